// Sparse softmax with fused dequantisation of the scores and re-quantisation of the
// probabilities (Section 5.3) for gfx950.
//
// One workgroup of 256 threads per (panel, score set).  A panel's scores are one contiguous block
// of nvec_p * V int32 in interchange order (V consecutive values per stored vector), and every
// row of the panel has the same number of entries, so the rows of a panel are reduced together.
//
//   softmax_wave_kernel<R>    panels of up to R * 256 scores: ONE WAVE per panel (four panels per
//                             workgroup), each lane keeps R pieces of four consecutive scores in
//                             registers; one read of the scores, one exponential per score, row
//                             reductions by lane exchanges, no barrier anywhere.
//   softmax_group_kernel<R,NW> panels of up to R * NW * 256 scores: the same with the NW waves of a
//                             workgroup sharing one panel (reductions finish through LDS).
//   softmax_general_kernel    any panel length: three passes over the scores in memory.
//
// The integer codes go out either in interchange order (int8 / int16) or straight in the device
// panel format that the SpMM kernels read (Section 4.3 lets the producer pick the format by its
// consumer): per chunk of 64 slots and group of 16 slots, [row v][16 slots] bytes; 16-bit codes as
// a high and a low signed-byte plane; padded slots zero.
#include "internal.h"

#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;

// largest code: int8 maximum, or the largest 16-bit value that splits into two signed bytes
__device__ __forceinline__ float code_max(int code_bits) { return (code_bits == 16) ? 32639.f : 127.f; }

// byte offset of element e = i * V + v (vector i of the panel, row v; V = 1 << vs) in the panel's
// device-format values; 16-bit codes (pb = 2): offset of the high plane, the low plane follows
// 16 * V bytes later
__device__ __forceinline__ int dev_offset(int e, int vs, int pb)
{
    const int i = e >> vs, v = e & ((1 << vs) - 1);
    return (((i >> 6) * MC_CHUNK + ((i >> 4) & 3) * 16) << vs) * pb + v * 16 + (i & 15);
}

// Combines the four per-lane values of every lane that holds the same rows: a lane's piece e0 =
// 4 * (tid + 256 k) starts at row e0 % V, i.e. rows 4 * (lane % 2) + r for V = 8, r for V = 4 and
// r % 2 for V = 2 (then components 0/2 and 1/3 belong together).  MAX: maximum, else sum.
template <bool MAX> __device__ __forceinline__ float comb(float x, float y) { return MAX ? fmaxf(x, y) : x + y; }

template <bool MAX> __device__ __forceinline__ v4f reduce_lanes(v4f x, int V)
{
    if (V == 2) {
        x.x = x.z = comb<MAX>(x.x, x.z);
        x.y = x.w = comb<MAX>(x.y, x.w);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float v = x[r];
        if (V < 8) v = comb<MAX>(v, __shfl_xor(v, 1, 64));
#pragma unroll
        for (int d = 2; d < 64; d <<= 1) v = comb<MAX>(v, __shfl_xor(v, d, 64));
        x[r] = v;
    }
    return x;
}

// ... and across the NW waves of a workgroup: lanes 0 and 1 of each wave publish their rows
template <bool MAX, int NW> __device__ __forceinline__ v4f reduce_rows(v4f x, int V, float (*red)[8], int lane, int w)
{
    x = reduce_lanes<MAX>(x, V);
    const int c = (V == 8) ? (lane & 1) : 0;
    if (lane < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[w][c * 4 + r] = x[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float v = red[0][c * 4 + r];
#pragma unroll
        for (int k = 1; k < NW; ++k) v = comb<MAX>(v, red[k][c * 4 + r]);
        x[r] = v;
    }
    return x;
}

// Scores -> codes for a panel handled by NT threads (one wave: NT = 64; a workgroup: NT = 256);
// thread t of them owns the pieces 4 * (t + NT * k), k < R.  reduce(x, is_max) finishes a row
// reduction over those threads; sync() orders the staged codes before they are copied out.
// C16: 16-bit codes (else 8-bit); DEV: device panel format (else interchange order) -- compile-time,
// so that the unrolled per-piece code carries no branches on the mode.
// The raw scores of one panel as the NT threads that handle it hold them: thread t owns the pieces
// 4 * (t + NT * k), k < R (only the whole ones are loaded), and thread 0 the half piece that V = 2
// with an odd number of vectors leaves at the end.
template <int R> struct PanelScores {
    v4i s[R];
    int t0, t1;      // the half piece (thread 0)
    int cnt;         // scores of the panel
    int64_t base;    // of its block in the score / code arrays
};

template <int R, int NT>
__device__ __forceinline__ void load_scores(const SoftmaxArgs &a, int panel, int batch, int t, PanelScores<R> &p)
{
    p.base = (int64_t)batch * a.batch_stride + (int64_t)a.row_ptr[panel] * a.V;
    p.cnt = (a.row_ptr[panel + 1] - a.row_ptr[panel]) * a.V;
    const int32_t *S = a.S + p.base;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int e0 = 4 * (t + NT * k);
        if (e0 + 4 <= p.cnt) __builtin_memcpy(&p.s[k], S + e0, 16);   // only 8-byte alignment is known (V = 2)
    }
    p.t0 = p.t1 = 0;
    if ((p.cnt & 3) != 0 && t == 0) {
        p.t0 = S[p.cnt - 2];
        p.t1 = S[p.cnt - 1];
    }
}

template <int R, int NT, bool C16, bool DEV, class Reduce, class Sync>
__device__ __forceinline__ void softmax_panel(const SoftmaxArgs &a, int panel, int batch, int t, const PanelScores<R> &p,
                                              uint8_t *stage, Reduce &&reduce, Sync &&sync)
{
    const int V = a.V, vs = (V == 8) ? 3 : (V == 4 ? 2 : 1);
    const int64_t base = p.base;
    const int cnt = p.cnt;

    // softmax in base 2: exp(x - max) = 2^(x * log2(e) - max2)
    const float scale2 = a.score_scale * LOG2E;
    const v4f absent = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    v4f x[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int e0 = 4 * (t + NT * k);
        const v4i s = p.s[k];
        x[k] = (e0 + 4 <= cnt) ? (v4f){(float)s.x * scale2, (float)s.y * scale2, (float)s.z * scale2, (float)s.w * scale2} : absent;
    }
    // the half piece: components 0, 1 = rows 0, 1 of the last vector
    const bool tail = (cnt & 3) != 0;
    v4f xt = absent;
    if (tail && t == 0) {
        xt.x = (float)p.t0 * scale2;
        xt.y = (float)p.t1 * scale2;
    }
    v4f m = {fmaxf(x[0].x, xt.x), fmaxf(x[0].y, xt.y), x[0].z, x[0].w};
#pragma unroll
    for (int k = 1; k < R; ++k) m = (v4f){fmaxf(m.x, x[k].x), fmaxf(m.y, x[k].y), fmaxf(m.z, x[k].z), fmaxf(m.w, x[k].w)};
    m = reduce(m, std::true_type{});

    v4f sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
        for (int r = 0; r < 4; ++r) x[k][r] = __builtin_amdgcn_exp2f(x[k][r] - m[r]); // absent entries: 2^-inf = 0
        sum += x[k];
    }
    xt.x = __builtin_amdgcn_exp2f(xt.x - m.x);
    xt.y = __builtin_amdgcn_exp2f(xt.y - m.y);
    sum.x += xt.x;
    sum.y += xt.y;
    sum = reduce(sum, std::false_type{});

    // p / s_p = e * (1 / (sum * s_p)): one division per row.  e * rinv is never negative, so the
    // code is min(., largest code) rounded to nearest even (v_cvt_pk_u8_f32 rounds that way and
    // drops the byte into place).
    const v4f rinv = {a.inv_s_p / sum.x, a.inv_s_p / sum.y, a.inv_s_p / sum.z, a.inv_s_p / sum.w};
    const float qmax = code_max(C16 ? 16 : 8);
    constexpr int pb = C16 ? 2 : 1;
    auto codes_of = [&](v4f e, unsigned &lo, unsigned &hi) {
        // 8 bit: lo = the four codes as bytes; 16 bit: lo, hi = codes 0, 1 and 2, 3 as halfwords
        lo = hi = 0;
        if (!C16) {
#pragma unroll
            for (int r = 0; r < 4; ++r) lo = __builtin_amdgcn_cvt_pk_u8_f32(fminf(e[r] * rinv[r], qmax), r, lo);
        } else {
            const unsigned q0 = (unsigned)rintf(fminf(e.x * rinv.x, qmax)), q1 = (unsigned)rintf(fminf(e.y * rinv.y, qmax));
            const unsigned q2 = (unsigned)rintf(fminf(e.z * rinv.z, qmax)), q3 = (unsigned)rintf(fminf(e.w * rinv.w, qmax));
            lo = q0 | (q1 << 16);
            hi = q2 | (q3 << 16);
        }
    };
    // one code into the staged device format
    auto stage_code = [&](int off, unsigned q) {
        if (C16) {
            const unsigned h = (q + 128) >> 8; // balanced split into two signed bytes
            stage[off] = (uint8_t)h;
            stage[off + 16 * V] = (uint8_t)(q - h * 256);
        } else {
            stage[off] = (uint8_t)q;
        }
    };
    auto code_at = [&](unsigned lo, unsigned hi, int r) -> unsigned {
        return C16 ? ((r < 2 ? lo : hi) >> (16 * (r & 1))) & 0xffffu : (lo >> (8 * r)) & 0xffu;
    };
    const bool aligned = (base & 3) == 0;  // else (V = 2 only) the block starts half a piece off
    const int cpad = (((cnt >> vs) + MC_CHUNK - 1) / MC_CHUNK * MC_CHUNK) << vs;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int e0 = 4 * (t + NT * k);
        const bool full = e0 + 4 <= cnt;
        unsigned lo, hi;
        codes_of(x[k], lo, hi);
        if (!DEV) {
            if (!full) continue;
            if (!C16) {
                int8_t *o = static_cast<int8_t *>(a.codes) + base + e0;
                if (aligned) {
                    *reinterpret_cast<unsigned *>(o) = lo;
                } else {
                    reinterpret_cast<uint16_t *>(o)[0] = (uint16_t)lo;
                    reinterpret_cast<uint16_t *>(o)[1] = (uint16_t)(lo >> 16);
                }
            } else {
                int16_t *o = static_cast<int16_t *>(a.codes) + base + e0;
                if (aligned) {
                    *reinterpret_cast<uint2 *>(o) = make_uint2(lo, hi);
                } else {
                    reinterpret_cast<unsigned *>(o)[0] = lo;
                    reinterpret_cast<unsigned *>(o)[1] = hi;
                }
            }
        } else if (e0 < cpad) {
            // a piece holds rows v .. v+3 of one vector (V >= 4: 16 bytes apart) or two vectors (V = 2);
            // beyond the panel's end the padded slots of the last chunk get code 0 (their e is 0), and the
            // half piece at the end is left to thread 0
            const int offa = dev_offset(e0, vs, pb), offb = (V == 2) ? dev_offset(e0 + 2, vs, pb) : offa + 32;
            if (full || e0 >= cnt) {
                stage_code(offa, code_at(lo, hi, 0));
                stage_code(offa + 16, code_at(lo, hi, 1));
            }
            stage_code(offb, code_at(lo, hi, 2));
            stage_code(offb + 16, code_at(lo, hi, 3));
        }
    }
    if (tail && t == 0) {
        unsigned lo, hi;
        codes_of(xt, lo, hi);
        if (!DEV) {
            if (!C16) *reinterpret_cast<uint16_t *>(static_cast<int8_t *>(a.codes) + base + cnt - 2) = (uint16_t)lo;
            else *reinterpret_cast<unsigned *>(static_cast<int16_t *>(a.codes) + base + cnt - 2) = lo;
        } else {
            const int off = dev_offset(cnt - 2, vs, pb);
            stage_code(off, code_at(lo, hi, 0));
            stage_code(off + 16, code_at(lo, hi, 1));
        }
    }
    if (DEV) {
        sync();
        const int s0 = a.panel_ptr[2 * panel]; // chunk-aligned first slot of the panel
        uint8_t *dst = a.dev_vals + (int64_t)batch * a.dev_batch_stride + (int64_t)(s0 / MC_CHUNK) * (MC_CHUNK * V * pb);
        for (int o = t * 16; o < cpad * pb; o += NT * 16)
            *reinterpret_cast<v4i *>(dst + o) = *reinterpret_cast<const v4i *>(stage + o);
    }
}

// four waves per SIMD: every panel of a 4096-panel launch is resident at once
template <int R, bool C16, bool DEV>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void softmax_wave_kernel(SoftmaxArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage[4][DEV ? R * 256 * (C16 ? 2 : 1) : 16]; // device-format codes, per wave
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int panel = blockIdx.x * 4 + w, batch = blockIdx.y, V = a.V;
    if (panel >= a.P || a.row_ptr[panel + 1] == a.row_ptr[panel]) return; // waves never meet in this kernel
    PanelScores<R> p;
    load_scores<R, 64>(a, panel, batch, lane, p);
    softmax_panel<R, 64, C16, DEV>(
        a, panel, batch, lane, p, stage[w],
        [&](v4f x, auto is_max) { return reduce_lanes<decltype(is_max)::value>(x, V); },
        [&]() {
            // LDS executes a wave's instructions in order; keep the compiler from moving the reads up
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_wave_barrier();
        });
}

// NW waves per panel (one workgroup per (panel, score set)): panels of up to R * NW * 256 scores; the
// row reductions finish through LDS.  Every barrier is reached by all waves (an empty panel is
// left before the first one).
template <int R, int NW, bool C16, bool DEV> __global__ __launch_bounds__(64 * NW) void softmax_group_kernel(SoftmaxArgs a)
{
    constexpr int NT = 64 * NW;
    __shared__ float red_max[NW][8], red_sum[NW][8];
    __shared__ __attribute__((aligned(16))) uint8_t stage[DEV ? R * NT * 4 * (C16 ? 2 : 1) : 16]; // device-format codes of the panel
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int panel = blockIdx.x, batch = blockIdx.y, V = a.V;
    if (a.row_ptr[panel + 1] == a.row_ptr[panel]) return;                 // uniform: before any barrier
    PanelScores<R> p;
    load_scores<R, NT>(a, panel, batch, tid, p);
    softmax_panel<R, NT, C16, DEV>(
        a, panel, batch, tid, p, stage,
        [&](v4f x, auto is_max) {
            constexpr bool MAX = decltype(is_max)::value;
            return reduce_rows<MAX, NW>(x, V, MAX ? red_max : red_sum, lane, w);
        },
        [&]() { __syncthreads(); });
}

// Thread t owns elements t, t+256, ... of the panel's score block; 256 % V == 0, so a thread
// always stays in row v = t % V.
__global__ __launch_bounds__(256) void softmax_general_kernel(SoftmaxArgs a)
{
    __shared__ float red[256];
    const int tid = threadIdx.x, panel = blockIdx.x, batch = blockIdx.y;
    const int V = a.V, v = tid % V;
    const int64_t base = (int64_t)batch * a.batch_stride + (int64_t)a.row_ptr[panel] * V;
    const int cnt = (a.row_ptr[panel + 1] - a.row_ptr[panel]) * V;
    const int32_t *S = a.S + base;

    const float scale2 = a.score_scale * LOG2E;
    float m = -INFINITY;
    for (int e = tid; e < cnt; e += 256) m = fmaxf(m, (float)S[e] * scale2);
    red[tid] = m;
    __syncthreads();
    m = -INFINITY;
    for (int t = v; t < 256; t += V) m = fmaxf(m, red[t]);
    __syncthreads();

    float sum = 0.f;
    for (int e = tid; e < cnt; e += 256) sum += __builtin_amdgcn_exp2f((float)S[e] * scale2 - m);
    red[tid] = sum;
    __syncthreads();
    sum = 0.f;
    for (int t = v; t < 256; t += V) sum += red[t];

    const float rinv = a.inv_s_p / sum;
    const float qmax = code_max(a.code_bits);
    if (a.codes) {
        for (int e = tid; e < cnt; e += 256) {
            const float q = fminf(fmaxf(rintf(__builtin_amdgcn_exp2f((float)S[e] * scale2 - m) * rinv), 0.f), qmax);
            if (a.code_bits == 16) static_cast<int16_t *>(a.codes)[base + e] = (int16_t)(int)q;
            else static_cast<int8_t *>(a.codes)[base + e] = (int8_t)(int)q;
        }
        return;
    }
    const int s0 = a.panel_ptr[2 * panel];
    const int cpad = (cnt / V + MC_CHUNK - 1) / MC_CHUNK * MC_CHUNK * V;
    const int pb = a.code_bits / 8, vs = (V == 8) ? 3 : (V == 4 ? 2 : 1);
    uint8_t *dst = a.dev_vals + (int64_t)batch * a.dev_batch_stride + (int64_t)(s0 / MC_CHUNK) * (MC_CHUNK * V * pb);
    for (int e = tid; e < cpad; e += 256) {
        int x = 0; // padded slots hold zeros
        if (e < cnt) x = (int)fminf(fmaxf(rintf(__builtin_amdgcn_exp2f((float)S[e] * scale2 - m) * rinv), 0.f), qmax);
        uint8_t *o = dst + dev_offset(e, vs, pb);
        if (a.code_bits == 16) {
            const int hi = (x + 128) >> 8;
            o[0] = (uint8_t)hi;
            o[16 * V] = (uint8_t)(x - hi * 256);
        } else {
            o[0] = (uint8_t)x;
        }
    }
}

} // namespace

template <bool C16, bool DEV> hipError_t launch_softmax_mode(const SoftmaxArgs &a, hipStream_t s)
{
    dim3 grid((unsigned)a.P, (unsigned)a.batch), grid4((unsigned)((a.P + 3) / 4), (unsigned)a.batch);
    const int64_t longest = (int64_t)a.max_panel_chunks * MC_CHUNK * a.V; // scores of the longest panel, padding included
    const int64_t units = (int64_t)a.P * a.batch;
    if (a.variant == 0 && longest <= 16 * 256) {
        // few panels: two waves per panel halve the time of the launch (5.9 -> 5.2 us for 512 panels of 3280
        // scores); many: one wave per panel (15.0 against 17.4 us for 4096 of them)
        if (units <= 1024) hipLaunchKernelGGL((softmax_group_kernel<8, 2, C16, DEV>), grid, dim3(128), 0, s, a);
        else hipLaunchKernelGGL((softmax_wave_kernel<16, C16, DEV>), grid4, dim3(256), 0, s, a);
    } else if (a.variant != 2 && longest <= 16 * 1024) {
        hipLaunchKernelGGL((softmax_group_kernel<16, 4, C16, DEV>), grid, dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL(softmax_general_kernel, grid, dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_softmax(const SoftmaxArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0) return hipSuccess;
    if (a.codes) return (a.code_bits == 16) ? launch_softmax_mode<true, false>(a, s) : launch_softmax_mode<false, false>(a, s);
    return (a.code_bits == 16) ? launch_softmax_mode<true, true>(a, s) : launch_softmax_mode<false, true>(a, s);
}
