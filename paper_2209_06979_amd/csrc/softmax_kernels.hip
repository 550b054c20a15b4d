// Sparse softmax with fused dequantisation of the scores and re-quantisation of the
// probabilities (Section 5.3) for gfx950.
//
// One workgroup of 256 threads per (panel, score set).  A panel's scores are one contiguous block
// of nvec_p * V int32 in interchange order (V consecutive values per stored vector), and every
// row of the panel has the same number of entries, so the rows of a panel are reduced together.
//
//   softmax_cached_kernel<R>  panels of up to R * 1024 scores: each thread keeps R pieces of four
//                             consecutive scores in registers; one read of the scores, one
//                             exponential per score, row reductions by lane exchanges.
//   softmax_general_kernel    any panel length: three passes over the scores in memory.
//
// The integer codes go out either in interchange order (int8 / int16) or straight in the device
// panel format that the SpMM kernels read (Section 4.3 lets the producer pick the format by its
// consumer): per chunk of 64 slots and group of 16 slots, [row v][16 slots] bytes; 16-bit codes as
// a high and a low signed-byte plane; padded slots zero.
#include "internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;

// largest code: int8 maximum, or the largest 16-bit value that splits into two signed bytes
__device__ __forceinline__ float code_max(int code_bits) { return (code_bits == 16) ? 32639.f : 127.f; }

// byte offset of (vector i of the panel, row v) in the panel's device-format values; 16-bit
// codes: offset of the high plane, the low plane follows 16 * V bytes later
__device__ __forceinline__ int dev_offset(int i, int v, int V, int pb)
{
    return (i / MC_CHUNK) * (MC_CHUNK * V * pb) + ((i % MC_CHUNK) / 16) * (16 * V * pb) + v * 16 + (i % 16);
}

// Combines the four per-lane values of every lane that holds the same rows: a lane's piece e0 =
// 4 * (tid + 256 k) starts at row e0 % V, i.e. rows 4 * (lane % 2) + r for V = 8, r for V = 4 and
// r % 2 for V = 2 (then components 0/2 and 1/3 belong together).  MAX: maximum, else sum.
template <bool MAX> __device__ __forceinline__ float comb(float x, float y) { return MAX ? fmaxf(x, y) : x + y; }

template <bool MAX> __device__ __forceinline__ v4f reduce_rows(v4f x, int V, float (*red)[8], int lane, int w)
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
    // across the four waves: lanes 0 and 1 of each wave publish their rows
    const int c = (V == 8) ? (lane & 1) : 0;
    if (lane < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[w][c * 4 + r] = x[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        x[r] = comb<MAX>(comb<MAX>(red[0][c * 4 + r], red[1][c * 4 + r]), comb<MAX>(red[2][c * 4 + r], red[3][c * 4 + r]));
    }
    return x;
}

template <int R> __global__ __launch_bounds__(256) void softmax_cached_kernel(SoftmaxArgs a)
{
    __shared__ float red_max[4][8], red_sum[4][8];
    __shared__ __attribute__((aligned(16))) uint8_t stage[R * 1024 * 2]; // device-format codes of the panel
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int panel = blockIdx.x, batch = blockIdx.y, V = a.V;
    const int64_t base = (int64_t)batch * a.batch_stride + (int64_t)a.row_ptr[panel] * V;
    const int cnt = (a.row_ptr[panel + 1] - a.row_ptr[panel]) * V;
    if (cnt == 0) return;
    const int32_t *S = a.S + base;

    // softmax in base 2: exp(x - max) = 2^(x * log2(e) - max2)
    const float scale2 = a.score_scale * LOG2E;
    v4f x[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int e0 = 4 * (tid + 256 * k);
        v4f f = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (e0 + 4 <= cnt) {
            v4i s;
            __builtin_memcpy(&s, S + e0, 16);   // only 4-byte alignment is known (V = 2 panels start anywhere)
            f = (v4f){(float)s.x * scale2, (float)s.y * scale2, (float)s.z * scale2, (float)s.w * scale2};
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (e0 + r < cnt) f[r] = (float)S[e0 + r] * scale2;
        }
        x[k] = f;
    }
    v4f m = x[0];
#pragma unroll
    for (int k = 1; k < R; ++k) m = (v4f){fmaxf(m.x, x[k].x), fmaxf(m.y, x[k].y), fmaxf(m.z, x[k].z), fmaxf(m.w, x[k].w)};
    m = reduce_rows<true>(m, V, red_max, lane, w);

    v4f sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
        for (int r = 0; r < 4; ++r) x[k][r] = __builtin_amdgcn_exp2f(x[k][r] - m[r]); // absent entries: 2^-inf = 0
        sum += x[k];
    }
    sum = reduce_rows<false>(sum, V, red_sum, lane, w);

    // p / s_p = e * (1 / (sum * s_p)): one division per row
    const v4f rinv = {a.inv_s_p / sum.x, a.inv_s_p / sum.y, a.inv_s_p / sum.z, a.inv_s_p / sum.w};
    const float qmax = code_max(a.code_bits);
    const int pb = a.code_bits / 8;
    const bool aligned = (base & 3) == 0;  // interchange order: whole pieces can go out as one store
    const int cpad = (cnt / V + MC_CHUNK - 1) / MC_CHUNK * MC_CHUNK * V;
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int e0 = 4 * (tid + 256 * k);
        int q[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) q[r] = (int)fminf(fmaxf(rintf(x[k][r] * rinv[r]), 0.f), qmax);
        if (a.codes) {
            if (e0 >= cnt) continue;
            if (a.code_bits == 8) {
                int8_t *o = static_cast<int8_t *>(a.codes) + base + e0;
                if (aligned && e0 + 4 <= cnt) {
                    *reinterpret_cast<int *>(o) = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (e0 + r < cnt) o[r] = (int8_t)q[r];
                }
            } else {
                int16_t *o = static_cast<int16_t *>(a.codes) + base + e0;
                if (aligned && e0 + 4 <= cnt) {
                    *reinterpret_cast<int2 *>(o) = make_int2(q[0] | (q[1] << 16), q[2] | (q[3] << 16));
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (e0 + r < cnt) o[r] = (int16_t)q[r];
                }
            }
        } else if (e0 < cpad) {
            // the padded slots of the last chunk take part with code 0 (their e is 0)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = e0 + r, off = dev_offset(e / V, e % V, V, pb);
                if (a.code_bits == 16) {
                    const int hi = (q[r] + 128) >> 8;
                    stage[off] = (uint8_t)hi;
                    stage[off + 16 * V] = (uint8_t)(q[r] - hi * 256);
                } else {
                    stage[off] = (uint8_t)q[r];
                }
            }
        }
    }
    if (!a.codes) {
        __syncthreads();
        const int s0 = a.panel_ptr[2 * panel]; // chunk-aligned first slot of the panel
        uint8_t *dst = a.dev_vals + (int64_t)batch * a.dev_batch_stride + (int64_t)(s0 / MC_CHUNK) * (MC_CHUNK * V * pb);
        for (int o = tid * 16; o < cpad * pb; o += 256 * 16)
            *reinterpret_cast<v4i *>(dst + o) = *reinterpret_cast<const v4i *>(stage + o);
    }
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
    const int pb = a.code_bits / 8;
    uint8_t *dst = a.dev_vals + (int64_t)batch * a.dev_batch_stride + (int64_t)(s0 / MC_CHUNK) * (MC_CHUNK * V * pb);
    for (int e = tid; e < cpad; e += 256) {
        int x = 0; // padded slots hold zeros
        if (e < cnt) x = (int)fminf(fmaxf(rintf(__builtin_amdgcn_exp2f((float)S[e] * scale2 - m) * rinv), 0.f), qmax);
        uint8_t *o = dst + dev_offset(e / V, v, V, pb);
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

hipError_t launch_softmax(const SoftmaxArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0) return hipSuccess;
    dim3 grid((unsigned)a.P, (unsigned)a.batch), block(256);
    const int64_t longest = (int64_t)a.max_panel_chunks * MC_CHUNK * a.V; // scores of the longest panel, padding included
    if (a.variant != 2 && longest <= 4 * 1024) hipLaunchKernelGGL(softmax_cached_kernel<4>, grid, block, 0, s, a);
    else if (a.variant != 2 && longest <= 16 * 1024) hipLaunchKernelGGL(softmax_cached_kernel<16>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(softmax_general_kernel, grid, block, 0, s, a);
    return hipGetLastError();
}
