// Scores and softmax of the attention layer in one kernel, for head dimensions and panel lengths the
// single fused attention kernel does not take (paper, Section 5.3: SDDMM -> softmax -> re-quantisation;
// Section 4.3: the producer writes the operand format of the following SpMM).
//
// One workgroup per (row panel of the mask, head).  Its WK waves take the panel's chunks of 64 vectors
// round-robin exactly as the SDDMM kernel does -- the chunk's 64 Kmat rows copied from global memory
// straight into LDS, read back as 128-bit MFMA operands against the panel's Q rows held in registers --
// but instead of writing int32 scores to memory they leave them in LDS, already scaled for a base-2
// exponential, as 8 rows x (padded panel length) floats.  After one barrier every wave owns some of the
// eight rows (row maximum, exponentials and row sum: two sweeps over LDS), and after a second barrier all
// threads turn the exponentials into integer codes and write them in the device panel format of the SpMM's
// sparse operand, 16 bytes per thread and whole kilobytes per wave (padded slots zero).  The int32 scores and fp32 probabilities never reach HBM: per stored score the
// layer's three-kernel form wrote 4 and read 4 bytes here and this kernel writes 1 (or 2) bytes.
//
// Rows of Q / Kmat of any length up to RB bytes that is a multiple of 16: the stage holds RB bytes per
// row, copy segments beyond the row end fetch segment 0 again, and the Q operand is zero there, so those
// bytes add nothing.
#include "internal.h"
#include "sddmm_tile.h"

namespace {

using namespace mcs;

constexpr float LOG2E = 1.4426950408889634f;

// PB: bits of Q / Kmat (8 or 4); RB: staged bytes per Kmat row (64, 128 or 256); WK: waves; C16: 16-bit codes
template <int PB, int RB, int WK, bool C16>
__global__ __launch_bounds__(64 * WK) void scores_softmax_kernel(ScoresArgs a)
{
    constexpr int LPR = RB / 16, NI = LPR, RPI = 64 / LPR, KC = RB / 64;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane / LPR, seg = lane % LPR;
    const int panel = blockIdx.x, head = blockIdx.y;
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    if (n <= 0) return;                                         // no stored vector: no slot to write
    const int nch = (n + MC_CHUNK - 1) / MC_CHUNK, npad = nch * MC_CHUNK;
    const int32_t *idx = a.slot_idx + s0;
    const uint8_t *Km = a.Km + (int64_t)head * a.in_head_stride;
    const uint8_t *Qpanel = a.Q + (int64_t)head * a.in_head_stride + (int64_t)panel * 8 * a.in_token_stride;
    // LDS: [WK stages of 64 * RB bytes][8 rows x xstride floats]; xstride = longest padded panel + 4 keeps the
    // rows 16 bytes apart modulo the banks
    char *stage = lds + w * (64 * RB);
    const int xstride = a.max_npad + 4;
    float *xs = reinterpret_cast<float *>(lds + WK * (64 * RB));
    float *rinv_s = xs + 8 * xstride;                               // one factor per row, for the last pass

    v4i qf[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qf[kc] = load_q<PB>(Qpanel, a.in_token_stride, 8, a.row_bytes, kc, j, g);
    int segoff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int sg = seg ^ i;
        segoff[i] = (sg * 16 < a.row_bytes) ? sg * 16 : 0;
    }

    const float scale2 = a.score_scale * LOG2E;
    const int nmy = (nch > w) ? (nch - w + WK - 1) / WK : 0;
    v4i idxv[NI / 4];
    auto load_idx = [&](int c) {
#pragma unroll
        for (int t = 0; t < NI / 4; ++t) idxv[t] = *reinterpret_cast<const v4i *>(idx + c * MC_CHUNK + rg * NI + 4 * t);
    };
    if (nmy > 0) load_idx(w);
    for (int k = 0; k < nmy; ++k) {
        const int c = w + k * WK;
        // copy instruction i: lane (rg, seg) copies segment seg ^ i of the row in slot rg * NI + i to LDS row i * RPI + rg
#pragma unroll
        for (int i = 0; i < NI; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t *)(Km + (int64_t)idxv[i >> 2][i & 3] * a.in_token_stride + segoff[i]),
                                             (lptr_t *)(stage + i * 1024), 16, 0, 0);
        const bool more = k + 1 < nmy;
        if (more) load_idx(c + WK);
        if (more) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NI / 4) : "memory"); // rows landed, indices may still fly
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int tl = 0; tl < 4; ++tl) {
            const int s = tl * 16 + j;              // slot within the chunk
            const int i = s % NI, r = s / NI;       // its copy instruction and row group
            const char *rowp = stage + i * 1024 + r * RB;
            v4i acc = {0, 0, 0, 0}, acc2 = {0, 0, 0, 0};
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                const v4i kf = *reinterpret_cast<const v4i *>(rowp + (((kc * 4 + g) ^ i) * 16));
                mma_step<PB>(qf[kc], kf, kf, acc, acc2);
            }
            acc = finish_tile<PB>(acc, acc2);
            asm volatile("" : "+v"(acc)); // (opaque to the optimiser: this compiler crashes when it sees the MFMA result converted to float element by element)
            // accumulator register r of lane (j, g) is row 4g + r of the vector in this slot; absent (padded)
            // slots enter the softmax as -infinity
            if (g < 2) {
                const int slot = c * MC_CHUNK + s;
                const bool real = slot < n;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) xs[(4 * g + rr) * xstride + slot] = real ? (float)acc[rr] * scale2 : -INFINITY;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // reads done before the rows are overwritten
    }
    __syncthreads();

    // ---- softmax of rows w, w + WK, ...: lane l sweeps the pieces of four slots l, l + 64, ... ----------
    const float qmax = C16 ? 32639.f : 127.f;
    uint8_t *dev = a.dev_vals + (int64_t)head * a.dev_batch_stride + (int64_t)(s0 / MC_CHUNK) * (MC_CHUNK * 8 * (C16 ? 2 : 1));
    static_assert(8 % WK == 0, "every wave owns the same number of rows");
    for (int rw = 0; rw < 8 / WK; ++rw) {
        const int row = w + rw * WK;
        float *x = xs + row * xstride;
        float m = -INFINITY;
        for (int p = lane; p < npad / 4; p += 64) {
            const v4f v = *reinterpret_cast<const v4f *>(x + 4 * p);
            m = fmaxf(fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)), m);
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
        float sum = 0.f;
        for (int p = lane; p < npad / 4; p += 64) {
            v4f v = *reinterpret_cast<const v4f *>(x + 4 * p);
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = __builtin_amdgcn_exp2f(v[r] - m); // absent entries: 2^-inf = 0
            *reinterpret_cast<v4f *>(x + 4 * p) = v;
            sum += (v.x + v.y) + (v.z + v.w);
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) sum += __shfl_xor(sum, d, 64);
        // p / s_p = e * (1 / (sum * s_p)): one factor per row, published for the pass that writes the codes
        if (lane == 0) rinv_s[row] = a.inv_s_p / sum;
    }
    __syncthreads();

    // ---- codes: a thread takes 16 consecutive slots (one sub-stride) of one row, which are 16 consecutive bytes of
    // the device format; neighbouring threads take the 8 rows of the same sub-stride (128 contiguous bytes), so a
    // wave writes whole kilobytes.  The code is min(e * rinv, largest code) rounded to nearest even. ----
    constexpr int PBY = C16 ? 2 : 1;
    for (int item = tid; item < (npad / 16) * 8; item += 64 * WK) {
        const int sub = item >> 3, row = item & 7;
        const float rinv = rinv_s[row];
        const float *x = xs + row * xstride + sub * 16;
        unsigned q8[4], hi[4], lo[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const v4f v = *reinterpret_cast<const v4f *>(x + 4 * t);
            q8[t] = hi[t] = lo[t] = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (!C16) {
                    q8[t] = __builtin_amdgcn_cvt_pk_u8_f32(fminf(v[r] * rinv, qmax), r, q8[t]);
                } else {
                    const unsigned q = (unsigned)rintf(fminf(v[r] * rinv, qmax));
                    const unsigned h = (q + 128) >> 8;               // balanced split into two signed bytes
                    hi[t] |= (h & 0xffu) << (8 * r);
                    lo[t] |= ((q - h * 256) & 0xffu) << (8 * r);
                }
            }
        }
        uint8_t *o = dev + (int64_t)sub * (16 * 8 * PBY) + row * 16;
        // (ordinary stores: the SpMM that follows finds the codes in L2; streaming stores cost it 3 us at 8 x 4096 x 64)
        if (!C16) {
            *reinterpret_cast<v4i *>(o) = (v4i){(int)q8[0], (int)q8[1], (int)q8[2], (int)q8[3]};
        } else {
            *reinterpret_cast<v4i *>(o) = (v4i){(int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
            *reinterpret_cast<v4i *>(o + 16 * 8) = (v4i){(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3]};
        }
    }
}

template <int PB, int RB, int WK, bool C16> hipError_t launch_one(const ScoresArgs &a, hipStream_t s)
{
    auto kern = scores_softmax_kernel<PB, RB, WK, C16>;
    const int lds = WK * 64 * RB + 8 * (a.max_npad + 4) * 4 + 32;
    if (lds > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)a.P, (unsigned)a.heads), dim3(64 * WK), lds, s, a);
    return hipGetLastError();
}

template <int PB, int RB, bool C16> hipError_t launch_wk(const ScoresArgs &a, int waves, hipStream_t s)
{
    if (waves >= 4) return launch_one<PB, RB, 4, C16>(a, s);
    return launch_one<PB, RB, 2, C16>(a, s);
}

template <int PB, bool C16> hipError_t launch_rb(const ScoresArgs &a, int waves, hipStream_t s)
{
    if (a.row_bytes <= 64) return launch_wk<PB, 64, C16>(a, waves, s);
    if (a.row_bytes <= 128) return launch_wk<PB, 128, C16>(a, waves, s);
    return launch_wk<PB, 256, C16>(a, waves, s);
}

} // namespace

// longest panel (in padded vectors) and longest row the kernel takes: the scores of a panel must fit LDS
int scores_softmax_max_npad(int row_bytes, int waves)
{
    const int rb = row_bytes <= 64 ? 64 : (row_bytes <= 128 ? 128 : 256);
    const int wk = waves >= 4 ? 4 : 2;
    return (160 * 1024 - wk * 64 * rb - 128) / 32 - 4;
}

hipError_t launch_scores_softmax(const ScoresArgs &a, int qkv_bits, int code_bits, int waves, hipStream_t s)
{
    if (a.P == 0 || a.heads == 0) return hipSuccess;
    if (a.row_bytes > 256 || a.row_bytes % 16 != 0) return hipErrorInvalidValue;
    if (qkv_bits == 4) return code_bits == 16 ? launch_rb<4, true>(a, waves, s) : launch_rb<4, false>(a, waves, s);
    return code_bits == 16 ? launch_rb<8, true>(a, waves, s) : launch_rb<8, false>(a, waves, s);
}
