// Fused quantized sparse self-attention for gfx950 (paper, Section 5.3): for one head and
// one row panel of the mask a workgroup runs SDDMM -> softmax -> int8 codes -> SpMM with
// the scores, probabilities and codes never leaving registers / LDS.
//
//   phase 0  every wave copies the Kmat rows named by its chunks of 64 mask vectors from
//            global memory straight into LDS (global_load_lds, 4 neighbouring lanes per
//            64-byte row, no registers in between).
//   phase 1  scores: one v_mfma_i32_16x16x64_i8 per 16 mask vectors (head dim 64 = one
//            MFMA); both operands are contiguous along the reduction (Section 4.3), so the
//            column operand is a plain 128-bit LDS read.  The same LDS region is then
//            refilled with the V rows of the same chunks while the softmax runs.
//   phase 2  fp32 softmax over the panel's stored entries; the row maximum and sum are
//            reduced over the 16 lanes that share a row and then over the 4 waves via LDS;
//            codes = clamp(rint(p / s_p), 0, 127) go to LDS in the row-major order the
//            SpMM row operand wants (16 consecutive slots per lane).
//   phase 3  SpMM (Section 4.2): ds_read_b64_tr_b8 hands each lane 8 reduction-consecutive
//            bytes of its own column of the V rows, which is the MFMA column-operand
//            layout, so no register transpose is needed.
//   phase 4  the 4 partial 8 x 64 tiles are summed through LDS, scaled by s_p * s_v and
//            stored as fp32 with 16-byte stores.
// LDS rows are 64 bytes; the 16-byte segments of a row are XOR-swizzled with the slot
// number so that the rows read together fall into different banks.
#include "internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v2i lds_v2i;

constexpr int AW = 4; // waves per workgroup

// XOR applied to the 16-byte segment number of slot r (r within a chunk of 64)
__device__ __forceinline__ int seg_swizzle(int r) { return ((r >> 1) & 3) ^ ((r >> 4) & 1); }

__device__ __forceinline__ float row16_max(float v)
{
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) v = fmaxf(v, __shfl_xor(v, m, 16));
    return v;
}
__device__ __forceinline__ float row16_sum(float v)
{
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) v += __shfl_xor(v, m, 16);
    return v;
}

typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

// CPW: chunks of 64 mask vectors per wave; a panel may hold up to AW * CPW * 64 vectors.
template <int CPW>
__global__ __launch_bounds__(64 * AW) void attention_fused_kernel(AttnArgs a)
{
    constexpr int DK = 64;
    constexpr int MAXPAD = AW * CPW * 64;
    constexpr int NP = CPW * 2;           // pairs of score tiles (2 x 16 vectors) per wave
    constexpr int PST = MAXPAD + 16;      // row stride of the code array
    __shared__ __attribute__((aligned(16))) char KVl[MAXPAD * DK]; // Kmat rows, then V rows, then partial tiles
    __shared__ __attribute__((aligned(16))) char Pl[8 * PST];
    __shared__ float red[2][AW][8];
    static_assert(MAXPAD * DK >= AW * 8 * DK * 4, "partial tiles must fit");

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int panel = blockIdx.x, head = blockIdx.y;
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    const int nch = (n + MC_CHUNK - 1) / MC_CHUNK;
    const int32_t *idx = a.slot_idx + s0;
    const int64_t hoff = (int64_t)head * a.head_stride;
    const uint8_t *Kh = a.Km + hoff, *Vh = a.Vm + hoff;
    float *Oh = a.O + hoff + (int64_t)panel * 8 * DK;

    if (n == 0) { // empty rows: zeros
        if (tid < 128) *reinterpret_cast<v4f *>(Oh + tid * 4) = (v4f){0.f, 0.f, 0.f, 0.f};
        return;
    }

    // ---- phase 0: Kmat rows of this wave's chunks -> LDS -----------------------------
    // lane l copies segment (l & 3) ^ swizzle of the row in slot i*16 + l/4; it lands at
    // byte i*1024 + l*16 of the chunk, i.e. row-major with 64-byte rows.
    unsigned roff[CPW][4];
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
        const int c = w + AW * cc;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rho = i * 16 + (lane >> 2);
            roff[cc][i] = 0;
            if (c < nch) roff[cc][i] = (unsigned)idx[c * MC_CHUNK + rho] * DK + (((lane & 3) ^ seg_swizzle(rho)) * 16);
        }
    }
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
        const int c = w + AW * cc;
        if (c < nch) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_global_load_lds((gptr_t *)(Kh + roff[cc][i]), (lptr_t *)(KVl + c * 4096 + i * 1024), 16, 0, 0);
        }
    }
    // Q rows twice: in MFMA rows 0..7 (q_lo) and in rows 8..15 (q_hi).  Two score tiles then
    // share one accumulator -- tile A from q_lo in rows 0..7, tile B from q_hi in rows 8..15 --
    // so that all 64 lanes carry real scores through the softmax.
    v4i q_lo = {0, 0, 0, 0}, q_hi = {0, 0, 0, 0};
    {
        const v4i qv = *reinterpret_cast<const v4i *>(a.Q + hoff + (int64_t)(panel * 8 + (j & 7)) * DK + g * 16);
        if (j < 8) q_lo = qv; else q_hi = qv;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- phase 1: scores; lane (j, g) owns row 4*(g&1) + r of tile 2*pr + (g >> 1) ------
    constexpr float LOG2E = 1.4426950408889634f;
    const float scale2 = a.score_scale * LOG2E; // softmax in base 2: exp(x - m) = 2^(x2 - m2)
    float x[NP][4];
    float mloc[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
        const int c = w + AW * cc;
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            v4i acc = {0, 0, 0, 0};
            if (c < nch) {
                const int rA = (2 * pr) * 16 + j, rB = rA + 16;
                const v4i kA = *reinterpret_cast<const v4i *>(KVl + c * 4096 + rA * 64 + ((g ^ seg_swizzle(rA)) * 16));
                const v4i kB = *reinterpret_cast<const v4i *>(KVl + c * 4096 + rB * 64 + ((g ^ seg_swizzle(rB)) * 16));
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_lo, kA, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_hi, kB, acc, 0, 0, 0);
            }
            const bool valid = c * MC_CHUNK + (2 * pr + (g >> 1)) * 16 + j < n;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                x[cc * 2 + pr][r] = valid ? (float)acc[r] * scale2 : -INFINITY;
                mloc[r] = fmaxf(mloc[r], x[cc * 2 + pr][r]);
            }
        }
    }
    // the Kmat rows have been consumed: refill the same LDS rows with the V rows
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
        const int c = w + AW * cc;
        if (c < nch) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_global_load_lds((gptr_t *)(Vh + roff[cc][i]), (lptr_t *)(KVl + c * 4096 + i * 1024), 16, 0, 0);
        }
    }

    // ---- phase 2: softmax over row 4*(g&1) + r ---------------------------------------------
    const int row0 = 4 * (g & 1);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        mloc[r] = row16_max(mloc[r]);
        mloc[r] = fmaxf(mloc[r], __shfl_xor(mloc[r], 32, 64));
    }
    if (j == 0 && g < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[0][w][row0 + r] = mloc[r];
    }
    __syncthreads();
    float m[4], sloc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = row0 + r;
        m[r] = fmaxf(fmaxf(red[0][0][row], red[0][1][row]), fmaxf(red[0][2][row], red[0][3][row]));
    }
#pragma unroll
    for (int t = 0; t < NP; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            x[t][r] = __builtin_amdgcn_exp2f(x[t][r] - m[r]);
            sloc[r] += x[t][r];
        }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        sloc[r] = row16_sum(sloc[r]);
        sloc[r] += __shfl_xor(sloc[r], 32, 64);
    }
    if (j == 0 && g < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[1][w][row0 + r] = sloc[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = row0 + r;
        const float sum = (red[1][0][row] + red[1][1][row]) + (red[1][2][row] + red[1][3][row]);
#pragma unroll
        for (int cc = 0; cc < CPW; ++cc) {
            const int c = w + AW * cc;
            if (c < nch) {
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    const float code = fminf(fmaxf(rintf(x[cc * 2 + pr][r] / sum * a.inv_s_p), 0.f), 127.f);
                    Pl[row * PST + c * MC_CHUNK + (2 * pr + (g >> 1)) * 16 + j] = (char)(int)code;
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // ---- phase 3: O_partial = codes * V over this wave's chunks -------------------------
    v4i o[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) o[ct] = (v4i){0, 0, 0, 0};
    const int src = lane & 15;
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
        const int c = w + AW * cc;
        if (c < nch) {
            v4i aop = {0, 0, 0, 0};
            if (j < 8) aop = *reinterpret_cast<const v4i *>(Pl + j * PST + c * MC_CHUNK + g * 16);
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                v2i d[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int r = g * 16 + 8 * h + (src >> 1);
                    const char *p = KVl + c * 4096 + r * 64 + ((ct ^ seg_swizzle(r)) * 16) + 8 * (src & 1);
                    d[h] = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)p);
                }
                const v4i bop = {d[0].x, d[0].y, d[1].x, d[1].y};
                o[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, bop, o[ct], 0, 0, 0);
            }
        }
    }

    // ---- phase 4: sum the waves' tiles, scale, store --------------------------------------
    __syncthreads(); // every wave is done with the V rows: reuse the region
    int *Ol = reinterpret_cast<int *>(KVl);
    if (g < 2) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) Ol[(w * 8 + 4 * g + r) * DK + ct * 16 + j] = o[ct][r];
    }
    __syncthreads();
    if (tid < 128) {
        const int row = tid >> 4, col = (tid & 15) * 4;
        v4i s = *reinterpret_cast<const v4i *>(&Ol[row * DK + col]);
#pragma unroll
        for (int ww = 1; ww < AW; ++ww) s += *reinterpret_cast<const v4i *>(&Ol[(ww * 8 + row) * DK + col]);
        const v4f f = {s.x * a.out_scale, s.y * a.out_scale, s.z * a.out_scale, s.w * a.out_scale};
        *reinterpret_cast<v4f *>(Oh + row * DK + col) = f;
    }
}

} // namespace

int attention_fused_max_vectors() { return AW * 2 * 64; }

hipError_t launch_attention_fused(const AttnArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.heads == 0) return hipSuccess;
    dim3 grid((unsigned)a.P, (unsigned)a.heads), block(64 * AW);
    hipLaunchKernelGGL((attention_fused_kernel<2>), grid, block, 0, s, a);
    return hipGetLastError();
}
