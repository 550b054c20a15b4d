// Fused quantized sparse self-attention for gfx950 (paper, Section 5.3): for one head and
// one row panel of the mask ONE WAVEFRONT runs SDDMM -> softmax -> int8 codes -> SpMM with
// the scores, probabilities and codes never leaving registers / LDS.  A wave never waits
// for another wave; latency is hidden by keeping ~16 such waves resident per CU, each
// with one 4 KB chunk of gathered rows in flight.
//
//   phase K  per chunk of 64 mask vectors: the Kmat rows named by the column indices are
//            copied from global memory straight into LDS (global_load_lds, 4 neighbouring
//            lanes per 64-byte row, no registers in between); one v_mfma_i32_16x16x64_i8
//            per 16 vectors gives the scores (head dim 64 = one MFMA; both operands are
//            contiguous along the reduction, Section 4.3).  The 8 Q rows sit in MFMA rows
//            0..7 for even tiles and in rows 8..15 for odd tiles, so two tiles share one
//            accumulator and all 64 lanes carry real scores.
//   softmax  fp32, base 2, over the panel's stored entries: in-lane over the tiles, DPP
//            rotations over the 16 lanes of a row, one cross-lane exchange for the two
//            tile parities; codes = clamp(rint(p / s_p), 0, 127) go to LDS as
//            [slot][8 rows] bytes (one 32-bit write per 4 codes).
//   phase V  SpMM (Section 4.2) per chunk: V rows are copied into the same LDS stage;
//            ds_read_b64_tr_b8 delivers both MFMA operands in place: the codes transposed
//            to [row][16 slots] and the V rows transposed to [column][16 slots].
//   output   the 8 x 64 tile goes through LDS once to be stored as fp32 with 16-byte stores.
// LDS rows are 64 bytes; slot s of a chunk lives in row (s % 4) * 16 + s / 4 (so that a
// lane's 4 column indices are consecutive) and its 16-byte segments are XOR-swizzled with
// s % 4 so that rows read together fall into different banks.
#include "internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v2i lds_v2i;
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

// max / sum over the 16 lanes of a DPP row via rotations by 1, 2, 4, 8 (VALU only)
template <int CTRL> __device__ __forceinline__ float dpp_rot(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, dpp_rot<0x121>(v)); // row_ror:1
    v = fmaxf(v, dpp_rot<0x122>(v));
    v = fmaxf(v, dpp_rot<0x124>(v));
    v = fmaxf(v, dpp_rot<0x128>(v));
    return v;
}
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_rot<0x121>(v);
    v += dpp_rot<0x122>(v);
    v += dpp_rot<0x124>(v);
    v += dpp_rot<0x128>(v);
    return v;
}

// MAXCH: longest panel in chunks of 64 vectors.
template <int MAXCH>
__global__ __launch_bounds__(64, 4) void attention_fused_kernel(AttnArgs a)
{
    constexpr int DK = 64;
    constexpr int NPR = MAXCH * 2; // pairs of score tiles
    __shared__ __attribute__((aligned(16))) char stage[4096];       // one chunk of gathered rows
    __shared__ __attribute__((aligned(16))) char Pl[MAXCH * 64 * 8]; // codes, [slot][8 rows]

    const int lane = threadIdx.x;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane >> 2, seg = lane & 3;
    const int panel = blockIdx.x, head = blockIdx.y;
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    const int nch = (n + MC_CHUNK - 1) / MC_CHUNK;
    const int32_t *idx = a.slot_idx + s0;
    const int64_t hoff = (int64_t)head * a.head_stride;
    const uint8_t *Kh = a.Km + hoff, *Vh = a.Vm + hoff;
    float *Oh = a.O + hoff + (int64_t)panel * 8 * DK;

    // Q rows twice: in MFMA rows 0..7 (q_lo) and in rows 8..15 (q_hi)
    v4i q_lo = {0, 0, 0, 0}, q_hi = {0, 0, 0, 0};
    {
        const v4i qv = *reinterpret_cast<const v4i *>(a.Q + hoff + (int64_t)(panel * 8 + (j & 7)) * DK + g * 16);
        if (j < 8) q_lo = qv; else q_hi = qv;
    }
    // lane (rg, seg), load instruction i: segment seg ^ i of the row in slot rg*4 + i
    int segoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) segoff[i] = (seg ^ i) * 16;
    auto gather = [&](const uint8_t *base, int c) {
        const v4i ix = *reinterpret_cast<const v4i *>(idx + c * MC_CHUNK + rg * 4);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t *)(base + (unsigned)ix[i] * DK + segoff[i]), (lptr_t *)(stage + i * 1024), 16, 0, 0);
    };

    // ---- phase K: scores; lane (j, g) owns row 4*(g&1) + r of tile 2*pr + (g >> 1) -----
    constexpr float LOG2E = 1.4426950408889634f;
    const float scale2 = a.score_scale * LOG2E; // softmax in base 2: exp(x - m) = 2^(x2 - m2)
    // K operand of tile tl: slot tl*16 + j -> LDS row (j&3)*16 + tl*4 + (j>>2), segment g ^ (j&3)
    const int krow = ((j & 3) * 16 + (j >> 2)) * 64 + ((g ^ (j & 3)) * 16);
    float x[NPR][4];
    float mrow[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) {
        if (c < nch) {
            gather(Kh, c);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            v4i acc = {0, 0, 0, 0};
            if (c < nch) {
                const v4i kA = *reinterpret_cast<const v4i *>(stage + krow + (2 * pr) * 256);
                const v4i kB = *reinterpret_cast<const v4i *>(stage + krow + (2 * pr + 1) * 256);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_lo, kA, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_hi, kB, acc, 0, 0, 0);
            }
            const bool valid = c * MC_CHUNK + (2 * pr + (g >> 1)) * 16 + j < n;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                x[c * 2 + pr][r] = valid ? (float)acc[r] * scale2 : -INFINITY;
                mrow[r] = fmaxf(mrow[r], x[c * 2 + pr][r]);
            }
        }
        if (c < nch) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // rows consumed before the next gather
    }

    // ---- softmax over row 4*(g&1) + r ---------------------------------------------------------
    float srow[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        mrow[r] = row16_max(mrow[r]);
        mrow[r] = fmaxf(mrow[r], __shfl_xor(mrow[r], 32, 64));
        if (mrow[r] == -INFINITY) mrow[r] = 0.f; // empty panel: keep exp2 away from inf - inf
    }
#pragma unroll
    for (int t = 0; t < NPR; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            x[t][r] = __builtin_amdgcn_exp2f(x[t][r] - mrow[r]);
            srow[r] += x[t][r];
        }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        srow[r] = row16_sum(srow[r]);
        srow[r] += __shfl_xor(srow[r], 32, 64);
    }
    // codes of slot (tile*16 + j), rows 4*(g&1) .. +3: one 32-bit LDS write
#pragma unroll
    for (int c = 0; c < MAXCH; ++c) {
        if (c < nch) {
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                unsigned packed = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float code = fminf(fmaxf(rintf(x[c * 2 + pr][r] / srow[r] * a.inv_s_p), 0.f), 127.f);
                    packed |= (unsigned)(int)code << (8 * r);
                }
                const int slot = c * MC_CHUNK + (2 * pr + (g >> 1)) * 16 + j;
                *reinterpret_cast<unsigned *>(Pl + slot * 8 + 4 * (g & 1)) = packed;
            }
        }
    }

    // ---- phase V: O = codes * V ------------------------------------------------------------------
    v4i o[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) o[ct] = (v4i){0, 0, 0, 0};
    const int src = lane & 15, ii = src >> 1;
    int vaddr[2], paddr[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int s = g * 16 + 8 * h + ii;   // slot within the chunk supplied by this lane
        vaddr[h] = (s & 3) * 1024 + (s >> 2) * 64 + ((s & 3) * 16) + 8 * (src & 1);
        paddr[h] = s * 8;
    }
    for (int c = 0; c < nch; ++c) {
        gather(Vh, c);
        // codes of this chunk, transposed to the MFMA row operand: row j < 8, slots g*16 .. +15
        const v2i p0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(Pl + c * 512 + paddr[0]));
        const v2i p1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(Pl + c * 512 + paddr[1]));
        v4i aop = {p0.x, p0.y, p1.x, p1.y};
        if (j >= 8) aop = (v4i){0, 0, 0, 0};
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            const v2i d0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(stage + (vaddr[0] ^ (ct * 16))));
            const v2i d1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(stage + (vaddr[1] ^ (ct * 16))));
            const v4i bop = {d0.x, d0.y, d1.x, d1.y};
            o[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, bop, o[ct], 0, 0, 0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }

    // ---- output: 8 x 64 tile through LDS, scaled, 16-byte stores ------------------------------
    int *Ol = reinterpret_cast<int *>(stage);
    if (g < 2) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) Ol[(4 * g + r) * DK + ct * 16 + j] = o[ct][r];
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int piece = h * 64 + lane, row = piece >> 4, col = (piece & 15) * 4;
        const v4i sres = *reinterpret_cast<const v4i *>(&Ol[row * DK + col]);
        const v4f f = {sres.x * a.out_scale, sres.y * a.out_scale, sres.z * a.out_scale, sres.w * a.out_scale};
        *reinterpret_cast<v4f *>(Oh + row * DK + col) = f;
    }
}

} // namespace

int attention_fused_max_vectors() { return 8 * 64; }

hipError_t launch_attention_fused(const AttnArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.heads == 0) return hipSuccess;
    dim3 grid((unsigned)a.P, (unsigned)a.heads), block(64);
    hipLaunchKernelGGL((attention_fused_kernel<8>), grid, block, 0, s, a);
    return hipGetLastError();
}
