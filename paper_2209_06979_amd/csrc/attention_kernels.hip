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
#include "lds_async.h"

namespace {

using namespace mcu;

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
    constexpr int GROUP = 5;       // memory instructions per chunk: 4 row copies + 1 index load
    __shared__ __attribute__((aligned(16))) char stage[2 * 4096];    // two chunks of gathered rows
    __shared__ __attribute__((aligned(16))) char Pl[MAXCH * 64 * 8]; // codes, [slot][8 rows]

    const int lane = threadIdx.x;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane >> 2, seg = lane & 3;
    // Workgroups are handed to the 8 XCDs round-robin by linear id.  With id = panel * heads +
    // head, an XCD only ever sees the heads congruent to its number, so its L2 has to hold the
    // Kmat and V rows of those heads (1/8 of the data for 8 heads) instead of all of them.
    const int head = blockIdx.x % a.heads, panel = blockIdx.x / a.heads;
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
    // Lane (rg, seg), copy instruction i: segment seg ^ i of the row in slot rg*4 + i.
    // One group of GROUP memory instructions per chunk: its 4 row copies, then the load of the
    // column indices of the chunk two steps ahead (clamped) into the registers the copies have
    // just consumed -- the index registers alternate with the chunk parity.
    int segoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) segoff[i] = (seg ^ i) * 16;
    const unsigned stage_u = lds_addr_uniform(stage);
    v4i ixv[2];
    auto issue = [&](const uint8_t *base, auto CC) {
        constexpr int c = CC;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            copy16_to_lds(base + (unsigned)ixv[c & 1][i] * DK + segoff[i], stage_u + (c & 1) * 4096 + i * 1024);
        const int cn = (c + 2 < nch) ? c + 2 : c;
        ixv[c & 1] = gload128(idx + cn * MC_CHUNK + rg * 4);
    };
    auto start_pipeline = [&](const uint8_t *base) {
        ixv[0] = gload128(idx + rg * 4);
        ixv[1] = gload128(idx + ((nch > 1) ? MC_CHUNK : 0) + rg * 4);
        vm_wait<0>();
        tie(ixv[0]);
        tie(ixv[1]);
        if (nch > 0) issue(base, std::integral_constant<int, 0>{});
        if (nch > 1) issue(base, std::integral_constant<int, 1>{});
    };
    // Chunk c (and the indices loaded with it) has landed when only the younger group, if
    // any, is still outstanding.
    auto wait_chunk = [&](auto CC) {
        constexpr int c = CC;
        if (c + 1 < nch) vm_wait<GROUP>(); else vm_wait<0>();
        tie(ixv[c & 1]);
    };

    // ---- phase K: scores; lane (j, g) owns row 4*(g&1) + r of tile 2*pr + (g >> 1) -----
    constexpr float LOG2E = 1.4426950408889634f;
    const float scale2 = a.score_scale * LOG2E; // softmax in base 2: exp(x - m) = 2^(x2 - m2)
    // K operand of tile tl: slot tl*16 + j -> LDS row (j&3)*16 + tl*4 + (j>>2), segment g ^ (j&3)
    const unsigned kaddr = lds_addr(stage) + ((j & 3) * 16 + (j >> 2)) * 64 + ((g ^ (j & 3)) * 16);
    float x[NPR][4];
    float mrow[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    start_pipeline(Kh);
    static_for<MAXCH>([&](auto C) {
        constexpr int c = C, ST = (c & 1) * 4096;
        v4i acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
        if (c < nch) {
            wait_chunk(C);
            v4i kA0 = lds_read128<ST>(kaddr), kB0 = lds_read128<ST + 256>(kaddr);
            v4i kA1 = lds_read128<ST + 512>(kaddr), kB1 = lds_read128<ST + 768>(kaddr);
            lds_wait(kA0, kB0, kA1, kB1);
            if (c + 2 < nch) issue(Kh, std::integral_constant<int, c + 2>{}); // the stage is free again
            acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_lo, kA0, acc0, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_hi, kB0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_lo, kA1, acc1, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_hi, kB1, acc1, 0, 0, 0);
        }
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            const v4i acc = pr ? acc1 : acc0;
            const bool valid = c * MC_CHUNK + (2 * pr + (g >> 1)) * 16 + j < n;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                x[c * 2 + pr][r] = valid ? (float)acc[r] * scale2 : -INFINITY;
                mrow[r] = fmaxf(mrow[r], x[c * 2 + pr][r]);
            }
        }
    });
    // all Kmat rows are consumed: start copying V rows while the softmax runs
    start_pipeline(Vh);

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
    unsigned vaddr[2][4], paddr[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int s = g * 16 + 8 * h + ii;   // slot within the chunk supplied by this lane
        const int base = (s & 3) * 1024 + (s >> 2) * 64 + ((s & 3) * 16) + 8 * (src & 1);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) vaddr[h][ct] = lds_addr(stage) + (base ^ (ct * 16));
        paddr[h] = lds_addr(Pl) + s * 8;
    }
    static_for<MAXCH>([&](auto C) {
        constexpr int c = C;
        if (c < nch) {
            wait_chunk(C);
            // codes of this chunk, transposed to the MFMA row operand: row j < 8, slots g*16 .. +15
            v2i p0 = lds_read_tr8<c * 512>(paddr[0]), p1 = lds_read_tr8<c * 512>(paddr[1]);
            v2i d[4][2];
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                d[ct][0] = lds_read_tr8<(c & 1) * 4096>(vaddr[0][ct]);
                d[ct][1] = lds_read_tr8<(c & 1) * 4096>(vaddr[1][ct]);
            }
            lds_wait(p0, p1, d[0][0], d[0][1], d[1][0], d[1][1], d[2][0], d[2][1], d[3][0], d[3][1]);
            if (c + 2 < nch) issue(Vh, std::integral_constant<int, c + 2>{});
            v4i aop = {p0.x, p0.y, p1.x, p1.y};
            if (j >= 8) aop = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                const v4i bop = {d[ct][0].x, d[ct][0].y, d[ct][1].x, d[ct][1].y};
                o[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, bop, o[ct], 0, 0, 0);
            }
        }
    });

    // ---- output: 8 x 64 tile through LDS, scaled, 16-byte stores ------------------------------
    vm_wait<0>();
    int *Ol = reinterpret_cast<int *>(stage);
    if (g < 2) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) Ol[(4 * g + r) * (DK + 4) + ct * 16 + j] = o[ct][r];
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int piece = h * 64 + lane, row = piece >> 4, col = (piece & 15) * 4;
        const v4i sres = *reinterpret_cast<const v4i *>(&Ol[row * (DK + 4) + col]);
        const v4f f = {sres.x * a.out_scale, sres.y * a.out_scale, sres.z * a.out_scale, sres.w * a.out_scale};
        *reinterpret_cast<v4f *>(Oh + row * DK + col) = f;
    }
}

} // namespace

int attention_fused_max_vectors() { return 8 * 64; }

hipError_t launch_attention_fused(const AttnArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.heads == 0) return hipSuccess;
    dim3 grid((unsigned)a.P * (unsigned)a.heads), block(64);
    hipLaunchKernelGGL((attention_fused_kernel<8>), grid, block, 0, s, a);
    return hipGetLastError();
}
