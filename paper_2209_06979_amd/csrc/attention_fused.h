// Fused quantized sparse self-attention for gfx950 (paper, Section 5.3): for one head and
// one row panel of the mask ONE WAVEFRONT runs SDDMM -> softmax -> int8 codes -> SpMM with
// the scores, probabilities and codes never leaving registers / LDS.  Latency is hidden by
// keeping a dozen such waves resident per CU, each with chunks of gathered rows in flight.
//
//   phase K  per chunk of 64 mask vectors: the Kmat rows named by the column indices are
//            copied from global memory straight into LDS (global_load_lds, no registers in
//            between); one v_mfma_i32_16x16x64_i8 per 16 vectors and 64 elements of the head
//            dimension gives the scores (head dim 64 = one MFMA, 128 = two; both operands are
//            contiguous along the reduction, Section 4.3).
//            The 8 Q rows sit in MFMA rows 0..7 for even tiles and in rows 8..15 for odd
//            tiles, so two tiles share one accumulator and all 64 lanes carry real scores.
//   softmax  fp32, base 2, over the panel's stored entries: in-lane over the tiles, DPP
//            rotations over the 16 lanes of a row, one cross-lane exchange for the two
//            tile parities; codes = clamp(rint(p / s_p), 0, 127) go to LDS as
//            [slot][8 rows] bytes (one 32-bit write per 4 codes).
//   phase V  SpMM (Section 4.2) per chunk: V rows are copied into the same LDS stages;
//            ds_read_b64_tr_b8 delivers both MFMA operands in place: the codes transposed
//            to [row][16 slots] and the V rows transposed to [column][16 slots].
//   output   the 8 x dk tile goes through LDS once to be stored as fp32 with 16-byte stores.
//
// Two variants (HPW = heads per workgroup):
//   HPW 1  any layout: the wave gathers the rows of its own head (64 bytes; 128 bytes for head
//          dimension 128 with 8-bit inputs) into its one LDS stage (8 KB of LDS per wave and
//          16 waves per CU for 64-byte rows).
//   HPW 2  token-major layout (the heads of a token are contiguous, as a QKV projection
//          writes them): two waves own two neighbouring heads and gather their 128 bytes of
//          a token with ONE request.  The L2 serves a 128-byte line at the cost of a 64-byte
//          half, so this halves the number of gather requests, which is what bounds the
//          kernel.  Each wave copies half of a chunk's rows; one s_barrier per chunk.
// LDS rows are as long as a gathered row (ROWB = HPW times the bytes of one head's row: 32 .. 128);
// slot s of a chunk lives in row (s % NIT) * (64/NIT) + s / NIT (NIT = ROWB/16 copy instructions
// per chunk, so that the column indices a lane needs are consecutive) and its 16-byte segments are
// XOR-swizzled with s % NIT so that rows read together fall into different banks.
#pragma once
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
__device__ __forceinline__ int row16_imax(int v)
{
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x121, 0xF, 0xF, false)); // row_ror:1
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x122, 0xF, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, false));
    v = max(v, __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false));
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

// MAXCH: longest panel in chunks of 64 vectors.  HPW: heads (= waves) per workgroup.
// PB: bits of the re-quantised softmax output.  16 ("16b-8b" layer): the code c <= 32639 is split
// into signed bytes c = 256*hi + lo (Section 4.4); the hi codes feed MFMA rows 0..7 and the lo
// codes rows 8..15 of the same instruction, and the output is (O_hi << 8) + O_lo.
// QB: bits of Q, Kmat and V.  4 ("8b-4b" layer): rows are 32 bytes of packed nibbles.  A nibble is
// widened in registers to an int8 worth 16 x its value (Section 4.4 without an int4 matrix unit):
// the even elements of a 16-byte piece in lane groups 0 and 1, the odd ones in groups 2 and 3, so
// the scores carry a factor 256 and the output a factor 16, removed by exact shifts.
// KS: waves that share one (panel, head) when a panel is longer than MAXCH chunks: wave ks takes
// chunks ks, ks + KS, ...; the waves exchange their row maxima and row sums through LDS and add up
// their partial output tiles at the end (three workgroup barriers in total).  With HPW 2 the
// workgroup has 2 * KS waves: pair ks (one wave per head) gathers its chunks into its own two
// stages, and since the per-chunk barrier is the workgroup's, every wave goes through the chunk
// loops as often as the pair with the most chunks does.
// DK: head dimension, 64 or 128.  Rows of 128 bytes (DK 128, 8-bit inputs) are gathered by one head per
// workgroup only; the 64-byte rows of DK 128 with 4-bit inputs behave like those of DK 64 with 8-bit ones.
// PAD: the head dimension is smaller than DK (any multiple of 16, of 32 for 4-bit inputs): a row has only
// a.real_pieces 16-byte pieces.  The copies of the missing pieces are left out, so the places they would
// land in keep the zeros written once at the start (place p of an LDS row always receives the same piece
// number, see the copy layout below); the Q registers of those pieces are zero as well.  Zero columns add
// nothing to a score and give zero output columns, which are not stored.  One head per workgroup only.
template <int MAXCH, int HPW, int PB, int QB, int KS, int DK, bool PAD = false>
__global__ __launch_bounds__(64 * HPW * KS, (((HPW == 1 && PB == 8 && KS == 1 && DK == 64) || (HPW == 2 && DK == 64 && QB == 8)) ? 4 : (KS == 8 ? 2 : 3)))
void attention_fused_kernel(AttnArgs a)
{
    static_assert(!PAD || HPW == 1, "shorter rows: one head per workgroup");
    static_assert(PB == 8 || PB == 16, "8- or 16-bit codes");
    static_assert(QB == 8 || QB == 4, "Q, K, V are 8-bit or packed 4-bit");
    static_assert(DK == 64 || (DK == 128 && (QB == 4 || HPW == 1)), "rows of 128 bytes: one head per workgroup");
    constexpr int NW = HPW * KS;         // waves per workgroup
    constexpr int PLANE = MAXCH * 512;   // bytes of one plane of codes, [slot][8 rows]
    constexpr int OTILE = (PB == 16 ? 16 : 8) * (DK + 4) * 4;                       // a wave's output tile, staged in the same area
    // HPW 2: the code area holds ONE chunk (codes are written right before they are read) and the
    // output tile is staged in the gather stages, which keeps a workgroup below 20 KB of LDS:
    // eight of them, i.e. all 2048 of a 8 x 4096 layer, are resident at once.
    constexpr bool SMALLP = (HPW == 2);
    constexpr int PSTRIDE = SMALLP ? 512 : PLANE;                                   // from the high to the low plane of the codes
    constexpr int PLB = SMALLP ? 512 * (PB / 8) : ((PLANE * (PB / 8) > OTILE) ? PLANE * (PB / 8) : OTILE); // bytes of that area
    constexpr int DKB = DK * QB / 8; // bytes of one head's row
    constexpr int KK = DK / 64;      // MFMA steps along the head dimension
    constexpr int NO = DK / 16;      // column tiles of the output
    constexpr int NPR = MAXCH * 2;   // pairs of score tiles
    constexpr int ROWB = DKB * HPW;  // bytes of a gathered row
    constexpr int LPR = ROWB / 16;   // lanes per row
    constexpr int NIT = LPR;         // copy instructions per chunk
    constexpr int NITW = DKB / 16;   // ... of which each wave issues this many (4; 2 for nibbles; 8 for head dimension 128)
    constexpr int SWZ = LPR - 1;
    constexpr int NIB = (int)0xF0F0F0F0;
    constexpr int STG = 64 * ROWB;   // bytes of one stage
    constexpr int NST = HPW;         // stages: one for a lone wave, two when two waves share the chunks
    static_assert(!SMALLP || OTILE <= STG, "with two heads per workgroup a wave's output tile is staged in one gather stage");
    __shared__ __attribute__((aligned(16))) char stage_all[NST * STG * KS];  // chunks of gathered rows (KS > 1: one stage per wave)
    __shared__ __attribute__((aligned(16))) char Pl_all[NW * PLB]; // codes, [plane][slot][8 rows], per wave
    __shared__ __attribute__((aligned(8))) char zeros[8];                      // row operand of the MFMA rows that carry no codes
    __shared__ int xch[2][HPW][KS][8];                                        // row maxima / row sums of the KS waves of a head

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = (HPW > 1) ? wave % HPW : 0;  // head within the workgroup
    const int ks = (KS > 1) ? wave / HPW : 0;  // share of the panel's chunks
    char *stage = stage_all + ks * (NST * STG);
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane / LPR, seg = lane % LPR;
    // Workgroups are handed to the 8 XCDs round-robin by linear id.  With id = panel * groups +
    // head group, an XCD only ever sees the head groups congruent to its number, so its L2 has
    // to hold the Kmat and V rows of those heads only.
    const int groups = a.heads / HPW;
    const int hgrp = blockIdx.x % groups;
    const int panel = a.panel_list ? a.panel_list[blockIdx.x / groups] : (int)(blockIdx.x / groups);
    const int head = hgrp * HPW + w;
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    const int nch = (n + MC_CHUNK - 1) / MC_CHUNK;
    const int32_t *idx = a.slot_idx + s0;
    const int64_t goff = (int64_t)hgrp * HPW * a.in_head_stride; // first head of the group
    const int64_t boff = (int64_t)blockIdx.y * a.in_batch_stride; // batch item
    const uint8_t *Kg = a.Km + boff + goff, *Vg = a.Vm + boff + goff;
    float *Oh = a.O + (int64_t)blockIdx.y * a.batch_stride + (int64_t)head * a.head_stride + (int64_t)panel * 8 * a.token_stride;
    char *Pl = Pl_all + wave * PLB;
    const int nloc = (nch > ks) ? (nch - ks + KS - 1) / KS : 0; // chunks of this wave: ks, ks + KS, ...
    // Waves that meet at a workgroup barrier per chunk all make as many passes as the busiest of them
    // (a pass without a chunk of its own is the barrier alone).
    constexpr bool LOCKSTEP = (HPW > 1 && KS > 1);
    const int npass = LOCKSTEP ? (nch + KS - 1) / KS : nloc;
    if (PB == 8 && lane < 2) reinterpret_cast<int *>(zeros)[lane] = 0; // every wave writes the same zeros: no race that matters
    if (PAD) {
        // the places of the pieces a row does not have: zero once, never written again
        for (int i = threadIdx.x; i < NST * STG * KS / 16; i += 64 * NW) reinterpret_cast<v4i *>(stage_all)[i] = (v4i){0, 0, 0, 0};
        __syncthreads(); // (waits for the writes, too: the copies below must land after them)
    }

    // Q rows twice: in MFMA rows 0..7 (q_lo) and in rows 8..15 (q_hi)
    v4i q_lo[KK], q_hi[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const uint8_t *qrow = a.Q + boff + (int64_t)head * a.in_head_stride + (int64_t)(panel * 8 + (j & 7)) * a.in_token_stride;
        v4i qv = {0, 0, 0, 0};
        if (!PAD || (QB == 8 ? 4 * kk + g : 2 * kk + (g & 1)) < a.real_pieces) { // (a piece the row does not have stays zero)
            if (QB == 8) {
                qv = *reinterpret_cast<const v4i *>(qrow + kk * 64 + g * 16);
            } else {
                const v4i raw = *reinterpret_cast<const v4i *>(qrow + kk * 32 + (g & 1) * 16);
                qv = (g < 2) ? ((raw << 4) & NIB) : (raw & NIB);
            }
        }
        q_lo[kk] = (j < 8) ? qv : (v4i){0, 0, 0, 0};
        q_hi[kk] = (j < 8) ? (v4i){0, 0, 0, 0} : qv;
    }
    // Copy instruction i of a chunk: lane (rg, seg) fetches segment seg ^ i of the row in slot
    // rg*NIT + i; it lands in LDS row i*(64/NIT) + rg.  Wave w issues instructions NITW*w .. +NITW-1,
    // whose column indices are consecutive slots: one 128-bit (64-bit) index load per chunk.
    typedef int ixv_t __attribute__((ext_vector_type(NITW)));
    unsigned segoff[NITW];
    bool live[NITW]; // PAD: whether the row has the piece this lane would fetch in instruction i
#pragma unroll
    for (int i = 0; i < NITW; ++i) {
        segoff[i] = (seg ^ ((NITW * w + i) & SWZ)) * 16;
        live[i] = !PAD || (int)(seg ^ ((NITW * w + i) & SWZ)) < a.real_pieces;
    }
    const unsigned stage_u = lds_addr_uniform(stage);  // this wave's stage(s)
    const int32_t *myidx = idx + rg * NIT + NITW * w;
    const unsigned tstride = (unsigned)a.in_token_stride;
    // issue(c): this wave's copies of chunk c into stage c % NST, from the column indices held
    // in ixn; then the indices of the following chunk are requested (an ordinary load that has
    // long arrived by the time they are needed: a vm_wait<0>() lies in between).
    ixv_t ixn = {};
    auto issue = [&](const uint8_t *base, int c) {
#pragma unroll
        for (int i = 0; i < NITW; ++i)
            if (!PAD || live[i])
                copy16_to_lds(base, __umul24(ixn[i], tstride) + segoff[i], stage_u + ((c / KS) % NST) * STG + (NITW * w + i) * 1024);
        ixn = *reinterpret_cast<const ixv_t *>(myidx + ((c + KS < nch) ? c + KS : c) * MC_CHUNK);
    };
    auto start_pipeline = [&](const uint8_t *base) {
        lgkm_wait();                               // no read of the stage is still in flight
        if (HPW > 1) __builtin_amdgcn_s_barrier(); // both waves are done with the stages
        if (nloc > 0) {
            ixn = *reinterpret_cast<const ixv_t *>(myidx + ks * MC_CHUNK);
            issue(base, ks);
        }
    };
    // Makes chunk c readable.  HPW 1: the next chunk is issued by release() once this one has
    // been read.  HPW 2: both halves have landed after the barrier, which also tells that
    // everybody is done reading the pair's previous chunk, so its next chunk can go into the other
    // stage now.  (c may lie beyond the panel's last chunk in a pass of waiting only.)
    auto acquire = [&](const uint8_t *base, int c) {
        vm_wait<0>();
        if (HPW > 1) {
            __builtin_amdgcn_s_barrier();
            if (c + KS < nch) issue(base, c + KS);
        }
    };
    auto release = [&](const uint8_t *base, int c) { // the reads of chunk c have been issued
        if (HPW == 1 && c + KS < nch) {
            lgkm_wait(); // ... and have returned: the one stage may be overwritten
            issue(base, c + KS);
        }
    };

    // ---- phase K: scores; lane (j, g) owns row 4*(g&1) + r of tile 2*pr + (g >> 1) -----
    // The integer scores stay in registers; only the last chunk can hold padded slots, which
    // are kept out of the row sum (and so out of the codes) below.
    // K operand of tile tl: slot s = tl*16 + j sits in LDS row (s % NIT)*(64/NIT) + s/NIT,
    // i.e. byte (j % NIT)*1024 + (j / NIT)*ROWB + tl*256; segment (NITW*w + piece) ^ (j % NIT), where
    // lane group g reads piece 4*kk + g of its head's row in MFMA step kk (8 bit) or piece 2*kk + g % 2
    // (4 bit: even elements of the piece for g < 2, odd elements for g >= 2, as on the Q side)
    const char *kaddr[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
        kaddr[kk] = stage + (j % NIT) * 1024 + (j / NIT) * ROWB + (((NITW * w + (QB == 8 ? 4 * kk + g : 2 * kk + (g & 1))) ^ (j % NIT)) * 16);
    auto kop = [&](v4i raw) -> v4i {
        if (QB == 8) return raw;
        return (g < 2) ? ((raw << 4) & NIB) : (raw & NIB);
    };
    v4i sc[NPR];
    int imax[4] = {INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN};
    const int tail = n - (nch - 1) * MC_CHUNK; // real vectors in the last chunk
    bool keep[2];                               // this lane's slots of the last chunk are real
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) keep[pr] = (2 * pr + (g >> 1)) * 16 + j < tail;
    start_pipeline(Kg);
    // (from here on c counts this wave's chunks; gc is the chunk's number in the panel)
    static_for<MAXCH>([&](auto C) {
        constexpr int c = C, ST = (c % NST) * STG;
        const int gc = ks + c * KS;
        if (c < npass) {
            acquire(Kg, gc);
            if (LOCKSTEP && c >= nloc) return;
            v4i kt[KK][4]; // tiles 0..3 of the chunk
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
#pragma unroll
                for (int tl = 0; tl < 4; ++tl) kt[kk][tl] = *reinterpret_cast<const v4i *>(kaddr[kk] + ST + tl * 256);
            release(Kg, gc);
            sc[2 * c] = (v4i){0, 0, 0, 0};
            sc[2 * c + 1] = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                sc[2 * c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_lo[kk], kop(kt[kk][0]), sc[2 * c], 0, 0, 0);
                sc[2 * c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_hi[kk], kop(kt[kk][1]), sc[2 * c], 0, 0, 0);
                sc[2 * c + 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_lo[kk], kop(kt[kk][2]), sc[2 * c + 1], 0, 0, 0);
                sc[2 * c + 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(q_hi[kk], kop(kt[kk][3]), sc[2 * c + 1], 0, 0, 0);
            }
            if (QB == 4) { // both operands carried a factor 16
                sc[2 * c] = sc[2 * c] >> 8;
                sc[2 * c + 1] = sc[2 * c + 1] >> 8;
            }
            // a padded slot repeats the panel's last real column, so its score duplicates a real
            // one and cannot change the row maximum: no masking here
#pragma unroll
            for (int r = 0; r < 4; ++r) imax[r] = max(imax[r], max(sc[2 * c][r], sc[2 * c + 1][r]));
        }
    });
    // all Kmat rows are consumed: start copying V rows while the softmax runs
    start_pipeline(Vg);

    // ---- softmax over row 4*(g&1) + r, in base 2: exp(x - max) = 2^((s - smax) * scale2) -----
    constexpr float LOG2E = 1.4426950408889634f;
    const float scale2 = a.score_scale * LOG2E;
    float m2[4], srow[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        imax[r] = row16_imax(imax[r]);
        imax[r] = max(imax[r], __shfl_xor(imax[r], 32, 64));
    }
    if (KS > 1) { // row 4*(g&1) + r: lanes 0 and 16 publish, everybody reads all waves
        if (lane == 0 || lane == 16) {
#pragma unroll
            for (int r = 0; r < 4; ++r) xch[0][w][ks][4 * (g & 1) + r] = imax[r];
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int k = 0; k < KS; ++k) imax[r] = max(imax[r], xch[0][w][k][4 * (g & 1) + r]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) m2[r] = (float)imax[r] * scale2;
    float x[NPR][4];
    static_for<MAXCH>([&](auto C) {
        constexpr int c = C;
        if (c < nloc) {
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    x[2 * c + pr][r] = __builtin_amdgcn_exp2f(__builtin_fmaf((float)sc[2 * c + pr][r], scale2, -m2[r]));
            if (ks + c * KS == nch - 1) {
                // the panel's last chunk: padded slots count for nothing.  (The empty statement keeps
                // this a branch taken once per wave instead of selects in every chunk.)
                asm volatile("" ::: "memory");
#pragma unroll
                for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                    for (int r = 0; r < 4; ++r) x[2 * c + pr][r] = keep[pr] ? x[2 * c + pr][r] : 0.f;
            }
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int r = 0; r < 4; ++r) srow[r] += x[2 * c + pr][r];
        }
    });
    float rinv[4]; // p / s_p = e * (1 / (sum * s_p)): one division per row instead of one per entry
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        srow[r] = row16_sum(srow[r]);
        srow[r] += __shfl_xor(srow[r], 32, 64);
    }
    if (KS > 1) { // every wave adds the partial sums in the same order: identical totals everywhere
        if (lane == 0 || lane == 16) {
#pragma unroll
            for (int r = 0; r < 4; ++r) xch[1][w][ks][4 * (g & 1) + r] = __builtin_bit_cast(int, srow[r]);
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            srow[r] = 0.f;
#pragma unroll
            for (int k = 0; k < KS; ++k) srow[r] += __builtin_bit_cast(float, xch[1][w][k][4 * (g & 1) + r]);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) rinv[r] = a.inv_s_p / srow[r];
    // ---- phase V: O = codes * V ------------------------------------------------------------------
    v4i o[NO];
#pragma unroll
    for (int ct = 0; ct < NO; ++ct) o[ct] = (v4i){0, 0, 0, 0};
    const int src = lane & 15, ii = src >> 1;
    int vbase[2];
    const char *paddr[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int s = g * 16 + 8 * h + ii;   // slot within the chunk supplied by this lane
        const int i = s % NIT, r = s / NIT;
        vbase[h] = i * 1024 + r * ROWB + (((NITW * w) ^ i) * 16) + 8 * (src & 1);
        // lanes 2t and 2t+1 supply the 8-byte pieces that end up in MFMA rows 0..7 and 8..15: the
        // codes and 8 zero bytes (PB 8), or the high and the low plane of the codes (PB 16)
        if (PB == 16) paddr[h] = Pl + s * 8 + (src & 1) * PSTRIDE;
        else paddr[h] = (src & 1) ? zeros : Pl + s * 8;
    }
    static_for<MAXCH>([&](auto C) {
        constexpr int c = C;
        const int gc = ks + c * KS;
        if (LOCKSTEP && c >= nloc) { // a pass of waiting only
            if (c < npass) acquire(Vg, gc);
            return;
        }
        if (c < nloc) {
            // Codes of this chunk's slots (tile*16 + j), rows 4*(g&1) .. +3: one 32-bit LDS write
            // per tile.  v_cvt_pk_u8_f32 rounds to nearest even and drops the byte into place; the
            // largest code is 127 (p / s_p exceeds it when s_p < 1/127), hence the minimum.
            // Done here, chunk by chunk, so that this ALU work overlaps the V copies in flight.
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                const int slot = (SMALLP ? 0 : c * MC_CHUNK) + (2 * pr + (g >> 1)) * 16 + j;
                if (PB == 8) {
                    unsigned packed = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) packed = __builtin_amdgcn_cvt_pk_u8_f32(fminf(x[2 * c + pr][r] * rinv[r], 127.f), r, packed);
                    *reinterpret_cast<unsigned *>(Pl + slot * 8 + 4 * (g & 1)) = packed;
                } else {
                    // code = clamp(rint(e * rinv), 0, 32639) (ties to even), hi = (code + 128) >> 8 in
                    // [0, 127], lo = code - 256 * hi in [-128, 127]: its low byte as it is
                    unsigned hi = 0, lo = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int code = (int)__builtin_rintf(fminf(x[2 * c + pr][r] * rinv[r], 32639.f));
                        hi |= (unsigned)((code + 128) >> 8) << (8 * r);
                        lo |= (unsigned)(code & 255) << (8 * r);
                    }
                    *reinterpret_cast<unsigned *>(Pl + slot * 8 + 4 * (g & 1)) = hi;
                    *reinterpret_cast<unsigned *>(Pl + PSTRIDE + slot * 8 + 4 * (g & 1)) = lo;
                }
            }
            acquire(Vg, gc);
            // the codes, transposed to the MFMA row operand: row j < 8, slots g*16 .. +15
            const int pstep = (SMALLP || (PB == 8 && (src & 1))) ? 0 : c * 512; // the zero bytes do not move
            const v2i p0 = lds_read_tr8(paddr[0] + pstep), p1 = lds_read_tr8(paddr[1] + pstep);
            v2i d[NITW][2];
#pragma unroll
            for (int ct = 0; ct < NITW; ++ct) {
                d[ct][0] = lds_read_tr8(stage + (c % NST) * STG + (vbase[0] ^ (ct * 16)));
                d[ct][1] = lds_read_tr8(stage + (c % NST) * STG + (vbase[1] ^ (ct * 16)));
            }
            release(Vg, gc);
            const v4i aop = {p0.x, p0.y, p1.x, p1.y};
#pragma unroll
            for (int ct = 0; ct < NITW; ++ct) {
                const v4i bop = {d[ct][0].x, d[ct][0].y, d[ct][1].x, d[ct][1].y};
                if (QB == 8) {
                    o[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, bop, o[ct], 0, 0, 0);
                } else { // byte j of the piece holds columns 32*ct + 2j (low nibble) and 2j + 1 (high nibble)
                    const v4i msk = {NIB, NIB, NIB, NIB};
                    o[2 * ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, (bop << 4) & msk, o[2 * ct], 0, 0, 0);
                    o[2 * ct + 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop, bop & msk, o[2 * ct + 1], 0, 0, 0);
                }
            }
        }
    });

    // ---- output: 8 x DK tile through this wave's code area, scaled, 16-byte stores -------------
    vm_wait<0>();
    if (SMALLP) {
        lgkm_wait();
        __builtin_amdgcn_s_barrier(); // nobody reads the stages any more: each wave takes one for its tile
    }
    int *Ol = reinterpret_cast<int *>(SMALLP ? stage_all + (ks * NST + w) * STG : Pl); // SMALLP: NST == HPW stages per pair
    if (g < 2 || PB == 16) {
#pragma unroll
        for (int ct = 0; ct < NO; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // the nibble products carry a factor 16; each plane's sum is shifted on its own
                if (QB == 8) Ol[(4 * g + r) * (DK + 4) + ct * 16 + j] = o[ct][r];
                else Ol[(4 * g + r) * (DK + 4) + (ct >> 1) * 32 + 2 * j + (ct & 1)] = o[ct][r] >> 4;
            }
    }
    lgkm_wait();
    if (KS > 1) __syncthreads(); else __builtin_amdgcn_wave_barrier();
    // the tile of wave k of this wave's head, and this thread's number among the 64 * KS threads of the head
    auto partial_tile = [&](int k) -> const int * {
        return reinterpret_cast<const int *>(SMALLP ? stage_all + (k * NST + w) * STG : Pl_all + k * PLB);
    };
    const int tih = ks * 64 + lane;
    if (a.out_f16) {
        // fp16: 8 rows x DK/8 pieces of 8 columns, one 16-byte store each
#pragma unroll
        for (int h = 0; h < (DK + 64 * KS - 1) / (64 * KS); ++h) {
            const int piece = tih + h * 64 * KS;
            if (piece >= DK) continue;
            const int row = piece / (DK / 8), col = (piece % (DK / 8)) * 8;
            if (PAD && col >= a.out_cols) continue;
            v4h hv[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                v4i sres = {0, 0, 0, 0}, slo = {0, 0, 0, 0};
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    const int *Ok = (KS > 1) ? partial_tile(k) : Ol;
                    sres += *reinterpret_cast<const v4i *>(&Ok[row * (DK + 4) + col + 4 * q]);
                    if (PB == 16) slo += *reinterpret_cast<const v4i *>(&Ok[(row + 8) * (DK + 4) + col + 4 * q]);
                }
                if (PB == 16) sres = (sres << 8) + slo;
                hv[q] = to_half4((v4f){sres.x * a.out_scale, sres.y * a.out_scale, sres.z * a.out_scale, sres.w * a.out_scale});
            }
            typedef _Float16 v8h __attribute__((ext_vector_type(8)));
            const int64_t off = (Oh - a.O) + (int64_t)row * a.token_stride + col;
            __builtin_nontemporal_store((v8h){hv[0].x, hv[0].y, hv[0].z, hv[0].w, hv[1].x, hv[1].y, hv[1].z, hv[1].w},
                                        reinterpret_cast<v8h *>(reinterpret_cast<_Float16 *>(a.O) + off));
        }
        return;
    }
    // 8 rows x DK/4 pieces of 4 columns; with KS waves all threads share the adding up of the partial tiles
#pragma unroll
    for (int h = 0; h < (2 * DK + 64 * KS - 1) / (64 * KS); ++h) {
        const int piece = tih + h * 64 * KS;
        if (piece >= 2 * DK) continue;
        const int row = piece / (DK / 4), col = (piece % (DK / 4)) * 4;
        if (PAD && col >= a.out_cols) continue;
        v4i sres = {0, 0, 0, 0}, slo = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            const int *Ok = (KS > 1) ? partial_tile(k) : Ol;
            sres += *reinterpret_cast<const v4i *>(&Ok[row * (DK + 4) + col]);
            if (PB == 16) slo += *reinterpret_cast<const v4i *>(&Ok[(row + 8) * (DK + 4) + col]);
        }
        if (PB == 16) sres = (sres << 8) + slo;
        const v4f f = {sres.x * a.out_scale, sres.y * a.out_scale, sres.z * a.out_scale, sres.w * a.out_scale};
        __builtin_nontemporal_store(f, reinterpret_cast<v4f *>(Oh + (int64_t)row * a.token_stride + col));
    }
}


} // namespace
