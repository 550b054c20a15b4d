// SDDMM and value-repack kernels for gfx950 (the sparse softmax lives in softmax_kernels.hip).
//
// SDDMM (paper, Section 4.3): a workgroup owns one row panel of the mask.  The panel's
// V rows of Q are the row operand of v_mfma_i32_16x16x64_i8 and stay in registers for
// the whole panel (the paper keeps this block in shared memory for its warps); the rows
// of Kmat named by 16 consecutive mask vectors are the column operand.  Both operands
// are contiguous along the reduction dimension, so no transpose is needed
// (Section 4.3.1): lane group g = lane/16 covers bytes 64*kc + 16*g .. +15 of a row on
// both sides.  The waves of a workgroup take the panel's chunks of 64 vectors round-robin
// and never have to meet: every chunk produces its own outputs.
// Two kernels:
//   sddmm_lds_kernel   rows of 64, 128, 256, 512 or 1024 bytes (sddmm_nib32_kernel: 32 bytes of nibbles): the 64 Kmat rows of a chunk are copied
//                      from global memory straight into LDS with coalesced 16-byte pieces
//                      (global_load_lds), then read as 128-bit MFMA operands; the
//                      16-byte segments are XOR-swizzled against bank conflicts.  Rows longer
//                      than 256 bytes pass through the stage 256 bytes at a time.
//   sddmm_direct_kernel any row length: each lane loads its 16 operand bytes from memory.
// int4 operands are widened in registers; int16 operands (L16-R16, Section 4.4) are split in
// registers into signed byte planes, the two Q planes stacked in the MFMA rows 0..7 / 8..15.
// The output is written in interchange (BCRS) order: V consecutive int32 per vector, or with the
// fused dequantisation of Section 5.3 V consecutive fp32 / fp16 values.
#include "internal.h"

#include "sddmm_tile.h"

namespace {

using namespace mcs;


// four fp32 values rounded to fp16 (to nearest even; beyond the fp16 range: infinity)
__device__ __forceinline__ v4h to_half4(v4f f) { return (v4h){(_Float16)f.x, (_Float16)f.y, (_Float16)f.z, (_Float16)f.w}; }

// DQ: fused dequantisation (Section 5.3).  A compile-time switch: the integer path keeps its
// straight-line stores, which the scheduler interleaves with the next tile's MFMAs.
// float_out 3 (only with DQ): the scores leave as integer codes clamp(rint(score * out_scale)) of 8 or 16 bits,
// written into the device panel format of a sparse operand with the mask's pattern (Section 4.3: the
// SDDMM writes the format the following SpMM reads); padded slots receive zeros.  s0: first slot of the panel.
template <bool DQ>
__device__ __forceinline__ void store_scores(const SddmmArgs &a, int64_t out0, int s0, int slot, int n, int g, v4i acc)
{
    if (DQ && a.float_out == 3) {
        if (4 * g >= a.V) return;
        const int64_t gs = (int64_t)s0 + slot;                 // slot of the whole matrix
        const int sub = (int)(gs % MC_CHUNK) / 16, b = (int)(gs % 16);
        const float qmax = (a.code_bits == 16) ? 32639.f : 127.f;
        uint8_t *chunk = a.dev_vals + (int64_t)blockIdx.y * a.dev_batch_stride + (gs / MC_CHUNK) * (MC_CHUNK * a.V * a.code_bits / 8);
        const int nr = a.V - 4 * g < 4 ? a.V - 4 * g : 4;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (r >= nr) break;
            // one fp32 product, rounded to nearest even, then clamped: the same arithmetic as the oracle's
            const float x = __builtin_rintf((float)acc[r] * a.out_scale);
            const int code = (slot < n) ? (int)__builtin_fminf(__builtin_fmaxf(x, -qmax), qmax) : 0;
            const int v = 4 * g + r;
            if (a.code_bits == 8) {
                chunk[sub * (16 * a.V) + v * 16 + b] = (uint8_t)code;
            } else {
                const int hi = (code + 128) >> 8, lo = code - hi * 256;   // two signed bytes: code = 256 * hi + lo
                chunk[sub * (32 * a.V) + v * 16 + b] = (uint8_t)hi;
                chunk[sub * (32 * a.V) + 16 * a.V + v * 16 + b] = (uint8_t)lo;
            }
        }
        return;
    }
    // accumulator register r of lane (j, g) is row 4g + r of vector `slot`
    if (slot < n && 4 * g < a.V) {
        const int64_t off = out0 + (int64_t)slot * a.V + 4 * g;
        if (!DQ) {
            int32_t *o = static_cast<int32_t *>(a.S) + off;
            if (a.V >= 4) __builtin_nontemporal_store(acc, reinterpret_cast<v4i *>(o));
            else __builtin_nontemporal_store((v2i){acc.x, acc.y}, reinterpret_cast<v2i *>(o));
        } else {
            const v4f f = {acc.x * a.out_scale, acc.y * a.out_scale, acc.z * a.out_scale, acc.w * a.out_scale};
            if (a.float_out == 1) {
                float *o = static_cast<float *>(a.S) + off;
                if (a.V >= 4) __builtin_nontemporal_store(f, reinterpret_cast<v4f *>(o));
                else { o[0] = f.x; o[1] = f.y; }
            } else {
                _Float16 *o = static_cast<_Float16 *>(a.S) + off;
                const v4h h = to_half4(f);
                if (a.V >= 4) __builtin_nontemporal_store(h, reinterpret_cast<v4h *>(o));
                else *reinterpret_cast<v2h *>(o) = (v2h){h.x, h.y};
            }
        }
    }
}


// RB: bytes of a Kmat row staged per pass (64, 128, 256, 512; 16-bit operands: from 128); SEGS: passes
// per chunk, a row has RB * SEGS bytes (the tiles' accumulators live across the passes, so long
// rows need no more LDS than short ones).  WK: waves per workgroup.
// U: 8- or 4-bit operands of which one or both are read as non-negative values (Section 4.4.1); the
// scheme is the one described at sddmm_unsigned_kernel below, here on rows staged in LDS.
template <int PB, int RB, int SEGS, int WK, bool DQ, bool U>
__global__ __launch_bounds__(64 * WK) void sddmm_lds_kernel(SddmmArgs a)
{
    constexpr int LPR = RB / 16, NI = LPR, RPI = 64 / LPR, KC = RB / StepBytes<PB>::value;
    static_assert(KC >= 1, "a row must fill at least one MFMA step");
    static_assert(!U || PB == 8 || PB == 4, "unsigned operands: 4 and 8 bits");
    constexpr int QR = (U && PB == 4) ? 2 : 1; // registers per step of the Q operand (unsigned nibbles are widened once, up front)
    __shared__ __attribute__((aligned(16))) char lds[WK * 64 * RB];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane / LPR, seg = lane % LPR;
    const int batch = blockIdx.y;
    // a unit of work: a whole panel, or (masks with very unequal panels) a range of its chunks
    int panel = blockIdx.x, cb = 0, ce = -1;
    if (a.items) {
        const v4i it = *reinterpret_cast<const v4i *>(a.items + 4 * blockIdx.x);
        panel = it.x; cb = it.y; ce = it.z;
    }
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    if (ce < 0) ce = (n + MC_CHUNK - 1) / MC_CHUNK;
    const int nch = ce - cb;
    const int32_t *idx = a.slot_idx + s0 + cb * MC_CHUNK;
    const int64_t out0 = (int64_t)batch * a.S_batch_stride + (int64_t)a.row_ptr[panel] * a.V;
    const uint8_t *Km = a.Kmat + (int64_t)batch * a.K_batch_stride;
    char *stage = lds + w * (64 * RB);

    v4i qf[KC * SEGS * QR];
    const uint8_t *Qpanel = a.Q + (int64_t)batch * a.Q_batch_stride + (int64_t)panel * a.V * a.ldq_bytes;
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const v4i nib = {NIBBLE_HI, NIBBLE_HI, NIBBLE_HI, NIBBLE_HI};
    const int qx1 = (U && a.lhs_unsigned) ? (int)0x80808080 : 0, kx1 = (U && a.rhs_unsigned) ? (int)0x80808080 : 0;
    const v4i qx = {qx1, qx1, qx1, qx1}, kx = {kx1, kx1, kx1, kx1};
    v4i rq = {0, 0, 0, 0}; // U: rows 4g .. 4g+3: sum over the reduction of the Q operand bytes
#pragma unroll
    for (int kc = 0; kc < KC * SEGS; ++kc) {
        const v4i raw = load_q<PB>(Qpanel, a.ldq_bytes, a.V, RB * SEGS, kc, j, g);
        if (!U) {
            qf[kc] = raw;
        } else {
            // rows of the panel: the operand bytes; MFMA row 8: all ones (it collects the sums of the Kmat
            // operand bytes of every output column); other rows: zero
#pragma unroll
            for (int t = 0; t < QR; ++t) {
                v4i q = (PB == 8) ? (raw ^ qx) : (((t == 0 ? (raw << 4) : raw) & nib) ^ qx);
                if (j >= a.V) q = (j == 8) ? ones : (v4i){0, 0, 0, 0};
                qf[kc * QR + t] = q;
                rq = __builtin_amdgcn_mfma_i32_16x16x64_i8(q, ones, rq, 0, 0, 0);
            }
        }
    }
    const int nred = RB * SEGS * (PB == 4 ? 2 : 1);                      // reduction elements
    const int cqck = (U && a.lhs_unsigned && a.rhs_unsigned) ? (PB == 4 ? 64 : 16384) * nred : 0;
    // load instruction i: lane (rg, seg) copies segment seg ^ i of the row (piece) in slot rg*NI + i
    // to LDS row i*RPI + rg (byte i*1024 + lane*16 of the stage)
    const int nmy = (nch > w) ? (nch - w + WK - 1) / WK : 0;
    v4i idxv[NI / 4];
    auto load_idx = [&](int c) {
#pragma unroll
        for (int t = 0; t < NI / 4; ++t) idxv[t] = *reinterpret_cast<const v4i *>(idx + c * MC_CHUNK + rg * NI + 4 * t);
    };
    if (nmy > 0) load_idx(w);
    for (int k = 0; k < nmy; ++k) {
        const int c = w + k * WK;
        v4i acc[4], acc2[4];
#pragma unroll
        for (int h = 0; h < SEGS; ++h) {
            if (h > 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // the previous pass has been read
            // (the column indices of this chunk are still needed by the later passes: the next
            // chunk's may only be requested after the last pass has issued its copies)
#pragma unroll
            for (int i = 0; i < NI; ++i)
                __builtin_amdgcn_global_load_lds((gptr_t *)(Km + (int64_t)idxv[i >> 2][i & 3] * a.ldk_bytes + h * RB + ((seg ^ i) * 16)),
                                                 (lptr_t *)(stage + i * 1024), 16, 0, 0);
            const bool more = (h == SEGS - 1) && (k + 1 < nmy);
            if (more) load_idx(c + WK);
            if (more) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NI / 4) : "memory"); // rows landed, indices may still fly
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int tl = 0; tl < 4; ++tl) {
                const int s = tl * 16 + j;              // slot within the chunk
                const int i = s % NI, r = s / NI;       // its load instruction and row group
                const char *rowp = stage + i * 1024 + r * RB;
                if (h == 0) acc[tl] = acc2[tl] = (v4i){0, 0, 0, 0};
#pragma unroll
                for (int kc = 0; kc < KC; ++kc) {
                    if (PB == 16) {
                        const v4i x = *reinterpret_cast<const v4i *>(rowp + (((kc * 8 + 2 * g) ^ i) * 16));
                        const v4i y = *reinterpret_cast<const v4i *>(rowp + (((kc * 8 + 2 * g + 1) ^ i) * 16));
                        v4i kh, kl;
                        split16(x, y, kh, kl);
                        mma_step<PB>(qf[h * KC + kc], kh, kl, acc[tl], acc2[tl]);
                    } else {
                        const v4i kf = *reinterpret_cast<const v4i *>(rowp + (((kc * 4 + g) ^ i) * 16));
                        if (!U) {
                            mma_step<PB>(qf[h * KC + kc], kf, kf, acc[tl], acc2[tl]);
                        } else if (PB == 8) {
                            acc[tl] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qf[h * KC + kc], kf ^ kx, acc[tl], 0, 0, 0);
                        } else {
                            acc[tl] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qf[(h * KC + kc) * 2], ((kf << 4) & nib) ^ kx, acc[tl], 0, 0, 0);
                            acc[tl] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qf[(h * KC + kc) * 2 + 1], (kf & nib) ^ kx, acc[tl], 0, 0, 0);
                        }
                    }
                }
                if (h == SEGS - 1) {
                    if (!U) {
                        store_scores<DQ>(a, out0, s0, (cb + c) * MC_CHUNK + s, n, g, finish_tile<PB>(acc[tl], acc2[tl]));
                    } else {
                        // sum (q'+cq)(k'+ck) = sum q'k' + ck sum q' + cq sum k' + cq ck n, with cq = ck = 128 in the
                        // scale the operand bytes carry (nibbles: 16 x their value)
                        v4i r = acc[tl];
                        const int cs = __shfl(r[0], 32 + j); // MFMA row 8 (lane group 2, register 0) of this lane's column
                        if (a.rhs_unsigned) r += rq << 7;
                        if (a.lhs_unsigned) r += (v4i){cs << 7, cs << 7, cs << 7, cs << 7};
                        if (PB == 4) r = r >> 8;
                        r += (v4i){cqck, cqck, cqck, cqck};
                        store_scores<DQ>(a, out0, s0, (cb + c) * MC_CHUNK + s, n, g, r);
                    }
                }
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // reads done before the rows are overwritten
    }
}

// Rows of 32 bytes of packed nibbles (Kd = 64 with 4-bit operands): one MFMA step per tile.  The 64
// reduction elements of a row fill the step exactly when lane groups 0 and 1 take the even elements
// of the two 16-byte pieces (low nibbles, shifted up) and groups 2 and 3 the odd ones (high nibbles),
// on both operand sides: sums do not depend on the order of their terms.  Both operands carry a
// factor 16.  Staging as in sddmm_lds_kernel: copy instruction i (of 2) brings the rows of the
// slots 2*rg + i, rg = lane / 2, into LDS rows i*32 + rg, pieces XOR-swizzled with i.
template <int WK, bool DQ, bool U>
__global__ __launch_bounds__(64 * WK) void sddmm_nib32_kernel(SddmmArgs a)
{
    constexpr int RB = 32;
    __shared__ __attribute__((aligned(16))) char lds[WK * 64 * RB];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane >> 1, seg = lane & 1;
    const int batch = blockIdx.y;
    int panel = blockIdx.x, cb = 0, ce = -1;
    if (a.items) {
        const v4i it = *reinterpret_cast<const v4i *>(a.items + 4 * blockIdx.x);
        panel = it.x; cb = it.y; ce = it.z;
    }
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    if (ce < 0) ce = (n + MC_CHUNK - 1) / MC_CHUNK;
    const int nch = ce - cb;
    const int32_t *idx = a.slot_idx + s0 + cb * MC_CHUNK;
    const int64_t out0 = (int64_t)batch * a.S_batch_stride + (int64_t)a.row_ptr[panel] * a.V;
    const uint8_t *Km = a.Kmat + (int64_t)batch * a.K_batch_stride;
    char *stage = lds + w * (64 * RB);

    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const v4i nib = {NIBBLE_HI, NIBBLE_HI, NIBBLE_HI, NIBBLE_HI};
    const int qx1 = (U && a.lhs_unsigned) ? (int)0x80808080 : 0, kx1 = (U && a.rhs_unsigned) ? (int)0x80808080 : 0;
    const v4i qx = {qx1, qx1, qx1, qx1}, kx = {kx1, kx1, kx1, kx1};
    // this lane's operand from 16 raw bytes: even elements (groups 0, 1) or odd elements (groups 2, 3)
    auto widen = [&](v4i raw) -> v4i { return ((g < 2) ? (raw << 4) : raw) & nib; };

    v4i qop = {0, 0, 0, 0};
    if (j < a.V) {
        const uint8_t *qrow = a.Q + (int64_t)batch * a.Q_batch_stride + (int64_t)(panel * a.V + j) * a.ldq_bytes;
        qop = widen(*reinterpret_cast<const v4i *>(qrow + (g & 1) * 16)) ^ qx;
    } else if (U && j == 8) {
        qop = ones; // MFMA row 8 collects the sums of the Kmat operand bytes of every output column
    }
    v4i rq = {0, 0, 0, 0}; // U: rows 4g .. 4g+3: sum over the reduction of the Q operand bytes
    if (U) rq = __builtin_amdgcn_mfma_i32_16x16x64_i8(qop, ones, rq, 0, 0, 0);
    const int cqck = (U && a.lhs_unsigned && a.rhs_unsigned) ? 64 * 64 : 0; // cq * ck per element, 64 elements

    const int nmy = (nch > w) ? (nch - w + WK - 1) / WK : 0;
    v2i idxv = {0, 0};
    if (nmy > 0) idxv = *reinterpret_cast<const v2i *>(idx + w * MC_CHUNK + rg * 2);
    for (int k = 0; k < nmy; ++k) {
        const int c = w + k * WK;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t *)(Km + (int64_t)idxv[i] * a.ldk_bytes + ((seg ^ i) * 16)),
                                             (lptr_t *)(stage + i * 1024), 16, 0, 0);
        if (k + 1 < nmy) {
            idxv = *reinterpret_cast<const v2i *>(idx + (c + WK) * MC_CHUNK + rg * 2);
            asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); // rows landed, indices may still fly
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
#pragma unroll
        for (int tl = 0; tl < 4; ++tl) {
            const int s = tl * 16 + j;              // slot within the chunk
            const int i = s & 1, r = s >> 1;        // its copy instruction and row group
            const v4i kf = *reinterpret_cast<const v4i *>(stage + i * 1024 + r * RB + (((g & 1) ^ i) * 16));
            v4i acc = {0, 0, 0, 0};
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(qop, widen(kf) ^ kx, acc, 0, 0, 0);
            if (U) {
                const int cs = __shfl(acc[0], 32 + j); // MFMA row 8 (lane group 2, register 0) of this lane's column
                if (a.rhs_unsigned) acc += rq << 7;
                if (a.lhs_unsigned) acc += (v4i){cs << 7, cs << 7, cs << 7, cs << 7};
            }
            acc = acc >> 8; // both operands carried a factor 16
            if (U) acc += (v4i){cqck, cqck, cqck, cqck};
            store_scores<DQ>(a, out0, s0, (cb + c) * MC_CHUNK + s, n, g, acc);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // reads done before the rows are overwritten
    }
}

// KC = number of MFMA steps along a row kept in registers (0: any length, Q re-read).
template <int PB, int KC, bool DQ>
__global__ __launch_bounds__(64 * SDDMM_WAVES) void sddmm_direct_kernel(SddmmArgs a)
{
    constexpr int STEP = StepBytes<PB>::value, LANEB = STEP / 4; // bytes per step / per lane and step
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int batch = blockIdx.y;
    int panel = blockIdx.x, cb = 0, ce = -1; // unit of work: a panel or a range of its chunks
    if (a.items) {
        const v4i it = *reinterpret_cast<const v4i *>(a.items + 4 * blockIdx.x);
        panel = it.x; cb = it.y; ce = it.z;
    }
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    // (codes written into an operand's device format also cover the padded slots of the last chunk, with zeros)
    const int tiles_all = (DQ && a.float_out == 3) ? (n + MC_CHUNK - 1) / MC_CHUNK * 4 : (n + 15) / 16;
    const int tile0 = 4 * cb, ntile = (ce < 0) ? tiles_all : min(tiles_all, 4 * ce);
    const int64_t out0 = (int64_t)batch * a.S_batch_stride + (int64_t)a.row_ptr[panel] * a.V;
    const uint8_t *Qpanel = a.Q + (int64_t)batch * a.Q_batch_stride + (int64_t)panel * a.V * a.ldq_bytes;
    const uint8_t *Km = a.Kmat + (int64_t)batch * a.K_batch_stride + g * LANEB;
    const int kc_n = (a.row_bytes + STEP - 1) / STEP;

    // this lane's piece of step kc of a Kmat row: (k, k2) = the operand (8 / 4 bit) or its planes
    auto load_k = [&](const uint8_t *kr, int kc, v4i &k, v4i &k2) {
        k = k2 = (v4i){0, 0, 0, 0};
        const int off = kc * STEP + g * LANEB;
        if (off < a.row_bytes) {
            const v4i x = *reinterpret_cast<const v4i *>(kr + kc * STEP);
            if (PB == 16) {
                v4i y = {0, 0, 0, 0};
                if (off + 16 < a.row_bytes) y = *reinterpret_cast<const v4i *>(kr + kc * STEP + 16);
                split16(x, y, k, k2);
            } else {
                k = x;
            }
        }
    };

    v4i qf[KC > 0 ? KC : 1];
    if (KC > 0) {
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[kc] = load_q<PB>(Qpanel, a.ldq_bytes, a.V, a.row_bytes, kc, j, g);
    }

    for (int t = tile0 + w; t < ntile; t += SDDMM_WAVES) {
        const int slot = t * 16 + j;
        const int row = a.slot_idx[s0 + slot]; // padded slots name a valid row
        const uint8_t *kr = Km + (int64_t)row * a.ldk_bytes;
        v4i acc = {0, 0, 0, 0}, acc2 = {0, 0, 0, 0};
        if (KC > 0) {
            v4i kf[KC > 0 ? KC : 1], kf2[KC > 0 ? KC : 1];
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) load_k(kr, kc, kf[kc], kf2[kc]);
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) mma_step<PB>(qf[kc], kf[kc], kf2[kc], acc, acc2);
        } else {
            for (int kc = 0; kc < kc_n; ++kc) {
                v4i k, k2;
                load_k(kr, kc, k, k2);
                const v4i q = load_q<PB>(Qpanel, a.ldq_bytes, a.V, a.row_bytes, kc, j, g);
                mma_step<PB>(q, k, k2, acc, acc2);
            }
        }
        store_scores<DQ>(a, out0, s0, slot, n, g, finish_tile<PB>(acc, acc2));
    }
}

// ---- unsigned 8- and 4-bit operands (Section 4.4.1), any row length ---------------------------
// The signed MFMA takes an unsigned value u as u - c (c = 128, or 8 for a nibble: one XOR of the
// top bit of the operand byte); sum (q'+cq)(k'+ck) = sum q'k' + ck sum q' + cq sum k' + cq ck n.
// sum q' per Q row comes from an MFMA against an all-ones column operand (once per wave), sum k'
// per gathered Kmat row from MFMA row 8, which is free (V <= 8) and is fed an all-ones row operand.
// Reduction bytes beyond the row end are zero on both sides before the XOR, so they take part in
// every term consistently and n counts them.
template <int PB, bool DQ>
__global__ __launch_bounds__(64 * SDDMM_WAVES) void sddmm_unsigned_kernel(SddmmArgs a)
{
    static_assert(PB == 8 || PB == 4, "unsigned operands: 4 and 8 bits");
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int batch = blockIdx.y;
    int panel = blockIdx.x, cb = 0, ce = -1; // unit of work: a panel or a range of its chunks
    if (a.items) {
        const v4i it = *reinterpret_cast<const v4i *>(a.items + 4 * blockIdx.x);
        panel = it.x; cb = it.y; ce = it.z;
    }
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    // (codes written into an operand's device format also cover the padded slots of the last chunk, with zeros)
    const int tiles_all = (DQ && a.float_out == 3) ? (n + MC_CHUNK - 1) / MC_CHUNK * 4 : (n + 15) / 16;
    const int tile0 = 4 * cb, ntile = (ce < 0) ? tiles_all : min(tiles_all, 4 * ce);
    const int64_t out0 = (int64_t)batch * a.S_batch_stride + (int64_t)a.row_ptr[panel] * a.V;
    const uint8_t *Qrow = a.Q + (int64_t)batch * a.Q_batch_stride + (int64_t)(panel * a.V + (j < a.V ? j : 0)) * a.ldq_bytes + g * 16;
    const uint8_t *Km = a.Kmat + (int64_t)batch * a.K_batch_stride + g * 16;
    const int kc_n = (a.row_bytes + 63) / 64;
    const int qx = a.lhs_unsigned ? (int)0x80808080 : 0, kx = a.rhs_unsigned ? (int)0x80808080 : 0;
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const v4i nib = {NIBBLE_HI, NIBBLE_HI, NIBBLE_HI, NIBBLE_HI};

    // operands of step kc: (q0, q1) row operands and (k0, k1) column operands; 8 bit uses the first of each
    auto q_ops = [&](int kc, v4i &q0, v4i &q1) {
        v4i raw = {0, 0, 0, 0};
        if (kc * 64 + g * 16 < a.row_bytes) raw = *reinterpret_cast<const v4i *>(Qrow + kc * 64);
        const v4i x = {qx, qx, qx, qx};
        if (PB == 8) { q0 = raw ^ x; q1 = q0; }
        else { q0 = ((raw << 4) & nib) ^ x; q1 = (raw & nib) ^ x; }
        if (j >= a.V) q0 = q1 = (j == 8) ? ones : (v4i){0, 0, 0, 0};
    };
    auto k_ops = [&](const uint8_t *kr, int kc, v4i &k0, v4i &k1) {
        v4i raw = {0, 0, 0, 0};
        if (kc * 64 + g * 16 < a.row_bytes) raw = *reinterpret_cast<const v4i *>(kr + kc * 64);
        const v4i x = {kx, kx, kx, kx};
        if (PB == 8) { k0 = raw ^ x; k1 = k0; }
        else { k0 = ((raw << 4) & nib) ^ x; k1 = (raw & nib) ^ x; }
    };

    v4i rq = {0, 0, 0, 0}; // rows 4g .. 4g+3: sum over the reduction of the Q operand bytes
    for (int kc = 0; kc < kc_n; ++kc) {
        v4i q0, q1;
        q_ops(kc, q0, q1);
        rq = __builtin_amdgcn_mfma_i32_16x16x64_i8(q0, ones, rq, 0, 0, 0);
        if (PB == 4) rq = __builtin_amdgcn_mfma_i32_16x16x64_i8(q1, ones, rq, 0, 0, 0);
    }
    const int nred = kc_n * (PB == 4 ? 128 : 64);                       // reduction elements, padding included
    const int cqck = (a.lhs_unsigned && a.rhs_unsigned) ? (PB == 4 ? 64 : 16384) * nred : 0;

    for (int t = tile0 + w; t < ntile; t += SDDMM_WAVES) {
        const int slot = t * 16 + j;
        const int row = a.slot_idx[s0 + slot]; // padded slots name a valid row
        const uint8_t *kr = Km + (int64_t)row * a.ldk_bytes;
        v4i acc = {0, 0, 0, 0};
        for (int kc = 0; kc < kc_n; ++kc) {
            v4i q0, q1, k0, k1;
            q_ops(kc, q0, q1);
            k_ops(kr, kc, k0, k1);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q0, k0, acc, 0, 0, 0);
            if (PB == 4) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q1, k1, acc, 0, 0, 0);
        }
        const int cs = __shfl(acc[0], 32 + j); // MFMA row 8 (lane group 2, register 0) of this lane's column
        if (a.rhs_unsigned) acc += rq << 7;
        if (a.lhs_unsigned) acc += (v4i){cs << 7, cs << 7, cs << 7, cs << 7};
        if (PB == 4) acc = acc >> 8;
        acc += (v4i){cqck, cqck, cqck, cqck};
        store_scores<DQ>(a, out0, s0, slot, n, g, acc);
    }
}

// ---- interchange-order values -> device panel format -------------------------------
// One workgroup per (panel, batch); a thread handles one padded slot (8/16 bit) or the
// slot pair (b, b+8) that shares bytes (4 bit).
__global__ __launch_bounds__(256) void repack_kernel(RepackArgs a)
{
    const int panel = blockIdx.x, batch = blockIdx.y, V = a.V;
    const int s0 = a.panel_ptr[2 * panel], n = a.panel_ptr[2 * panel + 1] - s0;
    const int npad = (n + MC_CHUNK - 1) / MC_CHUNK * MC_CHUNK;
    const uint8_t *src = a.src + (int64_t)batch * a.src_batch_stride;
    uint8_t *dst = a.dst + (int64_t)batch * a.dst_batch_stride;
    const int64_t vec0 = a.row_ptr[panel];
    if (a.bits == 8 || a.bits == 16) {
        const int cbytes = MC_CHUNK * V * a.bits / 8;
        for (int i = threadIdx.x; i < npad; i += 256) {
            const int s = s0 + i, g = (i % MC_CHUNK) / 16, b = i % 16;
            uint8_t *chunk = dst + (int64_t)(s / MC_CHUNK) * cbytes;
            for (int v = 0; v < V; ++v) {
                if (a.bits == 8) {
                    chunk[g * (16 * V) + v * 16 + b] = (i < n) ? src[(vec0 + i) * V + v] : (uint8_t)0;
                } else {
                    const int x = (i < n) ? reinterpret_cast<const int16_t *>(src)[(vec0 + i) * V + v] : 0;
                    const int hi = (x + 128) >> 8, lo = x - hi * 256;
                    chunk[g * (32 * V) + v * 16 + b] = (uint8_t)hi;
                    chunk[g * (32 * V) + 16 * V + v * 16 + b] = (uint8_t)lo;
                }
            }
        }
    } else { // 4 bits
        const int cbytes = MC_CHUNK * V / 2;
        for (int i2 = threadIdx.x; i2 < npad / 2; i2 += 256) {
            // pair index i2 -> (chunk, g, b < 8): slots i_lo = .. + b and i_hi = i_lo + 8
            const int ch = i2 / 32, g = (i2 % 32) / 8, b = i2 % 8;
            const int i_lo = ch * MC_CHUNK + g * 16 + b, i_hi = i_lo + 8;
            uint8_t *chunk = dst + (int64_t)(s0 / MC_CHUNK + ch) * cbytes;
            for (int v = 0; v < V; ++v) {
                int nl = 0, nh = 0;
                if (i_lo < n) {
                    const int64_t e = (vec0 + i_lo) * V + v;
                    nl = (src[e >> 1] >> ((e & 1) * 4)) & 15;
                }
                if (i_hi < n) {
                    const int64_t e = (vec0 + i_hi) * V + v;
                    nh = (src[e >> 1] >> ((e & 1) * 4)) & 15;
                }
                chunk[g * (8 * V) + v * 8 + b] = (uint8_t)(nl | (nh << 4));
            }
        }
    }
}

} // namespace

template <int PB, int RB, int SEGS, bool DQ, bool U> hipError_t launch_sddmm_lds(const SddmmArgs &a, int waves, hipStream_t s)
{
    dim3 grid((unsigned)(a.items ? a.n_units : a.P), (unsigned)a.batch);
    constexpr int MAXW = (64 * RB * 8 <= 65536) ? 8 : ((64 * RB * 4 <= 65536) ? 4 : 2); // 64 KB of stages per workgroup
    if (waves > MAXW) waves = MAXW;
    switch (waves) {
    case 1: hipLaunchKernelGGL((sddmm_lds_kernel<PB, RB, SEGS, 1, DQ, U>), grid, dim3(64), 0, s, a); break;
    case 2: hipLaunchKernelGGL((sddmm_lds_kernel<PB, RB, SEGS, 2, DQ, U>), grid, dim3(128), 0, s, a); break;
    case 4: hipLaunchKernelGGL((sddmm_lds_kernel<PB, RB, SEGS, (MAXW < 4 ? MAXW : 4), DQ, U>), grid, dim3(64 * (MAXW < 4 ? MAXW : 4)), 0, s, a); break;
    default: hipLaunchKernelGGL((sddmm_lds_kernel<PB, RB, SEGS, MAXW, DQ, U>), grid, dim3(64 * MAXW), 0, s, a); break;
    }
    return hipGetLastError();
}

template <int PB, bool DQ, bool U> hipError_t launch_sddmm_bits(const SddmmArgs &a, int waves, hipStream_t s)
{
    if (waves > 0) {
        if constexpr (PB == 4) {
            if (a.row_bytes == 32) { // 64 nibbles: one MFMA step
                dim3 grid((unsigned)(a.items ? a.n_units : a.P), (unsigned)a.batch);
                switch (waves) {
                case 1: hipLaunchKernelGGL((sddmm_nib32_kernel<1, DQ, U>), grid, dim3(64), 0, s, a); break;
                case 2: hipLaunchKernelGGL((sddmm_nib32_kernel<2, DQ, U>), grid, dim3(128), 0, s, a); break;
                case 4: hipLaunchKernelGGL((sddmm_nib32_kernel<4, DQ, U>), grid, dim3(256), 0, s, a); break;
                default: hipLaunchKernelGGL((sddmm_nib32_kernel<8, DQ, U>), grid, dim3(512), 0, s, a); break;
                }
                return hipGetLastError();
            }
        }
        if (a.row_bytes == 64 && PB != 16) return launch_sddmm_lds<(PB == 16 ? 8 : PB), 64, 1, DQ, U>(a, waves, s);
        if (a.row_bytes == 128) return launch_sddmm_lds<PB, 128, 1, DQ, U>(a, waves, s);
        if (a.row_bytes == 256) return launch_sddmm_lds<PB, 256, 1, DQ, U>(a, waves, s);
        // longer rows go through the stage in passes of 256 bytes: four waves per workgroup still fit
        // (a 512-byte stage leaves room for two; measured 15.6 -> 12.0 us for 16-bit operands at Kd = 256)
        if (a.row_bytes == 512) return launch_sddmm_lds<PB, 256, 2, DQ, U>(a, waves, s);
        if (a.row_bytes == 1024) return launch_sddmm_lds<PB, 256, 4, DQ, U>(a, waves, s);
    }
    dim3 grid((unsigned)(a.items ? a.n_units : a.P), (unsigned)a.batch), block(64 * SDDMM_WAVES);
    if constexpr (U) {
        hipLaunchKernelGGL((sddmm_unsigned_kernel<PB, DQ>), grid, block, 0, s, a); // any row length, operands straight from memory
    } else {
        const int kc = (a.row_bytes + StepBytes<PB>::value - 1) / StepBytes<PB>::value;
        if (kc == 1) hipLaunchKernelGGL((sddmm_direct_kernel<PB, 1, DQ>), grid, block, 0, s, a);
        else if (kc == 2) hipLaunchKernelGGL((sddmm_direct_kernel<PB, 2, DQ>), grid, block, 0, s, a);
        else if (kc <= 4) hipLaunchKernelGGL((sddmm_direct_kernel<PB, 4, DQ>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((sddmm_direct_kernel<PB, 0, DQ>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

template <bool DQ> hipError_t launch_sddmm_out(int bits, const SddmmArgs &a, int waves, hipStream_t s)
{
    if (a.lhs_unsigned || a.rhs_unsigned) {
        if (bits == 8) return launch_sddmm_bits<8, DQ, true>(a, waves, s);
        if (bits == 4) return launch_sddmm_bits<4, DQ, true>(a, waves, s);
        return hipErrorInvalidValue;
    }
    if (bits == 4) return launch_sddmm_bits<4, DQ, false>(a, waves, s);
    if (bits == 16) return launch_sddmm_bits<16, DQ, false>(a, waves, s);
    return launch_sddmm_bits<8, DQ, false>(a, waves, s);
}

hipError_t launch_sddmm(int bits, const SddmmArgs &a, int waves, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0) return hipSuccess;
    return a.float_out ? launch_sddmm_out<true>(bits, a, waves, s) : launch_sddmm_out<false>(bits, a, waves, s);
}

hipError_t launch_repack(const RepackArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0) return hipSuccess;
    dim3 grid((unsigned)a.P, (unsigned)a.batch), block(256);
    hipLaunchKernelGGL(repack_kernel, grid, block, 0, s, a);
    return hipGetLastError();
}

namespace {
// One thread per share (merged vector i, panel g of its group): vb bytes copied from the vector that fills it, or zeros.
__global__ __launch_bounds__(256) void merge_values_kernel(const int32_t *merge_src, const uint8_t *src, uint8_t *dst, int64_t shares, int vb)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= shares) return;
    const int64_t from = merge_src[t];
    for (int b = 0; b < vb; ++b) dst[t * vb + b] = (from >= 0) ? src[from * vb + b] : (uint8_t)0;
}
} // namespace

hipError_t launch_merge_values(const int32_t *merge_src, const uint8_t *src, uint8_t *dst, int64_t shares, int vb, hipStream_t s)
{
    if (shares == 0) return hipSuccess;
    hipLaunchKernelGGL(merge_values_kernel, dim3((unsigned)((shares + 255) / 256)), dim3(256), 0, s, merge_src, src, dst, shares, vb);
    return hipGetLastError();
}
