// SpMM kernels for gfx950: sparse A (V x 1 vectors, device panel format) times dense
// row-major B, exact int32 accumulation on v_mfma_i32_16x16x64_i8.
//
// Work split (paper, Section 4.2.1: one thread block per V x BS_n output tile, nnz/BS_k
// accumulation steps): a workgroup owns one row panel and BNB bytes of every gathered B
// row.  Its WK wavefronts share the panel's chunks of 64 vectors round-robin (each wave
// runs its own pipeline on a private LDS region, no barrier in the loop) and their
// partial tiles are summed through LDS at the end.
//
// One chunk step of a wave (the analogue of the "online transpose", Section 4.2.2):
//   1. the 64 lanes fetch the 64 B rows named by the chunk's column indices with
//      128-bit loads, LPR = BNB/16 neighbouring lanes per row (coalesced row segments);
//   2. the 16-byte pieces land in LDS lane-linear; which row a lane fetches and an XOR
//      on the segment number are chosen so that the later reads hit 64 distinct banks;
//   3. every lane reads 4 x 4 bytes (4 rows x 4 columns) per 16 reduction steps and
//      transposes them with 8 v_perm_b32, giving 4 registers of 4 reduction-consecutive
//      bytes for 4 neighbouring columns; the 4 registers feed 4 different MFMAs, so one
//      lane owns 4 consecutive output columns (int8 B) or 8 (int4 B);
//   4. int4 operands are widened in registers: a byte with the nibble in its top half is
//      16 x the signed nibble, so (x << 4) & 0xF0F0F0F0 and x & 0xF0F0F0F0 are valid int8
//      operands and the int32 sums are shifted right by 4 (or 8) at the end;
//   5. 16-bit A travels as two signed int8 planes in rows 0..7 (high) and 8..15 (low) of
//      the same MFMA (the "stacking" of Section 4.4) and is recombined as (hi<<8)+lo.
// The sum over a chunk does not depend on the order of its terms, so only the row /
// column ownership of the MFMA lanes matters, not the order of reduction bytes, as long
// as A and B use the same order; slot s of a chunk is reduction byte (s % 16) of lane
// group (s / 16) on both sides.
#include "internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

enum { PREC_L8R8 = 0, PREC_L8R4 = 1, PREC_L4R4 = 2, PREC_L16R8 = 3 };

// ---- geometry of the gather for a tile of BNB bytes per row ----------------------
// lane = rg * LPR + seg: row group and 16-byte segment.  Load instruction i of a chunk
// (i < NI = LPR) makes lane (rg, seg) fetch segment seg ^ swz(i) of the row in slot
// ld_slot(rg, i); its 16 bytes go to LDS byte i*1024 + lane*16.
template <int BNB> __device__ __forceinline__ int ld_slot(int rg, int i);
template <int BNB> __device__ __forceinline__ int ld_swz(int i);
// LDS byte address of the dword holding (slot g*16+b, tile bytes T*64+4j .. +3)
template <int BNB> __device__ __forceinline__ int rd_addr(int g, int j, int T, int b);

template <> __device__ __forceinline__ int ld_slot<64>(int rg, int i) { return (rg & 3) * 16 + (rg >> 2) * 4 + i; }
template <> __device__ __forceinline__ int ld_swz<64>(int) { return 0; }
template <> __device__ __forceinline__ int rd_addr<64>(int g, int j, int, int b)
{
    return (b & 3) * 1024 + ((b >> 2) * 4 + g) * 64 + j * 4;
}

template <> __device__ __forceinline__ int ld_slot<128>(int rg, int i)
{
    return (((rg & 1) << 1) | (i & 1)) * 16 + (rg >> 1) * 4 + (i >> 1);
}
template <> __device__ __forceinline__ int ld_swz<128>(int i) { return 4 * (i & 1); }
template <> __device__ __forceinline__ int rd_addr<128>(int g, int j, int T, int b)
{
    const int i = (b & 3) * 2 + (g & 1), rg = (b >> 2) * 2 + (g >> 1);
    const int seg = (T * 4 + (j >> 2)) ^ (4 * (i & 1));
    return i * 1024 + rg * 128 + seg * 16 + (j & 3) * 4;
}

template <> __device__ __forceinline__ int ld_slot<256>(int rg, int i) { return (i & 3) * 16 + rg * 4 + (i >> 2); }
template <> __device__ __forceinline__ int ld_swz<256>(int i) { return 4 * (i & 3); }
template <> __device__ __forceinline__ int rd_addr<256>(int g, int j, int T, int b)
{
    const int i = (b & 3) * 4 + g, rg = b >> 2;
    const int seg = (T * 4 + (j >> 2)) ^ (4 * g);
    return i * 1024 + rg * 256 + seg * 16 + (j & 3) * 4;
}

// 4 x 4 byte transpose: in r[k] = 4 columns of row k; out c[m] = rows 0..3 of column m.
__device__ __forceinline__ void transpose4x4(const unsigned r[4], unsigned c[4])
{
    const unsigned x0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u); // r0.b0 r1.b0 r0.b1 r1.b1
    const unsigned x1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u); // r0.b2 r1.b2 r0.b3 r1.b3
    const unsigned y0 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    const unsigned y1 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    c[0] = __builtin_amdgcn_perm(y0, x0, 0x05040100u);
    c[1] = __builtin_amdgcn_perm(y0, x0, 0x07060302u);
    c[2] = __builtin_amdgcn_perm(y1, x1, 0x05040100u);
    c[3] = __builtin_amdgcn_perm(y1, x1, 0x07060302u);
}

// Keeps the compiler from moving LDS traffic across a point where lanes of one wave
// exchange data through LDS (the hardware executes a wave's LDS operations in order).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// A operand of one chunk for this lane (row = lane % 16, lane group = lane / 16).
template <int MODE>
__device__ __forceinline__ v4i load_a(const uint8_t *vals, int64_t chunk, int V, int row, int g)
{
    v4i a = {0, 0, 0, 0};
    if (MODE == PREC_L16R8) {
        // [chunk][g][plane hi, lo][v][16]; high plane in rows 0..V-1, low plane in rows 8..8+V-1
        const int v = row & 7;
        if (v < V) a = *reinterpret_cast<const v4i *>(vals + chunk * (128 * V) + g * (32 * V) + (row >> 3) * (16 * V) + v * 16);
    } else if (MODE == PREC_L4R4) {
        // [chunk][g][v][8 bytes]: byte b = slot b (low nibble), slot b+8 (high nibble)
        if (row < V) {
            const v2i x = *reinterpret_cast<const v2i *>(vals + chunk * (32 * V) + g * (8 * V) + row * 8);
            a.x = (x.x << 4) & 0xF0F0F0F0;
            a.y = (x.y << 4) & 0xF0F0F0F0;
            a.z = x.x & 0xF0F0F0F0;
            a.w = x.y & 0xF0F0F0F0;
        }
    } else {
        if (row < V) a = *reinterpret_cast<const v4i *>(vals + chunk * (64 * V) + g * (16 * V) + row * 16);
    }
    return a;
}

template <int BNB, int WK, int MODE> struct SpmmCfg {
    static constexpr bool R4 = (MODE == PREC_L8R4 || MODE == PREC_L4R4);
    static constexpr int NT = BNB / 64;                 // groups of 64 tile bytes
    static constexpr int NACC = NT * 4 * (R4 ? 2 : 1);  // MFMA accumulators per lane (v4i each)
    static constexpr int STAGE = 64 * BNB;              // LDS bytes of one staged chunk
    static constexpr int RED = (WK - 1) * NACC * 1024;  // LDS bytes of the final reduction
    static constexpr int LDS = (WK * STAGE > RED) ? WK * STAGE : RED;
};

template <int BNB, int WK, int MODE>
__global__ __launch_bounds__(64 * WK) void spmm_kernel(SpmmArgs a)
{
    using Cfg = SpmmCfg<BNB, WK, MODE>;
    constexpr int LPR = BNB / 16, NI = LPR, NT = Cfg::NT, NACC = Cfg::NACC;
    constexpr bool R4 = Cfg::R4;
    __shared__ __attribute__((aligned(16))) char lds[Cfg::LDS];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane / LPR, seg = lane % LPR;
    const int ntiles = (a.row_bytes + BNB - 1) / BNB;
    const int panel = blockIdx.x / ntiles, tile = blockIdx.x % ntiles;
    const int batch = blockIdx.y;
    const int nb0 = tile * BNB;

    const int s0 = a.panel_ptr[2 * panel], s1 = a.panel_ptr[2 * panel + 1];
    const int nch = (s1 - s0 + MC_CHUNK - 1) / MC_CHUNK;
    const int64_t chunk0 = s0 / MC_CHUNK;
    const int32_t *idx = a.slot_idx + s0;
    const uint8_t *vals = a.vals + (int64_t)batch * a.vals_batch_stride;
    const uint8_t *Bb = a.B + (int64_t)batch * a.B_batch_stride + nb0;
    char *my = lds + w * Cfg::STAGE;

    v4i acc[NACC];
#pragma unroll
    for (int t = 0; t < NACC; ++t) acc[t] = (v4i){0, 0, 0, 0};

    // this lane's NI column indices of a chunk are NI/4 runs of 4 consecutive slots
    v4i idxv[NI / 4], idxn[NI / 4];
    v4i breg[NI];
    v4i a_next = {0, 0, 0, 0};

    auto load_idx = [&](int c, v4i (&dst)[NI / 4]) {
#pragma unroll
        for (int t = 0; t < NI / 4; ++t) {
            // run t starts at the slot of the first instruction that uses it
            const int i0 = (BNB == 64) ? 0 : t; // BNB 128: i = t, t+2, ..; BNB 256: i = t, t+4, ..
            dst[t] = *reinterpret_cast<const v4i *>(idx + c * MC_CHUNK + ld_slot<BNB>(rg, i0));
        }
    };
    auto pick_idx = [&](const v4i (&src)[NI / 4], int i) -> int {
        if (BNB == 64) return src[0][i];
        if (BNB == 128) return src[i & 1][i >> 1];
        return src[i & 3][i >> 2];
    };
    auto issue_b = [&](const v4i (&ix)[NI / 4]) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = pick_idx(ix, i);
            const int lseg = seg ^ ld_swz<BNB>(i);
            if (nb0 + lseg * 16 < a.row_bytes)
                breg[i] = *reinterpret_cast<const v4i *>(Bb + (int64_t)row * a.ldb_bytes + lseg * 16);
            else
                breg[i] = (v4i){0, 0, 0, 0};
        }
    };

    int c = w;
    if (c < nch) {
        load_idx(c, idxv);
        issue_b(idxv);
        a_next = load_a<MODE>(vals, chunk0 + c, a.V, j, g);
        if (c + WK < nch) load_idx(c + WK, idxn);
    }
    for (; c < nch; c += WK) {
#pragma unroll
        for (int i = 0; i < NI; ++i) *reinterpret_cast<v4i *>(my + i * 1024 + lane * 16) = breg[i];
        const v4i a_cur = a_next;
        if (c + WK < nch) {
            issue_b(idxn);
            a_next = load_a<MODE>(vals, chunk0 + c + WK, a.V, j, g);
            if (c + 2 * WK < nch) load_idx(c + 2 * WK, idxn);
        }
        wave_lds_fence();
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            unsigned r[16], cc[16];
#pragma unroll
            for (int b = 0; b < 16; ++b) r[b] = *reinterpret_cast<const unsigned *>(my + rd_addr<BNB>(g, j, T, b));
#pragma unroll
            for (int q = 0; q < 4; ++q) transpose4x4(&r[4 * q], &cc[4 * q]);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const v4i bop = {(int)cc[m], (int)cc[4 + m], (int)cc[8 + m], (int)cc[12 + m]};
                if (!R4) {
                    acc[T * 4 + m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, bop, acc[T * 4 + m], 0, 0, 0);
                } else {
                    const v4i lo = (bop << 4) & (v4i){(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
                    const v4i hi = bop & (v4i){(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
                    acc[(T * 4 + m) * 2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, lo, acc[(T * 4 + m) * 2], 0, 0, 0);
                    acc[(T * 4 + m) * 2 + 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, hi, acc[(T * 4 + m) * 2 + 1], 0, 0, 0);
                }
            }
        }
        wave_lds_fence();
    }

    // ---- sum the partial tiles of the WK waves (wave 0 keeps the result) ----------
    if (WK > 1) {
        __syncthreads();
        if (w > 0) {
#pragma unroll
            for (int t = 0; t < NACC; ++t)
                *reinterpret_cast<v4i *>(lds + ((w - 1) * NACC + t) * 1024 + lane * 16) = acc[t];
        }
        __syncthreads();
        if (w > 0) return;
#pragma unroll
        for (int ww = 1; ww < WK; ++ww)
#pragma unroll
            for (int t = 0; t < NACC; ++t)
                acc[t] += *reinterpret_cast<const v4i *>(lds + ((ww - 1) * NACC + t) * 1024 + lane * 16);
    }

    // ---- epilogue: accumulator register r of lane (j, g) is output row 4g + r --------
    if (MODE == PREC_L16R8) {
        // rows 8..15 (lanes 32..63) hold the low-plane sums of rows 0..7
#pragma unroll
        for (int t = 0; t < NACC; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const unsigned lo = (unsigned)__shfl_down(acc[t][r], 32, 64);
                acc[t][r] = (int)(((unsigned)acc[t][r] << 8) + lo);
            }
    } else if (MODE == PREC_L8R4) {
#pragma unroll
        for (int t = 0; t < NACC; ++t) acc[t] = acc[t] >> 4;
    } else if (MODE == PREC_L4R4) {
#pragma unroll
        for (int t = 0; t < NACC; ++t) acc[t] = acc[t] >> 8;
    }
    if (g >= 2) return;
    constexpr int CPB = R4 ? 2 : 1; // output columns per tile byte
    const int ncols = a.row_bytes * CPB;
#pragma unroll
    for (int T = 0; T < NT; ++T) {
        const int col = (nb0 + T * 64 + 4 * j) * CPB;
        if (col >= ncols) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * g + r;
            if (row >= a.V) continue;
            const int64_t off = (int64_t)batch * a.C_batch_stride + (int64_t)(panel * a.V + row) * a.ldc + col;
#pragma unroll
            for (int h = 0; h < CPB; ++h) {
                // R8: columns col..col+3 come from MFMAs m = 0..3; R4: 2m, 2m+1 from (m, lo/hi)
                const v4i o = R4 ? (v4i){acc[(T * 4 + 2 * h) * 2][r], acc[(T * 4 + 2 * h) * 2 + 1][r],
                                         acc[(T * 4 + 2 * h + 1) * 2][r], acc[(T * 4 + 2 * h + 1) * 2 + 1][r]}
                                 : (v4i){acc[T * 4][r], acc[T * 4 + 1][r], acc[T * 4 + 2][r], acc[T * 4 + 3][r]};
                if (a.float_out) {
                    const v4f f = {o.x * a.out_scale, o.y * a.out_scale, o.z * a.out_scale, o.w * a.out_scale};
                    *reinterpret_cast<v4f *>(static_cast<float *>(a.C) + off + 4 * h) = f;
                } else {
                    *reinterpret_cast<v4i *>(static_cast<int32_t *>(a.C) + off + 4 * h) = o;
                }
            }
        }
    }
}

template <int BNB, int WK, int MODE> hipError_t launch_one(const SpmmArgs &a, hipStream_t s)
{
    const int ntiles = (a.row_bytes + BNB - 1) / BNB;
    dim3 grid((unsigned)(a.P * ntiles), (unsigned)a.batch), block(64 * WK);
    hipLaunchKernelGGL((spmm_kernel<BNB, WK, MODE>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <int BNB, int MODE> hipError_t launch_wk(const SpmmArgs &a, int waves, hipStream_t s)
{
    switch (waves) {
    case 1: return launch_one<BNB, 1, MODE>(a, s);
    case 2: return launch_one<BNB, 2, MODE>(a, s);
    default: return launch_one<BNB, 4, MODE>(a, s);
    }
}

template <int MODE> hipError_t launch_mode(const SpmmArgs &a, int bnb, int waves, hipStream_t s)
{
    constexpr bool R4 = (MODE == PREC_L8R4 || MODE == PREC_L4R4);
    if (bnb == 64) return launch_wk<64, MODE>(a, waves, s);
    if (bnb == 256 && !R4) return launch_wk<256, (R4 ? PREC_L8R8 : MODE)>(a, waves, s);
    return launch_wk<128, MODE>(a, waves, s);
}

} // namespace

hipError_t launch_spmm(mc_prec prec, const SpmmArgs &a, int bnb, int waves, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0 || a.row_bytes == 0) return hipSuccess;
    switch (prec) {
    case MC_L8R8: return launch_mode<PREC_L8R8>(a, bnb, waves, s);
    case MC_L8R4: return launch_mode<PREC_L8R4>(a, bnb, waves, s);
    case MC_L4R4: return launch_mode<PREC_L4R4>(a, bnb, waves, s);
    case MC_L16R8: return launch_mode<PREC_L16R8>(a, bnb, waves, s);
    }
    return hipErrorInvalidValue;
}
