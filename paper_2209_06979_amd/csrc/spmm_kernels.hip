// SpMM kernels for gfx950: sparse A (V x 1 vectors, device panel format) times dense
// row-major B, exact int32 accumulation on v_mfma_i32_16x16x64_i8.
//
// Work split (paper, Section 4.2.1: one thread block per V x BS_n output tile, nnz/BS_k
// accumulation steps): a workgroup owns one row panel and BNB bytes of every gathered B
// row.  Its WK wavefronts share the panel's chunks of 64 vectors round-robin; each wave
// works on a private LDS region (no barrier in the loop) and the partial tiles are summed
// through LDS at the end.  Latency is hidden the MI355X way rather than with the software
// pipeline of the paper's Algorithm 1: a chunk in flight costs LDS, not registers, so the
// 160 KB of a CU are filled with many waves that each have one chunk in flight.
//
// One chunk step of a wave (the analogue of the "online transpose", Section 4.2.2):
//   1. the 64 lanes copy the 64 B rows named by the chunk's column indices from global
//      memory straight into LDS (global_load_lds, 16 bytes per lane, LPR = BNB/16
//      neighbouring lanes per row, so every row segment is one coalesced request); no
//      registers are spent on the data in flight;
//   2. ds_read_b64_tr_b8 reads an 8-row x 16-column byte block per 16-lane group and
//      hands every lane the 8 reduction-consecutive bytes of its own column, which is
//      exactly the MFMA column-operand layout: the transpose costs no ALU work;
//      the 16-byte segments of a row are XOR-swizzled with the load-instruction number so
//      that the 8 rows read together sit in 8 different bank groups;
//   3. int4 operands are widened in registers: a byte with the nibble in its top half is
//      16 x the signed nibble, so (x << 4) & 0xF0F0F0F0 and x & 0xF0F0F0F0 are valid int8
//      operands and the int32 sums are shifted right by 4 (or 8) at the end;
//   4. 16-bit A travels as two signed int8 planes in rows 0..7 (high) and 8..15 (low) of
//      the same MFMA (the "stacking" of Section 4.4) and is recombined as (hi<<8)+lo;
//   5. a 16-bit B row is gathered as it is and treated as a byte matrix of twice the width:
//      even byte columns hold the low (unsigned) bytes, odd ones the high (signed) bytes.
//      The MFMA is signed x signed, so a low byte u enters as u ^ 0x80 = u - 128 and the
//      missing 128 * sum_k A[m][k] comes from one extra MFMA per chunk against an all-ones
//      operand; the byte-column pairs are recombined as (hi<<8)+lo in the epilogue;
//   6. unsigned 8- or 4-bit operands (Section 4.4.1; kernels with U = true) use the same trick on
//      either side: an unsigned value u enters the signed MFMA as u - c (c = 128, or 8 for a
//      nibble, i.e. one XOR of the top bit of the operand byte), and
//      sum (a'+ca)(b'+cb) = sum a'b' + cb * sum a' + ca * sum b' + ca*cb*n.  The row sums of A come
//      from the all-ones MFMA of 5., the column sums of the gathered B rows from MFMA row 8,
//      which is free when A has one plane and is fed an all-ones row operand.
// The sum over a chunk does not depend on the order of its terms; slot s of a chunk is
// reduction byte (s % 16) of lane group (s / 16) on both the A and the B side.
#include "internal.h"
#include "lds_async.h"
#include "spmm_operand.h"

namespace {

using mcu::v4i;
using mcu::v2i;
using mcu::v4f;
using mcu::lds_v2i;
using mcu::load_a;
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

// NS: chunks in flight per wave.  1: the copies are issued through the compiler's builtin, which
// makes it wait for all of them before the first LDS read (any extent of B, any panel length).
// 2: the copies are issued from inline assembly into two alternating stages and only the older
// chunk is waited for (counted s_waitcnt); for waves with at most SPMM_PIPE_CHUNKS chunks; lane
// offsets are 32 bits, so B must span less than 4 GiB.
constexpr int SPMM_PIPE_CHUNKS = 4;

// Makes the compiler treat x as used and redefined here: a load into x that is still in flight is
// waited for at this point (and at no later one).
__device__ __forceinline__ void pin(v4i &x) { asm volatile("" : "+v"(x)); }
template <int BNB, int WK, int LB, int RB, bool U = false, int NS = 1> struct SpmmCfg {
    static constexpr bool R4 = (RB == 4), R16 = (RB == 16), L16 = (LB == 16);
    static_assert(!U || (!R16 && !L16), "unsigned operands: 4 and 8 bits");
    static constexpr int LPR = BNB / 16;                 // lanes (16-byte segments) per row
    static constexpr int NI = LPR;                       // load instructions per chunk
    static constexpr int RPI = 64 / LPR;                 // rows per load instruction
    static constexpr int SWZ = (LPR == 4) ? 3 : 7;       // bits of the instruction number used as swizzle
    static constexpr int XACC = LPR * (R4 ? 2 : 1);      // index of the accumulator of the all-ones MFMA (row sums of A)
    static constexpr int NACC = XACC + ((R16 || U) ? 1 : 0); // MFMA accumulators per lane (v4i each)
    static constexpr int STAGE = 64 * BNB;               // LDS bytes of one staged chunk
    static constexpr int COLS = BNB * (R4 ? 2 : 1);      // columns of the partial tile (byte columns for R16)
    static constexpr int OUTC = R16 ? BNB / 2 : COLS;    // output columns of the tile
    static constexpr int OROWS = L16 ? 16 : (U ? 12 : 8); // rows of a partial tile (U: row 8 holds column sums of B)
    static constexpr int TST = COLS + 4;                 // row stride (ints) of a partial tile: +4 keeps rows 4 apart in different banks
    static constexpr int OTILE = OROWS * TST * 4;        // bytes of one wave's partial tile
    static constexpr int PERWAVE = (NS * STAGE > OTILE) ? NS * STAGE : OTILE;
    static constexpr int LDS = WK * PERWAVE;
    // Which LDS row (within the RPI rows a load instruction writes) holds slot group r (slots r*NI .. r*NI+NI-1), and
    // back.  A transposing read's lane groups g and g + 1 (32 lanes, 256 bytes of banks) ask for slot groups 2g + h and
    // 2g + 2 + h (NI 8) or 4g + .. and 4g + 4 + .. (NI 4); in slot-group order those rows lie 256 bytes apart, i.e. in
    // the same banks, and every read took two conflict cycles.  Putting the bit g & 1 into address bit 7 instead
    // spreads them over all banks.
    static constexpr int row_of_group(int r)
    {
        return NI == 8 ? (((r & 1) << 2) | (r >> 1)) : (NI == 4 ? ((r & 9) | ((r & 2) << 1) | ((r & 4) >> 1)) : r);
    }
    static constexpr int group_of_row(int row)
    {
        return NI == 8 ? (((row & 3) << 1) | (row >> 2)) : (NI == 4 ? ((row & 9) | ((row & 2) << 1) | ((row & 4) >> 1)) : row);
    }
};

// Time stamps of a wave's progress (measurement aid: TR is true in one instantiation only, which
// mc_probe_spmm_phases launches; every other kernel carries none of this).  Ticks of the constant 100 MHz clock.
template <bool TR> struct PhaseClock {
    long long t[TR ? 10 : 1] = {};
    __device__ __forceinline__ void stamp(int k)
    {
        if constexpr (TR) {
            __builtin_amdgcn_sched_barrier(0);
            t[k] = wall_clock64();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
};

template <int BNB, int WK, int LB, int RB, bool U = false, int NS = 1, bool TR = false>
__global__ __launch_bounds__(64 * WK) void spmm_kernel(SpmmArgs a)
{
    using Cfg = SpmmCfg<BNB, WK, LB, RB, U, NS>;
    PhaseClock<TR> clk;
    clk.stamp(0);                                        // the wave has started
    constexpr int LPR = Cfg::LPR, NI = Cfg::NI, RPI = Cfg::RPI, NACC = Cfg::NACC, COLS = Cfg::COLS, TST = Cfg::TST;
    constexpr int OUTC = Cfg::OUTC;
    constexpr bool R4 = Cfg::R4, R16 = Cfg::R16, L16 = Cfg::L16;
    constexpr int XACC = Cfg::XACC;
    const int axor = (U && a.lhs_unsigned) ? (int)0x80808080 : 0, bxor = (U && a.rhs_unsigned) ? (int)0x80808080 : 0;
    __shared__ __attribute__((aligned(16))) char lds[Cfg::LDS];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int rg = lane / LPR, seg = lane % LPR;
    // workgroups of a unit: a.ntiles column tiles, a power of two when a.tile_shift >= 0
    const int unit = (a.tile_shift >= 0) ? (int)(blockIdx.x >> a.tile_shift) : (int)(blockIdx.x / a.ntiles);
    const int tile = (int)(blockIdx.x - unit * a.ntiles);
    const int batch = blockIdx.y;
    const int nb0 = tile * BNB;

    // a unit of work: a whole panel, or (matrices with very unequal panels) a range of its chunks
    int panel = unit, cb = 0, ce = -1, split = 0;
    if (a.items) {
        const v4i it = *reinterpret_cast<const v4i *>(a.items + 4 * unit);
        panel = it.x; cb = it.y; ce = it.z; split = it.w;
    }
    // Panels that all have the same number of chunks start at a computable slot: no trip to memory for the panel
    // pointers, on which every later load of the workgroup depends (padded slots carry zero values, so the real end
    // of the panel is not needed either).
    int s0;
    if (a.uniform_chunks > 0) {
        s0 = panel * a.uniform_chunks * MC_CHUNK;
        if (ce < 0) ce = a.uniform_chunks;
    } else {
        const v2i pp = *reinterpret_cast<const v2i *>(a.panel_ptr + 2 * panel); // first slot, end slot: one load
        s0 = pp.x;
        if (ce < 0) ce = (pp.y - s0 + MC_CHUNK - 1) / MC_CHUNK;
    }
    if constexpr (TR) {
        asm volatile("" ::"s"(s0), "s"(ce));             // (the stamp waits for the pointers)
        clk.stamp(1);                                    // kernel arguments and panel pointers have arrived
    }
    const int nch = ce - cb;                       // chunks of this unit: cb .. ce-1
    const int64_t chunk0 = s0 / MC_CHUNK + cb;
    const int32_t *idx = a.slot_idx + s0 + cb * MC_CHUNK;
    const uint8_t *vals = a.vals + (int64_t)batch * a.vals_batch_stride;
    const uint8_t *Bb = a.B + (int64_t)batch * a.B_batch_stride + nb0;
    char *stage = lds + w * Cfg::PERWAVE;

    v4i acc[NACC];
#pragma unroll
    for (int t = 0; t < NACC; ++t) acc[t] = (v4i){0, 0, 0, 0};

    // Load instruction i of a chunk: lane (rg, seg) copies segment seg ^ (i & SWZ) of the
    // row in slot group_of_row(rg)*NI + i to LDS byte i*1024 + lane*16, i.e. LDS row i*RPI + rg.  The NI
    // column indices a lane needs are consecutive slots: NI/4 128-bit index loads.
    // A segment beyond the row end is replaced by segment 0 (its columns are never stored),
    // so that every chunk issues exactly the same number of memory instructions.
    auto load_idx = [&](int c, v4i (&dst)[NI / 4]) {
#pragma unroll
        for (int t = 0; t < NI / 4; ++t) dst[t] = *reinterpret_cast<const v4i *>(idx + c * MC_CHUNK + Cfg::group_of_row(rg) * NI + 4 * t);
    };
    int segoff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        // (rows of 256 bytes: the row's parity picks the 128-byte half as well, for the same reason as row_of_group)
        const int lseg = seg ^ (i & Cfg::SWZ) ^ ((NI == 16) ? ((rg & 1) << 3) : 0);
        segoff[i] = (nb0 + lseg * 16 < a.row_bytes) ? lseg * 16 : 0;
    }
    const int nmy = (nch > w) ? (nch - w + WK - 1) / WK : 0; // chunks of this wave: w, w+WK, ...

    // piece pc of the finished tile = 4 columns of one of its 8 rows; this thread owns pieces tid, tid + 64 WK, ...
    const int ncols = R4 ? a.row_bytes * 2 : (R16 ? a.row_bytes / 2 : a.row_bytes);
    constexpr int PIECES = 8 * (OUTC / 4);
    constexpr int NPC = (PIECES + 64 * WK - 1) / (64 * WK);

    // LDS byte address (within a stage) of this lane's source piece for the transposing
    // read of half h (slots g*16 + 8h .. +7), before the column-tile XOR.
    const int src = lane & 15, ii = src >> 1;
    int rd_base[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int s = g * 16 + 8 * h + ii;
        const int i = s % NI, r = Cfg::row_of_group(s / NI);
        rd_base[h] = i * 1024 + r * BNB + (((i & Cfg::SWZ) ^ ((NI == 16) ? ((r & 1) << 3) : 0)) * 16) + 8 * (src & 1);
    }
    // R16: lanes that own an even byte column (low bytes) flip the top bit of every byte
    const int lowflip = (R16 && !(j & 1)) ? (int)0x80808080 : 0;
    // the A operand of chunk c of this wave's share, ready for the MFMA
    auto load_a_op = [&](int c) -> v4i {
        v4i av = load_a<LB>(vals, chunk0 + c, a.V, j, g);
        if (U) {
            if (j < a.V) av ^= (v4i){axor, axor, axor, axor};
            if (j == 8) av = (v4i){0x01010101, 0x01010101, 0x01010101, 0x01010101}; // row 8 collects the column sums of B
        }
        return av;
    };
    // all MFMAs of one chunk whose rows sit in the stage at st
    auto compute = [&](const char *st, v4i a_cur) {
#pragma unroll
        for (int ct = 0; ct < LPR; ++ct) {
            const v2i d0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(st + (rd_base[0] ^ (ct * 16))));
            const v2i d1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(st + (rd_base[1] ^ (ct * 16))));
            v4i bop = {d0.x, d0.y, d1.x, d1.y};
            if (R16) bop ^= (v4i){lowflip, lowflip, lowflip, lowflip};
            const v4i bx = {bxor, bxor, bxor, bxor};
            if (!R4) {
                if (U) bop ^= bx;
                acc[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, bop, acc[ct], 0, 0, 0);
            } else {
                const v4i msk = {(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
                v4i be = (bop << 4) & msk, bo = bop & msk;
                if (U) { be ^= bx; bo ^= bx; }
                acc[2 * ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, be, acc[2 * ct], 0, 0, 0);
                acc[2 * ct + 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, bo, acc[2 * ct + 1], 0, 0, 0);
            }
        }
        if (R16 || U) {
            const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
            acc[XACC] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, ones, acc[XACC], 0, 0, 0); // every column: sum over the chunk of A's row
        }
    };
    if (NS == 1) {
        v4i idxv[NI / 4];
        if (nmy > 0) load_idx(w, idxv);
        for (int k = 0; k < nmy; ++k) {
            const int c = w + k * WK;
#pragma unroll
            for (int i = 0; i < NI; ++i)
                __builtin_amdgcn_global_load_lds((gptr_t *)(Bb + (int64_t)idxv[i >> 2][i & 3] * a.ldb_bytes + segoff[i]),
                                                 (lptr_t *)(stage + i * 1024), 16, 0, 0);
            const v4i a_cur = load_a_op(c);
            if (k + 1 < nmy) load_idx(c + WK, idxv); // the copies above have consumed the old indices
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            compute(stage, a_cur);
            // the reads of the staged rows are complete before the next chunk overwrites them
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    } else {
        // Two chunks in flight (waves with at most MAXL chunks; the launcher guarantees it).
        // Every load that returns data in registers -- the column indices and A operands of ALL
        // the wave's chunks -- is issued up front and completed before the first copy: the
        // compiler schedules its own waits for such loads by counting the loads it knows of, and
        // such a wait in the middle of the loop would also wait for the copies it does not know
        // of.  The empty assembly statements below make the loaded registers "used" at this
        // point, so that the compiler's waits land here, where nothing else is in flight.  The
        // loop then contains copies (assembly, no register destination) and LDS reads only, and
        // vector-memory operations complete in issue order: "at most NI outstanding" right after
        // the NI copies of chunk k+1 means that chunk k has arrived.  (Row numbers and row strides are
        // below 2^24 here -- the launcher checks it -- so a lane's offset is one 24-bit multiply-add.)
        constexpr int MAXL = SPMM_PIPE_CHUNKS;
        const unsigned stage_u = mcu::lds_addr_uniform(stage);
        const unsigned ldb32 = (unsigned)a.ldb_bytes;
        v4i ix[MAXL][NI / 4], av[MAXL];
        mcu::static_for<MAXL>([&](auto Lc) {
            constexpr int l = decltype(Lc)::value;
#pragma unroll
            for (int t = 0; t < NI / 4; ++t) ix[l][t] = (v4i){0, 0, 0, 0};
            av[l] = (v4i){0, 0, 0, 0};
            if (l < nmy) {
                load_idx(w + l * WK, ix[l]);
                av[l] = load_a_op(w + l * WK);
            }
        });
        mcu::static_for<MAXL>([&](auto Lc) {
            constexpr int l = decltype(Lc)::value;
#pragma unroll
            for (int t = 0; t < NI / 4; ++t) pin(ix[l][t]);
            pin(av[l]);
        });
        auto issue = [&](int st, const v4i (&ixs)[NI / 4]) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
                mcu::copy16_to_lds(Bb, __umul24((unsigned)ixs[i >> 2][i & 3], ldb32) + (unsigned)segoff[i], stage_u + st * Cfg::STAGE + i * 1024);
        };
        clk.stamp(2);                                    // column indices and A operands have arrived
        if (nmy == 0) clk.stamp(3);                      // (a wave without chunks waits for no rows)
        if (nmy > 0) issue(0, ix[0]);
        mcu::static_for<MAXL>([&](auto Lc) {
            constexpr int l = decltype(Lc)::value;
            if (l < nmy) {
                if (l + 1 < MAXL && l + 1 < nmy) {
                    issue((l + 1) & 1, ix[(l + 1 < MAXL) ? l + 1 : l]);
                    mcu::vm_wait<NI>();
                } else {
                    mcu::vm_wait<0>();
                }
                if (l == 0) clk.stamp(3);                // the rows of the wave's first chunk have landed
                compute(stage + (l & 1) * Cfg::STAGE, av[l]);
                mcu::lgkm_wait(); // the reads of this stage have returned before it is refilled
            }
        });
    }

    // ---- partial tiles -> LDS (each wave into its own region), row-major int32 ----------
    // accumulator register r of lane (j, g) is output row 4g + r; MFMA ct covers tile bytes
    // 16*ct .. 16*ct+15, i.e. column 16*ct + j (R8) or columns 32*ct + 2j, 2j+1 (R4).
    // A one-plane operand of 16 rows (the merged copy of an operand) passes through the tile in two
    // halves of 8 rows: lane groups 0, 1 first, then 2, 3.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    clk.stamp(4);                                        // all chunks of the wave are in its accumulators
    int *tile_w = reinterpret_cast<int *>(stage);
    constexpr int OROWS = Cfg::OROWS;
    constexpr int SH = R4 ? (LB == 4 ? 8 : 4) : 0;       // scale carried by widened nibbles
    const int nhalf = (!L16 && !U && a.V > 8) ? 2 : 1;
    for (int hf = 0; hf < nhalf; ++hf) {
        if (hf) __syncthreads();                         // the first half's tiles have been read
        const int gg = g - 2 * hf;
        if (gg >= 0 && 4 * gg < OROWS) {
#pragma unroll
            for (int ct = 0; ct < LPR; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (!R4) {
                        tile_w[(4 * gg + r) * TST + ct * 16 + j] = acc[ct][r];
                    } else {
                        *reinterpret_cast<v2i *>(&tile_w[(4 * gg + r) * TST + ct * 32 + 2 * j]) = (v2i){acc[2 * ct][r], acc[2 * ct + 1][r]};
                    }
                }
            if ((R16 || U) && j == 0) { // the row sums ride in the padding column of the tile
#pragma unroll
                for (int r = 0; r < 4; ++r) tile_w[(4 * gg + r) * TST + COLS] = acc[XACC][r];
            }
        }
        if (hf == 0) clk.stamp(5);                       // partial tile written
        __syncthreads();
        if (hf == 0) clk.stamp(6);                       // the other waves' tiles are there too

        // ---- sum over the waves, finish the arithmetic, store 16 bytes per thread -------------
        // Every plane sum is exact in int32 (R4: after its shift); the recombinations wrap.
        // All LDS reads of a thread's pieces first (a piece beyond the tile reads the last one again), then the stores.
        v4i fin[NPC];
#pragma unroll
        for (int q = 0; q < NPC; ++q) {
            const int pc = (tid + q * 64 * WK < PIECES) ? tid + q * 64 * WK : PIECES - 1;
            const int row = pc / (OUTC / 4), col = (pc % (OUTC / 4)) * 4;
            const int tcol = R16 ? 2 * col : col;            // first column in the partial tile
            v4i s = {0, 0, 0, 0}, lo = {0, 0, 0, 0}, s2 = {0, 0, 0, 0}, lo2 = {0, 0, 0, 0}, cs = {0, 0, 0, 0};
            int rs = 0, rs_lo = 0;
#pragma unroll
            for (int ww = 0; ww < WK; ++ww) {
                const int *t = reinterpret_cast<const int *>(lds + ww * Cfg::PERWAVE);
                s += *reinterpret_cast<const v4i *>(&t[row * TST + tcol]);
                if (L16) lo += *reinterpret_cast<const v4i *>(&t[(row + 8) * TST + tcol]);
                if (U) {
                    cs += *reinterpret_cast<const v4i *>(&t[8 * TST + tcol]);
                    rs += t[row * TST + COLS];
                }
                if (R16) {
                    s2 += *reinterpret_cast<const v4i *>(&t[row * TST + tcol + 4]);
                    rs += t[row * TST + COLS];
                    if (L16) {
                        lo2 += *reinterpret_cast<const v4i *>(&t[(row + 8) * TST + tcol + 4]);
                        rs_lo += t[(row + 8) * TST + COLS];
                    }
                }
            }
            if (U) {
                // sum (a'+ca)(b'+cb): the operand bytes carry a' and b' (times 16 for nibbles), and
                // cb * 16^[R4] = ca * 16^[L4] = 128, so both corrections are the sums shifted by 7
                if (a.rhs_unsigned) s += (v4i){rs << 7, rs << 7, rs << 7, rs << 7};
                if (a.lhs_unsigned) s += cs << 7;
            }
            if (R4) { s = s >> SH; lo = lo >> SH; }
            if (U && a.lhs_unsigned && a.rhs_unsigned) {
                const int cc = (LB == 4 ? 8 : 128) * (RB == 4 ? 8 : 128) * (nch * MC_CHUNK); // ca * cb * slots (padded ones included: their a' is -ca)
                s += (v4i){cc, cc, cc, cc};
            }
            if (L16) { s = (s << 8) + lo; s2 = (s2 << 8) + lo2; rs = (rs << 8) + rs_lo; }
            if (R16) {
                // byte columns (low, high) of four B elements: A*b = (A*hi << 8) + A*(low ^ 0x80) + 128 * rowsum(A)
                const int fix = rs << 7;
                s = (v4i){(s.y << 8) + s.x + fix, (s.w << 8) + s.z + fix, (s2.y << 8) + s2.x + fix, (s2.w << 8) + s2.z + fix};
            }
            fin[q] = s;
        }
        if constexpr (TR) {
            if (hf == 0) {
                asm volatile("" ::"v"(fin[0]), "v"(fin[NPC - 1]));
                clk.stamp(7);                            // this thread's pieces are summed
            }
        }
#pragma unroll
        for (int q = 0; q < NPC; ++q) {
            const int pc = tid + q * 64 * WK;
            const int row = pc / (OUTC / 4) + 8 * hf, gcol = tile * OUTC + (pc % (OUTC / 4)) * 4;
            const int crow = panel * a.V + row;              // row of C
            if (pc >= PIECES || row >= a.V || crow >= a.rows || gcol >= ncols) continue;
            const v4i s = fin[q];
            const int64_t off = (int64_t)batch * a.C_batch_stride + (int64_t)crow * a.ldc + gcol;
            if (split && a.acc) {
                // a shared panel whose final values are rounded: the exact partial sums meet in int32 rows of their own
                int32_t *c = a.acc + (((int64_t)batch * a.n_split + (split - 1)) * a.V + row) * a.acc_ld + gcol;
                atomicAdd(c, s.x); atomicAdd(c + 1, s.y); atomicAdd(c + 2, s.z); atomicAdd(c + 3, s.w);
            } else if (a.float_out) {
                const v4f f = {s.x * a.out_scale, s.y * a.out_scale, s.z * a.out_scale, s.w * a.out_scale};
                if (a.float_out == 2) __builtin_nontemporal_store(mcu::to_half4(f), reinterpret_cast<mcu::v4h *>(static_cast<_Float16 *>(a.C) + off));
                else __builtin_nontemporal_store(f, reinterpret_cast<v4f *>(static_cast<float *>(a.C) + off));
            } else if (split) {
                // several units own this panel: exact, order-independent integer accumulation into rows
                // that were cleared before the launch
                int32_t *c = static_cast<int32_t *>(a.C) + off;
                atomicAdd(c, s.x); atomicAdd(c + 1, s.y); atomicAdd(c + 2, s.z); atomicAdd(c + 3, s.w);
            } else {
                __builtin_nontemporal_store(s, reinterpret_cast<v4i *>(static_cast<int32_t *>(a.C) + off));
            }
        }
    }
    if constexpr (TR) {
        clk.stamp(8);                                    // stores issued
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        clk.stamp(9);                                    // stores acknowledged
        if (a.trace && lane == 0) {
            long long *t = a.trace + ((int64_t)blockIdx.x * WK + w) * 10;
#pragma unroll
            for (int q = 0; q < 10; ++q) t[q] = clk.t[q];
        }
    }
}

template <int BNB, int WK, int LB, int RB, bool U, int NS> hipError_t launch_one(SpmmArgs a, hipStream_t s)
{
    a.ntiles = (a.row_bytes + BNB - 1) / BNB;
    a.tile_shift = -1;
    for (int sh = 0; sh < 31; ++sh)
        if ((1 << sh) == a.ntiles) a.tile_shift = sh;
    dim3 grid((unsigned)((a.items ? a.n_units : a.P) * a.ntiles), (unsigned)a.batch), block(64 * WK);
    hipLaunchKernelGGL((spmm_kernel<BNB, WK, LB, RB, U, NS>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <int BNB, int LB, int RB, bool U, int NS> hipError_t launch_ns(const SpmmArgs &a, int waves, hipStream_t s)
{
    // the per-wave LDS regions of a workgroup must fit 64 KB
    constexpr int MAXW = (SpmmCfg<BNB, 8, LB, RB, U, NS>::LDS <= 65536) ? 8 : ((SpmmCfg<BNB, 4, LB, RB, U, NS>::LDS <= 65536) ? 4 : ((SpmmCfg<BNB, 2, LB, RB, U, NS>::LDS <= 65536) ? 2 : 1));
    if (waves > MAXW) waves = MAXW;
    switch (waves) {
    case 1: return launch_one<BNB, 1, LB, RB, U, NS>(a, s);
    case 2: return launch_one<BNB, 2, LB, RB, U, NS>(a, s);
    case 4: return launch_one<BNB, (MAXW < 4 ? MAXW : 4), LB, RB, U, NS>(a, s);
    default: return launch_one<BNB, MAXW, LB, RB, U, NS>(a, s);
    }
}

template <int BNB, int LB, int RB, bool U = false> hipError_t launch_wk(const SpmmArgs &a, int waves, hipStream_t s)
{
    // two chunks in flight per wave whenever the lane offsets into B fit 32 bits (unsigned
    // operands keep to the one-chunk form to bound the number of kernels)
    // ... and no wave has more than SPMM_PIPE_CHUNKS chunks
    if constexpr (!U) if (a.stages == 2) {
        constexpr int MAXW2 = (SpmmCfg<BNB, 8, LB, RB, U, 2>::LDS <= 65536) ? 8 : ((SpmmCfg<BNB, 4, LB, RB, U, 2>::LDS <= 65536) ? 4 : ((SpmmCfg<BNB, 2, LB, RB, U, 2>::LDS <= 65536) ? 2 : 1));
        const int wv = waves > MAXW2 ? MAXW2 : (waves == 4 && MAXW2 < 4 ? MAXW2 : waves);
        if ((a.max_unit_chunks + wv - 1) / wv <= SPMM_PIPE_CHUNKS) return launch_ns<BNB, LB, RB, U, 2>(a, waves, s);
    }
    return launch_ns<BNB, LB, RB, U, 1>(a, waves, s);
}

// unsigned operands: tiles of 64 or 128 bytes
template <int LB, int RB> hipError_t launch_unsigned(const SpmmArgs &a, int bnb, int waves, hipStream_t s)
{
    if (bnb == 64) return launch_wk<64, LB, RB, true>(a, waves, s);
    return launch_wk<128, LB, RB, true>(a, waves, s);
}

template <int LB, int RB> hipError_t launch_mode(const SpmmArgs &a, int bnb, int waves, hipStream_t s)
{
    if (bnb == 64) return launch_wk<64, LB, RB>(a, waves, s);
    if (bnb == 256 && RB != 4) return launch_wk<256, (RB == 4 ? 8 : LB), (RB == 4 ? 8 : RB)>(a, waves, s);
    return launch_wk<128, LB, RB>(a, waves, s);
}

__global__ __launch_bounds__(256) void zero_rows_kernel(int32_t *C, int64_t ldc, int n, int V, const int32_t *panels)
{
    const int panel = panels[blockIdx.x];
    const int per_row = n / 4; // n is a multiple of 4 (16-byte pieces of int32)
    for (int p = threadIdx.x; p < V * per_row; p += 256) {
        const int row = p / per_row, col = (p % per_row) * 4;
        *reinterpret_cast<v4i *>(C + (int64_t)(panel * V + row) * ldc + col) = (v4i){0, 0, 0, 0};
    }
}

__global__ __launch_bounds__(256) void zero_ints_kernel(int32_t *p, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) reinterpret_cast<v4i *>(p)[i] = (v4i){0, 0, 0, 0};
}

__global__ __launch_bounds__(256) void finish_split_rows_kernel(const int32_t *acc, int n, int n_split, int V, const int32_t *panels,
                                                                void *C, int64_t ldc, int64_t C_batch_stride, int float_out, float scale)
{
    const int sp = blockIdx.x, batch = blockIdx.y, panel = panels[sp];
    const int per_row = n / 4;
    const int32_t *src = acc + ((int64_t)batch * n_split + sp) * V * n;
    for (int p = threadIdx.x; p < V * per_row; p += 256) {
        const int row = p / per_row, col = (p % per_row) * 4;
        const v4i s = *reinterpret_cast<const v4i *>(src + (int64_t)row * n + col);
        const v4f f = {s.x * scale, s.y * scale, s.z * scale, s.w * scale};
        const int64_t off = (int64_t)batch * C_batch_stride + (int64_t)(panel * V + row) * ldc + col;
        if (float_out == 2) *reinterpret_cast<mcu::v4h *>(static_cast<_Float16 *>(C) + off) = mcu::to_half4(f);
        else *reinterpret_cast<v4f *>(static_cast<float *>(C) + off) = f;
    }
}

} // namespace

hipError_t launch_zero_ints(int32_t *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t n4 = n / 4;
    hipLaunchKernelGGL(zero_ints_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, p, n4);
    return hipGetLastError();
}

hipError_t launch_finish_split_rows(const int32_t *acc, int n, int n_split, int V, int batch, const int32_t *panels, void *C,
                                    int64_t ldc, int64_t C_batch_stride, int float_out, float scale, hipStream_t s)
{
    if (n_split == 0 || batch == 0 || n == 0) return hipSuccess;
    hipLaunchKernelGGL(finish_split_rows_kernel, dim3((unsigned)n_split, (unsigned)batch), dim3(256), 0, s, acc, n, n_split, V, panels,
                       C, ldc, C_batch_stride, float_out, scale);
    return hipGetLastError();
}

hipError_t launch_zero_rows(int32_t *C, int64_t ldc, int n, int V, const int32_t *panels, int n_panels, hipStream_t s)
{
    if (n_panels == 0 || n == 0) return hipSuccess;
    hipLaunchKernelGGL(zero_rows_kernel, dim3((unsigned)n_panels), dim3(256), 0, s, C, ldc, n, V, panels);
    return hipGetLastError();
}

// The L8-R8 kernel on 128-byte tiles with two waves per panel and two chunks in flight, instrumented with time stamps
// (see PhaseClock): a.trace receives 10 stamps per wave, wave w of workgroup g at (g * 2 + w) * 10.
hipError_t launch_spmm_phase_probe(const SpmmArgs &a, hipStream_t s)
{
    if (a.P == 0 || a.row_bytes == 0) return hipSuccess;
    SpmmArgs b = a;
    b.ntiles = (a.row_bytes + 127) / 128;
    b.tile_shift = -1;
    for (int sh = 0; sh < 31; ++sh)
        if ((1 << sh) == b.ntiles) b.tile_shift = sh;
    hipLaunchKernelGGL((spmm_kernel<128, 2, 8, 8, false, 2, true>), dim3((unsigned)(a.P * b.ntiles)), dim3(128), 0, s, b);
    return hipGetLastError();
}

hipError_t launch_spmm(mc_prec prec, const SpmmArgs &a, int bnb, int waves, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0 || a.row_bytes == 0) return hipSuccess;
    if (a.lhs_unsigned || a.rhs_unsigned) {
        switch (prec) {
        case MC_L8R8: return launch_unsigned<8, 8>(a, bnb, waves, s);
        case MC_L8R4: return launch_unsigned<8, 4>(a, bnb, waves, s);
        case MC_L4R4: return launch_unsigned<4, 4>(a, bnb, waves, s);
        default: return hipErrorInvalidValue;
        }
    }
    switch (prec) {
    case MC_L8R8: return launch_mode<8, 8>(a, bnb, waves, s);
    case MC_L8R4: return launch_mode<8, 4>(a, bnb, waves, s);
    case MC_L4R4: return launch_mode<4, 4>(a, bnb, waves, s);
    case MC_L16R8: return launch_mode<16, 8>(a, bnb, waves, s);
    case MC_L16R16: return launch_mode<16, 16>(a, bnb, waves, s);
    case MC_L16R4:
    case MC_L12R4: return launch_mode<16, 4>(a, bnb, waves, s); // a 12-bit A is stored as two byte planes too
    }
    return hipErrorInvalidValue;
}
