// SpMM with the dense operand resident in LDS ("slab" form), for matrices dense enough that the
// rows of B named by the column indices are fetched many times over.
//
// The paper's kernel (Section 4.2) fetches, for every row panel, the B rows its vectors name and
// accepts that those rows have no reuse in on-chip memory.  On gfx950 a workgroup can hold
// 160 KB of LDS, and the transposing LDS read takes a per-lane address, so the "gather" can be
// served from LDS directly: a workgroup owns a 64-byte column tile of B and a group of row
// panels, walks over K in blocks of MC_KBLOCK rows, keeps the current block of its tile
// (64 KB) resident, and every chunk step reads its 64 rows straight out of that block -- the row
// numbers of the K-blocked format go into the addresses of ds_read_b64_tr_b8.  Per gathered byte
// this replaces one L2 -> LDS copy plus one LDS read by one LDS read, and B is fetched from L2
// once per workgroup instead of once per stored vector.
//
// Roles inside a workgroup: the last wave only fills (block b+1 into the second buffer while
// the others compute on block b; one workgroup barrier per block), the other waves own panels:
// the accumulators of a panel stay in the registers of its wave(s) over all K-blocks, so there
// is no partial-sum traffic and no atomic.  A row segment s of block row r sits at LDS position
// s ^ ((r >> 2) & 3) of the row: the eight rows of one transposing read then spread over the
// banks whatever their numbers are (measured: random rows read at 0.65 of the conflict-free rate).
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

constexpr int TILE_BYTES = 64;                       // bytes of a B row per workgroup
constexpr int BUF_BYTES = MC_KBLOCK * TILE_BYTES;     // one resident K-block of the tile
constexpr int SLAB_LDS = 2 * BUF_BYTES;               // two buffers: compute on one, fill the other

template <int LB, bool R4> struct SlabCfg {
    static constexpr bool L16 = (LB == 16);
    static constexpr int NACC = R4 ? 8 : 4;              // MFMA accumulators (v4i) per panel
    static constexpr int COLS = R4 ? 128 : 64;           // output columns of the tile
    static constexpr int OROWS = L16 ? 16 : 8;           // rows of a partial tile (two planes for a 16-bit A)
    static constexpr int TST = COLS + 4;                 // row stride (ints) of a staged tile
    static constexpr int PERWAVE = OROWS * TST * 4;      // bytes of one wave's staged tile
    static constexpr int SH = R4 ? (LB == 4 ? 8 : 4) : 0; // scale carried by widened nibbles
};

// Depth of the operand prefetch of a panel's chunk stream: the A operand and the row numbers of a chunk are
// requested PF chunks before they are used (they come from L2 or beyond; one chunk step is far shorter
// than that latency).
template <int PPW, bool R4> struct Prefetch { static constexpr int PF = 3; };

// PPW: panels per computing wave and pass (their accumulators live in registers at the same time)
template <int PPW, int LB, bool R4>
__global__ __launch_bounds__(1024) void spmm_slab_kernel(SlabArgs a)
{
    using Cfg = SlabCfg<LB, R4>;
    constexpr int NACC = Cfg::NACC, COLS = Cfg::COLS, TST = Cfg::TST, OROWS = Cfg::OROWS;
    constexpr int PF = Prefetch<PPW, R4>::PF;
    constexpr bool L16 = Cfg::L16;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform: everything derived from it stays in scalar registers
    // Workgroups go to the eight XCDs round-robin by their linear id.  The column tiles of one panel
    // group all read the same A operands, so they are given ids that are equal modulo 8: one XCD's L2
    // then fetches a group's A operands once for all tiles (and holds all of B, which is small).
    const int ntiles = (a.row_bytes + TILE_BYTES - 1) / TILE_BYTES;
    const int x = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int tile = q % ntiles, grp = (q / ntiles) * 8 + x, batch = blockIdx.y;
    if (grp >= a.groups) return;
    const int nb0 = tile * TILE_BYTES;
    const uint8_t *Bb = a.B + (int64_t)batch * a.B_batch_stride + nb0;
    const int nhalf = (!L16 && a.V > 8) ? 2 : 1;          // halves of 8 rows a finished tile is staged in
    const int slots = a.nc / a.wpp;                       // panels in work at the same time per PPW
    const int per_pass = slots * PPW;
    const int npass = (a.ppg + per_pass - 1) / per_pass;

    if (w >= a.nc) {
        // ---- the filling wave: block b of the tile -> buffer b & 1 -------------------------
        // Copy instruction i moves rows 16i .. 16i+15 of the block (four lanes per row); lane
        // (rr, pos) fetches the segment that belongs at LDS position pos of its row.  Segments
        // beyond the end of a B row are replaced by segment 0 (their columns are never stored),
        // rows beyond K by the last row (no chunk names them).
        const int rr = lane >> 2, pos = lane & 3;
        const int seg = pos ^ ((rr >> 2) & 3);
        const int segoff = (nb0 + seg * 16 < a.row_bytes) ? seg * 16 : 0;
        for (int pass = 0; pass < npass; ++pass) {
            for (int b = 0; b < a.nblk; ++b) {
                char *buf = lds + (b & 1) * BUF_BYTES;
                const int row0 = b * MC_KBLOCK;
                const int nrows = (a.K - row0 < MC_KBLOCK) ? a.K - row0 : MC_KBLOCK;
                const int ninstr = (nrows + 15) / 16;
                for (int i = w - a.nc; i < ninstr; i += a.nf) { // the filling waves take the copy instructions in turn
                    int r = row0 + i * 16 + rr;
                    if (r >= a.K) r = a.K - 1;
                    __builtin_amdgcn_global_load_lds((gptr_t *)(Bb + (int64_t)r * a.ldb_bytes + segoff), (lptr_t *)(buf + i * 1024), 16, 0, 0);
                }
                // block b has landed; the computing waves have finished block b-1, whose buffer the
                // next iteration overwrites
                asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
            }
            // the output stage of the computing waves uses the buffers: 2 barriers per panel of a wave and half of
            // its rows (a one-plane operand of 16 rows is staged in two halves), one more before the next pass may
            // fill again
            for (int i = 0; i < 2 * PPW * nhalf + (pass + 1 < npass ? 1 : 0); ++i) asm volatile("s_barrier" ::: "memory");
        }
        return;
    }

    // ---- computing waves ---------------------------------------------------------------------
    const int j = lane & 15, g = lane >> 4, ii = (lane & 15) >> 1, half = lane & 1;
    const int slot = w / a.wpp, k = w % a.wpp;            // this wave: panel slot, share of the panel's chunks
    const int g_begin = grp * a.ppg;
    const int g_end = (g_begin + a.ppg < a.P) ? g_begin + a.ppg : a.P;
    const uint8_t *vals = a.vals + (int64_t)batch * a.vals_batch_stride;
    const int ncols = R4 ? a.row_bytes * 2 : a.row_bytes;
    int *tile_w = reinterpret_cast<int *>(lds + w * Cfg::PERWAVE);

    for (int pass = 0; pass < npass; ++pass) {
        const int p_begin = g_begin + pass * per_pass;
        v4i acc[PPW][NACC];
        int bptr[PPW];            // lane l: first chunk of (panel, block l); lanes >= nblk: end of the panel
        int cur[PPW];             // this wave's next chunk of each of its panels
        // Operand prefetch.  The wave walks its (panel, block) lists in a fixed order (blocks outside, its
        // panels inside) and handles every list in groups of PF steps, a list of n chunks in max(1, ceil(n / PF))
        // groups whose surplus steps do nothing.  Step d of a group uses register set d and, after its MFMAs,
        // refills it with the operands of step d of the NEXT group (of the same list, or the first group of the
        // next list, which may lie beyond the coming barrier).  Every set is therefore loaded exactly PF steps
        // before its use, on every path, with compile-time set numbers and unconditional loads (a surplus step
        // loads some valid chunk again): the compiler's own counted waits are then exact -- a conditional load
        // or a rotation of the sets would make it copy registers, and a copy waits for the data.
        v4i ring_a[PF];
        int ring_r[PF];           // the two block rows this lane addresses: slot g*16 + ii (low half), g*16 + 8 + ii (high half)
        // (only loads: any arithmetic on the loaded registers here would have to wait for them)
        auto load_chunk = [&](int c, v4i &va, int &r) {
            va = mcu::load_a_raw<LB>(vals, c, a.V, j, g);
            r = reinterpret_cast<const int *>(a.blk_rows)[(int64_t)c * (MC_CHUNK / 2) + g * 8 + ii];
        };
        // this wave's chunks of list (panel i, block b): first, first + wpp, ... below the block's end
        auto list_len = [&](int first, int bend) { return first < bend ? (bend - first + a.wpp - 1) / a.wpp : 0; };
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
#pragma unroll
            for (int t = 0; t < NACC; ++t) acc[i][t] = (v4i){0, 0, 0, 0};
            const int p = p_begin + slot + i * slots;
            const bool valid = p < g_end;
            bptr[i] = valid ? a.blk_ptr[(int64_t)p * a.nblk + (lane < a.nblk ? lane : a.nblk)] : 0;
            cur[i] = __builtin_amdgcn_readlane(bptr[i], 0) + k;
        }
        {   // the first group of the first list
            const int len0 = list_len(cur[0], __builtin_amdgcn_readlane(bptr[0], 1));
#pragma unroll
            for (int d = 0; d < PF; ++d) load_chunk(len0 > 0 ? cur[0] + (d < len0 ? d : len0 - 1) * a.wpp : 0, ring_a[d], ring_r[d]);
        }

        for (int b = 0; b < a.nblk; ++b) {
            // block b has landed (the filling waves waited for their copies) and every wave is done with block
            // b-1 (its reads went into MFMAs that have been issued).  A bare barrier: the operand loads in
            // flight across it must not be waited for here.
            asm volatile("s_barrier" ::: "memory");
            const char *buf = lds + (b & 1) * BUF_BYTES;
            mcu::static_for<PPW>([&](auto Ic) {
                constexpr int i = decltype(Ic)::value;
                const int first = cur[i];
                const int len = list_len(first, __builtin_amdgcn_readlane(bptr[i], b + 1));
                const int ngroups = len > 0 ? (len + PF - 1) / PF : 1;
                // the list after this one: the wave's next panel in this block, or its first panel in the next block
                constexpr int ni = (i + 1 < PPW) ? i + 1 : 0;
                const int nb = (i + 1 < PPW) ? b : b + 1;
                const int nfirst = (i + 1 < PPW) ? cur[ni] : (PPW == 1 ? first + len * a.wpp : cur[0]);
                const int nlen = nb < a.nblk ? list_len(nfirst, __builtin_amdgcn_readlane(bptr[ni], nb + 1)) : 0;
                for (int gi = 0; gi < ngroups; ++gi) {
                    const bool last_group = gi + 1 == ngroups;
                    mcu::static_for<PF>([&](auto Dc) {
                        constexpr int d = decltype(Dc)::value;
                        const int pos = gi * PF + d;
                        if (pos < len) {
                            const v4i a_cur = mcu::finish_a<LB>(ring_a[d]);
                            const unsigned r0 = (unsigned)ring_r[d] & 0xFFFFu, r1 = (unsigned)ring_r[d] >> 16;
                            const unsigned o0 = r0 * TILE_BYTES + (((r0 >> 2) & 3) << 4) + 8 * half;
                            const unsigned o1 = r1 * TILE_BYTES + (((r1 >> 2) & 3) << 4) + 8 * half;
#pragma unroll
                            for (int ct = 0; ct < 4; ++ct) {
                                const v2i d0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(buf + (o0 ^ (ct * 16))));
                                const v2i d1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i *)(buf + (o1 ^ (ct * 16))));
                                const v4i bop = {d0.x, d0.y, d1.x, d1.y};
                                if (!R4) {
                                    acc[i][ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, bop, acc[i][ct], 0, 0, 0);
                                } else {
                                    const v4i msk = {(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
                                    const v4i be = (bop << 4) & msk, bo = bop & msk;
                                    acc[i][2 * ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, be, acc[i][2 * ct], 0, 0, 0);
                                    acc[i][2 * ct + 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a_cur, bo, acc[i][2 * ct + 1], 0, 0, 0);
                                }
                            }
                        }
                        // step d of the next group
                        int c;
                        if (!last_group) {
                            const int np = pos + PF;
                            c = first + (np < len ? np : len - 1) * a.wpp;
                        } else {
                            c = nlen > 0 ? nfirst + (d < nlen ? d : nlen - 1) * a.wpp : 0;
                        }
                        load_chunk(c, ring_a[d], ring_r[d]);
                    });
                }
                cur[i] = first + len * a.wpp;
            });
        }

        // ---- output: each wave stages its tile in its own LDS region; the waves of a panel then add their
        // tiles, finish the arithmetic and store 16 bytes per thread -------------------------------
        // accumulator register r of lane (j, g) is output row 4g + r; MFMA ct covers tile bytes 16ct .. 16ct+15,
        // i.e. column 16ct + j (8-bit B) or columns 32ct + 2j, 2j+1 (4-bit B)
#pragma unroll
        for (int i = 0; i < PPW; ++i) {
            for (int hf = 0; hf < nhalf; ++hf) {
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); // the slab (or the previous tiles) is no longer read
                const int gg = g - 2 * hf;                // lane groups 2 hf, 2 hf + 1 hold rows 8 hf .. 8 hf + 7 of a one-plane tile
                if (gg >= 0 && 4 * gg < OROWS) {
#pragma unroll
                    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if (!R4) tile_w[(4 * gg + r) * TST + ct * 16 + j] = acc[i][ct][r];
                            else *reinterpret_cast<v2i *>(&tile_w[(4 * gg + r) * TST + ct * 32 + 2 * j]) = (v2i){acc[i][2 * ct][r], acc[i][2 * ct + 1][r]};
                        }
                }
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); // the staged tiles are complete
                const int p = p_begin + slot + i * slots;
                if (p < g_end) {
                    constexpr int PIECES = 8 * (COLS / 4);
                    for (int pc = k * 64 + lane; pc < PIECES; pc += 64 * a.wpp) {
                        const int trow = pc / (COLS / 4), col = (pc % (COLS / 4)) * 4;
                        const int row = trow + 8 * hf, gcol = tile * COLS + col;
                        if (row >= a.V || p * a.V + row >= a.rows || gcol >= ncols) continue;
                        v4i s = {0, 0, 0, 0}, lo = {0, 0, 0, 0};
                        for (int ww = 0; ww < a.wpp; ++ww) {
                            const int *t = reinterpret_cast<const int *>(lds + (slot * a.wpp + ww) * Cfg::PERWAVE);
                            s += *reinterpret_cast<const v4i *>(&t[trow * TST + col]);
                            if (L16) lo += *reinterpret_cast<const v4i *>(&t[(trow + 8) * TST + col]);
                        }
                        // every plane sum is exact in int32 (4-bit B: after its shift); the recombination wraps
                        if (R4) { s = s >> Cfg::SH; lo = lo >> Cfg::SH; }
                        if (L16) s = (s << 8) + lo;
                        const int64_t off = (int64_t)batch * a.C_batch_stride + (int64_t)(p * a.V + row) * a.ldc + gcol;
                        if (a.float_out) {
                            const v4f f = {s.x * a.out_scale, s.y * a.out_scale, s.z * a.out_scale, s.w * a.out_scale};
                            if (a.float_out == 2) __builtin_nontemporal_store(mcu::to_half4(f), reinterpret_cast<mcu::v4h *>(static_cast<_Float16 *>(a.C) + off));
                            else __builtin_nontemporal_store(f, reinterpret_cast<v4f *>(static_cast<float *>(a.C) + off));
                        } else {
                            __builtin_nontemporal_store(s, reinterpret_cast<v4i *>(static_cast<int32_t *>(a.C) + off));
                        }
                    }
                }
            }
        }
        if (pass + 1 < npass) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); // the staged tiles have been read before the next pass fills the buffers
    }
}

template <int PPW, int LB, bool R4> hipError_t launch_one(const SlabArgs &a, hipStream_t s)
{
    auto kern = spmm_slab_kernel<PPW, LB, R4>;
    // more than 64 KB of LDS per workgroup has to be asked for
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, SLAB_LDS);
    if (e != hipSuccess) return e;
    const int ntiles = (a.row_bytes + TILE_BYTES - 1) / TILE_BYTES;
    // ids of the same panel group are equal modulo 8 (see the kernel): groups are rounded up to a multiple of 8
    dim3 grid((unsigned)((a.groups + 7) / 8 * 8 * ntiles), (unsigned)a.batch), block(64 * (a.nc + a.nf));
    hipLaunchKernelGGL(kern, grid, block, SLAB_LDS, s, a);
    return hipGetLastError();
}

template <int LB, bool R4> hipError_t launch_ppw(const SlabArgs &a, int ppw, hipStream_t s)
{
    if (ppw == 1) return launch_one<1, LB, R4>(a, s);
    if (ppw == 2) return launch_one<2, LB, R4>(a, s);
    if constexpr (!R4) {
        if (ppw == 4) return launch_one<4, LB, R4>(a, s);
    }
    return hipErrorInvalidValue;
}

// values in interchange order -> K-blocked value array, one thread per slot (8 / 16 bits) or per pair of
// slots (b, b + 8) that share bytes (4 bits)
__global__ __launch_bounds__(256) void repack_blocked_kernel(const int32_t *blk_src, const uint8_t *src, uint8_t *dst, int64_t nchunks,
                                                             int V, int bits)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (bits == 8 || bits == 16) {
        if (t >= nchunks * MC_CHUNK) return;
        const int i = (int)(t % MC_CHUNK), g = i / 16, b = i % 16;
        const int64_t vec = blk_src[t];
        uint8_t *chunk = dst + (t / MC_CHUNK) * (MC_CHUNK * V * bits / 8);
        for (int v = 0; v < V; ++v) {
            if (bits == 8) {
                chunk[g * (16 * V) + v * 16 + b] = (vec >= 0) ? src[vec * V + v] : (uint8_t)0;
            } else {
                const int x = (vec >= 0) ? reinterpret_cast<const int16_t *>(src)[vec * V + v] : 0;
                const int hi = (x + 128) >> 8, lo = x - hi * 256;
                chunk[g * (32 * V) + v * 16 + b] = (uint8_t)hi;
                chunk[g * (32 * V) + 16 * V + v * 16 + b] = (uint8_t)lo;
            }
        }
    } else {
        if (t >= nchunks * (MC_CHUNK / 2)) return;
        const int64_t ch = t / 32;
        const int g = (int)(t % 32) / 8, b = (int)(t % 8);
        const int64_t v_lo = blk_src[ch * MC_CHUNK + g * 16 + b], v_hi = blk_src[ch * MC_CHUNK + g * 16 + b + 8];
        uint8_t *chunk = dst + ch * (MC_CHUNK * V / 2);
        for (int v = 0; v < V; ++v) {
            int nl = 0, nh = 0;
            if (v_lo >= 0) { const int64_t e = v_lo * V + v; nl = (src[e >> 1] >> ((e & 1) * 4)) & 15; }
            if (v_hi >= 0) { const int64_t e = v_hi * V + v; nh = (src[e >> 1] >> ((e & 1) * 4)) & 15; }
            chunk[g * (8 * V) + v * 8 + b] = (uint8_t)(nl | (nh << 4));
        }
    }
}

} // namespace

int spmm_slab_lds_bytes() { return SLAB_LDS; }

hipError_t launch_spmm_slab(mc_prec prec, const SlabArgs &a, int ppw, hipStream_t s)
{
    if (a.P == 0 || a.batch == 0 || a.row_bytes == 0) return hipSuccess;
    switch (prec) {
    case MC_L8R8: return launch_ppw<8, false>(a, ppw, s);
    case MC_L8R4: return launch_ppw<8, true>(a, ppw, s);
    case MC_L4R4: return launch_ppw<4, true>(a, ppw, s);
    case MC_L16R8: return launch_ppw<16, false>(a, ppw, s);
    case MC_L16R4:
    case MC_L12R4: return launch_ppw<16, true>(a, ppw, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_repack_blocked(const int32_t *blk_src, const uint8_t *src, uint8_t *dst, int64_t nchunks, int V, int bits,
                                 hipStream_t s)
{
    if (nchunks == 0) return hipSuccess;
    const int64_t threads = nchunks * (bits == 4 ? MC_CHUNK / 2 : MC_CHUNK);
    hipLaunchKernelGGL(repack_blocked_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, blk_src, src, dst, nchunks, V, bits);
    return hipGetLastError();
}
