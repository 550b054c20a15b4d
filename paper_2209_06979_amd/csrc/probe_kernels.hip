// Measurement aid, not part of the arithmetic path: the gather of an SpMM and nothing else.
//
// The kernel has the work split, index loads and global->LDS row copies of spmm_kernel
// (workgroup = (panel, BNB bytes of every gathered B row), WK waves taking the panel's chunks
// round-robin, one chunk in flight per wave) but no A values, no LDS reads, no MFMA and no
// output tile.  Its run time is the floor that the memory system sets for "fetch the B rows
// named by these column indices into LDS in this launch shape"; the SpMM's time is reported
// as a multiple of it.  Every workgroup writes one word taken from its staged rows, which
// keeps the copies observable and lets a test check that the right rows arrived.
#include "internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

template <int BNB, int WK>
__global__ __launch_bounds__(64 * WK) void gather_probe_kernel(SpmmArgs a, int32_t *sink)
{
    constexpr int LPR = BNB / 16, NI = LPR, SWZ = (LPR == 4) ? 3 : 7;
    __shared__ __attribute__((aligned(16))) char lds[WK * 64 * BNB];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int rg = lane / LPR, seg = lane % LPR;
    const int ntiles = (a.row_bytes + BNB - 1) / BNB;
    const int panel = blockIdx.x / ntiles, tile = blockIdx.x % ntiles;
    const int nb0 = tile * BNB;
    // (the panel's first slot and chunk count as spmm_kernel finds them: computed when all panels are equally long)
    int s0, nch;
    if (a.uniform_chunks > 0) {
        s0 = panel * a.uniform_chunks * MC_CHUNK;
        nch = a.uniform_chunks;
    } else {
        const int2 pp = *reinterpret_cast<const int2 *>(a.panel_ptr + 2 * panel);
        s0 = pp.x;
        nch = (pp.y - s0 + MC_CHUNK - 1) / MC_CHUNK;
    }
    const int32_t *idx = a.slot_idx + s0;
    const uint8_t *Bb = a.B + nb0;
    char *stage = lds + w * (64 * BNB);

    int segoff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int lseg = seg ^ (i & SWZ);
        segoff[i] = (nb0 + lseg * 16 < a.row_bytes) ? lseg * 16 : 0;
    }
    const int nmy = (nch > w) ? (nch - w + WK - 1) / WK : 0;
    for (int k = 0; k < nmy; ++k) {
        const int c = w + k * WK;
        v4i idxv[NI / 4];
#pragma unroll
        for (int t = 0; t < NI / 4; ++t) idxv[t] = *reinterpret_cast<const v4i *>(idx + c * MC_CHUNK + rg * NI + 4 * t);
#pragma unroll
        for (int i = 0; i < NI; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t *)(Bb + (int64_t)idxv[i >> 2][i & 3] * a.ldb_bytes + segoff[i]),
                                             (lptr_t *)(stage + i * 1024), 16, 0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    // first word of wave 0's stage: bytes nb0 .. nb0+3 of the B row named by the first slot of
    // the last chunk that wave 0 copied (lane 0 of copy instruction 0 fetches segment 0)
    if (tid == 0) sink[blockIdx.x] = (nch > 0) ? *reinterpret_cast<const int32_t *>(lds) : 0;
}

template <int BNB> hipError_t launch_bnb(const SpmmArgs &a, int waves, int32_t *sink, hipStream_t s)
{
    const int ntiles = (a.row_bytes + BNB - 1) / BNB;
    dim3 grid((unsigned)(a.P * ntiles));
    constexpr int MAXW = (64 * BNB * 8 <= 65536) ? 8 : 4;
    if (waves > MAXW) waves = MAXW;
    switch (waves) {
    case 1: hipLaunchKernelGGL((gather_probe_kernel<BNB, 1>), grid, dim3(64), 0, s, a, sink); break;
    case 2: hipLaunchKernelGGL((gather_probe_kernel<BNB, 2>), grid, dim3(128), 0, s, a, sink); break;
    case 4: hipLaunchKernelGGL((gather_probe_kernel<BNB, 4>), grid, dim3(256), 0, s, a, sink); break;
    default: hipLaunchKernelGGL((gather_probe_kernel<BNB, MAXW>), grid, dim3(64 * MAXW), 0, s, a, sink); break;
    }
    return hipGetLastError();
}

// The matrix unit alone: every wave issues `iters` rounds of eight independent v_mfma_i32_16x16x64_i8 on
// registers (no memory traffic inside the loop); the sums go to `sink` so that nothing is optimised away.
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, int32_t *sink)
{
    v4i acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = (v4i){0, 0, 0, 0};
    const int l = threadIdx.x;
    v4i a = {l, l + 1, l + 2, l + 3}, b = {l * 3, l * 5, l * 7, l * 11};
    const long long c0 = __builtin_readcyclecounter(), t0 = wall_clock64();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[t], 0, 0, 0);
    }
    v4i s = acc[0];
#pragma unroll
    for (int t = 1; t < 8; ++t) s += acc[t];
    int out = s.x + s.y + s.z + s.w;
    // the first wave of the launch reports its own loop: shader-clock cycles and ticks of the constant 100 MHz clock
    const long long c1 = __builtin_readcyclecounter(), t1 = wall_clock64();
    if (blockIdx.x == 0 && l == 0) out = (int)(c1 - c0);
    if (blockIdx.x == 0 && l == 1) out = (int)(t1 - t0);
    sink[(size_t)blockIdx.x * 256 + l] = out;
}

} // namespace

hipError_t launch_mfma_probe(int workgroups, int iters, int32_t *sink, hipStream_t s)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, s, iters, sink);
    return hipGetLastError();
}

hipError_t launch_gather_probe(const SpmmArgs &a, int bnb, int waves, int32_t *sink, hipStream_t s)
{
    if (a.P == 0 || a.row_bytes == 0) return hipSuccess;
    if (bnb == 64) return launch_bnb<64>(a, waves, sink, s);
    if (bnb == 256) return launch_bnb<256>(a, waves, sink, s);
    return launch_bnb<128>(a, waves, sink, s);
}
