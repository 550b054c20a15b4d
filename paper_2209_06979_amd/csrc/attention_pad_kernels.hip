// Launchers of the fused attention kernel for head dimensions that do not fill its tile of 64 or 128
// elements (any multiple of 16; of 32 for 4-bit inputs): one head per workgroup, the missing pieces of
// every row read as zeros (see PAD in attention_fused.h).
#include "attention_fused.h"

namespace {
template <int PB, int QB, int DK> hipError_t launch_padded(const AttnArgs &a, int waves_per_panel, hipStream_t s)
{
    const dim3 grid((unsigned)a.P * (unsigned)a.heads, (unsigned)a.batch);
    if (waves_per_panel == 8) hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 8, DK, true>), grid, dim3(512), 0, s, a);
    else if (waves_per_panel == 4) hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 4, DK, true>), grid, dim3(256), 0, s, a);
    else if (waves_per_panel == 2) hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 2, DK, true>), grid, dim3(128), 0, s, a);
    else hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 1, DK, true>), grid, dim3(64), 0, s, a);
    return hipGetLastError();
}
} // namespace

// tile: 64 or 128, the kernel's head dimension; a.real_pieces * 16 bytes is what a row really has
// (fewer than tile * qkv_bits / 8), a.out_cols the real head dimension.
hipError_t launch_attention_fused_padded(const AttnArgs &a, int waves_per_panel, int p_bits, int qkv_bits, int tile, hipStream_t s)
{
    if (a.P == 0 || a.heads == 0 || a.batch == 0) return hipSuccess;
    if (a.real_pieces <= 0 || a.real_pieces * 16 >= tile * qkv_bits / 8 || a.out_cols <= 0 || a.out_cols >= tile) return hipErrorInvalidValue;
    if (tile == 128) {
        if (p_bits == 16) return (qkv_bits == 4) ? launch_padded<16, 4, 128>(a, waves_per_panel, s) : launch_padded<16, 8, 128>(a, waves_per_panel, s);
        return (qkv_bits == 4) ? launch_padded<8, 4, 128>(a, waves_per_panel, s) : launch_padded<8, 8, 128>(a, waves_per_panel, s);
    }
    if (tile != 64) return hipErrorInvalidValue;
    if (p_bits == 16) return (qkv_bits == 4) ? launch_padded<16, 4, 64>(a, waves_per_panel, s) : launch_padded<16, 8, 64>(a, waves_per_panel, s);
    return (qkv_bits == 4) ? launch_padded<8, 4, 64>(a, waves_per_panel, s) : launch_padded<8, 8, 64>(a, waves_per_panel, s);
}
