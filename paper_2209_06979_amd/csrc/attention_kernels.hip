// Launchers of the fused attention kernel for head dimensions 64 and 128 (rows that fill the kernel's tile).
#include "attention_fused.h"

int attention_fused_max_vectors() { return 8 * 8 * 64; }

template <int PB, int QB, int DK> hipError_t launch_pq(const AttnArgs &a, int heads_per_group, int waves_per_panel, hipStream_t s)
{
    if (heads_per_group == 2 && waves_per_panel == 8) return hipErrorInvalidValue;
    if (heads_per_group == 2) {
        // (16-bit codes with 4-bit Q/K/V: the two-plane output tile does not fit the stage; rows of 128
        // bytes: one head per workgroup)
        if constexpr ((PB == 16 && QB == 4) || (DK == 128 && QB == 8)) return hipErrorInvalidValue;
        else {
            const dim3 grid((unsigned)a.P * (unsigned)(a.heads / 2), (unsigned)a.batch);
            if (waves_per_panel == 4) hipLaunchKernelGGL((attention_fused_kernel<8, 2, PB, QB, 4, DK>), grid, dim3(512), 0, s, a);
            else if (waves_per_panel == 2) hipLaunchKernelGGL((attention_fused_kernel<8, 2, PB, QB, 2, DK>), grid, dim3(256), 0, s, a);
            else hipLaunchKernelGGL((attention_fused_kernel<8, 2, PB, QB, 1, DK>), grid, dim3(128), 0, s, a);
        }
    } else if (waves_per_panel == 8) {
        hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 8, DK>), dim3((unsigned)a.P * (unsigned)a.heads, (unsigned)a.batch), dim3(512), 0, s, a);
    } else if (waves_per_panel == 4) {
        hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 4, DK>), dim3((unsigned)a.P * (unsigned)a.heads, (unsigned)a.batch), dim3(256), 0, s, a);
    } else if (waves_per_panel == 2) {
        hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 2, DK>), dim3((unsigned)a.P * (unsigned)a.heads, (unsigned)a.batch), dim3(128), 0, s, a);
    } else {
        hipLaunchKernelGGL((attention_fused_kernel<8, 1, PB, QB, 1, DK>), dim3((unsigned)a.P * (unsigned)a.heads, (unsigned)a.batch), dim3(64), 0, s, a);
    }
    return hipGetLastError();
}

// waves_per_panel: 1, 2, 4 or 8 waves share the chunks of one (panel, head) (8: one head per workgroup only); a wave
// holds at most 8 chunks of scores in registers, so a panel may have up to 512 * waves_per_panel vectors.
// dk: 64 or 128
hipError_t launch_attention_fused(const AttnArgs &a, int heads_per_group, int waves_per_panel, int p_bits, int qkv_bits,
                                  int dk, hipStream_t s)
{
    if (a.P == 0 || a.heads == 0 || a.batch == 0) return hipSuccess;
    if (dk == 128) {
        if (p_bits == 16) return (qkv_bits == 4) ? launch_pq<16, 4, 128>(a, heads_per_group, waves_per_panel, s)
                                                 : launch_pq<16, 8, 128>(a, heads_per_group, waves_per_panel, s);
        return (qkv_bits == 4) ? launch_pq<8, 4, 128>(a, heads_per_group, waves_per_panel, s)
                               : launch_pq<8, 8, 128>(a, heads_per_group, waves_per_panel, s);
    }
    if (dk != 64) return hipErrorInvalidValue;
    if (p_bits == 16) return (qkv_bits == 4) ? launch_pq<16, 4, 64>(a, heads_per_group, waves_per_panel, s)
                                             : launch_pq<16, 8, 64>(a, heads_per_group, waves_per_panel, s);
    return (qkv_bits == 4) ? launch_pq<8, 4, 64>(a, heads_per_group, waves_per_panel, s)
                           : launch_pq<8, 8, 64>(a, heads_per_group, waves_per_panel, s);
}
