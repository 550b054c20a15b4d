// The sparse operand's side of one MFMA step, shared by the SpMM kernels.
#pragma once

#include "lds_async.h"

namespace mcu {

// A operand of one chunk for this lane (row = lane % 16, lane group = lane / 16).
// LB: stored width of A (4, 8 or 16 bits; a 12-bit operand is stored as 16).
template <int LB>
__device__ __forceinline__ v4i load_a(const uint8_t *vals, int64_t chunk, int V, int row, int g)
{
    v4i a = {0, 0, 0, 0};
    if (LB == 16) {
        // [chunk][g][plane hi, lo][v][16]; high plane in rows 0..V-1, low plane in rows 8..8+V-1
        const int v = row & 7;
        if (v < V) a = *reinterpret_cast<const v4i *>(vals + chunk * (128 * V) + g * (32 * V) + (row >> 3) * (16 * V) + v * 16);
    } else if (LB == 4) {
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


// The same operand in two steps, for kernels that request it several chunks ahead: load_a_raw only loads
// (so that nothing has to wait for the data yet), finish_a turns the loaded registers into the MFMA operand.
// MFMA rows beyond the V rows of a panel (whose results are never stored) receive a copy of row 0 instead
// of zeros: the load then needs no per-lane condition.
template <int LB>
__device__ __forceinline__ v4i load_a_raw(const uint8_t *vals, int64_t chunk, int V, int row, int g)
{
    if (LB == 16) {
        const int v = ((row & 7) < V) ? (row & 7) : 0;
        return *reinterpret_cast<const v4i *>(vals + chunk * (128 * V) + g * (32 * V) + (row >> 3) * (16 * V) + v * 16);
    } else if (LB == 4) {
        const int v = (row < V) ? row : 0;
        const v2i x = *reinterpret_cast<const v2i *>(vals + chunk * (32 * V) + g * (8 * V) + v * 8);
        return (v4i){x.x, x.y, 0, 0};
    } else {
        const int v = (row < V) ? row : 0;
        return *reinterpret_cast<const v4i *>(vals + chunk * (64 * V) + g * (16 * V) + v * 16);
    }
}
template <int LB> __device__ __forceinline__ v4i finish_a(v4i raw)
{
    if (LB == 4) return (v4i){(raw.x << 4) & (int)0xF0F0F0F0, (raw.y << 4) & (int)0xF0F0F0F0, raw.x & (int)0xF0F0F0F0, raw.y & (int)0xF0F0F0F0};
    return raw;
}

} // namespace mcu
