// One 16-vector tile step of the SDDMM (paper, Section 4.3), shared by the kernels that compute scores:
// operand widening / plane splitting in registers, the MFMA step and the Q operand load.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mcs {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

constexpr int SDDMM_WAVES = 4;
constexpr int NIBBLE_HI = (int)0xF0F0F0F0;

// Packed int4 -> two int8 operands holding 16 x the signed nibbles (even / odd elements).
__device__ __forceinline__ void widen4(v4i x, v4i &even, v4i &odd)
{
    const v4i m = {NIBBLE_HI, NIBBLE_HI, NIBBLE_HI, NIBBLE_HI};
    even = (x << 4) & m;
    odd = x & m;
}

// 16 little-endian int16 elements (x: the first 8, y: the last 8) -> their signed byte planes
// e = 256 * hi + lo with lo the low byte read as int8 and hi = (e + 128) >> 8 (Section 4.4 with
// both planes signed; needs e <= 32639).  Byte t of a plane register belongs to element t of
// the 32-byte piece on both operand sides, so the planes of Q and Kmat pair up term by term.
__device__ __forceinline__ void split16(v4i x, v4i y, v4i &hi, v4i &lo)
{
    typedef unsigned short v8us __attribute__((ext_vector_type(8)));
    const v8us half = {128, 128, 128, 128, 128, 128, 128, 128};
    const v4i xr = __builtin_bit_cast(v4i, (v8us)(__builtin_bit_cast(v8us, x) + half));
    const v4i yr = __builtin_bit_cast(v4i, (v8us)(__builtin_bit_cast(v8us, y) + half));
    // v_perm_b32 picks bytes from {first operand: bytes 4..7, second operand: bytes 0..3}
    constexpr unsigned EVEN = 0x06040200u, ODD = 0x07050301u;
    lo = (v4i){(int)__builtin_amdgcn_perm(x.y, x.x, EVEN), (int)__builtin_amdgcn_perm(x.w, x.z, EVEN),
               (int)__builtin_amdgcn_perm(y.y, y.x, EVEN), (int)__builtin_amdgcn_perm(y.w, y.z, EVEN)};
    hi = (v4i){(int)__builtin_amdgcn_perm(xr.y, xr.x, ODD), (int)__builtin_amdgcn_perm(xr.w, xr.z, ODD),
               (int)__builtin_amdgcn_perm(yr.y, yr.x, ODD), (int)__builtin_amdgcn_perm(yr.w, yr.z, ODD)};
}

// One reduction step of a 16-vector tile.  PB = operand width in bits.
//   8:  q, k are the operands.
//   4:  q, k hold packed nibbles; both are widened (16 x value) and multiplied pairwise.
//   16: q is ONE plane of the Q row (lanes 0..7 of a group of 16 carry the high plane of Q
//       rows 0..7, lanes 8..15 the low plane: the planes are stacked in the MFMA rows), kh / kl
//       are the planes of the Kmat piece; acc takes q x kh and acc2 takes q x kl.
template <int PB>
__device__ __forceinline__ void mma_step(v4i q, v4i k, v4i k2, v4i &acc, v4i &acc2)
{
    if (PB == 4) {
        v4i qe, qo, ke, ko;
        widen4(q, qe, qo);
        widen4(k, ke, ko);
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(qe, ke, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(qo, ko, acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(q, k, acc, 0, 0, 0);
        if (PB == 16) acc2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(q, k2, acc2, 0, 0, 0);
    }
}

// Finishes a tile's accumulators.  16 bit: rows 0..7 hold Qh.Kh (acc) and Qh.Kl (acc2), rows
// 8..15 (32 lanes further up) hold Ql.Kh and Ql.Kl; S = (QhKh << 16) + ((QhKl + QlKh) << 8) + QlKl.
template <int PB> __device__ __forceinline__ v4i finish_tile(v4i acc, v4i acc2)
{
    if (PB == 4) return acc >> 8; // both operands carried a factor 16
    if (PB == 16) {
        v4i up, up2;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            up[r] = __shfl_xor(acc[r], 32);
            up2[r] = __shfl_xor(acc2[r], 32);
        }
        return (acc << 16) + ((acc2 + up) << 8) + up2; // meaningful in lanes 0..31 only
    }
    return acc;
}

// Bytes of a row that one MFMA step consumes (64 operand bytes per plane).
template <int PB> struct StepBytes { static constexpr int value = (PB == 16) ? 128 : 64; };

// The Q operand of step kc for this lane, straight from memory (zero outside the panel's rows
// and beyond the row end).  j = lane % 16, g = lane / 16.
template <int PB>
__device__ __forceinline__ v4i load_q(const uint8_t *Qpanel, int64_t ldq_bytes, int V, int row_bytes, int kc, int j, int g)
{
    v4i q = {0, 0, 0, 0};
    if (PB == 16) {
        const int off = kc * 128 + g * 32;
        if ((j & 7) < V && off < row_bytes) {
            const uint8_t *p = Qpanel + (int64_t)(j & 7) * ldq_bytes + off;
            const v4i x = *reinterpret_cast<const v4i *>(p);
            v4i y = {0, 0, 0, 0};
            if (off + 16 < row_bytes) y = *reinterpret_cast<const v4i *>(p + 16);
            v4i hi, lo;
            split16(x, y, hi, lo);
            q = (j < 8) ? hi : lo;
        }
    } else {
        const int off = kc * 64 + g * 16;
        if (j < V && off < row_bytes) q = *reinterpret_cast<const v4i *>(Qpanel + (int64_t)j * ldq_bytes + off);
    }
    return q;
}

} // namespace mcs
