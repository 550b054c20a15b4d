// First step of the quantized attention layer (paper, Section 5.3): symmetric per-tensor
// quantisation of the projections' fp32 output to int8 or packed int4 codes.
//   absmax:   max |x| over the tensor (the scale is max|x| / qmax, taken by the caller)
//   quantize: q = clamp(rint(x / scale), -qmax, qmax), ties to even.
// Both are single passes over the tensor, 16 bytes per lane and load: pure HBM streaming.
// The code decision is taken as in double precision: an fp32 quotient decides unless it lies
// within 1e-3 of a rounding boundary, and only those lanes repeat the division in fp64.
#include "internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

__global__ void absmax_init_kernel(float *result) { *result = 0.f; }

// Each workgroup streams one contiguous span with eight independent 16-byte loads in flight per
// lane; the loads are non-temporal (the tensor is read once and is far larger than any cache).
// The result cell is read before the atomic: almost every workgroup finds a value at least as
// large already there and skips it (thousands of atomics on one address would otherwise cost
// more than the streaming itself).
__global__ __launch_bounds__(256) void absmax_kernel(const float *x, int64_t n, float *result)
{
    constexpr int U = 8;
    const v4f *xv = reinterpret_cast<const v4f *>(x);
    const int64_t nv = n / 4, per = (nv + gridDim.x - 1) / gridDim.x;
    const int64_t b = (int64_t)blockIdx.x * per, e = (b + per < nv) ? b + per : nv;
    float m = 0.f;
    auto take = [&](v4f v) { m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)))); };
    int64_t i = b + threadIdx.x;
    for (; i + (U - 1) * 256 < e; i += U * 256) {
        v4f v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(&xv[i + u * 256]);
#pragma unroll
        for (int u = 0; u < U; ++u) take(v[u]);
    }
    for (; i < e; i += 256) take(xv[i]);
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - nv * 4)) m = fmaxf(m, fabsf(x[nv * 4 + threadIdx.x]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    __shared__ float red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        // non-negative floats order like their bit patterns
        unsigned *cell = reinterpret_cast<unsigned *>(result);
        if (__float_as_uint(m) > __atomic_load_n(cell, __ATOMIC_RELAXED)) atomicMax(cell, __float_as_uint(m));
    }
}

// inv = 1 / scale rounded to fp32.  x * inv is within 1.5 units in the last place of x / scale,
// i.e. within 2e-5 for every quotient that is not clamped anyway, far inside the 1e-3 window in
// which the decision is handed to fp64.
__device__ __forceinline__ int code_of(float x, float scale, float inv, float qmax)
{
    const float r = x * inv;
    float q = rintf(r);
    if (fabsf(fabsf(r - truncf(r)) - 0.5f) < 1e-3f) q = (float)rint((double)x / (double)scale); // near a tie: decide in fp64
    return (int)fminf(fmaxf(q, -qmax), qmax);
}

// 8 elements per thread and unit: two 16-byte loads, one 8-byte (int8) or 4-byte (int4) store.  Each
// workgroup owns a contiguous span of units and keeps the loads of four units in flight per lane;
// loads and stores are non-temporal (everything is touched once).
template <int BITS> __global__ __launch_bounds__(256) void quantize_kernel(const float *x, int64_t n, float scale, uint8_t *q)
{
    constexpr int U = 4;
    const float qmax = (BITS == 8) ? 127.f : 7.f, inv = 1.f / scale;
    const v4f *xv = reinterpret_cast<const v4f *>(x);
    const int64_t n8 = n / 8, per = (n8 + gridDim.x - 1) / gridDim.x;
    const int64_t b = (int64_t)blockIdx.x * per, e = (b + per < n8) ? b + per : n8;
    auto emit = [&](int64_t i, v4f a, v4f c4) {
        const int c[8] = {code_of(a.x, scale, inv, qmax), code_of(a.y, scale, inv, qmax), code_of(a.z, scale, inv, qmax),
                          code_of(a.w, scale, inv, qmax), code_of(c4.x, scale, inv, qmax), code_of(c4.y, scale, inv, qmax),
                          code_of(c4.z, scale, inv, qmax), code_of(c4.w, scale, inv, qmax)};
        if (BITS == 8) {
            unsigned lo = 0, hi = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                lo |= (unsigned)(c[t] & 255) << (8 * t);
                hi |= (unsigned)(c[4 + t] & 255) << (8 * t);
            }
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            __builtin_nontemporal_store((v2u){lo, hi}, reinterpret_cast<v2u *>(q) + i);
        } else {
            unsigned w = 0;
#pragma unroll
            for (int t = 0; t < 8; ++t) w |= (unsigned)(c[t] & 15) << (4 * t); // element 2j in bits 3:0 of byte j
            __builtin_nontemporal_store(w, reinterpret_cast<unsigned *>(q) + i);
        }
    };
    int64_t i = b + threadIdx.x;
    for (; i + (U - 1) * 256 < e; i += U * 256) {
        v4f lo[U], hi[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            lo[u] = __builtin_nontemporal_load(&xv[2 * (i + u * 256)]);
            hi[u] = __builtin_nontemporal_load(&xv[2 * (i + u * 256) + 1]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) emit(i + u * 256, lo[u], hi[u]);
    }
    for (; i < e; i += 256) emit(i, xv[2 * i], xv[2 * i + 1]);
    // tail of fewer than 8 elements (n is even for 4-bit codes)
    if (blockIdx.x == 0) {
        const int64_t t0 = n8 * 8;
        if (BITS == 8) {
            if (threadIdx.x < (int)(n - t0)) q[t0 + threadIdx.x] = (uint8_t)(code_of(x[t0 + threadIdx.x], scale, inv, qmax) & 255);
        } else if (threadIdx.x < (int)((n - t0) / 2)) {
            const int64_t e = t0 + 2 * threadIdx.x;
            q[e / 2] = (uint8_t)((code_of(x[e], scale, inv, qmax) & 15) | ((code_of(x[e + 1], scale, inv, qmax) & 15) << 4));
        }
    }
}

// units of 256 threads' worth of work, at most `cap` workgroups (measured on 128 Mi elements: the
// read-only reduction is fastest with 512 .. 2048 workgroups, the read-write pass with about 16384)
inline unsigned grid_for(int64_t units, int64_t cap)
{
    const int64_t blocks = (units + 255) / 256;
    return (unsigned)(blocks < 1 ? 1 : (blocks > cap ? cap : blocks));
}

} // namespace

hipError_t launch_absmax(const float *x, int64_t n, float *result, hipStream_t s)
{
    hipLaunchKernelGGL(absmax_init_kernel, dim3(1), dim3(1), 0, s, result);
    if (n > 0) hipLaunchKernelGGL(absmax_kernel, dim3(grid_for(n / 4, 1024)), dim3(256), 0, s, x, n, result);
    return hipGetLastError();
}

hipError_t launch_quantize(const float *x, int64_t n, float scale, int bits, uint8_t *q, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    if (bits == 8) hipLaunchKernelGGL((quantize_kernel<8>), dim3(grid_for(n / 8, 16384)), dim3(256), 0, s, x, n, scale, q);
    else hipLaunchKernelGGL((quantize_kernel<4>), dim3(grid_for(n / 8, 16384)), dim3(256), 0, s, x, n, scale, q);
    return hipGetLastError();
}
