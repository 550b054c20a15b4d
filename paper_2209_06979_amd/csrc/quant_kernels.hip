// First step of the quantized attention layer (paper, Section 5.3): symmetric per-tensor
// quantisation of the projections' fp32 output to int8 or packed int4 codes.
//   absmax:   max |x| over the tensor (the scale is max|x| / qmax, taken by the caller)
//   quantize: q = clamp(rint(x / scale), -qmax, qmax), ties to even.
// Both are single passes over the tensor, 16 bytes per lane and load: pure HBM streaming.
// The code decision is taken as in double precision: the fp32 quotient decides unless it lies
// within 1e-3 of a rounding boundary, and only those lanes repeat the division in fp64.
#include "internal.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

__global__ void absmax_init_kernel(float *result) { *result = 0.f; }

__global__ __launch_bounds__(256) void absmax_kernel(const float *x, int64_t n, float *result)
{
    const int64_t nv = n / 4, stride = (int64_t)gridDim.x * 256;
    float m = 0.f;
    auto take = [&](v4f v) { m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)))); };
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < nv; i += 4 * stride) { // four independent 16-byte loads in flight per lane
        const v4f v0 = reinterpret_cast<const v4f *>(x)[i], v1 = reinterpret_cast<const v4f *>(x)[i + stride];
        const v4f v2 = reinterpret_cast<const v4f *>(x)[i + 2 * stride], v3 = reinterpret_cast<const v4f *>(x)[i + 3 * stride];
        take(v0); take(v1); take(v2); take(v3);
    }
    for (; i < nv; i += stride) take(reinterpret_cast<const v4f *>(x)[i]);
    if (blockIdx.x == 0 && threadIdx.x < (int)(n - nv * 4)) m = fmaxf(m, fabsf(x[nv * 4 + threadIdx.x]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    __shared__ float red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        // non-negative floats order like their bit patterns
        atomicMax(reinterpret_cast<unsigned *>(result), __float_as_uint(m));
    }
}

__device__ __forceinline__ int code_of(float x, float scale, float qmax)
{
    const float r = x / scale; // correctly rounded fp32 division
    float q = rintf(r);
    if (fabsf(fabsf(r - truncf(r)) - 0.5f) < 1e-3f) q = (float)rint((double)x / (double)scale); // near a tie: decide in fp64
    return (int)fminf(fmaxf(q, -qmax), qmax);
}

// 8 elements per thread and iteration: two 16-byte loads, one 8-byte (int8) or 4-byte (int4) store
template <int BITS> __global__ __launch_bounds__(256) void quantize_kernel(const float *x, int64_t n, float scale, uint8_t *q)
{
    const float qmax = (BITS == 8) ? 127.f : 7.f;
    const int64_t n8 = n / 8, stride = (int64_t)gridDim.x * 256;
#pragma unroll 2
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += stride) {
        const v4f a = reinterpret_cast<const v4f *>(x)[2 * i], b = reinterpret_cast<const v4f *>(x)[2 * i + 1];
        int c[8] = {code_of(a.x, scale, qmax), code_of(a.y, scale, qmax), code_of(a.z, scale, qmax), code_of(a.w, scale, qmax),
                    code_of(b.x, scale, qmax), code_of(b.y, scale, qmax), code_of(b.z, scale, qmax), code_of(b.w, scale, qmax)};
        if (BITS == 8) {
            unsigned lo = 0, hi = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                lo |= (unsigned)(c[t] & 255) << (8 * t);
                hi |= (unsigned)(c[4 + t] & 255) << (8 * t);
            }
            reinterpret_cast<uint2 *>(q)[i] = make_uint2(lo, hi);
        } else {
            unsigned w = 0;
#pragma unroll
            for (int t = 0; t < 8; ++t) w |= (unsigned)(c[t] & 15) << (4 * t); // element 2j in bits 3:0 of byte j
            reinterpret_cast<unsigned *>(q)[i] = w;
        }
    }
    // tail of fewer than 8 elements (n is even for 4-bit codes)
    if (blockIdx.x == 0) {
        const int64_t t0 = n8 * 8;
        if (BITS == 8) {
            if (threadIdx.x < (int)(n - t0)) q[t0 + threadIdx.x] = (uint8_t)(code_of(x[t0 + threadIdx.x], scale, qmax) & 255);
        } else if (threadIdx.x < (int)((n - t0) / 2)) {
            const int64_t e = t0 + 2 * threadIdx.x;
            q[e / 2] = (uint8_t)((code_of(x[e], scale, qmax) & 15) | ((code_of(x[e + 1], scale, qmax) & 15) << 4));
        }
    }
}

inline unsigned grid_for(int64_t units)
{
    const int64_t blocks = (units + 255) / 256;
    return (unsigned)(blocks < 1 ? 1 : (blocks > 8192 ? 8192 : blocks));
}

} // namespace

hipError_t launch_absmax(const float *x, int64_t n, float *result, hipStream_t s)
{
    hipLaunchKernelGGL(absmax_init_kernel, dim3(1), dim3(1), 0, s, result);
    if (n > 0) hipLaunchKernelGGL(absmax_kernel, dim3(grid_for(n / 4)), dim3(256), 0, s, x, n, result);
    return hipGetLastError();
}

hipError_t launch_quantize(const float *x, int64_t n, float scale, int bits, uint8_t *q, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    if (bits == 8) hipLaunchKernelGGL((quantize_kernel<8>), dim3(grid_for(n / 8)), dim3(256), 0, s, x, n, scale, q);
    else hipLaunchKernelGGL((quantize_kernel<4>), dim3(grid_for(n / 8)), dim3(256), 0, s, x, n, scale, q);
    return hipGetLastError();
}
