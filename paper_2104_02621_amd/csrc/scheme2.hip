// Comparison implementation of the paper's second scheme (Algorithm 5): the forward pass as one
// flat parallel loop over all small matrix products.  For every product the three operand
// positions (input capsule, kernel capsule, output capsule) are calculated beforehand into
// index arrays; the loop body reads them, multiplies one D1xD2 by one D2xD3 capsule and
// accumulates the D1xD3 result at the output position (atomic adds, since kh*kw*C products
// meet there).  For measurement only: capscaps_conv_fwd never takes this route.  The order of
// the atomic additions is not fixed, so results are reproducible only up to fp32 rounding.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "conv_shape.h"

namespace capscaps {
namespace {

template <typename T>
__device__ __forceinline__ float as_f32(T v);
template <>
__device__ __forceinline__ float as_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float as_f32<__half>(__half v) { return __half2float(v); }
template <>
__device__ __forceinline__ float as_f32<__hip_bfloat16>(__hip_bfloat16 v)
{
    return __bfloat162float(v);
}

// product index = ((((((n*Ho + x)*Wo + y)*M + m)*kh + p)*kw + q)*C + c)*D0 + d0
// index[3*i + 0/1/2] = capsule number in input (-1: the tap falls into the padding) / kernel /
// output; a capsule number times the capsule's element count is the element offset.
__global__ __launch_bounds__(256) void scheme2_index_kernel(int* __restrict__ index, ConvShape s,
                                                            size_t products)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= products) return;
    size_t r = i;
    const int d0 = (int)(r % s.D0); r /= s.D0;
    const int c = (int)(r % s.C);   r /= s.C;
    const int q = (int)(r % s.kw);  r /= s.kw;
    const int p = (int)(r % s.kh);  r /= s.kh;
    const int m = (int)(r % s.M);   r /= s.M;
    const int y = (int)(r % s.Wo);  r /= s.Wo;
    const int x = (int)(r % s.Ho);
    const int n = (int)(r / s.Ho);
    const int h = x * s.stride + p - s.pad, w = y * s.stride + q - s.pad;
    const bool inside = h >= 0 && h < s.H && w >= 0 && w < s.W;
    index[3 * i + 0] = inside ? (int)(((((size_t)n * s.H + h) * s.W + w) * s.C + c) * s.D0 + d0) : -1;
    index[3 * i + 1] = (int)(((((size_t)p * s.kw + q) * s.C + c) * s.M + m) * s.D0 + d0);
    index[3 * i + 2] = (int)(((((size_t)n * s.Ho + x) * s.Wo + y) * s.M + m) * s.D0 + d0);
}

template <typename T>
__global__ __launch_bounds__(256) void scheme2_kernel(const T* __restrict__ I,
                                                      const T* __restrict__ K,
                                                      float* __restrict__ O,
                                                      const int* __restrict__ index, int D1, int D2,
                                                      int D3, size_t products)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= products) return;
    const int ii = index[3 * i], ki = index[3 * i + 1], oi = index[3 * i + 2];
    if (ii < 0) return;
    const T* a = I + (size_t)ii * D1 * D2;
    const T* b = K + (size_t)ki * D2 * D3;
    float* o = O + (size_t)oi * D1 * D3;
    for (int d1 = 0; d1 < D1; ++d1)
        for (int d3 = 0; d3 < D3; ++d3) {
            float acc = 0.f;
            for (int d2 = 0; d2 < D2; ++d2)
                acc = fmaf(as_f32(a[d1 * D2 + d2]), as_f32(b[d2 * D3 + d3]), acc);
            atomicAdd(o + d1 * D3 + d3, acc);
        }
}

__global__ __launch_bounds__(256) void scheme2_zero_kernel(float* __restrict__ O, size_t elems)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < elems) O[i] = 0.f;
}

}  // namespace

size_t scheme2_products(const ConvShape& s)
{
    return (size_t)s.N * s.Ho * s.Wo * s.M * s.kh * s.kw * s.C * s.D0;
}

bool scheme2_supported(const ConvShape& s)
{
    // capsule numbers are 32-bit, the grid is one thread per product
    const long double lim = 2147483647.0L;
    if ((long double)s.N * s.H * s.W * s.C * s.D0 > lim) return false;
    if ((long double)s.N * s.Ho * s.Wo * s.M * s.D0 > lim) return false;
    if ((long double)s.kh * s.kw * s.C * s.M * s.D0 > lim) return false;
    const long double products =
        (long double)s.N * s.Ho * s.Wo * s.M * s.kh * s.kw * s.C * s.D0;
    return products / 256 < lim;
}

hipError_t launch_scheme2_index(const ConvShape& s, int* index, hipStream_t stream)
{
    const size_t products = scheme2_products(s);
    scheme2_index_kernel<<<(unsigned)((products + 255) / 256), 256, 0, stream>>>(index, s, products);
    return hipGetLastError();
}

hipError_t launch_scheme2(const ConvShape& s, const void* in, const void* kernel, float* out,
                          const int* index, hipStream_t stream)
{
    const size_t products = scheme2_products(s), elems = s.out_elems();
    scheme2_zero_kernel<<<(unsigned)((elems + 255) / 256), 256, 0, stream>>>(out, elems);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const unsigned blocks = (unsigned)((products + 255) / 256);
    if (s.dtype == 0)
        scheme2_kernel<float><<<blocks, 256, 0, stream>>>((const float*)in, (const float*)kernel,
                                                          out, index, s.D1, s.D2, s.D3, products);
    else if (s.dtype == 1)
        scheme2_kernel<__hip_bfloat16><<<blocks, 256, 0, stream>>>(
            (const __hip_bfloat16*)in, (const __hip_bfloat16*)kernel, out, index, s.D1, s.D2, s.D3,
            products);
    else
        scheme2_kernel<__half><<<blocks, 256, 0, stream>>>((const __half*)in, (const __half*)kernel,
                                                           out, index, s.D1, s.D2, s.D3, products);
    return hipGetLastError();
}

}  // namespace capscaps
