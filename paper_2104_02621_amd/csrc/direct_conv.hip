// Last-resort kernel of the capsule convolution forward pass (paper Algorithm 2): every thread
// owns one output element O[n,x,y,m,d0,d1,d3] and walks the window taps, the input channels and
// the contracted capsule index d2 with plain fp32 FMAs, reading global memory directly.  It runs
// any shape and any element type and serves what the wavefront-level path (wave_conv.hip) cannot
// stage in LDS (capsules of more than 64 row x column-quad pieces, windows too wide for LDS).
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "igemm_common.h"

namespace capscaps {
namespace {

template <typename T>
__device__ __forceinline__ float to_float(T v);
template <>
__device__ __forceinline__ float to_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_float<__half>(__half v) { return __half2float(v); }
template <>
__device__ __forceinline__ float to_float<__hip_bfloat16>(__hip_bfloat16 v)
{
    return __bfloat162float(v);
}

template <typename T>
__global__ __launch_bounds__(256) void direct_conv_kernel(const T* __restrict__ in,
                                                          const T* __restrict__ kernel,
                                                          float* __restrict__ out, ConvShape s,
                                                          size_t total)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    // e = ((((pix*M + m)*D0 + d0)*D1 + d1)*D3 + d3
    size_t r = e;
    const int d3 = (int)(r % s.D3); r /= s.D3;
    const int d1 = (int)(r % s.D1); r /= s.D1;
    const int d0 = (int)(r % s.D0); r /= s.D0;
    const int m = (int)(r % s.M);   r /= s.M;
    const int y = (int)(r % s.Wo);  r /= s.Wo;
    const int x = (int)(r % s.Ho);  r /= s.Ho;
    const int n = (int)r;

    const size_t in_caps = (size_t)s.D0 * s.D1 * s.D2;   // elements per input capsule
    const size_t k_caps = (size_t)s.D0 * s.D2 * s.D3;    // elements per kernel capsule
    const int h0 = x * s.stride - s.pad;
    const int w0 = y * s.stride - s.pad;
    float acc = 0.f;
    for (int p = 0; p < s.kh; ++p) {
        const int h = h0 + p;
        if (h < 0 || h >= s.H) continue;
        for (int q = 0; q < s.kw; ++q) {
            const int w = w0 + q;
            if (w < 0 || w >= s.W) continue;
            const T* ip = in + (((size_t)n * s.H + h) * s.W + w) * s.C * in_caps +
                          ((size_t)d0 * s.D1 + d1) * s.D2;
            const T* kp = kernel + (((size_t)p * s.kw + q) * s.C * s.M + m) * k_caps +
                          (size_t)d0 * s.D2 * s.D3 + d3;
            for (int c = 0; c < s.C; ++c) {
                for (int d2 = 0; d2 < s.D2; ++d2)
                    acc = fmaf(to_float(ip[d2]), to_float(kp[(size_t)d2 * s.D3]), acc);
                ip += in_caps;
                kp += (size_t)s.M * k_caps;
            }
        }
    }
    store1(out, (long long)e, acc, s.out16);
}

}  // namespace

hipError_t launch_direct(const ConvShape& s, const void* in, const void* kernel, float* out,
                         hipStream_t stream)
{
    if (wave_conv_eligible(s)) return launch_wave_conv(s, in, kernel, out, stream);
    const size_t total = s.out_elems();
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    switch (s.dtype) {
        case 0:
            direct_conv_kernel<float><<<grid, block, 0, stream>>>(
                (const float*)in, (const float*)kernel, out, s, total);
            break;
        case 1:
            direct_conv_kernel<__hip_bfloat16><<<grid, block, 0, stream>>>(
                (const __hip_bfloat16*)in, (const __hip_bfloat16*)kernel, out, s, total);
            break;
        case 2:
            direct_conv_kernel<__half><<<grid, block, 0, stream>>>(
                (const __half*)in, (const __half*)kernel, out, s, total);
            break;
        default:
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace capscaps
