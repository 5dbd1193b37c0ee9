// Measurement aid: the rate at which this GPU executes back-to-back matrix instructions on
// register operands (no memory, no LDS, no barriers), for the element types of the capsule
// convolution.  bench.py runs it next to the convolution so that the fraction of the published
// peak can be read against what the chip sustains on the same kind of data at its own clocks
// (on random data the clock under matrix load settles well below the 2.4 GHz of the published
// figure).  One workgroup of 4 waves per launched block; every wave keeps 16 independent
// accumulator tiles (4 x 4 MFMA 32x32, as the tuned kernels do) and 8 operand fragments.
#include <hip/hip_runtime.h>

#include "igemm_common.h"

namespace capscaps {
namespace {

// operands: per lane 8 fragments of 16 bytes, [block-independent] seed[frag][lane]
template <typename Tag>
__global__ __launch_bounds__(256) void mfma_yardstick_kernel(const chunk_t* __restrict__ seed,
                                                             float* __restrict__ sink, int iters)
{
    const int lane = threadIdx.x & 63;
    chunk_t a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = seed[i * 64 + lane];
        b[i] = seed[(4 + i) * 64 + lane];
    }
    float16v acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) Mma<Tag>::run(a[i], b[j], acc[i][j]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

// FLOPs one launch executes
double yardstick_flops(int dtype, int blocks, int iters)
{
    // per wave and iteration 16 x (32x32x16 multiply-adds), fp32: 16 x 4 x (32x32x2)
    const double per_wave_iter = dtype == 0 ? 16.0 * 4 * 2 * 32 * 32 * 2 : 16.0 * 2 * 32 * 32 * 16;
    return per_wave_iter * 4.0 * blocks * iters;
}

hipError_t launch_yardstick(int dtype, const void* seed, float* sink, int blocks, int iters,
                            hipStream_t stream)
{
    const chunk_t* sd = static_cast<const chunk_t*>(seed);
    if (dtype == 0)
        mfma_yardstick_kernel<f32_tag><<<blocks, 256, 0, stream>>>(sd, sink, iters);
    else if (dtype == 1)
        mfma_yardstick_kernel<bf16_tag><<<blocks, 256, 0, stream>>>(sd, sink, iters);
    else
        mfma_yardstick_kernel<f16_tag><<<blocks, 256, 0, stream>>>(sd, sink, iters);
    return hipGetLastError();
}

}  // namespace capscaps
