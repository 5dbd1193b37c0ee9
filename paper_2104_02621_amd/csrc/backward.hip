// Backward pass of the capsule convolution: gradients with respect to the input and to the
// kernel (the two results of the paper's Algorithm 4, taken as the derivative of Algorithm 2's
// sum, since the printed algorithm is garbled).  With G = dL/dO:
//
//   dI[n,h,w,c,d0] (D1xD2) = sum_{x*s+p-pad=h, y*s+q-pad=w, m}  G[n,x,y,m,d0] (D1xD3) . K[p,q,c,m,d0]^T
//   dK[p,q,c,m,d0] (D2xD3) = sum_{n,x,y}  I[n,x*s+p-pad,y*s+q-pad,c,d0]^T (D2xD1) . G[n,x,y,m,d0] (D1xD3)
//
// For stride 1 both are capsule convolutions themselves and run on the forward kernels:
//   dI = conv_fwd(G, K'),  K'[kh-1-p][kw-1-q][m][c][d0][d3][d2] = K[p][q][c][m][d0][d2][d3],
//        padding kh-1-pad (square windows), channels M -> C, capsules (D1xD3).(D3xD2);
//   dK = conv_fwd(I', G'), I' = I as [C][H][W][N][D0][D2][D1] (images <-> channels, capsules
//        transposed), G' = G as [H'][W'][N][M][D0][D1][D3] (the output gradient is the window),
//        same padding; the result [C][kh][kw][M][D0][D2][D3] is permuted into the kernel layout.
// The layout changes are done by one strided-gather kernel.  Other strides (and non-square
// windows for dI) take plain gather kernels, one thread per gradient element.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "conv_shape.h"

namespace capscaps {
namespace {

struct Permute7 {
    long long dst_dim[7];     // dense destination extents, last fastest
    long long src_stride[7];  // source stride (elements) of each destination coordinate
    long long src_base;       // source offset of destination element 0
};

template <typename T>
__global__ __launch_bounds__(256) void permute7_kernel(const T* __restrict__ src,
                                                       T* __restrict__ dst, Permute7 pm,
                                                       long long total)
{
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    long long r = id, off = pm.src_base;
#pragma unroll
    for (int k = 6; k >= 0; --k) {
        const long long c = r % pm.dst_dim[k];
        r /= pm.dst_dim[k];
        off += c * pm.src_stride[k];
    }
    dst[id] = src[off];
}

hipError_t launch_permute(const void* src, void* dst, const Permute7& pm, int elem_bytes,
                          hipStream_t stream)
{
    long long total = 1;
    for (int k = 0; k < 7; ++k) total *= pm.dst_dim[k];
    const long long blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (elem_bytes == 4)
        permute7_kernel<float><<<(unsigned)blocks, 256, 0, stream>>>((const float*)src, (float*)dst,
                                                                     pm, total);
    else
        permute7_kernel<unsigned short><<<(unsigned)blocks, 256, 0, stream>>>(
            (const unsigned short*)src, (unsigned short*)dst, pm, total);
    return hipGetLastError();
}

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }
template <>
__device__ __forceinline__ float to_f32<__hip_bfloat16>(__hip_bfloat16 v)
{
    return __bfloat162float(v);
}

// dI, any stride and window: one thread per element of dI, gather over taps, m and d3.
template <typename T>
__global__ __launch_bounds__(256) void bwd_input_direct_kernel(const T* __restrict__ G,
                                                               const T* __restrict__ K,
                                                               float* __restrict__ dI, ConvShape s,
                                                               size_t total)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    size_t r = e;
    const int d2 = (int)(r % s.D2); r /= s.D2;
    const int d1 = (int)(r % s.D1); r /= s.D1;
    const int d0 = (int)(r % s.D0); r /= s.D0;
    const int c = (int)(r % s.C);   r /= s.C;
    const int w = (int)(r % s.W);   r /= s.W;
    const int h = (int)(r % s.H);   r /= s.H;
    const int n = (int)r;
    const size_t g_caps = (size_t)s.D0 * s.D1 * s.D3, k_caps = (size_t)s.D0 * s.D2 * s.D3;
    float acc = 0.f;
    for (int p = 0; p < s.kh; ++p) {
        const int hx = h + s.pad - p;
        if (hx < 0 || hx % s.stride != 0 || hx / s.stride >= s.Ho) continue;
        for (int q = 0; q < s.kw; ++q) {
            const int wy = w + s.pad - q;
            if (wy < 0 || wy % s.stride != 0 || wy / s.stride >= s.Wo) continue;
            const int x = hx / s.stride, y = wy / s.stride;
            const T* gp = G + (((size_t)n * s.Ho + x) * s.Wo + y) * s.M * g_caps +
                          ((size_t)d0 * s.D1 + d1) * s.D3;
            const T* kp = K + (((size_t)p * s.kw + q) * s.C + c) * s.M * k_caps +
                          ((size_t)d0 * s.D2 + d2) * s.D3;
            for (int m = 0; m < s.M; ++m) {
                for (int d3 = 0; d3 < s.D3; ++d3)
                    acc = fmaf(to_f32(gp[d3]), to_f32(kp[d3]), acc);
                gp += g_caps;
                kp += k_caps;
            }
        }
    }
    dI[e] = acc;
}

// dK, any stride: one thread per element of dK, gather over images, output pixels and d1.
template <typename T>
__global__ __launch_bounds__(256) void bwd_kernel_direct_kernel(const T* __restrict__ I,
                                                                const T* __restrict__ G,
                                                                float* __restrict__ dK, ConvShape s,
                                                                size_t total)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    size_t r = e;
    const int d3 = (int)(r % s.D3); r /= s.D3;
    const int d2 = (int)(r % s.D2); r /= s.D2;
    const int d0 = (int)(r % s.D0); r /= s.D0;
    const int m = (int)(r % s.M);   r /= s.M;
    const int c = (int)(r % s.C);   r /= s.C;
    const int q = (int)(r % s.kw);
    const int p = (int)(r / s.kw);
    const size_t i_caps = (size_t)s.D0 * s.D1 * s.D2, g_caps = (size_t)s.D0 * s.D1 * s.D3;
    float acc = 0.f;
    for (int n = 0; n < s.N; ++n)
        for (int x = 0; x < s.Ho; ++x) {
            const int h = x * s.stride + p - s.pad;
            if (h < 0 || h >= s.H) continue;
            for (int y = 0; y < s.Wo; ++y) {
                const int w = y * s.stride + q - s.pad;
                if (w < 0 || w >= s.W) continue;
                const T* ip = I + ((((size_t)n * s.H + h) * s.W + w) * s.C + c) * i_caps +
                              (size_t)d0 * s.D1 * s.D2 + d2;
                const T* gp = G + ((((size_t)n * s.Ho + x) * s.Wo + y) * s.M + m) * g_caps +
                              (size_t)d0 * s.D1 * s.D3 + d3;
                for (int d1 = 0; d1 < s.D1; ++d1)
                    acc = fmaf(to_f32(ip[(size_t)d1 * s.D2]), to_f32(gp[(size_t)d1 * s.D3]), acc);
            }
        }
    dK[e] = acc;
}

template <typename Kern, typename... Args>
hipError_t launch_1d(Kern kern, size_t total, hipStream_t stream, Args... args)
{
    const size_t blocks = (total + 255) / 256;
    if (blocks == 0 || blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    kern<<<(unsigned)blocks, 256, 0, stream>>>(args..., total);
    return hipGetLastError();
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }
int elem_bytes(const ConvShape& s) { return s.dtype == 0 ? 4 : 2; }

// dI as a forward convolution of G with the flipped, transposed kernel
bool bwd_input_as_conv(const ConvShape& s)
{
    return s.stride == 1 && s.kh == s.kw && s.pad <= s.kh - 1;
}
ConvShape bwd_input_conv_shape(const ConvShape& s)
{
    // input G [N][Ho][Wo][M][D0][D1][D3], kernel K' [kh][kw][M][C][D0][D3][D2] -> dI [N][H][W][C][D0][D1][D2]
    return ConvShape{s.N, s.Ho, s.Wo, s.M, s.C, s.kh, s.kw, 1, s.kh - 1 - s.pad,
                     s.D0, s.D1, s.D3, s.D2, s.H, s.W, s.dtype};
}
// dK as a forward convolution of the re-laid-out input with the output gradient as the window
bool bwd_kernel_as_conv(const ConvShape& s) { return s.stride == 1; }
ConvShape bwd_kernel_conv_shape(const ConvShape& s)
{
    // input I' [C][H][W][N][D0][D2][D1], kernel G' [Ho][Wo][N][M][D0][D1][D3] -> [C][kh][kw][M][D0][D2][D3]
    return ConvShape{s.C, s.H, s.W, s.N, s.M, s.Ho, s.Wo, 1, s.pad,
                     s.D0, s.D2, s.D1, s.D3, s.kh, s.kw, s.dtype};
}

}  // namespace

size_t bwd_input_workspace_bytes(const ConvShape& s)
{
    if (!bwd_input_as_conv(s)) return 0;
    return align256(s.kernel_elems() * elem_bytes(s)) +
           forward_workspace_bytes(bwd_input_conv_shape(s));
}

size_t bwd_kernel_workspace_bytes(const ConvShape& s)
{
    if (!bwd_kernel_as_conv(s)) return 0;
    return align256(s.in_elems() * elem_bytes(s)) + align256(s.out_elems() * elem_bytes(s)) +
           align256(s.kernel_elems() * sizeof(float)) +
           forward_workspace_bytes(bwd_kernel_conv_shape(s));
}

int launch_bwd_input(const ConvShape& s, const void* dout, const void* kernel, float* din,
                     void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (bwd_input_as_conv(s)) {
        char* ws = static_cast<char*>(workspace);
        void* kflip = ws;
        const size_t used = align256(s.kernel_elems() * elem_bytes(s));
        // K'[p'][q'][m][c][d0][d3][d2] = K[kh-1-p'][kw-1-q'][c][m][d0][d2][d3]
        const long long sD3 = 1, sD2 = s.D3, sD0 = (long long)s.D2 * s.D3, sM = sD0 * s.D0,
                        sC = sM * s.M, sQ = sC * s.C, sP = sQ * s.kw;
        Permute7 pm{{s.kh, s.kw, s.M, s.C, s.D0, s.D3, s.D2},
                    {-sP, -sQ, sM, sC, sD0, sD3, sD2},
                    (long long)(s.kh - 1) * sP + (long long)(s.kw - 1) * sQ};
        hipError_t err = launch_permute(kernel, kflip, pm, elem_bytes(s), stream);
        if (err != hipSuccess) return status_from_hip(err);
        return forward_auto(bwd_input_conv_shape(s), dout, kflip, din, ws + used,
                            workspace_bytes - used, stream);
    }
    const size_t total = s.in_elems();
    hipError_t err;
    if (s.dtype == 0)
        err = launch_1d(bwd_input_direct_kernel<float>, total, stream, (const float*)dout,
                        (const float*)kernel, din, s);
    else if (s.dtype == 1)
        err = launch_1d(bwd_input_direct_kernel<__hip_bfloat16>, total, stream,
                        (const __hip_bfloat16*)dout, (const __hip_bfloat16*)kernel, din, s);
    else
        err = launch_1d(bwd_input_direct_kernel<__half>, total, stream, (const __half*)dout,
                        (const __half*)kernel, din, s);
    return status_from_hip(err);
}

int launch_bwd_kernel(const ConvShape& s, const void* input, const void* dout, float* dkernel,
                      void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (bwd_kernel_as_conv(s)) {
        char* ws = static_cast<char*>(workspace);
        void* in_t = ws;
        size_t used = align256(s.in_elems() * elem_bytes(s));
        void* g_t = ws + used;
        used += align256(s.out_elems() * elem_bytes(s));
        float* dk_t = reinterpret_cast<float*>(ws + used);
        used += align256(s.kernel_elems() * sizeof(float));
        // I'[c][h][w][n][d0][d2][d1] = I[n][h][w][c][d0][d1][d2]
        {
            const long long sD2 = 1, sD1 = s.D2, sD0 = (long long)s.D1 * s.D2, sC = sD0 * s.D0,
                            sW = sC * s.C, sH = sW * s.W, sN = sH * s.H;
            Permute7 pm{{s.C, s.H, s.W, s.N, s.D0, s.D2, s.D1}, {sC, sH, sW, sN, sD0, sD2, sD1}, 0};
            hipError_t err = launch_permute(input, in_t, pm, elem_bytes(s), stream);
            if (err != hipSuccess) return status_from_hip(err);
        }
        // G'[x][y][n][m][d0][d1][d3] = G[n][x][y][m][d0][d1][d3]
        {
            const long long caps = (long long)s.D0 * s.D1 * s.D3, sM = caps, sY = sM * s.M,
                            sX = sY * s.Wo, sN = sX * s.Ho;
            Permute7 pm{{s.Ho, s.Wo, s.N, s.M, s.D0, s.D1, s.D3},
                        {sX, sY, sN, sM, (long long)s.D1 * s.D3, s.D3, 1}, 0};
            hipError_t err = launch_permute(dout, g_t, pm, elem_bytes(s), stream);
            if (err != hipSuccess) return status_from_hip(err);
        }
        const int rc = forward_auto(bwd_kernel_conv_shape(s), in_t, g_t, dk_t, ws + used,
                                    workspace_bytes - used, stream);
        if (rc != 0) return rc;
        // dK[p][q][c][m][d0][d2][d3] = dK'[c][p][q][m][d0][d2][d3]
        const long long caps = (long long)s.D0 * s.D2 * s.D3, sM = caps, sQ = sM * s.M,
                        sP = sQ * s.kw, sC = sP * s.kh;
        Permute7 pm{{s.kh, s.kw, s.C, s.M, s.D0, s.D2, s.D3},
                    {sP, sQ, sC, sM, (long long)s.D2 * s.D3, s.D3, 1}, 0};
        return status_from_hip(launch_permute(dk_t, dkernel, pm, 4, stream));
    }
    const size_t total = s.kernel_elems();
    hipError_t err;
    if (s.dtype == 0)
        err = launch_1d(bwd_kernel_direct_kernel<float>, total, stream, (const float*)input,
                        (const float*)dout, dkernel, s);
    else if (s.dtype == 1)
        err = launch_1d(bwd_kernel_direct_kernel<__hip_bfloat16>, total, stream,
                        (const __hip_bfloat16*)input, (const __hip_bfloat16*)dout, dkernel, s);
    else
        err = launch_1d(bwd_kernel_direct_kernel<__half>, total, stream, (const __half*)input,
                        (const __half*)dout, dkernel, s);
    return status_from_hip(err);
}

}  // namespace capscaps
