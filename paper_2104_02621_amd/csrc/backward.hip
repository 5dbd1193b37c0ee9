// Backward pass of the capsule convolution: gradients with respect to the input and to the
// kernel (the two results of the paper's Algorithm 4, taken as the derivative of Algorithm 2's
// sum, since the printed algorithm is garbled).  With G = dL/dO:
//
//   dI[n,h,w,c,d0] (D1xD2) = sum_{x*s+p-pad=h, y*s+q-pad=w, m}  G[n,x,y,m,d0] (D1xD3) . K[p,q,c,m,d0]^T
//   dK[p,q,c,m,d0] (D2xD3) = sum_{n,x,y}  I[n,x*s+p-pad,y*s+q-pad,c,d0]^T (D2xD1) . G[n,x,y,m,d0] (D1xD3)
//
// dK has kernels of its own for the common capsule shapes (wgrad16.hip, wgrad32.hip: one GEMM per
// window tap over the output pixels the tap reaches); this file holds dI and the fallback for dK.
// For stride 1 both are capsule convolutions themselves and run on the forward kernels:
//   dI = conv_fwd(G, K'),  K'[kh-1-p][kw-1-q][m][c][d0][d3][d2] = K[p][q][c][m][d0][d2][d3],
//        padding kh-1-pad (square windows), channels M -> C, capsules (D1xD3).(D3xD2);
//   dK = conv_fwd(I', G'), I' = I as [C][H][W][N][D0][D2][D1] (images <-> channels, capsules
//        transposed), G' = G as [H'][W'][N][M][D0][D1][D3] (the output gradient is the window),
//        same padding; the result [C][kh][kw][M][D0][D2][D3] is permuted into the kernel layout.
// A stride s > 1 splits dI into s*s phases, the pixels with equal ((h+pad) mod s, (w+pad) mod s):
// phase (a,b) is a stride-1 convolution of G with the window taps p = a, a+s, ..., q = b, b+s, ...
// (flipped), whose output pixels lie s apart in dI.  Where every phase fits a tuned forward
// kernel (16-bit, or fp32 with enough rows for its four-wave tiles) that kernel runs each phase
// with its own row and column padding and writes through an output stride: no multiplication
// by zeros.  Otherwise the output gradient is spread out: G is copied into a zero
// buffer of the stride-1 output extent (H+2*pad-kh+1 rows), pixel (x,y) at (x*s, y*s).  The
// contraction then runs over s*s times the needed terms (the zeros), but on the matrix cores.
// The fully-connected layer's dI (one output pixel, window = image) is a 1x1 convolution whose
// output channels are the (h,w,c) of the input.  The layout changes are done by one strided
// copy kernel.  What these forms do not cover (dI with a non-square window or pad > kh-1)
// takes a plain gather kernel, one thread per element of dI.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "igemm_common.h"

namespace capscaps {
namespace {

// Strided copy over a 7-D index space: dst[dst_base + sum c_k*dst_stride_k] =
// src[src_base + sum c_k*src_stride_k] for every index c (last coordinate fastest).
struct Permute7 {
    long long dim[7];
    long long src_stride[7];
    long long src_base;
    long long dst_stride[7];
    long long dst_base;
};

// dense destination of extents dim[]: element strides of a row-major array
Permute7 gather_into_dense(const long long (&dim)[7], const long long (&src_stride)[7],
                           long long src_base)
{
    Permute7 pm{};
    long long st = 1;
    for (int k = 6; k >= 0; --k) {
        pm.dim[k] = dim[k];
        pm.src_stride[k] = src_stride[k];
        pm.dst_stride[k] = st;
        st *= dim[k];
    }
    pm.src_base = src_base;
    pm.dst_base = 0;
    return pm;
}

template <typename T>
__global__ __launch_bounds__(256) void permute7_kernel(const T* __restrict__ src,
                                                       T* __restrict__ dst, Permute7 pm,
                                                       long long total)
{
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    long long r = id, so = pm.src_base, dofs = pm.dst_base;
#pragma unroll
    for (int k = 6; k >= 0; --k) {
        const long long c = r % pm.dim[k];
        r /= pm.dim[k];
        so += c * pm.src_stride[k];
        dofs += c * pm.dst_stride[k];
    }
    dst[dofs] = src[so];
}

// bytes is a multiple of 16
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ dst, size_t chunks)
{
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id < chunks) dst[id] = make_uint4(0u, 0u, 0u, 0u);
}

hipError_t launch_fill_zero(void* dst, size_t bytes, hipStream_t stream)
{
    const size_t chunks = bytes / 16, blocks = (chunks + 255) / 256;
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    fill_zero_kernel<<<(unsigned)blocks, 256, 0, stream>>>(static_cast<uint4*>(dst), chunks);
    return hipGetLastError();
}

hipError_t launch_permute(const void* src, void* dst, const Permute7& pm, int elem_bytes,
                          hipStream_t stream)
{
    long long total = 1;
    for (int k = 0; k < 7; ++k) total *= pm.dim[k];
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

// dI, any stride, window and padding: one thread per element of dI, gather over taps, m, d3.
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
    store1(dI, (long long)e, acc, s.out16);
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

// extents of the output gradient spread out to stride 1
int spread_h(const ConvShape& s) { return s.H + 2 * s.pad - s.kh + 1; }
int spread_w(const ConvShape& s) { return s.W + 2 * s.pad - s.kw + 1; }
size_t spread_elems(const ConvShape& s)
{
    return (size_t)s.N * spread_h(s) * spread_w(s) * s.M * s.D0 * s.D1 * s.D3;
}

// One dimension of a phase of the strided input gradient: the positions h with (h + pad) mod s
// == a are h = s*U + a - pad for U in [lo, lo + count); they are reached through the `taps`
// window taps p = a + s*i.
struct PhaseDim {
    int taps, lo, count;
};
PhaseDim phase_dim(int extent, int k, int s, int pad, int a)
{
    PhaseDim d;
    d.taps = a < k ? (k - a + s - 1) / s : 0;
    d.lo = pad - a > 0 ? (pad - a + s - 1) / s : 0;
    const int top = extent - 1 + pad - a;  // s*U <= top
    const int hi = top >= 0 ? top / s : -1;
    d.count = hi - d.lo + 1 > 0 ? hi - d.lo + 1 : 0;
    return d;
}
// phase (a,b) as a forward convolution for the tuned kernels (16-bit or fp32)
ConvShape bwd_input_phase_shape(const ConvShape& s, const PhaseDim& ph, const PhaseDim& pw, int a,
                                int b)
{
    ConvShape f{s.N, s.Ho, s.Wo, s.M, s.C, ph.taps, pw.taps, 1, ph.taps - 1 - ph.lo,
                s.D0, s.D1, s.D3, s.D2, ph.count, pw.count, s.dtype};
    f.out16 = s.out16;
    f.pad_w_set = true;
    f.pad_w = pw.taps - 1 - pw.lo;
    f.out_view = true;
    const long long pix = (long long)s.C * s.D0 * s.D1 * s.D2;
    f.out_sn = (long long)s.H * s.W * pix;
    f.out_sx = (long long)s.stride * s.W * pix;
    f.out_sy = (long long)s.stride * pix;
    f.out_base = ((long long)(s.stride * ph.lo + a - s.pad) * s.W + (s.stride * pw.lo + b - s.pad)) * pix;
    f.out_alloc = (long long)s.in_elems();
    return f;
}
// which tuned kernel runs a phase: 16 = the 256x256-tile 16-bit kernel, 32 = the lane-per-row
// kernel (fp32, or 16-bit shapes the other one does not take), 0 = neither fits or fills the chip
int phase_kernel(const ConvShape& f)
{
    if (!mfma_supported(f)) return 0;
    if (f.dtype != 0 && mfma_tuned16_supported(f) &&
        (long long)f.N * f.Ho * f.Wo * f.D1 >= 256LL * 128)
        return 16;
    // the lane-per-row kernel with its four-wave tiles and an unsplit K loop
    if (mfma_dma32_supported(f) && igemm32_dma_preferred(f)) return 32;
    return 0;
}

// 16-bit layers with capsule columns of 4 elements: the phases that run on the lane-per-row
// kernel read the output gradient with its channels paired; it is paired once for all of them
bool phases_pair_dout(const ConvShape& s) { return s.dtype != 0 && s.D3 == 4 && s.M % 2 == 0; }

// every phase that has both pixels and taps must fit a tuned kernel and fill the chip
bool bwd_input_as_phases(const ConvShape& s)
{
    if (s.stride == 1 || s.stride > 4) return false;
    for (int a = 0; a < s.stride; ++a)
        for (int b = 0; b < s.stride; ++b) {
            const PhaseDim ph = phase_dim(s.H, s.kh, s.stride, s.pad, a);
            const PhaseDim pw = phase_dim(s.W, s.kw, s.stride, s.pad, b);
            if (ph.count == 0 || pw.count == 0 || ph.taps == 0 || pw.taps == 0) continue;
            const ConvShape f = bwd_input_phase_shape(s, ph, pw, a, b);
            if (phase_kernel(f) == 0) return false;
        }
    return true;
}

// zero the pixels (n, h0 + i*sh, w0 + j*sw), i < nh, j < nw, of a tensor [N][H][W][pix] of fp32
// (T = float) or 16-bit (T = unsigned short) elements
template <typename T>
__global__ __launch_bounds__(256) void zero_pixels_kernel(T* __restrict__ out, int H, int W,
                                                          long long pix, int h0, int sh, int nh,
                                                          int w0, int sw, int nw, size_t total)
{
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    size_t r = id;
    const long long e = (long long)(r % pix); r /= pix;
    const int j = (int)(r % nw); r /= nw;
    const int i = (int)(r % nh);
    const long long n = (long long)(r / nh);
    out[((n * H + h0 + (long long)i * sh) * W + w0 + (long long)j * sw) * pix + e] = T(0);
}

// fully-connected layer: one output pixel, the window is the whole unpadded image
bool bwd_input_as_fc(const ConvShape& s)
{
    return s.Ho == 1 && s.Wo == 1 && s.pad == 0 && s.kh == s.H && s.kw == s.W;
}
ConvShape bwd_input_fc_shape(const ConvShape& s)
{
    // input G [N][1][1][M][D0][D1][D3], kernel [1][1][M][(h,w,c)][D0][D3][D2] -> dI [N][(h,w,c)][D0][D1][D2]
    ConvShape f{s.N, 1, 1, s.M, s.kh * s.kw * s.C, 1, 1, 1, 0, s.D0, s.D1, s.D3, s.D2, 1, 1,
                s.dtype};
    f.out16 = s.out16;
    return f;
}
// dI as a forward convolution of the (spread-out) G with the flipped, transposed kernel
bool bwd_input_as_conv(const ConvShape& s) { return s.kh == s.kw && s.pad <= s.kh - 1; }
ConvShape bwd_input_conv_shape(const ConvShape& s)
{
    // input Gs [N][Hs][Ws][M][D0][D1][D3], kernel K' [kh][kw][M][C][D0][D3][D2] -> dI [N][H][W][C][D0][D1][D2]
    ConvShape f{s.N, spread_h(s), spread_w(s), s.M, s.C, s.kh, s.kw, 1, s.kh - 1 - s.pad,
                s.D0, s.D1, s.D3, s.D2, s.H, s.W, s.dtype};
    f.out16 = s.out16;
    return f;
}
// dK as a forward convolution of the re-laid-out input with the (spread-out) output gradient
// as the window
ConvShape bwd_kernel_conv_shape(const ConvShape& s)
{
    // input I' [C][H][W][N][D0][D2][D1], kernel G' [Hs][Ws][N][M][D0][D1][D3] -> [C][kh][kw][M][D0][D2][D3]
    return ConvShape{s.C, s.H, s.W, s.N, s.M, spread_h(s), spread_w(s), 1, s.pad,
                     s.D0, s.D2, s.D1, s.D3, s.kh, s.kw, s.dtype};
}

}  // namespace

size_t bwd_input_workspace_bytes(const ConvShape& s)
{
    const size_t kbytes = align256(s.kernel_elems() * elem_bytes(s));
    if (bwd_input_as_fc(s)) return kbytes + forward_workspace_bytes(bwd_input_fc_shape(s));
    if (bwd_input_as_phases(s)) {
        size_t fwd = 0;
        for (int a = 0; a < s.stride; ++a)
            for (int b = 0; b < s.stride; ++b) {
                const PhaseDim ph = phase_dim(s.H, s.kh, s.stride, s.pad, a);
                const PhaseDim pw = phase_dim(s.W, s.kw, s.stride, s.pad, b);
                if (ph.count == 0 || pw.count == 0 || ph.taps == 0 || pw.taps == 0) continue;
                ConvShape f = bwd_input_phase_shape(s, ph, pw, a, b);
                f.in_paired = phases_pair_dout(s);
                const size_t need = mfma_workspace_bytes(f);
                if (need > fwd) fwd = need;
            }
        // the phases' sub-kernels together are one kernel tensor
        return kbytes + fwd + (phases_pair_dout(s) ? align256(s.out_elems() * elem_bytes(s)) : 0);
    }
    if (!bwd_input_as_conv(s)) return 0;
    const size_t gbytes = s.stride > 1 ? align256(spread_elems(s) * elem_bytes(s)) : 0;
    return kbytes + gbytes + forward_workspace_bytes(bwd_input_conv_shape(s));
}

size_t bwd_kernel_workspace_bytes(const ConvShape& s)
{
    if (wgrad16_eligible(s)) return wgrad16_workspace_bytes(s);
    if (wgrad32_eligible(s)) return wgrad32_workspace_bytes(s);
    return align256(s.in_elems() * elem_bytes(s)) + align256(spread_elems(s) * elem_bytes(s)) +
           align256(s.kernel_elems() * sizeof(float)) +
           forward_workspace_bytes(bwd_kernel_conv_shape(s));
}

// `din` holds fp32 elements, or with s.out16 set 16-bit elements of that kind (every route's
// convolution shape carries s.out16 on, so its kernels round once at their stores).
int launch_bwd_input(const ConvShape& s, const void* dout, const void* kernel, float* din,
                     void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    const int eb = elem_bytes(s);
    const long long sD3 = 1, sD2 = s.D3, sD0 = (long long)s.D2 * s.D3, sM = sD0 * s.D0,
                    sC = sM * s.M, sQ = sC * s.C, sP = sQ * s.kw;
    if (bwd_input_as_fc(s)) {
        char* ws = static_cast<char*>(workspace);
        const size_t used = align256(s.kernel_elems() * eb);
        // K2[m][(h,w,c)][d0][d3][d2] = K[h][w][c][m][d0][d2][d3]; (h,w,c) is one index of stride sC
        ConvShape f = bwd_input_fc_shape(s);
        if (forward_auto_repacks_kernel(f)) {  // read in place, through the repack pass
            f.kernel_view = true;
            f.k_sc = sM;
            f.k_sm = sC;
            f.k_sd0 = sD0;
            f.k_sd2 = sD3;
            f.k_sd3 = sD2;
            return forward_auto(f, dout, kernel, din, ws + used, workspace_bytes - used, stream);
        }
        const Permute7 pm = gather_into_dense(
            {1, 1, s.M, (long long)s.kh * s.kw * s.C, s.D0, s.D3, s.D2},
            {0, 0, sM, sC, sD0, sD3, sD2}, 0);
        hipError_t err = launch_permute(kernel, ws, pm, eb, stream);
        if (err != hipSuccess) return status_from_hip(err);
        return forward_auto(f, dout, ws, din, ws + used, workspace_bytes - used, stream);
    }
    if (bwd_input_as_phases(s)) {
        char* ws = static_cast<char*>(workspace);
        const size_t kbytes = align256(s.kernel_elems() * eb);
        const long long pix = (long long)s.C * s.D0 * s.D1 * s.D2;
        size_t used = kbytes;
        const void* dout_paired = nullptr;
        if (phases_pair_dout(s)) {
            void* dst = ws + used;
            used += align256(s.out_elems() * eb);
            const hipError_t err = launch_pair_channels(dout, dst, (size_t)s.N * s.Ho * s.Wo, s.M,
                                                        s.D0 * s.D1, stream);
            if (err != hipSuccess) return status_from_hip(err);
            dout_paired = dst;
        }
        for (int a = 0; a < s.stride; ++a)
            for (int b = 0; b < s.stride; ++b) {
                const PhaseDim ph = phase_dim(s.H, s.kh, s.stride, s.pad, a);
                const PhaseDim pw = phase_dim(s.W, s.kw, s.stride, s.pad, b);
                if (ph.count == 0 || pw.count == 0) continue;  // no pixel of dI in this phase
                const int h0 = s.stride * ph.lo + a - s.pad, w0 = s.stride * pw.lo + b - s.pad;
                if (ph.taps == 0 || pw.taps == 0) {  // pixels no window reaches
                    const size_t total = (size_t)s.N * ph.count * pw.count * pix;
                    const size_t blocks = (total + 255) / 256;
                    if (blocks > 0x7fffffffULL) return status_from_hip(hipErrorInvalidValue);
                    if (s.out16 != 0)
                        zero_pixels_kernel<unsigned short><<<(unsigned)blocks, 256, 0, stream>>>(
                            reinterpret_cast<unsigned short*>(din), s.H, s.W, pix, h0, s.stride,
                            ph.count, w0, s.stride, pw.count, total);
                    else
                        zero_pixels_kernel<float><<<(unsigned)blocks, 256, 0, stream>>>(
                            din, s.H, s.W, pix, h0, s.stride, ph.count, w0, s.stride, pw.count,
                            total);
                    const hipError_t err = hipGetLastError();
                    if (err != hipSuccess) return status_from_hip(err);
                    continue;
                }
                // the phase's kernel Kab[i'][j'][m][c][d0][d3][d2] =
                // K[a + s*(taps_h-1-i')][b + s*(taps_w-1-j')][c][m][d0][d2][d3] is read in place:
                // the repack pass of the convolution takes it through strides
                ConvShape f = bwd_input_phase_shape(s, ph, pw, a, b);
                f.kernel_view = true;
                f.k_base = (long long)(a + s.stride * (ph.taps - 1)) * sP +
                           (long long)(b + s.stride * (pw.taps - 1)) * sQ;
                f.k_sp = -s.stride * sP;
                f.k_sq = -s.stride * sQ;
                f.k_sc = sM;   // the convolution's input channels are the layer's output channels
                f.k_sm = sC;
                f.k_sd0 = sD0;
                f.k_sd2 = sD3;  // ... and its contracted capsule index the layer's d3
                f.k_sd3 = sD2;
                const bool lane_per_row = phase_kernel(f) == 32;
                f.in_paired = lane_per_row && dout_paired != nullptr;
                const int rc = lane_per_row
                                   ? forward_tuned32(f, f.in_paired ? dout_paired : dout, kernel, din,
                                                     ws + used, workspace_bytes - used, stream)
                                   : forward_tuned16(f, dout, kernel, din, ws + used,
                                                     workspace_bytes - used, stream);
                if (rc != 0) return rc;
            }
        return 0;
    }
    if (bwd_input_as_conv(s)) {
        char* ws = static_cast<char*>(workspace);
        const void* kflip = ws;
        size_t used = align256(s.kernel_elems() * eb);
        // K'[p'][q'][m][c][d0][d3][d2] = K[kh-1-p'][kw-1-q'][c][m][d0][d2][d3]
        ConvShape f = bwd_input_conv_shape(s);
        hipError_t err = hipSuccess;
        if (forward_auto_repacks_kernel(f)) {  // read in place, through the repack pass
            f.kernel_view = true;
            f.k_base = (long long)(s.kh - 1) * sP + (long long)(s.kw - 1) * sQ;
            f.k_sp = -sP;
            f.k_sq = -sQ;
            f.k_sc = sM;
            f.k_sm = sC;
            f.k_sd0 = sD0;
            f.k_sd2 = sD3;
            f.k_sd3 = sD2;
            kflip = kernel;
        } else {
            const Permute7 pm = gather_into_dense({s.kh, s.kw, s.M, s.C, s.D0, s.D3, s.D2},
                                                  {-sP, -sQ, sM, sC, sD0, sD3, sD2},
                                                  (long long)(s.kh - 1) * sP + (long long)(s.kw - 1) * sQ);
            err = launch_permute(kernel, ws, pm, eb, stream);
            if (err != hipSuccess) return status_from_hip(err);
        }
        const void* g = dout;
        if (s.stride > 1) {
            // Gs[n][x*s][y*s] = G[n][x][y], zero elsewhere; a pixel (M capsules) moves as one run
            void* gs = ws + used;
            const size_t gbytes = align256(spread_elems(s) * eb);
            used += gbytes;
            err = launch_fill_zero(gs, gbytes, stream);
            if (err != hipSuccess) return status_from_hip(err);
            const long long pix = (long long)s.M * s.D0 * s.D1 * s.D3;
            Permute7 sp{};
            const long long dim[7] = {1, 1, 1, s.N, s.Ho, s.Wo, pix};
            const long long ss[7] = {0, 0, 0, (long long)s.Ho * s.Wo * pix, s.Wo * pix, pix, 1};
            const long long ds[7] = {0, 0, 0, (long long)spread_h(s) * spread_w(s) * pix,
                                     (long long)s.stride * spread_w(s) * pix, s.stride * pix, 1};
            for (int k = 0; k < 7; ++k) {
                sp.dim[k] = dim[k];
                sp.src_stride[k] = ss[k];
                sp.dst_stride[k] = ds[k];
            }
            err = launch_permute(dout, gs, sp, eb, stream);
            if (err != hipSuccess) return status_from_hip(err);
            g = gs;
        }
        return forward_auto(f, g, kflip, din, ws + used, workspace_bytes - used, stream);
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
    if (wgrad16_eligible(s))
        return status_from_hip(launch_wgrad16(s, input, dout, dkernel, workspace, stream));
    if (wgrad32_eligible(s))
        return status_from_hip(launch_wgrad32(s, input, dout, dkernel, workspace, stream));
    const int eb = elem_bytes(s);
    char* ws = static_cast<char*>(workspace);
    void* in_t = ws;
    size_t used = align256(s.in_elems() * eb);
    void* g_t = ws + used;
    const size_t gbytes = align256(spread_elems(s) * eb);
    used += gbytes;
    float* dk_t = reinterpret_cast<float*>(ws + used);
    used += align256(s.kernel_elems() * sizeof(float));
    // I'[c][h][w][n][d0][d2][d1] = I[n][h][w][c][d0][d1][d2]
    {
        const long long sD2 = 1, sD1 = s.D2, sD0 = (long long)s.D1 * s.D2, sC = sD0 * s.D0,
                        sW = sC * s.C, sH = sW * s.W, sN = sH * s.H;
        const Permute7 pm = gather_into_dense({s.C, s.H, s.W, s.N, s.D0, s.D2, s.D1},
                                              {sC, sH, sW, sN, sD0, sD2, sD1}, 0);
        hipError_t err = launch_permute(input, in_t, pm, eb, stream);
        if (err != hipSuccess) return status_from_hip(err);
    }
    // G'[x*s][y*s][n][m][d0][d1][d3] = G[n][x][y][m][d0][d1][d3], zero elsewhere
    {
        if (s.stride > 1) {
            hipError_t err = launch_fill_zero(g_t, gbytes, stream);
            if (err != hipSuccess) return status_from_hip(err);
        }
        const long long caps = (long long)s.D0 * s.D1 * s.D3, sM = caps, sY = sM * s.M,
                        sX = sY * s.Wo, sN = sX * s.Ho;
        Permute7 pm = gather_into_dense({s.Ho, s.Wo, s.N, s.M, s.D0, s.D1, s.D3},
                                        {sX, sY, sN, sM, (long long)s.D1 * s.D3, s.D3, 1}, 0);
        const long long pix = (long long)s.N * s.M * caps;  // one window tap of G'
        pm.dst_stride[0] = (long long)s.stride * spread_w(s) * pix;
        pm.dst_stride[1] = (long long)s.stride * pix;
        hipError_t err = launch_permute(dout, g_t, pm, eb, stream);
        if (err != hipSuccess) return status_from_hip(err);
    }
    const int rc = forward_auto(bwd_kernel_conv_shape(s), in_t, g_t, dk_t, ws + used,
                                workspace_bytes - used, stream);
    if (rc != 0) return rc;
    // dK[p][q][c][m][d0][d2][d3] = dK'[c][p][q][m][d0][d2][d3]
    const long long caps = (long long)s.D0 * s.D2 * s.D3, sM = caps, sQ = sM * s.M,
                    sP = sQ * s.kw, sC = sP * s.kh;
    const Permute7 pm = gather_into_dense({s.kh, s.kw, s.C, s.M, s.D0, s.D2, s.D3},
                                          {sP, sQ, sC, sM, (long long)s.D2 * s.D3, s.D3, 1}, 0);
    return status_from_hip(launch_permute(dk_t, dkernel, pm, 4, stream));
}

}  // namespace capscaps
