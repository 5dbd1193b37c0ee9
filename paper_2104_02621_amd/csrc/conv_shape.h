// Internal: geometry of one capsule-convolution call and the launchers of the compute paths.
// Notation follows the paper's Algorithm 2 (I, K, O; taps (p,q); channels c -> m) with the
// capsule indices d0 (batch), d1 (row), d2 (contracted), d3 (column).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace capscaps {

// Raises a kernel's dynamic-LDS limit to `bytes` the first time the kernel is launched on a
// device (the attribute stays set for the process), not on every launch: the call costs host
// time on exactly the launch-bound problems.  `done` is the caller's record for that kernel, one
// bit per device.
inline hipError_t set_dynamic_lds_once(const void* kern, int bytes,
                                       std::atomic<unsigned long long>& done)
{
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (err == hipSuccess && dev < 64) done.fetch_or(bit, std::memory_order_release);
    return err;
}

struct ConvShape {
    int N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3;
    int Ho, Wo;  // output extents
    int dtype;   // CAPSCAPS_FP32 / BF16 / FP16
    // output element type: 0 = fp32 (the accumulator as it is); CAPSCAPS_BF16 / FP16 = the
    // accumulator rounded to nearest even at the store (forward pass of 16-bit operands only)
    int out16 = 0;
    // Geometry overrides understood by the two tuned kernels only (launch_mfma with
    // MfmaKernel::Tuned16 or ::Dma32; everything else must be given shapes without them).  The backward
    // pass uses them to run a strided layer's input gradient as stride*stride convolutions
    // whose outputs interleave.  pad_w_set: the columns' padding is pad_w instead of pad; both
    // may then be negative (the window starts inside the image) and Ho, Wo are taken as given.
    // out_view: output pixel (n, x, y) is written at element out_base + n*out_sn + x*out_sx +
    // y*out_sy of `out` instead of densely.
    bool pad_w_set = false;
    int pad_w = 0;
    bool out_view = false;
    long long out_base = 0, out_sn = 0, out_sx = 0, out_sy = 0;
    long long out_alloc = 0;  // with out_view: elements of the whole tensor `out` points into
    // kernel_view (matrix-core paths only, honoured where the kernel tensor is repacked): kernel
    // element (p, q, c, m, d0, d2, d3) is read at element k_base + p*k_sp + q*k_sq + c*k_sc +
    // m*k_sm + d0*k_sd0 + d2*k_sd2 + d3*k_sd3 of `kernel` instead of densely (strides may be
    // negative: a flipped window).
    bool kernel_view = false;
    // in_paired (lane-per-row kernel, 16-bit capsule rows of 4 elements): `input` already is the
    // channel-paired copy [pixel][c/2][d0][d1][c%2][d2] (a caller that runs several convolutions
    // on one input pairs it once)
    bool in_paired = false;
    long long k_base = 0, k_sp = 0, k_sq = 0, k_sc = 0, k_sm = 0, k_sd0 = 0, k_sd2 = 0, k_sd3 = 0;
    int padw() const { return pad_w_set ? pad_w : pad; }
    bool plain() const { return !pad_w_set && !out_view && !kernel_view && !in_paired; }
    long long pixels() const { return (long long)N * Ho * Wo; }
    size_t in_elems() const { return (size_t)N * H * W * C * D0 * D1 * D2; }
    size_t kernel_elems() const { return (size_t)kh * kw * C * M * D0 * D2 * D3; }
    size_t out_elems() const { return (size_t)N * Ho * Wo * M * D0 * D1 * D3; }
};

// Wavefront-level small-matrix path: plain FMAs, any shape, any dtype.  No scratch.
// (`out` points to fp32 or, with s.out16, to 16-bit elements; likewise for launch_mfma)
// launch_direct takes the LDS-staged wave kernel (wave_conv.hip) where it can stage the shape,
// else a thread-per-element kernel.
hipError_t launch_direct(const ConvShape& s, const void* in, const void* kernel, float* out,
                         hipStream_t stream);
bool wave_conv_eligible(const ConvShape& s);
hipError_t launch_wave_conv(const ConvShape& s, const void* in, const void* kernel, float* out,
                            hipStream_t stream);

// Matrix-core path (LDS-staged implicit GEMM).  `mfma_supported` tells whether the path can
// run the shape; `mfma_workspace_bytes` is the scratch it needs (repacked kernel plus, for
// small problems, split-reduction partial sums).
enum class MfmaKernel { Auto, Generic, Tuned16, Dma32, Small };
bool mfma_supported(const ConvShape& s);
MfmaKernel mfma_auto_kernel(const ConvShape& s);  // what Auto resolves to (never Auto)
bool mfma_tuned16_supported(const ConvShape& s);
bool mfma_dma32_supported(const ConvShape& s);
bool mfma_small_supported(const ConvShape& s);
size_t mfma_workspace_bytes(const ConvShape& s);  // enough for every MfmaKernel choice (with
                                                  // s.out16: for Auto, the only choice then)
size_t mfma_auto_workspace_bytes(const ConvShape& s);  // for the kernel Auto resolves to only
hipError_t launch_mfma(const ConvShape& s, const void* in, const void* kernel, float* out,
                       void* workspace, hipStream_t stream, MfmaKernel which = MfmaKernel::Auto);

// The forward pass with the library's own path choice, and the scratch it needs (defined next
// to the C ABI); used by the backward pass, which for stride 1 is two forward convolutions.
// Both return a status code of the C ABI; `status_from_hip` maps a HIP error to one and
// records it for the ABI's diagnostic call.
size_t forward_workspace_bytes(const ConvShape& s);
int forward_auto(const ConvShape& s, const void* in, const void* kernel, float* out,
                 void* workspace, size_t workspace_bytes, hipStream_t stream);
// whether that choice is a matrix-core kernel, which takes the kernel tensor through a repack
// pass and therefore accepts s.kernel_view (the wavefront-level path reads it densely)
bool forward_auto_repacks_kernel(const ConvShape& s);
// the tuned 16-bit kernel, geometry overrides allowed (EUNSUPPORTED if it cannot run the shape)
int forward_tuned16(const ConvShape& s, const void* in, const void* kernel, float* out,
                    void* workspace, size_t workspace_bytes, hipStream_t stream);
// ... and the tuned fp32 kernel
int forward_tuned32(const ConvShape& s, const void* in, const void* kernel, float* out,
                    void* workspace, size_t workspace_bytes, hipStream_t stream);
int status_from_hip(hipError_t err);

// Backward pass (backward.hip): gradients with respect to input and kernel, fp32 results.
size_t bwd_input_workspace_bytes(const ConvShape& s);
size_t bwd_kernel_workspace_bytes(const ConvShape& s);
// Return a status code of the C ABI.
int launch_bwd_input(const ConvShape& s, const void* dout, const void* kernel, float* din,
                     void* workspace, size_t workspace_bytes, hipStream_t stream);
int launch_bwd_kernel(const ConvShape& s, const void* input, const void* dout, float* dkernel,
                      void* workspace, size_t workspace_bytes, hipStream_t stream);

// The paper's second scheme (Algorithm 5) as a comparison implementation (scheme2.hip).
bool scheme2_supported(const ConvShape& s);
size_t scheme2_products(const ConvShape& s);  // small matrix products = index triples
hipError_t launch_scheme2_index(const ConvShape& s, int* index, hipStream_t stream);
hipError_t launch_scheme2(const ConvShape& s, const void* in, const void* kernel, float* out,
                          const int* index, hipStream_t stream);

// Measurement aid (yardstick.hip): back-to-back matrix instructions on register operands.
double yardstick_flops(int dtype, int blocks, int iters);
hipError_t launch_yardstick(int dtype, const void* seed, float* sink, int blocks, int iters,
                            hipStream_t stream);

}  // namespace capscaps
