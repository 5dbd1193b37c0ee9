// C ABI of the capsule convolution (forward and backward pass): argument checking, path choice, launches.
// Declarations and their contracts are in include/capscaps.h.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/capscaps.h"
#include "conv_shape.h"

using capscaps::ConvShape;

namespace {

thread_local hipError_t g_last_hip_error = hipSuccess;

int hip_status(hipError_t err)
{
    if (err == hipSuccess) return CAPSCAPS_OK;
    g_last_hip_error = err;
    (void)hipGetLastError();  // leave no sticky error behind for the caller's next HIP call
    return CAPSCAPS_EHIP;
}

int fill_shape(ConvShape& s, int N, int H, int W, int C, int M, int kh, int kw, int stride, int pad,
               int D0, int D1, int D2, int D3, int dtype)
{
    if (N <= 0 || C <= 0 || M <= 0 || D0 <= 0 || D1 <= 0 || D2 <= 0 || D3 <= 0)
        return CAPSCAPS_EINVAL;
    if (dtype != CAPSCAPS_FP32 && dtype != CAPSCAPS_BF16 && dtype != CAPSCAPS_FP16)
        return CAPSCAPS_EINVAL;
    int Ho = 0, Wo = 0;
    const int rc = capscaps_out_shape(H, W, kh, kw, stride, pad, &Ho, &Wo);
    if (rc != CAPSCAPS_OK) return rc;
    // window taps are counted in 32 bits throughout (a window over a whole large scalar image,
    // 46341 x 46341 and up, would wrap)
    if ((long long)kh * kw > (1LL << 24)) return CAPSCAPS_EUNSUPPORTED;
    s = ConvShape{N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, Ho, Wo, dtype};
    // element counts must stay well inside 63 bits
    const long double big = (long double)N * H * W * C * D0 * D1 * D2;
    const long double bigo = (long double)N * Ho * Wo * M * D0 * D1 * D3;
    const long double bigk = (long double)kh * kw * C * M * D0 * D2 * D3;
    if (big > 1e17L || bigo > 1e17L || bigk > 1e17L) return CAPSCAPS_EINVAL;
    return CAPSCAPS_OK;
}

// Measured on MI355X (fp32 and bf16 layers with 3 .. 32 output columns (m, d3) and K from 4 to
// 288, the worked example of Fig. 2 among them): with 16-column tiles the matrix cores win even
// at 4 columns (12 of 16 columns of every tile are padding there, and they still finish first:
// the wavefront-level path spends more instructions staging an input value in LDS than
// multiplying it when few output columns use it).  The wavefront-level path wins
//   * where the contraction is so short (K up to 16 measured: a 1x1 or 2x2 window over one
//     channel of 4-element capsule rows) that a matrix-core tile's 64-value K slab is mostly
//     padding, and
//   * on layers of at most 8 output columns whose capsule rows are not multiples of 4 elements
//     (Fig. 2's 3x3x3 capsules: the matrix-core kernel then gathers element by element), once
//     the layer is large enough for throughput to count (a tiny one is latency-bound, and the
//     single-stage matrix-core kernel has the shorter latency);
// it also serves what the matrix-core path cannot address.
int choose_path(const ConvShape& s)
{
    if (!capscaps::mfma_supported(s)) return CAPSCAPS_PATH_DIRECT;
    const long long kdim = (long long)s.kh * s.kw * s.C * s.D2;
    const long long cols = (long long)s.M * s.D3;
    if (kdim <= 24) return CAPSCAPS_PATH_DIRECT;
    const double flops = 2.0 * (double)s.out_elems() * (double)kdim;
    if (cols <= 8 && (s.D2 % 4 != 0 || s.D3 % 4 != 0) && flops >= 5e7 && capscaps::wave_conv_eligible(s))
        return CAPSCAPS_PATH_DIRECT;
    switch (capscaps::mfma_auto_kernel(s)) {
        case capscaps::MfmaKernel::Tuned16: return CAPSCAPS_PATH_MFMA_TUNED16;
        case capscaps::MfmaKernel::Dma32: return CAPSCAPS_PATH_MFMA_TUNED32;
        case capscaps::MfmaKernel::Small: return CAPSCAPS_PATH_MFMA_SMALL;
        default: return CAPSCAPS_PATH_MFMA_GENERIC;
    }
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Scratch of the entry point that allocates nothing (capscaps_conv_fwd_static): a fixed array in
// every GPU's memory, there from the moment the library's code is loaded on that GPU until the
// process ends.  In host code the array's name stands for the symbol, not for a device address:
// the address on the current device is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[CAPSCAPS_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(void** ptr)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return hip_status(err);
    if (dev < 0 || dev >= kMaxDevices) return CAPSCAPS_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return hip_status(err);
        if (p == nullptr) return CAPSCAPS_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return CAPSCAPS_OK;
}

int run(const void* input, const void* kernel, void* out, const ConvShape& s, int path,
        void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    // the library's own choice needs scratch for the kernel it picks only; a forced path is
    // held to the size that covers every kernel (what the size query reports)
    const bool own_choice = path == CAPSCAPS_PATH_AUTO || path == CAPSCAPS_PATH_MFMA;
    if (path == CAPSCAPS_PATH_AUTO) path = choose_path(s);
    hipError_t err;
    if (path == CAPSCAPS_PATH_DIRECT) {
        err = capscaps::launch_direct(s, input, kernel, static_cast<float*>(out), stream);
    } else if (path == CAPSCAPS_PATH_MFMA || path == CAPSCAPS_PATH_MFMA_GENERIC ||
               path == CAPSCAPS_PATH_MFMA_TUNED16 || path == CAPSCAPS_PATH_MFMA_TUNED32 ||
               path == CAPSCAPS_PATH_MFMA_SMALL) {
        if (!capscaps::mfma_supported(s)) return CAPSCAPS_EUNSUPPORTED;
        if (path == CAPSCAPS_PATH_MFMA_TUNED16 && !capscaps::mfma_tuned16_supported(s))
            return CAPSCAPS_EUNSUPPORTED;
        if (path == CAPSCAPS_PATH_MFMA_TUNED32 && !capscaps::mfma_dma32_supported(s))
            return CAPSCAPS_EUNSUPPORTED;
        if (path == CAPSCAPS_PATH_MFMA_SMALL && !capscaps::mfma_small_supported(s))
            return CAPSCAPS_EUNSUPPORTED;
        const capscaps::MfmaKernel which =
            path == CAPSCAPS_PATH_MFMA           ? capscaps::MfmaKernel::Auto
            : path == CAPSCAPS_PATH_MFMA_GENERIC ? capscaps::MfmaKernel::Generic
            : path == CAPSCAPS_PATH_MFMA_TUNED16 ? capscaps::MfmaKernel::Tuned16
            : path == CAPSCAPS_PATH_MFMA_SMALL   ? capscaps::MfmaKernel::Small
                                                 : capscaps::MfmaKernel::Dma32;
        const size_t need = own_choice ? capscaps::mfma_auto_workspace_bytes(s)
                                       : capscaps::mfma_workspace_bytes(s);
        if (need > 0 && (workspace == nullptr || workspace_bytes < need))
            return CAPSCAPS_EWORKSPACE;
        if (need > 0 && misaligned(workspace)) return CAPSCAPS_EINVAL;
        err = capscaps::launch_mfma(s, input, kernel, static_cast<float*>(out), workspace, stream,
                                    which);
    } else {
        return CAPSCAPS_EINVAL;
    }
    return hip_status(err);
}

}  // namespace

namespace capscaps {

int status_from_hip(hipError_t err) { return hip_status(err); }

size_t forward_workspace_bytes(const ConvShape& s)
{
    return choose_path(s) == CAPSCAPS_PATH_DIRECT ? 0 : mfma_auto_workspace_bytes(s);
}

bool forward_auto_repacks_kernel(const ConvShape& s) { return choose_path(s) != CAPSCAPS_PATH_DIRECT; }

int forward_auto(const ConvShape& s, const void* in, const void* kernel, float* out,
                 void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (s.pad_w_set || s.out_view) return CAPSCAPS_EINVAL;
    if (s.kernel_view && !forward_auto_repacks_kernel(s)) return CAPSCAPS_EINVAL;
    return run(in, kernel, out, s, CAPSCAPS_PATH_AUTO, workspace, workspace_bytes, stream);
}

int forward_tuned16(const ConvShape& s, const void* in, const void* kernel, float* out,
                    void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    return run(in, kernel, out, s, CAPSCAPS_PATH_MFMA_TUNED16, workspace, workspace_bytes, stream);
}

int forward_tuned32(const ConvShape& s, const void* in, const void* kernel, float* out,
                    void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    return run(in, kernel, out, s, CAPSCAPS_PATH_MFMA_TUNED32, workspace, workspace_bytes, stream);
}

}  // namespace capscaps

extern "C" {

int capscaps_out_shape(int H, int W, int kh, int kw, int stride, int pad, int* Ho, int* Wo)
{
    if (Ho == nullptr || Wo == nullptr) return CAPSCAPS_EINVAL;
    if (H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return CAPSCAPS_EINVAL;
    if (pad > (1 << 28) || H > (1 << 28) || W > (1 << 28)) return CAPSCAPS_EINVAL;
    if (kh > H + 2 * pad || kw > W + 2 * pad) return CAPSCAPS_EINVAL;
    *Ho = (H + 2 * pad - kh) / stride + 1;
    *Wo = (W + 2 * pad - kw) / stride + 1;
    return CAPSCAPS_OK;
}

size_t capscaps_conv_fwd_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                         int stride, int pad, int D0, int D1, int D2, int D3,
                                         int dtype)
{
    ConvShape s;
    if (fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) != CAPSCAPS_OK)
        return 0;
    return capscaps::mfma_workspace_bytes(s);
}

int capscaps_select_path(int N, int H, int W, int C, int M, int kh, int kw, int stride, int pad,
                         int D0, int D1, int D2, int D3, int dtype)
{
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    return choose_path(s);
}

int capscaps_conv_fwd_path(const void* input, const void* kernel, void* out, int N, int H, int W,
                           int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                           int D2, int D3, int dtype, int path, void* workspace,
                           size_t workspace_bytes, void* stream)
{
    if (input == nullptr || kernel == nullptr || out == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(input) || misaligned(kernel) || misaligned(out)) return CAPSCAPS_EINVAL;
    if (path < CAPSCAPS_PATH_AUTO || path > CAPSCAPS_PATH_MFMA_SMALL) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    return run(input, kernel, out, s, path, workspace, workspace_bytes,
               static_cast<hipStream_t>(stream));
}

int capscaps_conv_fwd_ex(const void* input, const void* kernel, void* out, int N, int H, int W,
                         int C, int M, int kh, int kw, int stride, int pad, int D0, int D1, int D2,
                         int D3, int dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    return capscaps_conv_fwd_path(input, kernel, out, N, H, W, C, M, kh, kw, stride, pad, D0, D1,
                                  D2, D3, dtype, CAPSCAPS_PATH_AUTO, workspace, workspace_bytes,
                                  stream);
}

size_t capscaps_conv_fwd_out16_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                               int stride, int pad, int D0, int D1, int D2, int D3,
                                               int dtype)
{
    ConvShape s;
    if (dtype != CAPSCAPS_BF16 && dtype != CAPSCAPS_FP16) return 0;
    if (fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) != CAPSCAPS_OK)
        return 0;
    s.out16 = dtype;
    return capscaps::forward_workspace_bytes(s);
}

int capscaps_conv_fwd_out16(const void* input, const void* kernel, void* out, int N, int H, int W,
                            int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                            int D2, int D3, int dtype, void* workspace, size_t workspace_bytes,
                            void* stream)
{
    if (input == nullptr || kernel == nullptr || out == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(input) || misaligned(kernel) || misaligned(out)) return CAPSCAPS_EINVAL;
    if (dtype != CAPSCAPS_BF16 && dtype != CAPSCAPS_FP16) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    s.out16 = dtype;
    return run(input, kernel, out, s, CAPSCAPS_PATH_AUTO, workspace, workspace_bytes,
               static_cast<hipStream_t>(stream));
}

int capscaps_conv_fwd(const void* input, const void* kernel, void* out, int N, int H, int W, int C,
                      int M, int kh, int kw, int stride, int D0, int D1, int D2, int D3, int dtype,
                      void* stream)
{
    if (input == nullptr || kernel == nullptr || out == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(input) || misaligned(kernel) || misaligned(out)) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, 0, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int path = choose_path(s);
    const size_t need = path != CAPSCAPS_PATH_DIRECT ? capscaps::mfma_workspace_bytes(s) : 0;
    void* ws = nullptr;
    if (need > 0) {
        const hipError_t err = hipMallocAsync(&ws, need, st);
        if (err != hipSuccess) return hip_status(err);
    }
    const int status = run(input, kernel, out, s, path, ws, need, st);
    if (ws != nullptr) {
        const hipError_t err = hipFreeAsync(ws, st);
        if (err != hipSuccess && status == CAPSCAPS_OK) return hip_status(err);
    }
    return status;
}

int capscaps_conv_fwd_static(const void* input, const void* kernel, void* out, int N, int H, int W,
                             int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                             int D2, int D3, int dtype, void* stream)
{
    if (input == nullptr || kernel == nullptr || out == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(input) || misaligned(kernel) || misaligned(out)) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    // the scratch the library's own kernel choice needs must fit the fixed array
    if (capscaps::forward_workspace_bytes(s) > (size_t)CAPSCAPS_STATIC_SCRATCH_BYTES)
        return CAPSCAPS_ESCRATCH;
    void* ws = nullptr;
    const int rs = scratch_of_current_device(&ws);
    if (rs != CAPSCAPS_OK) return rs;
    return run(input, kernel, out, s, CAPSCAPS_PATH_AUTO, ws, (size_t)CAPSCAPS_STATIC_SCRATCH_BYTES,
               static_cast<hipStream_t>(stream));
}

size_t capscaps_conv_bwd_input_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                               int stride, int pad, int D0, int D1, int D2, int D3,
                                               int dtype)
{
    ConvShape s;
    if (fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) != CAPSCAPS_OK)
        return 0;
    return capscaps::bwd_input_workspace_bytes(s);
}

size_t capscaps_conv_bwd_kernel_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                                int stride, int pad, int D0, int D1, int D2,
                                                int D3, int dtype)
{
    ConvShape s;
    if (fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) != CAPSCAPS_OK)
        return 0;
    return capscaps::bwd_kernel_workspace_bytes(s);
}

int capscaps_conv_bwd_input(const void* dout, const void* kernel, void* dinput, int N, int H, int W,
                            int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                            int D2, int D3, int dtype, void* workspace, size_t workspace_bytes,
                            void* stream)
{
    if (dout == nullptr || kernel == nullptr || dinput == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(dout) || misaligned(kernel) || misaligned(dinput)) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    const size_t need = capscaps::bwd_input_workspace_bytes(s);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return CAPSCAPS_EWORKSPACE;
    if (need > 0 && misaligned(workspace)) return CAPSCAPS_EINVAL;
    return capscaps::launch_bwd_input(s, dout, kernel, static_cast<float*>(dinput), workspace,
                                      workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t capscaps_conv_bwd_input_out16_workspace_bytes(int N, int H, int W, int C, int M, int kh,
                                                     int kw, int stride, int pad, int D0, int D1,
                                                     int D2, int D3, int dtype)
{
    ConvShape s;
    if (dtype != CAPSCAPS_BF16 && dtype != CAPSCAPS_FP16) return 0;
    if (fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) != CAPSCAPS_OK)
        return 0;
    s.out16 = dtype;
    return capscaps::bwd_input_workspace_bytes(s);
}

int capscaps_conv_bwd_input_out16(const void* dout, const void* kernel, void* dinput, int N, int H,
                                  int W, int C, int M, int kh, int kw, int stride, int pad, int D0,
                                  int D1, int D2, int D3, int dtype, void* workspace,
                                  size_t workspace_bytes, void* stream)
{
    if (dout == nullptr || kernel == nullptr || dinput == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(dout) || misaligned(kernel) || misaligned(dinput)) return CAPSCAPS_EINVAL;
    if (dtype != CAPSCAPS_BF16 && dtype != CAPSCAPS_FP16) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    s.out16 = dtype;
    const size_t need = capscaps::bwd_input_workspace_bytes(s);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return CAPSCAPS_EWORKSPACE;
    if (need > 0 && misaligned(workspace)) return CAPSCAPS_EINVAL;
    return capscaps::launch_bwd_input(s, dout, kernel, static_cast<float*>(dinput), workspace,
                                      workspace_bytes, static_cast<hipStream_t>(stream));
}

int capscaps_conv_bwd_kernel(const void* input, const void* dout, void* dkernel, int N, int H,
                             int W, int C, int M, int kh, int kw, int stride, int pad, int D0,
                             int D1, int D2, int D3, int dtype, void* workspace,
                             size_t workspace_bytes, void* stream)
{
    if (input == nullptr || dout == nullptr || dkernel == nullptr) return CAPSCAPS_EINVAL;
    if (misaligned(input) || misaligned(dout) || misaligned(dkernel)) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    const size_t need = capscaps::bwd_kernel_workspace_bytes(s);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return CAPSCAPS_EWORKSPACE;
    if (need > 0 && misaligned(workspace)) return CAPSCAPS_EINVAL;
    return capscaps::launch_bwd_kernel(s, input, dout, static_cast<float*>(dkernel), workspace,
                                       workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t capscaps_scheme2_index_bytes(int N, int H, int W, int C, int M, int kh, int kw, int stride,
                                    int pad, int D0, int D1, int D2, int D3, int dtype)
{
    ConvShape s;
    if (fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype) != CAPSCAPS_OK)
        return 0;
    if (!capscaps::scheme2_supported(s)) return 0;
    return capscaps::scheme2_products(s) * 3 * sizeof(int);
}

int capscaps_scheme2_build_index(void* index, size_t index_bytes, int N, int H, int W, int C, int M,
                                 int kh, int kw, int stride, int pad, int D0, int D1, int D2,
                                 int D3, int dtype, void* stream)
{
    if (index == nullptr || misaligned(index)) return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    if (!capscaps::scheme2_supported(s)) return CAPSCAPS_EUNSUPPORTED;
    if (index_bytes < capscaps::scheme2_products(s) * 3 * sizeof(int)) return CAPSCAPS_EWORKSPACE;
    return hip_status(capscaps::launch_scheme2_index(s, static_cast<int*>(index),
                                                     static_cast<hipStream_t>(stream)));
}

int capscaps_scheme2_fwd(const void* input, const void* kernel, void* out, const void* index,
                         size_t index_bytes, int N, int H, int W, int C, int M, int kh, int kw,
                         int stride, int pad, int D0, int D1, int D2, int D3, int dtype,
                         void* stream)
{
    if (input == nullptr || kernel == nullptr || out == nullptr || index == nullptr)
        return CAPSCAPS_EINVAL;
    if (misaligned(input) || misaligned(kernel) || misaligned(out) || misaligned(index))
        return CAPSCAPS_EINVAL;
    ConvShape s;
    const int rc = fill_shape(s, N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, dtype);
    if (rc != CAPSCAPS_OK) return rc;
    if (!capscaps::scheme2_supported(s)) return CAPSCAPS_EUNSUPPORTED;
    if (index_bytes < capscaps::scheme2_products(s) * 3 * sizeof(int)) return CAPSCAPS_EWORKSPACE;
    return hip_status(capscaps::launch_scheme2(s, input, kernel, static_cast<float*>(out),
                                               static_cast<const int*>(index),
                                               static_cast<hipStream_t>(stream)));
}

double capscaps_mfma_yardstick_flops(int dtype, int blocks, int iters)
{
    if (dtype < 0 || dtype > 2 || blocks <= 0 || iters <= 0) return 0.0;
    return capscaps::yardstick_flops(dtype, blocks, iters);
}

int capscaps_mfma_yardstick(const void* seed, void* sink, int dtype, int blocks, int iters,
                            void* stream)
{
    if (seed == nullptr || sink == nullptr || misaligned(seed) || misaligned(sink))
        return CAPSCAPS_EINVAL;
    if (dtype < 0 || dtype > 2 || blocks <= 0 || blocks > (1 << 20) || iters <= 0 ||
        iters > (1 << 24))
        return CAPSCAPS_EINVAL;
    return hip_status(capscaps::launch_yardstick(dtype, seed, static_cast<float*>(sink), blocks,
                                                 iters, static_cast<hipStream_t>(stream)));
}

const char* capscaps_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

const char* capscaps_strerror(int status)
{
    switch (status) {
        case CAPSCAPS_OK: return "success";
        case CAPSCAPS_EINVAL: return "invalid argument";
        case CAPSCAPS_EWORKSPACE: return "workspace missing or too small";
        case CAPSCAPS_EUNSUPPORTED: return "path does not support this shape";
        case CAPSCAPS_EHIP: return "HIP runtime error";
        case CAPSCAPS_ESCRATCH:
            return "problem needs more scratch than the fixed buffer of the entry point that "
                   "allocates nothing";
        default: return "unknown status";
    }
}

}  // extern "C"
