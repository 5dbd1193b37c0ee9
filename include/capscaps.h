/*
 * capscaps -- capsule convolution (forward and backward pass) on AMD MI355X (gfx950).  C ABI.
 *
 * The operator (paper Sec. 1.2 and Algorithm 2, "General capsule convolution"; 3-D capsules
 * as in Fig. 2): for every image n, output pixel (x, y), output channel m and leading capsule
 * index d0, the D1 x D3 output capsule matrix is
 *
 *     O[n,x,y,m,d0] = sum over taps (p,q) and input channels c of
 *                     I[n, x*stride+p-pad, y*stride+q-pad, c, d0] (D1 x D2)  .  K[p,q,c,m,d0] (D2 x D3)
 *
 * with input pixels outside [0,H) x [0,W) contributing zero (pad = 0 is the paper's
 * operator; padding and the batch dimension N are extensions).  Cross-correlation, no
 * kernel flip.  The fully-connected capsule layer (Sec. 1.1) is the case kh = H, kw = W,
 * pad = 0; 2-D capsules are D0 = 1.
 *
 * Layouts: dense, row-major, last index fastest.
 *     input   [N ][H ][W ][C][D0][D1][D2]    element type given by `dtype`
 *     kernel  [kh][kw][C ][M][D0][D2][D3]    element type given by `dtype`
 *     out     [N ][H'][W'][M][D0][D1][D3]    always fp32 (the accumulator, unrounded)
 *     H' = floor((H + 2*pad - kh) / stride) + 1, W' likewise.
 *
 * Pointers: `input`, `kernel`, `out`, `workspace` are DEVICE pointers (HIP global memory on
 * the current device), 16-byte aligned, owned by the caller, not aliasing each other.
 * `input` and `kernel` are only read, `out` is overwritten (never accumulated into),
 * `workspace` is scratch whose contents are undefined afterwards.  `stream` is a
 * hipStream_t passed as void* (NULL = the default stream).  All work is enqueued on that
 * stream; no call here synchronises, so buffers must stay valid until the stream reaches the
 * end of the enqueued work.  The library keeps no global state between calls.  Calls that take a
 * `workspace` allocate nothing and enqueue only kernels, so they may be captured in a HIP graph
 * (capscaps_conv_fwd, which obtains its scratch itself, may not).
 *
 * Errors: functions returning int return CAPSCAPS_OK (0) or a negative status.  Arguments, the
 * workspace size and whether a path supports the shape are checked before the first launch: on
 * CAPSCAPS_EINVAL, CAPSCAPS_EWORKSPACE, CAPSCAPS_EUNSUPPORTED and CAPSCAPS_ESCRATCH nothing has
 * been enqueued and no buffer has been touched.  CAPSCAPS_EHIP reports a failing HIP call; a call
 * is a short sequence of launches (kernel repack, main kernel, fixed-order reduction; the backward
 * pass has a few more), so earlier launches of the sequence may already be enqueued: `out` and
 * `workspace` are undefined then.  Nothing is printed, nothing throws, nothing aborts.
 * The *_workspace_bytes queries return 0 both for "no scratch needed" and for invalid arguments;
 * capscaps_select_path (or the compute call itself) tells the two apart.
 */
#ifndef CAPSCAPS_H
#define CAPSCAPS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* every declaration below is an exported symbol of libcapscaps.so */
#pragma GCC visibility push(default)

/* element type of `input` and `kernel` */
#define CAPSCAPS_FP32 0
#define CAPSCAPS_BF16 1 /* bfloat16 in, fp32 accumulate, fp32 out */
#define CAPSCAPS_FP16 2 /* IEEE half in, fp32 accumulate, fp32 out */

/* status codes */
#define CAPSCAPS_OK 0
#define CAPSCAPS_EINVAL (-1)       /* null pointer, non-positive size, stride <= 0, pad < 0, kernel
                                      window larger than the padded input, unknown dtype/path,
                                      misaligned pointer */
#define CAPSCAPS_EWORKSPACE (-2)   /* workspace missing or smaller than required */
#define CAPSCAPS_EUNSUPPORTED (-3) /* the forced path cannot run this shape/dtype; a window of
                                      more than 2^24 taps */
#define CAPSCAPS_EHIP (-4)         /* a HIP call (launch, allocation) failed */
#define CAPSCAPS_ESCRATCH (-5)     /* capscaps_conv_fwd_static: the problem needs more scratch than
                                      CAPSCAPS_STATIC_SCRATCH_BYTES */

/* compute paths (for capscaps_conv_fwd_path / capscaps_select_path) */
#define CAPSCAPS_PATH_AUTO 0   /* library's choice */
#define CAPSCAPS_PATH_DIRECT 1 /* wavefront-level small-matrix path: plain FMAs, any shape */
#define CAPSCAPS_PATH_MFMA 2   /* LDS-staged implicit GEMM on the matrix cores (library picks
                                  the kernel variant) */
#define CAPSCAPS_PATH_MFMA_GENERIC 3 /* ... the any-shape variant (tiles 64..256, optional split
                                        of the K loop) */
#define CAPSCAPS_PATH_MFMA_TUNED16 4 /* ... the 256x256-tile variant for 16-bit types with
                                        D1 = D2 in {8, 16}; other shapes: CAPSCAPS_EUNSUPPORTED */
#define CAPSCAPS_PATH_MFMA_TUNED32 5 /* ... the lane-per-row variant with direct-to-LDS copies:
                                        fp32 capsule rows of 3, 4, 6, 8, 12 or 16 floats; 16-bit
                                        rows of 8, 16 or 32 elements (any D1, D3: non-square and
                                        vector capsules), and of 4 elements (4x4 capsules) with
                                        an even number of input channels, whose channels a
                                        pre-pass pairs in `workspace`; other shapes:
                                        CAPSCAPS_EUNSUPPORTED */
#define CAPSCAPS_PATH_MFMA_SMALL 6   /* ... the variant for small problems (a few thousand output
                                        rows, the fully-connected layer): one launch, kernel
                                        tensor read in place, 16-column tiles, fp32 matrix
                                        instructions for every element type */

/*
 * Output extents (Fig. 1 / Fig. 2: 5 with a 4-wide kernel at stride 1 gives 2).
 * Host-only, touches no GPU.  Returns CAPSCAPS_EINVAL if any size is non-positive,
 * stride <= 0, pad < 0 or the window does not fit the padded input; else writes *Ho, *Wo.
 */
int capscaps_out_shape(int H, int W, int kh, int kw, int stride, int pad, int* Ho, int* Wo);

/*
 * Capsule convolution forward (Algorithm 2), no padding: the signature of the operator as the
 * paper states it.  Scratch memory, if the chosen path needs any, is obtained and released
 * with stream-ordered allocation on `stream`.
 */
int capscaps_conv_fwd(const void* input, const void* kernel, void* out, int N, int H, int W, int C,
                      int M, int kh, int kw, int stride, int D0, int D1, int D2, int D3, int dtype,
                      void* stream);

/*
 * Same operator with symmetric zero padding `pad` and caller-provided scratch.
 * `workspace` must hold at least capscaps_conv_fwd_workspace_bytes(...) bytes for the same
 * arguments (it may be NULL when that is 0); too small -> CAPSCAPS_EWORKSPACE.
 */
int capscaps_conv_fwd_ex(const void* input, const void* kernel, void* out, int N, int H, int W,
                         int C, int M, int kh, int kw, int stride, int pad, int D0, int D1, int D2,
                         int D3, int dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * As capscaps_conv_fwd_ex, with the compute path forced (CAPSCAPS_PATH_*), so that both paths
 * can be measured on one shape.  CAPSCAPS_EUNSUPPORTED if that path cannot run the shape.
 * The workspace requirement is the one of capscaps_conv_fwd_workspace_bytes (which covers
 * every path).
 */
int capscaps_conv_fwd_path(const void* input, const void* kernel, void* out, int N, int H, int W,
                           int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                           int D2, int D3, int dtype, int path, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * As capscaps_conv_fwd_ex for 16-bit operands (dtype CAPSCAPS_BF16 or CAPSCAPS_FP16; fp32 ->
 * CAPSCAPS_EINVAL), with `out` holding elements of that same type: the fp32 accumulator is
 * rounded to nearest even once, at the store.  The output layout [N][H'][W'][M][D0][D1][D3] is the
 * input layout of a following layer (its C = M, its D2 = D3), so layers chain (the paper's
 * experiment is a five-layer stack, Sec. 3) without a conversion pass and with half the output
 * traffic.  `workspace` must hold capscaps_conv_fwd_out16_workspace_bytes(...) bytes (host-only;
 * 0 also for invalid arguments).
 */
size_t capscaps_conv_fwd_out16_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                               int stride, int pad, int D0, int D1, int D2, int D3,
                                               int dtype);
int capscaps_conv_fwd_out16(const void* input, const void* kernel, void* out, int N, int H, int W,
                            int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                            int D2, int D3, int dtype, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * capscaps_conv_fwd_ex for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * operator, arguments, layouts, kernels and results as capscaps_conv_fwd_ex, but the scratch
 * (repacked kernel, partial sums of split reductions) is a fixed array of
 * CAPSCAPS_STATIC_SCRATCH_BYTES in each GPU's memory that exists from the moment the library's
 * code is loaded on that GPU until the process ends.  The call allocates and frees nothing and
 * calls no allocating routine; a problem whose scratch does not fit returns CAPSCAPS_ESCRATCH
 * before anything is launched (all five benchmark configurations fit).  The device that holds the
 * buffers must be the current device.  The first call on a device looks up the array's address
 * there (make that call outside a graph capture).  All calls on one GPU share that GPU's array:
 * calls that may overlap on one GPU (different streams, or graphs replayed concurrently) race on
 * it and must be serialised by the caller; nothing in it needs to start at zero, every call
 * overwrites what it reads.
 */
#define CAPSCAPS_STATIC_SCRATCH_BYTES (80u << 20)
int capscaps_conv_fwd_static(const void* input, const void* kernel, void* out, int N, int H, int W,
                             int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                             int D2, int D3, int dtype, void* stream);

/*
 * Scratch bytes capscaps_conv_fwd_ex / _path need for these arguments (repacked kernel,
 * split-reduction partial sums).  Host-only.  Returns 0 also for invalid arguments (the
 * compute call reports those).
 */
size_t capscaps_conv_fwd_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                         int stride, int pad, int D0, int D1, int D2, int D3,
                                         int dtype);

/*
 * Which path CAPSCAPS_PATH_AUTO resolves to for these arguments (CAPSCAPS_PATH_DIRECT or one of
 * the CAPSCAPS_PATH_MFMA_* kernel variants), or a negative status for invalid arguments.
 * Host-only.
 */
int capscaps_select_path(int N, int H, int W, int C, int M, int kh, int kw, int stride, int pad,
                         int D0, int D1, int D2, int D3, int dtype);

/*
 * Backward pass (Algorithm 4, read as the derivative of Algorithm 2's sum: the printed
 * algorithm's index expressions are garbled).  With `dout` = dL/dO, laid out like `out` but
 * holding elements of type `dtype` (the gradient arrives in the storage type of the layer's
 * operands), both results are fp32 and overwritten, never accumulated into:
 *
 *   dinput [N][H][W][C][D0][D1][D2]:
 *     dI[n,h,w,c,d0] = sum over (x,y,p,q) with x*stride+p-pad = h, y*stride+q-pad = w, and m of
 *                      dO[n,x,y,m,d0] (D1 x D3) . transpose(K[p,q,c,m,d0]) (D3 x D2)
 *   dkernel [kh][kw][C][M][D0][D2][D3]:
 *     dK[p,q,c,m,d0] = sum over n and output pixels (x,y) whose tap (p,q) lies inside the image of
 *                      transpose(I[n,x*stride+p-pad,y*stride+q-pad,c,d0]) (D2 x D1) . dO[n,x,y,m,d0]
 *
 * The shape arguments are those of the forward call whose gradients are wanted.  The input
 * gradient is itself a capsule convolution of `dout` with the flipped, transposed kernel and runs
 * on the forward kernels (a stride s > 1 as s*s interleaved stride-1 convolutions where every one
 * of them fits a tuned kernel (see CAPSCAPS_PATH_MFMA_TUNED16 / _TUNED32) and has enough pixels,
 * else on `dout` spread out to stride 1 in `workspace`); the kernel gradient runs on dedicated
 * matrix-core kernels for 16-bit capsules of 8 or 16 rows (4-row ones that are 4x4 with even
 * channel counts, and ones of 1, 2 or 4 rows whose widths are multiples of 8) and fp32
 * capsules of 3, 4, 6, 8, 12 or 16 rows, else as a convolution with images and channels
 * exchanged.  Shapes none of these forms cover (a non-square window with pad > kh-1, ...) take
 * plain gather kernels, which need no workspace.  Pointer, stream and error rules as for the forward
 * calls; `workspace` must hold capscaps_conv_bwd_input_workspace_bytes(...) resp.
 * capscaps_conv_bwd_kernel_workspace_bytes(...) bytes for the same arguments (0 = may be NULL).
 */
int capscaps_conv_bwd_input(const void* dout, const void* kernel, void* dinput, int N, int H, int W,
                            int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                            int D2, int D3, int dtype, void* workspace, size_t workspace_bytes,
                            void* stream);
int capscaps_conv_bwd_kernel(const void* input, const void* dout, void* dkernel, int N, int H,
                             int W, int C, int M, int kh, int kw, int stride, int pad, int D0,
                             int D1, int D2, int D3, int dtype, void* workspace,
                             size_t workspace_bytes, void* stream);
/* Host-only; 0 also for invalid arguments (the compute call reports those). */
size_t capscaps_conv_bwd_input_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                               int stride, int pad, int D0, int D1, int D2, int D3,
                                               int dtype);
size_t capscaps_conv_bwd_kernel_workspace_bytes(int N, int H, int W, int C, int M, int kh, int kw,
                                                int stride, int pad, int D0, int D1, int D2,
                                                int D3, int dtype);

/*
 * As capscaps_conv_bwd_input for 16-bit operands (dtype CAPSCAPS_BF16 or CAPSCAPS_FP16; fp32 ->
 * CAPSCAPS_EINVAL), with `dinput` holding elements of that same type: every element is the fp32
 * sum of Algorithm 4's I_diff rounded to nearest even once, at the store.  The input gradient of a
 * layer is the output gradient of the layer below it (its `dout`, which arrives in the storage
 * type), so the backward pass through a stack (Sec. 3) chains without a conversion pass and with
 * half the store traffic.  Same kernels and routes as capscaps_conv_bwd_input; `workspace` must
 * hold capscaps_conv_bwd_input_out16_workspace_bytes(...) bytes (host-only; 0 also for invalid
 * arguments).
 */
size_t capscaps_conv_bwd_input_out16_workspace_bytes(int N, int H, int W, int C, int M, int kh,
                                                     int kw, int stride, int pad, int D0, int D1,
                                                     int D2, int D3, int dtype);
int capscaps_conv_bwd_input_out16(const void* dout, const void* kernel, void* dinput, int N, int H,
                                  int W, int C, int M, int kh, int kw, int stride, int pad, int D0,
                                  int D1, int D2, int D3, int dtype, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * Comparison implementation of the paper's second scheme (Algorithm 5; Sec. 2, last paragraph):
 * the three operand positions of every small matrix product are calculated beforehand
 * (capscaps_scheme2_build_index, once per shape), then one flat parallel loop multiplies and
 * accumulates each product at its output position with atomic adds.  Same operator, layouts,
 * pointer and stream rules as capscaps_conv_fwd_ex; fp32 out, overwritten.  For measurement
 * against the implicit-GEMM paths only: no capscaps_conv_fwd* call takes this route, and the
 * order of the atomic additions (hence the last bits of the result) is not fixed.
 * `index` is a device buffer of capscaps_scheme2_index_bytes(...) bytes (12 per product;
 * 0 = shape not supported: a tensor with 2^31 or more capsules, or 2^39 or more products), written
 * by _build_index and only read by _fwd.  Too small -> CAPSCAPS_EWORKSPACE.
 */
size_t capscaps_scheme2_index_bytes(int N, int H, int W, int C, int M, int kh, int kw, int stride,
                                    int pad, int D0, int D1, int D2, int D3, int dtype);
int capscaps_scheme2_build_index(void* index, size_t index_bytes, int N, int H, int W, int C, int M,
                                 int kh, int kw, int stride, int pad, int D0, int D1, int D2,
                                 int D3, int dtype, void* stream);
int capscaps_scheme2_fwd(const void* input, const void* kernel, void* out, const void* index,
                         size_t index_bytes, int N, int H, int W, int C, int M, int kh, int kw,
                         int stride, int pad, int D0, int D1, int D2, int D3, int dtype,
                         void* stream);

/*
 * Measurement aid, not part of the operator: `blocks` workgroups of 4 waves each execute
 * `iters` x 16 independent back-to-back matrix instructions (the ones the convolution kernels
 * use for `dtype`) on register operands -- no memory traffic, no LDS, no barriers -- so that a
 * convolution's fraction of the published peak can be read against what the chip sustains on
 * the same kind of data at its own clocks.  `seed`: 8 KB of device memory holding the operand
 * fragments (8 fragments x 64 lanes x 16 bytes of `dtype` elements; their values decide how
 * many bits toggle); `sink`: blocks * 256 floats, overwritten.  _flops returns the FLOPs one
 * such launch executes (0 for invalid arguments).  Time it with events on `stream`.
 */
int capscaps_mfma_yardstick(const void* seed, void* sink, int dtype, int blocks, int iters,
                            void* stream);
double capscaps_mfma_yardstick_flops(int dtype, int blocks, int iters);

/* Static, human-readable text for a status code.  Never NULL. */
const char* capscaps_strerror(int status);

/*
 * Diagnostic for CAPSCAPS_EHIP: the HIP runtime's own text for the error the calling thread's
 * most recent failing capscaps call ran into ("no error" if none has failed).  Thread-local;
 * the only state the library keeps.  Never NULL.
 */
const char* capscaps_last_hip_error(void);

#pragma GCC visibility pop

#ifdef __cplusplus
}
#endif
#endif /* CAPSCAPS_H */
