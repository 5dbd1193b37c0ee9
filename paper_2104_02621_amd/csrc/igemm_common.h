// Internal: types shared by the matrix-core kernels of the capsule convolution forward pass.
#pragma once
#include <hip/hip_runtime.h>

#include "conv_shape.h"

namespace capscaps {

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
typedef unsigned int chunk_t __attribute__((ext_vector_type(4)));  // 16 raw bytes

struct f32_tag { typedef float elem; };
struct f16_tag { typedef unsigned short elem; };
struct bf16_tag { typedef unsigned short elem; };

template <typename Tag>
struct Mma;
template <>
struct Mma<f16_tag> {
    static __device__ __forceinline__ void run(const chunk_t& a, const chunk_t& b, float16v& acc)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8v, a),
                                                     __builtin_bit_cast(half8v, b), acc, 0, 0, 0);
    }
};
template <>
struct Mma<bf16_tag> {
    static __device__ __forceinline__ void run(const chunk_t& a, const chunk_t& b, float16v& acc)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8v, a),
                                                      __builtin_bit_cast(bf16x8v, b), acc, 0, 0, 0);
    }
};
template <>
struct Mma<f32_tag> {
    // a chunk holds 4 K elements per lane half; element u of both halves forms the K pair of
    // one 32x32x2 instruction
    static __device__ __forceinline__ void run(const chunk_t& a, const chunk_t& b, float16v& acc)
    {
        const float4v fa = __builtin_bit_cast(float4v, a);
        const float4v fb = __builtin_bit_cast(float4v, b);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[u], fb[u], acc, 0, 0, 0);
    }
};

// fp32 -> 16-bit, round to nearest even (kind: 1 = bfloat16, 2 = IEEE half)
__device__ __forceinline__ unsigned short round_to_16(float v, int kind)
{
    if (kind == 2) {
        const _Float16 hv = (_Float16)v;
        return __builtin_bit_cast(unsigned short, hv);
    }
    const unsigned u = __builtin_bit_cast(unsigned, v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // NaN
    return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
// store 4 consecutive outputs starting at element `off` of `out`: fp32, or 16-bit if out16
__device__ __forceinline__ void store4(float* out, long long off, const float4v& v, int out16)
{
    if (out16 == 0) {
        *reinterpret_cast<float4v*>(out + off) = v;
    } else {
        typedef unsigned short us4 __attribute__((ext_vector_type(4)));
        us4 r = {round_to_16(v[0], out16), round_to_16(v[1], out16), round_to_16(v[2], out16),
                 round_to_16(v[3], out16)};
        *reinterpret_cast<us4*>(reinterpret_cast<unsigned short*>(out) + off) = r;
    }
}
__device__ __forceinline__ void store1(float* out, long long off, float v, int out16)
{
    if (out16 == 0)
        out[off] = v;
    else
        reinterpret_cast<unsigned short*>(out)[off] = round_to_16(v, out16);
}

struct IgemmParams {
    const void* in;
    const void* kp;  // repacked kernel
    float* out;      // final output, or split-K partial buffers [split][out_elems]
    int H, W, C, M, stride, pad, D0, D1, D2, D3, Ho, Wo, kw;
    long long rows;        // N*Ho*Wo*D1
    long long out_elems;   // per split
    long long pixsz;       // C*D0*D1*D2: elements per input pixel
    int cs;                // D0*D1*D2: input channel stride
    int cols, colsp;       // M*D3 and its padding to the column tile
    int KT;                // C*D2: K extent of one tap
    int KQP;               // chunks per tap, padded to a multiple of 8
    int d2c_shift;         // vector loader: log2(chunks per capsule row)
    unsigned d2_magic;     // half-chunk loader: ceil(2^32 / D2), K index / D2 as a multiplication; 0 = divide
    int spt;               // stages per tap
    int stages;            // ntaps * spt
    int stages_per_split;  // K-loop share of one split
    int nsplit;
    int ntaps;
    int row_tiles, col_tiles;
    long long in_bytes;    // size of the input tensor
    long long kp_records;  // size of the repacked kernel in bytes
    int out16;             // element type of the final output (0 = fp32), see ConvShape
    // tuned 16-bit kernel only (see ConvShape): column padding, strided output pixels
    int pad_w;
    int out_view;
    long long out_base, out_sn, out_sx, out_sy;
    // its epilogue may use buffer stores with 32-bit offsets from the tile's first pixel
    // (host-side test of D3 and of the tile's extent in the output); elements of the tensor
    // `out` points into
    int fast_store;
    long long out_alloc;
    // its launch order: tiles per image (0 = plain order), and how many of an image's first and
    // last row tiles have a shortened K loop (they are launched last)
    int lpt_timg, lpt_a, lpt_b;
    int bm;  // its tile height: 256 or 128 rows
    // its last, partial round of tiles: tiles tail_first.. are each cut into tail_split work
    // items over the channel groups of the K loop, which write fp32 partial results into
    // tail_partial [tail_split][tail_elems] (the output's last tail_elems elements, from pixel
    // tail_pix0 on); the caller adds them up.  tail_split = 0: off.
    int tail_first, tail_split, tail_pix0;
    // Launch order of the tuned kernel's first xcd_span work items (a multiple of 8 column-tile
    // groups; 0 = off): the hardware deals consecutive workgroups to the 8 XCDs in turn, and
    // with this set XCD j takes the j-th contiguous eighth of those tiles, so that all column
    // tiles of a row tile and its neighbouring row tiles read their input through one L2.
    int xcd_span;
    long long tail_elems;
    float* tail_partial;
};

// Shared launch helpers (igemm_conv.hip).  Repack: 16-byte chunks of `cw` valid K elements
// (zero-filled up to the slot's 4 floats / 8 halves); kgroup as documented at repack_kernel.
hipError_t launch_repack(const ConvShape& s, const void* kernel, void* kp, int cw, int KQP,
                         int colsp, int kgroup, size_t chunks, hipStream_t stream);
hipError_t launch_splitk_reduce(const float* partial, float* out, long long elems, int nsplit,
                                hipStream_t stream, int out16 = 0);

// fp32 kernel with direct-to-LDS copies (igemm32_dma.hip): capsule rows of 3k or 4k floats.
struct Dma32Params {
    const void* in;
    const void* kp;
    float* out;  // final output, or split-K partial buffers [split][out_elems]
    int H, W, C, M, stride, pad, D0, D1, D2, D3, Ho, Wo, kh, kw, ntaps;
    int pad_w;     // padding of the columns (pad: of the rows); either may be negative
    // out_mode bit 0 ("view"): output pixel (n, x, y) begins at element out_base + n*out_sn +
    // x*out_sx + y*out_sy; bits 1..2: 0 = fp32 output, 1 / 2 = bf16 / fp16 output (rounded at the
    // store).  One field: the kernel has no scalar register to spare.
    int out_mode;
    long long out_base, out_sn, out_sx, out_sy;
    long long rows, out_elems, pixsz, in_bytes, kp_bytes;
    int cs;        // D0*D1*D2: input channel stride (elements)
    int cols, colsp;
    int D2C;       // chunks per capsule row
    int kch;       // chunks per row and stage: 2 or 4
    int nstages;   // channel groups * taps
    int stages_per_split, nsplit;
    int row_tiles, col_tiles;
    // launch order: 0 = column tiles fastest, then row tiles, leading capsule index, K split;
    // > 0 = leading capsule index fastest, then column tiles, row tiles, and the first
    // xcd_span workgroups (a multiple of 8) permuted so that XCD j takes the j-th contiguous
    // eighth of the tiles (the hardware deals consecutive workgroups to the 8 XCDs in turn)
    int xcd_span;
    unsigned d3_magic;  // ceil(2^32 / D3): column index / D3 as a multiplication; 0 = divide
};
struct Dma32Plan {
    Dma32Params P;
    int cw, tn, nw, kqp;
    int dtype;          // 0: fp32; 1, 2: 16-bit capsule rows of 4 elements, channels paired
    long long blocks;
    size_t repack_bytes, partial_bytes;
    size_t pair_bytes;  // 16-bit: the input with its channels paired (same size as the input)
};
int igemm32_dma_chunk_width(const ConvShape& s);
Dma32Plan igemm32_dma_plan(const ConvShape& s);
bool igemm32_dma_eligible(const ConvShape& s);   // the kernel can run the shape
bool igemm32_dma_preferred(const ConvShape& s);  // ... and is the library's choice for it
hipError_t launch_igemm32_dma(const Dma32Plan& pl, hipStream_t stream);
// 16-bit operands: dst[pixel][c/2][d0][d1][c%2][4] = src[pixel][c][d0][d1][4] (8-byte units)
hipError_t launch_pair_channels(const ConvShape& s, const void* src, void* dst, hipStream_t stream);
// the same for any tensor [pixels][C][rows_per_capsule][4 halves]
hipError_t launch_pair_channels(const void* src, void* dst, size_t pixels, int C,
                                int rows_per_capsule, hipStream_t stream);

// Tuned 16-bit kernel (igemm16_fast.hip): 256x256 tiles, direct-to-LDS copies.
bool igemm16_fast_eligible(const ConvShape& s);   // the kernel can run the shape
bool igemm16_fast_preferred(const ConvShape& s);  // ... and is the library's choice for it
int igemm16_fast_tile_rows(const ConvShape& s);   // 256, 128, or 0 if not preferred
int igemm16_fast_kgroup(const ConvShape& s);      // chunks per K stage (repack order)
hipError_t launch_igemm16_fast(const IgemmParams& P, long long blocks, int dtype,
                               hipStream_t stream);

// Small-problem kernel (igemm_small.hip): one launch, kernel tensor read in place, 16-column
// tiles, K loop shared by the waves of a workgroup; honours ConvShape::kernel_view.
bool igemm_small_eligible(const ConvShape& s);   // the kernel can run the shape
bool igemm_small_preferred(const ConvShape& s);  // ... and is the library's choice for it
size_t igemm_small_workspace_bytes(const ConvShape& s);
hipError_t launch_igemm_small(const ConvShape& s, const void* in, const void* kernel, float* out,
                              void* workspace, hipStream_t stream);

// Kernel gradient on the matrix cores for 16-bit types, D1 in {8, 16} (wgrad16.hip).
bool wgrad16_eligible(const ConvShape& s);
size_t wgrad16_workspace_bytes(const ConvShape& s);
hipError_t launch_wgrad16(const ConvShape& s, const void* input, const void* dout, float* dkernel,
                          void* workspace, hipStream_t stream);
// ... and for fp32, capsule heights D1 of 3, 4, 6, 8, 12 or 16 floats (wgrad32.hip).
bool wgrad32_eligible(const ConvShape& s);
size_t wgrad32_workspace_bytes(const ConvShape& s);
hipError_t launch_wgrad32(const ConvShape& s, const void* input, const void* dout, float* dkernel,
                          void* workspace, hipStream_t stream);

}  // namespace capscaps
