// Matrix-core kernel of the capsule convolution forward pass (paper Algorithm 2) for SMALL
// problems: a few thousand output rows or fewer, any window -- among them the fully-connected
// capsule layer (Sec. 1.1: the window covers the whole input, one output pixel per image).
// Such problems are bound by launch and memory latency, not by arithmetic, so this kernel is
// one launch with a short body (two launches when the K loop is cut over workgroups):
//
//   * the kernel tensor is read in place (no repack pass): its (d2, d3) capsule matrices are
//     already K-major for the matrix instruction used here;
//   * same implicit GEMM as the large kernels -- rows (pixel, d1), columns (m, d3),
//     K = (tap, c, d2) -- on v_mfma_f32_16x16x4f32 tiles, so 16 columns fill a tile.  16-bit
//     operands are widened to fp32 while they are staged (exact), products and sums are fp32;
//   * a workgroup owns a tile of 16 or 32 rows x 16..64 columns; K is walked in slabs of 64
//     values staged through LDS, and the four waves share each slab's K range (wave w takes
//     K values 16w .. 16w+15), so no operand is read from LDS twice; their four partial tiles
//     are added through LDS in a fixed order at the end;
//   * the body is kept short on purpose: a launch this small executes most of its code exactly
//     once and pays for fetching it, so the K loop is not unrolled over a ring of stages (a ring
//     of 4 register sets measured 1.0 .. 1.5 us slower on both small configurations than the
//     single set used here); the loads of the next slab are issued before the matrix
//     instructions of the current one, and their address arithmetic is dealt out between those
//     instructions (one wave per SIMD issues one instruction at a time);
//   * a K loop too long for the few tiles of such a problem is cut over workgroups (config 4:
//     72 slabs per tile over 8 workgroups) and a fixed-order reduction kernel follows.
//
// LDS layouts (fp32 words): input side [row][K + 4]   (row stride 68: the 64 lanes of an
// operand read, 16 rows x 4 K values, fall into 64 different banks), kernel side [K][SB] with
// SB = 16, 48, 48 or 80 for 16..64 columns (same property for 4 K values x 16 columns).
#include <hip/hip_runtime.h>

#include "igemm_common.h"

namespace capscaps {
namespace {

// where kernel element (p, q, c, m, d0, d2, d3) lies in the tensor handed to the call (elements)
struct KStrides {
    long long base, sp, sq, sc, sm, sd0, sd2, sd3;
};

struct KStrides32 {  // the same in 32 bits, for the kernel (tensors here are below 2^31 bytes)
    int base, sp, sq, sc, sm, sd0, sd2, sd3;
};

struct Magic {
    unsigned mul, pass;
};

struct SmallParams {
    const void* in;
    const void* kernel;
    float* out;  // final output, or partial results [split][out_elems]
    int H, W, C, M, stride, pad, D0, D1, D2, D3, Ho, Wo, kw;
    int rows, cols;  // N*Ho*Wo*D1, M*D3
    int KT, Ktot;    // C*D2, ntaps*C*D2
    int hw;          // Ho*Wo
    int slabs, slabs_per_split, nsplit, row_tiles, col_tiles;
    long long out_elems;
    int pixsz, img_elems;        // elements per input pixel and per image
    int in_bytes, kernel_bytes;  // sizes of the two operand tensors (below 2^31)
    int cs;  // D0*D1*D2: input channel stride
    KStrides32 ks;
    // x / d as the upper half of x * ceil(2^32 / d), exact while x * d < 2^32 (host-checked);
    // d = 1 is (magic 0, pass -1): x / 1 = 0 + (x & -1), so the division is branch-free
    Magic mg_KT, mg_D2, mg_kw, mg_D1, mg_hw, mg_Wo, mg_D3;
    int out16;
};

// products of two values below 2^24 (pixel counts, channel strides: host-checked), low 32 bits
__device__ __forceinline__ unsigned umul24(int a, int b)
{
    return __umul24((unsigned)a, (unsigned)b);
}

__device__ __forceinline__ int mdiv(int x, Magic m)
{
    return (int)(__umulhi((unsigned)x, m.mul) + ((unsigned)x & m.pass));
}

// Operand loads are raw buffer loads: an offset at or beyond the descriptor's size reads as
// zero, so padding taps, rows, columns and K positions that do not exist are one out-of-range
// offset and every load is issued unconditionally -- the K loop then is straight-line code and
// the compiler's wait counts stay exact.
constexpr unsigned OOB = 0x80000000u;  // tensors handled here are smaller than 2^31 bytes

template <typename Tag>
struct Elem;
template <>
struct Elem<f32_tag> {
    static constexpr int BYTES = 4;
    static __device__ __forceinline__ float load1(__amdgpu_buffer_rsrc_t rs, unsigned off)
    {
        return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0));
    }
    static __device__ __forceinline__ float4v load4(__amdgpu_buffer_rsrc_t rs, unsigned off)
    {
        return __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
    }
};
template <>
struct Elem<bf16_tag> {
    static constexpr int BYTES = 2;
    static __device__ __forceinline__ float load1(__amdgpu_buffer_rsrc_t rs, unsigned off)
    {
        const unsigned v = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0);
        return __builtin_bit_cast(float, v << 16);
    }
    static __device__ __forceinline__ float4v load4(__amdgpu_buffer_rsrc_t rs, unsigned off)
    {
        typedef unsigned int u2 __attribute__((ext_vector_type(2)));
        const u2 w = __builtin_bit_cast(u2, __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 0));
        float4v r = {__builtin_bit_cast(float, w[0] << 16),
                     __builtin_bit_cast(float, w[0] & 0xffff0000u),
                     __builtin_bit_cast(float, w[1] << 16),
                     __builtin_bit_cast(float, w[1] & 0xffff0000u)};
        return r;
    }
};
template <>
struct Elem<f16_tag> {
    static constexpr int BYTES = 2;
    static __device__ __forceinline__ float load1(__amdgpu_buffer_rsrc_t rs, unsigned off)
    {
        const unsigned short v = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rs, off, 0, 0);
        return (float)__builtin_bit_cast(_Float16, v);
    }
    static __device__ __forceinline__ float4v load4(__amdgpu_buffer_rsrc_t rs, unsigned off)
    {
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        const h4 w = __builtin_bit_cast(h4, __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 0));
        float4v r = {(float)w[0], (float)w[1], (float)w[2], (float)w[3]};
        return r;
    }
};

constexpr int KS = 64;  // K values per slab

constexpr int small_sb(int bn) { return bn % 32 == 16 ? bn : bn + 16; }

// BMT, BNT: tile of 16*BMT rows x 16*BNT columns.  VECA: D2 % 4 == 0, input rows are read in
// 4-element pieces; VECB: D3 % 4 == 0 and d3 is the kernel tensor's fastest index, kernel
// capsule rows are read in 4-element pieces; otherwise element by element.
template <typename Tag, int BMT, int BNT, bool VECA, bool VECB>
__global__ __launch_bounds__(256) void igemm_small_kernel(const SmallParams P)
{
    constexpr int EB = Elem<Tag>::BYTES;
    constexpr int BM = 16 * BMT, BN = 16 * BNT;
    constexpr int SA = KS + 4, SB = small_sb(BN);
    constexpr int A_WORDS = BM * SA, B_WORDS = KS * SB, STAGE = A_WORDS + B_WORDS;
    constexpr int RS = BN + 4;  // row stride of a wave's partial tile in the final reduction
    constexpr int NA = VECA ? BMT : 4 * BMT;  // input-side load slots per thread and slab
    constexpr int NB = VECB ? BNT : 4 * BNT;  // kernel-side load slots
    static_assert(4 * BM * RS <= 2 * STAGE, "the reduction buffer reuses the stage buffers");
    __shared__ __attribute__((aligned(16))) float lds[2 * STAGE];

    int L = blockIdx.x;
    const int col_tile = L % P.col_tiles;
    L /= P.col_tiles;
    const int row_tile = L % P.row_tiles;
    L /= P.row_tiles;
    const int d0 = L % P.D0;
    const int split = L / P.D0;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int row0 = row_tile * BM, col0 = col_tile * BN;
    const __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(P.in), 0, (int)P.in_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_k = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(P.kernel), 0, (int)P.kernel_bytes, 0x00020000);

    // ---- input-side load slots: fixed rows of the tile, the K position moves with the slab
    // VECA: slot i = row (tid & 15) + 16 i, K piece 4 (tid >> 4) (the 16 lanes of a K piece
    // write 16 different bank groups of LDS);  else row (tid >> 6) + 4 i, K value tid & 63
    unsigned a_base[NA];  // element offset of (image, d0, d1) of the slot's row
    int a_ih0[NA], a_iw0[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int row_l = VECA ? (tid & 15) + 16 * i : (tid >> 6) + 4 * i;
        const int r = row0 + row_l;
        if (r < P.rows) {
            const int pixel = mdiv(r, P.mg_D1), d1 = r - pixel * P.D1;
            const int n = mdiv(pixel, P.mg_hw), rem = pixel - n * P.hw;
            const int x = mdiv(rem, P.mg_Wo), y = rem - x * P.Wo;
            a_ih0[i] = x * P.stride - P.pad;
            a_iw0[i] = y * P.stride - P.pad;
            a_base[i] = (unsigned)n * (unsigned)P.img_elems + (unsigned)((d0 * P.D1 + d1) * P.D2);
        } else {
            a_ih0[i] = -(1 << 30);  // no tap of such a row is ever inside the image
            a_iw0[i] = 0;
            a_base[i] = 0;
        }
    }
    // ---- kernel-side load slots.  VECB: K value 4 (tid >> 4) + (tid & 3) -- with VECA that is
    // the thread's input-side K piece plus 0..3, so one decomposition of the K position serves
    // both sides --, column piece 16 i + 4 ((tid >> 2) & 3): a quarter wave writes 16 different
    // bank groups of LDS;
    // else K value (tid >> 4) + 16 (i / BNT), column (tid & 15) + 16 (i % BNT)
    int b_base[NB];  // element offset of the slot's column (m, d3) and of d0
    bool b_ok[NB];   // the column exists
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int col = col0 + (VECB ? 16 * i + 4 * ((tid >> 2) & 3) : (tid & 15) + 16 * (i % BNT));
        b_ok[i] = col < P.cols;
        const int cc = b_ok[i] ? col : 0;
        const int m = mdiv(cc, P.mg_D3), d3 = cc - m * P.D3;
        b_base[i] = P.ks.base + m * P.ks.sm + d0 * P.ks.sd0 + d3 * P.ks.sd3;
    }

    // K position kk = (tap, c, d2) -> tap, offset of (c, d2) within an input pixel resp. a
    // kernel tap; kk past the end gives tap = -1
    auto split_k = [&](int kk, int& tap, int& p, int& q, int& c, int& d2) {
        const bool past = kk >= P.Ktot;
        kk = past ? 0 : kk;
        const int t = mdiv(kk, P.mg_KT);
        const int rem = kk - t * P.KT;
        c = mdiv(rem, P.mg_D2);
        d2 = rem - c * P.D2;
        p = mdiv(t, P.mg_kw);
        q = t - p * P.kw;
        tap = past ? -1 : t;
    };

    // the slab on its way from global memory to LDS
    float4v areg[VECA ? BMT : 1];
    float ascal[VECA ? 1 : 4 * BMT];
    float4v breg[VECB ? BNT : 1];
    float bscal[VECB ? 1 : 4 * BNT];

    // global loads of one slab (a slab past the end loads nothing but zeros)
    auto gload = [&](int slab) {
        const int k0 = slab * KS;
        int tap, p, q, c, d2;
        split_k(k0 + (VECA ? 4 * (tid >> 4) : (tid & 63)), tap, p, q, c, d2);
        {   // input side
            const unsigned koff = (unsigned)(umul24(c, P.cs) + d2);
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int ih = a_ih0[i] + p, iw = a_iw0[i] + q;
                const bool ok = tap >= 0 && (unsigned)ih < (unsigned)P.H &&
                                (unsigned)iw < (unsigned)P.W;
                const unsigned off =
                    ok ? (a_base[i] + umul24(umul24(ih, P.W) + iw, P.pixsz) + koff) * EB : OOB;
                if constexpr (VECA)
                    areg[i] = Elem<Tag>::load4(rs_in, off);
                else
                    ascal[i] = Elem<Tag>::load1(rs_in, off);
            }
        }
        if constexpr (VECB) {
            if constexpr (VECA) {
                d2 += tid & 3;  // same tap and channel: D2 is a multiple of 4
            } else {
                split_k(k0 + 4 * (tid >> 4) + (tid & 3), tap, p, q, c, d2);
            }
            const int koff = p * P.ks.sp + q * P.ks.sq + c * P.ks.sc + d2 * P.ks.sd2;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                breg[i] = Elem<Tag>::load4(
                    rs_k, (tap >= 0 && b_ok[i]) ? (unsigned)(b_base[i] + koff) * EB : OOB);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int tap, p, q, c, d2;
                split_k(k0 + (tid >> 4) + 16 * u, tap, p, q, c, d2);
                const int koff = p * P.ks.sp + q * P.ks.sq + c * P.ks.sc + d2 * P.ks.sd2;
#pragma unroll
                for (int j = 0; j < BNT; ++j) {
                    const int i = u * BNT + j;
                    bscal[i] = Elem<Tag>::load1(
                        rs_k, (tap >= 0 && b_ok[i]) ? (unsigned)(b_base[i] + koff) * EB : OOB);
                }
            }
        }
    };
    // the loaded slab -> LDS stage buffer `buf`
    auto lds_store = [&](int buf) {
        float* A = lds + buf * STAGE;
        float* B = A + A_WORDS;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if constexpr (VECA)
                *reinterpret_cast<float4v*>(A + ((tid & 15) + 16 * i) * SA + 4 * (tid >> 4)) =
                    areg[i];
            else
                A[((tid >> 6) + 4 * i) * SA + (tid & 63)] = ascal[i];
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if constexpr (VECB)
                *reinterpret_cast<float4v*>(B + (4 * (tid >> 4) + (tid & 3)) * SB + 16 * i +
                                            4 * ((tid >> 2) & 3)) = breg[i];
            else
                B[((tid >> 4) + 16 * (i / BNT)) * SB + (tid & 15) + 16 * (i % BNT)] = bscal[i];
        }
    };

    float4v acc[BNT][BMT];
#pragma unroll
    for (int a = 0; a < BNT; ++a)
#pragma unroll
        for (int b = 0; b < BMT; ++b) acc[a][b] = float4v{0.f, 0.f, 0.f, 0.f};

    // the matrix instruction's row operand is the kernel side (16 columns of the output), its
    // column operand the input side (16 rows): lane l supplies K value l / 16 of column resp.
    // row l % 16 and ends up with 4 consecutive columns 4 (l / 16) .. + 3 of output row l % 16
    const int lr = lane & 15, lk = lane >> 4;
    // operands of a whole slab for this wave (its 16 K values): 4 k-steps of BMT + BNT words
    float ib[4][BMT], ka[4][BNT];
    auto read_operands = [&](int buf) {
        const float* A = lds + buf * STAGE;
        const float* B = A + A_WORDS;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int kl = 16 * wave + 4 * t + lk;
#pragma unroll
            for (int b = 0; b < BMT; ++b) ib[t][b] = A[(16 * b + lr) * SA + kl];
#pragma unroll
            for (int a = 0; a < BNT; ++a) ka[t][a] = B[kl * SB + 16 * a + lr];
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int a = 0; a < BNT; ++a)
#pragma unroll
                for (int b = 0; b < BMT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(ka[t][a], ib[t][b], acc[a][b], 0, 0, 0);
    };

    const int s_begin = split * P.slabs_per_split;
    const int s_end = s_begin + P.slabs_per_split < P.slabs ? s_begin + P.slabs_per_split : P.slabs;

    // ---- K loop over the slabs [s_begin, s_end); LDS buffers alternate.  Every load, LDS store
    // and barrier is executed unconditionally (a slab past the end is zeros).
    gload(s_begin < s_end ? s_begin : P.slabs);
    lds_store(0);
    __syncthreads();
    int buf = 0;
    for (int cur = s_begin; cur < s_end; ++cur) {
        // One basic block: the operand reads of slab `cur` first, then the address arithmetic
        // and loads of slab cur + 1 dealt out between the matrix instructions (what is not
        // placed under a matrix instruction's 32 cycles adds to them).
        read_operands(buf);
        gload(cur + 1 < s_end ? cur + 1 : P.slabs);
        multiply();
        __builtin_amdgcn_sched_group_barrier(0x100, 4 * (BMT + BNT), 0);  // LDS reads
#pragma unroll
        for (int i = 0; i < 4 * BMT * BNT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x026, 5, 0);  // VALU, SALU, loads
        }
        lds_store(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // ---- the four waves' partial tiles, added in wave order, and the store
    float* red = lds;
#pragma unroll
    for (int a = 0; a < BNT; ++a)
#pragma unroll
        for (int b = 0; b < BMT; ++b)
            *reinterpret_cast<float4v*>(red + wave * (BM * RS) + (16 * b + lr) * RS + 16 * a + 4 * lk) =
                acc[a][b];
    __syncthreads();
    float* __restrict__ out = P.out + (long long)split * P.out_elems;
    const int caps_out = P.D0 * P.D1 * P.D3;
    for (int g = tid; g < BM * BN / 4; g += 256) {
        const int row_l = g / (BN / 4), cg = g - row_l * (BN / 4);
        const int r = row0 + row_l, col = col0 + 4 * cg;
        if (r >= P.rows || col >= P.cols) continue;
        const float* src = red + row_l * RS + 4 * cg;
        float4v v = *reinterpret_cast<const float4v*>(src);
#pragma unroll
        for (int w = 1; w < 4; ++w) v += *reinterpret_cast<const float4v*>(src + w * (BM * RS));
        const int pixel = mdiv(r, P.mg_D1), d1 = r - pixel * P.D1;
        const long long rbase = (long long)pixel * P.M * caps_out + (long long)(d0 * P.D1 + d1) * P.D3;
        if constexpr (VECB) {  // D3 % 4 == 0: the four columns are one capsule row piece
            const int m = mdiv(col, P.mg_D3), d3 = col - m * P.D3;
            store4(out, rbase + (long long)m * caps_out + d3, v, P.out16);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (col + u < P.cols) {
                    const int m = mdiv(col + u, P.mg_D3), d3 = col + u - m * P.D3;
                    store1(out, rbase + (long long)m * caps_out + d3, v[u], P.out16);
                }
            }
        }
    }
}

Magic magic_of(long long d)
{
    if (d <= 1) return Magic{0u, 0xffffffffu};
    return Magic{(unsigned)(((1ULL << 32) + d - 1) / d), 0u};
}

struct SmallPlan {
    SmallParams P;
    int bmt, bnt;
    bool veca, vecb;
    long long blocks;
    size_t partial_bytes;
};

KStrides kernel_strides(const ConvShape& s)
{
    KStrides ks;
    if (s.kernel_view) {
        ks = {s.k_base, s.k_sp, s.k_sq, s.k_sc, s.k_sm, s.k_sd0, s.k_sd2, s.k_sd3};
    } else {  // dense [kh][kw][C][M][D0][D2][D3]
        ks.base = 0;
        ks.sd3 = 1;
        ks.sd2 = s.D3;
        ks.sd0 = (long long)s.D2 * s.D3;
        ks.sm = ks.sd0 * s.D0;
        ks.sc = ks.sm * s.M;
        ks.sq = ks.sc * s.C;
        ks.sp = ks.sq * s.kw;
    }
    return ks;
}

SmallPlan small_plan(const ConvShape& s)
{
    SmallPlan pl{};
    SmallParams& P = pl.P;
    P.H = s.H; P.W = s.W; P.C = s.C; P.M = s.M; P.stride = s.stride; P.pad = s.pad;
    P.D0 = s.D0; P.D1 = s.D1; P.D2 = s.D2; P.D3 = s.D3; P.Ho = s.Ho; P.Wo = s.Wo; P.kw = s.kw;
    P.rows = (int)(s.pixels() * s.D1);
    P.cols = s.M * s.D3;
    P.KT = s.C * s.D2;
    P.Ktot = s.kh * s.kw * P.KT;
    P.hw = s.Ho * s.Wo;
    P.out_elems = (long long)s.out_elems();
    P.cs = s.D0 * s.D1 * s.D2;
    P.pixsz = s.C * P.cs;
    P.img_elems = s.H * s.W * P.pixsz;
    const int eb = s.dtype == 0 ? 4 : 2;
    P.in_bytes = (int)(s.in_elems() * eb);
    P.kernel_bytes = (int)(s.kernel_elems() * eb);
    const KStrides ks64 = kernel_strides(s);
    P.ks = KStrides32{(int)ks64.base, (int)ks64.sp, (int)ks64.sq, (int)ks64.sc,
                      (int)ks64.sm, (int)ks64.sd0, (int)ks64.sd2, (int)ks64.sd3};
    P.mg_KT = magic_of(P.KT); P.mg_D2 = magic_of(s.D2); P.mg_kw = magic_of(s.kw);
    P.mg_D1 = magic_of(s.D1); P.mg_hw = magic_of(P.hw); P.mg_Wo = magic_of(s.Wo);
    P.mg_D3 = magic_of(s.D3);
    P.out16 = s.out16;
    pl.bnt = P.cols <= 16 ? 1 : P.cols <= 32 ? 2 : P.cols <= 48 ? 3 : 4;
    pl.bmt = P.rows <= 16 ? 1 : 2;
    P.row_tiles = (P.rows + 16 * pl.bmt - 1) / (16 * pl.bmt);
    P.col_tiles = (P.cols + 16 * pl.bnt - 1) / (16 * pl.bnt);
    P.slabs = (P.Ktot + KS - 1) / KS;
    // The K loop is cut over workgroups when the tiles alone would leave CUs idle or give each
    // a long serial K loop: towards two workgroups per CU, every piece at least 4 slabs.
    const long long tiles = (long long)P.row_tiles * P.col_tiles * s.D0;
    int nsplit = 1;
    if (tiles < 512 && P.slabs >= 8) {
        nsplit = (int)(512 / tiles);
        if (nsplit > P.slabs / 4) nsplit = P.slabs / 4;
        if (nsplit < 1) nsplit = 1;
    }
    P.slabs_per_split = (P.slabs + nsplit - 1) / nsplit;
    P.nsplit = (P.slabs + P.slabs_per_split - 1) / P.slabs_per_split;
    pl.blocks = tiles * P.nsplit;
    // a partial-result pass is also how a 16-bit output is produced from split sums
    pl.partial_bytes = P.nsplit > 1 ? (size_t)P.nsplit * P.out_elems * sizeof(float) : 0;
    pl.veca = s.D2 % 4 == 0;
    const KStrides32& k = P.ks;
    pl.vecb = s.D3 % 4 == 0 && k.sd3 == 1 && k.base % 4 == 0 && k.sp % 4 == 0 && k.sq % 4 == 0 &&
              k.sc % 4 == 0 && k.sm % 4 == 0 && k.sd0 % 4 == 0 && k.sd2 % 4 == 0;
    return pl;
}

template <typename Tag, int BMT, int BNT>
hipError_t launch_vec(const SmallPlan& pl, hipStream_t stream)
{
    const dim3 grid((unsigned)pl.blocks), block(256);
    if (pl.veca && pl.vecb)
        igemm_small_kernel<Tag, BMT, BNT, true, true><<<grid, block, 0, stream>>>(pl.P);
    else if (pl.veca)
        igemm_small_kernel<Tag, BMT, BNT, true, false><<<grid, block, 0, stream>>>(pl.P);
    else if (pl.vecb)
        igemm_small_kernel<Tag, BMT, BNT, false, true><<<grid, block, 0, stream>>>(pl.P);
    else
        igemm_small_kernel<Tag, BMT, BNT, false, false><<<grid, block, 0, stream>>>(pl.P);
    return hipGetLastError();
}

template <typename Tag>
hipError_t launch_tile(const SmallPlan& pl, hipStream_t stream)
{
    if (pl.bmt == 1) {
        switch (pl.bnt) {
            case 1: return launch_vec<Tag, 1, 1>(pl, stream);
            case 2: return launch_vec<Tag, 1, 2>(pl, stream);
            case 3: return launch_vec<Tag, 1, 3>(pl, stream);
            default: return launch_vec<Tag, 1, 4>(pl, stream);
        }
    }
    switch (pl.bnt) {
        case 1: return launch_vec<Tag, 2, 1>(pl, stream);
        case 2: return launch_vec<Tag, 2, 2>(pl, stream);
        case 3: return launch_vec<Tag, 2, 3>(pl, stream);
        default: return launch_vec<Tag, 2, 4>(pl, stream);
    }
}

}  // namespace

bool igemm_small_eligible(const ConvShape& s)
{
    if (s.pad_w_set || s.out_view) return false;
    // 32-bit row, column and K indices, and exact divisions by multiplication (x * d < 2^32)
    const long long rows = s.pixels() * s.D1, cols = (long long)s.M * s.D3;
    const long long KT = (long long)s.C * s.D2, Ktot = (long long)s.kh * s.kw * KT;
    const long long hw = (long long)s.Ho * s.Wo;
    const long long lim = 1LL << 32;
    if (rows >= (1LL << 30) || cols >= (1LL << 24) || Ktot >= (1LL << 26)) return false;
    if (rows * s.D1 >= lim || s.pixels() * hw >= lim || hw * s.Wo >= lim) return false;
    if (cols * s.D3 >= lim || Ktot * KT >= lim || KT * s.D2 >= lim) return false;
    if ((long long)s.kh * s.kw * s.kw >= lim) return false;
    if ((long long)s.D0 * s.D1 * s.D2 >= (1LL << 24)) return false;
    // 24-bit multiplications of pixel positions and strides
    if ((long long)s.H * s.W >= (1LL << 24) || (long long)s.C * s.D0 * s.D1 * s.D2 >= (1LL << 24))
        return false;
    // operands are addressed with 32-bit byte offsets through buffer descriptors
    const long long eb = s.dtype == 0 ? 4 : 2;
    if ((long long)s.in_elems() * eb >= (1LL << 31) || (long long)s.kernel_elems() * eb >= (1LL << 31))
        return false;
    if (s.kernel_view) {  // a view must stay inside the tensor it rearranges
        const long long ext[7] = {s.kh, s.kw, s.C, s.M, s.D0, s.D2, s.D3};
        const long long str[7] = {s.k_sp, s.k_sq, s.k_sc, s.k_sm, s.k_sd0, s.k_sd2, s.k_sd3};
        long long lo = s.k_base, hi = s.k_base;
        for (int i = 0; i < 7; ++i) (str[i] < 0 ? lo : hi) += str[i] * (ext[i] - 1);
        if (lo < 0 || hi >= (long long)s.kernel_elems()) return false;
    }
    const long long tiles = ((rows + 31) / 32) * ((cols + 63) / 64) * s.D0;
    if (tiles * ((Ktot + KS - 1) / KS) >= (1LL << 31)) return false;
    return true;
}

// The library's choice for problems this small: the matrix instructions here run at the fp32
// rate whatever the operands' type, so 16-bit problems leave for the 16-bit kernels earlier.
bool igemm_small_preferred(const ConvShape& s)
{
    if (!igemm_small_eligible(s)) return false;
    // Measured against the any-shape kernel (three launches for problems this small) on
    // convolution and fully-connected shapes: fp32 problems win up to about 2.4e9 nominal FLOPs
    // and tie at 1e10; 16-bit problems win up to 3e8 -- up to 1.2e9 when the capsule rows are
    // shorter than the 8 elements that kernel moves in one piece.
    // A layer of very many tiles with a short K loop each (the fully-connected layer's input
    // gradient: a 1x1 convolution with 4608 output columns and K = 40) pays this kernel's fixed
    // cost per tile too often: measured 40 us against 29 us.
    const double flops = 2.0 * (double)s.out_elems() * s.kh * s.kw * s.C * s.D2;
    if (small_plan(s).blocks > 1024) return false;
    return flops <= (s.dtype == 0 ? 4e9 : s.D2 % 8 == 0 ? 4e8 : 1.5e9);
}

size_t igemm_small_workspace_bytes(const ConvShape& s)
{
    return igemm_small_eligible(s) ? small_plan(s).partial_bytes : 0;
}

hipError_t launch_igemm_small(const ConvShape& s, const void* in, const void* kernel, float* out,
                              void* workspace, hipStream_t stream)
{
    SmallPlan pl = small_plan(s);
    if (pl.blocks <= 0 || pl.blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    pl.P.in = in;
    pl.P.kernel = kernel;
    float* partial = static_cast<float*>(workspace);
    const bool split = pl.P.nsplit > 1;
    pl.P.out = split ? partial : out;
    if (split) pl.P.out16 = 0;  // the reduction rounds
    hipError_t err;
    switch (s.dtype) {
        case 0: err = launch_tile<f32_tag>(pl, stream); break;
        case 1: err = launch_tile<bf16_tag>(pl, stream); break;
        case 2: err = launch_tile<f16_tag>(pl, stream); break;
        default: return hipErrorInvalidValue;
    }
    if (err != hipSuccess || !split) return err;
    return launch_splitk_reduce(partial, out, pl.P.out_elems, pl.P.nsplit, stream, s.out16);
}

}  // namespace capscaps
