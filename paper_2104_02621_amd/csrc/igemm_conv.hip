// Matrix-core path of the capsule convolution forward pass (paper Algorithm 2), written as an
// implicit GEMM per leading capsule index d0:
//
//     rows     r = (pixel, d1)         pixel = (n, x, y) flattened          N*H'*W'*D1 of them
//     columns  j = (m, d3)                                                   M*D3 of them
//     K index  k = (tap, c, d2)        tap = (p, q)                          kh*kw*C*D2 of them
//
//     O[r][j] = sum_k I[pixel shifted by tap][c][d0][d1][d2] * K[tap][c][m][d0][d2][d3]
//
// The paper's scheme 1 (Algorithm 3) materialises the left operand (capsule im2col, then a
// copy per output channel) and the right operand (a copy per output pixel) in memory and sums
// the products in a separate pass; here the window addressing is index arithmetic while
// staging tiles into LDS, and the sum over taps and channels is the GEMM's K loop.
//
// Data movement unit: a 16-byte "chunk" = CH consecutive K elements of one row (CH = 8 for
// 16-bit types, 4 for fp32).  Per tap the K extent C*D2 is cut into chunks; a stage of the
// K loop covers 8 chunks of every row and column of the tile.  LDS holds a stage as
// [chunk 0..7][row or column][16 bytes], so the 32 lanes that feed one MFMA operand read 512
// contiguous bytes.  The kernel tensor is repacked once per call into
// Kp[d0][tap][chunk][column][CH] (zero-padded), which makes its stage loads plain contiguous
// copies and puts the contracted index innermost as the matrix cores want it.
//
// MFMA orientation: the matrix instruction's row operand is the kernel (columns j), its column
// operand the input (rows r).  Each lane then owns 4 consecutive j = 4 consecutive d3 of one
// output row, i.e. one 16-byte store.  Because both operands of an MFMA take their K elements
// in the same lane order, any fixed assignment of chunk halves to lanes is a valid K order.
#include <hip/hip_runtime.h>

#include "igemm_common.h"

namespace capscaps {
namespace {

// ---------------------------------------------------------------------------------------------
// Kernel repack: Kp[..][j][e] = K[tap][c][m][d0][d2][d3] with k = kq*CH+e = c*D2+d2,
// j = m*D3+d3; zero where k >= C*D2 or j >= M*D3.  One thread per 16-byte chunk.  Chunk order
// is the order in which the consuming kernel walks K:  kgroup = 0: [d0][tap][kq] (tap outermost);
// kgroup = g > 0: [d0][kq / g][tap][kq % g] (groups of g chunks outermost, tap inside).
// Where kernel element (p, q, c, m, d0, d2, d3) lies in the tensor handed to the call (elements).
struct KernelStrides {
    long long base, sp, sq, sc, sm, sd0, sd2, sd3;
};
template <typename E, int CH>
__global__ __launch_bounds__(256) void repack_kernel(const E* __restrict__ kernel,
                                                     E* __restrict__ kp, int ntaps, int kw, int D2,
                                                     int D3, int KT, int KQP, int cols, int colsp,
                                                     int kgroup, int cw, KernelStrides ks,
                                                     size_t total_chunks)
{
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= total_chunks) return;
    size_t r = id;
    const int j = (int)(r % colsp); r /= colsp;
    int kq, tap, d0;
    if (kgroup > 0) {
        const int kql = (int)(r % kgroup); r /= kgroup;
        tap = (int)(r % ntaps);            r /= ntaps;
        const int groups = KQP / kgroup;
        kq = (int)(r % groups) * kgroup + kql;
        d0 = (int)(r / groups);
    } else {
        kq = (int)(r % KQP);  r /= KQP;
        tap = (int)(r % ntaps);
        d0 = (int)(r / ntaps);
    }
    E v[CH];
#pragma unroll
    for (int e = 0; e < CH; ++e) {
        const int k = kq * cw + e;  // cw valid elements per chunk, the rest of the slot zero
        E x = 0;
        if (e < cw && k < KT && j < cols) {
            const int c = k / D2, d2 = k % D2, m = j / D3, d3 = j % D3;
            const int p = tap / kw, q = tap - p * kw;
            x = kernel[ks.base + p * ks.sp + q * ks.sq + c * ks.sc + m * ks.sm + d0 * ks.sd0 +
                       d2 * ks.sd2 + d3 * ks.sd3];
        }
        v[e] = x;
    }
    chunk_t out;
    __builtin_memcpy(&out, v, 16);
    reinterpret_cast<chunk_t*>(kp)[id] = out;
}

// Deterministic split-K reduction: out[e] = partial[0][e] + partial[1][e] + ... in that order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial,
                                                            float* __restrict__ out,
                                                            long long elems, int nsplit, int out16)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= elems) return;
    float acc = partial[e];
    for (int s = 1; s < nsplit; ++s) acc += partial[(long long)s * elems + e];
    store1(out, e, acc, out16);
}
// The same for element counts that are a multiple of 4: 16-byte loads, and the loads of 8 partial
// results in flight before their additions (which keep the order above).
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const float4v* __restrict__ partial,
                                                             float* __restrict__ out,
                                                             long long quads, int nsplit, int out16)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= quads) return;
    float4v acc = partial[e];
    int s = 1;
    for (; s + 8 <= nsplit; s += 8) {
        float4v v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(long long)(s + u) * quads + e];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; s < nsplit; ++s) acc += partial[(long long)s * quads + e];
    store4(out, 4 * e, acc, out16);
}

// ---------------------------------------------------------------------------------------------
// VB: bytes the input-side loader moves at a time.  16: a chunk never straddles a capsule row
// (D2 % CH == 0, D2/CH a power of two); 8: half a chunk never does (16-bit capsule rows of 4,
// 12, 20 .. elements, fp32 rows of 2, 6, 10 ..): two 8-byte loads per chunk; 0: element-wise.
// VB == 16 -> one
// 16-byte load per chunk; otherwise element-wise gather.   ST4: D3 % 4 == 0 -> 16-byte stores.
template <typename Tag, int VB, bool ST4, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) void igemm_kernel(const IgemmParams P)
{
    typedef typename Tag::elem E;
    constexpr int NT = 64 * WGM * WGN;
    constexpr int CH = 16 / (int)sizeof(E);
    constexpr int WM = BM / WGM, WN = BN / WGN;  // wave tile: rows (pixel,d1) x columns (m,d3)
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ACH = 8 * BM / NT, BCH = 8 * BN / NT;  // chunks per thread per stage
    constexpr int STAGE = 8 * (BM + BN);                 // chunks per LDS stage buffer
    static_assert(NT % BM == 0 && NT % BN == 0, "one row / column per loader thread");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tiles are made of 32x32 MFMA tiles");

    extern __shared__ chunk_t lds[];

    // ---- which tile: consecutive logical tiles go to the same XCD (blocks are dealt to the 8
    // XCDs round-robin), column tiles fastest so that neighbours share input rows in that L2.
    const int nb = gridDim.x;
    int L = blockIdx.x;
    {
        const int per = nb / 8, full = per * 8;
        if ((int)blockIdx.x < full) L = ((int)blockIdx.x % 8) * per + (int)blockIdx.x / 8;
    }
    const int col_tile = L % P.col_tiles;
    int rest = L / P.col_tiles;
    const int row_tile = rest % P.row_tiles;
    rest /= P.row_tiles;
    const int d0 = rest % P.D0;
    const int split = rest / P.D0;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int h = lane >> 5, lr = lane & 31;

    const long long row0 = (long long)row_tile * BM;
    const int col0 = col_tile * BN;

    // ---- loader set-up: this thread stages chunks of one fixed row of the tile
    const int a_row = tid % BM;
    const int a_kq0 = tid / BM;          // first chunk slot; slots advance by NT/BM
    constexpr int A_STEP = NT / BM;
    const long long rg = row0 + a_row;
    const bool row_ok = rg < P.rows;
    long long a_base = 0;
    int ih0 = 0, iw0 = 0;
    {
        const long long rr = row_ok ? rg : 0;
        const long long pixel = rr / P.D1;
        const int d1 = (int)(rr % P.D1);
        const int hw = P.Ho * P.Wo;
        const long long n = pixel / hw;
        const int rem = (int)(pixel % hw);
        const int x = rem / P.Wo, y = rem % P.Wo;
        ih0 = x * P.stride - P.pad;
        iw0 = y * P.stride - P.pad;
        a_base = ((n * P.H + ih0) * P.W + iw0) * P.pixsz + (long long)(d0 * P.D1 + d1) * P.D2;
    }
    const E* __restrict__ in = static_cast<const E*>(P.in);
    const int b_col = tid % BN;
    const int b_kq0 = tid / BN;
    constexpr int B_STEP = NT / BN;
    const chunk_t* __restrict__ kp = static_cast<const chunk_t*>(P.kp);

    chunk_t areg[ACH], breg[BCH];

    auto load_stage = [&](int st) {
        const int tap = st / P.spt;
        const int kq_stage = (st - tap * P.spt) * 8;
        const int p = tap / P.kw, q = tap - p * P.kw;
        const bool ok = row_ok && (unsigned)(ih0 + p) < (unsigned)P.H &&
                        (unsigned)(iw0 + q) < (unsigned)P.W;
        const E* src = in + a_base + ((long long)p * P.W + q) * P.pixsz;
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int kq = kq_stage + a_kq0 + i * A_STEP;
            chunk_t v = {0u, 0u, 0u, 0u};
            if (VB == 16) {
                const int k0 = kq * CH;
                if (ok && k0 < P.KT) {
                    const int c = kq >> P.d2c_shift;
                    const int d2 = k0 - c * P.D2;
                    v = *reinterpret_cast<const chunk_t*>(src + (long long)c * P.cs + d2);
                }
            } else if (VB == 8) {
                typedef unsigned int half_chunk_t __attribute__((ext_vector_type(2)));
                half_chunk_t piece[2] = {{0u, 0u}, {0u, 0u}};
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int k0 = kq * CH + u * (CH / 2);
                    if (ok && k0 < P.KT) {
                        const int c = P.d2_magic ? (int)__umulhi((unsigned)k0, P.d2_magic) : k0 / P.D2;
                        const int d2 = k0 - c * P.D2;
                        piece[u] = *reinterpret_cast<const half_chunk_t*>(src + (long long)c * P.cs + d2);
                    }
                }
                v = chunk_t{piece[0][0], piece[0][1], piece[1][0], piece[1][1]};
            } else {
                E tmp[CH];
#pragma unroll
                for (int e = 0; e < CH; ++e) {
                    const int k = kq * CH + e;
                    E xval = 0;
                    if (ok && k < P.KT) {
                        const int c = k / P.D2;
                        const int d2 = k - c * P.D2;
                        xval = src[(long long)c * P.cs + d2];
                    }
                    tmp[e] = xval;
                }
                __builtin_memcpy(&v, tmp, 16);
            }
            areg[i] = v;
        }
        const chunk_t* bsrc =
            kp + (((size_t)d0 * P.ntaps + tap) * P.KQP + kq_stage) * P.colsp + col0 + b_col;
#pragma unroll
        for (int i = 0; i < BCH; ++i) breg[i] = bsrc[(size_t)(b_kq0 + i * B_STEP) * P.colsp];
    };
    auto store_stage = [&](int buf) {
        chunk_t* A = lds + buf * STAGE;
        chunk_t* B = A + 8 * BM;
#pragma unroll
        for (int i = 0; i < ACH; ++i) A[(a_kq0 + i * A_STEP) * BM + a_row] = areg[i];
#pragma unroll
        for (int i = 0; i < BCH; ++i) B[(b_kq0 + i * B_STEP) * BN + b_col] = breg[i];
    };

    float16v acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int st_begin = split * P.stages_per_split;
    int st_end = st_begin + P.stages_per_split;
    if (st_end > P.stages) st_end = P.stages;

    if (st_begin < st_end) {
        load_stage(st_begin);
        store_stage(0);
    }
    __syncthreads();
    for (int st = st_begin; st < st_end; ++st) {
        const int buf = (st - st_begin) & 1;
        const bool more = st + 1 < st_end;
        if (more) load_stage(st + 1);
        const chunk_t* A = lds + buf * STAGE;
        const chunk_t* B = A + 8 * BM;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            chunk_t ka[TN], ib[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a) ka[a] = B[(2 * t + h) * BN + wn * WN + a * 32 + lr];
#pragma unroll
            for (int b = 0; b < TM; ++b) ib[b] = A[(2 * t + h) * BM + wm * WM + b * 32 + lr];
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int b = 0; b < TM; ++b) Mma<Tag>::run(ka[a], ib[b], acc[a][b]);
        }
        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane (h, lr) of MFMA tile (a, b) holds, in registers 4g..4g+3, columns
    // j = 8g + 4h + 0..3 of the tile for output row lr of the tile.
    float* __restrict__ out = P.out + (long long)split * P.out_elems;
    const int caps_out = P.D0 * P.D1 * P.D3;
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const long long orow = row0 + wm * WM + b * 32 + lr;
        if (orow >= P.rows) continue;
        const long long pixel = orow / P.D1;
        const int d1 = (int)(orow % P.D1);
        float* orow_ptr = out + pixel * P.M * caps_out + (long long)(d0 * P.D1 + d1) * P.D3;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j0 = col0 + wn * WN + a * 32 + 8 * g + 4 * h;
                if (ST4) {
                    if (j0 < P.cols) {
                        const int m = j0 / P.D3, d3 = j0 - m * P.D3;
                        float4v v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                                     acc[a][b][4 * g + 3]};
                        *reinterpret_cast<float4v*>(orow_ptr + (long long)m * caps_out + d3) = v;
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + u;
                        if (j < P.cols) {
                            const int m = j / P.D3, d3 = j - m * P.D3;
                            orow_ptr[(long long)m * caps_out + d3] = acc[a][b][4 * g + u];
                        }
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
struct TileChoice {
    int BM, BN;
};

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

struct Plan {
    IgemmParams P;
    TileChoice tile;
    int vb;  // bytes per input-side load: 16, 8, or 0 = element-wise
    bool st4;
    bool fast;  // tuned 16-bit kernel
    bool via_scratch;  // results go to fp32 scratch first, then through splitk_reduce_kernel
    size_t tail_bytes;  // tuned kernel: scratch for the partial results of its last round
    size_t repack_bytes, partial_bytes;
    long long blocks;
    int CH;
};

// Tile, split and padding decisions for a shape (host side, pure arithmetic).
Plan make_plan(const ConvShape& s, MfmaKernel which)
{
    Plan pl{};
    const int CH = s.dtype == 0 ? 4 : 8;
    pl.CH = CH;
    IgemmParams& P = pl.P;
    P.H = s.H; P.W = s.W; P.C = s.C; P.M = s.M; P.stride = s.stride; P.pad = s.pad;
    P.D0 = s.D0; P.D1 = s.D1; P.D2 = s.D2; P.D3 = s.D3; P.Ho = s.Ho; P.Wo = s.Wo; P.kw = s.kw;
    P.rows = s.pixels() * s.D1;
    P.out_elems = (long long)s.out_elems();
    P.pixsz = (long long)s.C * s.D0 * s.D1 * s.D2;
    P.cs = s.D0 * s.D1 * s.D2;
    P.cols = s.M * s.D3;
    P.KT = s.C * s.D2;
    P.ntaps = s.kh * s.kw;
    const int KQ = ceil_div(P.KT, CH);
    P.KQP = ceil_div(KQ, 8) * 8;
    P.spt = P.KQP / 8;
    P.stages = P.ntaps * P.spt;

    const int d2c = s.D2 / CH;
    const bool vec = (s.D2 % CH == 0) && (d2c & (d2c - 1)) == 0;
    pl.vb = vec ? 16 : s.D2 % (CH / 2) == 0 ? 8 : 0;
    P.d2c_shift = 0;
    if (vec)
        while ((1 << P.d2c_shift) < d2c) ++P.d2c_shift;
    // k / D2 by multiplication: exact while k * D2 < 2^32 (k < KT + 64)
    P.d2_magic = s.D2 > 1 && ((long long)P.KT + 64) * s.D2 < (1LL << 32)
                     ? (unsigned)(((1ULL << 32) + s.D2 - 1) / s.D2)
                     : 0u;
    pl.st4 = s.D3 % 4 == 0;

    // tile: the largest whose grid still gives every CU a few blocks; small problems take
    // small tiles and, if still short of blocks, split the K loop.
    const int kCUs = 256;
    const TileChoice choices[3] = {{256, 256}, {128, 128}, {64, 64}};
    pl.fast = which == MfmaKernel::Tuned16
                  ? igemm16_fast_eligible(s)
                  : which == MfmaKernel::Auto && igemm16_fast_preferred(s);
    int pick = 2;
    if (pl.fast) pick = 0;
    for (int i = 0; i < 3 && !pl.fast; ++i) {
        const long long blocks = (long long)ceil_div(P.rows, choices[i].BM) *
                                 ceil_div(P.cols, choices[i].BN) * s.D0;
        const bool fits_cols = P.cols >= choices[i].BN / 2 || i == 2;
        if (fits_cols && blocks >= 2 * kCUs) { pick = i; break; }
    }
    pl.tile = choices[pick];
    // tuned 16-bit kernel: 128-row tiles (two workgroups per CU) or 256-row tiles
    P.bm = 256;
    if (pl.fast && igemm16_fast_tile_rows(s) == 128) {
        P.bm = 128;
        pl.tile.BM = 128;
    }
    P.row_tiles = ceil_div(P.rows, pl.tile.BM);
    P.col_tiles = ceil_div(P.cols, pl.tile.BN);
    P.colsp = P.col_tiles * pl.tile.BN;
    long long blocks = (long long)P.row_tiles * P.col_tiles * s.D0;
    int nsplit = 1;
    if (blocks < kCUs && !pl.fast) {
        nsplit = ceil_div(2 * kCUs, blocks);
        if (nsplit > P.stages) nsplit = P.stages;
        if (nsplit > 64) nsplit = 64;
    }
    P.stages_per_split = ceil_div(P.stages, nsplit);
    P.nsplit = ceil_div(P.stages, P.stages_per_split);
    pl.blocks = blocks * P.nsplit;
    pl.repack_bytes = (size_t)s.D0 * P.ntaps * P.KQP * P.colsp * 16;
    // this kernel stores fp32 only: a 16-bit output goes through the fp32 scratch and the
    // reduction kernel, which then also converts
    pl.via_scratch = P.nsplit > 1 || (s.out16 != 0 && !pl.fast);
    pl.partial_bytes = pl.via_scratch ? (size_t)P.nsplit * P.out_elems * sizeof(float) : 0;
    P.in_bytes = (long long)s.in_elems() * (s.dtype == 0 ? 4 : 2);
    P.kp_records = (long long)pl.repack_bytes;
    P.out16 = s.out16;
    P.pad_w = s.padw();
    P.out_view = s.out_view ? 1 : 0;
    P.out_base = s.out_base; P.out_sn = s.out_sn; P.out_sx = s.out_sx; P.out_sy = s.out_sy;
    P.out_alloc = s.out_view ? s.out_alloc : P.out_elems;
    P.lpt_timg = P.lpt_a = P.lpt_b = 0;
    if (pl.fast && s.D0 == 1 && s.D1 > 0 && P.bm % s.D1 == 0) {
        // tiles of the tuned kernel hold 256/D1 consecutive pixels; when they do not straddle
        // images, count an image's leading (trailing) tiles all of whose pixels have a window
        // row above (below) the image
        const long long pix = P.bm / s.D1, hw = (long long)s.Ho * s.Wo;
        if (hw % pix == 0 && hw / pix < (1 << 20)) {
            const int timg = (int)(hw / pix);
            int a = 0, b = 0;
            while (a < timg && (((a + 1) * pix - 1) / s.Wo) * s.stride - s.pad < 0) ++a;
            while (b < timg - a &&
                   (((timg - 1 - b) * pix) / s.Wo) * s.stride - s.pad + s.kh - 1 >= s.H) ++b;
            if (a + b > 0 && a + b < timg) {
                P.lpt_timg = timg;
                P.lpt_a = a;
                P.lpt_b = b;
            }
        }
    }
    {
        // the tuned kernel's buffer-store epilogue: byte offsets from a tile's first output
        // pixel (a tile holds 256/D1 consecutive pixels, which may reach into following images)
        // plus one pixel's extent must stay below 2^31
        const long long pix_elems = (long long)s.M * s.D0 * s.D1 * s.D3;
        const long long tile_pix = 256 / (s.D1 > 0 ? s.D1 : 1) + 1;
        const long long hw = (long long)s.Ho * s.Wo;
        long long span;
        if (s.out_view) {
            const long long images = tile_pix / (hw > 0 ? hw : 1) + 2;
            span = images * (s.out_sn > 0 ? s.out_sn : 0) + pix_elems;
        } else {
            span = (tile_pix + 1) * pix_elems;
        }
        const bool d3_ok = s.D3 == 4 || s.D3 == 8 || s.D3 == 16 || s.D3 == 32;
        const bool strides_ok = !s.out_view || (s.out_sn >= 0 && s.out_sx >= 0 && s.out_sy >= 0);
        P.fast_store = d3_ok && strides_ok && span * 4 < (1LL << 31) - (1 << 20) ? 1 : 0;
    }
    // Tuned kernel, last round of tiles.  With T tiles on 256 CUs the last T % 256 tiles run
    // alone while the other CUs idle; when they are few, each is cut into several work items
    // over the channel groups of its K loop, so that the last round takes a fraction of a
    // tile's time; a reduction over the output's last pixels follows.  Only where the last
    // tiles in launch order are the output's last pixels (dense fp32 output, one leading
    // capsule index, plain launch order).
    P.tail_first = P.tail_split = P.tail_pix0 = 0;
    P.tail_elems = 0;
    P.tail_partial = nullptr;
    pl.tail_bytes = 0;
    if (pl.fast && s.D0 == 1 && !s.out_view && s.out16 == 0 && P.lpt_timg == 0 && P.nsplit == 1) {
        const long long T = (long long)P.row_tiles * P.col_tiles;
        const int R = (int)(T % kCUs);
        const int groups = P.KQP / igemm16_fast_kgroup(s);
        if (T > kCUs && R > 0 && R <= kCUs / 2 && R % P.col_tiles == 0 && groups >= 2) {
            int split = kCUs / R;
            if (split > groups) split = groups;
            if (split > 16) split = 16;
            const long long pix_per_tile = P.bm / s.D1;
            const long long pix0 = ((long long)P.row_tiles - R / P.col_tiles) * pix_per_tile;
            const long long pix_elems = (long long)s.M * s.D0 * s.D1 * s.D3;
            const long long elems = (s.pixels() - pix0) * pix_elems;
            if (split >= 2 && pix0 > 0 && pix0 < (1LL << 31) && elems > 0 &&
                (double)split * elems * 4 < (double)(1 << 30)) {
                P.tail_first = (int)(T - R);
                P.tail_split = split;
                P.tail_pix0 = (int)pix0;
                P.tail_elems = elems;
                pl.tail_bytes = (size_t)split * elems * sizeof(float);
                pl.blocks = (T - R) + (long long)R * split;
            }
        }
    }
    // Tuned kernel, launch order.  When the repacked kernel of one leading capsule index is
    // small (a few MB: every XCD can stream all of its column tiles through its 4 MB L2 once per
    // round of tiles), give each XCD a contiguous range of row tiles with all their column
    // tiles, so that the input is fetched by one L2 instead of one per column tile and
    // neighbouring row tiles share their halo rows there (config 3: 0.878 -> 0.855 ms).  With a
    // large repacked kernel that order thrashes the L2s (config 5: 2.5x the misses), and the
    // longest-tiles-first order has its own permutation.
    P.xcd_span = 0;
    if (pl.fast && P.lpt_timg == 0 && pl.repack_bytes / (size_t)s.D0 <= ((size_t)8 << 20)) {
        const long long whole = P.tail_split > 0 ? (long long)P.tail_first
                                                 : (long long)P.row_tiles * P.col_tiles * s.D0;
        const long long unit = 8LL * P.col_tiles;
        const long long span = whole / unit * unit;
        if (span > 0 && span < (1LL << 31)) P.xcd_span = (int)span;
    }
    if (pl.tail_bytes > pl.partial_bytes) pl.partial_bytes = pl.tail_bytes;
    return pl;
}

template <typename Tag, int VB, bool ST4, int BM, int BN>
hipError_t launch_tile(const Plan& pl, hipStream_t stream)
{
    auto kern = igemm_kernel<Tag, VB, ST4, BM, BN, 2, 2>;
    const size_t lds_bytes = (size_t)2 * 8 * (BM + BN) * 16;
    static std::atomic<unsigned long long> lds_set{0};
    hipError_t err = set_dynamic_lds_once(reinterpret_cast<const void*>(kern), (int)lds_bytes, lds_set);
    if (err != hipSuccess) return err;
    kern<<<dim3((unsigned)pl.blocks), dim3(256), lds_bytes, stream>>>(pl.P);
    return hipGetLastError();
}

template <typename Tag, int VB, bool ST4>
hipError_t launch_flags(const Plan& pl, hipStream_t stream)
{
    switch (pl.tile.BM) {
        case 256: return launch_tile<Tag, VB, ST4, 256, 256>(pl, stream);
        case 128: return launch_tile<Tag, VB, ST4, 128, 128>(pl, stream);
        default: return launch_tile<Tag, VB, ST4, 64, 64>(pl, stream);
    }
}

template <typename Tag>
hipError_t launch_typed(const Plan& pl, hipStream_t stream)
{
    if (pl.vb == 16) {
        return pl.st4 ? launch_flags<Tag, 16, true>(pl, stream)
                      : launch_flags<Tag, 16, false>(pl, stream);
    }
    if (pl.vb == 8) {
        return pl.st4 ? launch_flags<Tag, 8, true>(pl, stream)
                      : launch_flags<Tag, 8, false>(pl, stream);
    }
    return pl.st4 ? launch_flags<Tag, 0, true>(pl, stream)
                  : launch_flags<Tag, 0, false>(pl, stream);
}

bool shape_supported(const ConvShape& s)
{
    // 32-bit quantities inside the kernel
    const long long cols = (long long)s.M * s.D3, kt = (long long)s.C * s.D2;
    if (cols > (1 << 24) || kt > (1 << 24)) return false;
    if ((long long)s.D0 * s.D1 * s.D2 > (1 << 24)) return false;
    if ((long long)s.Ho * s.Wo > (1LL << 30)) return false;
    return true;
}

hipError_t launch_igemm(const ConvShape& s, const void* in, const void* kernel, float* out,
                        void* workspace, hipStream_t stream, MfmaKernel which)
{
    Plan pl = make_plan(s, which);
    if (pl.blocks <= 0 || pl.blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    char* ws = static_cast<char*>(workspace);
    void* kp = ws;
    float* partial = reinterpret_cast<float*>(ws + ((pl.repack_bytes + 255) & ~(size_t)255));
    pl.P.in = in;
    pl.P.kp = kp;
    pl.P.out = pl.via_scratch ? partial : out;

    const size_t chunks = pl.repack_bytes / 16;
    const int kgroup = pl.fast ? igemm16_fast_kgroup(s) : 0;
    hipError_t err = launch_repack(s, kernel, kp, pl.CH, pl.P.KQP, pl.P.colsp, kgroup, chunks, stream);
    if (err != hipSuccess) return err;

    if (pl.fast) {
        pl.P.tail_partial = partial;
        err = launch_igemm16_fast(pl.P, pl.blocks, s.dtype, stream);
        if (err != hipSuccess || pl.P.tail_split == 0) return err;
        const long long pix_elems = (long long)s.M * s.D0 * s.D1 * s.D3;
        return launch_splitk_reduce(partial, out + (long long)pl.P.tail_pix0 * pix_elems,
                                    pl.P.tail_elems, pl.P.tail_split, stream);
    }

    switch (s.dtype) {
        case 0: err = launch_typed<f32_tag>(pl, stream); break;
        case 1: err = launch_typed<bf16_tag>(pl, stream); break;
        case 2: err = launch_typed<f16_tag>(pl, stream); break;
        default: return hipErrorInvalidValue;
    }
    if (err != hipSuccess) return err;

    if (pl.via_scratch)
        err = launch_splitk_reduce(partial, out, pl.P.out_elems, pl.P.nsplit, stream, pl.P.out16);
    return err;
}

// scratch of the lane-per-row tuned kernel: repacked kernel, partial sums, paired input
size_t dma32_workspace_bytes(const Dma32Plan& pl)
{
    return ((pl.repack_bytes + 255) & ~(size_t)255) + ((pl.partial_bytes + 255) & ~(size_t)255) +
           pl.pair_bytes;
}

hipError_t launch_dma32(const ConvShape& s, const void* in, const void* kernel, float* out,
                        void* workspace, hipStream_t stream)
{
    Dma32Plan pl = igemm32_dma_plan(s);
    char* ws = static_cast<char*>(workspace);
    float* partial = reinterpret_cast<float*>(ws + ((pl.repack_bytes + 255) & ~(size_t)255));
    pl.P.in = in;
    pl.P.kp = ws;
    pl.P.out = pl.P.nsplit > 1 ? partial : out;
    hipError_t err = hipSuccess;
    if (pl.pair_bytes) {
        // 16-bit: the kernel reads the input with its channels paired, and 8 halves per chunk
        void* paired = ws + dma32_workspace_bytes(pl) - pl.pair_bytes;
        err = launch_pair_channels(s, in, paired, stream);
        if (err != hipSuccess) return err;
        pl.P.in = paired;
    }
    err = launch_repack(s, kernel, ws, s.dtype == 0 ? pl.cw : 8, pl.kqp, pl.P.colsp, pl.P.kch,
                        pl.repack_bytes / 16, stream);
    if (err != hipSuccess) return err;
    err = launch_igemm32_dma(pl, stream);
    if (err != hipSuccess) return err;
    if (pl.P.nsplit > 1)
        err = launch_splitk_reduce(partial, out, pl.P.out_elems, pl.P.nsplit, stream, s.out16);
    return err;
}

}  // namespace

hipError_t launch_repack(const ConvShape& s, const void* kernel, void* kp, int cw, int KQP,
                         int colsp, int kgroup, size_t chunks, hipStream_t stream)
{
    const unsigned rblocks = (unsigned)((chunks + 255) / 256);
    const int ntaps = s.kh * s.kw, KT = s.C * s.D2, cols = s.M * s.D3;
    KernelStrides ks;
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
    if (s.dtype == 0) {
        repack_kernel<float, 4><<<rblocks, 256, 0, stream>>>(
            (const float*)kernel, (float*)kp, ntaps, s.kw, s.D2, s.D3, KT, KQP, cols, colsp,
            kgroup, cw, ks, chunks);
    } else {
        repack_kernel<unsigned short, 8><<<rblocks, 256, 0, stream>>>(
            (const unsigned short*)kernel, (unsigned short*)kp, ntaps, s.kw, s.D2, s.D3, KT, KQP,
            cols, colsp, kgroup, cw, ks, chunks);
    }
    return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float* partial, float* out, long long elems, int nsplit,
                                hipStream_t stream, int out16)
{
    const bool quads = elems % 4 == 0 && (reinterpret_cast<uintptr_t>(partial) & 15u) == 0 &&
                       (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
    if (quads) {
        const unsigned blocks = (unsigned)((elems / 4 + 255) / 256);
        splitk_reduce4_kernel<<<blocks, 256, 0, stream>>>(
            reinterpret_cast<const float4v*>(partial), out, elems / 4, nsplit, out16);
    } else {
        const unsigned blocks = (unsigned)((elems + 255) / 256);
        splitk_reduce_kernel<<<blocks, 256, 0, stream>>>(partial, out, elems, nsplit, out16);
    }
    return hipGetLastError();
}

bool mfma_supported(const ConvShape& s) { return shape_supported(s); }

size_t mfma_workspace_bytes(const ConvShape& s)
{
    if (!shape_supported(s)) return 0;
    if (s.out16 != 0) {
        // 16-bit output is offered with the library's own kernel choice only
        const MfmaKernel which = mfma_auto_kernel(s);
        if (which == MfmaKernel::Dma32) return dma32_workspace_bytes(igemm32_dma_plan(s));
        if (which == MfmaKernel::Small) return igemm_small_workspace_bytes(s);
        const Plan pl = make_plan(s, which);
        return ((pl.repack_bytes + 255) & ~(size_t)255) + pl.partial_bytes;
    }
    size_t need = 0;
    for (MfmaKernel which : {MfmaKernel::Generic, MfmaKernel::Tuned16}) {
        if (which == MfmaKernel::Tuned16 && !igemm16_fast_eligible(s)) continue;
        const Plan pl = make_plan(s, which);
        const size_t bytes = ((pl.repack_bytes + 255) & ~(size_t)255) + pl.partial_bytes;
        if (bytes > need) need = bytes;
    }
    if (igemm32_dma_eligible(s)) {
        const size_t bytes = dma32_workspace_bytes(igemm32_dma_plan(s));
        if (bytes > need) need = bytes;
    }
    if (igemm_small_workspace_bytes(s) > need) need = igemm_small_workspace_bytes(s);
    return need;
}

size_t mfma_auto_workspace_bytes(const ConvShape& s)
{
    if (!shape_supported(s)) return 0;
    const MfmaKernel which = mfma_auto_kernel(s);
    if (which == MfmaKernel::Small) return igemm_small_workspace_bytes(s);
    if (which == MfmaKernel::Dma32) {
        return dma32_workspace_bytes(igemm32_dma_plan(s));
    }
    const Plan pl = make_plan(s, which);
    return ((pl.repack_bytes + 255) & ~(size_t)255) + pl.partial_bytes;
}

MfmaKernel mfma_auto_kernel(const ConvShape& s)
{
    if (igemm32_dma_preferred(s)) return MfmaKernel::Dma32;
    if (igemm16_fast_preferred(s)) return MfmaKernel::Tuned16;
    if (igemm_small_preferred(s)) return MfmaKernel::Small;
    return MfmaKernel::Generic;
}

bool mfma_dma32_supported(const ConvShape& s)
{
    return shape_supported(s) && igemm32_dma_eligible(s);
}

bool mfma_small_supported(const ConvShape& s)
{
    return shape_supported(s) && igemm_small_eligible(s);
}

bool mfma_tuned16_supported(const ConvShape& s)
{
    return shape_supported(s) && igemm16_fast_eligible(s);
}

hipError_t launch_mfma(const ConvShape& s, const void* in, const void* kernel, float* out,
                       void* workspace, hipStream_t stream, MfmaKernel which)
{
    // geometry overrides exist in the two tuned kernels only (a kernel view in all: it is the
    // repack pass that reads the kernel tensor)
    if ((s.pad_w_set || s.out_view) && !(which == MfmaKernel::Tuned16 && igemm16_fast_eligible(s)) &&
        !(which == MfmaKernel::Dma32 && igemm32_dma_eligible(s)))
        return hipErrorInvalidValue;
    if (which == MfmaKernel::Dma32 || (which == MfmaKernel::Auto && igemm32_dma_preferred(s)))
        return launch_dma32(s, in, kernel, out, workspace, stream);
    if (which == MfmaKernel::Small ||
        (which == MfmaKernel::Auto && mfma_auto_kernel(s) == MfmaKernel::Small))
        return launch_igemm_small(s, in, kernel, out, workspace, stream);
    return launch_igemm(s, in, kernel, out, workspace, stream, which);
}

}  // namespace capscaps
