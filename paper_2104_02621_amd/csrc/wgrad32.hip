// Kernel gradient of the capsule convolution for fp32 operands on the matrix cores: the same
// per-tap GEMM as wgrad16.hip (rows (c,d2), columns (m,d3), K = (n,x,y,d1) over the output
// pixels whose tap lies inside the image; the K_diff result of the paper's Algorithm 4 read as
// the derivative of Algorithm 2's sum), for capsule heights D1 of 3, 4, 6, 8, 12 or 16 floats.
//
// Unless the capsules are square (see NAT below), a pre-pass writes capsule-transposed copies
// It[n][h][w][c][d0][d2][d1] and Gt[n][x][y][m][d0][d3][d1], so the D1 contracted values of one
// (pixel, row) are contiguous.
// Data moves in 16-byte LDS slots of CW = 3 or 4 floats ("chunks", D1 = CW * D1C): a 12-byte
// buffer load lands at a 16-byte lane stride in LDS, so both widths read operands with one
// 16-byte LDS load per lane and feed CW MFMA 32x32x2 instructions from it (element u of the
// lower and of the upper half wave form the K pair of instruction u).
//
// fp32 layers have few rows and columns per tap (config 2: 96 x 96) and a very long K, so the
// tile is small -- 64*NW rows x 32*TN columns, wave w owning rows 64w..64w+63 against all
// columns -- and the K loop is split over image ranges (partial sums to scratch, added in a
// fixed order by the shared reduction kernel).  Lane i of a wave copies row 64w+i: a fixed
// lane offset plus the scalar offset of the pixel.  A stage is 4 chunks = 4/D1C pixels; ring of
// 3 LDS stages, one barrier per stage, several workgroups per CU overlap copies and MFMAs.
#include <hip/hip_runtime.h>

#include "igemm_common.h"
#include "lds_dma.h"

namespace capscaps {
namespace {

// KCH chunks per row and stage (2 for the two-wave tile unless a capsule column is 4 chunks,
// else 4), ring of NB stages:
// small stages keep the LDS footprint of a workgroup low, so that two or more waves share each
// SIMD and one wave's copies and scalar work run under another's MFMAs.
constexpr int stage_chunks(int d1c, int nw) { return d1c == 4 || nw == 4 ? 4 : 2; }
// waves per SIMD the kernel is compiled for: three where 168 registers hold the accumulators
// of the column tiles and a small stage's operands, else two
constexpr int waves_per_simd(int tn, int kch) { return tn <= 3 && kch == 2 ? 3 : 2; }
// three stages where six two-wave workgroups are to share a CU (24 KB each; measured on config 2
// against four stages and five workgroups: 0.98 against 1.07 ms), four for the other small stages
constexpr int ring_depth(int kch, int tn) { return kch == 2 && waves_per_simd(tn, kch) == 2 ? 4 : 3; }


struct Wgrad32Params {
    const void* it;  // capsule-transposed input
    const void* gt;  // capsule-transposed output gradient
    float* out;      // dK, or partial sums [split][kernel elements]
    int N, H, W, C, M, kw, stride, pad, D0, D1, D2, D3, Ho, Wo;
    int D1C;         // chunks per capsule column: D1 = CW * D1C, D1C in {1, 2, 4}
    int rows, cols;  // C*D2, M*D3
    int row_tiles, col_tiles, ntaps;
    int tiles;       // ntaps * D0 * row_tiles * col_tiles
    int natural;          // 1: it / gt are the input and the output gradient themselves
    unsigned d3_magic;    // ceil(2^32 / D3): column index / D3 as a multiplication; 0 = divide
    int nsplit;           // ranges the K loop (a tap's valid output pixels) is cut into
    long long items;      // tiles * nsplit = workgroups
    long long out_elems;  // elements of dK
    long long it_img_bytes, gt_img_bytes;
};

// dst[x][b][a] = src[x][a][b] for matrices of A x B floats.  One thread per element.
__global__ __launch_bounds__(256) void transpose_caps32_kernel(const float* __restrict__ src,
                                                               float* __restrict__ dst, int A,
                                                               int B, size_t total)
{
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int a = (int)(id % A);
    const size_t rest = id / A;
    const int b = (int)(rest % B);
    const size_t mat = rest / B;
    dst[id] = src[(mat * A + a) * B + b];
}

// NAT: the operands are the tensors themselves (square capsules, D1 = D2 = D3) instead of the
// capsule-transposed copies.  The copies are the same -- lane i then brings row (c, d1) with its
// d2 values where the transposed tensor has row (c, d2) with its d1 values, at the same byte
// offsets -- and the MFMA operands, single floats, are picked out of the slots one by one:
// row (c, d2) at K index (pixel, d1) is element d2 of slot (pixel, c, d1).
template <int CW, int TN, int NW, int KCH, bool NAT>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(waves_per_simd(TN, KCH)))) void wgrad32_kernel(const Wgrad32Params P)
{
    constexpr int NB = ring_depth(KCH, TN);
    constexpr int BM = 64 * NW, BN = 32 * TN, BNL = (BN + 63) / 64 * 64, TM = 2;
    constexpr int A_BYTES = KCH * BM * 16, B_BYTES = KCH * BNL * 16;
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int NBC = KCH * BNL / 64;  // column-side copies per stage, all waves
    constexpr int BPW = NBC / NW;        // ... per wave
    static_assert(NBC % NW == 0, "column copies divide evenly over the waves");
    constexpr int NCOPY = KCH + BPW;     // copies per wave and stage
    constexpr int OOB = (int)0x80000000u;
    // at a barrier the copies of the NB-2 most recent stages may still be in flight
    constexpr int KEEP = (NB - 2) * NCOPY;
    static_assert(KEEP < 64, "vmcnt is a 6-bit counter");
    constexpr int VMCNT_KEEP = 0x0F70 | (KEEP & 15) | ((KEEP >> 4) << 14);

    extern __shared__ char smem[];

    // ---- which item: each XCD (workgroups are dealt to the 8 XCDs in turn) gets a contiguous
    // range of items, image range slowest, so its resident workgroups read the same pixels
    long long item = blockIdx.x;
    {
        const long long per = P.items / 8;
        if (item < per * 8) item = (item % 8) * per + item / 8;
    }
    const int split = (int)(item / P.tiles);
    int rest = (int)(item % P.tiles);
    const int col_tile = rest % P.col_tiles;
    rest /= P.col_tiles;
    const int row_tile = rest % P.row_tiles;
    rest /= P.row_tiles;
    const int tap = rest % P.ntaps;
    const int d0 = rest / P.ntaps;
    const int tp = tap / P.kw, tq = tap - tp * P.kw;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, lr = lane & 31;

    // ---- the pixels of this item.  Per image the output pixels whose tap (tp, tq) reads a
    // real input pixel form a rectangle; the rectangles of all images, image after image, row
    // after row, are one sequence, of which this item contracts the range [t0, t1).
    const int s = P.stride;
    int nx, ny, x_lo, y_lo;
    {
        const int tx = P.pad - tp, ty = P.pad - tq;
        x_lo = tx > 0 ? (tx + s - 1) / s : 0;
        y_lo = ty > 0 ? (ty + s - 1) / s : 0;
        const int hx = P.H - 1 + tx, hy = P.W - 1 + ty;
        int x_hi = hx >= 0 ? hx / s : -1, y_hi = hy >= 0 ? hy / s : -1;
        if (x_hi > P.Ho - 1) x_hi = P.Ho - 1;
        if (y_hi > P.Wo - 1) y_hi = P.Wo - 1;
        nx = x_hi - x_lo + 1;
        ny = y_hi - y_lo + 1;
        if (nx <= 0 || ny <= 0) nx = ny = 0;
    }
    // every tap's sequence is cut into nsplit equal ranges
    const long long rect = (long long)nx * ny, total = rect * P.N;
    const long long tps = (total + P.nsplit - 1) / P.nsplit;
    long long t0 = (long long)split * tps;
    if (t0 > total) t0 = total;
    long long t1 = t0 + tps;
    if (t1 > total) t1 = total;
    const int npix = (int)(t1 - t0);
    const int n0 = npix > 0 ? (int)(t0 / rect) : 0;
    const int n_last = npix > 0 ? (int)((t1 - 1) / rect) : n0;
    const int r0 = npix > 0 ? (int)(t0 - (long long)n0 * rect) : 0;  // position in image n0
    const int xs = ny > 0 ? r0 / ny : 0, ys = ny > 0 ? r0 - xs * ny : 0;
    const int ipix = P.C * P.D0 * P.D2 * P.D1 * 4;  // bytes per pixel of It / Gt
    const int gpix = P.M * P.D0 * P.D3 * P.D1 * 4;
    const int i_step = s * ipix, g_step = gpix;
    const int i_rowjump = (s * P.W - (ny - 1) * s) * ipix, g_rowjump = (P.Wo - (ny - 1)) * gpix;
    const int i_imgjump = (P.H * P.W - nx * s * P.W) * ipix, g_imgjump = (P.Ho * P.Wo - nx * P.Wo) * gpix;
    // offsets are relative to image n0
    int i_cur = (((x_lo + xs) * s - (P.pad - tp)) * P.W + ((y_lo + ys) * s - (P.pad - tq))) * ipix;
    int g_cur = ((x_lo + xs) * P.Wo + y_lo + ys) * gpix;
    int left = npix, yl = ny - ys, xl = nx - xs;
    const int n1 = n_last + 1;

    const char* it_base = static_cast<const char*>(P.it) + (long long)n0 * P.it_img_bytes;
    const char* gt_base = static_cast<const char*>(P.gt) + (long long)n0 * P.gt_img_bytes;
    const rsrc_t rs_it = make_rsrc(it_base, (unsigned)((n1 - n0) * P.it_img_bytes));
    const rsrc_t rs_gt = make_rsrc(gt_base, (unsigned)((n1 - n0) * P.gt_img_bytes));
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;

    // ---- per-lane constants: byte offset of the lane's row (column) within a pixel, or the
    // out-of-range mark past the last row (column): those copy zeros
    unsigned a_voff;
    {
        const int R = row_tile * BM + wave * 64 + lane;
        const int c = R / P.D2, d2 = R - c * P.D2;
        a_voff = R < P.rows ? (unsigned)((((c * P.D0 + d0) * P.D2 + d2) * P.D1) * 4) : (unsigned)OOB;
    }
    unsigned b_voff[BPW];
#pragma unroll
    for (int j = 0; j < BPW; ++j) {
        const int blk = wave * BPW + j;                 // chunk blk / (BNL/64), column block blk % ..
        const int jl = (blk % (BNL / 64)) * 64 + lane;  // column within the tile
        const int J = col_tile * BN + jl;
        const int m = J / P.D3, d3 = J - m * P.D3;
        b_voff[j] = (jl < BN && J < P.cols)
                        ? (unsigned)((((m * P.D0 + d0) * P.D3 + d3) * P.D1) * 4)
                        : (unsigned)OOB;
    }

    const int pps = KCH / P.D1C;                     // pixels per stage
    const int d1c_shift = P.D1C == 1 ? 0 : P.D1C == 2 ? 1 : 2;
    const int nstages = (npix + pps - 1) / pps;
    const int nstages_pad = (nstages + NB - 1) / NB * NB;  // surplus stages contract zeros

    // copies of the next stage (scalar pixel walk: the stage's pixels, each the next valid
    // output pixel of the tap's rectangle, image after image; past the last one zero fill)
    auto issue_stage = [&](int slot) {
        const unsigned stage = lds0 + slot * STAGE_BYTES;
        int i_soff[KCH], g_soff[KCH];
#pragma unroll
        for (int j = 0; j < KCH; ++j) {
            i_soff[j] = OOB;
            g_soff[j] = OOB;
            if (j < pps) {
                if (left > 0) {
                    i_soff[j] = i_cur;
                    g_soff[j] = g_cur;
                }
                --left;
                --yl;
                if (yl != 0) {
                    i_cur += i_step;
                    g_cur += g_step;
                } else {
                    yl = ny;
                    --xl;
                    i_cur += i_rowjump;
                    g_cur += g_rowjump;
                    if (xl == 0) {
                        xl = nx;
                        i_cur += i_imgjump;
                        g_cur += g_imgjump;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < KCH; ++q) {
            const int slot_px = q >> d1c_shift, part = q - (slot_px << d1c_shift);
            int px = i_soff[0];
#pragma unroll
            for (int k = 1; k < KCH; ++k) px = slot_px == k ? i_soff[k] : px;
            copy_to_lds_dwords<CW>(rs_it, stage + (q * BM + 64 * wave) * 16, a_voff,
                                   px == OOB ? OOB : px + part * CW * 4);
        }
#pragma unroll
        for (int j = 0; j < BPW; ++j) {
            const int blk = wave * BPW + j;
            const int q = blk / (BNL / 64);
            const int slot_px = q >> d1c_shift, part = q - (slot_px << d1c_shift);
            int px = g_soff[0];
#pragma unroll
            for (int k = 1; k < KCH; ++k) px = slot_px == k ? g_soff[k] : px;
            copy_to_lds_dwords<CW>(rs_gt, stage + A_BYTES + blk * 1024, b_voff[j],
                                   px == OOB ? OOB : px + part * CW * 4);
        }
    };

    float16v acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // row tiles of this wave that hold at least one real row (the others would multiply zeros)
    bool row_tile_live[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) row_tile_live[b] = row_tile * BM + 64 * wave + b * 32 < P.rows;

    // NAT: byte offsets of this lane's operands.  MFMA k-pair j takes K index 2j (lower half
    // wave) and 2j+1 (upper half) of the stage's KCH*CW indices (pixel, d1).
    constexpr int NPAIR = KCH * CW / 2;
    int na_base[TM], nb_base[TN], na_k[NPAIR], nb_k[NPAIR];
    if constexpr (NAT) {
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int rl = 64 * wave + 32 * b + lr;  // row within the tile
            const int c_l = rl / P.D2, d2 = rl - c_l * P.D2;
            const bool real = row_tile * BM + rl < P.rows;
            na_base[b] = real ? ((d2 / CW) * BM + c_l * P.D1) * 16 + (d2 % CW) * 4 : 0;
        }
#pragma unroll
        for (int a = 0; a < TN; ++a) {
            const int jl = a * 32 + lr;  // column within the tile
            const int m_l = jl / P.D3, d3 = jl - m_l * P.D3;
            const bool real = col_tile * BN + jl < P.cols;
            nb_base[a] = A_BYTES + (real ? ((d3 / CW) * BNL + m_l * P.D1) * 16 + (d3 % CW) * 4 : 0);
        }
#pragma unroll
        for (int j = 0; j < NPAIR; ++j) {
            const int k = 2 * j + h;
            const int p = k / P.D1, d1 = k - p * P.D1;
            na_k[j] = (p * P.D1C * BM + d1) * 16;
            nb_k[j] = (p * P.D1C * BNL + d1) * 16;
        }
    }

    // A stage's operands are read from LDS in one go, the copies (and the scalar pixel walk) of
    // a later stage are issued while those reads are on their way, then the stage's matrix
    // instructions run: one LDS latency per stage is exposed instead of one per K pair
    // (config 2: 1.05 -> 1.00 ms).
    constexpr int NREAD = NAT ? NPAIR : KCH / 2;
    float kb1[NAT ? NREAD : 1][TN], ia1[NAT ? NREAD : 1][TM];
    float4v kb4[NAT ? 1 : NREAD][TN], ia4[NAT ? 1 : NREAD][TM];
    auto read_stage = [&](int slot) {
        const char* stage = smem + slot * STAGE_BYTES;
        if constexpr (NAT) {
#pragma unroll
            for (int j = 0; j < NPAIR; ++j) {
#pragma unroll
                for (int a = 0; a < TN; ++a)
                    kb1[j][a] = *reinterpret_cast<const float*>(stage + nb_base[a] + nb_k[j]);
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    ia1[j][b] = *reinterpret_cast<const float*>(stage + na_base[b] + na_k[j]);
            }
        } else {
#pragma unroll
            for (int t = 0; t < KCH / 2; ++t) {
                // lanes 0..31 take chunk 2t, lanes 32..63 chunk 2t+1
#pragma unroll
                for (int a = 0; a < TN; ++a)
                    kb4[t][a] = *reinterpret_cast<const float4v*>(
                        stage + A_BYTES + ((2 * t + h) * BNL + a * 32 + lr) * 16);
#pragma unroll
                for (int b = 0; b < TM; ++b)
                    ia4[t][b] = *reinterpret_cast<const float4v*>(
                        stage + ((2 * t + h) * BM + 64 * wave + b * 32 + lr) * 16);
            }
        }
    };
    auto multiply_stage = [&]() {
        if constexpr (NAT) {
#pragma unroll
            for (int j = 0; j < NPAIR; ++j)
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    if (!row_tile_live[b]) continue;  // wave-uniform
#pragma unroll
                    for (int a = 0; a < TN; ++a)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(kb1[j][a], ia1[j][b],
                                                                         acc[a][b], 0, 0, 0);
                }
        } else {
#pragma unroll
            for (int t = 0; t < KCH / 2; ++t)
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    if (!row_tile_live[b]) continue;  // wave-uniform
#pragma unroll
                    for (int u = 0; u < CW; ++u)
#pragma unroll
                        for (int a = 0; a < TN; ++a)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                                kb4[t][a][u], ia4[t][b][u], acc[a][b], 0, 0, 0);
                }
        }
    };

    // ---- prologue: NB-1 stages in flight, the first one landed
    static_for<NB - 1>([&](auto S0) { issue_stage(decltype(S0)::value); });
    __builtin_amdgcn_s_waitcnt(VMCNT_KEEP);
    __syncthreads();

    // ---- main loop: copy stage s+NB-1 into the slot read in iteration s-1, contract stage s
    for (int st = 0; st < nstages_pad; st += NB) {
        static_for<NB>([&](auto SLOT) {
            constexpr int slot = decltype(SLOT)::value;
            read_stage(slot);
            issue_stage((slot + NB - 1) % NB);
            multiply_stage();
            // this wave's copies of the next stage have landed, its reads of this stage are
            // done; after the barrier both hold for every wave
            __builtin_amdgcn_s_waitcnt(VMCNT_KEEP & 0xF0FF);
            __syncthreads();
        });
    }
    // the copies of the surplus stages still write (zeros) into this workgroup's LDS
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // ---- epilogue: lane (h, lr) of tile (a, b) holds in registers 4g..4g+3 the columns
    // 8g + 4h + 0..3 of the tile for row lr of the tile
    float* __restrict__ out = P.out + (long long)split * P.out_elems;
    const long long caps = (long long)P.D0 * P.D2 * P.D3;
    const bool st4 = (P.D3 & 3) == 0;
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const int R = row_tile * BM + 64 * wave + b * 32 + lr;
        if (R >= P.rows) continue;
        const int c = R / P.D2, d2 = R - c * P.D2;
        float* orow = out + ((long long)tap * P.C + c) * P.M * caps +
                      ((long long)d0 * P.D2 + d2) * P.D3;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j0 = col_tile * BN + a * 32 + 8 * g + 4 * h;
                if (st4) {
                    if (j0 < P.cols) {
                        const int m = j0 / P.D3, d3 = j0 - m * P.D3;
                        float4v v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                                     acc[a][b][4 * g + 3]};
                        *reinterpret_cast<float4v*>(orow + (long long)m * caps + d3) = v;
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + u;
                        if (j < P.cols) {
                            // j / D3 by multiplication (exact while j * D3 < 2^32, which the host has checked)
                            const int m = P.d3_magic ? (int)__umulhi((unsigned)j, P.d3_magic) : j / P.D3;
                            const int d3 = j - m * P.D3;
                            orow[(long long)m * caps + d3] = acc[a][b][4 * g + u];
                        }
                    }
                }
            }
        }
    }
}

struct Wgrad32Plan {
    Wgrad32Params P;
    int cw, tn, nw;
    size_t it_bytes, gt_bytes, partial_bytes;
};

int ceil_div_i(long long a, long long b) { return (int)((a + b - 1) / b); }
size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// Valid floats per chunk: 4 or 3, such that a capsule column of D1 floats is 1, 2 or 4 chunks.
int chunk_width(const ConvShape& s)
{
    for (int cw : {4, 3}) {
        if (s.D1 % cw) continue;
        const int d1c = s.D1 / cw;
        if (d1c == 1 || d1c == 2 || d1c == 4) return cw;
    }
    return 0;
}

// Fewest ranges such that the images one range touches (N/nsplit + 3) stay below 2^31 bytes;
// 0 if a single image is already too large for that.
long long split_lower_bound(const ConvShape& s)
{
    const long long it_img = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * 4;
    const long long gt_img = (long long)s.Ho * s.Wo * s.M * s.D0 * s.D1 * s.D3 * 4;
    const long long img_max = it_img > gt_img ? it_img : gt_img;
    const long long imgs_cap = ((1LL << 31) - 1) / (img_max > 0 ? img_max : 1);
    if (imgs_cap < 4) return 0;
    return (s.N + (imgs_cap - 3) - 1) / (imgs_cap - 3);
}

// Tiles and the split of the K loop (host side, pure arithmetic).
Wgrad32Plan make_plan(const ConvShape& s)
{
    Wgrad32Plan pl{};
    Wgrad32Params& P = pl.P;
    pl.cw = chunk_width(s);
    P.N = s.N; P.H = s.H; P.W = s.W; P.C = s.C; P.M = s.M; P.kw = s.kw; P.stride = s.stride;
    P.pad = s.pad; P.D0 = s.D0; P.D1 = s.D1; P.D2 = s.D2; P.D3 = s.D3; P.Ho = s.Ho; P.Wo = s.Wo;
    P.D1C = pl.cw ? s.D1 / pl.cw : 1;
    P.rows = s.C * s.D2;
    P.cols = s.M * s.D3;
    pl.tn = P.cols <= 32 ? 1 : P.cols <= 64 ? 2 : P.cols <= 96 ? 3 : 4;
    pl.nw = P.rows <= 128 ? 2 : 4;
    P.row_tiles = ceil_div_i(P.rows, 64 * pl.nw);
    P.col_tiles = ceil_div_i(P.cols, 32 * pl.tn);
    P.ntaps = s.kh * s.kw;
    P.tiles = P.ntaps * s.D0 * P.row_tiles * P.col_tiles;
    P.out_elems = (long long)s.kernel_elems();
    P.d3_magic = s.D3 > 1 && (long long)s.M * s.D3 * s.D3 < (1LL << 32)
                     ? (unsigned)(((1ULL << 32) + s.D3 - 1) / s.D3)
                     : 0u;  // 0: divide
    P.it_img_bytes = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * 4;
    P.gt_img_bytes = (long long)s.Ho * s.Wo * s.M * s.D0 * s.D1 * s.D3 * 4;
    // square capsules whose tiles begin at whole channels need no transposed copies
    P.natural = s.D1 == s.D2 && s.D1 == s.D3 &&
                (P.row_tiles == 1 || (64 * pl.nw) % s.D2 == 0) &&
                (P.col_tiles == 1 || (32 * pl.tn) % s.D3 == 0);
    pl.it_bytes = P.natural ? 0 : (size_t)s.N * P.it_img_bytes;
    pl.gt_bytes = P.natural ? 0 : (size_t)s.N * P.gt_img_bytes;

    // Split of the K loop (a tap's valid output pixels, at most N*Ho*Wo) over workgroups.  The
    // workgroups resident at a time are bounded by LDS and registers; the split aims at one
    // full round of them and keeps at least 16 stages per workgroup.  A range of N*rect/nsplit
    // pixels touches at most N/nsplit + 3 images: their bytes must stay below 2^31 (a lower
    // bound on nsplit), and the partial sums below 1 GiB (an upper bound).
    const int kch = stage_chunks(P.D1C, pl.nw);
    const size_t lds = (size_t)ring_depth(kch, pl.tn) * kch * (64 * pl.nw + (32 * pl.tn + 63) / 64 * 64) * 16;
    long long per_cu = (long long)(160 * 1024 / lds);
    const int wps = waves_per_simd(pl.tn, kch);  // by registers
    if (per_cu > 4 * wps / pl.nw) per_cu = 4 * wps / pl.nw;
    if (per_cu < 1) per_cu = 1;
    const long long slots = 256 * per_cu;
    const long long full = (long long)s.N * s.Ho * s.Wo;
    long long want = slots / P.tiles;
    if (want < 1) want = 1;
    const long long min_pix = 16LL * (kch / P.D1C);
    if (want > (full + min_pix - 1) / min_pix) want = (full + min_pix - 1) / min_pix;
    if (want > 3072) want = 3072;
    while (want > 1 && (double)want * P.out_elems * 4 > (double)(1 << 30)) --want;
    const long long lo = split_lower_bound(s);
    if (want < lo) want = lo;
    P.nsplit = (int)want;
    P.items = (long long)P.nsplit * P.tiles;
    pl.partial_bytes = P.nsplit > 1 ? (size_t)P.nsplit * P.out_elems * sizeof(float) : 0;
    return pl;
}

hipError_t launch_transpose32(const void* src, void* dst, size_t nmat, int A, int B,
                              hipStream_t stream)
{
    const size_t total = nmat * (size_t)A * B;
    const size_t blocks = (total + 255) / 256;
    if (blocks == 0 || blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    transpose_caps32_kernel<<<(unsigned)blocks, 256, 0, stream>>>(
        static_cast<const float*>(src), static_cast<float*>(dst), A, B, total);
    return hipGetLastError();
}

template <int CW, int TN, int NW, int KCH, bool NAT>
hipError_t launch_nat(const Wgrad32Params& P, hipStream_t stream)
{
    constexpr int BM = 64 * NW, BNL = (32 * TN + 63) / 64 * 64;
    auto kern = wgrad32_kernel<CW, TN, NW, KCH, NAT>;
    const size_t lds_bytes = (size_t)ring_depth(KCH, TN) * KCH * (BM + BNL) * 16;
    static std::atomic<unsigned long long> lds_set{0};
    hipError_t err = set_dynamic_lds_once(reinterpret_cast<const void*>(kern), (int)lds_bytes, lds_set);
    if (err != hipSuccess) return err;
    kern<<<dim3((unsigned)P.items), dim3(64 * NW), lds_bytes, stream>>>(P);
    return hipGetLastError();
}

template <int CW, int TN, int NW, int KCH>
hipError_t launch_kch(const Wgrad32Params& P, hipStream_t stream)
{
    return P.natural ? launch_nat<CW, TN, NW, KCH, true>(P, stream)
                     : launch_nat<CW, TN, NW, KCH, false>(P, stream);
}

template <int CW, int TN, int NW>
hipError_t launch_one(const Wgrad32Params& P, hipStream_t stream)
{
    if constexpr (NW == 4)
        return launch_kch<CW, TN, NW, 4>(P, stream);
    else
        return P.D1C == 4 ? launch_kch<CW, TN, NW, 4>(P, stream)
                          : launch_kch<CW, TN, NW, 2>(P, stream);
}

template <int CW, int NW>
hipError_t launch_tn(const Wgrad32Params& P, int tn, hipStream_t stream)
{
    switch (tn) {
        case 1: return launch_one<CW, 1, NW>(P, stream);
        case 2: return launch_one<CW, 2, NW>(P, stream);
        case 3: return launch_one<CW, 3, NW>(P, stream);
        default: return launch_one<CW, 4, NW>(P, stream);
    }
}

}  // namespace

bool wgrad32_eligible(const ConvShape& s)
{
    if (s.dtype != 0) return false;
    if (chunk_width(s) == 0) return false;
    // 31-bit byte offsets within one image of either tensor, 31-bit counts
    const long long it_img = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * 4;
    const long long gt_img = (long long)s.Ho * s.Wo * s.M * s.D0 * s.D1 * s.D3 * 4;
    if (it_img >= (1LL << 31) || gt_img >= (1LL << 31)) return false;
    if ((long long)s.stride * s.W * s.C * s.D0 * s.D1 * s.D2 * 4 >= (1LL << 30)) return false;
    if ((long long)s.C * s.D2 >= (1 << 24) || (long long)s.M * s.D3 >= (1 << 24)) return false;
    const long long tiles = (long long)s.kh * s.kw * s.D0 * (((long long)s.C * s.D2 + 127) / 128) *
                            (((long long)s.M * s.D3 + 31) / 32);
    const long long lo = split_lower_bound(s);
    if (lo == 0 || lo > 3072) return false;
    if ((double)lo * (double)s.kernel_elems() * 4 > (double)(1 << 30) && lo > 1) return false;
    if (tiles * 3072 >= (1LL << 31)) return false;  // the split never exceeds 3072 ranges
    if ((long long)s.N * s.Ho * s.Wo >= (1LL << 31)) return false;  // pixel counts are 32-bit
    return true;
}

size_t wgrad32_workspace_bytes(const ConvShape& s)
{
    const Wgrad32Plan pl = make_plan(s);
    return align256(pl.it_bytes) + align256(pl.gt_bytes) + pl.partial_bytes;
}

hipError_t launch_wgrad32(const ConvShape& s, const void* input, const void* dout, float* dkernel,
                          void* workspace, hipStream_t stream)
{
    Wgrad32Plan pl = make_plan(s);
    char* ws = static_cast<char*>(workspace);
    void* it = ws;
    void* gt = ws + align256(pl.it_bytes);
    float* partial = reinterpret_cast<float*>(ws + align256(pl.it_bytes) + align256(pl.gt_bytes));
    hipError_t err = hipSuccess;
    if (pl.P.natural) {
        pl.P.it = input;
        pl.P.gt = dout;
    } else {
        err = launch_transpose32(input, it, (size_t)s.N * s.H * s.W * s.C * s.D0, s.D1, s.D2, stream);
        if (err != hipSuccess) return err;
        err = launch_transpose32(dout, gt, (size_t)s.N * s.Ho * s.Wo * s.M * s.D0, s.D1, s.D3, stream);
        if (err != hipSuccess) return err;
        pl.P.it = it;
        pl.P.gt = gt;
    }
    pl.P.out = pl.P.nsplit > 1 ? partial : dkernel;
    if (pl.cw == 3)
        err = pl.nw == 4 ? launch_tn<3, 4>(pl.P, pl.tn, stream) : launch_tn<3, 2>(pl.P, pl.tn, stream);
    else
        err = pl.nw == 4 ? launch_tn<4, 4>(pl.P, pl.tn, stream) : launch_tn<4, 2>(pl.P, pl.tn, stream);
    if (err != hipSuccess) return err;
    if (pl.P.nsplit > 1)
        err = launch_splitk_reduce(partial, dkernel, pl.P.out_elems, pl.P.nsplit, stream);
    return err;
}

}  // namespace capscaps
