// Kernel gradient of the capsule convolution (the K_diff result of the paper's Algorithm 4,
// taken as the derivative of Algorithm 2's sum) on the matrix cores, for 16-bit element types
// and D1 in {8, 16}, and for capsules of 1, 2 and 4 rows (see the end of this comment).  With G = dL/dO, per window tap (p,q) and leading capsule index d0 it is
// one GEMM
//
//     rows     r = (c, d2)                                           C*D2 of them
//     columns  j = (m, d3)                                           M*D3 of them
//     K index  k = (n, x, y, d1)   over the output pixels whose tap (p,q) lies inside the image
//
//     dK[p,q,c,m,d0,d2,d3] = sum_k I[n, x*s+p-pad, y*s+q-pad, c, d0, d1, d2] * G[n, x, y, m, d0, d1, d3]
//
// In both tensors the contracted index d1 is the slower one of a capsule, so a pre-pass writes
// capsule-transposed copies It[n][h][w][c][d0][d2][d1] and Gt[n][x][y][m][d0][d3][d1]: the D1
// values a matrix instruction wants side by side are then 16 or 32 contiguous bytes, and for
// one pixel the 256 rows (or columns) of a tile are one contiguous run (D0 = 1) of It (Gt).
//
// A workgroup owns one 256 x 256 tile of one tap (of two or four taps where the rows fill at
// most half or a quarter of it: see NT at the kernel) and a range of the tap's pixel sequence
// (the valid output pixels, a rectangle per image, image after image; the sequence is cut into
// equal ranges when the tiles alone do not fill the chip; partial sums go to scratch and are
// added in a fixed order by a second kernel).  It walks only those pixels, so no multiplication
// by padding zeros is done and any stride costs the same.  A K stage is 32 contracted values = 32/D1 pixels; per stage each wave copies 64 rows
// and 64 columns (4 x 1 KB each) straight into LDS with buffer loads whose scalar offset is
// the pixel.  The K loop has the shape of the tuned forward kernel's: a ring of 4 LDS stages,
// operand fragments double-buffered in registers, one barrier per stage, copies and the scalar
// pixel walk dealt out between the MFMAs.
//
// LDS stage: [side: It rows, Gt columns][chunk 0..3][row 0..255][16 bytes]; chunk kc holds d1
// values (kc % (D1/8))*8 .. +7 of pixel kc / (D1/8) of the stage.  Operand reads are 512
// contiguous bytes per 32 lanes.
//
// When D2 and D3 are multiples of 8 there is no pre-pass (template flag OWN): the two tensors
// are copied to LDS as they lie in memory, a 16-byte chunk being 8 consecutive rows (c, d2) of
// one (pixel, d1) line, and the matrix instruction's operands are gathered by the transposing
// LDS read ds_read_b64_tr_b16: of a 16-lane group, lane 4a + b supplies the address of 4 rows
// (b) of one line (a), and lane i receives row i's values from the four lines.  A stage then
// holds 32 lines of 256 rows.  One copy instruction brings a unit of 8 lines x 64 rows (for
// 8-row capsules: 8 whole capsules of 128 contiguous bytes; for 16-row ones: 4 half capsules of
// 256 contiguous bytes), consecutive lanes taking consecutive memory; LDS per side is
// [line / 8][row / 64][the unit's 64 chunks in lane order].  Within a unit the line index of
// every other pair of chunk columns is XORed with 4, which makes the 16 chunks a half-wave
// reads (4 lines x 32 rows) fall into 16 different 16-byte columns of the 64 banks.  Which
// (pixel, d1) pair sits in which of an instruction's 16 contraction slots is the same on both
// sides, which is all the contraction needs.
//
// 4x4 capsules (D1 = D2 = D3 = 4, even channel counts) take the same path on channel-paired copies
// of both tensors, [pixel][c/2][d0][d1][c%2][4 halves] (a pre-pass at HBM speed): 8 consecutive
// rows (c, d2) of a line are then one 16-byte chunk as above.  A pixel has only 4 lines, so a
// stage is 8 pixels and a copy's 8 lines are two pixels: the second pixel's offset travels in
// the lane offset of its lanes.  Capsules of 4, 2 or 1 rows whose widths are multiples of 8 are
// read in place; with 2 or 1 rows a stage is 16 or 32 pixels, which the lanes follow one each
// (see VW in the kernel).
#include <hip/hip_runtime.h>

#include "igemm_common.h"
#include "lds_dma.h"

namespace capscaps {
namespace {

struct WgradParams {
    const void* it;  // capsule-transposed input
    const void* gt;  // capsule-transposed output gradient
    float* out;      // dK, or partial sums [split][kernel elements]
    int N, H, W, C, M, kw, stride, pad, D0, D2, D3, Ho, Wo;
    int rows, cols;  // C*D2, M*D3
    int row_tiles, col_tiles, ntaps;
    int tiles;       // ntap_items * D0 * row_tiles * col_tiles
    int nt;          // window taps per tile: 1, or with at most 128 / 64 rows 2 / 4 (see NT in the kernel)
    int ntap_items;  // ceil(ntaps / nt)
    int nsplit;      // ranges a tap's pixel sequence is cut into
    long long items;      // tiles * nsplit = workgroups
    long long out_elems;  // elements of dK
    long long it_img_bytes, gt_img_bytes;
};

// dst[x][b][a] = src[x][a][b] for `nmat` matrices of A x B 16-bit elements, A % 8 == 0 (so a
// matrix is a whole number of 16-byte chunks).  A workgroup moves `mpb` whole matrices through
// LDS: 16-byte loads and stores, both contiguous across the lanes; the transposition is the
// 2-byte gather from LDS in between.  cpm = chunks per matrix = (A/8)*B <= 256.
__global__ __launch_bounds__(256) void transpose_caps_kernel(const chunk_t* __restrict__ src,
                                                             chunk_t* __restrict__ dst, int A,
                                                             int B, int cpm, int mpb,
                                                             size_t chunks)
{
    __shared__ chunk_t tile[256];
    const size_t base = (size_t)blockIdx.x * mpb * cpm;
    const int t = threadIdx.x;
    const bool mine = t < mpb * cpm && base + t < chunks;
    if (mine) tile[t] = src[base + t];
    __syncthreads();
    if (!mine) return;
    const int a8n = A / 8;
    const int a8 = t % a8n;
    const int rest = t / a8n;
    const int b = rest % B, mat = rest / B;
    const unsigned short* m = reinterpret_cast<const unsigned short*>(tile) + mat * A * B;
    unsigned short v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = m[(a8 * 8 + e) * B + b];
    chunk_t out;
    __builtin_memcpy(&out, v, 16);
    dst[base + t] = out;
}

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v lds_short4v;

// NT > 1: layers with at most 128 (64) rows (c, d2) would leave half (three quarters) of the
// 256-row tile empty; their tiles hold NT = 2 (4) consecutive window taps instead, tap NT*i + k in
// rows k*256/NT onwards.  All multiply the same output-gradient pixels, so the column side is
// shared; the row side of tap k is the input k taps further on, a constant byte distance that
// travels in the lane offsets of the waves that copy that tap's rows (a wave copies 64 rows: one
// tap's).  The pixels walked are the bounding rectangle of the taps' rectangles; where a wave's
// own tap reads outside the image its row-side copies are zero fill (decided per pixel from the
// walker's row and column counters).
template <typename Tag, int D1, bool OWN, int NT = 1>
__global__ __launch_bounds__(256) void wgrad16_kernel(const WgradParams P)
{
    constexpr int KCH = 4, NB = 4;
    constexpr int D1C = D1 >= 8 ? D1 / 8 : 1;  // chunks per pixel and row (copies per pixel, D1 >= 8)
    constexpr int PPS = 32 / D1;               // pixels per stage
    static_assert(D1 >= 8 || OWN, "short capsules are read in place (or as channel-paired tensors)");
    // capsules of one or two rows: 32 or 16 pixels per stage are too many for the scalar walk;
    // every lane follows one pixel of the stage instead (vector arithmetic), and a copy, whose 8
    // lines are PPC pixels, fetches its lanes' pixel offsets with a cross-lane read
    constexpr bool VW = D1 <= 2;
    constexpr int PPC = VW ? 8 / D1 : 1;
    constexpr int NWM = 2, NWN = 2;
    constexpr int BM = 256, BN = 256;
    constexpr int SIDE_BYTES = KCH * BM * 16, STAGE_BYTES = 2 * SIDE_BYTES;
    constexpr int WM = BM / NWM, WN = BN / NWN, TM = WM / 32, TN = WN / 32;
    constexpr int NMMA = TM * TN;
    constexpr int NFRAG = TN + TM;
    constexpr int NCOPY = 2 * KCH;  // copies per wave and stage
    constexpr int OOB = (int)0x80000000u;
    constexpr int KEEP = (NB - 2) * NCOPY;
    static_assert(KEEP < 64, "vmcnt is a 6-bit counter");
    constexpr int VMCNT_KEEP = 0x0F70 | (KEEP & 15) | ((KEEP >> 4) << 14);
    static_assert(D1 == 1 || D1 == 2 || D1 == 4 || D1 == 8 || D1 == 16, "D1");
    static_assert(NMMA == 16 && KCH == 4, "the schedule below is written for this shape");
    constexpr bool PAIR = NT > 1;
    constexpr int RT = BM / NT;  // tile rows per tap
    static_assert(NT == 1 || NT == 2 || NT == 4, "taps per tile");
    static_assert(!PAIR || (OWN && !VW && WM == 128), "several taps per tile: in-place reads, scalar walk");

    extern __shared__ char smem[];

    // ---- which item.  Consecutive workgroups go to the 8 XCDs in turn; each XCD is handed a
    // contiguous range of items, ordered pixel range slowest, then tap, then tile, so the
    // workgroups resident on one XCD at a time read the same pixels of It and Gt through its L2.
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
    const int tap = NT * (rest % P.ntap_items);
    const int d0 = rest / P.ntap_items;
    const int tp = tap / P.kw, tq = tap - tp * P.kw;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // (several taps per tile) the tap whose rows this wave copies
    const int k_mine = PAIR ? wave * NT / 4 : 0;
    const int tap_m = tap + k_mine;
    const int tp_m = tap_m / P.kw, tq_m = tap_m - tp_m * P.kw;
    const int wm = wave % NWM, wn = wave / NWM;
    const int h = lane >> 5, lr = lane & 31;

    // ---- the pixels of this item.  Per image the output pixels (x, y) whose tap (tp, tq) reads a
    // real input pixel form a rectangle; the rectangles of all images, image after image, row
    // after row, are one sequence, which is cut into nsplit equal ranges: this item contracts the
    // range [t0, t1), which begins at pixel (xs, ys) of the rectangle of image n0.
    const int s = P.stride;
    int nx, ny, x_lo, y_lo;
    // (several taps per tile) this wave's own tap lies inside the image where the walker's counters satisfy
    // xb <= rows left <= xa and yb <= pixels left in the row <= ya
    int pv_xa = 0, pv_xb = 0, pv_ya = 0, pv_yb = 0;
    if constexpr (!PAIR) {
        const int tx = P.pad - tp, ty = P.pad - tq;  // need x*s >= tx and x*s <= H-1+tx
        x_lo = tx > 0 ? (tx + s - 1) / s : 0;
        y_lo = ty > 0 ? (ty + s - 1) / s : 0;
        const int hx = P.H - 1 + tx, hy = P.W - 1 + ty;
        int x_hi = hx >= 0 ? hx / s : -1, y_hi = hy >= 0 ? hy / s : -1;
        if (x_hi > P.Ho - 1) x_hi = P.Ho - 1;
        if (y_hi > P.Wo - 1) y_hi = P.Wo - 1;
        nx = x_hi - x_lo + 1;
        ny = y_hi - y_lo + 1;
        if (nx <= 0 || ny <= 0) nx = ny = 0;
    } else {
        // rectangle [xl, xh] x [yl, yh] of a tap; empty: xh < xl
        auto tap_rect = [&](int tp_, int tq_, int& xl, int& xh, int& yl, int& yh) {
            const int tx = P.pad - tp_, ty = P.pad - tq_;
            xl = tx > 0 ? (tx + s - 1) / s : 0;
            yl = ty > 0 ? (ty + s - 1) / s : 0;
            const int hx = P.H - 1 + tx, hy = P.W - 1 + ty;
            xh = hx >= 0 ? hx / s : -1;
            yh = hy >= 0 ? hy / s : -1;
            if (xh > P.Ho - 1) xh = P.Ho - 1;
            if (yh > P.Wo - 1) yh = P.Wo - 1;
            if (xh < xl || yh < yl) {
                xl = yl = 0;
                xh = yh = -1;
            }
        };
        // bounding rectangle of the taps that exist and meet the image; this wave's own rectangle
        int x_hi = -1, y_hi = -1, mxl = 0, mxh = -1, myl = 0, myh = -1;
        x_lo = y_lo = 0;
        bool any = false;
#pragma unroll
        for (int k = 0; k < NT; ++k) {
            const int tk = tap + k;
            if (tk >= P.ntaps) break;
            int xl, xh, yl, yh;
            tap_rect(tk / P.kw, tk % P.kw, xl, xh, yl, yh);
            if (k == k_mine) {
                mxl = xl; mxh = xh; myl = yl; myh = yh;
            }
            if (xh < xl) continue;
            if (!any) {
                x_lo = xl; x_hi = xh; y_lo = yl; y_hi = yh;
                any = true;
            } else {
                x_lo = xl < x_lo ? xl : x_lo; x_hi = xh > x_hi ? xh : x_hi;
                y_lo = yl < y_lo ? yl : y_lo; y_hi = yh > y_hi ? yh : y_hi;
            }
        }
        nx = x_hi - x_lo + 1;
        ny = y_hi - y_lo + 1;
        if (nx <= 0 || ny <= 0) nx = ny = 0;
        // pixel (x, y) of the walk has nx - (x - x_lo) rows and ny - (y - y_lo) pixels left
        pv_xa = nx - (mxl - x_lo); pv_xb = nx - (mxh - x_lo);
        pv_ya = ny - (myl - y_lo); pv_yb = ny - (myh - y_lo);
        if (mxh < mxl) pv_xa = -1;  // never
        // all of these are the same in every lane; say so (they feed scalar instructions)
        x_lo = __builtin_amdgcn_readfirstlane(x_lo); y_lo = __builtin_amdgcn_readfirstlane(y_lo);
        nx = __builtin_amdgcn_readfirstlane(nx); ny = __builtin_amdgcn_readfirstlane(ny);
        pv_xa = __builtin_amdgcn_readfirstlane(pv_xa); pv_xb = __builtin_amdgcn_readfirstlane(pv_xb);
        pv_ya = __builtin_amdgcn_readfirstlane(pv_ya); pv_yb = __builtin_amdgcn_readfirstlane(pv_yb);
    }
    const long long rect = (long long)nx * ny, total = rect * P.N;
    const long long tps = (total + P.nsplit - 1) / P.nsplit;
    long long t0 = (long long)split * tps;
    if (t0 > total) t0 = total;
    long long t1 = t0 + tps;
    if (t1 > total) t1 = total;
    const int npix = (int)(t1 - t0);
    const int n0 = npix > 0 ? (int)(t0 / rect) : 0;
    const int n1 = npix > 0 ? (int)((t1 - 1) / rect) + 1 : n0 + 1;
    const int r0 = npix > 0 ? (int)(t0 - (long long)n0 * rect) : 0;  // position in image n0
    const int xs = ny > 0 ? r0 / ny : 0, ys = ny > 0 ? r0 - xs * ny : 0;
    const int ipix = P.C * P.D0 * P.D2 * D1 * 2;  // bytes per pixel of It / Gt
    const int gpix = P.M * P.D0 * P.D3 * D1 * 2;
    const int i_step = s * ipix, g_step = gpix;
    // from the last pixel of a rectangle row to the first of the next row; from there, after
    // the last row, on to the first row of the next image
    const int i_rowjump = (s * P.W - (ny - 1) * s) * ipix, g_rowjump = (P.Wo - (ny - 1)) * gpix;
    const int i_imgjump = (P.H * P.W - nx * s * P.W) * ipix, g_imgjump = (P.Ho * P.Wo - nx * P.Wo) * gpix;
    // one walker over the pixel sequence with a position in either tensor
    // (several taps per tile) the walker follows the first tap's input pixel, which at the border
    // lies up to `pad` rows and pixels before the image, and a later tap's lies up to kw - 1 pixels
    // before that one: the descriptor's base is moved down by both, and the offsets up, so that all stay
    // non-negative.  Only offsets of pixels inside an image are ever dereferenced.
    const int bias_walk = PAIR ? (P.pad * P.W + P.pad) * ipix : 0;
    const int bias_lane = PAIR ? P.kw * ipix : 0;
    int i_cur = (((x_lo + xs) * s - (P.pad - tp)) * P.W + ((y_lo + ys) * s - (P.pad - tq))) * ipix + bias_walk;
    int g_cur = ((x_lo + xs) * P.Wo + y_lo + ys) * gpix;
    int w_left = npix, w_yl = ny - ys, w_xl = nx - xs;

    const unsigned long long it_base = reinterpret_cast<unsigned long long>(P.it) +
                                       (unsigned long long)((long long)n0 * P.it_img_bytes) -
                                       (unsigned long long)(bias_walk + bias_lane);
    const char* gt_base = static_cast<const char*>(P.gt) + (long long)n0 * P.gt_img_bytes;
    const rsrc_t rs_it = make_rsrc(reinterpret_cast<const void*>(it_base),
                                   (unsigned)((n1 - n0) * P.it_img_bytes + bias_walk + bias_lane));
    const rsrc_t rs_gt = make_rsrc(gt_base, (unsigned)((n1 - n0) * P.gt_img_bytes));
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    // this wave copies rows (and columns) wave*64 .. +63 of the tile, all chunks (OWN: copy kc
    // brings lines 8*kc .. +7 of those rows)
    const unsigned lds_a = __builtin_amdgcn_readfirstlane((int)(lds0 + wave * 1024));
    const unsigned lds_b = lds_a + SIDE_BYTES;

    // ---- per-lane constants: byte offset of the lane's row (column) within a pixel, or the
    // out-of-range mark for rows (columns) past the end: those copy zeros
    unsigned a_voff, b_voff;
    int pair_hi_a = 0, pair_hi_b = 0, bp_a = 0, bp_b = 0;
    // OWN: place of chunk (line l8, chunk column r8) in its unit, and back.  `wide`: two chunk
    // columns per capsule row (capsule width a multiple of 16), else one.
    auto unit_slot = [](bool wide, int l8, int r8) {
        const int l = l8 ^ (((r8 >> 1) & 1) * 4);
        return wide ? (r8 >> 1) * 16 + l * 2 + (r8 & 1) : r8 * 8 + l;
    };
    const bool a_wide = P.D2 % 16 == 0, b_wide = P.D3 % 16 == 0;
    if constexpr (OWN) {
        const int ra = a_wide ? (lane >> 4) * 2 + (lane & 1) : lane >> 3;
        const int la = (a_wide ? (lane & 15) >> 1 : lane & 7) ^ (((ra >> 1) & 1) * 4);
        // (several taps per tile: the wave's 64 rows are rows of its own tap.  There the lanes of rows
        // past the last one copy row 0 again instead of carrying the out-of-range mark -- those
        // tile rows are never stored -- so that a lane offset plus a pixel's out-of-range mark
        // can never wrap around to the bytes before the tensor that the moved base covers.)
        const int R_pair = (wave * 64 + ra * 8) % RT;
        const int R = PAIR ? (R_pair < P.rows ? R_pair : 0) : row_tile * BM + (wave * 8 + ra) * 8;
        const int c = R / P.D2, d2 = R - c * P.D2;
        if constexpr (VW) {
            // line la % D1 of pixel la / D1 of the copy
            a_voff = R < P.rows ? (unsigned)(((((c * P.D0 + d0) * D1 + (la % D1)) * P.D2) + d2) * 2) : (unsigned)OOB;
        } else if constexpr (D1 == 4) {
            // line la % 4 of the pixel (la / 4: which of the copy's two pixels); 4x4 capsules:
            // channel-paired tensor, chunk R / 8 of the line is 16 bytes of its own
            if (P.D2 == 4)
                a_voff = R < P.rows ? (unsigned)((((R >> 3) * P.D0 + d0) * D1 + (la & 3)) * 16) : (unsigned)OOB;
            else
                a_voff = R < P.rows ? (unsigned)(((((c * P.D0 + d0) * D1 + (la & 3)) * P.D2) + d2) * 2) : (unsigned)OOB;
        } else
            a_voff = R < P.rows ? (unsigned)(((((c * P.D0 + d0) * D1 + la) * P.D2) + d2) * 2) : (unsigned)OOB;
        if constexpr (PAIR) {
            // this wave's tap's input pixel relative to the first tap's
            const int delta = ((tp_m - tp) * P.W + (tq_m - tq)) * ipix;
            a_voff += (unsigned)(bias_lane + delta);
        }
        const int rb = b_wide ? (lane >> 4) * 2 + (lane & 1) : lane >> 3;
        const int lb = (b_wide ? (lane & 15) >> 1 : lane & 7) ^ (((rb >> 1) & 1) * 4);
        const int J = col_tile * BN + (wave * 8 + rb) * 8;
        const int m = J / P.D3, d3 = J - m * P.D3;
        if constexpr (VW) {
            b_voff = J < P.cols ? (unsigned)(((((m * P.D0 + d0) * D1 + (lb % D1)) * P.D3) + d3) * 2) : (unsigned)OOB;
        } else if constexpr (D1 == 4) {
            if (P.D3 == 4)
                b_voff = J < P.cols ? (unsigned)((((J >> 3) * P.D0 + d0) * D1 + (lb & 3)) * 16) : (unsigned)OOB;
            else
                b_voff = J < P.cols ? (unsigned)(((((m * P.D0 + d0) * D1 + (lb & 3)) * P.D3) + d3) * 2) : (unsigned)OOB;
        } else
            b_voff = J < P.cols ? (unsigned)(((((m * P.D0 + d0) * D1 + lb) * P.D3) + d3) * 2) : (unsigned)OOB;
        // 4-row capsules: a copy's 8 lines are two pixels; all ones in the lanes of the second
        pair_hi_a = -(int)(la >> 2);
        pair_hi_b = -(int)(lb >> 2);
        // (vector walk) byte address, for the cross-lane read, of the lane that follows this
        // lane's pixel of copy 0
        bp_a = (la / D1) * 4;
        bp_b = (lb / D1) * 4;
    } else {
        const int R = row_tile * BM + wave * 64 + lane;
        const int c = R / P.D2, d2 = R - c * P.D2;
        a_voff = R < P.rows ? (unsigned)((((c * P.D0 + d0) * P.D2 + d2) * D1) * 2) : (unsigned)OOB;
        const int J = col_tile * BN + wave * 64 + lane;
        const int m = J / P.D3, d3 = J - m * P.D3;
        b_voff = J < P.cols ? (unsigned)((((m * P.D0 + d0) * P.D3 + d3) * D1) * 2) : (unsigned)OOB;
    }
    // Operand reads.  OWN: lane (h, lr) supplies, for the line group j = 0, 1 of its half h, the
    // address of line (lr % 16) / 4 of that group, rows 16*(lr / 16) + 4*(lr % 4) .. +3 of a
    // 32-row block; the block's place in the stage is added at the read.
    unsigned a_rd[2], b_rd[2];
    if constexpr (OWN) {
        const int g16 = lr >> 4, li = (lr & 15) >> 2, quad = lr & 3;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int l8 = j * 4 + li, r8 = 2 * g16 + (quad >> 1);
            a_rd[j] = (unsigned)(h * 4096 + wm * 2048 + unit_slot(a_wide, l8, r8) * 16 + (quad & 1) * 8);
            b_rd[j] = (unsigned)(SIDE_BYTES + h * 4096 + wn * 2048 + unit_slot(b_wide, l8, r8) * 16 +
                                 (quad & 1) * 8);
        }
    } else {
        a_rd[0] = a_rd[1] = (unsigned)((h * BM + wm * WM + lr) * 16);
        b_rd[0] = b_rd[1] = (unsigned)(SIDE_BYTES + (h * BN + wn * WN + lr) * 16);
    }
    // byte distance of 8 lines (the second half of a 16-row capsule) in either tensor
    const int a_half = OWN ? 16 * P.D2 : 16, b_half = OWN ? 16 * P.D3 : 16;

    float16v acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int nstages = (npix + PPS - 1) / PPS;
    const int nstages_pad = (nstages + NB - 1) / NB * NB;  // surplus stages contract zeros

    // Pixel offsets of the stage whose It copies go out next (a_soff) and of the stage whose
    // Gt copies go out next (g_soff): the same stage, the Gt copies follow one k-step later.
    // All scalar.
    int a_soff[VW ? 1 : PPS], g_soff[VW ? 1 : PPS];
    // One pixel step of the walker, in four branch-free pieces that the main loop puts into
    // different gaps between MFMAs: (0) record the pixel's offsets for slot j of the stage, or
    // past the last pixel the out-of-range mark (zero fill, touches no memory); (1) count down
    // the rectangle row and pick the steps; (2) apply them; (3) at the end of an image jump to
    // the next one.  Written out instruction by instruction: the compiler's code for these
    // selects was two to three times as long, and a volatile statement also stays in the gap
    // it is written in.
    int i_inc = 0, g_inc = 0;
    auto walk = [&](int j, int piece) {
        if (piece == 0) {
            asm volatile("s_cmp_gt_i32 %2, 0\n\t"
                         "s_cselect_b32 %0, %3, 0x80000000\n\t"
                         "s_cselect_b32 %1, %4, 0x80000000\n\t"
                         "s_add_i32 %2, %2, -1"
                         : "=&s"(a_soff[j]), "=&s"(g_soff[j]), "+s"(w_left)
                         : "s"(i_cur), "s"(g_cur)
                         : "scc");
            if constexpr (PAIR) {
                // this wave's tap outside the image at this pixel: zero fill
                asm volatile("s_cmp_gt_i32 %1, %3\n\t"
                             "s_cselect_b32 %0, 0x80000000, %0\n\t"
                             "s_cmp_lt_i32 %1, %4\n\t"
                             "s_cselect_b32 %0, 0x80000000, %0\n\t"
                             "s_cmp_gt_i32 %2, %5\n\t"
                             "s_cselect_b32 %0, 0x80000000, %0\n\t"
                             "s_cmp_lt_i32 %2, %6\n\t"
                             "s_cselect_b32 %0, 0x80000000, %0"
                             : "+s"(a_soff[j])
                             : "s"(w_xl), "s"(w_yl), "s"(pv_xa), "s"(pv_xb), "s"(pv_ya), "s"(pv_yb)
                             : "scc");
            }
        } else if (piece == 1) {
            // next pixel of the rectangle row, or (row done) first pixel of the next row
            asm volatile("s_add_i32 %0, %0, -1\n\t"
                         "s_cmp_eq_u32 %0, 0\n\t"
                         "s_cselect_b32 %2, %5, %4\n\t"
                         "s_cselect_b32 %3, %7, %6\n\t"
                         "s_cselect_b32 %0, %8, %0\n\t"
                         "s_subb_u32 %1, %1, 0"
                         : "+s"(w_yl), "+s"(w_xl), "=&s"(i_inc), "=&s"(g_inc)
                         : "s"(i_step), "s"(i_rowjump), "s"(g_step), "s"(g_rowjump), "s"(ny)
                         : "scc");
        } else if (piece == 2) {
            asm volatile("s_add_i32 %0, %0, %2\n\t"
                         "s_add_i32 %1, %1, %3"
                         : "+s"(i_cur), "+s"(g_cur)
                         : "s"(i_inc), "s"(g_inc)
                         : "scc");
        } else {
            // rectangle done: on to the next image
            int ji, jg;
            asm volatile("s_cmp_eq_u32 %0, 0\n\t"
                         "s_cselect_b32 %3, %5, 0\n\t"
                         "s_cselect_b32 %4, %6, 0\n\t"
                         "s_cselect_b32 %0, %7, %0\n\t"
                         "s_add_i32 %1, %1, %3\n\t"
                         "s_add_i32 %2, %2, %4"
                         : "+s"(w_xl), "+s"(i_cur), "+s"(g_cur), "=&s"(ji), "=&s"(jg)
                         : "s"(i_imgjump), "s"(g_imgjump), "s"(nx)
                         : "scc");
        }
    };
    // ---- vector walk (VW): lane j follows pixel j of the stage whose offsets are being worked out:
    // its place (vx, vy) in the tap's rectangle, its image vn (relative to n0) and how many pixels
    // of the range begin at or after it (v_left <= 0: past the end).  A stage on, every lane moves
    // PPS pixels forward: two divisions of small numbers (by the rectangle's width and height),
    // done as a float multiplication with one correction step (exact for quotients below 2^20).
    int vx = xs, vy = ys, vn = 0, v_left = npix - lane;
    const int ny1 = ny > 0 ? ny : 1, nx1 = nx > 0 ? nx : 1;
    const float inv_ny = 1.0f / (float)ny1, inv_nx = 1.0f / (float)nx1;
    auto small_div = [](int a, int d, float inv) {
        int q = (int)((float)a * inv);
        const int r = a - q * d;
        q += r >= d ? 1 : 0;
        q -= r < 0 ? 1 : 0;
        return q;
    };
    auto vw_step_y = [&](int step) {
        vy += step;
        const int q = small_div(vy, ny1, inv_ny);
        vy -= q * ny1;
        vx += q;
        asm volatile("" : "+v"(vx), "+v"(vy));
    };
    auto vw_step_x = [&]() {
        const int q = small_div(vx, nx1, inv_nx);
        vx -= q * nx1;
        vn += q;
        asm volatile("" : "+v"(vx), "+v"(vn));
    };
    // offsets of the lane's pixel in either tensor, relative to image n0 (or the out-of-range mark)
    const int vi_base = ((x_lo * s - (P.pad - tp)) * P.W + (y_lo * s - (P.pad - tq))) * ipix;
    const int vg_base = (x_lo * P.Wo + y_lo) * gpix;
    const int vi_img = (int)P.it_img_bytes, vg_img = (int)P.gt_img_bytes;
    const int vi_row = s * P.W * ipix, vg_row = P.Wo * gpix;
    auto vw_offset_i = [&]() -> unsigned {
        unsigned o = (unsigned)(vn * vi_img + vx * vi_row + vy * i_step + vi_base);
        o = v_left > 0 ? o : (unsigned)OOB;
        asm volatile("" : "+v"(o));
        return o;
    };
    auto vw_offset_g = [&]() -> unsigned {
        unsigned o = (unsigned)(vn * vg_img + vx * vg_row + vy * g_step + vg_base);
        o = v_left > 0 ? o : (unsigned)OOB;
        asm volatile("" : "+v"(o));
        return o;
    };
    // offsets in use: i_offs for the next It copies, g_offs for the next Gt copies (lane j: pixel j)
    unsigned i_offs = 0, g_offs = 0, i_new = 0, g_new = 0;
    if constexpr (VW) {
        vw_step_y(lane);  // lane j starts j pixels into the range
        vw_step_x();
    }
    // pixel offsets of a copy's lanes, fetched one gap ahead of the copy
    int bp_val_a = 0, bp_val_b = 0;
    auto fetch_a = [&](int kc) {
        bp_val_a = __builtin_amdgcn_ds_bpermute(bp_a + kc * PPC * 4, (int)i_offs);
    };
    auto fetch_b = [&](int kc) {
        bp_val_b = __builtin_amdgcn_ds_bpermute(bp_b + kc * PPC * 4, (int)g_offs);
    };
    auto copy_a = [&](auto SLOT, auto KC) {
        constexpr int slot = decltype(SLOT)::value, kc = decltype(KC)::value;
        if constexpr (VW) {
            copy_to_lds_16B<slot * STAGE_BYTES + kc * BM * 16>(rs_it, lds_a, a_voff + (unsigned)bp_val_a, 0, 0);
        } else if constexpr (D1 == 4) {
            // the pixel's offset travels in the lane offset (an out-of-range mark in either
            // pixel keeps that pixel's lanes out of range)
            const int lo = a_soff[2 * kc], hi = a_soff[2 * kc + 1];
            const unsigned v = a_voff + (unsigned)lo + ((unsigned)(hi - lo) & (unsigned)pair_hi_a);
            copy_to_lds_16B<slot * STAGE_BYTES + kc * BM * 16>(rs_it, lds_a, v, 0, 0);
        } else {
            copy_to_lds_16B<slot * STAGE_BYTES + kc * BM * 16>(rs_it, lds_a, a_voff, a_soff[kc / D1C],
                                                               (kc % D1C) * a_half);
        }
    };
    auto copy_b = [&](auto SLOT, auto KC) {
        constexpr int slot = decltype(SLOT)::value, kc = decltype(KC)::value;
        if constexpr (VW) {
            copy_to_lds_16B<slot * STAGE_BYTES + kc * BN * 16>(rs_gt, lds_b, b_voff + (unsigned)bp_val_b, 0, 0);
        } else if constexpr (D1 == 4) {
            const int lo = g_soff[2 * kc], hi = g_soff[2 * kc + 1];
            const unsigned v = b_voff + (unsigned)lo + ((unsigned)(hi - lo) & (unsigned)pair_hi_b);
            copy_to_lds_16B<slot * STAGE_BYTES + kc * BN * 16>(rs_gt, lds_b, v, 0, 0);
        } else {
            copy_to_lds_16B<slot * STAGE_BYTES + kc * BN * 16>(rs_gt, lds_b, b_voff, g_soff[kc / D1C],
                                                               (kc % D1C) * b_half);
        }
    };
    // operand fragment f of k-step t from ring slot: f < TN column side (Gt), else row side (It)
    auto read_frag = [&](int slot, int t, int f) -> chunk_t {
        const char* stage = smem + slot * STAGE_BYTES;
        if constexpr (OWN) {
            // lines 16t + 8h .. +7 of 32-row block f: two transposing reads of four lines each
            const int ff = f < TN ? f : f - TN;
            const char* p = stage + t * 8192 + (ff / 2) * 1024 + (ff % 2) * 512;
            struct { short4v lo, hi; } v;
            v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v*)(p + (f < TN ? b_rd[0] : a_rd[0])));
            v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v*)(p + (f < TN ? b_rd[1] : a_rd[1])));
            return __builtin_bit_cast(chunk_t, v);
        }
        if (f < TN)
            return *reinterpret_cast<const chunk_t*>(stage + b_rd[0] + (2 * t * BN + f * 32) * 16);
        return *reinterpret_cast<const chunk_t*>(stage + a_rd[0] + (2 * t * BM + (f - TN) * 32) * 16);
    };

    // An MFMA has no side effect the compiler must order, so by itself it may drift away from
    // the gap it is written in; the two empty volatile statements around it (which do keep their
    // order among the copies and scheduling barriers) hold its accumulator, and so the MFMA,
    // in place.
    auto pinned_mma = [&](const chunk_t& ka, const chunk_t& ib, float16v& c) {
        asm volatile("" : "+a"(c));
        Mma<Tag>::run(ka, ib, c);
        asm volatile("" : "+a"(c));
    };

    // ---- prologue: stages 0..NB-2 whole and the It side of stage NB-1
    if constexpr (VW) {
        static_for<NB - 1>([&](auto S0) {
            i_offs = vw_offset_i();
            g_offs = vw_offset_g();
            static_for<KCH>([&](auto KC) {
                fetch_a(decltype(KC)::value);
                copy_a(S0, KC);
            });
            static_for<KCH>([&](auto KC) {
                fetch_b(decltype(KC)::value);
                copy_b(S0, KC);
            });
            vw_step_y(PPS);
            vw_step_x();
            v_left -= PPS;
        });
        i_offs = vw_offset_i();
        g_offs = vw_offset_g();
        static_for<KCH>([&](auto KC) {
            fetch_a(decltype(KC)::value);
            copy_a(std::integral_constant<int, NB - 1>{}, KC);
        });
    } else {
        static_for<NB - 1>([&](auto S0) {
#pragma unroll
            for (int j = 0; j < PPS; ++j)
#pragma unroll
                for (int piece = 0; piece < 4; ++piece) walk(j, piece);
            static_for<KCH>([&](auto KC) { copy_a(S0, KC); });
            static_for<KCH>([&](auto KC) { copy_b(S0, KC); });
        });
#pragma unroll
        for (int j = 0; j < PPS; ++j)
#pragma unroll
            for (int piece = 0; piece < 4; ++piece) walk(j, piece);
        static_for<KCH>([&](auto KC) { copy_a(std::integral_constant<int, NB - 1>{}, KC); });
    }
    {
        constexpr int keep0 = (NB - 2) * NCOPY + KCH;
        static_assert(keep0 < 64, "vmcnt is a 6-bit counter");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (keep0 & 15) | ((keep0 >> 4) << 14));
    }
    __syncthreads();
    chunk_t frag[2][NFRAG];
#pragma unroll
    for (int f = 0; f < NFRAG; ++f) frag[0][f] = read_frag(0, 0, f);

    // ---- main loop, unrolled over the ring so that slots are compile-time constants.
    // Iteration st: k-step 0 issues the Gt copies of stage st+NB-1 (one after every fourth
    // MFMA); after the barrier, k-step 1 issues the It copies of stage st+NB into the slot just
    // released.  The walk over the pixels of stage st+NB runs through both k-steps: pixel j's
    // first piece after the last Gt copy that still reads the previous
    // stage's offset of slot j (k-step 0) and before the first It copy that reads the new one
    // (k-step 1).  Gaps 0..15 are k-step 0's, 16..31 k-step 1's.
    constexpr int NPIECE = VW ? 0 : 4 * PPS;
    constexpr auto piece_gap = [](int q) {
        // four pixels per stage: the second halves of both k-steps, whose gaps hold no operand
        // reads (config 3: 2.7 % faster than pieces in the read gaps); two pixels: measured the
        // other way round (config 5: 2 % slower in the second halves)
        constexpr int four[16] = {8, 9, 10, 11, 12, 13, 14, 15, 24, 25, 26, 27, 28, 29, 30, 31};
        constexpr int two[8] = {7, 8, 9, 11, 15, 16, 17, 19};
        // eight pixels: 32 pieces spread over gaps 3 .. 29; pixel j's first piece falls after the
        // Gt copy of chunk j / 2 (gap 4 (j / 2) + 2) and before the It copy of that chunk (gap
        // 18 + 4 (j / 2))
        return PPS == 8 ? 3 + q * 27 / 32 : PPS == 4 ? four[q] : two[q];
    };
    static_assert(VW || PPS == 8 || PPS == 4 || PPS == 2, "the walk's schedule is written for these stage shapes");
    for (int st = 0; st < nstages_pad; st += NB) {
        static_for<NB>([&](auto SLOT) {
            constexpr int slot = decltype(SLOT)::value;
            constexpr int slot_next = (slot + 1) % NB;
            typedef std::integral_constant<int, (slot + NB - 1) % NB> SlotPrev;
            static_for<NMMA>([&](auto I) {
                constexpr int i = decltype(I)::value;
                pinned_mma(frag[0][i / TM], frag[0][TN + i % TM], acc[i / TM][i % TM]);
                if constexpr (i < NFRAG) frag[1][i] = read_frag(slot, 1, i);
                if constexpr (VW) {
                    // the Gt copies' pixel offsets are fetched two gaps ahead; the lanes move on
                    // to the next stage's pixels, whose offsets take effect after the last Gt copy
                    if constexpr (i % 4 == 0) fetch_b(i / 4);
                    if constexpr (i == 1) vw_step_y(PPS);
                    if constexpr (i == 3) {
                        vw_step_x();
                        v_left -= PPS;
                    }
                    if constexpr (i == 5) i_new = vw_offset_i();
                    if constexpr (i == 7) g_new = vw_offset_g();
                    if constexpr (i == NMMA - 1) {
                        i_offs = i_new;
                        g_offs = g_new;
                        asm volatile("" : "+v"(i_offs), "+v"(g_offs));
                    }
                }
                if constexpr (i % 4 == 2) copy_b(SlotPrev{}, std::integral_constant<int, i / 4>{});
                static_for<NPIECE>([&](auto Q) {
                    constexpr int q = decltype(Q)::value;
                    if constexpr (piece_gap(q) == i) walk(q / 4, q % 4);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
            __builtin_amdgcn_s_waitcnt(VMCNT_KEEP & 0xF0FF);  // and lgkmcnt(0)
            __syncthreads();
            static_for<NMMA>([&](auto I) {
                constexpr int i = decltype(I)::value;
                pinned_mma(frag[1][i / TM], frag[1][TN + i % TM], acc[i / TM][i % TM]);
                if constexpr (i < NFRAG) frag[0][i] = read_frag(slot_next, 0, i);
                if constexpr (VW && i % 4 == 0) fetch_a(i / 4);
                if constexpr (i % 4 == 2) copy_a(SLOT, std::integral_constant<int, i / 4>{});
                static_for<NPIECE>([&](auto Q) {
                    constexpr int q = decltype(Q)::value;
                    if constexpr (piece_gap(q) == NMMA + i) walk(q / 4, q % 4);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    }
    // the copies of the surplus stages still write (zeros) into this workgroup's LDS
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // ---- epilogue: lane (h, lr) of MFMA tile (a, b) holds in registers 4g..4g+3 the columns
    // 8g + 4h + 0..3 of that tile for its row lr
    float* __restrict__ out = P.out + (long long)split * P.out_elems;
    const long long caps = (long long)P.D0 * P.D2 * P.D3;
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        // (several taps per tile: tile row Rt is row Rt % RT of tap Rt / RT)
        const int Rt = wm * WM + b * 32 + lr;
        const int R = PAIR ? Rt % RT : row_tile * BM + Rt;
        const int tap_out = PAIR ? tap + Rt / RT : tap;
        if (R >= P.rows || tap_out >= P.ntaps) continue;
        const int c = R / P.D2, d2 = R - c * P.D2;
        float* orow = out + ((long long)tap_out * P.C + c) * P.M * caps +
                      ((long long)d0 * P.D2 + d2) * P.D3;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j0 = col_tile * BN + wn * WN + a * 32 + 8 * g + 4 * h;
                if (j0 < P.cols) {
                    const int m = j0 / P.D3, d3 = j0 - m * P.D3;
                    float4v v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                                 acc[a][b][4 * g + 3]};
                    *reinterpret_cast<float4v*>(orow + (long long)m * caps + d3) = v;
                }
            }
        }
    }
}

struct WgradPlan {
    WgradParams P;
    size_t it_bytes, gt_bytes, partial_bytes;
};

int ceil_div_i(long long a, long long b) { return (int)((a + b - 1) / b); }

// Window taps a tile can hold (NT in the kernel): 4 with at most 64 rows, 2 with at most 128
int taps_per_tile(const ConvShape& s)
{
    const bool paired4 = s.D1 == 4 && s.D2 == 4 && s.D3 == 4 && s.C % 2 == 0 && s.M % 2 == 0;
    const bool in_place = s.D2 % 8 == 0 && s.D3 % 8 == 0;
    if (!((s.D1 == 4 || s.D1 == 8 || s.D1 == 16) && (in_place || paired4))) return 1;
    const long long rows = (long long)s.C * s.D2, ntaps = (long long)s.kh * s.kw;
    if (rows <= 64 && ntaps >= 3) return 4;
    if (rows <= 128 && ntaps >= 2) return 2;
    return 1;
}

// Tiles and the split over images (host side, pure arithmetic).
WgradPlan make_plan(const ConvShape& s)
{
    WgradPlan pl{};
    WgradParams& P = pl.P;
    P.N = s.N; P.H = s.H; P.W = s.W; P.C = s.C; P.M = s.M; P.kw = s.kw; P.stride = s.stride;
    P.pad = s.pad; P.D0 = s.D0; P.D2 = s.D2; P.D3 = s.D3; P.Ho = s.Ho; P.Wo = s.Wo;
    P.rows = s.C * s.D2;
    P.cols = s.M * s.D3;
    P.row_tiles = ceil_div_i(P.rows, 256);
    P.col_tiles = ceil_div_i(P.cols, 256);
    P.ntaps = s.kh * s.kw;
    P.out_elems = (long long)s.kernel_elems();
    P.it_img_bytes = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * 2;
    P.gt_img_bytes = (long long)s.Ho * s.Wo * s.M * s.D0 * s.D1 * s.D3 * 2;
    pl.it_bytes = (size_t)s.N * P.it_img_bytes;
    pl.gt_bytes = (size_t)s.N * P.gt_img_bytes;
    // Two or four window taps per tile where the rows fill at most half or a quarter of it (tensors read in place or
    // as channel-paired copies, capsules of 4, 8 or 16 rows); the byte offsets, moved up by the
    // reach of the padding and of the window's width, must still fit 31 bits for one image.
    const long long pair_bias = ((long long)s.pad * s.W + s.pad + s.kw) * s.C * s.D0 * s.D1 * s.D2 * 2;
    P.nt = P.it_img_bytes + 2 * pair_bias + 3 * (long long)s.W * s.C * s.D0 * s.D1 * s.D2 * 2 <
                   (1LL << 31) - (1 << 20)
               ? taps_per_tile(s)
               : 1;
    P.ntap_items = (P.ntaps + P.nt - 1) / P.nt;
    P.tiles = P.ntap_items * s.D0 * P.row_tiles * P.col_tiles;

    // Ranges per tap: the cost of a choice is (rounds of 256 workgroups) x (pixels per workgroup
    // + the fixed cost of a workgroup, about 15 us, in pixel units).  A range of N*rect/nsplit
    // pixels touches at most N/nsplit + 2 images, whose byte offsets must stay below 2^31 (where
    // two images already exceed that, every range is one image); the partial sums stay below 1 GiB.
    const long long img_max = P.it_img_bytes > P.gt_img_bytes ? P.it_img_bytes : P.gt_img_bytes;
    const long long room =
        (1LL << 31) - 1 -
        (P.nt > 1 ? 2 * pair_bias + 3 * (long long)s.W * s.C * s.D0 * s.D1 * s.D2 * 2 + (1 << 20) : 0);
    const long long imgs_cap = room / (img_max > 0 ? img_max : 1);  // images a range may touch
    const double pix_total = (double)s.N * s.Ho * s.Wo;
    const double fixed = 1120.0 / s.D1;  // D1 = 16: 70 pixels
    int nsplit_min = 1, nsplit_max = s.N;
    if (imgs_cap < 3) {
        nsplit_min = s.N;  // image-aligned ranges
    } else {
        nsplit_min = ceil_div_i(s.N, imgs_cap - 2);
        // at least 16 stages per range
        const long long by_len = (long long)(pix_total / (16.0 * 32 / s.D1));
        nsplit_max = (int)(by_len < 1 ? 1 : by_len > 4096 ? 4096 : by_len);
        if (nsplit_max < nsplit_min) nsplit_max = nsplit_min;
    }
    double best = 0;
    int best_split = nsplit_min;
    for (int nsplit = nsplit_min; nsplit <= nsplit_max; ++nsplit) {
        if (nsplit > nsplit_min && (double)nsplit * P.out_elems * 4 > (double)(1 << 30)) break;
        const long long items = (long long)nsplit * P.tiles;
        const double rounds = (double)((items + 255) / 256);
        const double cost = rounds * (pix_total / nsplit + fixed);
        // (a finer cut must be cheaper by a margin; measured on config 5: 16 ranges, 9 full rounds,
        // 15.14 ms against 15.54 ms for 7 ranges in 3.94 rounds, which this model puts level)
        if (nsplit == nsplit_min || cost < best * 0.995) {
            best = cost;
            best_split = nsplit;
        }
    }
    P.nsplit = best_split;
    P.items = (long long)P.nsplit * P.tiles;
    pl.partial_bytes = P.nsplit > 1 ? (size_t)P.nsplit * P.out_elems * sizeof(float) : 0;
    return pl;
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

hipError_t launch_transpose(const void* src, void* dst, size_t nmat, int A, int B,
                            hipStream_t stream)
{
    const int cpm = (A / 8) * B;  // <= 256: checked by wgrad16_eligible
    const int mpb = 256 / cpm;
    const size_t chunks = nmat * (size_t)cpm;
    const size_t blocks = (nmat + mpb - 1) / mpb;
    if (blocks == 0 || blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    transpose_caps_kernel<<<(unsigned)blocks, 256, 0, stream>>>(
        static_cast<const chunk_t*>(src), static_cast<chunk_t*>(dst), A, B, cpm, mpb, chunks);
    return hipGetLastError();
}

template <typename Tag, int D1, bool OWN, int NT = 1>
hipError_t launch_kernel(const WgradParams& P, hipStream_t stream)
{
    auto kern = wgrad16_kernel<Tag, D1, OWN, NT>;
    const size_t lds_bytes = (size_t)4 * 2 * 4 * 256 * 16;  // ring of 4 stages of 32 KB
    static std::atomic<unsigned long long> lds_set{0};
    hipError_t err = set_dynamic_lds_once(reinterpret_cast<const void*>(kern), (int)lds_bytes, lds_set);
    if (err != hipSuccess) return err;
    kern<<<dim3((unsigned)P.items), dim3(256), lds_bytes, stream>>>(P);
    return hipGetLastError();
}

}  // namespace

bool wgrad16_eligible(const ConvShape& s)
{
    if (s.dtype != 1 && s.dtype != 2) return false;
    // 4x4 capsules with even channel counts run on channel-paired copies of both tensors
    // ... and 4-row capsules whose widths are multiples of 8 are read in place
    const bool paired = s.D1 == 4 && s.D2 == 4 && s.D3 == 4 && s.C % 2 == 0 && s.M % 2 == 0;
    // ... as are capsules of one or two rows (vector capsules)
    const bool four_in_place = (s.D1 == 4 || s.D1 == 2 || s.D1 == 1) && s.D2 % 8 == 0 && s.D3 % 8 == 0;
    if (s.D1 != 8 && s.D1 != 16 && !paired && !four_in_place) return false;
    if (s.D3 % 4 != 0) return false;
    if (!paired && !four_in_place && ((s.D1 / 8) * s.D2 > 256 || (s.D1 / 8) * s.D3 > 256))
        return false;  // the transpose's tile
    // 31-bit byte offsets within one image of either tensor, 31-bit row/column/pixel counts
    const long long it_img = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * 2;
    const long long gt_img = (long long)s.Ho * s.Wo * s.M * s.D0 * s.D1 * s.D3 * 2;
    if (it_img >= (1LL << 31) || gt_img >= (1LL << 31)) return false;
    if ((long long)s.stride * s.W * s.C * s.D0 * s.D1 * s.D2 * 2 >= (1LL << 30)) return false;
    if ((long long)s.C * s.D2 >= (1 << 24) || (long long)s.M * s.D3 >= (1 << 24)) return false;
    const long long tiles = (long long)s.kh * s.kw * s.D0 * (((long long)s.C * s.D2 + 255) / 256) *
                            (((long long)s.M * s.D3 + 255) / 256);
    if (tiles * (s.N > 4096 ? s.N : 4096) >= (1LL << 31)) return false;  // tiles x ranges
    return true;
}

// Both tensors can be read as they lie in memory when 8 consecutive rows (c, d2) and columns
// (m, d3) of a line are one aligned 16-byte chunk.
static bool reads_in_place(const ConvShape& s) { return s.D2 % 8 == 0 && s.D3 % 8 == 0; }

size_t wgrad16_workspace_bytes(const ConvShape& s)
{
    const WgradPlan pl = make_plan(s);
    if (reads_in_place(s)) return pl.partial_bytes;
    // transposed copies, or (4x4 capsules) channel-paired ones, of both tensors
    return align256(pl.it_bytes) + align256(pl.gt_bytes) + pl.partial_bytes;
}

hipError_t launch_wgrad16(const ConvShape& s, const void* input, const void* dout, float* dkernel,
                          void* workspace, hipStream_t stream)
{
    WgradPlan pl = make_plan(s);
    char* ws = static_cast<char*>(workspace);
    const bool own = reads_in_place(s);
    float* partial;
    hipError_t err = hipSuccess;
    if (own) {
        pl.P.it = input;
        pl.P.gt = dout;
        partial = reinterpret_cast<float*>(ws);
    } else if (s.D1 == 4) {
        // 4x4 capsules: [pixel][c/2][d0][d1][c%2][d2], so that 8 consecutive rows (c, d2) of a line
        // are one 16-byte chunk; the kernel then reads them like tensors it takes in place
        void* it = ws;
        void* gt = ws + align256(pl.it_bytes);
        partial = reinterpret_cast<float*>(ws + align256(pl.it_bytes) + align256(pl.gt_bytes));
        err = launch_pair_channels(input, it, (size_t)s.N * s.H * s.W, s.C, s.D0 * s.D1, stream);
        if (err != hipSuccess) return err;
        err = launch_pair_channels(dout, gt, (size_t)s.N * s.Ho * s.Wo, s.M, s.D0 * s.D1, stream);
        if (err != hipSuccess) return err;
        pl.P.it = it;
        pl.P.gt = gt;
    } else {
        void* it = ws;
        void* gt = ws + align256(pl.it_bytes);
        partial = reinterpret_cast<float*>(ws + align256(pl.it_bytes) + align256(pl.gt_bytes));
        err = launch_transpose(input, it, (size_t)s.N * s.H * s.W * s.C * s.D0, s.D1, s.D2, stream);
        if (err != hipSuccess) return err;
        err = launch_transpose(dout, gt, (size_t)s.N * s.Ho * s.Wo * s.M * s.D0, s.D1, s.D3, stream);
        if (err != hipSuccess) return err;
        pl.P.it = it;
        pl.P.gt = gt;
    }
    pl.P.out = pl.P.nsplit > 1 ? partial : dkernel;
    if (pl.P.nt == 4) {  // four window taps per tile
        if (s.D1 == 4)
            err = s.dtype == 2 ? launch_kernel<f16_tag, 4, true, 4>(pl.P, stream)
                               : launch_kernel<bf16_tag, 4, true, 4>(pl.P, stream);
        else if (s.D1 == 8)
            err = s.dtype == 2 ? launch_kernel<f16_tag, 8, true, 4>(pl.P, stream)
                               : launch_kernel<bf16_tag, 8, true, 4>(pl.P, stream);
        else
            err = s.dtype == 2 ? launch_kernel<f16_tag, 16, true, 4>(pl.P, stream)
                               : launch_kernel<bf16_tag, 16, true, 4>(pl.P, stream);
    } else if (pl.P.nt == 2) {  // two window taps per tile
        if (s.D1 == 4)
            err = s.dtype == 2 ? launch_kernel<f16_tag, 4, true, 2>(pl.P, stream)
                               : launch_kernel<bf16_tag, 4, true, 2>(pl.P, stream);
        else if (s.D1 == 8)
            err = s.dtype == 2 ? launch_kernel<f16_tag, 8, true, 2>(pl.P, stream)
                               : launch_kernel<bf16_tag, 8, true, 2>(pl.P, stream);
        else
            err = s.dtype == 2 ? launch_kernel<f16_tag, 16, true, 2>(pl.P, stream)
                               : launch_kernel<bf16_tag, 16, true, 2>(pl.P, stream);
    } else if (s.D1 == 4) {  // in place, or on the channel-paired copies
        err = s.dtype == 2 ? launch_kernel<f16_tag, 4, true>(pl.P, stream)
                           : launch_kernel<bf16_tag, 4, true>(pl.P, stream);
    } else if (s.D1 == 2) {
        err = s.dtype == 2 ? launch_kernel<f16_tag, 2, true>(pl.P, stream)
                           : launch_kernel<bf16_tag, 2, true>(pl.P, stream);
    } else if (s.D1 == 1) {
        err = s.dtype == 2 ? launch_kernel<f16_tag, 1, true>(pl.P, stream)
                           : launch_kernel<bf16_tag, 1, true>(pl.P, stream);
    } else if (s.dtype == 2) {
        if (own)
            err = s.D1 == 16 ? launch_kernel<f16_tag, 16, true>(pl.P, stream)
                             : launch_kernel<f16_tag, 8, true>(pl.P, stream);
        else
            err = s.D1 == 16 ? launch_kernel<f16_tag, 16, false>(pl.P, stream)
                             : launch_kernel<f16_tag, 8, false>(pl.P, stream);
    } else {
        if (own)
            err = s.D1 == 16 ? launch_kernel<bf16_tag, 16, true>(pl.P, stream)
                             : launch_kernel<bf16_tag, 8, true>(pl.P, stream);
        else
            err = s.D1 == 16 ? launch_kernel<bf16_tag, 16, false>(pl.P, stream)
                             : launch_kernel<bf16_tag, 8, false>(pl.P, stream);
    }
    if (err != hipSuccess) return err;
    if (pl.P.nsplit > 1)
        err = launch_splitk_reduce(partial, dkernel, pl.P.out_elems, pl.P.nsplit, stream);
    return err;
}

}  // namespace capscaps
