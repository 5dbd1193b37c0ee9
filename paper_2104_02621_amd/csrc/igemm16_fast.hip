// Tuned matrix-core kernel of the capsule convolution forward pass for 16-bit element types
// and capsule dimensions D1 = D2 in {8, 16}: the shapes where the contraction is dense enough
// to be bound by the MFMA rate.  Same implicit GEMM as igemm_conv.hip (rows (pixel,d1),
// columns (m,d3), K = (tap, c, d2); paper Algorithm 2), but
//
//   * global -> LDS copies are buffer loads that write LDS directly (no VGPR staging, no
//     ds_write): one wave instruction moves 64 chunks of 16 bytes = 1 KB ("block");
//   * all per-block addressing is wave-uniform (SGPR): a block never mixes pixels, so the
//     window tap and the channel offset are scalar adds, and a tap that falls into the padding
//     is an out-of-range buffer offset, which the hardware answers with zeros;
//   * the K loop runs channel group outermost and window tap innermost: the kh*kw shifted
//     windows of one channel group are fetched in consecutive stages, so all but the first
//     touch of an input byte are L2 hits (tap-outermost order re-streams the whole input
//     window from HBM once per tap);
//   * the K loop is one branch-free basic block per stage in which the copies of the stages
//     NB-1 and NB ahead (one after every fourth MFMA) and the LDS operand reads of the next
//     k-step sit between the MFMAs of the current k-step (operand fragments are
//     double-buffered in registers).
//
// Tile: 256 rows x 256 columns, 4 waves of 128 x 128 (4 x 4 MFMA 32x32x16 tiles, 256
// accumulator registers).  A K stage is KCH chunks (KCH*8 elements) per row; LDS holds a ring
// of NB stages.  One barrier per stage: it is placed before the last k-step of the stage, when
// the wave holds that k-step's operands in registers, so the MFMAs of that k-step overlap the
// first operand reads of the next stage.
//
// LDS layout of one stage
//   input side:  4*KCH blocks.  A pixel of the tile contributes, per stage, KCH chunks for
//                each of its D1 rows = KCH*D1/64 blocks, in global memory order
//                [channel][d1][d2-half]; blocks are spaced 1024+APAD bytes and (D2 = 16) the
//                two halves of a row swap places for d1 >= 8, so the 16 lanes of a quarter
//                wave always touch 16 distinct 16-byte bank groups when reading MFMA operands.
//   kernel side: [chunk 0..KCH-1][column 0..255][16 bytes], copied verbatim from the repacked
//                kernel (repacked in the same stage order); operand reads are 512 contiguous
//                bytes per 32 lanes.
#include <hip/hip_runtime.h>

#include "igemm_common.h"
#include "lds_dma.h"

namespace capscaps {
namespace {

// Input-side block geometry.  A block is the 64 chunks one wave-wide copy moves.  Either a
// pixel's stage data fills one or more blocks (PPB = 1, BPP blocks per pixel, each holding CPB
// channels as [channel][d1][d2-half]), or two pixels share a block (PPB = 2, D1 = D2 = 8 with 4
// chunks per stage: [channel 0..3][pixel 0..1][d1 0..7], the lower half wave copies one pixel,
// the upper half the other).
template <int D1, int D2, int KCH, int BM>
struct ALayout {
    static constexpr int D2C = D2 / 8;             // chunks per capsule row
    static constexpr int G = D1 * D2C;             // chunks per (pixel, channel)
    static constexpr int PPB = (KCH * D1 >= 64) ? 1 : 64 / (KCH * D1);  // pixels per block
    static constexpr int BPP = (PPB == 1) ? KCH * D1 / 64 : 1;  // blocks per pixel (PPB = 1)
    static constexpr int CPB = 64 / (G * PPB);     // channels per block
    static constexpr int PIX = BM / D1;            // pixels per tile
    static constexpr int NBLK = BM * KCH / 64;     // input-side blocks per stage
    // padding between blocks so that lanes of a quarter wave that belong to different pixels
    // fall into different bank groups
    static constexpr int APAD = (G == 8 && PPB == 1) ? 128 : 0;
    static constexpr int ABLK = 1024 + APAD;
    static_assert(D1 == 8 || D1 == 16, "D1");
    static_assert(D2 == 8 || D2 == 16, "D2");
    static_assert(KCH == 4 || KCH == 8, "chunks per stage");
    static_assert(PPB == 1 || (PPB == 2 && D2C == 1), "at most two pixels share a block");
    static_assert(PPB * BPP * 64 == PPB * PPB * KCH * D1 || PPB == 1, "block geometry");
    static_assert(CPB * BPP * D2C == KCH, "blocks of a pixel cover the stage's channels");
    // the two 16-byte halves of a 32-byte capsule row trade places for the upper rows
    static __device__ __forceinline__ int swz(int d1)
    {
        return (D2C == 2 && D1 == 16) ? (d1 >> 3) & 1 : 0;
    }
    // lane of a copy -> element offset of its chunk within the pixel's stage data
    // (cs = channel stride in elements), and which of the block's pixels it belongs to
    static __device__ __forceinline__ int lane_elem_offset(int lane, int cs)
    {
        if (PPB == 1) {
            const int csub = lane / G, g = lane % G, d1 = g / D2C, sh = g % D2C;
            return csub * cs + d1 * D2 + ((sh ^ swz(d1)) * 8);
        }
        const int csub = lane / 16, d1 = lane % 8;
        return csub * cs + d1 * D2;
    }
    static __device__ __forceinline__ int lane_pixel(int lane) { return PPB == 1 ? 0 : (lane >> 3) & 1; }
    // byte position, within the stage's input region, of chunk (pixel pl of the tile, stage
    // channel c_l, row d1, row half)
    static __device__ __forceinline__ int chunk_pos(int pl, int c_l, int d1, int half)
    {
        if (PPB == 1)
            return (pl * BPP + c_l / CPB) * ABLK +
                   ((c_l % CPB) * G + d1 * D2C + (half ^ swz(d1))) * 16;
        return (pl / 2) * ABLK + (c_l * 16 + (pl % 2) * 8 + d1) * 16;
    }
};

// KCH: chunks (of 8 K elements) per row and stage; NB: LDS stage buffers in the ring.
// OUT16: the output has the operands' 16-bit type (rounded at the store) instead of fp32.
// BM: rows of the tile, 256 (one workgroup per CU, 128 x 128 per wave) or 128 (64 x 128 per wave,
// half the registers and LDS, so that two workgroups share a CU and one's set-up, epilogue and
// waits run under the other's MFMAs).
template <typename Tag, int D1, int D2, int KCH, int NB, bool OUT16, int BM>
__global__ __launch_bounds__(256, BM == 256 ? 1 : 2) void igemm16_fast_kernel(const IgemmParams P)
{
    constexpr int OUT_KIND = !OUT16 ? 0 : std::is_same<Tag, f16_tag>::value ? 2 : 1;
    typedef ALayout<D1, D2, KCH, BM> AL;
    constexpr int NWM = 2, NWN = 2, NW = 4;
    constexpr int BN = 256;
    constexpr int D2C = AL::D2C, CPB = AL::CPB, BPP = AL::BPP, PPB = AL::PPB, PIX = AL::PIX;
    constexpr int ABLK = AL::ABLK, NBLK = AL::NBLK, NBLK_B = BN * KCH / 64;
    constexpr int A_BYTES = NBLK * ABLK, B_BYTES = NBLK_B * 1024, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int WM = BM / NWM, WN = BN / NWN, TM = WM / 32, TN = WN / 32;
    constexpr int NMMA = TM * TN;    // MFMAs per k-step = slots for side operations
    constexpr int KS = KCH / 2;      // MFMA k-steps (16 K elements) per stage
    constexpr int BWA = NBLK / NW;   // input-side blocks per wave and stage
    constexpr int BWB = NBLK_B / NW; // kernel-side blocks per wave and stage
    constexpr int PPW = BWA * PPB / BPP;  // pixels whose blocks this wave loads
    constexpr int NFRAG = TN + TM;   // operand fragments per k-step
    constexpr int NCOPY = BWA + BWB; // copies per wave and stage
    static_assert(BM == 256 || BM == 128, "tile rows");
    static_assert(BWA % BPP == 0 && PPW >= 1, "a wave loads whole pixels");
    static_assert(NFRAG <= NMMA && PPW <= NMMA / 2, "side operations fit between the MFMAs");
    static_assert(KS % 2 == 0, "register double buffer alternates per k-step");
    // s_waitcnt vmcnt(n), other counters untouched (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
    constexpr int KEEP = (NB - 2) * NCOPY;  // copies that may still be in flight at a barrier
    static_assert(KEEP < 64, "vmcnt is a 6-bit counter");
    constexpr int VMCNT_KEEP = 0x0F70 | (KEEP & 15) | ((KEEP >> 4) << 14);

    extern __shared__ char smem[];

    // ---- tile: column tiles fastest in launch order.  The hardware deals consecutive
    // workgroups to the 8 XCDs in turn, so with 4 (or 2, or 8) column tiles every XCD works on
    // one column tile and on every other row tile: its L2 streams a single column tile of the
    // repacked kernel for all its resident workgroups, and vertically adjacent row tiles, which
    // share input halo rows, meet in the same L2.  Measured on config 5: 2.5x fewer L2 misses
    // than handing each XCD a contiguous range of tiles covering all column tiles.
    // Longest tiles first: the row tiles on an image's first and last rows, whose K loop is
    // shorter (see tap_lo / tap_hi below), are launched after all others, so that they fill the
    // last round of tiles instead of leaving CUs idle at the end (the host's plan says how many
    // such tiles an image has; 0 = launch order is tile order).
    // Work items past tail_first are pieces of the last tiles: tile and piece of its K loop.
    int L = blockIdx.x;
    int tail_piece = -1;
    if (P.tail_split > 0 && L >= P.tail_first) {
        const int k = L - P.tail_first;
        L = P.tail_first + k / P.tail_split;
        tail_piece = k - (k / P.tail_split) * P.tail_split;
    }
    if (L < P.xcd_span) L = (L & 7) * (P.xcd_span >> 3) + (L >> 3);
    const int col_tile = L % P.col_tiles;
    int rest = L / P.col_tiles;
    int row_tile = rest % P.row_tiles;
    const int d0 = rest / P.row_tiles;
    if (P.lpt_timg > 0) {
        const int ab = P.lpt_a + P.lpt_b, mid = P.lpt_timg - ab;
        const int full = (P.row_tiles / P.lpt_timg) * mid;
        if (row_tile < full) {
            const int n = row_tile / mid;
            row_tile = n * P.lpt_timg + P.lpt_a + (row_tile - n * mid);
        } else {
            const int r2 = row_tile - full, n = r2 / ab, u = r2 - n * ab;
            row_tile = n * P.lpt_timg + (u < P.lpt_a ? u : P.lpt_timg - ab + u);
        }
    }

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % NWM, wn = wave / NWM;
    const int h = lane >> 5, lr = lane & 31;
    const int col0 = col_tile * BN;

    // ---- the pixels whose input blocks this wave copies.  Per pixel (all scalar): the byte
    // offset of its window's first input pixel from in_base (meaningful together with an
    // in-range tap), and a bit mask over the window taps: bit t set = tap t reads a real input
    // pixel, clear = it falls into the padding or the output pixel does not exist.  The mask is
    // a wave ballot: lane t evaluates tap t.
    const int hw = P.Ho * P.Wo;
    // pixel indices fit 32 bits (checked by the launcher): 32-bit divisions keep the set-up short
    const int npix = (int)(P.rows / D1);
    const int pg0 = row_tile * PIX;
    const int n_first = pg0 / hw;
    const long long img_elems = (long long)P.H * P.W * P.pixsz;
    const unsigned short* in_base =
        static_cast<const unsigned short*>(P.in) + (long long)n_first * img_elems;
    const int pix_bytes = (int)(P.pixsz * 2);
    const int tap_p = lane / P.kw, tap_q = lane - tap_p * P.kw;  // this lane's tap
    int pix_off[PPW];
    unsigned long long tap_ok[PPW];
#pragma unroll
    for (int j = 0; j < PPW; ++j) {
        const int pg = pg0 + wave * PPW + j;
        const bool exists = pg < npix;
        const int pgc = exists ? pg : pg0;
        const int n_rel = pgc / hw - n_first;
        const int rem = pgc - (pgc / hw) * hw;
        const int x = rem / P.Wo, y = rem - x * P.Wo;
        const int ih0 = x * P.stride - P.pad, iw0 = y * P.stride - P.pad_w;
        const bool ok = exists && lane < P.ntaps && (unsigned)(ih0 + tap_p) < (unsigned)P.H &&
                        (unsigned)(iw0 + tap_q) < (unsigned)P.W;
        tap_ok[j] = __builtin_amdgcn_ballot_w64(ok);
        pix_off[j] = __builtin_amdgcn_readfirstlane(
            (int)((((long long)n_rel * P.H + ih0) * P.W + iw0) * pix_bytes) + d0 * D1 * D2 * 2);
    }
    // Window rows that no pixel of the whole tile can use (the tile lies on the image's first
    // or last rows and the window row falls into the padding) are left out of the K loop: the
    // tile then runs taps [tap_lo, tap_hi) only.  The tap masks of the four waves are combined
    // through LDS (free until the first copy is issued).
    int tap_lo = 0, tap_hi = P.ntaps;
    {
        unsigned long long mine = 0;
#pragma unroll
        for (int j = 0; j < PPW; ++j) mine |= tap_ok[j];
        unsigned long long* share = reinterpret_cast<unsigned long long*>(smem);
        if (lane == 0) share[wave] = mine;
        __syncthreads();
        unsigned long long all = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) all |= share[w];
        const unsigned all_lo = __builtin_amdgcn_readfirstlane((int)(unsigned)all);
        const unsigned all_hi = __builtin_amdgcn_readfirstlane((int)(unsigned)(all >> 32));
        const unsigned long long live = ((unsigned long long)all_hi << 32) | all_lo;
        __syncthreads();  // everyone has read before any copy may land here
        if (live != 0) {
            const unsigned long long row_bits = P.kw >= 64 ? ~0ull : (1ull << P.kw) - 1;
            int p_lo = 0, p_hi = P.ntaps / P.kw;
            while (p_lo < p_hi - 1 && ((live >> (p_lo * P.kw)) & row_bits) == 0) ++p_lo;
            while (p_hi - 1 > p_lo && ((live >> ((p_hi - 1) * P.kw)) & row_bits) == 0) --p_hi;
            tap_lo = p_lo * P.kw;
            tap_hi = p_hi * P.kw;
        }
    }
    long long in_left = P.in_bytes - (long long)n_first * img_elems * 2;
    if (in_left > 0x7fffffffLL) in_left = 0x7fffffffLL;
    const rsrc_t rs_in = make_rsrc(in_base, (unsigned)in_left);
    const rsrc_t rs_kp = make_rsrc(P.kp, (unsigned)P.kp_records);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    // LDS byte addresses of this wave's first input block and first kernel block in slot 0
    const unsigned lds_a = __builtin_amdgcn_readfirstlane((int)(lds0 + wave * BWA * ABLK));
    const unsigned lds_b = __builtin_amdgcn_readfirstlane((int)(lds0 + A_BYTES + wave * BWB * 1024));

    // ---- per-lane constants
    // input block: byte offset of the lane's chunk within its pixel's stage data
    const unsigned a_voff = (unsigned)(AL::lane_elem_offset(lane, P.cs) * 2);
    const int a_hi = -AL::lane_pixel(lane);  // all ones in the lanes that copy a block's 2nd pixel
    const unsigned b_voff = (unsigned)lane * 16u;
    // operand reads: MFMA row tile b covers rows wm*WM + b*32 + lr of the tile; lane half h
    // takes chunk 2t + h of the stage: channel (2t+h)/D2C, row half (2t+h)%D2C
    unsigned a_rd;  // byte offset within the stage's input region, for b = 0, t = 0
    {
        const int r = wm * WM + lr;
        a_rd = (unsigned)AL::chunk_pos(r / D1, h / D2C, r % D1, h % D2C);
    }
    const unsigned b_rd = (unsigned)(A_BYTES + (h * BN + wn * WN + lr) * 16);

    float16v acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // ---- K loop state (scalar).  Stage s covers channel group s / ntaps (KCH chunks =
    // KCH/D2C channels) at window tap s % ntaps.  The input-side state describes the stage
    // whose input copies go out next, the kernel-side state (one offset) the stage whose kernel
    // copies go out next; in the steady state the input side runs one stage ahead.
    const int groups = P.KQP / KCH;
    // channel groups of this work item: all, or one piece of a tile of the last round
    int g_first = 0, g_count = groups;
    if (tail_piece >= 0) {
        const int per = (groups + P.tail_split - 1) / P.tail_split;
        g_first = tail_piece * per;
        g_count = g_first >= groups ? 0 : (groups - g_first < per ? groups - g_first : per);
    }
    const int nlive = tap_hi - tap_lo;                      // taps per channel group that run
    const int nstages = nlive * g_count;
    const int nstages_pad = (nstages + NB - 1) / NB * NB;  // surplus stages contract zeros
    const int c_step = (KCH / D2C) * P.cs * 2;             // bytes per channel group
    const int kp_step = KCH * P.colsp * 16;                 // repacked kernel bytes per stage
    const int kp_wrap = (P.ntaps - nlive + 1) * kp_step;    // last live tap -> first of next group
    const int row_skip = (P.W - P.kw + 1) * pix_bytes;     // last tap of a window row -> next row
    const int tap_off0 = (tap_lo / P.kw) * P.W * pix_bytes;
    int a_stage = 0, tap = tap_lo, tap_q_cur = 0, tap_off = tap_off0, c_off = g_first * c_step;
    constexpr int DEAD_TAP = 63;  // no window has a 64th tap (checked by the launcher)
    int tap_sel = nstages > 0 ? tap_lo : DEAD_TAP;
    int kp_off = (int)(((((long long)d0 * groups + g_first) * P.ntaps + tap_lo) * KCH * P.colsp +
                        col0) * 16);
    int kp_left = nlive;  // kernel-side stages until the next channel group
    // kernel-side state -> next stage
    // (Scalar arithmetic has no side effect the compiler must order, so by itself it may drift
    // out of the gap between MFMAs it is written in; the empty volatile statements, which do
    // keep their order among the copies and scheduling barriers, hold its inputs and results in
    // place.)
    auto advance_b = [&]() {
        asm volatile("" : "+s"(kp_left), "+s"(kp_off));
        --kp_left;
        const bool wrap = kp_left == 0;
        kp_off += wrap ? kp_wrap : kp_step;
        kp_left = wrap ? nlive : kp_left;
        asm volatile("" : "+s"(kp_left), "+s"(kp_off));
    };
    int b_const[BWB];
#pragma unroll
    for (int j = 0; j < BWB; ++j) {
        const int bb = wave * BWB + j;
        b_const[j] = ((bb / 4) * P.colsp + (bb % 4) * 64) * 16;
    }
    int a_soff[PPW];  // per pixel: byte offset of the current tap's input pixel, or OOB

    // All of the following is scalar arithmetic (nothing on the vector pipe that could hold up
    // the MFMAs); the main loop deals it out in small pieces between the MFMAs.
    // offset of the input-side stage's copies for pixel j
    // (three scalar instructions, written out: bit tap_sel of the pixel's tap mask picks the
    // address or the out-of-range mark; tap_sel is the input-side stage's tap, or the always
    // clear bit 63 past the last stage, whose copies then fill zeros and touch no memory)
    auto stage_offset = [&](int j) {
        asm volatile("s_add_i32 %0, %3, %4\n\t"
                     "s_bitcmp1_b64 %1, %2\n\t"
                     "s_cselect_b32 %0, %0, 0x80000000"
                     : "=&s"(a_soff[j])
                     : "s"(tap_ok[j]), "s"(tap_sel), "s"(pix_off[j]), "s"(tap_off)
                     : "scc");
    };
    // input-side state -> next stage, in five pieces (0 .. 4 in this order)
    auto advance_a = [&](int piece) {
        asm volatile("" : "+s"(a_stage), "+s"(tap), "+s"(tap_q_cur), "+s"(tap_off), "+s"(c_off));
        if (piece == 0) {
            ++a_stage;
            ++tap;
            ++tap_q_cur;
        } else if (piece == 1) {
            const bool row_end = tap_q_cur == P.kw;
            tap_q_cur = row_end ? 0 : tap_q_cur;
            tap_off += row_end ? row_skip : pix_bytes;
        } else if (piece == 4) {
            tap_sel = a_stage < nstages ? tap : DEAD_TAP;
        } else if (piece == 2) {
            // window done (tap == tap_hi): next channel group ... (pieces 2 and 3 are written
            // out so that they stay selects: the compiler makes a branch of them in some slots)
            int step;
            asm volatile("s_cmp_eq_u32 %2, %3\n\t"
                         "s_cselect_b32 %1, %4, 0\n\t"
                         "s_add_i32 %0, %0, %1"
                         : "+s"(c_off), "=&s"(step)
                         : "s"(tap), "s"(tap_hi), "s"(c_step)
                         : "scc");
        } else {
            // ... first live tap (piece 3)
            asm volatile("s_cmp_eq_u32 %0, %3\n\t"
                         "s_cselect_b32 %0, %4, %0\n\t"
                         "s_cselect_b32 %1, 0, %1\n\t"
                         "s_cselect_b32 %2, %5, %2"
                         : "+s"(tap), "+s"(tap_q_cur), "+s"(tap_off)
                         : "s"(tap_hi), "s"(tap_lo), "s"(tap_off0)
                         : "scc");
        }
        asm volatile("" : "+s"(a_stage), "+s"(tap), "+s"(tap_q_cur), "+s"(tap_off), "+s"(c_off),
                     "+s"(tap_sel));
    };
    // (two pixels per block) the lane offsets of the next input copy, set by prepare_a in the
    // gap before the copy's own
    unsigned a_voff2 = 0;
    // input copy J (0 .. BWA-1) of the input-side stage / kernel copy J of the kernel-side stage
    auto copy_a = [&](auto SLOT, auto J) {
        constexpr int slot = decltype(SLOT)::value, j = decltype(J)::value;
        if constexpr (PPB == 1) {
            constexpr int pj = j / BPP, part = j % BPP;
            copy_to_lds_16B<slot * STAGE_BYTES + j * ABLK>(rs_in, lds_a, a_voff, a_soff[pj],
                                                           c_off + part * CPB * P.cs * 2);
        } else {
            // two pixels per block: the pixel's offset travels in the lane offset (wrapping
            // arithmetic; an out-of-range mark in either half keeps that half out of range)
            copy_to_lds_16B<slot * STAGE_BYTES + j * ABLK>(rs_in, lds_a, a_voff2, c_off, 0);
        }
    };
    auto prepare_a = [&](int j) {
        asm volatile("" : "+s"(a_soff[2 * j]), "+s"(a_soff[2 * j + 1]));
        const int lo = a_soff[2 * j], hi = a_soff[2 * j + 1];
        a_voff2 = a_voff + (unsigned)lo + ((unsigned)(hi - lo) & (unsigned)a_hi);
        asm volatile("" : "+v"(a_voff2));
    };
    auto copy_b = [&](auto SLOT, auto J) {
        constexpr int slot = decltype(SLOT)::value, j = decltype(J)::value;
        // beyond the repacked kernel (surplus stages) the range check returns zeros
        copy_to_lds_16B<slot * STAGE_BYTES + j * 1024>(rs_kp, lds_b, b_voff, kp_off, b_const[j]);
    };

    // operand fragment f of k-step t from ring slot: f < TN kernel side, else input side
    auto read_frag = [&](int slot, int t, int f) -> chunk_t {
        const char* stage = smem + slot * STAGE_BYTES;
        if (f < TN)
            return *reinterpret_cast<const chunk_t*>(stage + b_rd + (2 * t * BN + f * 32) * 16);
        const int b = f - TN;
        // chunk index +2t = channel +2t/D2C (row half unchanged); rows +32b = pixels +32b/D1.
        // The lane's own (pixel, channel, d1, half) at b = t = 0 adds no carry: positions are
        // affine in the pixel (steps of 32/D1) and channel advance (CPB, blocks per pixel even).
        const int off = AL::chunk_pos(b * 32 / D1, 2 * t / D2C, 0, 0) - AL::chunk_pos(0, 0, 0, 0);
        return *reinterpret_cast<const chunk_t*>(stage + a_rd + off);
    };

    // ---- schedule of the side operations.  A stage is two k-steps of NMMA = 16 MFMAs; per
    // wave it needs 4 input copies and 4 kernel copies: one copy after every fourth MFMA
    // keeps the copy queue shallow.  In the k-step after the barrier of iteration s go the input
    // copies of stage s+NB, into the ring slot that iteration has just finished reading (the
    // last k-step's operands are in registers); in the first k-step of iteration s+1 go that
    // stage's kernel copies, and, dealt out over the other gaps, the scalar arithmetic that
    // moves the input-side state on by one stage.  No gap holds more than a handful of
    // instructions, so the next MFMA is always issued before the matrix pipe runs dry.
    // With the 128-row tile a k-step has 8 MFMAs and a wave 2 input copies; two workgroups share
    // the CU then, so a fuller gap in one wave is covered by the other wave of the SIMD.
    static_assert(KS == 2 && BWB == 4 && (NMMA == 16 || NMMA == 8), "the schedule is written for these shapes");
    // gap (index of the MFMA it follows) of: kernel copy j (k-step 0), input copy j (k-step 1),
    // piece of the input-side advance, tap lookup of pixel j (k-step 0, after the advance)
    constexpr auto copy_b_gap = [](int j) { return NMMA == 16 ? 4 * j + 2 : 2 * j + 1; };
    constexpr auto copy_a_gap = [](int j) { return NMMA == 16 ? 4 * j + 2 : 4 * j + 3; };
    // (the seventh and eighth lookup go into k-step 1 -- NMMA + g: its gap g, before the copy
    // that uses the pixel)
    constexpr auto advance_gap = [](int piece) {
        constexpr int wide[5] = {0, 1, 3, 4, 5}, narrow[5] = {0, 1, 2, 2, 3};
        return NMMA == 16 ? wide[piece] : narrow[piece];
    };
    constexpr auto lookup_gap = [](int j) {
        constexpr int wide[8] = {7, 8, 9, 11, 12, 13, NMMA + 7, NMMA + 8};
        return NMMA == 16 ? wide[j] : 4 + j;
    };
    // with two waves per SIMD the MFMAs are held in their gaps explicitly (a pure instruction
    // may otherwise drift across the scheduling barriers)
    auto mma = [&](const chunk_t& ka, const chunk_t& ib, float16v& c) {
        if constexpr (BM == 128) asm volatile("" : "+a"(c));
        Mma<Tag>::run(ka, ib, c);
        if constexpr (BM == 128) asm volatile("" : "+a"(c));
    };

    // ---- prologue: stages 0..NB-2 whole and the input side of stage NB-1, wait for stage 0,
    // fetch its first fragments
    static_for<NB - 1>([&](auto S0) {
#pragma unroll
        for (int j = 0; j < PPW; ++j) stage_offset(j);
        static_for<BWA>([&](auto J) {
            if constexpr (PPB == 2) prepare_a(decltype(J)::value);
            copy_a(S0, J);
        });
        static_for<BWB>([&](auto J) { copy_b(S0, J); });
        advance_a(0);
        advance_a(1);
        advance_a(2);
        advance_a(3);
        advance_a(4);
        advance_b();
    });
#pragma unroll
    for (int j = 0; j < PPW; ++j) stage_offset(j);
    static_for<BWA>([&](auto J) {
        if constexpr (PPB == 2) prepare_a(decltype(J)::value);
        copy_a(std::integral_constant<int, NB - 1>{}, J);
    });
    // the accumulators are cleared here, while the first copies are on their way (left to
    // itself the compiler clears them after the wait)
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) asm volatile("" : "+a"(acc[a][b]));
    {
        constexpr int keep0 = (NB - 2) * NCOPY + BWA;
        static_assert(keep0 < 64, "vmcnt is a 6-bit counter");
        __builtin_amdgcn_s_waitcnt(0x0F70 | (keep0 & 15) | ((keep0 >> 4) << 14));
    }
    __syncthreads();
    chunk_t frag[2][NFRAG];
#pragma unroll
    for (int f = 0; f < NFRAG; ++f) frag[0][f] = read_frag(0, 0, f);

    // ---- main loop, unrolled over the ring so that slots are compile-time constants
    for (int st = 0; st < nstages_pad; st += NB) {
        static_for<NB>([&](auto SLOT) {
            constexpr int slot = decltype(SLOT)::value;
            constexpr int slot_next = (slot + 1) % NB;
            typedef std::integral_constant<int, (slot + NB - 1) % NB> SlotPrev;
            // k-step 0: kernel copies of the stage NB-1 ahead; input-side state -> stage NB ahead
            static_for<NMMA>([&](auto I) {
                constexpr int i = decltype(I)::value;
                mma(frag[0][i / TM], frag[0][TN + i % TM], acc[i / TM][i % TM]);
                if constexpr (i < NFRAG) frag[1][i] = read_frag(slot, 1, i);
                static_for<BWB>([&](auto J) {
                    if constexpr (copy_b_gap(decltype(J)::value) == i) copy_b(SlotPrev{}, J);
                });
                static_for<5>([&](auto PC) {
                    if constexpr (advance_gap(decltype(PC)::value) == i) advance_a(decltype(PC)::value);
                });
                static_for<PPW>([&](auto J) {
                    if constexpr (lookup_gap(decltype(J)::value) == i) stage_offset(decltype(J)::value);
                });
                if constexpr (i == NMMA - 1) advance_b();
                __builtin_amdgcn_sched_barrier(0);
            });
            // everything this wave still needs from `slot` is in registers; its copies of the
            // next stage have landed; after the barrier that holds for all waves
            __builtin_amdgcn_s_waitcnt(VMCNT_KEEP & 0xF0FF);  // and lgkmcnt(0)
            __syncthreads();
            // k-step 1: input copies of the stage NB ahead into the slot just released
            static_for<NMMA>([&](auto I) {
                constexpr int i = decltype(I)::value;
                mma(frag[1][i / TM], frag[1][TN + i % TM], acc[i / TM][i % TM]);
                if constexpr (i < NFRAG) frag[0][i] = read_frag(slot_next, 0, i);
                static_for<PPW>([&](auto J) {
                    if constexpr (lookup_gap(decltype(J)::value) == NMMA + i)
                        stage_offset(decltype(J)::value);
                });
                static_for<BWA>([&](auto J) {
                    if constexpr (PPB == 2 && copy_a_gap(decltype(J)::value) - 1 == i)
                        prepare_a(decltype(J)::value);
                    if constexpr (copy_a_gap(decltype(J)::value) == i) copy_a(SLOT, J);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    }

    // the copies of the surplus stages still write (zeros) into this workgroup's LDS
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // ---- epilogue: lane (h, lr) of MFMA tile (a, b) holds in registers 4g..4g+3 the columns
    // 8g + 4h + 0..3 of that tile for its output row lr.
    const int caps_out = P.D0 * D1 * P.D3;
    // a piece of a tile writes into its own copy of the output's last pixels
    const long long tail_shift = (long long)P.tail_pix0 * P.M * caps_out;
    float* __restrict__ out =
        tail_piece < 0 ? P.out : P.tail_partial + (long long)tail_piece * P.tail_elems - tail_shift;
    const long long out_alloc = tail_piece < 0 ? P.out_alloc : tail_shift + P.tail_elems;
    const int d3_shift = 31 - __builtin_clz(P.D3);
    // element offset of an output pixel
    auto pixel_offset = [&](int pixel) -> long long {
        if (!P.out_view) return (long long)pixel * P.M * caps_out;
        // the output pixels of this call interleave with other calls'
        const int n = pixel / hw, rem = pixel - n * hw;
        const int x = rem / P.Wo, y = rem - x * P.Wo;
        return P.out_base + n * P.out_sn + x * P.out_sx + y * P.out_sy;
    };
    if (P.fast_store && col0 + BN <= P.cols) {
        // Whole column tile, D3 in {4, 8, 16, 32} (the host's test): the position of a store is
        // (lane part) + (part that depends on a and g only), without carries between the two.
        // So each lane keeps one 32-bit byte offset per row tile b, relative to the tile's first
        // pixel; the (a, g) part is a scalar offset of a buffer store, and rows past the last
        // pixel carry the out-of-range mark, which the range check drops.  No per-store vector
        // arithmetic is left (the general form below costs about 50 instructions per store).
        constexpr int ES = OUT16 ? 2 : 4;
        const long long tile_base = pixel_offset(pg0);
        const int jl = col0 + wn * WN + 4 * h;
        const int lane_col = (jl >> d3_shift) * caps_out + (jl & (P.D3 - 1));
        unsigned voff[TM];
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int r = wm * WM + b * 32 + lr;
            const int pixel = pg0 + r / D1;
            const int d1 = r % D1;
            const long long rel = pixel_offset(pixel < npix ? pixel : pg0) - tile_base +
                                  (d0 * D1 + d1) * P.D3 + lane_col;
            voff[b] = pixel < npix ? (unsigned)(rel * ES) : 0x80000000u;
        }
        long long bytes_left = (out_alloc - tile_base) * ES;
        if (bytes_left > 0x7fffffffLL) bytes_left = 0x7fffffffLL;
        const unsigned long long base_addr =
            reinterpret_cast<unsigned long long>(out) + (unsigned long long)(tile_base * ES);
        const unsigned base_lo = __builtin_amdgcn_readfirstlane((int)(unsigned)base_addr);
        const unsigned base_hi = __builtin_amdgcn_readfirstlane((int)(unsigned)(base_addr >> 32));
        const __amdgpu_buffer_rsrc_t rs_out = __builtin_amdgcn_make_buffer_rsrc(
            reinterpret_cast<void*>(((unsigned long long)base_hi << 32) | base_lo), 0,
            __builtin_amdgcn_readfirstlane((int)bytes_left), 0x00020000);
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int delta = a * 32 + 8 * g;
                const int soff = ((delta >> d3_shift) * caps_out + (delta & (P.D3 - 1))) * ES;
#pragma unroll
                for (int b = 0; b < TM; ++b) {
                    const float4v v = {acc[a][b][4 * g], acc[a][b][4 * g + 1],
                                       acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
                    if constexpr (OUT16) {
                        typedef unsigned int u2 __attribute__((ext_vector_type(2)));
                        const u2 w = {(unsigned)round_to_16(v[0], OUT_KIND) |
                                          ((unsigned)round_to_16(v[1], OUT_KIND) << 16),
                                      (unsigned)round_to_16(v[2], OUT_KIND) |
                                          ((unsigned)round_to_16(v[3], OUT_KIND) << 16)};
                        __builtin_amdgcn_raw_buffer_store_b64(w, rs_out, voff[b], soff, 0);
                    } else {
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(chunk_t, v),
                                                               rs_out, voff[b], soff, 0);
                    }
                }
            }
        }
        return;
    }
    // general form: ragged column tile, other D3.  Columns advance in steps of 8, so (m, d3) of
    // a column is found by shifts when D3 is a power of two, by division otherwise.
    const bool d3_pow2 = (P.D3 & (P.D3 - 1)) == 0;
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const int r = wm * WM + b * 32 + lr;
        const int pixel = pg0 + r / D1;
        if (pixel >= npix) continue;
        const int d1 = r % D1;
        const long long orow_off = pixel_offset(pixel) + (long long)(d0 * D1 + d1) * P.D3;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j0 = col0 + wn * WN + a * 32 + 8 * g + 4 * h;
                if (j0 < P.cols) {
                    const int m = d3_pow2 ? j0 >> d3_shift : j0 / P.D3;
                    const int d3 = j0 - m * P.D3;
                    float4v v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                                 acc[a][b][4 * g + 3]};
                    store4(out, orow_off + (long long)m * caps_out + d3, v, OUT_KIND);
                }
            }
        }
    }
}

template <int D1, int D2>
struct FastConfig;  // chunks per stage and ring depth chosen per capsule size
template <>
struct FastConfig<16, 16> { static constexpr int KCH = 4, NB = 4; };
template <>
struct FastConfig<8, 8> { static constexpr int KCH = 4, NB = 4; };

template <typename Tag, int D1, int D2>
hipError_t launch_one(const IgemmParams& P, long long blocks, hipStream_t stream)
{
    constexpr int KCH = FastConfig<D1, D2>::KCH;
    if (P.bm == 128) {
        // two workgroups per CU: a ring of 3 stages of 24..25.6 KB each
        constexpr int NB = 3;
        typedef ALayout<D1, D2, KCH, 128> AL;
        auto kern = P.out16 ? igemm16_fast_kernel<Tag, D1, D2, KCH, NB, true, 128>
                            : igemm16_fast_kernel<Tag, D1, D2, KCH, NB, false, 128>;
        const size_t lds_bytes = (size_t)NB * (AL::NBLK * AL::ABLK + 256 * KCH * 16);
        static std::atomic<unsigned long long> lds_set[2] = {{0}, {0}};
        hipError_t err = set_dynamic_lds_once(reinterpret_cast<const void*>(kern), (int)lds_bytes,
                                              lds_set[P.out16 ? 1 : 0]);
        if (err != hipSuccess) return err;
        kern<<<dim3((unsigned)blocks), dim3(256), lds_bytes, stream>>>(P);
        return hipGetLastError();
    }
    constexpr int NB = FastConfig<D1, D2>::NB;
    typedef ALayout<D1, D2, KCH, 256> AL;
    auto kern = P.out16 ? igemm16_fast_kernel<Tag, D1, D2, KCH, NB, true, 256>
                        : igemm16_fast_kernel<Tag, D1, D2, KCH, NB, false, 256>;
    const size_t lds_bytes = (size_t)NB * AL::NBLK * (AL::ABLK + 1024);
    static std::atomic<unsigned long long> lds_set[2] = {{0}, {0}};
    hipError_t err = set_dynamic_lds_once(reinterpret_cast<const void*>(kern), (int)lds_bytes,
                                          lds_set[P.out16 ? 1 : 0]);
    if (err != hipSuccess) return err;
    kern<<<dim3((unsigned)blocks), dim3(256), lds_bytes, stream>>>(P);
    return hipGetLastError();
}

template <typename Tag>
hipError_t launch_dims(const IgemmParams& P, long long blocks, hipStream_t stream)
{
    if (P.D1 == 16 && P.D2 == 16) return launch_one<Tag, 16, 16>(P, blocks, stream);
    if (P.D1 == 8 && P.D2 == 8) return launch_one<Tag, 8, 8>(P, blocks, stream);
    return hipErrorInvalidValue;
}

}  // namespace

bool igemm16_fast_eligible(const ConvShape& s)
{
    if (s.dtype != 1 && s.dtype != 2) return false;
    if (!((s.D1 == 16 && s.D2 == 16) || (s.D1 == 8 && s.D2 == 8))) return false;
    if (s.D3 % 4 != 0) return false;
    if ((s.C * s.D2) % 64 != 0) return false;  // whole K stages per channel group
    if (s.kh * s.kw > 63) return false;        // one bit of the tap masks per window tap, bit 63 kept clear
    // 31-bit byte offsets: a tile's input window spans at most the images its 256/D1 pixels
    // touch; the repacked kernel is addressed from its start
    const long long img_bytes = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * 2;
    const long long hw = (long long)s.Ho * s.Wo;
    const long long pix = 256 / s.D1;
    const long long images_spanned = (pix + hw - 2) / hw + 1;
    if (images_spanned * img_bytes >= (1LL << 31)) return false;
    const long long colsp = ((long long)s.M * s.D3 + 255) / 256 * 256;
    const long long kp_bytes = (long long)s.D0 * s.kh * s.kw * (s.C * s.D2 / 8) * colsp * 16;
    if (kp_bytes >= (1LL << 31) - (1 << 24)) return false;
    if ((long long)s.pixels() >= (1LL << 31) - 256) return false;  // 32-bit pixel indices
    return true;
}

// Tile height the kernel would use: 256 rows when that gives every CU a tile and the K loop is
// long, else 128 rows (half the work per tile, two workgroups per CU; 6 % slower per FLOP on
// config 5), 0 when even those are too few: such problems use the generic kernel's small tiles
// and split K loop.
int igemm16_fast_tile_rows(const ConvShape& s)
{
    if (!igemm16_fast_eligible(s)) return 0;
    const long long colsp = ((long long)s.M * s.D3 + 255) / 256 * 256;
    const long long rows = (long long)s.pixels() * s.D1;
    // short K loops (measured on 36 .. 144 stages of 32 K elements): up to 72 stages the
    // half-height tile is 2 .. 6 % faster, because the other workgroup on the CU covers a
    // tile's set-up and stores; at 144 stages the full tile is 4 % faster
    const long long stages = (long long)s.kh * s.kw * s.C * s.D2 / 32;
    const bool short_k = stages <= 96 && (rows + 127) / 128 * (colsp / 256) * s.D0 >= 512;
    if (!short_k && (rows + 255) / 256 * (colsp / 256) * s.D0 >= 256) return 256;
    if ((rows + 127) / 128 * (colsp / 256) * s.D0 >= 256) return 128;
    return 0;
}

bool igemm16_fast_preferred(const ConvShape& s) { return igemm16_fast_tile_rows(s) != 0; }

int igemm16_fast_kgroup(const ConvShape& s)
{
    return s.D1 == 16 ? FastConfig<16, 16>::KCH : FastConfig<8, 8>::KCH;
}

hipError_t launch_igemm16_fast(const IgemmParams& P, long long blocks, int dtype,
                               hipStream_t stream)
{
    return dtype == 2 ? launch_dims<f16_tag>(P, blocks, stream)
                      : launch_dims<bf16_tag>(P, blocks, stream);
}

}  // namespace capscaps
