// fp32 matrix-core kernel of the capsule convolution forward pass with direct-to-LDS copies.
// Same implicit GEMM as the other igemm kernels (rows (pixel,d1), columns (m,d3),
// K = (tap, c, d2); paper Algorithm 2).  It serves capsule rows of 3 floats (D2 a multiple of
// 3: the 3x3x3 capsules of the paper's Fig. 2) as well as multiples of 4.
//
// Unit of data movement: a 16-byte LDS slot holding CW = 3 or 4 consecutive d2 of one capsule
// row ("chunk").  For CW = 3 the copy is a 12-byte buffer load, which the hardware places at
// a 16-byte lane stride in LDS, so both cases read operands with one 16-byte LDS load per lane
// and feed CW MFMA 32x32x2 instructions from it (element u of the lower and of the upper half
// wave form the K pair of instruction u; the fourth float of a 3-float slot is never used).
//
// Tile: 64*NW rows x 32*TN columns; wave w copies and contracts rows 64w..64w+63 (two MFMA
// row tiles) against all TN column tiles.  Lane i of a wave copies row 64w+i: its byte offset,
// with the out-of-range mark where the current tap falls into the padding, sits in one VGPR
// and is refreshed once per stage from a per-lane bit mask over the taps; everything else
// (tap, channel group, chunk) is a scalar offset.  K runs channel group outermost, tap inside,
// 4 chunks per stage, ring of 3 LDS stages, one barrier per stage; the K loop can be split over
// blocks (partial sums are reduced in a fixed order by the caller's reduce kernel).
//
// The same kernel serves 16-bit operands (one MFMA 32x32x16 per chunk pair and tile instead of CW
// fp32 ones).  Capsule rows of 8, 16 or 32 halves are, in units of 4 bytes, rows of 4, 8 or 16
// "floats": nothing else changes (any D1 and D3: non-square and vector capsules, which the
// 256x256-tile 16-bit kernel does not take).  Rows of 4 halves (4x4 capsules) no 16-byte copy can
// stage as they lie in memory: the 8 K values a 16-bit matrix instruction takes
// per lane are the rows of two channels, 32 bytes apart.  A pre-pass (pair_channels_kernel, at
// HBM speed) writes the input with channels paired, [pixel][c/2][d0][d1][c%2][d2]; in units of
// 4 bytes that is an fp32 layer with half the channels and rows of 4 "floats", so every offset
// and copy of this kernel stays as it is, and a chunk pair feeds one MFMA 32x32x16 per tile.
#include <hip/hip_runtime.h>

#include "igemm_common.h"
#include "lds_dma.h"

namespace capscaps {
namespace {

// KCH chunks per row and stage, ring of NB stages.  Small stages (2 chunks) halve the LDS
// footprint of a workgroup, so that more of them share a CU and one wave's copies and waits run
// under the others' MFMAs; they need capsule rows of at most 2 chunks.  With up to three column
// tiles the kernel is compiled for four waves per SIMD (126 registers: the accumulators and a
// small stage's operands) and takes a ring of three stages, so that four four-wave workgroups
// share a CU (config 2: 0.877 -> 0.860 ms against three workgroups with a ring of four);
// elsewhere the compiler's own register budget and the deeper ring of the small stages.
constexpr int waves_per_simd(int tn, int nw, int kch) { return nw == 4 && tn <= 3 && kch == 2 ? 4 : 1; }
// The 16-bit-output variants are held to the waves per SIMD their fp32-output twins reach by
// themselves (32 TN accumulator registers and about 30 others): left alone, the compiler reads
// all accumulators out for the rounding at once (146 registers more with four column tiles), one
// wave per SIMD remains, and a layer of 64 channels of 4x4 capsules runs 35 % slower with 16-bit
// than with fp32 output.
constexpr int waves_per_simd_out16(int tn, int nw, int kch)
{
    return waves_per_simd(tn, nw, kch) > 1 ? waves_per_simd(tn, nw, kch) : tn == 1 ? 6 : tn == 2 ? 4 : 3;
}
constexpr int ring_depth(int kch, int tn, int nw) { return kch == 2 && waves_per_simd(tn, nw, kch) == 1 ? 4 : 3; }

// Tag: f32_tag, or a 16-bit tag for capsule rows of 4 halves whose channels a pre-pass has paired
// (pair_channels_kernel): a 16-byte chunk then holds the 8 K values (c, c+1) x d2 of one row, all
// offsets are those of an fp32 layer with half the channels and rows of 4 floats, and a chunk pair
// feeds one 16-bit MFMA 32x32x16 per tile instead of CW fp32 ones.
// OUT16 (16-bit operands only): the output has the operands' type, rounded at the store.
template <typename Tag, int CW, int TN, int NW, int KCH, bool OUT16 = false>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(OUT16 ? waves_per_simd_out16(TN, NW, KCH) : waves_per_simd(TN, NW, KCH)))) void igemm32_dma_kernel(const Dma32Params P)
{
    constexpr bool F32 = std::is_same<Tag, f32_tag>::value;
    static_assert(!(F32 && OUT16), "fp32 operands have fp32 output");
    // a compile-time constant: with the choice made at run time the register allocator fails
    // to keep the copies' buffer descriptors in scalar registers
    constexpr int o16 = !OUT16 ? 0 : std::is_same<Tag, f16_tag>::value ? 2 : 1;
    static_assert(F32 || CW == 4, "16-bit chunks are whole 16-byte slots");
    constexpr int NB = ring_depth(KCH, TN, NW);
    constexpr int BM = 64 * NW, BN = 32 * TN, BNL = (BN + 63) / 64 * 64, TM = 2;
    constexpr int A_BYTES = KCH * BM * 16, B_BYTES = KCH * BNL * 16;
    constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int NBC = KCH * BNL / 64;  // kernel-side copies per stage, all waves
    constexpr int BPW = NBC / NW;        // ... per wave
    static_assert(NBC % NW == 0, "kernel copies divide evenly over the waves");
    constexpr int NCOPY = KCH + BPW;     // copies per wave and stage
    constexpr int OOB = (int)0x80000000u;
    // at a barrier the copies of the NB-2 most recent stages may still be in flight
    constexpr int KEEP = (NB - 2) * NCOPY;
    static_assert(KEEP < 64, "vmcnt is a 6-bit counter");
    constexpr int VMCNT_KEEP = 0x0F70 | (KEEP & 15) | ((KEEP >> 4) << 14);

    extern __shared__ char smem[];

    // ---- tile: column tiles fastest, then row tiles, leading capsule index, K split
    int L = blockIdx.x;
    int col_tile, row_tile, d0, split;
    if (P.xcd_span > 0) {
        // the D0 tiles of one (row tile, column tile) read the same input lines and write into
        // the same output lines: they run at the same time on one XCD and meet in its L2
        if (L < P.xcd_span) L = (L & 7) * (P.xcd_span >> 3) + (L >> 3);
        d0 = L % P.D0;
        int rest = L / P.D0;
        col_tile = rest % P.col_tiles;
        rest /= P.col_tiles;
        row_tile = rest % P.row_tiles;
        split = rest / P.row_tiles;
    } else {
        col_tile = L % P.col_tiles;
        int rest = L / P.col_tiles;
        row_tile = rest % P.row_tiles;
        rest /= P.row_tiles;
        d0 = rest % P.D0;
        split = rest / P.D0;
    }

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = lane >> 5, lr = lane & 31;
    const long long row0 = (long long)row_tile * BM;
    const int col0 = col_tile * BN;

    // ---- this lane's row: byte offset of its capsule row in the window's first input pixel,
    // relative to the first image the tile touches, and the bit mask of taps that read a real
    // input pixel
    const int hw = P.Ho * P.Wo;
    const long long n_first = (row0 / P.D1) / hw;
    const long long img_bytes = (long long)P.H * P.W * P.pixsz * 4;
    const int pix_bytes = (int)(P.pixsz * 4);
    // Lane offsets must not be negative (the hardware adds lane and scalar offset without
    // wrapping), but a window's first pixel may lie in the padding: the descriptor's base is
    // moved back by the largest such distance and every lane offset forward by the same.
    // Nothing is read below the tensor: only in-range taps are ever addressed.
    const int bias = ((P.pad > 0 ? P.pad : 0) * P.W + (P.pad_w > 0 ? P.pad_w : 0)) * pix_bytes;
    const char* in_base = static_cast<const char*>(P.in) + n_first * img_bytes - bias;
    int row_off;
    unsigned long long tap_ok = 0;
    {
        const long long rg = row0 + 64 * wave + lane;
        const bool exists = rg < P.rows;
        const long long rr = exists ? rg : row0;
        const long long pixel = rr / P.D1;
        const int d1 = (int)(rr % P.D1);
        const int n_rel = (int)(pixel / hw - n_first);
        const int rem = (int)(pixel % hw);
        const int x = rem / P.Wo, y = rem - x * P.Wo;
        const int ih0 = x * P.stride - P.pad, iw0 = y * P.stride - P.pad_w;
        row_off = (int)((((long long)n_rel * P.H + ih0) * P.W + iw0) * pix_bytes) +
                  (d0 * P.D1 + d1) * P.D2 * 4 + bias;
        if (exists) {
            int t = 0;
            for (int p = 0; p < P.kh; ++p)
                for (int q = 0; q < P.kw; ++q, ++t)
                    if ((unsigned)(ih0 + p) < (unsigned)P.H && (unsigned)(iw0 + q) < (unsigned)P.W)
                        tap_ok |= 1ull << t;
        }
    }
    long long in_left = P.in_bytes - n_first * img_bytes + bias;
    if (in_left > 0x7fffffffLL) in_left = 0x7fffffffLL;
    const rsrc_t rs_in = make_rsrc(in_base, (unsigned)in_left);
    rsrc_t rs_none = rs_in;  // nothing addressable: every lane stores zeros
    rs_none[2] = 0;
    const rsrc_t rs_kp = make_rsrc(P.kp, (unsigned)P.kp_bytes);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;

    // ---- K loop state of the next stage to copy (all scalar)
    const int st_begin = split * P.stages_per_split;
    int st_end = st_begin + P.stages_per_split;
    if (st_end > P.nstages) st_end = P.nstages;
    const int my_stages = st_end - st_begin;
    const int my_stages_pad = (my_stages + NB - 1) / NB * NB;
    const int chan_per_group = KCH / P.D2C;                  // D2C is 1, 2 or 4
    const int g_step = chan_per_group * P.cs * 4;           // bytes per channel group
    const int kp_step = KCH * P.colsp * 16;
    const int row_skip = (P.W - P.kw + 1) * pix_bytes;
    int issued = 0;
    int tap = st_begin % P.ntaps, grp = st_begin / P.ntaps;
    int tap_q = tap % P.kw;
    int tap_off = ((tap / P.kw) * P.W + tap_q) * pix_bytes;
    int g_off = grp * g_step;
    int c0 = grp * chan_per_group;  // first channel of the group
    int kp_off = (int)((((long long)d0 * P.nstages + st_begin) * KCH * P.colsp + col0) * 16);
    int q_off[KCH], q_chan[KCH];
#pragma unroll
    for (int q = 0; q < KCH; ++q) {
        q_chan[q] = q / P.D2C;
        q_off[q] = (q_chan[q] * P.cs + (q % P.D2C) * CW) * 4;
    }
    int b_const[BPW];
#pragma unroll
    for (int j = 0; j < BPW; ++j) {
        const int c = wave * BPW + j;
        b_const[j] = ((c / (BNL / 64)) * P.colsp + (c % (BNL / 64)) * 64) * 16;
    }
    const unsigned b_voff = (unsigned)lane * 16u;

    auto issue_stage = [&](int slot) {
        const bool live = issued < my_stages;
        const unsigned stage = lds0 + slot * STAGE_BYTES;
        // input side: this lane's row, chunks 0..KCH-1 of the stage
        const bool ok = live && ((tap_ok >> tap) & 1ull) != 0;
        const unsigned voff = ok ? (unsigned)row_off : (unsigned)OOB;
        const int s_base = tap_off + g_off;
#pragma unroll
        for (int q = 0; q < KCH; ++q) {
            const bool chan_ok = c0 + q_chan[q] < P.C;  // last group may be partial
            copy_to_lds_dwords<CW>(chan_ok ? rs_in : rs_none, stage + (q * BM + 64 * wave) * 16, voff,
                            s_base + q_off[q]);
        }
        // kernel side: this wave's share of the stage's KCH x BNL chunks
#pragma unroll
        for (int j = 0; j < BPW; ++j) {
            const int c = wave * BPW + j;
            copy_to_lds_dwords<4>(rs_kp, stage + A_BYTES + c * 1024, b_voff,
                           live ? kp_off + b_const[j] : OOB);
        }
        // next stage: next tap, after the last tap the next channel group
        ++issued;
        kp_off += kp_step;
        ++tap;
        ++tap_q;
        const bool row_end = tap_q == P.kw;
        tap_q = row_end ? 0 : tap_q;
        tap_off += row_end ? row_skip : pix_bytes;
        if (tap == P.ntaps) {
            tap = 0;
            tap_q = 0;
            tap_off = 0;
            g_off += g_step;
            c0 += chan_per_group;
        }
    };

    float16v acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    auto compute_stage = [&](int slot) {
        const char* stage = smem + slot * STAGE_BYTES;
#pragma unroll
        for (int t = 0; t < KCH / 2; ++t) {
            // lanes 0..31 take chunk 2t, lanes 32..63 chunk 2t+1
            float4v ka[TN], ib[TM];
#pragma unroll
            for (int a = 0; a < TN; ++a)
                ka[a] = *reinterpret_cast<const float4v*>(
                    stage + A_BYTES + ((2 * t + h) * BNL + a * 32 + lr) * 16);
#pragma unroll
            for (int b = 0; b < TM; ++b)
                ib[b] = *reinterpret_cast<const float4v*>(
                    stage + ((2 * t + h) * BM + 64 * wave + b * 32 + lr) * 16);
            if constexpr (F32) {
#pragma unroll
                for (int u = 0; u < CW; ++u)
#pragma unroll
                    for (int a = 0; a < TN; ++a)
#pragma unroll
                        for (int b = 0; b < TM; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(ka[a][u], ib[b][u],
                                                                             acc[a][b], 0, 0, 0);
            } else {
#pragma unroll
                for (int a = 0; a < TN; ++a)
#pragma unroll
                    for (int b = 0; b < TM; ++b)
                        Mma<Tag>::run(__builtin_bit_cast(chunk_t, ka[a]),
                                      __builtin_bit_cast(chunk_t, ib[b]), acc[a][b]);
            }
        }
    };

    // ---- prologue: NB-1 stages in flight, the first one landed
    static_for<NB - 1>([&](auto S0) { issue_stage(decltype(S0)::value); });
    __builtin_amdgcn_s_waitcnt(VMCNT_KEEP);
    __syncthreads();

    // ---- main loop: copy stage s+NB-1 into the slot read in iteration s-1, contract stage s
    for (int st = 0; st < my_stages_pad; st += NB) {
        static_for<NB>([&](auto SLOT) {
            constexpr int slot = decltype(SLOT)::value;
            issue_stage((slot + NB - 1) % NB);
            compute_stage(slot);
            // this wave's copies of the next stage have landed, its reads of this stage are
            // done; after the barrier both hold for every wave
            __builtin_amdgcn_s_waitcnt(VMCNT_KEEP & 0xF0FF);
            __syncthreads();
        });
    }

    // ---- epilogue: lane (h, lr) of tile (a, b) holds in registers 4g..4g+3 the columns
    // 8g + 4h + 0..3 of the tile for output row lr of the tile
    // (partial sums of a split K loop are fp32; the reduction rounds)
    float* __restrict__ out = P.out + (long long)split * P.out_elems;
    const int caps_out = P.D0 * P.D1 * P.D3;
    const bool st4 = (P.D3 & 3) == 0;
#pragma unroll
    for (int b = 0; b < TM; ++b) {
        const long long orow = row0 + 64 * wave + b * 32 + lr;
        if (orow >= P.rows) continue;
        const long long pixel = orow / P.D1;
        const int d1 = (int)(orow % P.D1);
        long long pix_at = pixel * P.M * caps_out;
        if (P.out_mode & 1) {
            const long long n = pixel / hw;
            const int rem = (int)(pixel - n * hw);
            const int x = rem / P.Wo, y = rem - x * P.Wo;
            pix_at = P.out_base + n * P.out_sn + x * P.out_sx + y * P.out_sy;
        }
        const long long orow_off = pix_at + (long long)(d0 * P.D1 + d1) * P.D3;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j0 = col0 + a * 32 + 8 * g + 4 * h;
                if (st4) {
                    if (j0 < P.cols) {
                        const int m = j0 / P.D3, d3 = j0 - m * P.D3;
                        float4v v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                                     acc[a][b][4 * g + 3]};
                        if constexpr (F32)
                            *reinterpret_cast<float4v*>(out + orow_off + (long long)m * caps_out + d3) = v;
                        else
                            store4(out, orow_off + (long long)m * caps_out + d3, v, o16);
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + u;
                        if (j < P.cols) {
                            // j / D3 by multiplication (exact while j * D3 < 2^32, which the host has checked)
                            const int m = P.d3_magic ? (int)__umulhi((unsigned)j, P.d3_magic) : j / P.D3;
                            const int d3 = j - m * P.D3;
                            if constexpr (F32)
                                out[orow_off + (long long)m * caps_out + d3] = acc[a][b][4 * g + u];
                            else
                                store1(out, orow_off + (long long)m * caps_out + d3, acc[a][b][4 * g + u], o16);
                        }
                    }
                }
            }
        }
    }
}

template <typename Tag, int CW, int TN, int NW, int KCH, bool OUT16 = false>
hipError_t launch_kch(const Dma32Params& P, long long blocks, hipStream_t stream)
{
    constexpr int BM = 64 * NW, BNL = (32 * TN + 63) / 64 * 64;
    auto kern = igemm32_dma_kernel<Tag, CW, TN, NW, KCH, OUT16>;
    const size_t lds_bytes = (size_t)ring_depth(KCH, TN, NW) * KCH * (BM + BNL) * 16;
    static std::atomic<unsigned long long> lds_set{0};
    hipError_t err = set_dynamic_lds_once(reinterpret_cast<const void*>(kern), (int)lds_bytes, lds_set);
    if (err != hipSuccess) return err;
    kern<<<dim3((unsigned)blocks), dim3(64 * NW), lds_bytes, stream>>>(P);
    return hipGetLastError();
}

// 2-chunk stages where the column copies still divide over the waves; 16-bit output straight from
// the kernel (16-bit operands) unless a split K loop leaves fp32 partial sums for the reduction
template <typename Tag, int CW, int TN, int NW>
hipError_t launch_one(const Dma32Params& P, long long blocks, hipStream_t stream)
{
    constexpr bool F32 = std::is_same<Tag, f32_tag>::value;
    const bool o16 = !F32 && (P.out_mode >> 1) != 0 && P.nsplit == 1;
    if constexpr ((2 * ((32 * TN + 63) / 64)) % NW == 0) {
        if (P.kch == 2) {
            if constexpr (!F32) {
                if (o16) return launch_kch<Tag, CW, TN, NW, 2, true>(P, blocks, stream);
            }
            return launch_kch<Tag, CW, TN, NW, 2>(P, blocks, stream);
        }
    }
    if constexpr (!F32) {
        if (o16) return launch_kch<Tag, CW, TN, NW, 4, true>(P, blocks, stream);
    }
    return launch_kch<Tag, CW, TN, NW, 4>(P, blocks, stream);
}

template <typename Tag, int CW, int NW>
hipError_t launch_tn(const Dma32Params& P, int tn, long long blocks, hipStream_t stream)
{
    switch (tn) {
        case 1: return launch_one<Tag, CW, 1, NW>(P, blocks, stream);
        case 2: return launch_one<Tag, CW, 2, NW>(P, blocks, stream);
        case 3: return launch_one<Tag, CW, 3, NW>(P, blocks, stream);
        default: return launch_one<Tag, CW, 4, NW>(P, blocks, stream);
    }
}

// 8-byte units: dst[pixel][c/2][d0*D1 + d1][c%2] = src[pixel][c][d0*D1 + d1]; a thread moves
// the two units of one (pixel, channel pair, row): one 16-byte store
__global__ __launch_bounds__(256) void pair_channels_kernel(const uint2* __restrict__ src,
                                                            uint4* __restrict__ dst, int C,
                                                            int rows_per_capsule, size_t pairs)
{
    const size_t id = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= pairs) return;
    size_t r = id;
    const int row = (int)(r % rows_per_capsule); r /= rows_per_capsule;
    const int c2 = (int)(r % (C / 2));
    const size_t pixel = r / (C / 2);
    const uint2* p = src + (pixel * C + 2 * c2) * rows_per_capsule + row;
    const uint2 lo = p[0], hi = p[rows_per_capsule];
    dst[id] = uint4{lo.x, lo.y, hi.x, hi.y};
}

inline int ceil_div_ll(long long a, long long b) { return (int)((a + b - 1) / b); }

}  // namespace

// Valid floats per 16-byte chunk: 4 or 3, such that a capsule row is 1, 2 or 4 chunks (so that
// the 4 chunks of a stage never split a row); 0 if neither fits.
int igemm32_dma_chunk_width(const ConvShape& s)
{
    // 16-bit operands: capsule rows of 8, 16 or 32 halves are rows of 4, 8 or 16 "floats" as they
    // lie in memory; rows of 4 halves need an even number of channels, which a pre-pass pairs so
    // that a chunk is (c, c+1) x 4 halves
    if (s.dtype != 0) {
        if (s.D2 == 8 || s.D2 == 16 || s.D2 == 32) return 4;
        return s.D2 == 4 && s.C % 2 == 0 ? 4 : 0;
    }
    for (int cw : {4, 3}) {
        if (s.D2 % cw) continue;
        const int d2c = s.D2 / cw;
        if (d2c == 1 || d2c == 2 || d2c == 4) return cw;
    }
    return 0;
}

bool igemm32_dma_eligible(const ConvShape& s)
{
    const int cw = igemm32_dma_chunk_width(s);
    if (cw == 0) return false;
    if (s.kh * s.kw > 64) return false;                   // one mask bit per window tap
    const int es = s.dtype == 0 ? 4 : 2;
    const long long img_bytes = (long long)s.H * s.W * s.C * s.D0 * s.D1 * s.D2 * es;
    const long long hw = (long long)s.Ho * s.Wo;
    const long long pix = (256 + s.D1 - 1) / s.D1 + 1;
    const long long images_spanned = (pix + hw - 2) / hw + 1;
    const long long bias = ((long long)(s.pad > 0 ? s.pad : 0) * s.W + (s.padw() > 0 ? s.padw() : 0)) *
                           s.C * s.D0 * s.D1 * s.D2 * es;
    if (images_spanned * img_bytes + bias >= (1LL << 31)) return false;
    const Dma32Plan pl = igemm32_dma_plan(s);
    // an output view is written by the kernel itself: no partial sums over a split K loop
    if (s.out_view && (pl.P.nsplit != 1 || s.out_sn < 0 || s.out_sx < 0 || s.out_sy < 0)) return false;
    if ((long long)pl.repack_bytes >= (1LL << 31) - (1 << 24)) return false;
    return pl.blocks > 0 && pl.blocks < 0x7fffffffLL;
}

// Tile, split and padding decisions (host side, pure arithmetic).
Dma32Plan igemm32_dma_plan(const ConvShape& s)
{
    Dma32Plan pl{};
    Dma32Params& P = pl.P;
    const int cw = igemm32_dma_chunk_width(s);
    pl.cw = cw;
    pl.dtype = s.dtype;
    // 16-bit operands: in units of 4 bytes the channel-paired input is an fp32 layer with half
    // the channels and capsule rows of 4 "floats"
    const bool paired = s.dtype != 0 && s.D2 == 4;
    const int C = paired ? s.C / 2 : s.C;
    const int D2 = s.dtype == 0 ? s.D2 : paired ? 4 : s.D2 / 2;
    pl.pair_bytes = paired && !s.in_paired ? (size_t)s.in_elems() * 2 : 0;
    P.H = s.H; P.W = s.W; P.C = C; P.M = s.M; P.stride = s.stride; P.pad = s.pad;
    P.pad_w = s.padw();
    P.out_mode = (s.out_view ? 1 : 0) | (s.out16 << 1);
    P.out_base = s.out_base; P.out_sn = s.out_sn; P.out_sx = s.out_sx; P.out_sy = s.out_sy;
    P.D0 = s.D0; P.D1 = s.D1; P.D2 = D2; P.D3 = s.D3; P.Ho = s.Ho; P.Wo = s.Wo;
    P.kh = s.kh; P.kw = s.kw; P.ntaps = s.kh * s.kw;
    P.rows = s.pixels() * s.D1;
    P.out_elems = (long long)s.out_elems();
    P.pixsz = (long long)C * s.D0 * s.D1 * D2;
    P.cs = s.D0 * s.D1 * D2;
    P.cols = s.M * s.D3;
    P.D2C = cw ? D2 / cw : 1;
    const int KK = C * P.D2C;                   // chunks per row and tap
    pl.tn = P.cols <= 32 ? 1 : P.cols <= 64 ? 2 : P.cols <= 96 ? 3 : 4;
    // four waves per block (256 rows) when that still fills the chip, else one (64 rows)
    {
        const int bn = 32 * pl.tn;
        const long long big = (long long)ceil_div_ll(s.pixels() * s.D1, 256) * ((P.cols + bn - 1) / bn) * s.D0;
        pl.nw = big >= 256 ? 4 : 1;
    }
    // chunks per stage: 2 for the four-wave tile with wide column tiles and short capsule rows
    // (measured on config 2: 0.955 ms against 0.987 ms), else 4
    // (16-bit: 8-chunk stages, one workgroup per CU, measured 22 % slower than 4-chunk ones; 2-chunk
    // stages 4 .. 5 % faster, as for fp32)
    // (16-bit vector capsules, whose consecutive rows are different pixels: a lane's 4 chunks are
    // one 64-byte run of memory; 11 .. 26 % faster than 2-chunk stages.  fp32: 2 % slower)
    const int KCH = (pl.nw == 4 && pl.tn >= 3 && P.D2C <= 2 && !(s.dtype != 0 && s.D1 <= 2)) ? 2 : 4;
    P.kch = KCH;
    const int groups = (KK + KCH - 1) / KCH;
    pl.kqp = groups * KCH;
    P.nstages = groups * P.ntaps;
    const int BN = 32 * pl.tn;
    P.col_tiles = (P.cols + BN - 1) / BN;
    P.colsp = P.col_tiles * BN;
    P.row_tiles = ceil_div_ll(P.rows, 64 * pl.nw);
    const long long tiles = (long long)P.row_tiles * P.col_tiles * s.D0;
    int nsplit = 1;
    if (tiles < 256) {
        nsplit = ceil_div_ll(512, tiles);
        if (nsplit > P.nstages) nsplit = P.nstages;
        if (nsplit > 64) nsplit = 64;
    }
    P.stages_per_split = (P.nstages + nsplit - 1) / nsplit;
    P.nsplit = (P.nstages + P.stages_per_split - 1) / P.stages_per_split;
    pl.blocks = tiles * P.nsplit;
    pl.repack_bytes = (size_t)s.D0 * P.nstages * KCH * P.colsp * 16;
    pl.partial_bytes = P.nsplit > 1 ? (size_t)P.nsplit * P.out_elems * sizeof(float) : 0;
    P.in_bytes = (long long)s.in_elems() * (s.dtype == 0 ? 4 : 2);
    P.kp_bytes = (long long)pl.repack_bytes;
    P.d3_magic = s.D3 > 1 && (long long)s.M * s.D3 * s.D3 < (1LL << 32)
                     ? (unsigned)(((1ULL << 32) + s.D3 - 1) / s.D3)
                     : 0u;  // 0: divide
    P.xcd_span = 0;
    // (config 2: 0.90 -> 0.82 ms; with a repacked kernel far beyond the 4 MB of an L2 every
    // XCD would stream all of it per round of tiles, so large ones keep the plain order)
    if (pl.repack_bytes <= ((size_t)8 << 20)) {
        const long long unit = 8LL * s.D0 * P.col_tiles;
        const long long span = pl.blocks / unit * unit;
        if (span > 0 && span < (1LL << 31)) P.xcd_span = (int)span;
    }
    return pl;
}

bool igemm32_dma_preferred(const ConvShape& s)
{
    if (!igemm32_dma_eligible(s)) return false;
    // measured on MI355X: 1.8x faster than the generic kernel on config 2 (many 256-row tiles);
    // on problems so small that the K loop is split the generic kernel's 64x64 tiles win
    // 16-bit: square capsules of 8 or 16 rows belong to the 256x256-tile kernel, which is 1.12 ..
    // 1.17x faster on whole column tiles (configs 3 and 5: 0.92 against 1.03 ms, 14.2 against
    // 16.6 ms) -- unless its 256-column tiles pad the columns much further than this kernel's
    // 128-column ones (320 or 384 columns: this kernel 14 % and 7 % faster)
    if (s.dtype != 0 && igemm16_fast_preferred(s)) {
        const long long cols = (long long)s.M * s.D3;
        const long long pad256 = (cols + 255) / 256 * 256, pad128 = (cols + 127) / 128 * 128;
        if (pad256 * 100 < pad128 * 115) return false;
    }
    const Dma32Plan pl = igemm32_dma_plan(s);
    return pl.nw == 4 && pl.P.nsplit == 1;
}

hipError_t launch_igemm32_dma(const Dma32Plan& pl, hipStream_t stream)
{
    if (pl.dtype == 1)
        return pl.nw == 4 ? launch_tn<bf16_tag, 4, 4>(pl.P, pl.tn, pl.blocks, stream)
                          : launch_tn<bf16_tag, 4, 1>(pl.P, pl.tn, pl.blocks, stream);
    if (pl.dtype == 2)
        return pl.nw == 4 ? launch_tn<f16_tag, 4, 4>(pl.P, pl.tn, pl.blocks, stream)
                          : launch_tn<f16_tag, 4, 1>(pl.P, pl.tn, pl.blocks, stream);
    if (pl.cw == 3)
        return pl.nw == 4 ? launch_tn<f32_tag, 3, 4>(pl.P, pl.tn, pl.blocks, stream)
                          : launch_tn<f32_tag, 3, 1>(pl.P, pl.tn, pl.blocks, stream);
    return pl.nw == 4 ? launch_tn<f32_tag, 4, 4>(pl.P, pl.tn, pl.blocks, stream)
                      : launch_tn<f32_tag, 4, 1>(pl.P, pl.tn, pl.blocks, stream);
}

hipError_t launch_pair_channels(const void* src, void* dst, size_t pixels, int C,
                                int rows_per_capsule, hipStream_t stream)
{
    const size_t pairs = pixels * (size_t)(C / 2) * rows_per_capsule;  // 16 bytes each
    const size_t blocks = (pairs + 255) / 256;
    if (blocks == 0 || blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    pair_channels_kernel<<<(unsigned)blocks, 256, 0, stream>>>(
        static_cast<const uint2*>(src), static_cast<uint4*>(dst), C, rows_per_capsule, pairs);
    return hipGetLastError();
}

hipError_t launch_pair_channels(const ConvShape& s, const void* src, void* dst, hipStream_t stream)
{
    return launch_pair_channels(src, dst, (size_t)s.N * s.H * s.W, s.C, s.D0 * s.D1, stream);
}

}  // namespace capscaps
