// Wavefront-level small-matrix path of the capsule convolution forward pass (paper Sec. 1.3:
// "many small matrix multiplications"; Algorithm 2): for shapes whose (m, d3) extent is too
// narrow to fill a matrix-core tile (the worked example of Fig. 2 has 3 columns).
//
// A wave owns groups of G = 4 consecutive output pixels.  Its lanes are laid over the output
// capsules of such a group: lane = (pixel group, output channel m, capsule row d1, quad of
// capsule columns d3), and every lane keeps G x 4 accumulators -- the same (m, d1, d3 quad) of
// the group's G pixels -- so the contraction over d2 runs in registers: per contracted value
// one 16-byte LDS read brings the lane's 4 kernel-capsule columns, G 4-byte reads bring the
// input-capsule values of the G pixels (lanes that share d1 read the same word), and 4 G plain
// fp32 FMAs follow: one LDS cycle per FMA instruction, which is the rate the four SIMDs of a CU
// consume them at.
//
// Staging, once per window row p and channel chunk: the workgroup (4 waves, one tile of output
// channels) copies the kernel capsules K[p, 0..kw, chunk, m tile] into LDS, each wave copies
// the window row of its own pixels I[pixel + (p, 0..kw), chunk]; both with coalesced global
// loads (consecutive lanes walk a pixel's contiguous capsule data), widened to fp32 on the way,
// padding taps staged as zeros.  Two barriers per stage.
#include <hip/hip_runtime.h>

#include "igemm_common.h"

namespace capscaps {
namespace {

constexpr int G = 4;  // output pixels per pixel group (accumulator rows per lane)

struct WMagic {
    unsigned mul, pass;  // x / d = mulhi(x, mul) + (x & pass); d = 1 is (0, -1)
};
__device__ __forceinline__ int wdiv(int x, WMagic m)
{
    return (int)(__umulhi((unsigned)x, m.mul) + ((unsigned)x & m.pass));
}
WMagic wmagic(long long d)
{
    if (d <= 1) return WMagic{0u, 0xffffffffu};
    return WMagic{(unsigned)(((1ULL << 32) + d - 1) / d), 0u};
}

struct WaveParams {
    const void* in;
    const void* kernel;
    float* out;
    int H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3, Ho, Wo;
    int pixels;        // N*Ho*Wo
    int hw;            // Ho*Wo
    int Mt, m_tiles;   // output channels per workgroup, tiles of them
    int D3q, D3p;      // quads of capsule columns, columns padded to whole quads
    int LE;            // lanes per pixel group: Mt*D1*D3q
    int PGW;           // pixel groups per wave
    int CC;            // channels per stage
    int R;             // D1*D2: elements of one input capsule slice
    int cs;            // D0*D1*D2: input channel stride
    long long pixsz, img_elems;
    long long k_sp, k_sq, k_sc, k_sm, k_sd0;  // kernel tensor strides (dense layout)
    int ks_words;      // LDS words of the kernel stage
    int is_words;      // LDS words of one wave's input stage
    WMagic mg_hw, mg_Wo, mg_LE, mg_D1D3q, mg_D3q, mg_kwCCR, mg_CCR, mg_R, mg_MtD3, mg_D3;
    int out16;
};

template <typename E>
__device__ __forceinline__ float widen(E v);
template <>
__device__ __forceinline__ float widen<float>(float v) { return v; }
struct bf16_bits { unsigned short v; };
struct f16_bits { unsigned short v; };
template <>
__device__ __forceinline__ float widen<bf16_bits>(bf16_bits b)
{
    return __builtin_bit_cast(float, (unsigned)b.v << 16);
}
template <>
__device__ __forceinline__ float widen<f16_bits>(f16_bits b)
{
    return (float)__builtin_bit_cast(_Float16, b.v);
}

template <typename E>
__global__ __launch_bounds__(256) void wave_conv_kernel(const WaveParams P)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const E* __restrict__ in = static_cast<const E*>(P.in);
    const E* __restrict__ kern = static_cast<const E*>(P.kernel);

    int L = blockIdx.x;
    const int m_tile = L % P.m_tiles;
    L /= P.m_tiles;
    const int d0 = L % P.D0;
    const int ptile = L / P.D0;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int m0 = m_tile * P.Mt;
    const int ppw = P.PGW * G;                          // pixels per wave
    const int pix0 = (ptile * 4 + wave) * ppw;          // first pixel of this wave

    float* Ks = smem;                                   // [kw][CC][D2][Mt][D3p]
    float* Is = smem + P.ks_words + wave * P.is_words;  // [ppw][kw][CC][D1][D2]
    int* origin = reinterpret_cast<int*>(smem + P.ks_words + 4 * P.is_words) + wave * 3 * 64;
    // per pixel of the wave: image, first window row and column (may lie in the padding)
    if (lane < ppw) {
        const int pixel = pix0 + lane;
        int n = -1, ih0 = 0, iw0 = 0;
        if (pixel < P.pixels) {
            n = wdiv(pixel, P.mg_hw);
            const int rem = pixel - n * P.hw;
            const int x = wdiv(rem, P.mg_Wo), y = rem - x * P.Wo;
            ih0 = x * P.stride - P.pad;
            iw0 = y * P.stride - P.pad;
        }
        origin[3 * lane] = n;
        origin[3 * lane + 1] = ih0;
        origin[3 * lane + 2] = iw0;
    }

    // this lane's output capsule piece: pixel group, channel, row, column quad
    const int pgl = wdiv(lane, P.mg_LE);
    const int slot = lane - pgl * P.LE;
    const int mt = wdiv(slot, P.mg_D1D3q);
    const int r1 = slot - mt * (P.D1 * P.D3q);
    const int d1 = wdiv(r1, P.mg_D3q), d3q = r1 - d1 * P.D3q;
    const bool lane_on = pgl < P.PGW && m0 + mt < P.M;

    float4v acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = float4v{0.f, 0.f, 0.f, 0.f};

    const int kwCCR = P.kw * P.CC * P.R, CCR = P.CC * P.R;
    const int is_count = ppw * kwCCR;                   // words of the wave's input stage
    const int MtD3 = P.Mt * P.D3;
    const int ks_row = P.D2 * MtD3;                     // kernel elements per (q, c)

    for (int p = 0; p < P.kh; ++p) {
        for (int c0 = 0; c0 < P.C; c0 += P.CC) {
            const int cc = P.C - c0 < P.CC ? P.C - c0 : P.CC;
            __syncthreads();  // the previous stage has been consumed (and `origin` is written)
            // ---- kernel capsules of window row p, channels c0.., this channel tile
            for (int qc = 0; qc < P.kw * cc; ++qc) {
                const int q = qc / cc, c = qc - q * cc;  // uniform
                const long long kbase = p * P.k_sp + q * P.k_sq + (long long)(c0 + c) * P.k_sc +
                                        d0 * P.k_sd0;
                float* dst = Ks + (q * P.CC + c) * (P.D2 * P.Mt * P.D3p);
                // (loads of 4 rounds in flight before their LDS stores: a stage is latency-bound)
                for (int f0 = tid; f0 < ks_row; f0 += 4 * 256) {
                    float v[4];
                    int at[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int f = f0 + 256 * u;
                        const int d2 = wdiv(f, P.mg_MtD3), r = f - d2 * MtD3;
                        const int mm = wdiv(r, P.mg_D3), d3 = r - mm * P.D3;
                        v[u] = 0.f;
                        at[u] = f < ks_row ? (d2 * P.Mt + mm) * P.D3p + d3 : -1;
                        if (f < ks_row && m0 + mm < P.M)
                            v[u] = widen<E>(kern[kbase + (long long)(m0 + mm) * P.k_sm + d2 * P.D3 + d3]);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (at[u] >= 0) dst[at[u]] = v[u];
                }
            }
            // ---- this wave's window rows: [pixel][q][c][d1][d2]; consecutive lanes walk a
            // pixel's contiguous capsule data
            for (int f0 = lane; f0 < is_count; f0 += 4 * 64) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int f = f0 + 64 * u < is_count ? f0 + 64 * u : 0;
                    const int ps = wdiv(f, P.mg_kwCCR), r = f - ps * kwCCR;
                    const int q = wdiv(r, P.mg_CCR), r2 = r - q * CCR;
                    const int c = wdiv(r2, P.mg_R), e = r2 - c * P.R;
                    const int n = origin[3 * ps], ih = origin[3 * ps + 1] + p,
                              iw = origin[3 * ps + 2] + q;
                    v[u] = 0.f;
                    if (n >= 0 && c < cc && (unsigned)ih < (unsigned)P.H && (unsigned)iw < (unsigned)P.W)
                        v[u] = widen<E>(in[n * P.img_elems + ((long long)ih * P.W + iw) * P.pixsz +
                                           (long long)(c0 + c) * P.cs + d0 * P.R + e]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (f0 + 64 * u < is_count) Is[f0 + 64 * u] = v[u];
            }
            __syncthreads();
            if (!lane_on) continue;
            // ---- contraction over (q, c, d2) in registers
            const float* kq = Ks + mt * P.D3p + 4 * d3q;
            const float* iq = Is + pgl * G * kwCCR + d1 * P.D2;
            for (int q = 0; q < P.kw; ++q) {
                for (int c = 0; c < cc; ++c) {
                    const float* kc = kq + (q * P.CC + c) * (P.D2 * P.Mt * P.D3p);
                    const float* ic = iq + q * CCR + c * P.R;
                    for (int d2 = 0; d2 < P.D2; ++d2) {
                        const float4v kv = *reinterpret_cast<const float4v*>(kc + d2 * P.Mt * P.D3p);
#pragma unroll
                        for (int g = 0; g < G; ++g) {
                            const float iv = ic[g * kwCCR + d2];
                            acc[g][0] = fmaf(iv, kv[0], acc[g][0]);
                            acc[g][1] = fmaf(iv, kv[1], acc[g][1]);
                            acc[g][2] = fmaf(iv, kv[2], acc[g][2]);
                            acc[g][3] = fmaf(iv, kv[3], acc[g][3]);
                        }
                    }
                }
            }
        }
    }

    if (!lane_on) return;
    const long long caps_out = (long long)P.D0 * P.D1 * P.D3;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int pixel = pix0 + pgl * G + g;
        if (pixel >= P.pixels) continue;
        const long long base = ((long long)pixel * P.M + m0 + mt) * caps_out +
                               (long long)(d0 * P.D1 + d1) * P.D3 + 4 * d3q;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (4 * d3q + u < P.D3) store1(P.out, base + u, acc[g][u], P.out16);
    }
}

struct WavePlan {
    WaveParams P;
    long long blocks;
    size_t lds_bytes;
    bool ok;
};

WavePlan wave_plan(const ConvShape& s)
{
    WavePlan pl{};
    WaveParams& P = pl.P;
    pl.ok = false;
    if (!s.plain()) return pl;
    P.H = s.H; P.W = s.W; P.C = s.C; P.M = s.M; P.kh = s.kh; P.kw = s.kw; P.stride = s.stride;
    P.pad = s.pad; P.D0 = s.D0; P.D1 = s.D1; P.D2 = s.D2; P.D3 = s.D3; P.Ho = s.Ho; P.Wo = s.Wo;
    if (s.pixels() >= (1LL << 30)) return pl;
    P.pixels = (int)s.pixels();
    P.hw = s.Ho * s.Wo;
    P.D3q = (s.D3 + 3) / 4;
    P.D3p = 4 * P.D3q;
    const long long per_channel = (long long)s.D1 * P.D3q;  // lanes one output channel takes
    if (per_channel > 64) return pl;
    P.Mt = (int)(64 / per_channel);
    if (P.Mt > s.M) P.Mt = s.M;
    P.m_tiles = (s.M + P.Mt - 1) / P.Mt;
    P.LE = (int)(P.Mt * per_channel);
    P.PGW = 64 / P.LE;
    if (P.PGW > 16) P.PGW = 16;  // at most 64 pixels per wave
    // a small problem spreads over more workgroups with fewer pixel groups per wave
    while (P.PGW > 1 && (long long)P.pixels < 256LL * 4 * P.PGW * G) P.PGW /= 2;
    P.R = s.D1 * s.D2;
    P.cs = s.D0 * P.R;
    P.pixsz = (long long)s.C * P.cs;
    P.img_elems = (long long)s.H * s.W * P.pixsz;
    if ((long long)s.D1 * s.D2 >= (1 << 20) || (long long)s.kw * s.C * P.R >= (1LL << 24)) return pl;
    P.k_sd0 = (long long)s.D2 * s.D3;
    P.k_sm = P.k_sd0 * s.D0;
    P.k_sc = P.k_sm * s.M;
    P.k_sq = P.k_sc * s.C;
    P.k_sp = P.k_sq * s.kw;
    // channels per stage: as many as fit 60 KB of LDS
    const long long budget = 60 * 1024 / 4 - 4 * 3 * 64;
    auto words = [&](int cc, long long& ks, long long& is) {
        ks = (long long)s.kw * cc * s.D2 * P.Mt * P.D3p;
        is = ((long long)P.PGW * G * s.kw * cc * P.R + 3) / 4 * 4;
        return ks + 4 * is;
    };
    long long ks = 0, is = 0;
    int cc = s.C < 64 ? s.C : 64;
    while (cc > 1 && words(cc, ks, is) > budget) cc = (cc + 1) / 2;
    while (words(cc, ks, is) > budget && P.PGW > 1) P.PGW /= 2;
    if (words(cc, ks, is) > budget) return pl;
    P.CC = cc;
    P.ks_words = (int)ks;
    P.is_words = (int)is;
    pl.lds_bytes = (size_t)(ks + 4 * is + 4 * 3 * 64) * 4;
    const long long ppb = 4LL * P.PGW * G;  // pixels per workgroup
    pl.blocks = (P.pixels + ppb - 1) / ppb * P.m_tiles * s.D0;
    if (pl.blocks <= 0 || pl.blocks >= (1LL << 31)) return pl;
    P.mg_hw = wmagic(P.hw); P.mg_Wo = wmagic(s.Wo); P.mg_LE = wmagic(P.LE);
    P.mg_D1D3q = wmagic(per_channel); P.mg_D3q = wmagic(P.D3q);
    P.mg_kwCCR = wmagic((long long)s.kw * cc * P.R); P.mg_CCR = wmagic((long long)cc * P.R);
    P.mg_R = wmagic(P.R); P.mg_MtD3 = wmagic((long long)P.Mt * s.D3); P.mg_D3 = wmagic(s.D3);
    // exactness of the multiplicative divisions (x * d < 2^32)
    if ((long long)P.pixels * P.hw >= (1LL << 32) || (long long)P.hw * s.Wo >= (1LL << 32)) return pl;
    const long long is_count = (long long)P.PGW * G * s.kw * cc * P.R;
    if (is_count * s.kw * cc * P.R >= (1LL << 32)) return pl;
    if ((long long)s.D2 * P.Mt * s.D3 * P.Mt * s.D3 >= (1LL << 32)) return pl;
    P.out16 = s.out16;
    pl.ok = true;
    return pl;
}

}  // namespace

bool wave_conv_eligible(const ConvShape& s) { return wave_plan(s).ok; }

hipError_t launch_wave_conv(const ConvShape& s, const void* in, const void* kernel, float* out,
                            hipStream_t stream)
{
    WavePlan pl = wave_plan(s);
    if (!pl.ok) return hipErrorInvalidValue;
    pl.P.in = in;
    pl.P.kernel = kernel;
    pl.P.out = out;
    const dim3 grid((unsigned)pl.blocks), block(256);
    switch (s.dtype) {
        case 0: wave_conv_kernel<float><<<grid, block, pl.lds_bytes, stream>>>(pl.P); break;
        case 1: wave_conv_kernel<bf16_bits><<<grid, block, pl.lds_bytes, stream>>>(pl.P); break;
        case 2: wave_conv_kernel<f16_bits><<<grid, block, pl.lds_bytes, stream>>>(pl.P); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace capscaps
