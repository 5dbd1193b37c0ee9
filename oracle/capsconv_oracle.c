/*
 * Capsule-convolution forward pass: plain CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct statement of what the operator computes.  Only the
 * tests, the smoke check and the CPU-baseline leg of the bench may call it; the GPU library
 * never does, and the two share no code.
 *
 * Definition followed (paper Sec. 1.2, Algorithm 2 "General capsule convolution", and the
 * worked example of Fig. 2): every output capsule is the sum, over the kernel window and
 * the input channels, of (input capsule matrix) x (kernel capsule matrix).  A capsule with a
 * leading dimension D0 (Fig. 2 uses 3x3x3 capsules) is a batch of D0 independent D1xD2
 * matrices; the leading index is carried through, never contracted (Algorithm 2's innermost
 * loop variable c selects one matrix of the batch for input, kernel and output alike).
 *
 * Readings of the paper taken here:
 *   - indices are 0-based; the loops accumulate into an output that starts at zero;
 *   - the product is  O_caps (D1xD3) += I_caps (D1xD2) . K_caps (D2xD3)   (Sec. 1.2);
 *   - cross-correlation: input row = row_offset + tap row, no kernel flip (Algorithm 2);
 *   - row_offset = x * stride (Algorithm 2); symmetric zero padding `pad` is an extension,
 *     pad = 0 is the paper's operator;  H' = floor((H + 2 pad - kh) / stride) + 1;
 *   - a batch dimension N is added outermost; images are independent.
 *
 * Logical tensors (dense, row-major, last index fastest):
 *   I[n][h][w][c][d0][d1][d2]      N x H  x W  x C x D0 x D1 x D2
 *   K[p][q][c][m][d0][d2][d3]      kh x kw x C x M x D0 x D2 x D3   (order of Fig. 2's caption)
 *   O[n][x][y][m][d0][d1][d3]      N x H' x W' x M x D0 x D1 x D3
 *
 * Element values arrive as float (already rounded to the run's storage type by the caller);
 * every product and every sum is formed in double.  Results are returned in double.
 * Optionally the sum of absolute values of the products, S = sum |I| * |K|, is returned per
 * output element: it is the natural scale for a summation-order error bound.
 */
#include <stddef.h>
#include <stdlib.h>

typedef struct {
    int N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3;
} capsconv_dims;

static int out_extent(int in, int k, int stride, int pad)
{
    int span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* logical-index accessors: no flattening tricks anywhere else */
static double I_at(const float *I, const capsconv_dims *g, int n, int h, int w, int c, int d0,
                   int d1, int d2)
{
    size_t idx = ((((((size_t)n * g->H + h) * g->W + w) * g->C + c) * g->D0 + d0) * g->D1 + d1) *
                     g->D2 + d2;
    return (double)I[idx];
}

static double K_at(const float *K, const capsconv_dims *g, int p, int q, int c, int m, int d0,
                   int d2, int d3)
{
    size_t idx = ((((((size_t)p * g->kw + q) * g->C + c) * g->M + m) * g->D0 + d0) * g->D2 + d2) *
                     g->D3 + d3;
    return (double)K[idx];
}

/*
 * One output capsule (n, x, y, m): all D0 x D1 x D3 elements, written to o[d0][d1][d3]
 * (and s[d0][d1][d3] if s is not NULL).  Algorithm 2's body: for every input channel and
 * every window tap, one small matrix product per leading index d0, accumulated.
 */
static void one_capsule(const float *I, const float *K, const capsconv_dims *g, int n, int x,
                        int y, int m, double *o, double *s)
{
    const int D0 = g->D0, D1 = g->D1, D2 = g->D2, D3 = g->D3;
    for (int e = 0; e < D0 * D1 * D3; ++e) {
        o[e] = 0.0;
        if (s) s[e] = 0.0;
    }
    const int row_offset = x * g->stride - g->pad;
    const int col_offset = y * g->stride - g->pad;
    for (int c = 0; c < g->C; ++c) {
        for (int p = 0; p < g->kh; ++p) {
            for (int q = 0; q < g->kw; ++q) {
                const int h = row_offset + p;
                const int w = col_offset + q;
                if (h < 0 || h >= g->H || w < 0 || w >= g->W) continue; /* zero padding */
                for (int d0 = 0; d0 < D0; ++d0) {
                    /* matrix_multiply(I-capsule, K-capsule) accumulated into the O-capsule */
                    for (int d1 = 0; d1 < D1; ++d1) {
                        for (int d3 = 0; d3 < D3; ++d3) {
                            double acc = 0.0, absacc = 0.0;
                            for (int d2 = 0; d2 < D2; ++d2) {
                                double a = I_at(I, g, n, h, w, c, d0, d1, d2);
                                double b = K_at(K, g, p, q, c, m, d0, d2, d3);
                                double prod = a * b;
                                acc += prod;
                                absacc += prod < 0 ? -prod : prod;
                            }
                            o[(d0 * D1 + d1) * D3 + d3] += acc;
                            if (s) s[(d0 * D1 + d1) * D3 + d3] += absacc;
                        }
                    }
                }
            }
        }
    }
}

/* Output extents; returns 0 on success, -1 if the arguments describe no valid operator. */
int capsconv_oracle_out_shape(int H, int W, int kh, int kw, int stride, int pad, int *Ho, int *Wo)
{
    if (H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return -1;
    if (kh > H + 2 * pad || kw > W + 2 * pad) return -1;
    *Ho = out_extent(H, kh, stride, pad);
    *Wo = out_extent(W, kw, stride, pad);
    return 0;
}

/*
 * Full tensor.  O (and S, if not NULL) must hold N*H'*W'*M*D0*D1*D3 doubles.
 * Returns 0, or -1 on invalid dimensions.
 */
int capsconv_oracle_fwd(const float *I, const float *K, double *O, double *S, int N, int H, int W,
                        int C, int M, int kh, int kw, int stride, int pad, int D0, int D1, int D2,
                        int D3)
{
    capsconv_dims g = {N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3};
    int Ho, Wo;
    if (N <= 0 || C <= 0 || M <= 0 || D0 <= 0 || D1 <= 0 || D2 <= 0 || D3 <= 0) return -1;
    if (capsconv_oracle_out_shape(H, W, kh, kw, stride, pad, &Ho, &Wo)) return -1;
    const size_t caps = (size_t)D0 * D1 * D3;
    const long long npix = (long long)N * Ho * Wo;
#pragma omp parallel for schedule(dynamic, 4)
    for (long long pix = 0; pix < npix; ++pix) {
        const int n = (int)(pix / ((long long)Ho * Wo));
        const int x = (int)((pix / Wo) % Ho);
        const int y = (int)(pix % Wo);
        for (int m = 0; m < M; ++m) {
            size_t base = ((size_t)pix * M + m) * caps;
            one_capsule(I, K, &g, n, x, y, m, O + base, S ? S + base : NULL);
        }
    }
    return 0;
}

/*
 * Subset: `count` output capsules listed as quadruples (n, x, y, m) in `which`
 * (4*count ints).  O (and S) receive count * D0*D1*D3 doubles, in list order.
 * Returns 0, -1 on invalid dimensions, -2 if a listed capsule is out of range.
 */
int capsconv_oracle_fwd_subset(const float *I, const float *K, double *O, double *S, int N, int H,
                               int W, int C, int M, int kh, int kw, int stride, int pad, int D0,
                               int D1, int D2, int D3, const int *which, long long count)
{
    capsconv_dims g = {N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3};
    int Ho, Wo;
    if (N <= 0 || C <= 0 || M <= 0 || D0 <= 0 || D1 <= 0 || D2 <= 0 || D3 <= 0) return -1;
    if (capsconv_oracle_out_shape(H, W, kh, kw, stride, pad, &Ho, &Wo)) return -1;
    for (long long i = 0; i < count; ++i) {
        const int *w4 = which + 4 * i;
        if (w4[0] < 0 || w4[0] >= N || w4[1] < 0 || w4[1] >= Ho || w4[2] < 0 || w4[2] >= Wo ||
            w4[3] < 0 || w4[3] >= M)
            return -2;
    }
    const size_t caps = (size_t)D0 * D1 * D3;
#pragma omp parallel for schedule(dynamic, 8)
    for (long long i = 0; i < count; ++i) {
        const int *w4 = which + 4 * i;
        one_capsule(I, K, &g, w4[0], w4[1], w4[2], w4[3], O + (size_t)i * caps,
                    S ? S + (size_t)i * caps : NULL);
    }
    return 0;
}

/*
 * ---------------------------------------------------------------------------------------------
 * Backward pass (the two results of the paper's Algorithm 4: Input_diff and Kernel_diff).
 * The printed algorithm is garbled (a one-argument batched multiply, Input_diff typed as a
 * D1 x D3 capsule), so the definition taken here is the derivative of Algorithm 2's sum, which
 * is what any backward pass of that operator must produce.  With G = dL/dO:
 *
 *   dI[n,h,w,c,d0] (D1 x D2) = sum over (x,p) with x*stride+p-pad = h, (y,q) with y*stride+q-pad = w,
 *                              and m of   G[n,x,y,m,d0] (D1 x D3) . K[p,q,c,m,d0]^T (D3 x D2)
 *   dK[p,q,c,m,d0] (D2 x D3) = sum over n, x, y with an in-range input pixel of
 *                              I[n,x*stride+p-pad,y*stride+q-pad,c,d0]^T (D2 x D1) . G[n,x,y,m,d0] (D1 x D3)
 *
 * Both are written in gather form (one output element at a time), so there is nothing to
 * synchronise and every sum has a fixed order.  Products and sums in double.
 */
static double G_at(const float *G, const capsconv_dims *g, int Ho, int Wo, int n, int x, int y,
                   int m, int d0, int d1, int d3)
{
    size_t idx = ((((((size_t)n * Ho + x) * Wo + y) * g->M + m) * g->D0 + d0) * g->D1 + d1) *
                     g->D3 + d3;
    return (double)G[idx];
}

/* dI: N*H*W*C*D0*D1*D2 doubles.  Returns 0, or -1 on invalid dimensions. */
int capsconv_oracle_bwd_input(const float *G, const float *K, double *dI, int N, int H, int W,
                              int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                              int D2, int D3)
{
    capsconv_dims g = {N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3};
    int Ho, Wo;
    if (N <= 0 || C <= 0 || M <= 0 || D0 <= 0 || D1 <= 0 || D2 <= 0 || D3 <= 0) return -1;
    if (capsconv_oracle_out_shape(H, W, kh, kw, stride, pad, &Ho, &Wo)) return -1;
    const long long npix = (long long)N * H * W;
#pragma omp parallel for schedule(dynamic, 4)
    for (long long pix = 0; pix < npix; ++pix) {
        const int n = (int)(pix / ((long long)H * W));
        const int h = (int)((pix / W) % H);
        const int w = (int)(pix % W);
        for (int c = 0; c < C; ++c)
            for (int d0 = 0; d0 < D0; ++d0)
                for (int d1 = 0; d1 < D1; ++d1)
                    for (int d2 = 0; d2 < D2; ++d2) {
                        double acc = 0.0;
                        for (int p = 0; p < kh; ++p) {
                            const int hx = h + pad - p; /* = x * stride */
                            if (hx < 0 || hx % stride != 0 || hx / stride >= Ho) continue;
                            for (int q = 0; q < kw; ++q) {
                                const int wy = w + pad - q;
                                if (wy < 0 || wy % stride != 0 || wy / stride >= Wo) continue;
                                const int x = hx / stride, y = wy / stride;
                                for (int m = 0; m < M; ++m)
                                    for (int d3 = 0; d3 < D3; ++d3)
                                        acc += G_at(G, &g, Ho, Wo, n, x, y, m, d0, d1, d3) *
                                               K_at(K, &g, p, q, c, m, d0, d2, d3);
                            }
                        }
                        dI[((((size_t)pix * C + c) * D0 + d0) * D1 + d1) * D2 + d2] = acc;
                    }
    }
    return 0;
}

/* dK: kh*kw*C*M*D0*D2*D3 doubles.  Returns 0, or -1 on invalid dimensions. */
int capsconv_oracle_bwd_kernel(const float *I, const float *G, double *dK, int N, int H, int W,
                               int C, int M, int kh, int kw, int stride, int pad, int D0, int D1,
                               int D2, int D3)
{
    capsconv_dims g = {N, H, W, C, M, kh, kw, stride, pad, D0, D1, D2, D3};
    int Ho, Wo;
    if (N <= 0 || C <= 0 || M <= 0 || D0 <= 0 || D1 <= 0 || D2 <= 0 || D3 <= 0) return -1;
    if (capsconv_oracle_out_shape(H, W, kh, kw, stride, pad, &Ho, &Wo)) return -1;
    const long long ncaps = (long long)kh * kw * C * M;
#pragma omp parallel for schedule(dynamic, 1)
    for (long long kc = 0; kc < ncaps; ++kc) {
        const int m = (int)(kc % M);
        const int c = (int)((kc / M) % C);
        const int q = (int)((kc / ((long long)M * C)) % kw);
        const int p = (int)(kc / ((long long)M * C * kw));
        for (int d0 = 0; d0 < D0; ++d0)
            for (int d2 = 0; d2 < D2; ++d2)
                for (int d3 = 0; d3 < D3; ++d3) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int x = 0; x < Ho; ++x) {
                            const int h = x * stride + p - pad;
                            if (h < 0 || h >= H) continue;
                            for (int y = 0; y < Wo; ++y) {
                                const int w = y * stride + q - pad;
                                if (w < 0 || w >= W) continue;
                                for (int d1 = 0; d1 < D1; ++d1)
                                    acc += I_at(I, &g, n, h, w, c, d0, d1, d2) *
                                           G_at(G, &g, Ho, Wo, n, x, y, m, d0, d1, d3);
                            }
                        }
                    dK[(((size_t)kc * D0 + d0) * D2 + d2) * D3 + d3] = acc;
                }
    }
    return 0;
}

/* Number of OpenMP threads the loops above will use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int capsconv_oracle_threads(void) { return omp_get_max_threads(); }
#else
int capsconv_oracle_threads(void) { return 1; }
#endif
