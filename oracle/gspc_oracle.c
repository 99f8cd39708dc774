/*
 * CPU oracle for the forward grouped 2-D convolution (NCHW, g groups).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be linked or called from it; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Everything is double precision: callers widen fp32 (or bf16-rounded) data
 * to double, which is exact, so the only rounding left is the fp64 summation.
 *
 * What each routine follows in the paper (arXiv 2006.09791):
 *   - oracle_conv2d_grouped : the definition of G(g) in Section II and Fig. 2
 *     (filter oc reads only the Cin/g channels of its group), tensor shapes of
 *     Section III-B, index expression oh*S+kh / ow*S+kw of Algorithm 1's
 *     convolution stage (no kernel flip), zero padding ("padded input").
 *   - oracle_macs           : the MAC formula of Section IV-B (Eq. 2).
 *   - oracle_conv2d_standard: Section II's standard convolution S, written
 *     with no notion of groups at all (used to pin the grouped routine).
 *   - oracle_alg1_*         : the four stages of Algorithm 1 (Section III-B)
 *     restated with the printed listing's slips corrected (7-D W', 6-D X',
 *     6-D Y', 4-D Y) for tile sizes T_O | KPG, T_I | CPG.
 *   - oracle_alg1_conv_vec  : the convolution stage with the T_O filters of a
 *     tile as one vector and (group, image) pairs over the cores, the CPU
 *     schedule of Sections III-B / III-C; a timed baseline, pinned bit-identical
 *     to oracle_alg1_conv.
 *   - relu / add / maxpool  : the non-convolution ops of the ResNet-style
 *     stacks of Section IV-A, needed to chain layers end to end.
 *
 * Readings taken where the printed algorithm is garbled:
 *   - kernel reshape reads W[j*KPG + k*T_O + co][c*T_I + ci][h][w] (the
 *     printed index drops the tile index k);
 *   - X' spans the padded extent (H+2p, W+2p) and holds zeros outside the
 *     image; loop bounds are exclusive; output dims are
 *     floor((H + 2p - KH)/S) + 1.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int out_dim(int in, int k, int stride, int pad)
{
    int span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

int oracle_out_dim(int in, int k, int stride, int pad)
{
    return out_dim(in, k, stride, pad);
}

/* Eq. 2: MACs = N * Cin * Cout * Kh * Kw * Hout * Wout / g */
uint64_t oracle_macs(int N, int Cin, int Cout, int KH, int KW, int Hout,
                     int Wout, int groups)
{
    uint64_t num = (uint64_t)N * (uint64_t)Cin * (uint64_t)Cout *
                   (uint64_t)KH * (uint64_t)KW * (uint64_t)Hout * (uint64_t)Wout;
    return num / (uint64_t)groups;
}

/*
 * Seven nested loops n, oc, oh, ow, c, kh, kw.
 *   x [N][Cin][H][W], w [Cout][Cin/g][KH][KW], y [N][Cout][Hout][Wout]
 *   absacc (nullable): sum of |x*w| per output, for error-bound diagnostics.
 *   macs   (nullable): incremented once per innermost iteration, taps that
 *                      land on padding included (Eq. 2 counts them).
 *   threads: >1 splits the (n, oc) loop nest over that many OpenMP threads;
 *            each output is still one thread's plain serial sum.
 * Returns 0, or -1 on bad arguments.
 */
int oracle_conv2d_grouped(const double *x, const double *w, int N, int Cin,
                          int H, int W, int Cout, int KH, int KW, int stride,
                          int pad, int groups, double *y, double *absacc,
                          uint64_t *macs, int threads)
{
    if (!x || !w || !y) return -1;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || KH <= 0 ||
        KW <= 0 || stride <= 0 || pad < 0 || groups <= 0)
        return -1;
    if (Cin % groups || Cout % groups) return -1;
    const int CPG = Cin / groups, KPG = Cout / groups;
    const int Hout = out_dim(H, KH, stride, pad);
    const int Wout = out_dim(W, KW, stride, pad);
    if (Hout <= 0 || Wout <= 0) return -1;
    uint64_t total = 0;
    (void)threads;

#ifdef _OPENMP
#pragma omp parallel for collapse(2) reduction(+ : total) num_threads(threads > 0 ? threads : 1)
#endif
    for (int n = 0; n < N; ++n) {
        for (int oc = 0; oc < Cout; ++oc) {
            const int j = oc / KPG; /* group of this filter */
            for (int oh = 0; oh < Hout; ++oh) {
                for (int ow = 0; ow < Wout; ++ow) {
                    double s = 0.0, a = 0.0;
                    for (int c = 0; c < CPG; ++c) {
                        for (int kh = 0; kh < KH; ++kh) {
                            for (int kw = 0; kw < KW; ++kw) {
                                const int ih = oh * stride - pad + kh;
                                const int iw = ow * stride - pad + kw;
                                double xv = 0.0;
                                if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                                    xv = x[(((size_t)n * Cin + (size_t)j * CPG + c) * H + ih) * W + iw];
                                const double wv =
                                    w[(((size_t)oc * CPG + c) * KH + kh) * KW + kw];
                                s += xv * wv;
                                a += fabs(xv * wv);
                                ++total;
                            }
                        }
                    }
                    const size_t o = (((size_t)n * Cout + oc) * Hout + oh) * Wout + ow;
                    y[o] = s;
                    if (absacc) absacc[o] = a;
                }
            }
        }
    }
    if (macs) *macs = total;
    return 0;
}

/*
 * Same sum as above for a chosen subset of output channels only:
 * y_sel [N][n_sel][Hout][Wout] holds channel oc_sel[i] at position i.
 * Lets a full-batch layer be checked on sampled channels.
 */
int oracle_conv2d_grouped_channels(const double *x, const double *w, int N,
                                   int Cin, int H, int W, int Cout, int KH,
                                   int KW, int stride, int pad, int groups,
                                   const int *oc_sel, int n_sel, double *y_sel,
                                   int threads)
{
    if (!x || !w || !y_sel || !oc_sel || n_sel <= 0) return -1;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || KH <= 0 ||
        KW <= 0 || stride <= 0 || pad < 0 || groups <= 0)
        return -1;
    if (Cin % groups || Cout % groups) return -1;
    const int CPG = Cin / groups, KPG = Cout / groups;
    const int Hout = out_dim(H, KH, stride, pad);
    const int Wout = out_dim(W, KW, stride, pad);
    if (Hout <= 0 || Wout <= 0) return -1;
    for (int i = 0; i < n_sel; ++i)
        if (oc_sel[i] < 0 || oc_sel[i] >= Cout) return -1;
    (void)threads;

#ifdef _OPENMP
#pragma omp parallel for collapse(2) num_threads(threads > 0 ? threads : 1)
#endif
    for (int n = 0; n < N; ++n) {
        for (int i = 0; i < n_sel; ++i) {
            const int oc = oc_sel[i];
            const int j = oc / KPG;
            for (int oh = 0; oh < Hout; ++oh) {
                for (int ow = 0; ow < Wout; ++ow) {
                    double s = 0.0;
                    for (int c = 0; c < CPG; ++c)
                        for (int kh = 0; kh < KH; ++kh)
                            for (int kw = 0; kw < KW; ++kw) {
                                const int ih = oh * stride - pad + kh;
                                const int iw = ow * stride - pad + kw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                s += x[(((size_t)n * Cin + (size_t)j * CPG + c) * H + ih) * W + iw] *
                                     w[(((size_t)oc * CPG + c) * KH + kh) * KW + kw];
                            }
                    y_sel[(((size_t)n * n_sel + i) * Hout + oh) * Wout + ow] = s;
                }
            }
        }
    }
    return 0;
}

/*
 * Standard convolution S: every filter reads every input channel.  Written
 * without any group logic, over an explicitly zero-padded copy of the input,
 * so that it shares neither the channel mapping nor the border handling of
 * the grouped routine.  w [Cout][Cin][KH][KW].
 */
int oracle_conv2d_standard(const double *x, const double *w, int N, int Cin,
                           int H, int W, int Cout, int KH, int KW, int stride,
                           int pad, double *y)
{
    if (!x || !w || !y) return -1;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || KH <= 0 ||
        KW <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int Hp = H + 2 * pad, Wp = W + 2 * pad;
    const int Hout = out_dim(H, KH, stride, pad);
    const int Wout = out_dim(W, KW, stride, pad);
    if (Hout <= 0 || Wout <= 0) return -1;
    double *xp = (double *)calloc((size_t)N * Cin * Hp * Wp, sizeof(double));
    if (!xp) return -2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Cin; ++c)
            for (int h = 0; h < H; ++h)
                memcpy(xp + (((size_t)n * Cin + c) * Hp + h + pad) * Wp + pad,
                       x + (((size_t)n * Cin + c) * H + h) * W,
                       (size_t)W * sizeof(double));
    for (int n = 0; n < N; ++n)
        for (int oc = 0; oc < Cout; ++oc)
            for (int oh = 0; oh < Hout; ++oh)
                for (int ow = 0; ow < Wout; ++ow) {
                    double s = 0.0;
                    for (int c = 0; c < Cin; ++c)
                        for (int kh = 0; kh < KH; ++kh)
                            for (int kw = 0; kw < KW; ++kw)
                                s += xp[(((size_t)n * Cin + c) * Hp + oh * stride + kh) * Wp +
                                        ow * stride + kw] *
                                     w[(((size_t)oc * Cin + c) * KH + kh) * KW + kw];
                    y[(((size_t)n * Cout + oc) * Hout + oh) * Wout + ow] = s;
                }
    free(xp);
    return 0;
}

/* ------------------------------------------------------------------------
 * Algorithm 1, taken stage by stage.  KPG = Cout/g, CPG = Cin/g,
 * KT = KPG/T_O, CT = CPG/T_I (exact division required).
 * ---------------------------------------------------------------------- */

/* Stage 1.  W [Cout][CPG][KH][KW] -> W' [g][KT][CT][KH][KW][T_I][T_O] */
int oracle_alg1_pack_kernels(const double *w, int Cin, int Cout, int KH, int KW,
                             int groups, int T_I, int T_O, double *wp)
{
    if (!w || !wp || groups <= 0 || Cin % groups || Cout % groups) return -1;
    const int CPG = Cin / groups, KPG = Cout / groups;
    if (T_I <= 0 || T_O <= 0 || T_I > CPG || T_O > KPG) return -1; /* Eq. 1 */
    if (CPG % T_I || KPG % T_O) return -1;
    const int KT = KPG / T_O, CT = CPG / T_I;
    size_t o = 0;
    for (int j = 0; j < groups; ++j)
        for (int k = 0; k < KT; ++k)
            for (int c = 0; c < CT; ++c)
                for (int h = 0; h < KH; ++h)
                    for (int ww = 0; ww < KW; ++ww)
                        for (int ci = 0; ci < T_I; ++ci)
                            for (int co = 0; co < T_O; ++co) {
                                const int oc = j * KPG + k * T_O + co;
                                const int ic = c * T_I + ci;
                                wp[o++] = w[(((size_t)oc * CPG + ic) * KH + h) * KW + ww];
                            }
    return 0;
}

/* Stage 2.  X [N][Cin][H][W] -> X' [g][N][CT][H+2p][T_I][W+2p], zeros in the border */
int oracle_alg1_pack_inputs(const double *x, int N, int Cin, int H, int W,
                            int pad, int groups, int T_I, double *xp)
{
    if (!x || !xp || groups <= 0 || Cin % groups || pad < 0) return -1;
    const int CPG = Cin / groups;
    if (T_I <= 0 || T_I > CPG || CPG % T_I) return -1;
    const int CT = CPG / T_I, Hp = H + 2 * pad, Wp = W + 2 * pad;
    size_t o = 0;
    for (int j = 0; j < groups; ++j)
        for (int n = 0; n < N; ++n)
            for (int C = 0; C < CT; ++C)
                for (int h = 0; h < Hp; ++h)
                    for (int c = 0; c < T_I; ++c)
                        for (int ww = 0; ww < Wp; ++ww) {
                            const int ih = h - pad, iw = ww - pad;
                            const int ch = C * T_I + c + CPG * j;
                            double v = 0.0;
                            if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                                v = x[(((size_t)n * Cin + ch) * H + ih) * W + iw];
                            xp[o++] = v;
                        }
    return 0;
}

/* Stage 3.  Y' [g][N][KT][Hout][Wout][T_O] from W' and X'. */
int oracle_alg1_conv(const double *xp, const double *wp, int N, int Cin, int H,
                     int W, int Cout, int KH, int KW, int stride, int pad,
                     int groups, int T_I, int T_O, double *yp)
{
    if (!xp || !wp || !yp || groups <= 0 || Cin % groups || Cout % groups) return -1;
    const int CPG = Cin / groups, KPG = Cout / groups;
    if (T_I <= 0 || T_O <= 0 || CPG % T_I || KPG % T_O) return -1;
    const int KT = KPG / T_O, CT = CPG / T_I;
    const int Hp = H + 2 * pad, Wp = W + 2 * pad;
    const int Hout = out_dim(H, KH, stride, pad);
    const int Wout = out_dim(W, KW, stride, pad);
    if (Hout <= 0 || Wout <= 0) return -1;
    size_t o = 0;
    for (int j = 0; j < groups; ++j)
        for (int n = 0; n < N; ++n)
            for (int occ = 0; occ < KT; ++occ)
                for (int oh = 0; oh < Hout; ++oh)
                    for (int ow = 0; ow < Wout; ++ow)
                        for (int ocb = 0; ocb < T_O; ++ocb) {
                            double yv = 0.0;
                            for (int c = 0; c < CPG; ++c)
                                for (int kh = 0; kh < KH; ++kh)
                                    for (int kw = 0; kw < KW; ++kw) {
                                        /* X'[j][n][c/T_I][oh*S+kh][c%T_I][ow*S+kw] */
                                        const size_t xi =
                                            (((((size_t)j * N + n) * CT + c / T_I) * Hp +
                                              (oh * stride + kh)) * T_I + c % T_I) * Wp +
                                            (ow * stride + kw);
                                        /* W'[j][occ][c/T_I][kh][kw][c%T_I][ocb] */
                                        const size_t wi =
                                            ((((((size_t)j * KT + occ) * CT + c / T_I) * KH + kh) * KW +
                                              kw) * T_I + c % T_I) * T_O + ocb;
                                        yv += xp[xi] * wp[wi];
                                    }
                            yp[o++] = yv;
                        }
    return 0;
}

/*
 * Stage 3 as Section III-B / III-C schedule it on a CPU: the innermost T_O
 * filters of a tile are one vector (they are contiguous in W' and in Y'), the
 * input value is broadcast, and the (group, image) pairs are spread over the
 * cores.  TIMED BASELINE ONLY ("the paper's method on the host"): nothing is
 * checked against it.  Every output still sums its products in (c, kh, kw)
 * order, one multiply and one add each, so the result is bit-identical to
 * oracle_alg1_conv (pinned in the tests).  Same arguments as oracle_alg1_conv;
 * threads > 1 splits the (group, image) loop nest over OpenMP threads.
 */
#define ALG1_MAX_TO 64
#if defined(__x86_64__) && defined(__GNUC__) && !defined(__clang__)
__attribute__((target_clones("avx512f", "avx2", "default")))
#endif
int oracle_alg1_conv_vec(const double *xp, const double *wp, int N, int Cin, int H,
                         int W, int Cout, int KH, int KW, int stride, int pad,
                         int groups, int T_I, int T_O, double *yp, int threads)
{
    if (!xp || !wp || !yp || groups <= 0 || Cin % groups || Cout % groups) return -1;
    const int CPG = Cin / groups, KPG = Cout / groups;
    if (T_I <= 0 || T_O <= 0 || T_O > ALG1_MAX_TO || CPG % T_I || KPG % T_O) return -1;
    const int KT = KPG / T_O, CT = CPG / T_I;
    const int Hp = H + 2 * pad, Wp = W + 2 * pad;
    const int Hout = out_dim(H, KH, stride, pad);
    const int Wout = out_dim(W, KW, stride, pad);
    if (Hout <= 0 || Wout <= 0) return -1;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) num_threads(threads > 0 ? threads : 1)
#endif
    for (int j = 0; j < groups; ++j)
        for (int n = 0; n < N; ++n)
            for (int occ = 0; occ < KT; ++occ)
                for (int oh = 0; oh < Hout; ++oh)
                    for (int ow = 0; ow < Wout; ++ow) {
                        double acc[ALG1_MAX_TO];
                        for (int ocb = 0; ocb < T_O; ++ocb) acc[ocb] = 0.0;
                        for (int c = 0; c < CPG; ++c)
                            for (int kh = 0; kh < KH; ++kh)
                                for (int kw = 0; kw < KW; ++kw) {
                                    const double xv =
                                        xp[(((((size_t)j * N + n) * CT + c / T_I) * Hp + (oh * stride + kh)) * T_I +
                                            c % T_I) * Wp + (ow * stride + kw)];
                                    const double *wv =
                                        wp + ((((((size_t)j * KT + occ) * CT + c / T_I) * KH + kh) * KW + kw) * T_I +
                                              c % T_I) * T_O;
#pragma omp simd
                                    for (int ocb = 0; ocb < T_O; ++ocb) acc[ocb] += xv * wv[ocb];
                                }
                        double *out = yp + (((((size_t)j * N + n) * KT + occ) * Hout + oh) * Wout + ow) * T_O;
                        for (int ocb = 0; ocb < T_O; ++ocb) out[ocb] = acc[ocb];
                    }
    return 0;
}

/* Stage 4.  Y' [g][N][KT][Hout][Wout][T_O] -> Y [N][Cout][Hout][Wout] */
int oracle_alg1_unpack_outputs(const double *yp, int N, int Cout, int Hout,
                               int Wout, int groups, int T_O, double *y)
{
    if (!yp || !y || groups <= 0 || Cout % groups) return -1;
    const int KPG = Cout / groups;
    if (T_O <= 0 || KPG % T_O) return -1;
    const int KT = KPG / T_O;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Cout; ++c)
            for (int h = 0; h < Hout; ++h)
                for (int ww = 0; ww < Wout; ++ww) {
                    const int j = c / KPG;
                    const int occ = (c / T_O) % KT;
                    const int ocb = (c % T_O) % KPG;
                    y[(((size_t)n * Cout + c) * Hout + h) * Wout + ww] =
                        yp[(((((size_t)j * N + n) * KT + occ) * Hout + h) * Wout + ww) * T_O + ocb];
                }
    return 0;
}

/* ------------------------------------------------------------------------
 * Chain helpers.
 * ---------------------------------------------------------------------- */
void oracle_relu(const double *x, size_t count, double *y)
{
    for (size_t i = 0; i < count; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

void oracle_add(const double *a, const double *b, size_t count, double *y)
{
    for (size_t i = 0; i < count; ++i) y[i] = a[i] + b[i];
}

/* Max pooling over K x K windows; positions outside the image are ignored
 * (equivalent to -inf padding).  x [N][C][H][W] -> y [N][C][Hout][Wout]. */
int oracle_maxpool2d(const double *x, int N, int C, int H, int W, int K,
                     int stride, int pad, double *y)
{
    if (!x || !y || N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 ||
        stride <= 0 || pad < 0 || 2 * pad > K)
        return -1;
    const int Hout = out_dim(H, K, stride, pad);
    const int Wout = out_dim(W, K, stride, pad);
    if (Hout <= 0 || Wout <= 0) return -1;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < Hout; ++oh)
                for (int ow = 0; ow < Wout; ++ow) {
                    double m = -INFINITY;
                    for (int kh = 0; kh < K; ++kh)
                        for (int kw = 0; kw < K; ++kw) {
                            const int ih = oh * stride - pad + kh;
                            const int iw = ow * stride - pad + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const double v = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            if (v > m) m = v;
                        }
                    y[(((size_t)n * C + c) * Hout + oh) * Wout + ow] = m;
                }
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
