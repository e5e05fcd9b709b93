/*
 * CPU oracle for the group-wise int8 quantized Winograd F(m,3) convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct loops written from
 * the paper; nothing in the product path may call into this file, and this
 * file shares no code, header, table or constant with the HIP kernels.
 *
 * What each function follows:
 *   oracle_direct_conv_f64      left side of the Winograd identity (Section
 *                               "Winograd convolution", first equation): the
 *                               3x3 stride-1 zero-pad-1 cross-correlation.
 *   oracle_winograd_f64         the four un-quantized stages W=GwG^T, X=B^T x B,
 *                               Y=W.X, y=A^T Y A of the same section, in fp64,
 *                               with any supplied matrices.
 *   oracle_weight_transform_quant   W=GwG^T (offline stage) followed by the
 *                               uniform symmetric quantizer (Section "Related
 *                               work", quantizer equation) applied per group of
 *                               `g` input channels.
 *   oracle_input_transform_quant    X=B^T x B followed by the same quantizer
 *                               with dynamic abs-max scales (Section "Learnable
 *                               Winograd transform scales", last sentence
 *                               before "Random Gaussian noise ...").
 *   oracle_contract             the quantized Hadamard product summed over input
 *                               channels, Y ~ s_qW s_qX Q(W) Q(X) (second of the
 *                               three quantized-stage equations), exact int32
 *                               per group, rescaled in fp64.
 *   oracle_output_transform     y=A^T Y A plus bias, fp64.
 *
 * Readings the paper leaves open (all stated again in the design notes):
 *   - groups run along input channels, contiguous, one scale per
 *     (tap, tile, group) for activations and (tap, out-channel, group) for
 *     weights;
 *   - symmetric int8, range [-127,127], scale s = absmax/127;
 *   - the quotient x/s is evaluated as x*r with r = 127/absmax (one rounded
 *     division per group, one rounded multiply per element), then rounded to
 *     nearest with ties to even;
 *   - groups whose absmax is below 127*FLT_MIN quantize to all-zero, scale 0;
 *   - the fp32 transforms are fused-multiply-add chains, left factor first,
 *     inner index ascending, starting from +0;
 *   - tiles that overhang the image read zeros and drop the outputs that fall
 *     outside.
 *
 * Layouts (all dense, row-major, last index fastest):
 *   x   [N][H][W][Cin]  fp32          w    [Cout][Cin][3][3] fp32
 *   Xq  [n*n][T][Cin]   int8          sX   [n*n][T][Cin/g]   fp32
 *   Wq  [n*n][Cout][Cin] int8         sW   [n*n][Cin/g][Cout] fp32
 *   P   [n*n][T][Cin/g][Cout] int32   M    [n*n][T][Cout]    fp64
 *   y   [N][H][W][Cout]
 * with n = m+2, tile grid TH=ceil(H/m), TW=ceil(W/m), T=N*TH*TW and tile id
 * (b*TH+th)*TW+tw; tap id t = i*n+j.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MAXN 8

static int cdiv(int a, int b) { return (a + b - 1) / b; }

/* ------------------------------------------------------------------ O-A */
void oracle_direct_conv_f64(const float *x, const float *w, const float *bias,
                            double *y, int N, int H, int W, int Cin, int Cout)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int h = 0; h < H; ++h)
            for (int q = 0; q < W; ++q)
                for (int o = 0; o < Cout; ++o) {
                    double acc = bias ? (double)bias[o] : 0.0;
                    for (int u = 0; u < 3; ++u) {
                        int hh = h + u - 1;
                        if (hh < 0 || hh >= H) continue;
                        for (int v = 0; v < 3; ++v) {
                            int ww = q + v - 1;
                            if (ww < 0 || ww >= W) continue;
                            const float *xp = x + (((size_t)b * H + hh) * W + ww) * Cin;
                            const float *wp = w + (size_t)o * Cin * 9 + u * 3 + v;
                            for (int c = 0; c < Cin; ++c)
                                acc += (double)xp[c] * (double)wp[(size_t)c * 9];
                        }
                    }
                    y[(((size_t)b * H + h) * W + q) * Cout + o] = acc;
                }
}

/* ------------------------------------------------------------------ O-B */
/* BT is n x n, G is n x 3, AT is m x n, all fp64 row-major. */
void oracle_winograd_f64(const float *x, const float *w, const float *bias,
                         const double *BT, const double *G, const double *AT,
                         double *y, int N, int H, int W, int Cin, int Cout, int m)
{
    const int n = m + 2, TH = cdiv(H, m), TW = cdiv(W, m);
    double *Wt = (double *)malloc((size_t)Cout * Cin * n * n * sizeof(double));
    for (int o = 0; o < Cout; ++o)
        for (int c = 0; c < Cin; ++c) {
            const float *k = w + ((size_t)o * Cin + c) * 9;
            double U[MAXN][3];
            for (int i = 0; i < n; ++i)
                for (int b = 0; b < 3; ++b) {
                    double s = 0.0;
                    for (int a = 0; a < 3; ++a) s += G[i * 3 + a] * (double)k[a * 3 + b];
                    U[i][b] = s;
                }
            double *dst = Wt + ((size_t)o * Cin + c) * n * n;
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    double s = 0.0;
                    for (int a = 0; a < 3; ++a) s += U[i][a] * G[j * 3 + a];
                    dst[i * n + j] = s;
                }
        }
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int th = 0; th < TH; ++th) {
            double *X = (double *)malloc((size_t)Cin * n * n * sizeof(double));
            for (int tw = 0; tw < TW; ++tw) {
                for (int c = 0; c < Cin; ++c) {
                    double d[MAXN][MAXN], Tm[MAXN][MAXN];
                    for (int i = 0; i < n; ++i)
                        for (int j = 0; j < n; ++j) {
                            int hh = th * m - 1 + i, ww = tw * m - 1 + j;
                            d[i][j] = (hh >= 0 && hh < H && ww >= 0 && ww < W)
                                ? (double)x[(((size_t)b * H + hh) * W + ww) * Cin + c] : 0.0;
                        }
                    for (int i = 0; i < n; ++i)
                        for (int j = 0; j < n; ++j) {
                            double s = 0.0;
                            for (int k = 0; k < n; ++k) s += BT[i * n + k] * d[k][j];
                            Tm[i][j] = s;
                        }
                    for (int i = 0; i < n; ++i)
                        for (int j = 0; j < n; ++j) {
                            double s = 0.0;
                            for (int k = 0; k < n; ++k) s += Tm[i][k] * BT[j * n + k];
                            X[(size_t)c * n * n + i * n + j] = s;
                        }
                }
                for (int o = 0; o < Cout; ++o) {
                    double Y[MAXN][MAXN];
                    for (int t = 0; t < n * n; ++t) {
                        double s = 0.0;
                        for (int c = 0; c < Cin; ++c)
                            s += Wt[((size_t)o * Cin + c) * n * n + t] * X[(size_t)c * n * n + t];
                        Y[t / n][t % n] = s;
                    }
                    for (int a = 0; a < m; ++a)
                        for (int e = 0; e < m; ++e) {
                            int hh = th * m + a, ww = tw * m + e;
                            if (hh >= H || ww >= W) continue;
                            double s = 0.0;
                            for (int i = 0; i < n; ++i)
                                for (int j = 0; j < n; ++j)
                                    s += AT[a * n + i] * Y[i][j] * AT[e * n + j];
                            y[(((size_t)b * H + hh) * W + ww) * Cout + o] =
                                s + (bias ? (double)bias[o] : 0.0);
                        }
                }
            }
            free(X);
        }
    free(Wt);
}

/* ------------------------------------------------------- the quantizer */
/* Uniform symmetric quantizer of one group with codes in [-qmax, qmax]
 * (qmax = 127 for 8 bits, 7 for 4 bits): `count` values at stride `vs` ->
 * `count` codes at stride `qs`; returns the group's scale a/qmax. */
static float quantize_group_q(const float *v, size_t vs, int count, int8_t *q, size_t qs, float qmax)
{
    float a = 0.0f;
    for (int k = 0; k < count; ++k) {
        float t = fabsf(v[k * vs]);
        if (t > a) a = t;
    }
    if (!(a >= qmax * FLT_MIN)) {
        for (int k = 0; k < count; ++k) q[k * qs] = 0;
        return 0.0f;
    }
    const float s = a / qmax;
    const float r = qmax / a;
    for (int k = 0; k < count; ++k) {
        float z = rintf(v[k * vs] * r);
        if (z > qmax) z = qmax;
        if (z < -qmax) z = -qmax;
        q[k * qs] = (int8_t)z;
    }
    return s;
}

static float quantize_group(const float *v, size_t vs, int count, int8_t *q, size_t qs)
{
    return quantize_group_q(v, vs, count, q, qs, 127.0f);
}

/* largest code of a `bits`-wide symmetric quantizer */
static float qmax_of(int bits) { return (float)((1 << (bits - 1)) - 1); }

/* exported for the quantizer's own tests */
float oracle_quantize_group(const float *v, int count, int8_t *q)
{
    return quantize_group(v, 1, count, q, 1);
}

float oracle_quantize_group_bits(const float *v, int count, int bits, int8_t *q)
{
    return quantize_group_q(v, 1, count, q, 1, qmax_of(bits));
}

/* The quantizer equation of Section "Related work" read to the letter, x_int =
 * clamp(round(x / s)) with s = a / 127 and one IEEE division per element.  Not used by any
 * pipeline here: it only measures how far the reading x * (127 / a) of quantize_group_q is
 * from the text (the two differ where x / s falls within a rounding error of a half-integer). */
float oracle_quantize_group_literal(const float *v, int count, int8_t *q)
{
    float a = 0.0f;
    for (int k = 0; k < count; ++k) {
        float t = fabsf(v[k]);
        if (t > a) a = t;
    }
    if (!(a >= 127.0f * FLT_MIN)) {
        for (int k = 0; k < count; ++k) q[k] = 0;
        return 0.0f;
    }
    const float s = a / 127.0f;
    for (int k = 0; k < count; ++k) {
        float z = rintf(v[k] / s);
        if (z > 127.0f) z = 127.0f;
        if (z < -127.0f) z = -127.0f;
        q[k] = (int8_t)z;
    }
    return s;
}

/* -------------------------------------------------- stage 4 (offline) */
void oracle_weight_transform_quant(const float *w, const float *G, int Cin, int Cout,
                                   int m, int g, int8_t *Wq, float *sW, float *Wf)
{
    const int n = m + 2, n2 = n * n, groups = Cin / g;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Cout; ++o) {
        float *buf = (float *)malloc((size_t)Cin * n2 * sizeof(float));
        for (int c = 0; c < Cin; ++c) {
            const float *k = w + ((size_t)o * Cin + c) * 9;
            float U[MAXN][3];
            for (int i = 0; i < n; ++i)
                for (int b = 0; b < 3; ++b) {
                    float acc = 0.0f;
                    for (int a = 0; a < 3; ++a) acc = fmaf(G[i * 3 + a], k[a * 3 + b], acc);
                    U[i][b] = acc;
                }
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    float acc = 0.0f;
                    for (int a = 0; a < 3; ++a) acc = fmaf(U[i][a], G[j * 3 + a], acc);
                    buf[(size_t)(i * n + j) * Cin + c] = acc;
                }
        }
        for (int t = 0; t < n2; ++t) {
            if (Wf)
                memcpy(Wf + ((size_t)t * Cout + o) * Cin, buf + (size_t)t * Cin,
                       (size_t)Cin * sizeof(float));
            for (int gi = 0; gi < groups; ++gi)
                sW[((size_t)t * groups + gi) * Cout + o] =
                    quantize_group(buf + (size_t)t * Cin + gi * g, 1, g,
                                   Wq + ((size_t)t * Cout + o) * Cin + gi * g, 1);
        }
        free(buf);
    }
}

/* ------------------------------------------------------------ stage 1 */
void oracle_input_transform_quant(const float *x, const float *BT, int N, int H, int W,
                                  int Cin, int m, int g, int8_t *Xq, float *sX, float *Xf)
{
    const int n = m + 2, n2 = n * n, groups = Cin / g;
    const int TH = cdiv(H, m), TW = cdiv(W, m);
    const size_t T = (size_t)N * TH * TW;
#pragma omp parallel for schedule(static)
    for (long tau = 0; tau < (long)T; ++tau) {
        const int tw = (int)(tau % TW), th = (int)((tau / TW) % TH), b = (int)(tau / ((long)TW * TH));
        float *buf = (float *)malloc((size_t)Cin * n2 * sizeof(float));
        for (int c = 0; c < Cin; ++c) {
            float d[MAXN][MAXN], Tm[MAXN][MAXN];
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    int hh = th * m - 1 + i, ww = tw * m - 1 + j;
                    d[i][j] = (hh >= 0 && hh < H && ww >= 0 && ww < W)
                        ? x[(((size_t)b * H + hh) * W + ww) * Cin + c] : 0.0f;
                }
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    float acc = 0.0f;
                    for (int k = 0; k < n; ++k) acc = fmaf(BT[i * n + k], d[k][j], acc);
                    Tm[i][j] = acc;
                }
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j) {
                    float acc = 0.0f;
                    for (int k = 0; k < n; ++k) acc = fmaf(Tm[i][k], BT[j * n + k], acc);
                    buf[(size_t)(i * n + j) * Cin + c] = acc;
                }
        }
        for (int t = 0; t < n2; ++t) {
            if (Xf)
                memcpy(Xf + ((size_t)t * T + tau) * Cin, buf + (size_t)t * Cin,
                       (size_t)Cin * sizeof(float));
            for (int gi = 0; gi < groups; ++gi)
                sX[((size_t)t * T + tau) * groups + gi] =
                    quantize_group(buf + (size_t)t * Cin + gi * g, 1, g,
                                   Xq + ((size_t)t * T + tau) * Cin + gi * g, 1);
        }
        free(buf);
    }
}

/* ------------------------------------------------------------ stage 2 */
/* P may be NULL.  M is [n2][T][Cout] fp64. */
void oracle_contract(const int8_t *Xq, const float *sX, const int8_t *Wq, const float *sW,
                     long T, int Cin, int Cout, int n2, int g, int32_t *P, double *M)
{
    const int groups = Cin / g;
#pragma omp parallel for collapse(2) schedule(static)
    for (int t = 0; t < n2; ++t)
        for (long tau = 0; tau < T; ++tau) {
            const int8_t *xr = Xq + ((size_t)t * T + tau) * Cin;
            for (int o = 0; o < Cout; ++o) {
                const int8_t *wr = Wq + ((size_t)t * Cout + o) * Cin;
                double acc = 0.0;
                for (int gi = 0; gi < groups; ++gi) {
                    int32_t p = 0;
                    for (int c = gi * g; c < (gi + 1) * g; ++c)
                        p += (int32_t)xr[c] * (int32_t)wr[c];
                    if (P) P[(((size_t)t * T + tau) * groups + gi) * Cout + o] = p;
                    acc += (double)p * (double)sX[((size_t)t * T + tau) * groups + gi]
                                     * (double)sW[((size_t)t * groups + gi) * Cout + o];
                }
                M[((size_t)t * T + tau) * Cout + o] = acc;
            }
        }
}

/* ------------------------------------------------------------ stage 3 */
/* AT is m x n fp32 (promoted to fp64).  y64 and y32 may each be NULL. */
void oracle_output_transform(const double *M, const float *AT, const float *bias,
                             int N, int H, int W, int Cout, int m, double *y64, float *y32)
{
    const int n = m + 2, TH = cdiv(H, m), TW = cdiv(W, m);
    const size_t T = (size_t)N * TH * TW;
#pragma omp parallel for schedule(static)
    for (long tau = 0; tau < (long)T; ++tau) {
        const int tw = (int)(tau % TW), th = (int)((tau / TW) % TH), b = (int)(tau / ((long)TW * TH));
        for (int o = 0; o < Cout; ++o)
            for (int a = 0; a < m; ++a)
                for (int e = 0; e < m; ++e) {
                    int hh = th * m + a, ww = tw * m + e;
                    if (hh >= H || ww >= W) continue;
                    double s = 0.0;
                    for (int i = 0; i < n; ++i)
                        for (int j = 0; j < n; ++j)
                            s += (double)AT[a * n + i]
                               * M[((size_t)(i * n + j) * T + tau) * Cout + o]
                               * (double)AT[e * n + j];
                    if (bias) s += (double)bias[o];
                    size_t idx = (((size_t)b * H + hh) * W + ww) * Cout + o;
                    if (y64) y64[idx] = s;
                    if (y32) y32[idx] = (float)s;
                }
    }
}

/* brute-force integer contraction with a different loop nest, for the
 * self-check of oracle_contract on tiny shapes: P2[t][tau][gi][o]. */
void oracle_contract_bruteforce(const int8_t *Xq, const int8_t *Wq, long T, int Cin,
                                int Cout, int n2, int g, int64_t *P2)
{
    const int groups = Cin / g;
    memset(P2, 0, (size_t)n2 * T * groups * Cout * sizeof(int64_t));
    for (int c = 0; c < Cin; ++c)
        for (int o = 0; o < Cout; ++o)
            for (long tau = 0; tau < T; ++tau)
                for (int t = 0; t < n2; ++t)
                    P2[(((size_t)t * T + tau) * groups + c / g) * Cout + o] +=
                        (int64_t)Xq[((size_t)t * T + tau) * Cin + c] *
                        (int64_t)Wq[((size_t)t * Cout + o) * Cin + c];
}

/* ======================================================================
 * The comparison point of the paper's runtime section ("Runtime
 * improvements": group-wise quantized STANDARD convolution layers): the same
 * 3x3 stride-1 zero-pad-1 convolution with the same quantizer, but without
 * the Winograd transforms.  Reading (the paper gives no formula for it):
 * groups run along input channels as in the Winograd path; activations get
 * one dynamic scale per (pixel, group), weights one scale per
 * (filter tap, out-channel, group); every (tap, group) int32 dot product is
 * rescaled by its two scales and summed:
 *   y[b,h,w,o] = bias[o] + sum_{u,v} sum_G  P * sx[pixel(h+u-1,w+v-1)][G] * sw[u,v][G][o],
 *   P = sum_{c in G} xq[pixel][c] * wq[u,v][o][c]          (exact int32).
 * Layouts: xq [N*H*W][Cin] int8, sx [N*H*W][Cin/g] fp32,
 *          wq [9][Cout][Cin] int8 (tap t = u*3+v), sw [9][Cin/g][Cout] fp32.
 * ====================================================================== */
void oracle_quantize_pixels(const float *x, long P, int Cin, int g, int8_t *xq, float *sx)
{
    const int groups = Cin / g;
#pragma omp parallel for schedule(static)
    for (long p = 0; p < P; ++p)
        for (int gi = 0; gi < groups; ++gi)
            sx[p * groups + gi] = quantize_group(x + (size_t)p * Cin + (size_t)gi * g, 1, g,
                                                 xq + (size_t)p * Cin + (size_t)gi * g, 1);
}

/* `bits` = width of the weight codes: 8 (W8A8) or 4 (the W4A8 rows of the paper's tables:
 * the same symmetric abs-max quantizer with codes in [-7, 7]; activations stay 8-bit). */
void oracle_quantize_filters_bits(const float *w, int Cin, int Cout, int g, int bits, int8_t *wq,
                                  float *sw)
{
    const int groups = Cin / g;
    const float qmax = qmax_of(bits);
    for (int t = 0; t < 9; ++t)
        for (int o = 0; o < Cout; ++o)
            for (int gi = 0; gi < groups; ++gi)
                sw[((size_t)t * groups + gi) * Cout + o] =
                    quantize_group_q(w + ((size_t)o * Cin + (size_t)gi * g) * 9 + t, 9, g,
                                     wq + ((size_t)t * Cout + o) * Cin + (size_t)gi * g, 1, qmax);
}

void oracle_quantize_filters(const float *w, int Cin, int Cout, int g, int8_t *wq, float *sw)
{
    oracle_quantize_filters_bits(w, Cin, Cout, g, 8, wq, sw);
}

/* y64 and y32 may each be NULL. */
void oracle_direct_qconv(const int8_t *xq, const float *sx, const int8_t *wq, const float *sw,
                         const float *bias, int N, int H, int W, int Cin, int Cout, int g,
                         double *y64, float *y32)
{
    const int groups = Cin / g;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int h = 0; h < H; ++h)
            for (int q = 0; q < W; ++q)
                for (int o = 0; o < Cout; ++o) {
                    double acc = bias ? (double)bias[o] : 0.0;
                    for (int u = 0; u < 3; ++u) {
                        const int hh = h + u - 1;
                        if (hh < 0 || hh >= H) continue;
                        for (int v = 0; v < 3; ++v) {
                            const int ww = q + v - 1;
                            if (ww < 0 || ww >= W) continue;
                            const size_t pix = ((size_t)b * H + hh) * W + ww;
                            const int t = u * 3 + v;
                            const int8_t *xr = xq + pix * Cin;
                            const int8_t *wr = wq + ((size_t)t * Cout + o) * Cin;
                            for (int gi = 0; gi < groups; ++gi) {
                                int32_t p = 0;
                                for (int c = gi * g; c < (gi + 1) * g; ++c)
                                    p += (int32_t)xr[c] * (int32_t)wr[c];
                                acc += (double)p * (double)sx[pix * groups + gi]
                                                 * (double)sw[((size_t)t * groups + gi) * Cout + o];
                            }
                        }
                    }
                    const size_t idx = (((size_t)b * H + h) * W + q) * Cout + o;
                    if (y64) y64[idx] = acc;
                    if (y32) y32[idx] = (float)acc;
                }
}

/* ======================================================================
 * Group-wise quantized linear layer y = x W^T + bias (the paper applies the
 * same group-wise quantization to all linear layers and to the attention
 * matrix products, Section "Experiments", first paragraph): rows of x
 * [R][Cin] get one dynamic scale per (row, group) - oracle_quantize_pixels
 * with P = R - and the weight matrix W [Cout][Cin] one scale per
 * (output row, group):  y[r][o] = bias[o] + sum_G P * sx[r][G] * sw[G][o].
 * Layouts: wq [Cout][Cin] int8, sw [Cin/g][Cout] fp32.
 * ====================================================================== */
void oracle_quantize_weight_rows_bits(const float *w, int Cin, int Cout, int g, int bits,
                                      int8_t *wq, float *sw)
{
    const int groups = Cin / g;
    const float qmax = qmax_of(bits);
    for (int o = 0; o < Cout; ++o)
        for (int gi = 0; gi < groups; ++gi)
            sw[(size_t)gi * Cout + o] =
                quantize_group_q(w + (size_t)o * Cin + (size_t)gi * g, 1, g,
                                 wq + (size_t)o * Cin + (size_t)gi * g, 1, qmax);
}

void oracle_quantize_weight_rows(const float *w, int Cin, int Cout, int g, int8_t *wq, float *sw)
{
    oracle_quantize_weight_rows_bits(w, Cin, Cout, g, 8, wq, sw);
}

/* y64 and y32 may each be NULL. */
void oracle_linear_q(const int8_t *xq, const float *sx, const int8_t *wq, const float *sw,
                     const float *bias, long R, int Cin, int Cout, int g, double *y64, float *y32)
{
    const int groups = Cin / g;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < R; ++r)
        for (int o = 0; o < Cout; ++o) {
            double acc = bias ? (double)bias[o] : 0.0;
            for (int gi = 0; gi < groups; ++gi) {
                int32_t p = 0;
                for (int c = gi * g; c < (gi + 1) * g; ++c)
                    p += (int32_t)xq[(size_t)r * Cin + c] * (int32_t)wq[(size_t)o * Cin + c];
                acc += (double)p * (double)sx[(size_t)r * groups + gi] * (double)sw[(size_t)gi * Cout + o];
            }
            if (y64) y64[(size_t)r * Cout + o] = acc;
            if (y32) y32[(size_t)r * Cout + o] = (float)acc;
        }
}
