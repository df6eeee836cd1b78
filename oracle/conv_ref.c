/*
 * CPU oracle, numeric half.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may call, link or import this file.  It shares no code with the HIP
 * library.
 *
 * What it computes: the stored activation of one fused layer, written out from
 * its plain definition.  The paper's manager treats each operator output as the
 * unit it releases and regenerates (DELTA, Sec. 3, Assumption 1: every tensor is
 * the output of an operator; Sec. 5.5 names ConvForward, BNForward and
 * PoolingForward as the regenerated operators).  The layer itself is the
 * textbook one (He et al., ResNet v1):
 *
 *   z[n,p,q,k] = sum_{r,s,c} x[n, p*stride + r - pad, q*stride + s - pad, c] * w[k,r,s,c]
 *   u = gamma_k * (z - mean_k) / sqrt(var_k + eps) + beta_k      (frozen statistics)
 *   v = u + residual[n,p,q,k]                                    (if present)
 *   y = max(v, 0)                                                (if relu)
 *
 * Operands are taken at their storage precision (the exact fp32 or bf16 bit
 * patterns), all arithmetic is fp64, and y is rounded once, to nearest even,
 * to the storage type.  Loops are the naive seven-deep nest; OpenMP splits the
 * two outermost loops only.
 *
 * Pins (tests/test_oracle_numeric.py): 1x1 case equals a matrix product,
 * centre-tap identity, all-ones padding counts, linearity, stride subsampling,
 * BN identity and closed forms, bf16 rounding on hand-picked bit patterns.
 *
 * Backward of the same layer (oracle_conv_bn_act_bwd): the backward half of the
 * training iteration whose tensor accesses DELTA's planner follows (Sec. 3,
 * Assumptions 1-3: the backward pass reads the stored forward activations).  It is
 * the chain rule of the four lines above, written out; all in fp64, nothing rounded.
 * Pins (tests/test_oracle_backward.py): central finite differences of the forward
 * function, the adjoint identity <g, conv(x')> = <conv^T(g), x'>, the 1x1 case as
 * two matrix products, and the mask/scale factors on hand-made cases.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* bf16 bit pattern -> exact double */
static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bf16 bit pattern, one rounding, ties to even.  bf16 = 1 sign, 8 exponent,
 * 7 fraction bits: the spacing of representable values around v is 2^(e-7) with
 * e = floor(log2 |v|), and 2^-133 in the subnormal range (e < -126). */
uint16_t oracle_double_to_bf16(double v)
{
    uint32_t u;
    float f;
    if (isnan(v)) return 0x7FC0;
    if (isinf(v)) return v > 0 ? 0x7F80 : 0xFF80;
    if (v == 0.0) return signbit(v) ? 0x8000 : 0x0000;
    int e = ilogb(v);
    if (e < -126) e = -126;
    double ulp = ldexp(1.0, e - 7);
    double r = nearbyint(v / ulp) * ulp;      /* default rounding mode: nearest, ties to even */
    if (fabs(r) >= ldexp(1.0, 128)) return v > 0 ? 0x7F80 : 0xFF80;
    f = (float)r;                              /* exact: r has at most 8 significant bits */
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

double oracle_bf16_to_double(uint16_t b) { return bf16_to_double(b); }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double *widen(int dtype, const void *src, size_t n)
{
    double *d = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!d) return NULL;
    if (dtype == ORACLE_F32) {
        const float *s = (const float *)src;
        for (size_t i = 0; i < n; ++i) d[i] = (double)s[i];
    } else {
        const uint16_t *s = (const uint16_t *)src;
        for (size_t i = 0; i < n; ++i) d[i] = bf16_to_double(s[i]);
    }
    return d;
}

/*
 * One fused layer.  x: [N,H,W,Cin], w: [Cout,R,S,Cin], res: [N,P,Q,Cout] or NULL,
 * gamma/beta/mean/var: fp32 [Cout] (gamma == NULL means no batch-norm: u = z),
 * y: [N,P,Q,Cout] in the storage type, y64 (optional): the same values before
 * the final rounding.  Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_conv_bn_act(int dtype, const void *x, const void *w, const void *res,
                       const float *gamma, const float *beta, const float *mean,
                       const float *var, double eps,
                       int N, int H, int W, int Cin, int Cout, int R, int S,
                       int stride, int pad, int relu, void *y, double *y64)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || N < 0 || H <= 0 || W <= 0 ||
        Cin <= 0 || Cout <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
    if (P <= 0 || Q <= 0) return -1;
    const size_t nx = (size_t)N * H * W * Cin, nw = (size_t)Cout * R * S * Cin;
    const size_t ny = (size_t)N * P * Q * Cout;
    double *xd = widen(dtype, x, nx), *wd = widen(dtype, w, nw);
    double *rd = res ? widen(dtype, res, ny) : NULL;
    if (!xd || !wd || (res && !rd)) { free(xd); free(wd); free(rd); return -1; }

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < Cout; ++k) {
                    double z = 0.0;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * stride + r - pad;
                        if (h < 0 || h >= H) continue;          /* zero padding */
                        for (int s = 0; s < S; ++s) {
                            const int ww = q * stride + s - pad;
                            if (ww < 0 || ww >= W) continue;
                            const double *xp = xd + (((size_t)n * H + h) * W + ww) * Cin;
                            const double *wp = wd + (((size_t)k * R + r) * S + s) * Cin;
                            for (int c = 0; c < Cin; ++c) z += xp[c] * wp[c];
                        }
                    }
                    double u = z;
                    if (gamma)
                        u = (double)gamma[k] * (z - (double)mean[k]) /
                                sqrt((double)var[k] + eps) + (double)beta[k];
                    const size_t o = (((size_t)n * P + p) * Q + q) * Cout + k;
                    if (rd) u += rd[o];
                    if (relu && !(u > 0.0)) u = (u != u) ? u : 0.0;   /* NaN passes through */
                    if (y64) y64[o] = u;
                    if (dtype == ORACLE_F32) ((float *)y)[o] = (float)u;
                    else ((uint16_t *)y)[o] = oracle_double_to_bf16(u);
                }
    free(xd); free(wd); free(rd);
    return 0;
}

/* Max pooling (PoolingForward), window R x S, padding excluded from the maximum. */
int oracle_maxpool(int dtype, const void *x, int N, int H, int W, int C, int R, int S,
                   int stride, int pad, void *y)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || stride <= 0) return -1;
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (P <= 0 || Q <= 0) return -1;
    double *xd = widen(dtype, x, (size_t)N * H * W * C);
    if (!xd) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int c = 0; c < C; ++c) {
                    double m = -INFINITY;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            const int h = p * stride + r - pad, ww = q * stride + s - pad;
                            if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                            const double v = xd[(((size_t)n * H + h) * W + ww) * C + c];
                            if (v > m) m = v;
                        }
                    const size_t o = (((size_t)n * P + p) * Q + q) * C + c;
                    if (dtype == ORACLE_F32) ((float *)y)[o] = (float)m;
                    else ((uint16_t *)y)[o] = oracle_double_to_bf16(m);
                }
    free(xd);
    return 0;
}

/* Global average pooling over H x W. */
int oracle_avgpool(int dtype, const void *x, int N, int H, int W, int C, void *y)
{
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    double *xd = widen(dtype, x, (size_t)N * H * W * C);
    if (!xd) return -1;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double a = 0.0;
            for (int i = 0; i < H * W; ++i) a += xd[((size_t)n * H * W + i) * C + c];
            a /= (double)(H * W);
            if (dtype == ORACLE_F32) ((float *)y)[(size_t)n * C + c] = (float)a;
            else ((uint16_t *)y)[(size_t)n * C + c] = oracle_double_to_bf16(a);
        }
    free(xd);
    return 0;
}

/*
 * Backward of one fused layer with frozen batch-norm statistics.  Given gy = dL/dy:
 *
 *   gpre[n,p,q,k] = gy[n,p,q,k] * [y[n,p,q,k] > 0]     (if relu; the subgradient at 0 is 0;
 *                                                        y is the STORED forward output)
 *                 = gy[n,p,q,k]                         (otherwise)
 *   dL/dres = gpre                                      (the residual enters v with weight 1)
 *   gz[n,p,q,k] = gpre[n,p,q,k] * gamma_k / sqrt(var_k + eps)          (gz = gpre without BN)
 *   gx[n,h,w,c]  = sum over (p,q,k,r,s) with h = p*stride + r - pad, w = q*stride + s - pad
 *                  of gz[n,p,q,k] * w[k,r,s,c]
 *   gw[k,r,s,c]  = sum over (n,p,q) with that (h,w) inside the image of gz[n,p,q,k] * x[n,h,w,c]
 *
 * x, w, y, gy at storage precision; gx64 [N,H,W,Cin], gw64 [Cout,R,S,Cin], gpre64 [N,P,Q,Cout]
 * in fp64 (any of the three may be NULL).  gamma == NULL: no batch-norm.  y may be NULL when
 * relu == 0.  Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_conv_bn_act_bwd(int dtype, const void *x, const void *w, const void *y, const void *gy,
                           const float *gamma, const float *var, double eps,
                           int N, int H, int W, int Cin, int Cout, int R, int S,
                           int stride, int pad, int relu,
                           double *gx64, double *gw64, double *gpre64)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || N < 0 || H <= 0 || W <= 0 ||
        Cin <= 0 || Cout <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0 || !gy || (relu && !y))
        return -1;
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
    if (P <= 0 || Q <= 0) return -1;
    const size_t nx = (size_t)N * H * W * Cin, nw = (size_t)Cout * R * S * Cin;
    const size_t ny = (size_t)N * P * Q * Cout;
    double *xd = widen(dtype, x, nx), *wd = widen(dtype, w, nw), *gd = widen(dtype, gy, ny);
    double *yd = relu ? widen(dtype, y, ny) : NULL;
    double *gz = (double *)malloc((ny ? ny : 1) * sizeof(double));
    if (!xd || !wd || !gd || (relu && !yd) || !gz) { free(xd); free(wd); free(gd); free(yd); free(gz); return -1; }

    for (size_t o = 0; o < ny; ++o) {
        const int k = (int)(o % (size_t)Cout);
        double g = gd[o];
        if (relu && !(yd[o] > 0.0)) g = 0.0;
        if (gpre64) gpre64[o] = g;
        if (gamma) g *= (double)gamma[k] / sqrt((double)var[k] + eps);
        gz[o] = g;
    }
    if (gx64) {
        memset(gx64, 0, nx * sizeof(double));
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n)                      /* images are independent */
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q)
                    for (int k = 0; k < Cout; ++k) {
                        const double g = gz[(((size_t)n * P + p) * Q + q) * Cout + k];
                        for (int r = 0; r < R; ++r) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int ww = q * stride + s - pad;
                                if (ww < 0 || ww >= W) continue;
                                double *gp = gx64 + (((size_t)n * H + h) * W + ww) * Cin;
                                const double *wp = wd + (((size_t)k * R + r) * S + s) * Cin;
                                for (int c = 0; c < Cin; ++c) gp[c] += g * wp[c];
                            }
                        }
                    }
    }
    if (gw64) {
        memset(gw64, 0, nw * sizeof(double));
#pragma omp parallel for schedule(static)
        for (int k = 0; k < Cout; ++k)                   /* output channels are independent */
            for (int n = 0; n < N; ++n)
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q) {
                        const double g = gz[(((size_t)n * P + p) * Q + q) * Cout + k];
                        for (int r = 0; r < R; ++r) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int ww = q * stride + s - pad;
                                if (ww < 0 || ww >= W) continue;
                                const double *xp = xd + (((size_t)n * H + h) * W + ww) * Cin;
                                double *gp = gw64 + (((size_t)k * R + r) * S + s) * Cin;
                                for (int c = 0; c < Cin; ++c) gp[c] += g * xp[c];
                            }
                        }
                    }
    }
    free(xd); free(wd); free(gd); free(yd); free(gz);
    return 0;
}
