/*
 * CPU checker for the fused block  conv -> per-channel affine -> (+ residual) -> (ReLU)
 * and its analytic backward.  TEST INFRASTRUCTURE ONLY: it is called by the tests, by the
 * smoke check and by the benchmark's "cpu_baseline" leg, never by the product path, and it
 * shares no code with the GPU kernels.
 *
 * The paper replaces step 1 (model forward pass) and step 3 (model backward pass) of the
 * training loop by compiled code (section "SOL principle", the four atomic steps of the
 * training loop; listing "training loop") and keeps step 2, an L1 loss, in the framework.
 * It prints no formulas; what is computed here is the textbook definition of each of
 * those steps for one ResNet-50-style block, written as plain direct loops in fp64:
 *
 *   forward   z[n,co,ho,wo] = sum_{ci,kh,kw} x[n,ci,ho*s-p+kh,wo*s-p+kw] * w[co,ci,kh,kw]
 *             (taps outside the image contribute nothing; cross-correlation, no bias)
 *             v = scale[co]*z + shift[co] (+ r[n,co,ho,wo]);   y = relu ? max(v,0) : v
 *   loss      L = mean |y - t|,   dy = sign(y - t) / numel,   sign(0) = 0
 *   backward  g = relu ? (y > 0 ? dy : 0) : dy          dres = g
 *             dshift[co] = sum g       dscale[co] = sum g*z
 *             dx[n,ci,hi,wi] += g*scale[co]*w[co,ci,kh,kw]
 *             dw[co,ci,kh,kw] += g*scale[co]*x[n,ci,hi,wi]          (in-bounds taps only)
 *
 * Layout: activations [N][C][H][W], weights [C_out][C_in][KH][KW], all double.
 * There is no blocking, no vector intrinsics and no reordering beyond "which outermost
 * independent loop the OpenMP threads split".
 *
 * Pins (tests/test_oracle_*.py): closed forms on all-ones inputs, centre-delta weights,
 * 1x1 convolution == matrix product (numpy), stride-2 == subsampled stride-1, linearity,
 * central finite differences and adjoint identities for dx/dW/dscale/dshift, the ReLU
 * invariant, an independent library convolution + autograd in float64, hand-picked
 * bfloat16 rounding cases.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int N, H, W, C_in, C_out, KH, KW, stride, pad, relu;
} orc_desc;

static int out_h(const orc_desc* d) { return (d->H + 2 * d->pad - d->KH) / d->stride + 1; }
static int out_w(const orc_desc* d) { return (d->W + 2 * d->pad - d->KW) / d->stride + 1; }

int orc_out_h(const orc_desc* d) { return out_h(d); }
int orc_out_w(const orc_desc* d) { return out_w(d); }

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

double orc_now(void) {
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return (double)ts.tv_sec + 1e-9 * (double)ts.tv_nsec;
}

#define X_AT(n, c, h, w_) x[(((size_t)(n) * d->C_in + (c)) * d->H + (h)) * d->W + (w_)]
#define W_AT(co, ci, kh, kw) w[(((size_t)(co) * d->C_in + (ci)) * d->KH + (kh)) * d->KW + (kw)]
#define O_IDX(n, co, ho, wo) ((((size_t)(n) * d->C_out + (co)) * Ho + (ho)) * Wo + (wo))

/* Plain convolution (cross-correlation), the seven loops n, co, ho, wo, ci, kh, kw. */
void orc_conv(const orc_desc* d, const double* x, const double* w, double* z) {
    const int Ho = out_h(d), Wo = out_w(d);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int co = 0; co < d->C_out; ++co)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    double acc = 0.0;
                    for (int ci = 0; ci < d->C_in; ++ci)
                        for (int kh = 0; kh < d->KH; ++kh)
                            for (int kw = 0; kw < d->KW; ++kw) {
                                const int hi = ho * d->stride - d->pad + kh;
                                const int wi = wo * d->stride - d->pad + kw;
                                if (hi < 0 || hi >= d->H || wi < 0 || wi >= d->W) continue;
                                acc += X_AT(n, ci, hi, wi) * W_AT(co, ci, kh, kw);
                            }
                    z[O_IDX(n, co, ho, wo)] = acc;
                }
}

/* Forward of the block.  res may be NULL; z_out (the raw convolution) may be NULL. */
void orc_block_fwd(const orc_desc* d, const double* x, const double* w, const double* scale,
                   const double* shift, const double* res, double* z_out, double* y) {
    const int Ho = out_h(d), Wo = out_w(d);
    const size_t total = (size_t)d->N * d->C_out * Ho * Wo;
    double* z = z_out ? z_out : (double*)malloc(total * sizeof(double));
    orc_conv(d, x, w, z);
    for (int n = 0; n < d->N; ++n)
        for (int co = 0; co < d->C_out; ++co)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    const size_t i = O_IDX(n, co, ho, wo);
                    double v = scale[co] * z[i] + shift[co];
                    if (res) v += res[i];
                    y[i] = d->relu ? (v > 0.0 ? v : 0.0) : v;
                }
    if (!z_out) free(z);
}

/* Step 2 of the training loop: mean absolute error and its gradient w.r.t. y. */
double orc_l1_loss(const double* y, const double* t, long numel) {
    double s = 0.0;
    for (long i = 0; i < numel; ++i) s += fabs(y[i] - t[i]);
    return s / (double)numel;
}

void orc_l1_grad(const double* y, const double* t, long numel, double* dy) {
    const double inv = 1.0 / (double)numel;
    for (long i = 0; i < numel; ++i) {
        const double diff = y[i] - t[i];
        dy[i] = diff > 0.0 ? inv : (diff < 0.0 ? -inv : 0.0);
    }
}

/*
 * Backward of the block, scatter form over the same seven loops.
 * dx and dres may be NULL.  dw, dscale, dshift are overwritten.
 * The raw convolution z needed by dscale is recomputed here from x and w.
 */
void orc_block_bwd(const orc_desc* d, const double* dy, const double* x, const double* w,
                   const double* y, const double* scale, double* dx, double* dw, double* dscale,
                   double* dshift, double* dres) {
    const int Ho = out_h(d), Wo = out_w(d);
    const size_t total = (size_t)d->N * d->C_out * Ho * Wo;
    double* g = (double*)malloc(total * sizeof(double));
    double* z = (double*)malloc(total * sizeof(double));
    orc_conv(d, x, w, z);
    for (size_t i = 0; i < total; ++i) g[i] = d->relu ? (y[i] > 0.0 ? dy[i] : 0.0) : dy[i];
    if (dres) memcpy(dres, g, total * sizeof(double));

    for (int co = 0; co < d->C_out; ++co) {
        double sb = 0.0, ss = 0.0;
        for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    const size_t i = O_IDX(n, co, ho, wo);
                    sb += g[i];
                    ss += g[i] * z[i];
                }
        dshift[co] = sb;
        dscale[co] = ss;
    }

    if (dx) {
        memset(dx, 0, (size_t)d->N * d->C_in * d->H * d->W * sizeof(double));
#pragma omp parallel for schedule(static)
        for (int n = 0; n < d->N; ++n)                   /* images never share a dx element */
            for (int co = 0; co < d->C_out; ++co)
                for (int ho = 0; ho < Ho; ++ho)
                    for (int wo = 0; wo < Wo; ++wo) {
                        const double gs = g[O_IDX(n, co, ho, wo)] * scale[co];
                        if (gs == 0.0) continue;
                        for (int ci = 0; ci < d->C_in; ++ci)
                            for (int kh = 0; kh < d->KH; ++kh)
                                for (int kw = 0; kw < d->KW; ++kw) {
                                    const int hi = ho * d->stride - d->pad + kh;
                                    const int wi = wo * d->stride - d->pad + kw;
                                    if (hi < 0 || hi >= d->H || wi < 0 || wi >= d->W) continue;
                                    dx[(((size_t)n * d->C_in + ci) * d->H + hi) * d->W + wi] +=
                                        gs * W_AT(co, ci, kh, kw);
                                }
                    }
    }

    memset(dw, 0, (size_t)d->C_out * d->C_in * d->KH * d->KW * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int co = 0; co < d->C_out; ++co)                /* output channels never share a dw element */
        for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    const double gs = g[O_IDX(n, co, ho, wo)] * scale[co];
                    if (gs == 0.0) continue;
                    for (int ci = 0; ci < d->C_in; ++ci)
                        for (int kh = 0; kh < d->KH; ++kh)
                            for (int kw = 0; kw < d->KW; ++kw) {
                                const int hi = ho * d->stride - d->pad + kh;
                                const int wi = wo * d->stride - d->pad + kw;
                                if (hi < 0 || hi >= d->H || wi < 0 || wi >= d->W) continue;
                                dw[(((size_t)co * d->C_in + ci) * d->KH + kh) * d->KW + kw] +=
                                    gs * X_AT(n, ci, hi, wi);
                            }
                }
    free(g);
    free(z);
}

/* 3x3-style max-pool over [N][C][H][W] (padding never wins: it is -inf). */
void orc_maxpool(int N, int C, int H, int W, int k, int stride, int pad, const double* x, double* y) {
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
#pragma omp parallel for schedule(static)
    for (long nc = 0; nc < (long)N * C; ++nc)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                double m = -INFINITY;
                for (int kh = 0; kh < k; ++kh)
                    for (int kw = 0; kw < k; ++kw) {
                        const int hi = ho * stride - pad + kh, wi = wo * stride - pad + kw;
                        if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                        const double v = x[((size_t)nc * H + hi) * W + wi];
                        if (v > m) m = v;
                    }
                y[((size_t)nc * Ho + ho) * Wo + wo] = m;
            }
}

/*
 * Round a double to the nearest bfloat16 value (8 significant bits, binary32 exponent
 * range, gradual underflow), ties to even, in one rounding step.
 */
double orc_bf16_rne(double v) {
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    (void)frexp(v, &e);                  /* |v| = m * 2^e with 0.5 <= m < 1 */
    int q = e - 8;                       /* weight of the last kept bit */
    if (q < -133) q = -133;              /* smallest subnormal is 2^-133 */
    const double r = nearbyint(ldexp(v, -q));   /* exact scaling; default mode = ties to even */
    double out = ldexp(r, q);
    if (fabs(out) > 0x1.FEp127) out = copysign(INFINITY, v);
    return out;
}

void orc_quantize_bf16(const double* in, double* out, long n) {
    for (long i = 0; i < n; ++i) out[i] = orc_bf16_rne(in[i]);
}

/* ------------------------------------------------------------------------------------
 * Single-output versions of the same definitions, for spot checks at sizes where the
 * full loops above would take minutes.  idx holds 4 ints per point.
 * ---------------------------------------------------------------------------------- */

/* idx = (n, co, ho, wo).  v_out: pre-activation; y_out: block output; mag_out (nullable):
 * |scale|*sum|x*w| + |shift| + |r|, the magnitude that bounds the rounding of v. */
void orc_fwd_points(const orc_desc* d, const double* x, const double* w, const double* scale,
                    const double* shift, const double* res, long npts, const int* idx,
                    double* v_out, double* y_out, double* mag_out) {
    const int Ho = out_h(d), Wo = out_w(d);
#pragma omp parallel for schedule(static)
    for (long p = 0; p < npts; ++p) {
        const int n = idx[4 * p], co = idx[4 * p + 1], ho = idx[4 * p + 2], wo = idx[4 * p + 3];
        double acc = 0.0, mag = 0.0;
        for (int ci = 0; ci < d->C_in; ++ci)
            for (int kh = 0; kh < d->KH; ++kh)
                for (int kw = 0; kw < d->KW; ++kw) {
                    const int hi = ho * d->stride - d->pad + kh;
                    const int wi = wo * d->stride - d->pad + kw;
                    if (hi < 0 || hi >= d->H || wi < 0 || wi >= d->W) continue;
                    const double t = X_AT(n, ci, hi, wi) * W_AT(co, ci, kh, kw);
                    acc += t;
                    mag += fabs(t);
                }
        double v = scale[co] * acc + shift[co];
        mag = fabs(scale[co]) * mag + fabs(shift[co]);
        if (res) {
            v += res[O_IDX(n, co, ho, wo)];
            mag += fabs(res[O_IDX(n, co, ho, wo)]);
        }
        v_out[p] = v;
        y_out[p] = d->relu ? (v > 0.0 ? v : 0.0) : v;
        if (mag_out) mag_out[p] = mag;
    }
}

/* idx = (n, ci, hi, wi): dx at that input element (gather over the taps that reach it). */
void orc_dx_points(const orc_desc* d, const double* dy, const double* y, const double* w,
                   const double* scale, long npts, const int* idx, double* out) {
    const int Ho = out_h(d), Wo = out_w(d);
#pragma omp parallel for schedule(static)
    for (long p = 0; p < npts; ++p) {
        const int n = idx[4 * p], ci = idx[4 * p + 1], hi = idx[4 * p + 2], wi = idx[4 * p + 3];
        double acc = 0.0;
        for (int co = 0; co < d->C_out; ++co)
            for (int kh = 0; kh < d->KH; ++kh)
                for (int kw = 0; kw < d->KW; ++kw) {
                    const int th = hi + d->pad - kh, tw = wi + d->pad - kw;
                    if (th < 0 || tw < 0 || th % d->stride || tw % d->stride) continue;
                    const int ho = th / d->stride, wo = tw / d->stride;
                    if (ho >= Ho || wo >= Wo) continue;
                    const size_t i = O_IDX(n, co, ho, wo);
                    const double g = d->relu ? (y[i] > 0.0 ? dy[i] : 0.0) : dy[i];
                    acc += g * scale[co] * W_AT(co, ci, kh, kw);
                }
        out[p] = acc;
    }
}

/* idx = (co, ci, kh, kw): dw at that weight element. */
void orc_dw_points(const orc_desc* d, const double* dy, const double* y, const double* x,
                   const double* scale, long npts, const int* idx, double* out) {
    const int Ho = out_h(d), Wo = out_w(d);
#pragma omp parallel for schedule(static)
    for (long p = 0; p < npts; ++p) {
        const int co = idx[4 * p], ci = idx[4 * p + 1], kh = idx[4 * p + 2], kw = idx[4 * p + 3];
        double acc = 0.0;
        for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    const int hi = ho * d->stride - d->pad + kh;
                    const int wi = wo * d->stride - d->pad + kw;
                    if (hi < 0 || hi >= d->H || wi < 0 || wi >= d->W) continue;
                    const size_t i = O_IDX(n, co, ho, wo);
                    const double g = d->relu ? (y[i] > 0.0 ? dy[i] : 0.0) : dy[i];
                    acc += g * scale[co] * X_AT(n, ci, hi, wi);
                }
        out[p] = acc;
    }
}

/* dshift and dscale of the listed output channels (dscale recomputes z along the way). */
void orc_affine_grad_channels(const orc_desc* d, const double* dy, const double* y, const double* x,
                              const double* w, long nch, const int* ch, double* dscale_out,
                              double* dshift_out) {
    const int Ho = out_h(d), Wo = out_w(d);
#pragma omp parallel for schedule(static)
    for (long p = 0; p < nch; ++p) {
        const int co = ch[p];
        double sb = 0.0, ss = 0.0;
        for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    const size_t i = O_IDX(n, co, ho, wo);
                    const double g = d->relu ? (y[i] > 0.0 ? dy[i] : 0.0) : dy[i];
                    if (g == 0.0) continue;
                    double z = 0.0;
                    for (int ci = 0; ci < d->C_in; ++ci)
                        for (int kh = 0; kh < d->KH; ++kh)
                            for (int kw = 0; kw < d->KW; ++kw) {
                                const int hi = ho * d->stride - d->pad + kh;
                                const int wi = wo * d->stride - d->pad + kw;
                                if (hi < 0 || hi >= d->H || wi < 0 || wi >= d->W) continue;
                                z += X_AT(n, ci, hi, wi) * W_AT(co, ci, kh, kw);
                            }
                    sb += g;
                    ss += g * z;
                }
        dshift_out[p] = sb;
        dscale_out[p] = ss;
    }
}
