/*
 * CPU oracle for the EOQ full-int8 training step -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, direct loops written from the definitions in the paper
 * (Section 3.2.1: forward Eq.2, backward Eq.3, parameter gradients Eq.4).
 * Nothing here is shared with the HIP library; only tests, the smoke check
 * and the CPU-baseline leg of the benchmark may load this file's library.
 *
 * Conventions: activations / errors are NHWC int8 codes, weights are KRSC
 * int8 codes, "conv" is cross-correlation with zero padding.  Every sum is
 * accumulated in int64 and must fit int32 (the functions return the number
 * of elements that did not fit; 0 means success).
 *
 * OpenMP is used on outermost loops only; integer sums are order-free, so
 * the bits do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t N, H, W, C; /* input tensor, NHWC            */
    int32_t K, R, S;    /* filters K x R x S x C (KRSC)   */
    int32_t stride, pad;
} eo_conv_desc;

static int out_dim(int in, int pad, int k, int st) { return (in + 2 * pad - k) / st + 1; }

int eo_out_h(const eo_conv_desc *d) { return out_dim(d->H, d->pad, d->R, d->stride); }
int eo_out_w(const eo_conv_desc *d) { return out_dim(d->W, d->pad, d->S, d->stride); }

static int fits32(int64_t v) { return v >= INT32_MIN && v <= INT32_MAX; }

/* Eq.2, x2 before quantisation: acc[n,p,q,k] = sum_{r,s,c} u[n,p*st+r-pad,q*st+s-pad,c] * w[k,r,s,c] */
long eo_conv_fwd(const eo_conv_desc *d, const int8_t *u, const int8_t *w, int32_t *acc)
{
    const int P = eo_out_h(d), Q = eo_out_w(d);
    long bad = 0;
#pragma omp parallel for collapse(2) reduction(+ : bad) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < d->K; ++k) {
                    int64_t s64 = 0;
                    for (int r = 0; r < d->R; ++r) {
                        const int h = p * d->stride + r - d->pad;
                        if (h < 0 || h >= d->H) continue;
                        for (int s = 0; s < d->S; ++s) {
                            const int x = q * d->stride + s - d->pad;
                            if (x < 0 || x >= d->W) continue;
                            const int8_t *up = u + (((size_t)n * d->H + h) * d->W + x) * d->C;
                            const int8_t *wp = w + (((size_t)k * d->R + r) * d->S + s) * d->C;
                            for (int c = 0; c < d->C; ++c) s64 += (int64_t)up[c] * (int64_t)wp[c];
                        }
                    }
                    if (!fits32(s64)) ++bad;
                    acc[(((size_t)n * P + p) * Q + q) * d->K + k] = (int32_t)s64;
                }
    return bad;
}

/* Eq.3, e4 before quantisation (error times the transposed weights):
 * dx[n,h,x,c] = sum_{k,r,s} e[n,p,q,k] * w[k,r,s,c]  over the (p,q) with  h = p*st+r-pad, x = q*st+s-pad */
long eo_conv_bwd_data(const eo_conv_desc *d, const int8_t *e, const int8_t *w, int32_t *dx)
{
    const int P = eo_out_h(d), Q = eo_out_w(d);
    long bad = 0;
#pragma omp parallel for collapse(2) reduction(+ : bad) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int h = 0; h < d->H; ++h) {
            int64_t *tmp = (int64_t *)malloc(sizeof(int64_t) * (size_t)d->C);
            for (int x = 0; x < d->W; ++x) {
                for (int c = 0; c < d->C; ++c) tmp[c] = 0;
                for (int r = 0; r < d->R; ++r) {
                    const int ph = h + d->pad - r;
                    if (ph < 0 || ph % d->stride) continue;
                    const int p = ph / d->stride;
                    if (p >= P) continue;
                    for (int s = 0; s < d->S; ++s) {
                        const int qw = x + d->pad - s;
                        if (qw < 0 || qw % d->stride) continue;
                        const int q = qw / d->stride;
                        if (q >= Q) continue;
                        const int8_t *ep = e + (((size_t)n * P + p) * Q + q) * d->K;
                        for (int k = 0; k < d->K; ++k) {
                            const int64_t ev = ep[k];
                            const int8_t *wp = w + (((size_t)k * d->R + r) * d->S + s) * d->C;
                            for (int c = 0; c < d->C; ++c) tmp[c] += ev * (int64_t)wp[c];
                        }
                    }
                }
                int32_t *o = dx + (((size_t)n * d->H + h) * d->W + x) * d->C;
                for (int c = 0; c < d->C; ++c) {
                    if (!fits32(tmp[c])) ++bad;
                    o[c] = (int32_t)tmp[c];
                }
            }
            free(tmp);
        }
    return bad;
}

/* Eq.4, g_w before quantisation:
 * g[k,r,s,c] = sum_{n,p,q} e[n,p,q,k] * u[n,p*st+r-pad,q*st+s-pad,c] */
long eo_conv_bwd_weight(const eo_conv_desc *d, const int8_t *e, const int8_t *u, int32_t *g)
{
    const int P = eo_out_h(d), Q = eo_out_w(d);
    const size_t rsc = (size_t)d->R * d->S * d->C;
    long bad = 0;
#pragma omp parallel for reduction(+ : bad) schedule(dynamic, 1)
    for (int k = 0; k < d->K; ++k) {
        int64_t *g64 = (int64_t *)calloc(rsc, sizeof(int64_t));
        for (int n = 0; n < d->N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int64_t ev = e[(((size_t)n * P + p) * Q + q) * d->K + k];
                    for (int r = 0; r < d->R; ++r) {
                        const int h = p * d->stride + r - d->pad;
                        if (h < 0 || h >= d->H) continue;
                        for (int s = 0; s < d->S; ++s) {
                            const int x = q * d->stride + s - d->pad;
                            if (x < 0 || x >= d->W) continue;
                            const int8_t *up = u + (((size_t)n * d->H + h) * d->W + x) * d->C;
                            int64_t *gp = g64 + ((size_t)r * d->S + s) * d->C;
                            for (int c = 0; c < d->C; ++c) gp[c] += ev * (int64_t)up[c];
                        }
                    }
                }
        for (size_t i = 0; i < rsc; ++i) {
            if (!fits32(g64[i])) ++bad;
            g[(size_t)k * rsc + i] = (int32_t)g64[i];
        }
        free(g64);
    }
    return bad;
}

/* Max pooling on int8 codes (the stem of the ImageNet-shaped nets; the block the
 * paper builds on uses a 3x3/2 pool).  Padding cells never win; ties go to the
 * first cell in (r,s) scan order.  arg[] receives r*S+s of the winner. */
void eo_maxpool_fwd(int N, int H, int W, int C, int R, int S, int stride, int pad,
                    const int8_t *a, int8_t *y, uint8_t *arg)
{
    const int P = out_dim(H, pad, R, stride), Q = out_dim(W, pad, S, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int c = 0; c < C; ++c) {
                    int best = -1000, bi = 0;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * stride + r - pad;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int x = q * stride + s - pad;
                            if (x < 0 || x >= W) continue;
                            const int v = a[(((size_t)n * H + h) * W + x) * C + c];
                            if (v > best) { best = v; bi = r * S + s; }
                        }
                    }
                    const size_t o = (((size_t)n * P + p) * Q + q) * C + c;
                    y[o] = (int8_t)best;
                    arg[o] = (uint8_t)bi;
                }
}

/* Backward of the pool: each output error is routed to its winner; overlapping
 * windows add (integer sum, kept wide). */
void eo_maxpool_bwd(int N, int H, int W, int C, int R, int S, int stride, int pad,
                    const int8_t *e, const uint8_t *arg, int32_t *d)
{
    const int P = out_dim(H, pad, R, stride), Q = out_dim(W, pad, S, stride);
    memset(d, 0, sizeof(int32_t) * (size_t)N * H * W * C);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int c = 0; c < C; ++c) {
                    const size_t o = (((size_t)n * P + p) * Q + q) * C + c;
                    const int r = arg[o] / S, s = arg[o] % S;
                    const int h = p * stride + r - pad, x = q * stride + s - pad;
                    d[(((size_t)n * H + h) * W + x) * C + c] += e[o];
                }
}

/* ------------------------------------------------------------------------
 * Float head: the last layer is the one part the paper leaves unquantised
 * (Section 5.1).  fp64 with a fixed operation order so that the error that
 * re-enters the integer chain is reproducible bit for bit:
 *   feat   = sum / (128*HW)                    (mean of the real activations)
 *   logit  = b + sum_k feat_k * W_jk           sequential fma, ascending k
 *   p      = softmax with max subtraction, exp by the routine below,
 *            denominator summed in ascending j
 *   loss   = mean_n ( log(sum) - (logit_y - max) )
 *   dlogit = (p - onehot) / N
 *   dfeat  = sum_j dlogit_j * W_jk             sequential fma, ascending j
 *   d_out  = (float)(dfeat / HW)               error w.r.t. each real activation
 *   dW_jk  = sum_n dlogit_nj * feat_nk, db_j = sum_n dlogit_nj   ascending n
 * Build with -ffp-contract=off.
 * ---------------------------------------------------------------------- */
static double head_exp(double x)
{
    /* exp for x <= 0: k = rint(x*log2e); r = x - k*ln2 (two-part ln2); degree-13
     * Taylor polynomial by Horner with fma; scale by 2^k. */
    static const double LOG2E = 0x1.71547652b82fep+0;
    static const double LN2_HI = 0x1.62e42feep-1;
    static const double LN2_LO = 0x1.a39ef35793c76p-33;
    if (x < -700.0) x = -700.0;
    const double k = rint(x * LOG2E);
    double r = fma(k, -LN2_HI, x);
    r = fma(k, -LN2_LO, r);
    double p = 1.0 / 6227020800.0; /* 1/13! */
    p = fma(p, r, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)k);
}

double eo_head_exp(double x) { return head_exp(x); }

void eo_head(int N, int F, int J, int HW, const int32_t *gap_sum, const double *Wfc, const double *bfc,
             const int32_t *labels, double *loss_out, float *d_out, double *dW, double *db,
             double *logits_out /* [N][J], may be NULL */)
{
    double *feat = (double *)malloc(sizeof(double) * (size_t)N * F);
    double *dl = (double *)malloc(sizeof(double) * (size_t)N * J);
    double *lossn = (double *)malloc(sizeof(double) * (size_t)N);
    const double denom = 128.0 * (double)HW;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < F; ++k) feat[(size_t)n * F + k] = (double)gap_sum[(size_t)n * F + k] / denom;
        double *lg = dl + (size_t)n * J;
        for (int j = 0; j < J; ++j) {
            double a = bfc[j];
            for (int k = 0; k < F; ++k) a = fma(feat[(size_t)n * F + k], Wfc[(size_t)j * F + k], a);
            lg[j] = a;
            if (logits_out) logits_out[(size_t)n * J + j] = a;
        }
        double m = lg[0];
        for (int j = 1; j < J; ++j) if (lg[j] > m) m = lg[j];
        const double xy = lg[labels[n]] - m;
        double sum = 0.0;
        for (int j = 0; j < J; ++j) { lg[j] = head_exp(lg[j] - m); sum = sum + lg[j]; }
        lossn[n] = log(sum) - xy;
        for (int j = 0; j < J; ++j) {
            const double p = lg[j] / sum;
            lg[j] = (p - (j == labels[n] ? 1.0 : 0.0)) / (double)N;
        }
        for (int k = 0; k < F; ++k) {
            double a = 0.0;
            for (int j = 0; j < J; ++j) a = fma(lg[j], Wfc[(size_t)j * F + k], a);
            d_out[(size_t)n * F + k] = (float)(a / (double)HW);
        }
    }
    double loss = 0.0;
    for (int n = 0; n < N; ++n) loss = loss + lossn[n];
    *loss_out = loss / (double)N;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < J; ++j) {
        double b = 0.0;
        for (int n = 0; n < N; ++n) b = b + dl[(size_t)n * J + j];
        db[j] = b;
        for (int k = 0; k < F; ++k) {
            double a = 0.0;
            for (int n = 0; n < N; ++n) a = fma(dl[(size_t)n * J + j], feat[(size_t)n * F + k], a);
            dW[(size_t)j * F + k] = a;
        }
    }
    free(feat);
    free(dl);
    free(lossn);
}
