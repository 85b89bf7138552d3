/*
 * tao_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-purpose CPU evaluation of the per-operator tolerance
 * engine of "TAO: Tolerance-Aware Optimistic Verification for Floating-Point
 * Neural Networks" (Sec. 3.1 bound templates, Sec. 5.3 error profile, Sec. 5.4
 * leaf check, App. A.1-A.2 constants).  It exists so that tests, the smoke
 * check and the benchmark's cpu_baseline leg have something independent to
 * compare the GPU library with.  It shares no source, header, table or helper
 * with the GPU library and must never be called from the product path.
 *
 * Arithmetic: every bound is evaluated in IEEE binary64 with the rounding mode
 * set toward +infinity, so each printed formula is an upper enclosure of its
 * real-number value (quantities that must be lower bounds -- 1-sigma, 1-c*u,
 * w_lo, a lower sqrt -- are formed as -(RU(-x))).  Products of two binary32
 * numbers are exact in binary64.  The final value is converted to binary32,
 * again rounding up.  The check/profile step instead uses round-to-nearest
 * binary64, because there the arithmetic itself is the definition.
 *
 * No blocking, fusion or reordering: loops run in the order of the formulas.
 * OpenMP, when enabled, only distributes independent output rows.
 *
 * Pins (see tests/): gamma_k closed forms (App. A.1 Eq. gamma-def), the
 * summation bound of App. A.2 Eq. det-sum by exact-rational brute force, the
 * printed softmax template of Sec. 3.1 at first order, high-precision brute
 * force soundness for every template, exhaustive-range sweeps for the unary
 * templates, and an exact order-statistic cross-check of the histogram
 * percentiles.  Templates the paper names but does not print (LayerNorm,
 * RMSNorm, BatchNorm-affine, GELU, SiLU, mean) are derived from the primitive
 * rule of Sec. 3.1: "parity unpinned by the paper" for their exact constants.
 * They are pinned from below by soundness (brute force over executions) and
 * from above by the first-order worst case of the canonical algorithm under the
 * model of App. A.1, derived independently of the chains written here.
 */
#include <fenv.h>
#include <math.h>
#include <stdint.h>
#include <string.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define TAOO_NBINS 2048

/* Floating-point model of App. A.1 plus the intrinsic-accuracy constants that
 * Sec. 3.1 takes from the math library's documentation (relative error of the
 * intrinsic in units of u; Sec. 3.1 prints 2u for exp). */
typedef struct {
    double u;        /* unit roundoff, 2^-24 for binary32 (App. A.1) */
    int mode;        /* 0: deterministic gamma_k; 1: probabilistic gamma~_k(lambda) (Sec. 3.1) */
    double lambda;   /* 4 in the paper */
    double c_exp, c_erf, c_rsqrt, c_div;
    unsigned flags;  /* bit 0: add underflow terms (off: App. A.1 excludes underflow) */
    double c_log, c_sin, c_cos, c_tanh, c_pow;   /* further library functions, units of u */
} taoo_model;

typedef struct {
    uint64_t n;
    uint64_t violations;
    uint64_t nan_count;
    float max_rel;
    uint32_t accept;
    uint32_t p50_bin, p99_bin, p999_bin;
    float p50, p99, p999;
    uint32_t pad_;
    uint64_t hist[TAOO_NBINS];
} taoo_profile;

enum { TAOO_LAYERNORM = 0, TAOO_RMSNORM = 1, TAOO_BN_AFFINE = 2, TAOO_SUM = 3, TAOO_MEAN = 4 };
enum { TAOO_GELU_ERF = 0, TAOO_SILU = 1, TAOO_MUL = 2, TAOO_ADD = 3, TAOO_RELU = 4,
       TAOO_SUB = 5, TAOO_DIV = 6, TAOO_EXACT = 7, TAOO_SQRT = 8, TAOO_RSQRT = 9, TAOO_EXP = 10,
       TAOO_LOG = 11, TAOO_SIN = 12, TAOO_COS = 13, TAOO_TANH = 14, TAOO_POW = 15, TAOO_SIGMOID = 16,
       TAOO_GELU_TANH = 17 };

/* ------------------------------------------------------------------ helpers */

/* lower bound of (1 - x) while the mode is upward: -(RU(x - 1)). */
static double one_minus_lo(double x) { volatile double t = x - 1.0; return -t; }
/* lower bound of (a - b) while the mode is upward. */
static double sub_lo(double a, double b) { volatile double t = b - a; return -t; }
/* lower bound of (a + b) while the mode is upward. */
static double add_lo(double a, double b) { volatile double t = (-a) - b; return -t; }

/* libm calls are made in round-to-nearest (their error bound is stated for
 * that mode) and then widened by a few ulps. */
static double exp_up(double x) {
    int m = fegetround(); fesetround(FE_TONEAREST);
    volatile double v = exp(x);
    fesetround(m);
    return v * (1.0 + 0x1p-50);
}
static double expm1_up(double x) {
    int m = fegetround(); fesetround(FE_TONEAREST);
    volatile double v = expm1(x);
    fesetround(m);
    return v * (1.0 + 0x1p-50);
}
/* sqrt is correctly rounded in the current mode; the predecessor of the
 * upward-rounded root is a lower bound. */
static double sqrt_lo(double x) {
    volatile double r = sqrt(x);
    if (r * r == x) return r;   /* only an over-estimate is possible; equality test is a shortcut */
    return nextafter(r, 0.0);
}

/* Gamma(k): App. A.1 Eq. (gamma-def) in mode 0, the probabilistic constant of
 * Sec. 3.1 / App. A.2 in mode 1.  Returns NaN when k*u >= 1 (constant undefined). */
double taoo_gamma(long k, const taoo_model *md) {
    int saved = fegetround(); fesetround(FE_UPWARD);
    double r;
    if (k <= 0) { r = 0.0; }
    else if (md->mode == 0) {
        volatile double ku = (double)k * md->u;
        double den = one_minus_lo(ku);
        r = (den > 0.0) ? ku / den : NAN;
    } else {
        volatile double sq = sqrt((double)k);
        volatile double t1 = md->lambda * sq * md->u;
        volatile double t2 = ((double)k * md->u * md->u) / one_minus_lo(md->u);
        volatile double arg = t1 + t2;
        r = (arg < 1.0) ? expm1_up(arg) : NAN;
    }
    fesetround(saved);
    return r;
}

/* --------------------------------------------------- T1: linear / matmul    */
/* tau_ij = Gamma(K') * ( sum_k |a_ik||w_jk| + |b_j| ),  K' = K (+1 with bias).
 * Sec. 3.1: reductions take gamma_k with the k of the output element; the
 * dot-product form is the summation bound of App. A.2 with one extra rounding
 * per product.  trans_w = 0: W is [N,K] (row j holds the weights of output j);
 * trans_w = 1: W is [K,N]. */
int taoo_bound_linear(const float *A, const float *W, const float *bias, float *tau,
                      long M, long N, long K, long lda, long ldw, long ldt, int trans_w,
                      long batch, long strideA, long strideW, long strideT,
                      const taoo_model *md) {
    long Kp = K + (bias ? 1 : 0);
    double G = taoo_gamma(Kp, md);
    if (!(G == G)) return -4;
    for (long b = 0; b < batch; ++b) {
        const float *Ab = A + b * strideA, *Wb = W + b * strideW;
        float *Tb = tau + b * strideT;
#pragma omp parallel for schedule(static)
        for (long i = 0; i < M; ++i) {
            int saved = fegetround(); fesetround(FE_UPWARD);
            for (long j = 0; j < N; ++j) {
                volatile double S = 0.0;
                for (long k = 0; k < K; ++k) {
                    double a = fabs((double)Ab[i * lda + k]);
                    double w = fabs((double)(trans_w ? Wb[k * ldw + j] : Wb[j * ldw + k]));
                    S = S + a * w;            /* product exact, sum rounded up */
                }
                if (bias) S = S + fabs((double)bias[j]);
                volatile double t = G * S;
                /* optional gradual-underflow term: each of the K' roundings may lose 2^-150 */
                if (md->flags & 1u) t = t + (double)Kp * 0x1p-149;
                Tb[i * ldt + j] = (float)t;   /* rounds up: mode is upward */
            }
            fesetround(saved);
        }
    }
    return 0;
}

/* 2-D convolution as a reduction (Sec. 3.1: conv takes gamma_k with the k of the
 * output element; operator list of the appendix: Conv2D).  Input x[Nb][H][W][C],
 * filter w[Cout][R][S][C], output tau[Nb][OH][OW][Cout], all contiguous:
 *   tau[n,oh,ow,co] = Gamma(K') ( sum_{r,s,c} |x[n, oh*sh-ph+r*dh, ow*sw-pw+s*dw, c]| |w[co,r,s,c]| + |b_co| )
 * with K = R*S*C for every output element and K' = K (+1 with bias).  Taps that
 * fall into the zero padding are exact zeros: they add nothing to the sum and
 * keep their place in the count (a larger k stays sound).  Terms are added in
 * the order (r, s, c). */
int taoo_bound_conv2d(const float *x, const float *w, const float *bias, float *tau,
                      long Nb, long H, long W, long C, long Cout, long R, long S,
                      long sh, long sw, long ph, long pw, long dh, long dw,
                      const taoo_model *md) {
    if (sh < 1 || sw < 1 || dh < 1 || dw < 1 || ph < 0 || pw < 0) return -2;
    long OH = (H + 2 * ph - dh * (R - 1) - 1) / sh + 1;
    long OW = (W + 2 * pw - dw * (S - 1) - 1) / sw + 1;
    if (H + 2 * ph - dh * (R - 1) - 1 < 0 || W + 2 * pw - dw * (S - 1) - 1 < 0) return -2;
    long K = R * S * C, Kp = K + (bias ? 1 : 0);
    double G = taoo_gamma(Kp, md);
    if (!(G == G)) return -4;
#pragma omp parallel for schedule(static)
    for (long pix = 0; pix < Nb * OH * OW; ++pix) {
        int saved = fegetround(); fesetround(FE_UPWARD);
        long n = pix / (OH * OW), oh = (pix / OW) % OH, ow = pix % OW;
        for (long co = 0; co < Cout; ++co) {
            volatile double Sum = 0.0;
            for (long r = 0; r < R; ++r) {
                long ih = oh * sh - ph + r * dh;
                for (long s = 0; s < S; ++s) {
                    long iw = ow * sw - pw + s * dw;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;   /* padding: exact zeros */
                    const float *xp = x + ((n * H + ih) * W + iw) * C;
                    const float *wp = w + ((co * R + r) * S + s) * C;
                    for (long c = 0; c < C; ++c)
                        Sum = Sum + fabs((double)xp[c]) * fabs((double)wp[c]);
                }
            }
            if (bias) Sum = Sum + fabs((double)bias[co]);
            volatile double t = G * Sum;
            if (md->flags & 1u) t = t + (double)Kp * 0x1p-149;
            tau[pix * Cout + co] = (float)t;    /* rounds up */
        }
        fesetround(saved);
    }
    return 0;
}

/* --------------------------------------------------- T3: softmax            */
/* Sec. 3.1 "Minimal example: softmax", made rigorous by closing each
 * first-order step (exp(a)-1 <= a+a^2, 1/(1-c*u), S* >= S^(1-sigma)),
 * expressed through the computed output y = fl(e/S):
 *   a_j   = u (|x_j| + |m|)                               (eps_z)
 *   rho_j = (a_j (1+a_j) + c_exp u) / (1 - c_exp u)       (eps_e / e)
 *   q_j   = y_j / (1-u)                                   (>= e_j / S)
 *   sigma = Gamma(n-1) sum q_j + (1+Gamma(n-1)) sum rho_j q_j   (eps_S / S)
 *   tau_i = q_i rho_i + q_i (1+rho_i) sigma/(1-sigma) + u y_i
 * Entries with x_j = -inf are masked (tau = 0, not summed); n stays `cols`. */
int taoo_bound_softmax(const float *x, const float *y, float *tau, long rows, long cols, long ld,
                       const taoo_model *md) {
    double G = taoo_gamma(cols - 1, md);
    if (!(G == G)) return -4;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int saved = fegetround(); fesetround(FE_UPWARD);
        const float *xr = x + r * ld, *yr = y + r * ld;
        float *tr = tau + r * ld;
        const double u = md->u;
        double m = -INFINITY; int bad = 0;
        for (long j = 0; j < cols; ++j) {
            double v = (double)xr[j];
            if (v != v || v == INFINITY) bad = 1;
            if (v > m) m = v;
        }
        if (m == -INFINITY) bad = 1;
        const double inv1mu_den = one_minus_lo(u);
        const double cden = one_minus_lo(md->c_exp * u);
        volatile double Wsum = 0.0, Rsum = 0.0;
        if (!bad) {
            for (long j = 0; j < cols; ++j) {
                double v = (double)xr[j];
                if (v == -INFINITY) continue;
                volatile double a = u * (fabs(v) + fabs(m));
                volatile double rho = (a * (1.0 + a) + md->c_exp * u) / cden;
                volatile double q = fabs((double)yr[j]) / inv1mu_den;
                Wsum = Wsum + q;
                Rsum = Rsum + rho * q;
            }
        }
        volatile double sigma = G * Wsum + (1.0 + G) * Rsum;
        if (bad || !(sigma < 1.0)) {
            for (long j = 0; j < cols; ++j) tr[j] = NAN;
            fesetround(saved);
            continue;
        }
        volatile double sfac = sigma / one_minus_lo(sigma);
        for (long j = 0; j < cols; ++j) {
            double v = (double)xr[j];
            if (v == -INFINITY) { tr[j] = 0.0f; continue; }
            volatile double a = u * (fabs(v) + fabs(m));
            volatile double rho = (a * (1.0 + a) + md->c_exp * u) / cden;
            volatile double yj = fabs((double)yr[j]);
            volatile double q = yj / inv1mu_den;
            volatile double t = q * rho + q * (1.0 + rho) * sfac + u * yj;
            tr[j] = (float)t;
        }
        fesetround(saved);
    }
    return 0;
}

/* --------------------------------------------------- T2, T4-T6: row ops     */

/* lower bound of a*b for a,b >= 0 while the mode is upward. */
static double mul_lo(double a, double b) { volatile double t = (-a) * b; return -t; }

/* Error of a value divided by n in one or two roundings (a division, or a
 * multiplication by a rounded reciprocal):  (E/n + c_div u |v|) / (1 - c_div u). */
static double div_n_err(double E, double absv, long n, const taoo_model *md) {
    volatile double cu = md->c_div * md->u;
    volatile double num = E / (double)n + cu * absv;
    return num / one_minus_lo(cu);
}

/* Tail shared by LayerNorm and RMSNorm.  v* (the exact mean of squares) lies
 * in [v_lo, v_up]; E_v bounds |v^ - v*|.  With w = v + eps and r = w^-1/2:
 *   E_w = (E_v + u w*)/(1-u),  w_lo = w* - E_w  (must be > 0),
 *   E_r = 1/2 E_w w_lo^-3/2 + c_rsqrt u w_lo^-1/2,  R = r* + E_r.
 * Returns 0 when w_lo <= 0 (the template gives no finite bound). */
static int rsqrt_tail(double v_lo, double v_up, double E_v, double eps, const taoo_model *md,
                      double *rstar_up, double *E_r, double *R) {
    const double u = md->u;
    volatile double w_up = v_up + eps;
    volatile double E_w = (E_v + u * w_up) / one_minus_lo(u);
    volatile double nw = -v_lo - eps;           /* -nw is a lower bound of w* */
    double wstar_lo = -nw;
    double w_lo = sub_lo(wstar_lo, E_w);
    if (!(w_lo > 0.0)) return 0;
    double s_lo = sqrt_lo(w_lo);
    volatile double inv_s = 1.0 / s_lo;         /* >= w_lo^-1/2 */
    volatile double inv_s3 = inv_s / w_lo;      /* >= w_lo^-3/2 */
    volatile double er = 0.5 * E_w * inv_s3 + md->c_rsqrt * u * inv_s;
    volatile double rs = 1.0 / sqrt_lo(wstar_lo);   /* >= r* */
    volatile double RR = rs + er;
    *E_r = er; *rstar_up = rs; *R = RR;
    return 1;
}

/* kind = LAYERNORM: canonical two-pass algorithm
 *   mu = sum(x)/n; d = x - mu; v = sum(d^2)/n; w = v + eps; r = rsqrt(w); y = d r g + b.
 * Each step is bounded by the primitive rule of Sec. 3.1 (propagated + fresh
 * rounding), reductions by Gamma(n-1), the divisions by n through c_div, the
 * rsqrt through c_rsqrt.  Starred (exact) quantities are enclosed in binary64:
 *   E_s = Gamma(n-1) sum|x|;  E_mu = (E_s/n + c_div u |mu*|)/(1 - c_div u)
 *   E_d = (E_mu + u|d*|)/(1-u);  D = |d*| + E_d
 *   E_q = E_d (|d*| + D) + u D^2;  Q = D^2 (1+u)
 *   E_t = Gamma(n-1) sum Q + sum E_q;  E_v = (E_t/n + c_div u v*)/(1 - c_div u)
 *   (E_w, w_lo, E_r, R as in rsqrt_tail)
 *   E_h = D E_r + r* E_d + u D R;  H = |d*| r* + E_h
 *   E_p = |g| E_h + u |g| H;  tau = E_p + u |y|.
 * kind = RMSNORM: y = g (x rsqrt(mean(x^2) + eps)):
 *   E_t = (Gamma(n-1)(1+u) + u) sum x^2, then E_v .. R as above,
 *   tau = |x g| (E_r + u R) + u |y|.
 * kind = BN_AFFINE: y = x s_c + t_c per column: tau = u |x s| (1+u) + u |y|.
 * kind = SUM / MEAN over the last dimension, one tau per row
 *   (App. A.2 Eq. det-sum): sum: Gamma(n-1) sum|x|;
 *   mean: Gamma(n-1) sum|x| / n + |y| c_div u / (1 - c_div u).
 * `eps_in` is rounded to the binary32 value the operator actually adds.
 * g == NULL means g = 1.
 * y == NULL (the caller has no re-executed output at hand): the fresh-rounding term u|y| of
 * Sec. 3.1 is taken at an upper bound Y >= |y| of every canonical execution instead, formed from
 * the exact intermediates and their error bounds:
 *   LAYERNORM  Y = (|d*| r* |g| + E_p + |b|)(1+u)      (y = fl(p^ + b), |p^ - p*| <= E_p)
 *   RMSNORM    Y = |x g| R (1+u)^2                      (y = fl(g fl(x r^)), r^ <= R)
 *   BN_AFFINE  Y = (|x s|(1+u) + |t|)(1+u)              (y = fl(fl(x s) + t), or one fused rounding)
 *   MEAN       Y = (sum|x| / n)(1 + Gamma(n-1))(1 + c_div u)
 * b (the additive term) enters a bound only through this Y. */
int taoo_bound_norm(int kind, const float *x, const float *y, const float *g, const float *b,
                    double eps_in, float *tau, long rows, long cols, long ld,
                    const taoo_model *md) {
    const long n = cols;
    double G = taoo_gamma(n - 1, md);
    if (!(G == G)) return -4;
    const double eps = (double)(float)eps_in;
    const double u = md->u;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int saved = fegetround(); fesetround(FE_UPWARD);
        const float *xr = x + r * ld;
        if (kind == TAOO_SUM || kind == TAOO_MEAN) {
            volatile double sa = 0.0;
            for (long i = 0; i < n; ++i) sa = sa + fabs((double)xr[i]);
            volatile double t = G * sa;
            if (kind == TAOO_MEAN) {
                volatile double cu = md->c_div * u;
                volatile double Y;
                if (y) Y = fabs((double)y[r]);
                else Y = (sa / (double)n) * (1.0 + G) * (1.0 + cu);
                t = t / (double)n + Y * (cu / one_minus_lo(cu));
            }
            tau[r] = (float)t;
        } else if (kind == TAOO_BN_AFFINE) {
            const float *yr = y ? y + r * ld : NULL; float *tr = tau + r * ld;
            for (long i = 0; i < n; ++i) {
                double xs = fabs((double)xr[i] * (double)g[i]);           /* exact product */
                volatile double Y;
                if (yr) Y = fabs((double)yr[i]);
                else Y = (xs * (1.0 + u) + (b ? fabs((double)b[i]) : 0.0)) * (1.0 + u);
                volatile double t = u * xs * (1.0 + u) + u * Y;
                tr[i] = (float)t;
            }
        } else if (kind == TAOO_RMSNORM) {
            const float *yr = y ? y + r * ld : NULL; float *tr = tau + r * ld;
            volatile double s2_up = 0.0, ns2 = 0.0;    /* upper sum, negated lower sum of x^2 */
            for (long i = 0; i < n; ++i) {
                double xi = (double)xr[i];
                double sq = xi * xi;                    /* exact: 48 significant bits */
                s2_up = s2_up + sq;
                ns2 = ns2 - sq;
            }
            volatile double E_t = (G * (1.0 + u) + u) * s2_up;
            volatile double v_up = s2_up / (double)n;
            volatile double nv = ns2 / (double)n;
            double v_lo = -nv;
            double E_v = div_n_err(E_t, v_up, n, md);
            double rs, E_r, R;
            if (!rsqrt_tail(v_lo, v_up, E_v, eps, md, &rs, &E_r, &R)) {
                for (long i = 0; i < n; ++i) tr[i] = NAN;
            } else {
                for (long i = 0; i < n; ++i) {
                    double gi = g ? (double)g[i] : 1.0;
                    double xg = fabs((double)xr[i] * gi);                 /* exact */
                    volatile double Y;
                    if (yr) Y = fabs((double)yr[i]);
                    else Y = xg * R * (1.0 + u) * (1.0 + u);
                    volatile double t = xg * (E_r + u * R) + u * Y;
                    tr[i] = (float)t;
                }
            }
        } else { /* LAYERNORM */
            const float *yr = y ? y + r * ld : NULL; float *tr = tau + r * ld;
            volatile double s_up = 0.0, ns = 0.0, sabs = 0.0;
            for (long i = 0; i < n; ++i) {
                double xi = (double)xr[i];
                s_up = s_up + xi; ns = ns - xi; sabs = sabs + fabs(xi);
            }
            volatile double mu_up = s_up / (double)n;
            volatile double nmu = ns / (double)n;
            double mu_lo = -nmu;                         /* mu* lies in [mu_lo, mu_up] */
            volatile double E_s = G * sabs;
            double absmu = fmax(fabs(mu_lo), fabs(mu_up));
            double E_mu = div_n_err(E_s, absmu, n, md);
            volatile double sQ = 0.0, sEq = 0.0, sd2_up = 0.0, nsd2 = 0.0;
            for (long i = 0; i < n; ++i) {
                double xi = (double)xr[i];
                volatile double dhi = xi - mu_lo;        /* >= d* */
                double dlo = sub_lo(xi, mu_up);          /* <= d* */
                double ad_up = fmax(fabs(dhi), fabs(dlo));               /* >= |d*| */
                double ad_lo = (dlo > 0.0) ? dlo : ((dhi < 0.0) ? -dhi : 0.0);   /* <= |d*| */
                volatile double E_d = (E_mu + u * ad_up) / one_minus_lo(u);
                volatile double D = ad_up + E_d;
                volatile double E_q = E_d * (ad_up + D) + u * D * D;
                volatile double Q = D * D * (1.0 + u);
                sQ = sQ + Q; sEq = sEq + E_q;
                sd2_up = sd2_up + ad_up * ad_up;
                nsd2 = nsd2 - mul_lo(ad_lo, ad_lo);
            }
            volatile double E_t = G * sQ + sEq;
            volatile double v_up = sd2_up / (double)n;
            volatile double nv = nsd2 / (double)n;
            double v_lo = -nv;
            double E_v = div_n_err(E_t, v_up, n, md);
            double rs, E_r, R;
            if (!rsqrt_tail(v_lo, v_up, E_v, eps, md, &rs, &E_r, &R)) {
                for (long i = 0; i < n; ++i) tr[i] = NAN;
            } else {
                for (long i = 0; i < n; ++i) {
                    double xi = (double)xr[i];
                    volatile double dhi = xi - mu_lo;
                    double dlo = sub_lo(xi, mu_up);
                    double ad_up = fmax(fabs(dhi), fabs(dlo));
                    volatile double E_d = (E_mu + u * ad_up) / one_minus_lo(u);
                    volatile double D = ad_up + E_d;
                    volatile double E_h = D * E_r + rs * E_d + u * D * R;
                    volatile double H = ad_up * rs + E_h;
                    double ag = g ? fabs((double)g[i]) : 1.0;
                    volatile double E_p = ag * E_h + u * ag * H;
                    volatile double Y;
                    if (yr) Y = fabs((double)yr[i]);
                    else Y = (ad_up * rs * ag + E_p + (b ? fabs((double)b[i]) : 0.0)) * (1.0 + u);
                    volatile double t = E_p + u * Y;
                    tr[i] = (float)t;
                }
            }
        }
        fesetround(saved);
    }
    return 0;
}

/* --------------------------------------------------- T7, T8: elementwise    */
/* GELU (erf form): y = fl(0.5 x) * fl(1 + erf(fl(x k))), k = fl(1/sqrt 2):
 *   t* = x/sqrt2, E_t = (2u+u^2)|t*|, t_lo = max(0,|t*|-E_t),
 *   G' = (2/sqrt pi) exp(-t_lo^2), A = min(1, (2/sqrt pi)|t*|(1+4u)),
 *   E_g = G' E_t + c_erf u A,  tau = (|x|/2) E_g + u|y| (1 + 1/(1-u)).
 * GELU (tanh form): y = fl(0.5 x) * fl(1 + tanh(p^)), p^ the binary32 evaluation of
 *   p* = b (x + a x^3), b = sqrt(2/pi), a = 0.044715, in either association
 *   (b*(x + a*x*x*x) or b*x*(1 + a*x*x)); both terms have the sign of x and pass
 *   through at most 7 roundings, the two constants' included:
 *   E_p = Gamma(7)|p*|, p_lo = max(0,|p*|-E_p), G' = sech^2(p_lo) = 4q/(1+q)^2 with
 *   q = exp(-2 p_lo), A = min(1, |p*|(1+Gamma(7))), E_T = G' E_p + c_tanh u A,
 *   tau = (|x|/2) E_T + u|y| (1 + 1/(1-u)).
 * SiLU: y = fl(x / fl(1 + exp(-x))): c' = c_exp u/(1-c_exp u), w = (c'+u)/(1-u),
 *   tau = |y| (w/(1-u) + u).
 * MUL / ADD / SUB / SQRT: one correctly rounded operation, tau = u|y|.
 * RELU / EXACT (Neg, Abs, Max, Min, max-pooling, masked fill, data movement): tau = 0.
 * DIV, RSQRT, EXP, LOG, SIN, COS, TANH, POW: a library function whose result is
 *   within c u of the exact one relatively, y = y*(1+d), |d| <= c u, so
 *   |y - y*| <= c u |y*| <= |y| c u/(1 - c u); c = c_div, c_rsqrt, c_exp, c_log,
 *   c_sin, c_cos, c_tanh, c_pow.  (Inputs are exact: operator-local scope.)
 * SIGMOID: y = fl(1 / fl(1 + exp(-x))): the SiLU factor (the numerator is exact
 *   in both).
 * (Sec. 3.1 primitive rule; App. A.3 lists these operators, no template printed.) */
int taoo_bound_act(int kind, const float *x, const float *x2, const float *y, float *tau, long n,
                   const taoo_model *md) {
    (void)x2;
    const double u = md->u;
    if (kind < 0 || kind > TAOO_GELU_TANH) return -3;
    if ((kind == TAOO_GELU_ERF || kind == TAOO_GELU_TANH) && !x && n > 0) return -1;
#pragma omp parallel
    {
        int saved = fegetround(); fesetround(FE_UPWARD);
        const double inv_sqrt2_up = 0x1.6a09e667f3bcdp-1;   /* 1/sqrt 2, rounded up   */
        const double inv_sqrt2_lo = 0x1.6a09e667f3bccp-1;   /* 1/sqrt 2, rounded down */
        const double two_rsqrtpi_up = 0x1.20dd750429b6ep+0; /* 2/sqrt pi, rounded up  */
        volatile double c1 = md->c_exp * u / one_minus_lo(md->c_exp * u);
        volatile double om = (c1 + u) / one_minus_lo(u);
        volatile double silu_f = om / one_minus_lo(u) + u;
        volatile double fresh2 = u * (1.0 + 1.0 / one_minus_lo(u));
        double cf = -1.0;                                   /* library-function kinds */
        switch (kind) {
            case TAOO_DIV: cf = md->c_div; break;   case TAOO_RSQRT: cf = md->c_rsqrt; break;
            case TAOO_EXP: cf = md->c_exp; break;   case TAOO_LOG: cf = md->c_log; break;
            case TAOO_SIN: cf = md->c_sin; break;   case TAOO_COS: cf = md->c_cos; break;
            case TAOO_TANH: cf = md->c_tanh; break; case TAOO_POW: cf = md->c_pow; break;
            default: break;
        }
        volatile double lib_f = (cf >= 0.0) ? (cf * u) / one_minus_lo(cf * u) : 0.0;
        const double beta_up = 0x1.9884533d43651p-1, beta_lo = 0x1.9884533d43650p-1;   /* sqrt(2/pi) */
        const double a_up = 0x1.6e4e26d4801f8p-5, a_lo = 0x1.6e4e26d4801f7p-5;         /* 0.044715  */
        volatile double g7 = (7.0 * u) / one_minus_lo(7.0 * u);
#pragma omp for schedule(static)
        for (long i = 0; i < n; ++i) {
            volatile double t;
            double ay = fabs((double)y[i]);
            if (kind == TAOO_GELU_ERF) {
                double ax = fabs((double)x[i]);
                volatile double ts = ax * inv_sqrt2_up;                  /* >= |t*| */
                volatile double E_t = (2.0 * u + u * u) * ts;
                double t_lo = sub_lo(mul_lo(ax, inv_sqrt2_lo), E_t);     /* <= |t*| - E_t */
                if (t_lo < 0.0) t_lo = 0.0;
                double sq_lo = mul_lo(t_lo, t_lo);
                volatile double Gp = two_rsqrtpi_up * exp_up(-sq_lo);
                volatile double A = two_rsqrtpi_up * ts * (1.0 + 4.0 * u);
                if (A > 1.0) A = 1.0;
                volatile double E_g = Gp * E_t + md->c_erf * u * A;
                t = 0.5 * ax * E_g + ay * fresh2;
            } else if (kind == TAOO_GELU_TANH) {
                double ax = fabs((double)x[i]);
                double x2 = ax * ax;                                     /* exact */
                volatile double poly_up = 1.0 + a_up * x2;
                volatile double ps = beta_up * ax * poly_up;             /* >= |p*| */
                double poly_lo = add_lo(1.0, mul_lo(a_lo, x2));          /* <= 1 + a x^2 */
                double p_dn = mul_lo(mul_lo(beta_lo, ax), poly_lo);      /* <= |p*| */
                volatile double E_p = g7 * ps;
                double p_lo = sub_lo(p_dn, E_p);
                if (p_lo < 0.0) p_lo = 0.0;
                volatile double q = exp_up(-2.0 * p_lo);                 /* -2 p_lo exact; q >= exp(-2 p_lo) */
                if (q > 1.0) q = 1.0;
                double den_lo = mul_lo(add_lo(1.0, q), add_lo(1.0, q));  /* <= (1+q)^2 */
                volatile double Gp = (4.0 * q) / den_lo;
                if (Gp > 1.0) Gp = 1.0;                                  /* sech^2 <= 1 */
                volatile double A = ps * (1.0 + g7);
                if (A > 1.0) A = 1.0;
                volatile double E_T = Gp * E_p + md->c_tanh * u * A;
                t = 0.5 * ax * E_T + ay * fresh2;
            } else if (kind == TAOO_SILU || kind == TAOO_SIGMOID) {
                t = ay * silu_f;
            } else if (kind == TAOO_MUL || kind == TAOO_ADD || kind == TAOO_SUB || kind == TAOO_SQRT) {
                t = u * ay;
            } else if (cf >= 0.0) {
                t = ay * lib_f;
            } else {
                t = 0.0;
            }
            tau[i] = (float)t;
        }
        fesetround(saved);
    }
    return 0;
}

/* Rotary position embedding (operator list of App. A.3: Sin/Cos tables times the
 * activations; Sec. 3.1: a reduction of k terms takes gamma_k).  Each output is a
 * two-term dot product of exact inputs,
 *   y_a = x_a cos - x_b sin,   y_b = x_b cos + x_a sin,
 * so tau_a = Gamma(2) (|x_a cos| + |x_b sin|), tau_b = Gamma(2) (|x_b cos| + |x_a sin|)
 * for any order and with or without fused multiply-add.  x, tau: [rows][d];
 * cos, sin: [npos][d/2]; row r uses table row (r / inner) % npos.  Pairs (a, b):
 * (j, j + d/2) when interleaved == 0, (2j, 2j + 1) otherwise. */
int taoo_bound_rope(const float *x, const float *cs, const float *sn, float *tau,
                    long rows, long d, long inner, long npos, int interleaved, const taoo_model *md) {
    if (d < 0 || (d & 1) || inner < 1 || npos < 1 || rows < 0) return -2;
    double G = taoo_gamma(2, md);
    if (!(G == G)) return -4;
    long h = d / 2;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int saved = fegetround(); fesetround(FE_UPWARD);
        const float *xr = x + r * d, *cr = cs + ((r / inner) % npos) * h, *sr = sn + ((r / inner) % npos) * h;
        float *tr = tau + r * d;
        for (long j = 0; j < h; ++j) {
            long a = interleaved ? 2 * j : j, b = interleaved ? 2 * j + 1 : j + h;
            double xa = fabs((double)xr[a]), xb = fabs((double)xr[b]);
            double c = fabs((double)cr[j]), sv = fabs((double)sr[j]);
            volatile double sa = xa * c + xb * sv;      /* products exact, sum rounded up */
            volatile double sb = xb * c + xa * sv;
            volatile double ta = G * sa, tb = G * sb;
            if (md->flags & 1u) { ta = ta + 2.0 * 0x1p-149; tb = tb + 2.0 * 0x1p-149; }
            tr[a] = (float)ta; tr[b] = (float)tb;
        }
        fesetround(saved);
    }
    return 0;
}

/* --------------------------------------------------- check + profile        */
/* Leaf check of Sec. 5.4 and relative-error profile of Sec. 5.3 / Sec. 3.2
 * Eq. (2), in round-to-nearest binary64:
 *   d = |c - r|; violation <=> !(d <= alpha tau); e = d / (|r| + eps); e32 = (float)e.
 * Histogram key: NaN -> 2047, else bits(e32) >> 20 (8 bins per octave).
 * Percentile p = num/den: rank = max(1, ceil(n num/den)), nearest rank on the
 * bins, reported as the bin index and the bin's upper edge. */
static uint32_t bin_of(float e32) {
    if (e32 != e32) return TAOO_NBINS - 1;
    uint32_t bits; memcpy(&bits, &e32, 4);
    return bits >> 20;
}
static float bin_upper_edge(uint32_t b) {
    if (b >= TAOO_NBINS - 1) return NAN;
    if (b >= 2039) return INFINITY;
    uint32_t bits = (b + 1u) << 20; float f; memcpy(&f, &bits, 4); return f;
}
static uint32_t rank_bin(const uint64_t *hist, uint64_t n, uint64_t num, uint64_t den) {
    if (n == 0) return 0;
    /* ceil(n*num/den) without overflow for n < 2^53 */
    unsigned __int128 prod = (unsigned __int128)n * num;
    uint64_t rank = (uint64_t)((prod + den - 1) / den);
    if (rank < 1) rank = 1;
    uint64_t cum = 0;
    for (uint32_t b = 0; b < TAOO_NBINS; ++b) { cum += hist[b]; if (cum >= rank) return b; }
    return TAOO_NBINS - 1;
}

int taoo_check_and_profile(const float *claimed, const float *ref, const float *tau, long n,
                           double alpha, double eps_rel, taoo_profile *out) {
    int saved = fegetround(); fesetround(FE_TONEAREST);
    memset(out, 0, sizeof(*out));
    out->n = (uint64_t)n;
    float mx = 0.0f;
    for (long i = 0; i < n; ++i) {
        volatile double c = (double)claimed[i], r = (double)ref[i];
        volatile double d = fabs(c - r);
        volatile double T = alpha * (double)tau[i];
        if (!(d <= T)) out->violations++;
        volatile double den = fabs(r) + eps_rel;
        volatile double e = d / den;
        float e32 = (float)e;
        if (e32 != e32) out->nan_count++;
        else if (e32 > mx) mx = e32;
        out->hist[bin_of(e32)]++;
    }
    out->max_rel = mx;
    out->accept = (out->violations == 0) ? 1u : 0u;
    out->p50_bin = rank_bin(out->hist, out->n, 1, 2);
    out->p99_bin = rank_bin(out->hist, out->n, 99, 100);
    out->p999_bin = rank_bin(out->hist, out->n, 999, 1000);
    out->p50 = bin_upper_edge(out->p50_bin);
    out->p99 = bin_upper_edge(out->p99_bin);
    out->p999 = bin_upper_edge(out->p999_bin);
    fesetround(saved);
    return 0;
}

/* Element-wise relative errors e32 alone (same arithmetic as above), so a test
 * can compute exact order statistics with a sort and compare bins. */
int taoo_rel_errors(const float *claimed, const float *ref, long n, double eps_rel, float *e32_out) {
    int saved = fegetround(); fesetround(FE_TONEAREST);
    for (long i = 0; i < n; ++i) {
        volatile double c = (double)claimed[i], r = (double)ref[i];
        volatile double d = fabs(c - r);
        volatile double den = fabs(r) + eps_rel;
        volatile double e = d / den;
        e32_out[i] = (float)e;
    }
    fesetround(saved);
    return 0;
}

/* --------------------------------------------------- error profiles on the paper's grid */
/* Sec. 5.3 (and Sec. 3.2 Eq. 1-2): absolute and relative element-wise errors between the
 * proposer's and the challenger's output, their percentile profiles on the 22-point grid
 * P = {1, 5, 10, ..., 95, 99, 100}, and the selection statistic
 *   p_max = max_p { p_abs(p)/thr_abs(p), p_rel(p)/thr_rel(p) },  offending iff p_max > 1.
 * Percentiles are nearest-rank on the fixed 2048-edge histogram (bin = bits(e32) >> 20, NaN ->
 * 2047) and reported as the bin's upper edge, capped by the exact maximum (so p = 100 is the
 * maximum itself).
 * Ratios are binary64 quotients of the reported value and the threshold; NaN ratios (0/0) are
 * skipped; without thresholds p_max = NaN and offending = 0. */
#define TAOO_NGRID 22
typedef struct {
    uint64_t n;
    uint64_t nan_count;
    float max_abs, max_rel;
    float abs_p[TAOO_NGRID], rel_p[TAOO_NGRID];
    uint32_t abs_bin[TAOO_NGRID], rel_bin[TAOO_NGRID];
    double p_max;
    uint32_t offending;
    uint32_t pad_;
    uint64_t hist_abs[TAOO_NBINS], hist_rel[TAOO_NBINS];
} taoo_error_profile;

static int grid_percent(int g) { return g == 0 ? 1 : (g <= 19 ? 5 * g : (g == 20 ? 99 : 100)); }

int taoo_profile_errors(const float *claimed, const float *ref, long n, double eps_rel,
                        const float *thr_abs, const float *thr_rel, taoo_error_profile *out) {
    int saved = fegetround(); fesetround(FE_TONEAREST);
    memset(out, 0, sizeof(*out));
    out->n = (uint64_t)n;
    float mxa = 0.0f, mxr = 0.0f;
    for (long i = 0; i < n; ++i) {
        volatile double c = (double)claimed[i], r = (double)ref[i];
        volatile double d = fabs(c - r);
        volatile double den = fabs(r) + eps_rel;
        volatile double e = d / den;
        float a32 = (float)d, e32 = (float)e;
        if (e32 != e32) out->nan_count++;
        else if (e32 > mxr) mxr = e32;
        if (a32 == a32 && a32 > mxa) mxa = a32;
        out->hist_abs[bin_of(a32)]++;
        out->hist_rel[bin_of(e32)]++;
    }
    out->max_abs = mxa; out->max_rel = mxr;
    double pmax = NAN;
    for (int g = 0; g < TAOO_NGRID; ++g) {
        int pct = grid_percent(g);
        out->abs_bin[g] = rank_bin(out->hist_abs, out->n, (uint64_t)pct, 100);
        out->rel_bin[g] = rank_bin(out->hist_rel, out->n, (uint64_t)pct, 100);
        out->abs_p[g] = bin_upper_edge(out->abs_bin[g]);
        out->rel_p[g] = bin_upper_edge(out->rel_bin[g]);
        /* a percentile cannot exceed the exact maximum (p = 100 is the maximum itself) */
        if (n > 0 && out->abs_bin[g] < TAOO_NBINS - 1 && out->abs_p[g] > mxa) out->abs_p[g] = mxa;
        if (n > 0 && out->rel_bin[g] < TAOO_NBINS - 1 && out->rel_p[g] > mxr) out->rel_p[g] = mxr;
        if (thr_abs && thr_rel) {
            volatile double ra = (double)out->abs_p[g] / (double)thr_abs[g];
            volatile double rr = (double)out->rel_p[g] / (double)thr_rel[g];
            if (ra == ra && !(pmax >= ra)) pmax = ra;
            if (rr == rr && !(pmax >= rr)) pmax = rr;
        }
    }
    out->p_max = pmax;
    out->offending = (pmax > 1.0) ? 1u : 0u;
    fesetround(saved);
    return 0;
}
size_t taoo_error_profile_size(void) { return sizeof(taoo_error_profile); }

/* ------------------------------------------------- calibration: envelope and thresholds */
/* Sec. 3.2: the device- and input-agnostic profile of an operator is the max-envelope, per grid
 * point p, of the percentile profiles of all (device pair, input) runs,
 *   P_abs(p) = max_r P_abs^(r)(p),   P_rel(p) = max_r P_rel^(r)(p),
 * and the committed thresholds are alpha times it (alpha = 3 in the paper):
 *   thr_abs(p) = alpha P_abs(p),     thr_rel(p) = alpha P_rel(p).
 * Here: NaN profile entries are skipped by the maximum (NaN only if every run is NaN there);
 * the product is one IEEE binary64 multiplication, rounded UP to binary32, so a threshold is
 * never below alpha times the envelope.  count >= 1, alpha >= 0. */
int taoo_calibrate_thresholds(const taoo_error_profile *profiles, long count, double alpha,
                              float *env_abs, float *env_rel, float *thr_abs, float *thr_rel) {
    if (count < 1 || !(alpha >= 0.0)) return -1;
    int saved = fegetround(); fesetround(FE_TONEAREST);
    for (int g = 0; g < TAOO_NGRID; ++g) {
        float ma = NAN, mr = NAN;
        for (long r = 0; r < count; ++r) {
            float a = profiles[r].abs_p[g], e = profiles[r].rel_p[g];
            if (a == a && !(ma >= a)) ma = a;
            if (e == e && !(mr >= e)) mr = e;
        }
        if (env_abs) env_abs[g] = ma;
        if (env_rel) env_rel[g] = mr;
        volatile double ta = alpha * (double)ma, tr = alpha * (double)mr;
        fesetround(FE_UPWARD);
        volatile float fa = (float)ta, fr = (float)tr;      /* smallest binary32 >= product */
        fesetround(FE_TONEAREST);
        thr_abs[g] = fa; thr_rel[g] = fr;
    }
    fesetround(saved);
    return 0;
}

int taoo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
size_t taoo_profile_size(void) { return sizeof(taoo_profile); }
