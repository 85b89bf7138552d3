// Row-wise bound kernels: tao_bound_softmax and tao_bound_norm.
//
// One "row group" of TPR threads (a wavefront, or a whole 256-thread workgroup
// for long rows) owns one row.  The row is read once with 16-byte loads and
// kept in registers (V vectors per thread); row statistics are accumulated in
// binary64 and combined with wavefront shuffles (plus one LDS exchange when the
// group spans four wavefronts); the bound is written once.  HBM traffic is the
// algorithmic minimum: each input element read once, each tau written once.
// Rows longer than 8192 columns take the V == 0 variant, which re-reads the row
// from global memory in each pass instead of caching it.
//
// Formulas: Sec. 3.1 softmax template closed to second order; LayerNorm,
// RMSNorm, BatchNorm-affine, sum and mean (operators of App. A.3) from the
// primitive rule of Sec. 3.1 with Gamma(n-1) for the reductions (App. A.2).
#include "tao_check.hpp"
#include "tao_device.hpp"
#include "tao_host.hpp"

namespace tao {

constexpr int kRowThreads = 256;

struct RowConsts {
    double u;          // unit roundoff
    double G;          // Gamma(cols - 1), upper
    double inv1mu;     // >= 1/(1-u)
    double ce_u;       // c_exp * u
    double inv1mce;    // >= 1/(1 - c_exp u)
    double cd_u;       // c_div * u
    double inv1mcd;    // >= 1/(1 - c_div u)
    double cr_u;       // c_rsqrt * u
    double eps;        // (double)(float)eps
    double inv_n;      // 1/cols (nearest; covered by the guard factor)
    double mean_f;     // c_div u / (1 - c_div u), upper
    double m;          // rounding margin of a bound of this row length (see make_consts)
};

// Factors of the final upper rounding (up32g) for a rounding margin m.
struct UpFactors {
    double mul, sub;
    __device__ __forceinline__ explicit UpFactors(double m) : mul(1.0 + 0x1p-24 + fmax(0x1p-32, 2.0 * m)), sub(1.0 + m) {}
};

// ---- reductions over the TPR threads of a row group (result in every thread) ----
template <int TPR>
__device__ __forceinline__ void group_sum(double* v, int count, double* smem) {
    for (int i = 0; i < count; ++i) v[i] = wave_sum(v[i]);
    if (TPR > kWave) {
        const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
        // every reduction of a kernel has its own 16-double slot of smem, so one barrier is enough
        if (lane == 0) for (int i = 0; i < count; ++i) smem[wave * 4 + i] = v[i];
        __syncthreads();
        for (int i = 0; i < count; ++i) {
            double s = 0;
            for (int w = 0; w < TPR / kWave; ++w) s += smem[w * 4 + i];
            v[i] = s;
        }
    }
}
template <int TPR>
__device__ __forceinline__ void group_max_or(float& m, int& flag, double* smem) {
    m = wave_max(m);
    flag = wave_or(flag);
    if (TPR > kWave) {
        const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
        if (lane == 0) { smem[wave * 4] = (double)m; smem[wave * 4 + 1] = (double)flag; }
        __syncthreads();
        float mm = -INFINITY; int ff = 0;
        for (int w = 0; w < TPR / kWave; ++w) { mm = fmaxf(mm, (float)smem[w * 4]); ff |= (int)smem[w * 4 + 1]; }
        m = mm; flag = ff;
    }
}

#define TAO_ROW_PROLOGUE                                                              \
    constexpr int RPB = kRowThreads / TPR;                                            \
    constexpr bool CACHED = (V > 0);                                                  \
    __shared__ double smem[2 * 16]; /* one slot per reduction of the kernel */        \
    const int lt = threadIdx.x % TPR;                                                 \
    const long row = (long)blockIdx.x * RPB + threadIdx.x / TPR;                      \
    const bool active = row < rows;                                                   \
    const long limit = active ? cols : 0; /* idle groups see an empty row */          \
    const long roff = active ? row * ld : 0;                                          \
    const int nv = CACHED ? V : (int)((cols + TPR * 4 - 1) / (TPR * 4));              \
    (void)smem;

#define TAO_VEC_INDEX(v) (((long)(v) * TPR + lt) * 4)

// ------------------------------------------------------------------ softmax
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void softmax_bound(
    const float* __restrict__ x, const float* __restrict__ y, float* __restrict__ tau,
    long rows, long cols, long ld, int vec_ok, RowConsts k) {
    TAO_ROW_PROLOGUE
    float4 xv[CACHED ? V : 1], yv[CACHED ? V : 1];
    float m = -INFINITY; int bad = 0;
    for (int v = 0; v < nv; ++v) {
        const float4 X = load4<CACHED>(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, -INFINITY);
        if (CACHED) { xv[v] = X; yv[v] = load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f); }
        const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) { bad |= (e[c] != e[c]) | (e[c] == INFINITY); m = fmaxf(m, e[c]); }
    }
    group_max_or<TPR>(m, bad, smem);
    if (m == -INFINITY) bad = 1;
    // a = u(|x| + |m|) and rho = (a(1+a) + c u)/(1 - c u) as three fused multiply-adds:
    //   a = fma(u, |x|, u|m|);  rho = fma(fma(a, a, a), inv, c u inv)
    const double uam = k.u * fabs((double)m);
    const double ce_inv = k.ce_u * k.inv1mce;
    double acc[2] = {0.0, 0.0};                                  // sum q, sum rho q
    // q and rho of the cached elements are kept for the last pass only while registers allow
    // (a wavefront-wide row of 2048 columns recomputes them: six operations per element)
    constexpr bool KEEP = CACHED && V <= 4;
    double qv[KEEP ? V * 4 : 1], rv[KEEP ? V * 4 : 1];
    // masked entries (x = -inf) take |x| = 0 and y = 0: then q = 0 drops them from both sums
    // and from tau without a select on binary64 values
    auto q_rho = [&](float xe, float ye, double& q, double& rho) __attribute__((always_inline)) {
        const bool masked = xe == -INFINITY;
        const double ax = (double)(masked ? 0.f : fabsf(xe));
        const double a = fma(k.u, ax, uam);
        rho = fma(fma(a, a, a), k.inv1mce, ce_inv);
        q = (double)(masked ? 0.f : fabsf(ye)) * k.inv1mu;
    };
    for (int v = 0; v < nv; ++v) {
        const float4 X = CACHED ? xv[v] : load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, -INFINITY);
        const float4 Y = CACHED ? yv[v] : load4(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            double q, rho;
            q_rho(xe[c], ye[c], q, rho);
            acc[0] += q; acc[1] = fma(rho, q, acc[1]);
            if (KEEP) { qv[v * 4 + c] = q; rv[v * 4 + c] = rho; }
        }
    }
    group_sum<TPR>(acc, 2, smem + 16);
    const double sigma = k.G * acc[0] + (1.0 + k.G) * acc[1];
    if (!(sigma < 1.0)) bad = 1;
    // tau = q rho + q (1+rho) sfac + u y  with y = q (1-u) <= q:
    //     = q (rho (1 + sfac) + (sfac + u)); a row without a finite bound gets NaN through the
    // two row constants (0 * NaN = NaN also covers its masked entries)
    const double sfac = sigma / (1.0 - sigma);
    const double w1 = bad ? NAN : 1.0 + sfac;
    const double w0 = bad ? NAN : sfac + k.u;
    // (an error of the sums enters sfac amplified by 1/(1 - sigma): the margin follows)
    const UpFactors up(k.m * (1.0 + 2.0 / (1.0 - sigma)));
    for (int v = 0; v < nv; ++v) {
        float4 X = make_float4(0.f, 0.f, 0.f, 0.f), Y = X;
        if (!CACHED) {
            X = load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, -INFINITY);
            Y = load4(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        } else if (!KEEP) {
            X = xv[v]; Y = yv[v];
        }
        const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
        float te[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            double q, rho;
            if (KEEP) { q = qv[v * 4 + c]; rho = rv[v * 4 + c]; }
            else q_rho(xe[c], ye[c], q, rho);
            te[c] = up32g(q * fma(rho, w1, w0), up.mul, up.sub);
        }
        store4(tau + roff, TAO_VEC_INDEX(v), limit, vec_ok, make_float4(te[0], te[1], te[2], te[3]));
    }
}

// ---- softmax bound checked in registers (the bound is never stored) --------------------------
// Same arithmetic as softmax_bound element by element, followed by the leaf check of
// tao_check_and_profile on (claimed, y, tau) with tau first rounded to binary32 as it would have
// been stored.  Workgroups of 1024 threads walk the rows (1024 / TPR at a time), keep the
// histogram of relative errors in LDS and leave one partial per workgroup, like the streaming
// check pass; the same finalising kernel turns the partials into the profile.  HBM traffic:
// x, y and claimed read once (12 B per element), nothing written.
template <int TPR>
__device__ __forceinline__ void wide_group_sum(double* v, int count, double* smem) {
    for (int i = 0; i < count; ++i) v[i] = wave_sum(v[i]);
    if (TPR > kWave) {
        const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
        const int first = (threadIdx.x / TPR) * (TPR / kWave);       // first wavefront of this row group
        if (lane == 0) for (int i = 0; i < count; ++i) smem[wave * 4 + i] = v[i];
        __syncthreads();
        for (int i = 0; i < count; ++i) {
            double s = 0;
            for (int w = 0; w < TPR / kWave; ++w) s += smem[(first + w) * 4 + i];
            v[i] = s;
        }
    }
}
template <int TPR>
__device__ __forceinline__ void wide_group_max_or(float& m, int& flag, double* smem) {
    m = wave_max(m);
    flag = wave_or(flag);
    if (TPR > kWave) {
        const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
        const int first = (threadIdx.x / TPR) * (TPR / kWave);
        if (lane == 0) { smem[wave * 4] = (double)m; smem[wave * 4 + 1] = (double)flag; }
        __syncthreads();
        float mm = -INFINITY; int ff = 0;
        for (int w = 0; w < TPR / kWave; ++w) { mm = fmaxf(mm, (float)smem[(first + w) * 4]); ff |= (int)smem[(first + w) * 4 + 1]; }
        m = mm; flag = ff;
    }
}

template <int TPR, int V>
__global__ __launch_bounds__(kCheckThreads) void softmax_check(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ claimed,
    long rows, long cols, long ld, int vec_ok, RowConsts k, double alpha, double eps_rel,
    unsigned int* __restrict__ ws_hist, unsigned int* __restrict__ ws_coarse, BlockStats* __restrict__ ws_stats) {
    constexpr int RPB = kCheckThreads / TPR;
    constexpr bool CACHED = (V > 0);
    __shared__ unsigned int hist[kBins * kReplicas];
    __shared__ unsigned int red[3 * (kCheckThreads / kWave)];
    __shared__ double smem[2 * 4 * (kCheckThreads / kWave)];       // one slot per reduction of a row
    const int tid = threadIdx.x;
    for (int i = tid; i < kBins * kReplicas; i += kCheckThreads) hist[i] = 0;
    __syncthreads();
    ThreadAcc acc_chk;
    const int rep = tid & (kReplicas - 1);
    const int lt = tid % TPR;
    const int nv = CACHED ? V : (int)((cols + TPR * 4 - 1) / (TPR * 4));
    const long nblocks = (rows + RPB - 1) / RPB;
    // every thread of the workgroup takes the same number of trips (the reductions hold barriers)
    for (long rb = blockIdx.x; rb < nblocks; rb += gridDim.x) {
        const long row = rb * RPB + tid / TPR;
        const bool active = row < rows;
        const long limit = active ? cols : 0;
        const long roff = active ? row * ld : 0;
        float4 xv[CACHED ? V : 1], yv[CACHED ? V : 1];
        float m = -INFINITY; int bad = 0;
        for (int v = 0; v < nv; ++v) {
            const float4 X = load4<CACHED>(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, -INFINITY);
            if (CACHED) { xv[v] = X; yv[v] = load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f); }
            const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) { bad |= (e[c] != e[c]) | (e[c] == INFINITY); m = fmaxf(m, e[c]); }
        }
        wide_group_max_or<TPR>(m, bad, smem);
        if (m == -INFINITY) bad = 1;
        const double uam = k.u * fabs((double)m);
        const double ce_inv = k.ce_u * k.inv1mce;
        double acc[2] = {0.0, 0.0};
        auto q_rho = [&](float xe, float ye, double& q, double& rho) __attribute__((always_inline)) {
            const bool masked = xe == -INFINITY;
            const double ax = (double)(masked ? 0.f : fabsf(xe));
            const double a = fma(k.u, ax, uam);
            rho = fma(fma(a, a, a), k.inv1mce, ce_inv);
            q = (double)(masked ? 0.f : fabsf(ye)) * k.inv1mu;
        };
        for (int v = 0; v < nv; ++v) {
            const float4 X = CACHED ? xv[v] : load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, -INFINITY);
            const float4 Y = CACHED ? yv[v] : load4(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
            const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                double q, rho;
                q_rho(xe[c], ye[c], q, rho);
                acc[0] += q; acc[1] = fma(rho, q, acc[1]);
            }
        }
        wide_group_sum<TPR>(acc, 2, smem + 4 * (kCheckThreads / kWave));
        const double sigma = k.G * acc[0] + (1.0 + k.G) * acc[1];
        if (!(sigma < 1.0)) bad = 1;
        const double sfac = sigma / (1.0 - sigma);
        const double w1 = bad ? NAN : 1.0 + sfac;
        const double w0 = bad ? NAN : sfac + k.u;
        const UpFactors up(k.m * (1.0 + 2.0 / (1.0 - sigma)));
        for (int v = 0; v < nv; ++v) {
            const long idx = TAO_VEC_INDEX(v);
            if (idx >= limit) continue;
            const float4 X = CACHED ? xv[v] : load4(x + roff, idx, limit, vec_ok, -INFINITY);
            const float4 Y = CACHED ? yv[v] : load4(y + roff, idx, limit, vec_ok, 0.f);
            const float4 C = load4<true>(claimed + roff, idx, limit, vec_ok, 0.f);
            const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w}, ce[4] = {C.x, C.y, C.z, C.w};
            if (idx + 3 < limit) {                           // a whole vector: four chains side by side
                float te[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    double q, rho;
                    q_rho(xe[c], ye[c], q, rho);
                    te[c] = up32g(q * fma(rho, w1, w0), up.mul, up.sub);
                }
                check_four(ce, ye, te, alpha, eps_rel, hist, rep, acc_chk);
                continue;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (idx + c >= limit) break;
                double q, rho;
                q_rho(xe[c], ye[c], q, rho);
                const float t = up32g(q * fma(rho, w1, w0), up.mul, up.sub);
                check_one(ce[c], ye[c], t, alpha, eps_rel, hist, rep, acc_chk);
            }
        }
    }
    __syncthreads();
    flush_block_stats(acc_chk, red, ws_stats);
    flush_histogram(hist, ws_hist + (size_t)blockIdx.x * kBins, ws_coarse + blockIdx.x * kGroups);
}

// tail shared by LayerNorm and RMSNorm: from v*, E_v to (r*, E_r, R); ok = finite bound
// amp: how much a relative error of the row sums is amplified on its way into E_r (the sums enter
// through the difference w_lo = w - E_w, and E_r falls with w_lo at most like its power -3/2)
__device__ __forceinline__ bool rsqrt_tail(double vstar, double E_v, const RowConsts& k,
                                           double& rs, double& E_r, double& R, double& amp) {
    const double w = vstar + k.eps;
    const double E_w = (E_v + k.u * w) * k.inv1mu;
    const double w_lo = w - E_w;
    const bool ok = w_lo > 0.0;
    amp = (w + E_w) / w_lo;
    const double inv_s = 1.0 / sqrt(w_lo);
    const double inv_s3 = inv_s / w_lo;
    E_r = 0.5 * E_w * inv_s3 + k.cr_u * inv_s;
    rs = 1.0 / sqrt(w);
    R = rs + E_r;
    return ok;
}

// ------------------------------------------------------------------ LayerNorm
// Chain of the template (E_s, E_mu, E_d, D, E_q, Q, E_t, E_v, E_w, w_lo, E_r, R, E_h, H, E_p).
// Per element only |d| = |x - mu| varies, and everything downstream is a polynomial in it with
// non-negative coefficients:
//   E_d = u' |d| + E'      (u' = u/(1-u), E' = E_mu/(1-u));   D = |d| + E_d = (1+u')|d| + E'
// so the two sums the variance bound needs,
//   sum Q   = (1+u) sum D^2,   sum E_q = sum E_d(|d| + D) + u sum D^2,
// follow from n, sum|d| and sum d^2, and the per-element tail
//   E_p/|g| = (1+u) E_h + u r|d|,  E_h = D (E_r + u R) + r E_d
// collapses to K1 |d| + K0.  Same real-number formula as the step-by-step chain; the different
// binary64 rounding (a few 2^-53) is covered by the rounding margin of up32g.
// From E_mu, sum|d|, sum d^2 to the per-element coefficients: E_p/|g| = K1 |d| + K0.
__device__ __forceinline__ void layernorm_tail(double E_mu, double s_ad, double s_d2, double n, const RowConsts& k,
                                               double& K1, double& K0, double& amp, double* rs_out = nullptr) {
    const double up = k.u * k.inv1mu, Ep = E_mu * k.inv1mu;       // u', E'
    const double c1 = 1.0 + up;
    const double sD2 = c1 * c1 * s_d2 + 2.0 * c1 * Ep * s_ad + n * Ep * Ep;           // sum D^2
    const double sEdD = up * (1.0 + c1) * s_d2 + Ep * (up + 1.0 + c1) * s_ad + n * Ep * Ep;  // sum E_d(|d|+D)
    const double E_t = k.G * (1.0 + k.u) * sD2 + sEdD + k.u * sD2;
    const double vstar = s_d2 * k.inv_n;
    const double E_v = (E_t * k.inv_n + k.cd_u * vstar) * k.inv1mcd;
    double rs, E_r, R;
    const bool ok = rsqrt_tail(vstar, E_v, k, rs, E_r, R, amp);
    const double hc = E_r + k.u * R;                              // E_h = D hc + r E_d
    K1 = (1.0 + k.u) * (c1 * hc + rs * up) + k.u * rs;
    K0 = ok ? (1.0 + k.u) * Ep * (hc + rs) : NAN;                 // NaN row when the bound is not finite
    if (rs_out) *rs_out = rs;
}

// GROUPED (GroupNorm): a row is one (sample, group) of a channel-major tensor, cols = channels per
// group x positions; column c takes the affine scale of channel (row % groups) * cpg + c / hw.
struct GroupGeom { unsigned hw, cpg, groups; };
// NOY: the caller has no re-executed output; the fresh-rounding term u|y| is then taken at the upper
// bound Y = (|d| r |g| + E_p + |b|)(1+u) of |y| over all canonical executions (b: the additive term,
// which enters a bound only here).
template <int TPR, int V, bool GROUPED, bool NOY = false>
__device__ __forceinline__ void layernorm_body(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_g, const RowConsts& k,
    GroupGeom gg, const float* __restrict__ b = nullptr, int vec_b = 0) {
    static_assert(!(NOY && GROUPED), "GroupNorm takes the re-executed output");
    TAO_ROW_PROLOGUE
    // the four scales of the vector that starts at column idx
    const float* gb = (GROUPED && g && active) ? g + (unsigned long)(row % (long)gg.groups) * gg.cpg : g;
    auto scales = [&](long idx) {
        if (!g) return make_float4(1.f, 1.f, 1.f, 1.f);
        if (!GROUPED) return load4(g, idx, limit, vec_g, 1.f);
        float ge[4] = {1.f, 1.f, 1.f, 1.f};
        if (idx < limit) {
            unsigned ch = (unsigned)idx / gg.hw, rem = (unsigned)idx - ch * gg.hw;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (idx + c < limit) ge[c] = gb[ch];
                if (++rem == gg.hw) { rem = 0; ++ch; }
            }
        }
        return make_float4(ge[0], ge[1], ge[2], ge[3]);
    };
    // a cached row also requests y and g up front: their latency then overlaps the reductions
    constexpr bool CACHE_Y = CACHED;
    float4 xv[CACHED ? V : 1], yv[CACHE_Y ? V : 1], gv[CACHE_Y ? V : 1];
    double a1[2] = {0.0, 0.0};                                   // sum x, sum |x|
    for (int v = 0; v < nv; ++v) {
        const float4 X = load4<CACHED>(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        if (CACHED) xv[v] = X;
        if (CACHE_Y) {
            // (without y the registers hold |b| instead)
            yv[v] = NOY ? (b ? load4(b, TAO_VEC_INDEX(v), limit, vec_b, 0.f) : make_float4(0.f, 0.f, 0.f, 0.f))
                        : load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
            gv[v] = scales(TAO_VEC_INDEX(v));
        }
        const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) { a1[0] += (double)e[c]; a1[1] += (double)fabsf(e[c]); }
    }
    group_sum<TPR>(a1, 2, smem);
    const double n = (double)cols;
    const double mu = a1[0] * k.inv_n;
    const double E_mu = ((k.G * a1[1]) * k.inv_n + k.cd_u * fabs(mu)) * k.inv1mcd;
    double a2[2] = {0.0, 0.0};                                   // sum |d|, sum d^2
    for (int v = 0; v < nv; ++v) {
        const float4 X = CACHED ? xv[v] : load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // padding lanes (beyond the row) hold x = 0 and must not count: d = 0 for them
            const double d = (TAO_VEC_INDEX(v) + c < limit) ? (double)e[c] - mu : 0.0;
            a2[0] += fabs(d);
            a2[1] = fma(d, d, a2[1]);
        }
    }
    group_sum<TPR>(a2, 2, smem + 16);
    double K1, K0, amp, rs;
    layernorm_tail(E_mu, a2[0], a2[1], n, k, K1, K0, amp, &rs);
    const UpFactors up(k.m * (1.0 + 2.0 * amp));
    for (int v = 0; v < nv; ++v) {
        const float4 X = CACHED ? xv[v] : load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        const float4 Y = CACHE_Y ? yv[v]
                       : NOY ? (b ? load4(b, TAO_VEC_INDEX(v), limit, vec_b, 0.f) : make_float4(0.f, 0.f, 0.f, 0.f))
                             : load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        const float4 Gv = CACHE_Y ? gv[v] : scales(TAO_VEC_INDEX(v));
        const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
        const float ge[4] = {Gv.x, Gv.y, Gv.z, Gv.w};
        float te[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double ad = fabs((double)xe[c] - mu);
            const double ag = (double)fabsf(ge[c]);
            const double ep = ag * fma(K1, ad, K0);
            // |y|, or its upper bound (|d| r |g| + E_p + |b|)(1+u)
            const double Yb = NOY ? (ad * rs * ag + ep + (double)fabsf(ye[c])) * (1.0 + k.u) : (double)fabsf(ye[c]);
            te[c] = up32g(fma(k.u, Yb, ep), up.mul, up.sub);
        }
        store4(tau + roff, TAO_VEC_INDEX(v), limit, vec_ok, make_float4(te[0], te[1], te[2], te[3]));
    }
}
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void layernorm_bound(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_g, RowConsts k) {
    layernorm_body<TPR, V, false>(x, y, g, tau, rows, cols, ld, vec_ok, vec_g, k, GroupGeom());
}
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void layernorm_bound_noy(
    const float* __restrict__ x, const float* __restrict__ g, const float* __restrict__ b,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_g, int vec_b, RowConsts k) {
    layernorm_body<TPR, V, false, true>(x, nullptr, g, tau, rows, cols, ld, vec_ok, vec_g, k, GroupGeom(), b, vec_b);
}
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void groupnorm_bound(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, RowConsts k, GroupGeom gg) {
    layernorm_body<TPR, V, true>(x, y, g, tau, rows, cols, ld, vec_ok, 0, k, gg);
}

// ---- GroupNorm rows longer than the cached variants hold: the row is cut into chunks of
// kChunk columns, one workgroup each, so that a few very long rows still fill the chip.  Three
// passes, each reading its chunk once: (a) sum x, sum |x|; (b) the mean from the partials of
// (a), then sum |d|, sum d^2; (c) all four sums, the row's coefficients, the bound.  Partials
// live in a caller-supplied workspace, four binary64 values per (row, chunk); every workgroup
// adds them up in the same order, so all chunks of a row see identical row constants.
constexpr long kSplitMaxRows = 512;                            // from here on one workgroup per row
constexpr int kChunkVecs = 8;                                  // float4 per thread
constexpr long kChunk = (long)kRowThreads * kChunkVecs * 4;    // 8192 columns

struct ChunkPos { long row, c0, limit; int s; };
__device__ __forceinline__ ChunkPos chunk_pos(long cols, unsigned nchunk) {
    ChunkPos p;
    p.row = blockIdx.x / nchunk; p.s = (int)(blockIdx.x % nchunk);
    p.c0 = (long)p.s * kChunk;
    p.limit = cols - p.c0 < kChunk ? cols - p.c0 : kChunk;      // columns of this chunk
    return p;
}
// sum over the chunks of a row of partial `which` .. `which + 1` (same order in every workgroup)
__device__ __forceinline__ void chunk_totals(const double* __restrict__ part, unsigned nchunk, int which,
                                             double* out2, double* smem) {
    double a[2] = {0.0, 0.0};
    for (unsigned s = threadIdx.x; s < nchunk; s += kRowThreads) { a[0] += part[s * 4 + which]; a[1] += part[s * 4 + which + 1]; }
    group_sum<kRowThreads>(a, 2, smem);
    out2[0] = a[0]; out2[1] = a[1];
}
__global__ __launch_bounds__(kRowThreads) void groupnorm_sums_a(const float* __restrict__ x, double* __restrict__ ws,
                                                                long cols, unsigned nchunk, int vec_ok) {
    __shared__ double smem[16];
    const ChunkPos p = chunk_pos(cols, nchunk);
    const float* xr = x + p.row * cols + p.c0;
    double a[2] = {0.0, 0.0};
#pragma unroll
    for (int v = 0; v < kChunkVecs; ++v) {
        const float4 X = load4<false>(xr, ((long)v * kRowThreads + threadIdx.x) * 4, p.limit, vec_ok, 0.f);
        const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) { a[0] += (double)e[c]; a[1] += (double)fabsf(e[c]); }
    }
    group_sum<kRowThreads>(a, 2, smem);
    if (threadIdx.x == 0) { double* o = ws + ((long)blockIdx.x) * 4; o[0] = a[0]; o[1] = a[1]; }
}
__global__ __launch_bounds__(kRowThreads) void groupnorm_sums_b(const float* __restrict__ x, double* __restrict__ ws,
                                                                long cols, unsigned nchunk, int vec_ok, RowConsts k) {
    __shared__ double smem[32];
    const ChunkPos p = chunk_pos(cols, nchunk);
    double t[2];
    chunk_totals(ws + p.row * nchunk * 4, nchunk, 0, t, smem);
    const double mu = t[0] * k.inv_n;
    const float* xr = x + p.row * cols + p.c0;
    double a[2] = {0.0, 0.0};
#pragma unroll
    for (int v = 0; v < kChunkVecs; ++v) {
        const long idx = ((long)v * kRowThreads + threadIdx.x) * 4;
        const float4 X = load4<false>(xr, idx, p.limit, vec_ok, 0.f);
        const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double d = (idx + c < p.limit) ? (double)e[c] - mu : 0.0;
            a[0] += fabs(d);
            a[1] = fma(d, d, a[1]);
        }
    }
    group_sum<kRowThreads>(a, 2, smem + 16);
    if (threadIdx.x == 0) { double* o = ws + ((long)blockIdx.x) * 4; o[2] = a[0]; o[3] = a[1]; }
}
__global__ __launch_bounds__(kRowThreads) void groupnorm_apply(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g, float* __restrict__ tau,
    const double* __restrict__ ws, long cols, unsigned nchunk, int vec_ok, RowConsts k, GroupGeom gg) {
    __shared__ double smem[32];
    const ChunkPos p = chunk_pos(cols, nchunk);
    double t1[2], t2[2];
    chunk_totals(ws + p.row * nchunk * 4, nchunk, 0, t1, smem);
    chunk_totals(ws + p.row * nchunk * 4, nchunk, 2, t2, smem + 16);
    const double n = (double)cols;
    const double mu = t1[0] * k.inv_n;
    const double E_mu = ((k.G * t1[1]) * k.inv_n + k.cd_u * fabs(mu)) * k.inv1mcd;
    double K1, K0, amp;
    layernorm_tail(E_mu, t2[0], t2[1], n, k, K1, K0, amp);
    const UpFactors up(k.m * (1.0 + 2.0 * amp));
    const long roff = p.row * cols + p.c0;
    const float* gb = g ? g + (unsigned long)(p.row % (long)gg.groups) * gg.cpg : nullptr;
#pragma unroll 2
    for (int v = 0; v < kChunkVecs; ++v) {
        const long idx = ((long)v * kRowThreads + threadIdx.x) * 4;
        if (idx >= p.limit) break;
        const float4 X = load4<true>(x + roff, idx, p.limit, vec_ok, 0.f);
        const float4 Y = load4<true>(y + roff, idx, p.limit, vec_ok, 0.f);
        float ge[4] = {1.f, 1.f, 1.f, 1.f};
        if (gb) {
            const unsigned col = (unsigned)(p.c0 + idx);
            unsigned ch = col / gg.hw, rem = col - ch * gg.hw;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (idx + c < p.limit) ge[c] = gb[ch];
                if (++rem == gg.hw) { rem = 0; ++ch; }
            }
        }
        const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
        float te[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double ad = fabs((double)xe[c] - mu);
            const double ep = (double)fabsf(ge[c]) * fma(K1, ad, K0);
            te[c] = up32g(fma(k.u, (double)fabsf(ye[c]), ep), up.mul, up.sub);
        }
        store4(tau + roff, idx, p.limit, vec_ok, make_float4(te[0], te[1], te[2], te[3]));
    }
}

// ------------------------------------------------------------------ RMSNorm
// NOY: no re-executed output; u|y| is taken at Y = |x g| R (1+u)^2 >= |y|.
template <int TPR, int V, bool NOY>
__device__ __forceinline__ void rmsnorm_body(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_g, const RowConsts& k) {
    TAO_ROW_PROLOGUE
    float4 xv[CACHED ? V : 1], yv[(CACHED && !NOY) ? V : 1], gv[CACHED ? V : 1];
    double a1[1] = {0.0};
    for (int v = 0; v < nv; ++v) {
        const float4 X = load4<CACHED>(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        if (CACHED) {
            xv[v] = X;
            if (!NOY) yv[v] = load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
            gv[v] = g ? load4(g, TAO_VEC_INDEX(v), limit, vec_g, 1.f) : make_float4(1.f, 1.f, 1.f, 1.f);
        }
        const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) a1[0] += (double)e[c] * (double)e[c];
    }
    group_sum<TPR>(a1, 1, smem);
    const double E_t = (k.G * (1.0 + k.u) + k.u) * a1[0];
    const double vstar = a1[0] * k.inv_n;
    const double E_v = (E_t * k.inv_n + k.cd_u * vstar) * k.inv1mcd;
    double rs, E_r, R, amp;
    const bool ok = rsqrt_tail(vstar, E_v, k, rs, E_r, R, amp);
    const double f = E_r + k.u * R;
    const double fy = k.u * R * (1.0 + k.u) * (1.0 + k.u);           // NOY: u Y / |x g|
    const UpFactors up(k.m * (1.0 + 2.0 * amp));
    for (int v = 0; v < nv; ++v) {
        const float4 X = CACHED ? xv[v] : load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        const float4 Y = NOY ? make_float4(0.f, 0.f, 0.f, 0.f)
                             : (CACHED ? yv[v] : load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f));
        const float4 Gv = CACHED ? gv[v] : (g ? load4(g, TAO_VEC_INDEX(v), limit, vec_g, 1.f) : make_float4(1.f, 1.f, 1.f, 1.f));
        const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
        const float ge[4] = {Gv.x, Gv.y, Gv.z, Gv.w};
        float te[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double xg = fabs((double)xe[c] * (double)ge[c]);
            const double t = NOY ? xg * f + xg * fy : xg * f + k.u * fabs((double)ye[c]);
            te[c] = ok ? up32g(t, up.mul, up.sub) : NAN;
        }
        store4(tau + roff, TAO_VEC_INDEX(v), limit, vec_ok, make_float4(te[0], te[1], te[2], te[3]));
    }
}
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void rmsnorm_bound(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_g, RowConsts k) {
    rmsnorm_body<TPR, V, false>(x, y, g, tau, rows, cols, ld, vec_ok, vec_g, k);
}
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void rmsnorm_bound_noy(
    const float* __restrict__ x, const float* __restrict__ g,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_g, RowConsts k) {
    rmsnorm_body<TPR, V, true>(x, nullptr, g, tau, rows, cols, ld, vec_ok, vec_g, k);
}

// LayerNorm / RMSNorm bounds checked on the spot: the structure of softmax_check (1024-thread
// workgroups that walk the rows, kCheckThreads / TPR rows at a time, one partial histogram each)
// with the arithmetic of layernorm_body / rmsnorm_bound, operation for operation, so that the bound
// compared in registers is the binary32 value the bound kernels store.
template <bool RMS, int TPR, int V>
__global__ __launch_bounds__(kCheckThreads) void norm_check(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ g, const float* __restrict__ claimed,
    long rows, long cols, long ld, int vec_ok, int vec_g, RowConsts k, double alpha, double eps_rel,
    unsigned int* __restrict__ ws_hist, unsigned int* __restrict__ ws_coarse, BlockStats* __restrict__ ws_stats) {
    constexpr int RPB = kCheckThreads / TPR;
    constexpr bool CACHED = (V > 0);
    __shared__ unsigned int hist[kBins * kReplicas];
    __shared__ unsigned int red[3 * (kCheckThreads / kWave)];
    __shared__ double smem[2 * 4 * (kCheckThreads / kWave)];       // one slot per reduction of a row
    const int tid = threadIdx.x;
    for (int i = tid; i < kBins * kReplicas; i += kCheckThreads) hist[i] = 0;
    __syncthreads();
    ThreadAcc acc_chk;
    const int rep = tid & (kReplicas - 1);
    const int lt = tid % TPR;
    const int nv = CACHED ? V : (int)((cols + TPR * 4 - 1) / (TPR * 4));
    const long nblocks = (rows + RPB - 1) / RPB;
    const double n = (double)cols;
    auto scales = [&](long idx, long limit) {
        return g ? load4(g, idx, limit, vec_g, 1.f) : make_float4(1.f, 1.f, 1.f, 1.f);
    };
    // every thread of the workgroup takes the same number of trips (the reductions hold barriers)
    for (long rb = blockIdx.x; rb < nblocks; rb += gridDim.x) {
        const long row = rb * RPB + tid / TPR;
        const bool active = row < rows;
        const long limit = active ? cols : 0;
        const long roff = active ? row * ld : 0;
        float4 xv[CACHED ? V : 1], yv[CACHED ? V : 1], gv[CACHED ? V : 1];
        double a1[2] = {0.0, 0.0};                 // RMS: sum x^2;  LayerNorm: sum x, sum |x|
        for (int v = 0; v < nv; ++v) {
            const float4 X = load4<CACHED>(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
            if (CACHED) {
                xv[v] = X;
                yv[v] = load4<true>(y + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
                gv[v] = scales(TAO_VEC_INDEX(v), limit);
            }
            const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (RMS) a1[0] += (double)e[c] * (double)e[c];
                else { a1[0] += (double)e[c]; a1[1] += (double)fabsf(e[c]); }
            }
        }
        wide_group_sum<TPR>(a1, RMS ? 1 : 2, smem);
        double mu = 0.0, K1 = 0.0, K0 = 0.0, f = 0.0, amp = 1.0;
        bool ok = true;
        if (RMS) {
            const double E_t = (k.G * (1.0 + k.u) + k.u) * a1[0];
            const double vstar = a1[0] * k.inv_n;
            const double E_v = (E_t * k.inv_n + k.cd_u * vstar) * k.inv1mcd;
            double rs, E_r, R;
            ok = rsqrt_tail(vstar, E_v, k, rs, E_r, R, amp);
            f = E_r + k.u * R;
        } else {
            mu = a1[0] * k.inv_n;
            const double E_mu = ((k.G * a1[1]) * k.inv_n + k.cd_u * fabs(mu)) * k.inv1mcd;
            double a2[2] = {0.0, 0.0};                                   // sum |d|, sum d^2
            for (int v = 0; v < nv; ++v) {
                const float4 X = CACHED ? xv[v] : load4(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
                const float e[4] = {X.x, X.y, X.z, X.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const double d = (TAO_VEC_INDEX(v) + c < limit) ? (double)e[c] - mu : 0.0;
                    a2[0] += fabs(d);
                    a2[1] = fma(d, d, a2[1]);
                }
            }
            wide_group_sum<TPR>(a2, 2, smem + 4 * (kCheckThreads / kWave));
            layernorm_tail(E_mu, a2[0], a2[1], n, k, K1, K0, amp);
        }
        const UpFactors up(k.m * (1.0 + 2.0 * amp));
        for (int v = 0; v < nv; ++v) {
            const long idx = TAO_VEC_INDEX(v);
            if (idx >= limit) continue;
            const float4 X = CACHED ? xv[v] : load4(x + roff, idx, limit, vec_ok, 0.f);
            const float4 Y = CACHED ? yv[v] : load4<true>(y + roff, idx, limit, vec_ok, 0.f);
            const float4 Gv = CACHED ? gv[v] : scales(idx, limit);
            const float4 C = load4<true>(claimed + roff, idx, limit, vec_ok, 0.f);
            const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w};
            const float ge[4] = {Gv.x, Gv.y, Gv.z, Gv.w}, ce[4] = {C.x, C.y, C.z, C.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (idx + c >= limit) break;
                float t;
                if (RMS) {
                    const double xg = fabs((double)xe[c] * (double)ge[c]);
                    const double tt = xg * f + k.u * fabs((double)ye[c]);
                    t = ok ? up32g(tt, up.mul, up.sub) : NAN;
                } else {
                    const double ad = fabs((double)xe[c] - mu);
                    const double ep = (double)fabsf(ge[c]) * fma(K1, ad, K0);
                    t = up32g(fma(k.u, (double)fabsf(ye[c]), ep), up.mul, up.sub);
                }
                check_one(ce[c], ye[c], t, alpha, eps_rel, hist, rep, acc_chk);
            }
        }
    }
    __syncthreads();
    flush_block_stats(acc_chk, red, ws_stats);
    flush_histogram(hist, ws_hist + (size_t)blockIdx.x * kBins, ws_coarse + blockIdx.x * kGroups);
}

// ------------------------------------------------------------------ sum / mean
template <int TPR, int V>
__global__ __launch_bounds__(kRowThreads) void summean_bound(
    const float* __restrict__ x, const float* __restrict__ y, float* __restrict__ tau,
    long rows, long cols, long ld, int vec_ok, int is_mean, RowConsts k) {
    TAO_ROW_PROLOGUE
    double a1[1] = {0.0};
    for (int v = 0; v < nv; ++v) {
        const float4 X = load4<true>(x + roff, TAO_VEC_INDEX(v), limit, vec_ok, 0.f);
        a1[0] += fabs((double)X.x) + fabs((double)X.y) + fabs((double)X.z) + fabs((double)X.w);
    }
    group_sum<TPR>(a1, 1, smem);
    if (active && lt == 0) {
        double t = k.G * a1[0];
        // (mean without y: |y| <= (sum|x| / n)(1 + Gamma)(1 + c_div u))
        if (is_mean) t = t * k.inv_n + (y ? fabs((double)y[row]) : a1[0] * k.inv_n * (1.0 + k.G) * (1.0 + k.cd_u)) * k.mean_f;
        const UpFactors up(k.m);
        tau[row] = up32g(t, up.mul, up.sub);
    }
}

// ------------------------------------------------------------------ BatchNorm-affine
// tau = u |x s_c| (1+u) + u |y|, column c = flat index mod cols; one thread per 4 columns.
// NOY: no re-executed output (y is then the shift t or NULL, indexed by column like s): u|y| is taken at
// Y = (|x s|(1+u) + |t|)(1+u) >= |y|.
template <bool NOY>
__global__ __launch_bounds__(kRowThreads) void bn_affine_bound(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ s,
    float* __restrict__ tau, long rows, long cols, long ld, int vec_ok, int vec_s, double u) {
    const long vpr = (cols + 3) / 4;                       // vectors per row
    const long total = rows * vpr;
    // flat grid-stride walk over (row, vector) pairs; the pair is advanced by additions only
    // (one division per thread, before the loop)
    const long stride = (long)gridDim.x * blockDim.x;
    const long srow = stride / vpr, sjv = stride - srow * vpr;
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long row = i / vpr, jv = i - row * vpr;
    for (; i < total; i += stride, row += srow, jv += sjv) {
        if (jv >= vpr) { jv -= vpr; ++row; }
        const long j = jv * 4;
        const float4 X = load4<true>(x + row * ld, j, cols, vec_ok, 0.f);
        const float4 Y = NOY ? (y ? load4(y, j, cols, 0, 0.f) : make_float4(0.f, 0.f, 0.f, 0.f))
                             : load4<true>(y + row * ld, j, cols, vec_ok, 0.f);
        const float4 S = load4(s, j, cols, vec_s, 0.f);
        const float xe[4] = {X.x, X.y, X.z, X.w}, ye[4] = {Y.x, Y.y, Y.z, Y.w}, se[4] = {S.x, S.y, S.z, S.w};
        float te[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double xs = fabs((double)xe[c] * (double)se[c]);
            const double Yb = NOY ? (xs * (1.0 + u) + fabs((double)ye[c])) * (1.0 + u) : fabs((double)ye[c]);
            const double t = u * xs * (1.0 + u) + u * Yb;
            te[c] = up32g(t, kUpMul, 1.0 + 0x1p-48);
        }
        store4(tau + row * ld, j, cols, vec_ok, make_float4(te[0], te[1], te[2], te[3]));
    }
}

// Pick the row-group shape for a row length and launch KERNEL<TPR, V>.  A single wavefront owns
// a row of up to WMAX columns (no barrier, no LDS exchange); longer rows take a workgroup.
// Measured: beyond 1024 columns the registers of a wavefront-wide cached row cut the occupancy
// to two wavefronts per SIMD and the kernels lose a third of their bandwidth, so WMAX = 1024.
// Rows of 513 .. 768 columns (a common hidden size) take three vectors per lane rather than four:
// fewer registers, one more wavefront per SIMD (LayerNorm 62 -> 68 %, RMSNorm 67 -> 75 % of the HBM roofline).
#define TAO_DISPATCH_ROWS(KERNEL, WMAX, rows, cols, stream, ...)                                    \
    do {                                                                                            \
        const long c_ = (cols);                                                                     \
        auto grid_ = [&](int tpr) { return dim3((unsigned)(((rows) + (kRowThreads / tpr) - 1) / (kRowThreads / tpr))); }; \
        if (c_ <= 256)       hipLaunchKernelGGL((KERNEL<64, 1>), grid_(64), dim3(kRowThreads), 0, stream, __VA_ARGS__);   \
        else if (c_ <= 512)  hipLaunchKernelGGL((KERNEL<64, 2>), grid_(64), dim3(kRowThreads), 0, stream, __VA_ARGS__);   \
        else if (c_ <= 768)  hipLaunchKernelGGL((KERNEL<64, 3>), grid_(64), dim3(kRowThreads), 0, stream, __VA_ARGS__);   \
        else if (c_ <= 1024) hipLaunchKernelGGL((KERNEL<64, 4>), grid_(64), dim3(kRowThreads), 0, stream, __VA_ARGS__);   \
        else if (c_ <= 2048 && WMAX >= 2048) hipLaunchKernelGGL((KERNEL<64, 8>), grid_(64), dim3(kRowThreads), 0, stream, __VA_ARGS__);  \
        else if (c_ <= 4096 && WMAX >= 4096) hipLaunchKernelGGL((KERNEL<64, 16>), grid_(64), dim3(kRowThreads), 0, stream, __VA_ARGS__); \
        else if (c_ <= 2048) hipLaunchKernelGGL((KERNEL<256, 2>), grid_(256), dim3(kRowThreads), 0, stream, __VA_ARGS__); \
        else if (c_ <= 4096) hipLaunchKernelGGL((KERNEL<256, 4>), grid_(256), dim3(kRowThreads), 0, stream, __VA_ARGS__); \
        else if (c_ <= 8192) hipLaunchKernelGGL((KERNEL<256, 8>), grid_(256), dim3(kRowThreads), 0, stream, __VA_ARGS__); \
        else                 hipLaunchKernelGGL((KERNEL<256, 0>), grid_(256), dim3(kRowThreads), 0, stream, __VA_ARGS__); \
    } while (0)

// variance: the operator divides by a computed variance (LayerNorm, RMSNorm, GroupNorm).  Its
// template subtracts the variance's own error bound, about Gamma(n-1) times the variance, from the
// variance: beyond Gamma(n-1) = 1/2 the difference has lost its relative accuracy (and soon its
// sign), so such rows are refused rather than bounded by noise.
static int make_consts(const tao_fp_model& md, long cols, double eps, RowConsts* k, bool variance = false) {
    const double G = gamma_up(cols - 1, md);
    if (!(G == G) || (variance && G > 0.5)) return TAO_ERR_K_RANGE;
    const double u = md.u;
    k->u = u; k->G = G;
    k->inv1mu = widen(1.0 / (1.0 - u));
    k->ce_u = md.c_exp * u;
    k->inv1mce = widen(1.0 / (1.0 - md.c_exp * u));
    k->cd_u = md.c_div * u;
    k->inv1mcd = widen(1.0 / (1.0 - md.c_div * u));
    k->cr_u = md.c_rsqrt * u;
    k->eps = (double)(float)eps;
    k->inv_n = 1.0 / (double)cols;
    k->mean_f = widen(k->cd_u * k->inv1mcd);
    // Rounding margin of the emitted bound.  The row sums are formed here in round-to-nearest
    // binary64 (each thread a sequential part, then a tree: at most cols 2^-53 below the real sum),
    // and a reference that adds the row sequentially with upward rounding sits up to cols 2^-52
    // above it; the scalar chain after the sums adds a few dozen roundings.  m covers both for a
    // bound that depends on the sums with unit sensitivity; the kernels scale it where a sum enters
    // through a difference (1 - sigma of the softmax, the lower end w_lo of the variance).
    k->m = ((double)cols + 130.0) * 0x1p-51;
    if (!(md.c_exp * u < 0.5) || !(md.c_div * u < 0.5)) return TAO_ERR_MODEL;
    return TAO_OK;
}

}  // namespace tao

extern "C" {

int tao_bound_softmax(const float* x, const float* y_ref, float* tau, long rows, long cols, long ld,
                      const tao_fp_model* model, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (rows < 0 || cols < 0 || ld < cols) return TAO_ERR_SHAPE;
    if (rows == 0 || cols == 0) return TAO_OK;
    if (!x || !y_ref || !tau) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(tau, 4)) return TAO_ERR_ALIGN;
    RowConsts k;
    rc = make_consts(md, cols, 0.0, &k);
    if (rc != TAO_OK) return rc;
    const int vec_ok = aligned(x, 16) && aligned(y_ref, 16) && aligned(tau, 16) && (ld % 4 == 0);
    hipStream_t st = (hipStream_t)stream;
    TAO_DISPATCH_ROWS(softmax_bound, 1024, rows, cols, st, x, y_ref, tau, rows, cols, ld, vec_ok, k);
    return launch_status();
}

int tao_bound_norm(int kind, const float* x, const float* y_ref, const float* gamma_or_scale,
                   const float* beta_or_shift, double eps, float* tau, long rows, long cols, long ld,
                   const tao_fp_model* model, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (kind < TAO_NORM_LAYERNORM || kind > TAO_NORM_MEAN) return TAO_ERR_KIND;
    if (rows < 0 || cols < 0 || ld < cols) return TAO_ERR_SHAPE;
    if (rows == 0) return TAO_OK;
    if (cols == 0 && kind != TAO_NORM_SUM && kind != TAO_NORM_MEAN) return TAO_OK;
    if (cols == 0) return TAO_ERR_SHAPE;
    if (!x || !tau) return TAO_ERR_NULL;
    if (kind == TAO_NORM_BN_AFFINE && !gamma_or_scale) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(tau, 4) || !aligned(gamma_or_scale, 4) || !aligned(beta_or_shift, 4))
        return TAO_ERR_ALIGN;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return TAO_ERR_SHAPE;
    RowConsts k;
    rc = make_consts(md, cols, eps, &k, kind == TAO_NORM_LAYERNORM || kind == TAO_NORM_RMSNORM);
    if (rc != TAO_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int vec_x = aligned(x, 16) && (ld % 4 == 0);
    const int vec_ok = vec_x && aligned(y_ref, 16) && aligned(tau, 16);      // (a NULL y_ref counts as aligned)
    const int vec_g = aligned(gamma_or_scale, 16), vec_b = aligned(beta_or_shift, 16);
    const float* g = gamma_or_scale;
    const float* b = beta_or_shift;
    switch (kind) {
        case TAO_NORM_LAYERNORM:
            if (y_ref) TAO_DISPATCH_ROWS(layernorm_bound, 1024, rows, cols, st, x, y_ref, g, tau, rows, cols, ld, vec_ok, vec_g, k);
            else       TAO_DISPATCH_ROWS(layernorm_bound_noy, 1024, rows, cols, st, x, g, b, tau, rows, cols, ld, vec_ok, vec_g, vec_b, k);
            break;
        case TAO_NORM_RMSNORM:
            if (y_ref) TAO_DISPATCH_ROWS(rmsnorm_bound, 1024, rows, cols, st, x, y_ref, g, tau, rows, cols, ld, vec_ok, vec_g, k);
            else       TAO_DISPATCH_ROWS(rmsnorm_bound_noy, 1024, rows, cols, st, x, g, tau, rows, cols, ld, vec_ok, vec_g, k);
            break;
        case TAO_NORM_BN_AFFINE: {
            const long total = rows * ((cols + 3) / 4);
            long blocks = (total + kRowThreads - 1) / kRowThreads;
            if (blocks > 256L * 64) blocks = 256L * 64;    // grid-stride beyond 64 workgroups per CU
            if (y_ref) hipLaunchKernelGGL(bn_affine_bound<false>, dim3((unsigned)blocks), dim3(kRowThreads), 0, st, x, y_ref, g,
                                          tau, rows, cols, ld, vec_ok, vec_g, md.u);
            else       hipLaunchKernelGGL(bn_affine_bound<true>, dim3((unsigned)blocks), dim3(kRowThreads), 0, st, x, b, g,
                                          tau, rows, cols, ld, vec_ok, vec_g, md.u);
            break;
        }
        default: {
            const int is_mean = (kind == TAO_NORM_MEAN);
            TAO_DISPATCH_ROWS(summean_bound, 1024, rows, cols, st, x, y_ref, tau, rows, cols, ld, vec_x, is_mean, k);
            break;
        }
    }
    return launch_status();
}

size_t tao_groupnorm_workspace_bytes(long batch, long channels, long positions, long groups) {
    using namespace tao;
    if (batch <= 0 || channels <= 0 || positions <= 0 || groups < 1 || channels % groups) return 0;
    const __int128 cols = (__int128)(channels / groups) * positions;
    if (cols <= 8192 || cols >= (1L << 31) || batch * groups >= kSplitMaxRows) return 0;   // the row kernels need none
    const long nchunk = (long)((cols + kChunk - 1) / kChunk);
    return (size_t)batch * (size_t)groups * (size_t)nchunk * 4 * sizeof(double);
}

int tao_bound_groupnorm(const float* x, const float* y_ref, const float* gamma, const float* beta, double eps,
                        float* tau, long batch, long channels, long positions, long groups,
                        const tao_fp_model* model, void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    (void)beta;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (batch < 0 || channels < 0 || positions < 0 || groups < 1 || channels % groups) return TAO_ERR_SHAPE;
    const long cpg = channels / groups;
    if (positions >= (1L << 31) || cpg >= (1L << 31) || groups >= (1L << 31)) return TAO_ERR_SHAPE;
    if ((__int128)cpg * positions >= (1L << 31) || (__int128)batch * groups >= (1L << 40)) return TAO_ERR_SHAPE;
    const long rows = batch * groups, cols = cpg * positions;
    if (rows == 0 || cols == 0) return TAO_OK;
    if (!x || !tau || !y_ref) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(tau, 4) || !aligned(gamma, 4)) return TAO_ERR_ALIGN;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return TAO_ERR_SHAPE;
    RowConsts k;
    rc = make_consts(md, cols, eps, &k, true);
    if (rc != TAO_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int vec_ok = aligned(x, 16) && aligned(y_ref, 16) && aligned(tau, 16) && (cols % 4 == 0);
    GroupGeom gg;
    gg.hw = (unsigned)positions; gg.cpg = (unsigned)cpg; gg.groups = (unsigned)groups;
    // rows the cached variants hold, or enough rows to fill the chip with one workgroup each
    // (measured: 1024 rows of 25088 run at 42 % of the HBM roofline that way, 32 % in chunks;
    // 256 rows of 40960 at 20 % against 32 %)
    if (cols <= 8192 || rows >= kSplitMaxRows) {
        TAO_DISPATCH_ROWS(groupnorm_bound, 1024, rows, cols, st, x, y_ref, gamma, tau, rows, cols, cols, vec_ok, k, gg);
        return launch_status();
    }
    const long nchunk = (cols + kChunk - 1) / kChunk;
    if ((__int128)rows * nchunk >= (1L << 31)) return TAO_ERR_SHAPE;
    const size_t need = (size_t)rows * (size_t)nchunk * 4 * sizeof(double);
    if (!ws || ws_bytes < need || !aligned(ws, 8)) return TAO_ERR_WORKSPACE;
    double* part = static_cast<double*>(ws);
    const dim3 grid((unsigned)(rows * nchunk)), blk(kRowThreads);
    hipLaunchKernelGGL(groupnorm_sums_a, grid, blk, 0, st, x, part, cols, (unsigned)nchunk, vec_ok);
    hipLaunchKernelGGL(groupnorm_sums_b, grid, blk, 0, st, x, part, cols, (unsigned)nchunk, vec_ok, k);
    hipLaunchKernelGGL(groupnorm_apply, grid, blk, 0, st, x, y_ref, gamma, tau, part, cols, (unsigned)nchunk, vec_ok, k, gg);
    return launch_status();
}

int tao_bound_check_norm(int kind, const float* x, const float* y_ref, const float* gamma, const float* beta,
                         double eps, const float* claimed, long rows, long cols, long ld,
                         double alpha, double eps_rel, const tao_fp_model* model, tao_profile* out,
                         void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    (void)beta;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (kind != TAO_NORM_LAYERNORM && kind != TAO_NORM_RMSNORM) return TAO_ERR_KIND;
    if (!out || !ws) return out ? TAO_ERR_WORKSPACE : TAO_ERR_NULL;
    if (rows < 0 || cols < 0 || ld < cols || !(eps >= 0.0) || !std::isfinite(eps)) return TAO_ERR_SHAPE;
    if (!(alpha >= 0.0) || !std::isfinite(alpha) || !(eps_rel >= 0.0) || !std::isfinite(eps_rel)) return TAO_ERR_SHAPE;
    const long n = rows * cols;
    if (rows > 0 && cols > 0 && n / cols != rows) return TAO_ERR_SHAPE;
    if (n >= (1L << 36)) return TAO_ERR_SHAPE;                      // 32-bit per-workgroup counters
    if (n > 0 && (!x || !y_ref || !claimed)) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(claimed, 4) || !aligned(gamma, 4) || !aligned(out, 8))
        return TAO_ERR_ALIGN;
    if (!aligned(ws, 256) || ws_bytes < check_workspace_bytes()) return TAO_ERR_WORKSPACE;
    RowConsts k;
    rc = make_consts(md, cols > 0 ? cols : 1, eps, &k, true);
    if (rc != TAO_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int vec_ok = aligned(x, 16) && (ld % 4 == 0) && aligned(y_ref, 16) && aligned(claimed, 16);
    const int vec_g = aligned(gamma, 16);
    const CheckWorkspace w = carve_check_workspace(ws);
    int nblocks = 1;
    const bool rms = kind == TAO_NORM_RMSNORM;
    auto launch = [&](auto kernel, int tpr, long r, long c, long l) {
        const long rb = (r + (kCheckThreads / tpr) - 1) / (kCheckThreads / tpr);
        nblocks = (int)(rb < 1 ? 1 : (rb < kMaxCheckBlocks ? rb : kMaxCheckBlocks));
        hipLaunchKernelGGL(kernel, dim3(nblocks), dim3(kCheckThreads), 0, st, x, y_ref, gamma, claimed, r, c, l,
                           vec_ok, vec_g, k, alpha, eps_rel, w.hist, w.coarse, w.stats);
    };
    // at most two vectors per thread for RMSNorm and one, up to 1024 columns, for LayerNorm (its
    // second reduction and the check's binary64 division leave no more room under the 128-register
    // limit of a 1024-thread workgroup): longer rows take wider groups, or re-read the row
#define TAO_NORM_CHECK(RMS, TPR, V) launch(norm_check<RMS, TPR, V>, TPR, rows, cols, ld)
    if (n == 0) {
        if (rms) launch(norm_check<true, 64, 1>, 64, 0L, 1L, 1L); else launch(norm_check<false, 64, 1>, 64, 0L, 1L, 1L);
    } else if (rms) {
        if (cols <= 256)       TAO_NORM_CHECK(true, 64, 1);
        else if (cols <= 512)  TAO_NORM_CHECK(true, 64, 2);
        else if (cols <= 1024) TAO_NORM_CHECK(true, 256, 1);
        else if (cols <= 2048) TAO_NORM_CHECK(true, 256, 2);
        else if (cols <= 4096) TAO_NORM_CHECK(true, 512, 2);
        else if (cols <= 8192) TAO_NORM_CHECK(true, 1024, 2);
        else                   TAO_NORM_CHECK(true, 1024, 0);
    } else {
        if (cols <= 256)       TAO_NORM_CHECK(false, 64, 1);
        else if (cols <= 1024) TAO_NORM_CHECK(false, 256, 1);
        else                   TAO_NORM_CHECK(false, 1024, 0);     // wider cached rows spill: re-read instead
    }
#undef TAO_NORM_CHECK
    launch_profile_reduce(w, nblocks, (unsigned long long)n, out, st);
    return launch_status();
}

int tao_bound_check_softmax(const float* x, const float* y_ref, const float* claimed, long rows, long cols, long ld,
                            double alpha, double eps_rel, const tao_fp_model* model, tao_profile* out,
                            void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (!out || !ws) return out ? TAO_ERR_WORKSPACE : TAO_ERR_NULL;
    if (rows < 0 || cols < 0 || ld < cols || !(eps_rel >= 0.0)) return TAO_ERR_SHAPE;
    const long n = rows * cols;
    if (rows > 0 && cols > 0 && n / cols != rows) return TAO_ERR_SHAPE;
    if (n >= (1L << 36)) return TAO_ERR_SHAPE;                      // 32-bit per-workgroup counters
    if (n > 0 && (!x || !y_ref || !claimed)) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(claimed, 4) || !aligned(out, 8)) return TAO_ERR_ALIGN;
    if (!aligned(ws, 256) || ws_bytes < check_workspace_bytes()) return TAO_ERR_WORKSPACE;
    RowConsts k;
    rc = make_consts(md, cols > 0 ? cols : 1, 0.0, &k);
    if (rc != TAO_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const CheckWorkspace w = carve_check_workspace(ws);
    const int vec_ok = aligned(x, 16) && aligned(y_ref, 16) && aligned(claimed, 16) && (ld % 4 == 0);
    int nblocks = 1;
    if (n > 0) {
        auto launch = [&](auto kernel, int tpr) {
            const long rb = (rows + (kCheckThreads / tpr) - 1) / (kCheckThreads / tpr);
            nblocks = (int)(rb < kMaxCheckBlocks ? rb : kMaxCheckBlocks);
            hipLaunchKernelGGL(kernel, dim3(nblocks), dim3(kCheckThreads), 0, st, x, y_ref, claimed, rows, cols, ld,
                               vec_ok, k, alpha, eps_rel, w.hist, w.coarse, w.stats);
        };
        // at most two vectors per thread (the check's binary64 division leaves no room for more
        // under the 128-register limit of a 1024-thread workgroup): longer rows take wider groups
        if (cols <= 256)       launch(softmax_check<64, 1>, 64);
        else if (cols <= 512)  launch(softmax_check<64, 2>, 64);
        else if (cols <= 1024) launch(softmax_check<256, 1>, 256);
        else if (cols <= 2048) launch(softmax_check<256, 2>, 256);
        else if (cols <= 4096) launch(softmax_check<512, 2>, 512);
        else if (cols <= 8192) launch(softmax_check<1024, 2>, 1024);
        else                   launch(softmax_check<1024, 0>, 1024);
    } else {
        // nothing to examine: an empty partial, so that the profile reports n = 0
        hipLaunchKernelGGL((softmax_check<64, 1>), dim3(1), dim3(kCheckThreads), 0, st, x, y_ref, claimed, 0L, 1L, 1L,
                           0, k, alpha, eps_rel, w.hist, w.coarse, w.stats);
    }
    launch_profile_reduce(w, nblocks, (unsigned long long)n, out, st);
    return launch_status();
}

}  // extern "C"
