// tao_bound_act: element-wise bounds for GELU (erf and tanh forms), SiLU / sigmoid,
// one-step arithmetic and library functions, exact operators; tao_bound_rope: the
// rotary embedding (operators of App. A.3, bounded with the primitive rule of
// Sec. 3.1: propagated error through the derivative plus u|f^| fresh rounding per
// step).  One grid-stride streaming pass with 16-byte loads each; HBM-bound.
#include "tao_device.hpp"
#include "tao_host.hpp"
#include "tao_check.hpp"

namespace tao {

struct ActConsts {
    double u;
    double c_erf_u;        // c_erf * u
    double et_f;           // 2u + u^2
    double fresh2;         // u (1 + 1/(1-u)), upper
    double silu_f;         // w/(1-u) + u with w = (c_exp u/(1-c_exp u) + u)/(1-u), upper
    double a_f;            // (2/sqrt pi)(1 + 4u), upper
    double scale_f;        // factor of the one-step kinds: u, or c u/(1 - c u), upper
    double g7;             // Gamma(7), upper (tanh-form GELU: roundings of the polynomial)
    double c_tanh_u;       // c_tanh * u
};
// kernel variants beyond the public kinds' own: every one-step kind is |y| * scale_f
constexpr int kKindScale = 100;

constexpr double kInvSqrt2Up = 0x1.6a09e667f3bcdp-1;     // 1/sqrt(2) rounded up
constexpr double kInvSqrt2Lo = 0x1.6a09e667f3bccp-1;     // 1/sqrt(2) rounded down
constexpr double kTwoRsqrtPiUp = 0x1.20dd750429b6ep+0;   // 2/sqrt(pi) rounded up
constexpr double kBetaUp = 0x1.9884533d43651p-1, kBetaLo = 0x1.9884533d43650p-1;   // sqrt(2/pi)
constexpr double kCubicUp = 0x1.6e4e26d4801f8p-5, kCubicLo = 0x1.6e4e26d4801f7p-5; // 0.044715

// exp(-s) for s >= 0 with relative error below 2^-40 (covered, with the few
// roundings around it, by the guard factor): s = k ln2 + r, |r| <= ln2/2, degree-11
// Taylor polynomial of exp(-r) (remainder 0.35^12/12! < 1e-14), scaled by 2^-k.
__device__ __forceinline__ double exp_neg(double s) {
    if (s > 745.0) return 0x1p-1074;                       // never report exactly 0
    const double kf = rint(s * 0x1.71547652b82fep+0);      // s / ln 2
    const double r = fma(-kf, 0x1.62e42fefa39efp-1, s) - kf * 0x1.abc9e3b39803fp-56;   // s - k ln2
    const double x = -r;
    double p = 1.0 / 39916800.0;
    p = fma(p, x, 1.0 / 3628800.0);
    p = fma(p, x, 1.0 / 362880.0);
    p = fma(p, x, 1.0 / 40320.0);
    p = fma(p, x, 1.0 / 5040.0);
    p = fma(p, x, 1.0 / 720.0);
    p = fma(p, x, 1.0 / 120.0);
    p = fma(p, x, 1.0 / 24.0);
    p = fma(p, x, 1.0 / 6.0);
    p = fma(p, x, 0.5);
    p = fma(p, x, 1.0);
    p = fma(p, x, 1.0);
    return ldexp(p, -(int)kf);
}

template <int KIND>
__device__ __forceinline__ float act_one(float x, float y, const ActConsts& k) {
    const double ay = fabs((double)y);
    double t;
    if (KIND == TAO_ACT_GELU_ERF) {
        const double ax = fabs((double)x);
        if (!(ax <= 0x1.fffffep+127)) return __builtin_nanf("");        // infinite or NaN operand: no bound
        const double ts = ax * kInvSqrt2Up;                      // >= |t*|
        const double E_t = k.et_f * ts;
        double t_lo = ax * kInvSqrt2Lo * (1.0 - 0x1p-52) - E_t;  // <= |t*| - E_t (one ulp of slack
        t_lo = fmax(t_lo * (1.0 - 0x1p-51), 0.0);                //    for the two roundings)
        const double sq_lo = t_lo * t_lo * (1.0 - 0x1p-52);
        const double Gp = kTwoRsqrtPiUp * exp_neg(sq_lo);
        const double A = fmin(k.a_f * ts, 1.0);
        const double E_g = Gp * E_t + k.c_erf_u * A;
        t = 0.5 * ax * E_g + ay * k.fresh2;
    } else if (KIND == TAO_ACT_GELU_TANH) {
        // each product below is rounded to nearest; the factors (1 +- 2^-50) turn the few
        // roundings of a line into an upper or a lower bound
        const double ax = fabs((double)x);
        if (!(ax <= 0x1.fffffep+127)) return __builtin_nanf("");        // infinite or NaN operand: no bound
        const double x2 = ax * ax;                                            // exact (48 bits)
        const double ps = kBetaUp * ax * (1.0 + kCubicUp * x2) * (1.0 + 0x1p-50);   // >= |p*|
        const double p_dn = kBetaLo * ax * (1.0 + kCubicLo * x2) * (1.0 - 0x1p-50); // <= |p*|
        const double E_p = k.g7 * ps * (1.0 + 0x1p-51);
        const double p_lo = fmax((p_dn - E_p) * (1.0 - 0x1p-51), 0.0);
        const double q = fmin(exp_neg(2.0 * p_lo) * (1.0 + 0x1p-39), 1.0);    // >= exp(-2 p_lo)
        const double Gp = fmin(4.0 * q / ((1.0 + q) * (1.0 + q)) * (1.0 + 0x1p-50), 1.0);  // >= sech^2(p_lo)
        const double A = fmin(ps * (1.0 + k.g7) * (1.0 + 0x1p-51), 1.0);
        const double E_T = Gp * E_p + k.c_tanh_u * A;
        t = 0.5 * ax * E_T + ay * k.fresh2;
    } else if (KIND == TAO_ACT_SILU) {
        // one product with a factor that already carries its margin (widened on the host; u itself for
        // the correctly rounded kinds, where the product is exact): nothing is added to a subnormal result
        return up32g(ay * k.silu_f, kUpMul, 1.0);
    } else if (KIND == kKindScale) {
        return up32g(ay * k.scale_f, kUpMul, 1.0);
    } else {
        return 0.f;
    }
    return up32g(t);
}

template <int KIND>
__global__ __launch_bounds__(256) void act_bound(const float* __restrict__ x, const float* __restrict__ y,
                                                  float* __restrict__ tau, long n, int vec_ok, ActConsts k) {
    constexpr bool NEEDS_X = (KIND == TAO_ACT_GELU_ERF || KIND == TAO_ACT_GELU_TANH);
    const long nvec = vec_ok ? (n >> 2) : 0;
    const long stride = (long)gridDim.x * blockDim.x;
    const long t0 = (long)blockIdx.x * blockDim.x + threadIdx.x;
    for (long i = t0; i < nvec; i += stride) {
        float4 X = make_float4(0.f, 0.f, 0.f, 0.f);
        if (NEEDS_X) X = ntload4(reinterpret_cast<const float4*>(x) + i);
        const float4 Y = ntload4(reinterpret_cast<const float4*>(y) + i);
        float4 T;
        T.x = act_one<KIND>(X.x, Y.x, k); T.y = act_one<KIND>(X.y, Y.y, k);
        T.z = act_one<KIND>(X.z, Y.z, k); T.w = act_one<KIND>(X.w, Y.w, k);
        ntstore4(reinterpret_cast<float4*>(tau) + i, T);
    }
    for (long i = (nvec << 2) + t0; i < n; i += stride)
        tau[i] = act_one<KIND>(NEEDS_X ? x[i] : 0.f, y[i], k);
}

// The same bound checked on the spot (Sec. 5.4 / 5.3): the structure of the streaming check pass
// (1024-thread workgroups, one partial histogram each), with tau formed in registers from y (and
// x) instead of loaded -- 8 or 12 bytes per element where the two passes move 20 or 24.
template <int KIND>
__global__ __launch_bounds__(kCheckThreads) void act_check(
    const float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ claimed, long n, int vec_ok,
    ActConsts k, double alpha, double eps_rel,
    unsigned int* __restrict__ ws_hist, unsigned int* __restrict__ ws_coarse, BlockStats* __restrict__ ws_stats) {
    constexpr bool NEEDS_X = (KIND == TAO_ACT_GELU_ERF || KIND == TAO_ACT_GELU_TANH);
    __shared__ unsigned int hist[kBins * kReplicas];
    __shared__ unsigned int red[3 * (kCheckThreads / kWave)];
    const int tid = threadIdx.x;
    for (int i = tid; i < kBins * kReplicas; i += kCheckThreads) hist[i] = 0;
    __syncthreads();
    ThreadAcc acc;
    const int rep = tid & (kReplicas - 1);
    const long nvec = vec_ok ? (n >> 2) : 0;
    const long stride = (long)gridDim.x * kCheckThreads;
    for (long i = (long)blockIdx.x * kCheckThreads + tid; i < nvec; i += stride) {
        float4 X = make_float4(0.f, 0.f, 0.f, 0.f);
        if (NEEDS_X) X = ntload4(reinterpret_cast<const float4*>(x) + i);
        const float4 Y = ntload4(reinterpret_cast<const float4*>(y) + i);
        const float4 C = ntload4(reinterpret_cast<const float4*>(claimed) + i);
        check_one(C.x, Y.x, act_one<KIND>(X.x, Y.x, k), alpha, eps_rel, hist, rep, acc);
        check_one(C.y, Y.y, act_one<KIND>(X.y, Y.y, k), alpha, eps_rel, hist, rep, acc);
        check_one(C.z, Y.z, act_one<KIND>(X.z, Y.z, k), alpha, eps_rel, hist, rep, acc);
        check_one(C.w, Y.w, act_one<KIND>(X.w, Y.w, k), alpha, eps_rel, hist, rep, acc);
    }
    for (long i = (nvec << 2) + (long)blockIdx.x * kCheckThreads + tid; i < n; i += stride)
        check_one(claimed[i], y[i], act_one<KIND>(NEEDS_X ? x[i] : 0.f, y[i], k), alpha, eps_rel, hist, rep, acc);
    flush_block_stats(acc, red, ws_stats);
    flush_histogram(hist, ws_hist + (size_t)blockIdx.x * kBins, ws_coarse + blockIdx.x * kGroups);
}

// Rotary embedding: one thread per output pair and float4 of a half (pairs (j, j + d/2)) or per
// float4 of interleaved pairs.  Tables are read through the cache (every head of a position
// shares a row), activations and bounds stream.  The bounds go to a sink: stored (rope_bound) or
// checked on the spot against the claimed and the re-executed output (rope_check).
struct StoreSink {
    float* tau;
    __device__ __forceinline__ void put4(long idx, float4 t) { ntstore4(reinterpret_cast<float4*>(tau + idx), t); }
    __device__ __forceinline__ void put1(long idx, float t) { tau[idx] = t; }
};
struct CheckSink {
    const float* y; const float* claimed; double alpha, eps_rel; unsigned int* hist; int rep; ThreadAcc acc;
    __device__ __forceinline__ void put1(long idx, float t) { check_one(claimed[idx], y[idx], t, alpha, eps_rel, hist, rep, acc); }
    __device__ __forceinline__ void put4(long idx, float4 t) {
        const float4 Y = ntload4(reinterpret_cast<const float4*>(y + idx));
        const float4 C = ntload4(reinterpret_cast<const float4*>(claimed + idx));
        check_one(C.x, Y.x, t.x, alpha, eps_rel, hist, rep, acc); check_one(C.y, Y.y, t.y, alpha, eps_rel, hist, rep, acc);
        check_one(C.z, Y.z, t.z, alpha, eps_rel, hist, rep, acc); check_one(C.w, Y.w, t.w, alpha, eps_rel, hist, rep, acc);
    }
};

template <bool INTERLEAVED, bool VEC, class Sink>
__device__ __forceinline__ void rope_body(const float* __restrict__ x, const float* __restrict__ cs, const float* __restrict__ sn,
                                          long rows, int d, long inner, long npos, double g2, double uflow, Sink& sink) {
    const int h = d >> 1;
    // work items per row: h/4 vectors of a half, or d/4 vectors of interleaved pairs (2 pairs each);
    // the scalar variants take one pair per item
    const int per_row = VEC ? (INTERLEAVED ? d >> 2 : h >> 2) : h;
    const long total = rows * per_row;
    const long stride = (long)gridDim.x * blockDim.x;
    auto one = [&](float xa, float xb, float c, float s, float& ta, float& tb) {
        const double ca = fabs((double)c), sa = fabs((double)s), a = fabs((double)xa), b = fabs((double)xb);
        ta = up32g(g2 * (a * ca + b * sa) + uflow, kUpMul, 1.0 + 0x1p-48);   // (three round-to-nearest operations)
        tb = up32g(g2 * (b * ca + a * sa) + uflow, kUpMul, 1.0 + 0x1p-48);
    };
    for (long w = (long)blockIdx.x * blockDim.x + threadIdx.x; w < total; w += stride) {
        const long r = w / per_row;
        const int j = (int)(w - r * per_row);
        const long t = (r / inner) % npos;
        const float* xr = x + r * d;
        const long base = r * d;
        const float* cr = cs + t * h; const float* sr = sn + t * h;
        if (VEC && !INTERLEAVED) {
            const float4 A = ntload4(reinterpret_cast<const float4*>(xr) + j);
            const float4 B = ntload4(reinterpret_cast<const float4*>(xr + h) + j);
            const float4 C = reinterpret_cast<const float4*>(cr)[j];
            const float4 S = reinterpret_cast<const float4*>(sr)[j];
            float4 TA, TB;
            one(A.x, B.x, C.x, S.x, TA.x, TB.x); one(A.y, B.y, C.y, S.y, TA.y, TB.y);
            one(A.z, B.z, C.z, S.z, TA.z, TB.z); one(A.w, B.w, C.w, S.w, TA.w, TB.w);
            sink.put4(base + 4L * j, TA);
            sink.put4(base + h + 4L * j, TB);
        } else if (VEC) {
            const float4 X = ntload4(reinterpret_cast<const float4*>(xr) + j);      // pairs 2j, 2j+1
            const float2 C = reinterpret_cast<const float2*>(cr)[j];
            const float2 S = reinterpret_cast<const float2*>(sr)[j];
            float4 T;
            one(X.x, X.y, C.x, S.x, T.x, T.y); one(X.z, X.w, C.y, S.y, T.z, T.w);
            sink.put4(base + 4L * j, T);
        } else {
            const int a = INTERLEAVED ? 2 * j : j, b = INTERLEAVED ? 2 * j + 1 : j + h;
            float ta, tb;
            one(xr[a], xr[b], cr[j], sr[j], ta, tb);
            sink.put1(base + a, ta);
            sink.put1(base + b, tb);
        }
    }
}

template <bool INTERLEAVED, bool VEC>
__global__ __launch_bounds__(256) void rope_bound(const float* __restrict__ x, const float* __restrict__ cs,
                                                   const float* __restrict__ sn, float* __restrict__ tau,
                                                   long rows, int d, long inner, long npos, double g2, double uflow) {
    StoreSink sink{tau};
    rope_body<INTERLEAVED, VEC>(x, cs, sn, rows, d, inner, npos, g2, uflow, sink);
}

template <bool INTERLEAVED, bool VEC>
__global__ __launch_bounds__(kCheckThreads) void rope_check(
    const float* __restrict__ x, const float* __restrict__ cs, const float* __restrict__ sn,
    const float* __restrict__ y, const float* __restrict__ claimed,
    long rows, int d, long inner, long npos, double g2, double uflow, double alpha, double eps_rel,
    unsigned int* __restrict__ ws_hist, unsigned int* __restrict__ ws_coarse, BlockStats* __restrict__ ws_stats) {
    __shared__ unsigned int hist[kBins * kReplicas];
    __shared__ unsigned int red[3 * (kCheckThreads / kWave)];
    for (int i = threadIdx.x; i < kBins * kReplicas; i += kCheckThreads) hist[i] = 0;
    __syncthreads();
    CheckSink sink{y, claimed, alpha, eps_rel, hist, (int)(threadIdx.x & (kReplicas - 1)), ThreadAcc()};
    rope_body<INTERLEAVED, VEC>(x, cs, sn, rows, d, inner, npos, g2, uflow, sink);
    flush_block_stats(sink.acc, red, ws_stats);
    flush_histogram(hist, ws_hist + (size_t)blockIdx.x * kBins, ws_coarse + blockIdx.x * kGroups);
}

}  // namespace tao

extern "C" {

// Validates kind and model and fills the constants of the element-wise kernels.
static int act_setup(int kind, const tao_fp_model* model, tao::ActConsts* out) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (kind < TAO_ACT_GELU_ERF || kind > TAO_ACT_GELU_TANH) return TAO_ERR_KIND;
    const double u = md.u;
    if (!(md.c_exp * u < 0.5)) return TAO_ERR_MODEL;
    ActConsts k;
    k.u = u;
    k.c_erf_u = md.c_erf * u;
    k.et_f = widen(2.0 * u + u * u);
    const double inv1mu = widen(1.0 / (1.0 - u));
    k.fresh2 = widen(u * (1.0 + inv1mu));
    const double c1 = widen(md.c_exp * u / (1.0 - md.c_exp * u));
    const double om = widen((c1 + u) * inv1mu);
    k.silu_f = widen(om * inv1mu + u);
    k.a_f = widen(kTwoRsqrtPiUp * (1.0 + 4.0 * u));
    k.g7 = widen(7.0 * u / (1.0 - 7.0 * u));
    k.c_tanh_u = md.c_tanh * u;
    // one-step kinds: a correctly rounded operation (u), or a library function accurate to c u
    double cf = -1.0;
    switch (kind) {
        case TAO_ACT_DIV: cf = md.c_div; break;    case TAO_ACT_RSQRT: cf = md.c_rsqrt; break;
        case TAO_ACT_EXP: cf = md.c_exp; break;    case TAO_ACT_LOG: cf = md.c_log; break;
        case TAO_ACT_SIN: cf = md.c_sin; break;    case TAO_ACT_COS: cf = md.c_cos; break;
        case TAO_ACT_TANH: cf = md.c_tanh; break;  case TAO_ACT_POW: cf = md.c_pow; break;
        default: break;
    }
    if (cf >= 0.0 && !(cf * u < 0.5)) return TAO_ERR_MODEL;
    k.scale_f = cf >= 0.0 ? widen(cf * u / (1.0 - cf * u)) : u;
    *out = k;
    return TAO_OK;
}

int tao_bound_act(int kind, const float* x, const float* x2, const float* y_ref, float* tau, long n,
                  const tao_fp_model* model, void* stream) {
    using namespace tao;
    (void)x2;
    ActConsts k;
    int rc = act_setup(kind, model, &k);
    if (rc != TAO_OK) return rc;
    if (n < 0) return TAO_ERR_SHAPE;
    if (n == 0) return TAO_OK;
    const bool needs_x = kind == TAO_ACT_GELU_ERF || kind == TAO_ACT_GELU_TANH;
    if (!y_ref || !tau || (needs_x && !x)) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(tau, 4)) return TAO_ERR_ALIGN;
    const int vec_ok = aligned(y_ref, 16) && aligned(tau, 16) && (!needs_x || aligned(x, 16));
    // up to 64 workgroups of 256 threads per CU, grid-stride beyond that (sweeping 2 .. 128 per
    // CU at 8 M .. 100 M elements: the kernels with more arithmetic keep gaining up to 32 - 64)
    long blocks = (n / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 256L * 64) blocks = 256L * 64;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)blocks), blk(256);
    switch (kind) {
        case TAO_ACT_GELU_ERF: hipLaunchKernelGGL(act_bound<TAO_ACT_GELU_ERF>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        case TAO_ACT_GELU_TANH: hipLaunchKernelGGL(act_bound<TAO_ACT_GELU_TANH>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        case TAO_ACT_SILU: case TAO_ACT_SIGMOID:
            hipLaunchKernelGGL(act_bound<TAO_ACT_SILU>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        case TAO_ACT_RELU: case TAO_ACT_EXACT:
            hipLaunchKernelGGL(act_bound<TAO_ACT_RELU>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        default:        // MUL, ADD, SUB, SQRT and the library functions
            hipLaunchKernelGGL(act_bound<kKindScale>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
    }
    return launch_status();
}

int tao_bound_check_act(int kind, const float* x, const float* x2, const float* y_ref, const float* claimed,
                        long n, double alpha, double eps_rel, const tao_fp_model* model, tao_profile* out,
                        void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    (void)x2;
    ActConsts k;
    int rc = act_setup(kind, model, &k);
    if (rc != TAO_OK) return rc;
    if (!out || !ws) return out ? TAO_ERR_WORKSPACE : TAO_ERR_NULL;
    if (n < 0 || n >= (1L << 36) || !(alpha >= 0.0) || !std::isfinite(alpha) || !(eps_rel >= 0.0) || !std::isfinite(eps_rel))
        return TAO_ERR_SHAPE;
    const bool needs_x = kind == TAO_ACT_GELU_ERF || kind == TAO_ACT_GELU_TANH;
    if (n > 0 && (!y_ref || !claimed || (needs_x && !x))) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(claimed, 4) || !aligned(out, 8)) return TAO_ERR_ALIGN;
    if (!aligned(ws, 256) || ws_bytes < check_workspace_bytes()) return TAO_ERR_WORKSPACE;
    const int vec_ok = aligned(y_ref, 16) && aligned(claimed, 16) && (!needs_x || aligned(x, 16));
    long want = (n + (long)kCheckThreads * 16 - 1) / ((long)kCheckThreads * 16);
    const int nblocks = (int)(want < 1 ? 1 : (want > kMaxCheckBlocks ? kMaxCheckBlocks : want));
    const CheckWorkspace w = carve_check_workspace(ws);
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)nblocks), blk(kCheckThreads);
#define TAO_ACT_CHECK(K) hipLaunchKernelGGL(act_check<K>, grid, blk, 0, st, x, y_ref, claimed, n, vec_ok, k, alpha, eps_rel, \
                                            w.hist, w.coarse, w.stats)
    switch (kind) {
        case TAO_ACT_GELU_ERF: TAO_ACT_CHECK(TAO_ACT_GELU_ERF); break;
        case TAO_ACT_GELU_TANH: TAO_ACT_CHECK(TAO_ACT_GELU_TANH); break;
        case TAO_ACT_SILU: case TAO_ACT_SIGMOID: TAO_ACT_CHECK(TAO_ACT_SILU); break;
        case TAO_ACT_RELU: case TAO_ACT_EXACT: TAO_ACT_CHECK(TAO_ACT_RELU); break;
        default: TAO_ACT_CHECK(kKindScale); break;
    }
#undef TAO_ACT_CHECK
    launch_profile_reduce(w, nblocks, (unsigned long long)n, out, st);
    return launch_status();
}

int tao_bound_rope(const float* x, const float* cos_table, const float* sin_table, float* tau,
                   long rows, long d, long inner, long npos, int interleaved,
                   const tao_fp_model* model, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (rows < 0 || d < 0 || (d & 1) || inner < 1 || npos < 1 || d >= (1L << 30)) return TAO_ERR_SHAPE;
    const double g2 = gamma_up(2, md);
    if (!(g2 == g2)) return TAO_ERR_K_RANGE;
    if (rows == 0 || d == 0) return TAO_OK;
    if (!x || !cos_table || !sin_table || !tau) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(cos_table, 4) || !aligned(sin_table, 4) || !aligned(tau, 4)) return TAO_ERR_ALIGN;
    const double uflow = (md.flags & TAO_FLAG_UNDERFLOW_TERMS) ? 2.0 * 0x1p-149 : 0.0;
    // 16-byte accesses: rows and halves 16-byte aligned (d a multiple of 8; of 4 when interleaved)
    const bool vec = aligned(x, 16) && aligned(tau, 16) && aligned(cos_table, 16) && aligned(sin_table, 16) &&
                     (interleaved ? d % 4 == 0 : d % 8 == 0);
    const long per_row = vec ? (interleaved ? d / 4 : d / 8) : d / 2;
    long blocks = (rows * per_row + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 256L * 64) blocks = 256L * 64;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)blocks), blk(256);
    if (interleaved) {
        if (vec) hipLaunchKernelGGL((rope_bound<true, true>), grid, blk, 0, st, x, cos_table, sin_table, tau, rows, (int)d, inner, npos, g2, uflow);
        else     hipLaunchKernelGGL((rope_bound<true, false>), grid, blk, 0, st, x, cos_table, sin_table, tau, rows, (int)d, inner, npos, g2, uflow);
    } else {
        if (vec) hipLaunchKernelGGL((rope_bound<false, true>), grid, blk, 0, st, x, cos_table, sin_table, tau, rows, (int)d, inner, npos, g2, uflow);
        else     hipLaunchKernelGGL((rope_bound<false, false>), grid, blk, 0, st, x, cos_table, sin_table, tau, rows, (int)d, inner, npos, g2, uflow);
    }
    return launch_status();
}

int tao_bound_check_rope(const float* x, const float* cos_table, const float* sin_table, const float* y_ref,
                         const float* claimed, long rows, long d, long inner, long npos, int interleaved,
                         double alpha, double eps_rel, const tao_fp_model* model, tao_profile* out,
                         void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (!out || !ws) return out ? TAO_ERR_WORKSPACE : TAO_ERR_NULL;
    if (rows < 0 || d < 0 || (d & 1) || inner < 1 || npos < 1 || d >= (1L << 30)) return TAO_ERR_SHAPE;
    if (!(alpha >= 0.0) || !std::isfinite(alpha) || !(eps_rel >= 0.0) || !std::isfinite(eps_rel)) return TAO_ERR_SHAPE;
    if (rows > 0 && d > 0 && rows > ((1L << 36) - 1) / d) return TAO_ERR_SHAPE;   // 32-bit per-workgroup counters
    const double g2 = gamma_up(2, md);
    if (!(g2 == g2)) return TAO_ERR_K_RANGE;
    const long n = rows * d;
    if (n > 0 && (!x || !cos_table || !sin_table || !y_ref || !claimed)) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(cos_table, 4) || !aligned(sin_table, 4) || !aligned(y_ref, 4) || !aligned(claimed, 4) ||
        !aligned(out, 8)) return TAO_ERR_ALIGN;
    if (!aligned(ws, 256) || ws_bytes < check_workspace_bytes()) return TAO_ERR_WORKSPACE;
    const double uflow = (md.flags & TAO_FLAG_UNDERFLOW_TERMS) ? 2.0 * 0x1p-149 : 0.0;
    const bool vec = aligned(x, 16) && aligned(y_ref, 16) && aligned(claimed, 16) && aligned(cos_table, 16) &&
                     aligned(sin_table, 16) && (interleaved ? d % 4 == 0 : d % 8 == 0);
    const long per_row = vec ? (interleaved ? d / 4 : d / 8) : d / 2;
    long want = (rows * per_row + (long)kCheckThreads * 4 - 1) / ((long)kCheckThreads * 4);
    const int nblocks = (int)(want < 1 ? 1 : (want > kMaxCheckBlocks ? kMaxCheckBlocks : want));
    const CheckWorkspace w = carve_check_workspace(ws);
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)nblocks), blk(kCheckThreads);
#define TAO_ROPE_CHECK(I, V) hipLaunchKernelGGL((rope_check<I, V>), grid, blk, 0, st, x, cos_table, sin_table, y_ref, claimed, \
                                                rows, (int)d, inner, npos, g2, uflow, alpha, eps_rel, w.hist, w.coarse, w.stats)
    if (interleaved) { if (vec) TAO_ROPE_CHECK(true, true); else TAO_ROPE_CHECK(true, false); }
    else             { if (vec) TAO_ROPE_CHECK(false, true); else TAO_ROPE_CHECK(false, false); }
#undef TAO_ROPE_CHECK
    launch_profile_reduce(w, nblocks, (unsigned long long)n, out, st);
    return launch_status();
}

}  // extern "C"
