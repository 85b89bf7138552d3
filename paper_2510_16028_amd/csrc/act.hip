// tao_bound_act: element-wise bounds for GELU (erf form), SiLU, Mul/Add and ReLU
// (operators of App. A.3, bounded with the primitive rule of Sec. 3.1: propagated
// error through the derivative plus u|f^| fresh rounding per step).  One
// grid-stride streaming pass with 16-byte loads; HBM-bound.
#include "tao_device.hpp"
#include "tao_host.hpp"

namespace tao {

struct ActConsts {
    double u;
    double c_erf_u;        // c_erf * u
    double et_f;           // 2u + u^2
    double fresh2;         // u (1 + 1/(1-u)), upper
    double silu_f;         // w/(1-u) + u with w = (c_exp u/(1-c_exp u) + u)/(1-u), upper
    double a_f;            // (2/sqrt pi)(1 + 4u), upper
};

constexpr double kInvSqrt2Up = 0x1.6a09e667f3bcdp-1;     // 1/sqrt(2) rounded up
constexpr double kInvSqrt2Lo = 0x1.6a09e667f3bccp-1;     // 1/sqrt(2) rounded down
constexpr double kTwoRsqrtPiUp = 0x1.20dd750429b6ep+0;   // 2/sqrt(pi) rounded up

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
        const double ts = ax * kInvSqrt2Up;                      // >= |t*|
        const double E_t = k.et_f * ts;
        double t_lo = ax * kInvSqrt2Lo * (1.0 - 0x1p-52) - E_t;  // <= |t*| - E_t (one ulp of slack
        t_lo = fmax(t_lo * (1.0 - 0x1p-51), 0.0);                //    for the two roundings)
        const double sq_lo = t_lo * t_lo * (1.0 - 0x1p-52);
        const double Gp = kTwoRsqrtPiUp * exp_neg(sq_lo);
        const double A = fmin(k.a_f * ts, 1.0);
        const double E_g = Gp * E_t + k.c_erf_u * A;
        t = 0.5 * ax * E_g + ay * k.fresh2;
    } else if (KIND == TAO_ACT_SILU) {
        t = ay * k.silu_f;
    } else if (KIND == TAO_ACT_MUL || KIND == TAO_ACT_ADD) {
        t = k.u * ay;
    } else {
        return 0.f;
    }
    return up32g(t);
}

template <int KIND>
__global__ __launch_bounds__(256) void act_bound(const float* __restrict__ x, const float* __restrict__ y,
                                                  float* __restrict__ tau, long n, int vec_ok, ActConsts k) {
    constexpr bool NEEDS_X = (KIND == TAO_ACT_GELU_ERF);
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

}  // namespace tao

extern "C" {

int tao_bound_act(int kind, const float* x, const float* x2, const float* y_ref, float* tau, long n,
                  const tao_fp_model* model, void* stream) {
    using namespace tao;
    (void)x2;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (kind < TAO_ACT_GELU_ERF || kind > TAO_ACT_RELU) return TAO_ERR_KIND;
    if (n < 0) return TAO_ERR_SHAPE;
    if (n == 0) return TAO_OK;
    if (!y_ref || !tau || (kind == TAO_ACT_GELU_ERF && !x)) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y_ref, 4) || !aligned(tau, 4)) return TAO_ERR_ALIGN;
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
    const int vec_ok = aligned(y_ref, 16) && aligned(tau, 16) && (kind != TAO_ACT_GELU_ERF || aligned(x, 16));
    // up to 64 workgroups of 256 threads per CU, grid-stride beyond that (sweeping 2 .. 128 per
    // CU at 8 M .. 100 M elements: the kernels with more arithmetic keep gaining up to 32 - 64)
    long blocks = (n / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 256L * 64) blocks = 256L * 64;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)blocks), blk(256);
    switch (kind) {
        case TAO_ACT_GELU_ERF: hipLaunchKernelGGL(act_bound<TAO_ACT_GELU_ERF>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        case TAO_ACT_SILU: hipLaunchKernelGGL(act_bound<TAO_ACT_SILU>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        case TAO_ACT_MUL: hipLaunchKernelGGL(act_bound<TAO_ACT_MUL>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        case TAO_ACT_ADD: hipLaunchKernelGGL(act_bound<TAO_ACT_ADD>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
        default: hipLaunchKernelGGL(act_bound<TAO_ACT_RELU>, grid, blk, 0, st, x, y_ref, tau, n, vec_ok, k); break;
    }
    return launch_status();
}

}  // extern "C"
