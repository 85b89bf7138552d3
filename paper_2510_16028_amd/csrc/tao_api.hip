// Entry points that need no kernel of their own: model defaults, Gamma on the
// host, status strings, and the helpers declared in tao_host.hpp.
#include "tao_host.hpp"

namespace tao {

thread_local int g_last_hip_error = 0;

int resolve_model(const tao_fp_model* m, tao_fp_model* out) {
    if (!m) { tao_default_model(out); return TAO_OK; }
    *out = *m;
    auto ok = [](double c) { return std::isfinite(c) && c >= 0.0; };
    if (!(out->u > 0.0) || !(out->u <= 0x1p-10)) return TAO_ERR_MODEL;
    if (out->mode != TAO_MODE_DETERMINISTIC && out->mode != TAO_MODE_PROBABILISTIC) return TAO_ERR_MODEL;
    if (out->mode == TAO_MODE_PROBABILISTIC && !(std::isfinite(out->lambda) && out->lambda > 0.0))
        return TAO_ERR_MODEL;
    if (!ok(out->c_exp) || !ok(out->c_erf) || !ok(out->c_rsqrt) || !ok(out->c_div)) return TAO_ERR_MODEL;
    if (!ok(out->c_log) || !ok(out->c_sin) || !ok(out->c_cos) || !ok(out->c_tanh) || !ok(out->c_pow)) return TAO_ERR_MODEL;
    if (out->flags & ~(TAO_FLAG_UNDERFLOW_TERMS | TAO_FLAG_FAST_ACCUM | TAO_FLAG_CHECK_IN_EPILOGUE)) return TAO_ERR_MODEL;
    return TAO_OK;
}

// gamma_k = k u / (1 - k u) (App. A.1 Eq. gamma-def); gamma~_k(lambda) =
// exp(lambda sqrt(k) u + k u^2/(1-u)) - 1 (Sec. 3.1, App. A.2).
double gamma_up(long k, const tao_fp_model& m) {
    if (k <= 0) return 0.0;
    if (m.mode == TAO_MODE_DETERMINISTIC) {
        double ku = (double)k * m.u;
        if (!(ku < 1.0)) return NAN;
        double den = (1.0 - ku) * (1.0 - 0x1p-52);
        return widen(ku / den);
    }
    double arg = widen(m.lambda * std::sqrt((double)k) * m.u) + widen((double)k * m.u * m.u / (1.0 - m.u));
    arg = widen(arg);
    if (!(arg < 1.0)) return NAN;
    return widen(std::expm1(arg));
}

}  // namespace tao

extern "C" {

void tao_default_model(tao_fp_model* m) {
    if (!m) return;
    m->u = 0x1p-24;
    m->mode = TAO_MODE_DETERMINISTIC;
    m->lambda = 4.0;
    m->c_exp = 2.0; m->c_erf = 2.0; m->c_rsqrt = 2.0; m->c_div = 2.0;
    m->flags = 0;
    m->c_log = 2.0; m->c_sin = 4.0; m->c_cos = 4.0; m->c_tanh = 4.0; m->c_pow = 8.0;
}

double tao_gamma(long k, const tao_fp_model* model) {
    tao_fp_model md;
    if (tao::resolve_model(model, &md) != TAO_OK) return NAN;
    return tao::gamma_up(k, md);
}

int tao_last_hip_error(void) { return tao::g_last_hip_error; }

const char* tao_status_string(int s) {
    switch (s) {
        case TAO_OK: return "ok";
        case TAO_ERR_NULL: return "required pointer is NULL";
        case TAO_ERR_SHAPE: return "bad shape, leading dimension or stride";
        case TAO_ERR_ALIGN: return "pointer not sufficiently aligned";
        case TAO_ERR_K_RANGE: return "reduction depth k with k*u >= 1: gamma_k undefined";
        case TAO_ERR_MODEL: return "tao_fp_model field out of range";
        case TAO_ERR_KIND: return "unknown operator kind";
        case TAO_ERR_LAUNCH: return "HIP error (see tao_last_hip_error)";
        case TAO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        default: return "unknown status";
    }
}

}  // extern "C"
