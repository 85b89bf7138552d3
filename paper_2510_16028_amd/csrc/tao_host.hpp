// Host-side helpers of the C ABI: status handling, model validation and the
// scalar constants (Gamma, guard factors) that the kernels take as arguments.
#pragma once
#include <hip/hip_runtime.h>
#include <cmath>
#include <atomic>
#include <cstdint>
#include "tao.h"

namespace tao {

extern thread_local int g_last_hip_error;

// Per-device "done once" mark for settings that a device keeps (the dynamic LDS limit of a kernel):
// bit d of `done` is set once device d has them.  Two threads that race both apply the setting,
// which is idempotent.
struct OncePerDevice {
    std::atomic<unsigned long long> done{0};
    template <class F> hipError_t run(F&& apply) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const unsigned long long bit = 1ull << (dev & 63);
        if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
        e = apply();
        if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
        return e;
    }
};

inline int launch_status() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { g_last_hip_error = (int)e; return TAO_ERR_LAUNCH; }
    return TAO_OK;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Returns TAO_OK and fills *out with the validated model (defaults when m == NULL).
int resolve_model(const tao_fp_model* m, tao_fp_model* out);

// Upper enclosures in binary64 (round-to-nearest evaluation widened by a few ulps).
double gamma_up(long k, const tao_fp_model& m);            // NaN when undefined
inline double widen(double v) { return v * (1.0 + 0x1p-49); }   // for v >= 0

// Every kernel evaluates its formula in round-to-nearest binary64; a margin that dominates the
// accumulated binary64 rounding keeps the emitted bound at or above the real-number value.  The
// matrix kernel multiplies by this factor and rounds up exactly (up32); the streaming kernels fold
// a margin into their upper rounding (up32g): a fixed one for element-wise work, one that grows
// with the row length ((cols + 130) 2^-51, at least 2^-33) for the row kernels.
constexpr double kGuard = 1.0 + 0x1p-32;

}  // namespace tao
