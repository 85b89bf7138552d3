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

// Shape checks of a 2-D convolution (channels-last input [batch][H][W][C], filters [Cout][R][S][C]) and the
// shape of its implicit patch-matrix product: M = batch OH OW rows, K = R S C columns.
inline int conv_geometry(long batch, long H, long W, long C, long Cout, long R, long S,
                         long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w,
                         long* OH, long* OW, long* M, long* K) {
    if (batch < 0 || H < 0 || W < 0 || C < 0 || Cout < 0 || R < 1 || S < 1) return TAO_ERR_SHAPE;
    if (stride_h < 1 || stride_w < 1 || dil_h < 1 || dil_w < 1 || pad_h < 0 || pad_w < 0) return TAO_ERR_SHAPE;
    const long lim = 1L << 28;       // each extent, so that coordinate arithmetic stays in 32 bits
    if (H >= lim || W >= lim || C >= lim || R >= lim || S >= lim || Cout >= lim || batch >= lim ||
        stride_h >= lim || stride_w >= lim || dil_h >= lim || dil_w >= lim || pad_h >= lim || pad_w >= lim) return TAO_ERR_SHAPE;
    if (dil_h * (R - 1) >= lim || dil_w * (S - 1) >= lim) return TAO_ERR_SHAPE;
    const long eh = H + 2 * pad_h - dil_h * (R - 1) - 1, ew = W + 2 * pad_w - dil_w * (S - 1) - 1;
    if (eh < 0 || ew < 0) return TAO_ERR_SHAPE;          // filter larger than the padded input
    *OH = eh / stride_h + 1; *OW = ew / stride_w + 1;
    const __int128 M128 = (__int128)batch * *OH * *OW, K128 = (__int128)R * S * C;
    if (M128 >= (1L << 31) || K128 >= (1L << 31) || *OH * *OW >= (1L << 31)) return TAO_ERR_SHAPE;
    *M = (long)M128; *K = (long)K128;
    if ((__int128)batch * H * W * C >= ((__int128)1 << 61) || (__int128)*M * Cout >= ((__int128)1 << 61)) return TAO_ERR_SHAPE;
    return TAO_OK;
}

// Every kernel evaluates its formula in round-to-nearest binary64; a margin that dominates the
// accumulated binary64 rounding keeps the emitted bound at or above the real-number value.  The
// matrix kernel multiplies by this factor and rounds up exactly (up32); the streaming kernels fold
// a margin into their upper rounding (up32g): a fixed one for element-wise work, one that grows
// with the row length ((cols + 130) 2^-51, at least 2^-33) for the row kernels.
constexpr double kGuard = 1.0 + 0x1p-32;

}  // namespace tao
