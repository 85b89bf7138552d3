// Pieces of the leaf check (Sec. 5.4) and relative-error profile (Sec. 5.3; Sec. 3.2 Eq. 2) shared by
// the streaming check pass and by bound kernels that check their bound in registers instead of
// storing it: the per-element step, the per-workgroup counters, the workspace layout and the
// launch of the finalising kernel.
#pragma once
#include "tao_hist.hpp"
#include "tao_host.hpp"

namespace tao {

constexpr int kCheckThreads = 1024;          // one workgroup per CU: one partial histogram per CU
constexpr int kMaxCheckBlocks = kMaxPartials;
constexpr int kReduceBlocks = kGroups;

struct BlockStats {          // one per pass-1 workgroup, in the workspace after the histograms
    unsigned long long violations;
    unsigned long long nans;
    unsigned int max_bits;   // bit pattern of the largest non-NaN error (errors are >= 0)
    unsigned int pad;
};

struct ThreadAcc {
    unsigned int violations = 0, nans = 0, max_bits = 0;
};

// The arithmetic of one element: violation flag, bin of the relative error, its bits.  A claimed
// value that equals the re-executed one bit for bit (and is finite) has d = 0 exactly, so the error is
// 0 (NaN for 0/0) without the binary64 division; whole wavefronts of such elements -- the masked
// half of a causal softmax, exact operators -- skip the division's instructions altogether.
// SHORTCUT = false leaves the test out: straight-line code, which a caller that unrolls many elements
// (the matrix kernel's epilogue) wants more than the shortcut.
struct CheckedElement { bool violation, is_nan; unsigned int bin, bits; };
template <bool SHORTCUT = true>
__device__ __forceinline__ CheckedElement check_arith(float c, float r, float t, double alpha, double eps_rel) {
    CheckedElement o;
    const double rd = (double)r;
    const double T = alpha * (double)t;
    const double den = fabs(rd) + eps_rel;
    if (SHORTCUT && c == r && fabsf(c) != INFINITY) {
        o.violation = !(0.0 <= T);
        o.is_nan = !(den > 0.0);                             // 0/0
        o.bits = 0u;
        o.bin = o.is_nan ? (unsigned)(kBins - 1) : 0u;
        return o;
    }
    const double d = fabs((double)c - rd);
    o.violation = !(d <= T);
    const double e = d / den;
    const float e32 = (float)e;
    o.bin = error_bin(e32, o.is_nan);
    o.bits = __float_as_uint(e32);
    return o;
}

// Four elements at once, as straight-line code: the four chains of dependent binary64 operations are
// independent of one another, so the compiler interleaves them and a wavefront does not sit out the
// latency of every operation of every element in turn (element by element, each behind its own test
// for the shortcut, that is what happened).  The shortcut is taken for the four together or not at
// all; the full arithmetic returns the shortcut's result for an element that qualifies (d = 0, e = 0 or
// 0/0), so the profile does not depend on the route.
template <int R = kReplicas>
__device__ __forceinline__ void check_four(const float (&c)[4], const float (&r)[4], const float (&t)[4], double alpha,
                                           double eps_rel, unsigned int* hist, int rep, ThreadAcc& acc) {
    bool same = true;
#pragma unroll
    for (int i = 0; i < 4; ++i) same = same && c[i] == r[i] && fabsf(c[i]) != INFINITY;
    CheckedElement o[4];
    if (same) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = check_arith<true>(c[i], r[i], t[i], alpha, eps_rel);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = check_arith<false>(c[i], r[i], t[i], alpha, eps_rel);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc.violations += o[i].violation;
        acc.nans += o[i].is_nan;
        acc.max_bits = max(acc.max_bits, o[i].is_nan ? 0u : o[i].bits);
        atomicAdd(&hist[o[i].bin * R + rep], 1u);
    }
}

// R: copies of every bin in the LDS histogram `hist` (copy `rep` is used).
template <int R = kReplicas>
__device__ __forceinline__ void check_one(float c, float r, float t, double alpha, double eps_rel,
                                          unsigned int* hist, int rep, ThreadAcc& acc) {
    const CheckedElement o = check_arith(c, r, t, alpha, eps_rel);
    acc.violations += o.violation;
    acc.nans += o.is_nan;
    if (!o.is_nan) acc.max_bits = max(acc.max_bits, o.bits);
    atomicAdd(&hist[o.bin * R + rep], 1u);
}

// Workgroup totals of the per-thread counters (kCheckThreads threads) into ws_stats[blockIdx.x];
// red: 3 * (kCheckThreads / kWave) words of LDS.  Contains one barrier.
__device__ __forceinline__ void flush_block_stats(const ThreadAcc& acc, unsigned int* red, BlockStats* __restrict__ ws_stats) {
    const int tid = threadIdx.x;
    unsigned int v = acc.violations, q = acc.nans, m = acc.max_bits;
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        v += __shfl_xor(v, o, kWave);
        q += __shfl_xor(q, o, kWave);
        m = max(m, (unsigned int)__shfl_xor(m, o, kWave));
    }
    const int wave = tid / kWave;
    if ((tid & (kWave - 1)) == 0) { red[wave * 3] = v; red[wave * 3 + 1] = q; red[wave * 3 + 2] = m; }
    __syncthreads();
    if (tid == 0) {
        BlockStats s{0, 0, 0, 0};
        for (int w = 0; w < kCheckThreads / kWave; ++w) {
            s.violations += red[w * 3]; s.nans += red[w * 3 + 1];
            s.max_bits = max(s.max_bits, red[w * 3 + 2]);
        }
        ws_stats[blockIdx.x] = s;
    }
}

// The caller's workspace: kMaxCheckBlocks partial histograms, their coarse group counts, the counters.
struct CheckWorkspace {
    unsigned int* hist; unsigned int* coarse; BlockStats* stats;
};
constexpr size_t check_workspace_bytes() {
    return (size_t)kMaxCheckBlocks * ((kBins + kGroups) * sizeof(unsigned int) + sizeof(BlockStats));
}
inline CheckWorkspace carve_check_workspace(void* ws) {
    CheckWorkspace w;
    w.hist = (unsigned int*)ws;
    w.coarse = w.hist + (size_t)kMaxCheckBlocks * kBins;
    w.stats = (BlockStats*)(w.coarse + (size_t)kMaxCheckBlocks * kGroups);
    return w;
}
// Enqueue the finalising kernel over the partials of `nblocks` pass-1 workgroups (defined with the check pass).
void launch_profile_reduce(const CheckWorkspace& w, int nblocks, unsigned long long n, tao_profile* out, hipStream_t st);

}  // namespace tao
