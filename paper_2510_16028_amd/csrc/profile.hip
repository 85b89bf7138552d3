// tao_profile_errors: absolute and relative element-wise errors between two outputs of one
// operator (Sec. 3.2 Eq. 1-2), their percentile profiles on the 22-point grid
// P = {1, 5, 10, ..., 95, 99, 100} (Sec. 3.2 / Sec. 5.3) and the selection statistic
//     p_max = max_p { p_abs(p)/thr_abs(p), p_rel(p)/thr_rel(p) },   offending iff p_max > 1
// that the dispute game uses to pick the child to descend into (Sec. 5.3).
//
// Pass 1 (errors_pass): grid-stride over 16-byte vectors of both inputs; per element IEEE
// binary64 arithmetic (no contraction), two lane-replicated 2048-bin LDS histograms, partial
// histograms and counters to the workspace (no global atomics: the result does not depend on
// scheduling).  Pass 2 (errors_reduce): one workgroup per 64 bins of either histogram sums the
// partials and locates the 22 nearest-rank percentiles.  Pass 3 (errors_finalize, one small
// workgroup): exact maxima, percentile values capped by the maximum, threshold ratios.
#include "tao_hist.hpp"
#include "tao_host.hpp"

namespace tao {

constexpr int kErrThreads = 1024;            // one workgroup per CU
constexpr int kErrReplicas = 4;              // two histograms of 4 x 2048 counters: 64 KB of LDS
constexpr int kGrid = TAO_NGRID;

struct ErrStats {            // one per pass-1 workgroup
    unsigned long long nans;
    unsigned int max_abs_bits, max_rel_bits;   // bit patterns of the largest non-NaN errors (>= 0)
};

__device__ __forceinline__ unsigned int grid_percent(int g) {
    return g == 0 ? 1u : (g <= 19 ? 5u * (unsigned)g : (g == 20 ? 99u : 100u));
}

__device__ __forceinline__ void error_one(float c, float r, double eps_rel, unsigned int* hist_a,
                                          unsigned int* hist_r, int rep, unsigned int& nans,
                                          unsigned int& max_a, unsigned int& max_r) {
    const double cd = (double)c, rd = (double)r;
    const double d = fabs(cd - rd);
    const double den = fabs(rd) + eps_rel;
    const double e = d / den;
    const float a32 = (float)d, e32 = (float)e;
    bool an, en;
    const unsigned int ba = error_bin(a32, an), be = error_bin(e32, en);
    nans += en;
    if (!en) max_r = max(max_r, __float_as_uint(e32));
    if (!an) max_a = max(max_a, __float_as_uint(a32));
    atomicAdd(&hist_a[ba * kErrReplicas + rep], 1u);
    atomicAdd(&hist_r[be * kErrReplicas + rep], 1u);
}

__global__ __launch_bounds__(kErrThreads) void errors_pass(
    const float* __restrict__ claimed, const float* __restrict__ ref, long n, int vec_ok, double eps_rel,
    unsigned int* __restrict__ ws_hist_a, unsigned int* __restrict__ ws_hist_r,
    unsigned int* __restrict__ ws_coarse_a, unsigned int* __restrict__ ws_coarse_r,
    ErrStats* __restrict__ ws_stats) {
    __shared__ unsigned int hist_a[kBins * kErrReplicas], hist_r[kBins * kErrReplicas];
    __shared__ unsigned int red[3 * (kErrThreads / kWave)];
    const int tid = threadIdx.x;
    for (int i = tid; i < kBins * kErrReplicas; i += kErrThreads) { hist_a[i] = 0; hist_r[i] = 0; }
    __syncthreads();

    unsigned int nans = 0, max_a = 0, max_r = 0;
    const int rep = tid & (kErrReplicas - 1);
    const long nvec = vec_ok ? (n >> 2) : 0;
    const long stride = (long)gridDim.x * kErrThreads;
    for (long i = (long)blockIdx.x * kErrThreads + tid; i < nvec; i += stride) {
        const float4 c4 = ntload4(reinterpret_cast<const float4*>(claimed) + i);
        const float4 r4 = ntload4(reinterpret_cast<const float4*>(ref) + i);
        error_one(c4.x, r4.x, eps_rel, hist_a, hist_r, rep, nans, max_a, max_r);
        error_one(c4.y, r4.y, eps_rel, hist_a, hist_r, rep, nans, max_a, max_r);
        error_one(c4.z, r4.z, eps_rel, hist_a, hist_r, rep, nans, max_a, max_r);
        error_one(c4.w, r4.w, eps_rel, hist_a, hist_r, rep, nans, max_a, max_r);
    }
    // scalar remainder (everything when the inputs are not 16-byte aligned)
    for (long i = (nvec << 2) + (long)blockIdx.x * kErrThreads + tid; i < n; i += stride)
        error_one(claimed[i], ref[i], eps_rel, hist_a, hist_r, rep, nans, max_a, max_r);

#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        nans += __shfl_xor(nans, o, kWave);
        max_a = max(max_a, (unsigned int)__shfl_xor(max_a, o, kWave));
        max_r = max(max_r, (unsigned int)__shfl_xor(max_r, o, kWave));
    }
    const int wave = tid / kWave;
    if ((tid & (kWave - 1)) == 0) { red[wave * 3] = nans; red[wave * 3 + 1] = max_a; red[wave * 3 + 2] = max_r; }
    __syncthreads();
    if (tid == 0) {
        ErrStats s{0, 0, 0};
        for (int w = 0; w < kErrThreads / kWave; ++w) {
            s.nans += red[w * 3];
            s.max_abs_bits = max(s.max_abs_bits, red[w * 3 + 1]);
            s.max_rel_bits = max(s.max_rel_bits, red[w * 3 + 2]);
        }
        ws_stats[blockIdx.x] = s;
    }
    flush_histogram<kErrReplicas>(hist_a, ws_hist_a + (size_t)blockIdx.x * kBins, ws_coarse_a + blockIdx.x * kGroups);
    flush_histogram<kErrReplicas>(hist_r, ws_hist_r + (size_t)blockIdx.x * kBins, ws_coarse_r + blockIdx.x * kGroups);
}

// workgroups 0 .. 31: absolute-error histogram; 32 .. 63: relative-error histogram
__global__ __launch_bounds__(kReduceThreads) void errors_reduce(
    const unsigned int* __restrict__ ws_hist_a, const unsigned int* __restrict__ ws_hist_r,
    const unsigned int* __restrict__ ws_coarse_a, const unsigned int* __restrict__ ws_coarse_r,
    int nblocks, unsigned long long n, tao_error_profile* out) {
    __shared__ unsigned long long smem[kReduceThreads + kReduceWaves];
    RankQuery q[kGrid];
#pragma unroll
    for (int g = 0; g < kGrid; ++g) { q[g].num = grid_percent(g); q[g].den = 100u; }
    const bool rel = blockIdx.x >= (unsigned)kGroups;
    const int grp = rel ? blockIdx.x - kGroups : blockIdx.x;
    if (!rel) reduce_group<kGrid>(ws_hist_a, ws_coarse_a, nblocks, grp, n, out->hist_abs, q, out->abs_bin, out->abs_p, smem);
    else      reduce_group<kGrid>(ws_hist_r, ws_coarse_r, nblocks, grp, n, out->hist_rel, q, out->rel_bin, out->rel_p, smem);
}

__global__ __launch_bounds__(256) void errors_finalize(const ErrStats* __restrict__ ws_stats, int nblocks,
                                                        unsigned long long n, const float* __restrict__ thr_abs,
                                                        const float* __restrict__ thr_rel, tao_error_profile* out) {
    __shared__ unsigned long long wq[4];
    __shared__ unsigned int wa[4], wr[4];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    unsigned long long qn = 0; unsigned int ma = 0, mr = 0;
    for (int k = tid; k < nblocks; k += 256) {
        qn += ws_stats[k].nans; ma = max(ma, ws_stats[k].max_abs_bits); mr = max(mr, ws_stats[k].max_rel_bits);
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        qn += __shfl_xor(qn, o, kWave);
        ma = max(ma, (unsigned int)__shfl_xor(ma, o, kWave));
        mr = max(mr, (unsigned int)__shfl_xor(mr, o, kWave));
    }
    if (lane == 0) { wq[wave] = qn; wa[wave] = ma; wr[wave] = mr; }
    __syncthreads();
    if (tid != 0) return;
    qn = 0; ma = 0; mr = 0;
    for (int w = 0; w < 4; ++w) { qn += wq[w]; ma = max(ma, wa[w]); mr = max(mr, wr[w]); }
    const float max_abs = __uint_as_float(ma), max_rel = __uint_as_float(mr);
    out->n = n; out->nan_count = qn; out->max_abs = max_abs; out->max_rel = max_rel; out->pad_ = 0;
    double pmax = NAN;
    for (int g = 0; g < kGrid; ++g) {
        unsigned int ba = out->abs_bin[g], br = out->rel_bin[g];
        float pa = out->abs_p[g], pr = out->rel_p[g];
        if (n == 0) { ba = br = 0; pa = pr = bin_upper_edge(0); }
        // a percentile cannot exceed the exact maximum (p = 100 is the maximum itself)
        if (n > 0 && ba < (unsigned)(kBins - 1) && pa > max_abs) pa = max_abs;
        if (n > 0 && br < (unsigned)(kBins - 1) && pr > max_rel) pr = max_rel;
        out->abs_bin[g] = ba; out->rel_bin[g] = br; out->abs_p[g] = pa; out->rel_p[g] = pr;
        if (thr_abs && thr_rel) {
            const double ra = (double)pa / (double)thr_abs[g];
            const double rr = (double)pr / (double)thr_rel[g];
            if (ra == ra && !(pmax >= ra)) pmax = ra;       // NaN ratios (0/0) are skipped
            if (rr == rr && !(pmax >= rr)) pmax = rr;
        }
    }
    out->p_max = pmax;
    out->offending = (pmax > 1.0) ? 1u : 0u;
}

// Calibration (Sec. 3.2): per grid point the maximum over the runs' percentile values (NaN entries
// skipped) and alpha times it, the product one binary64 multiplication rounded up to binary32.
// One thread per (kind, grid point); the runs are read with independent strided loads.
__global__ __launch_bounds__(64) void calibrate_kernel(const tao_error_profile* __restrict__ profiles, long count,
                                                       double alpha, float* __restrict__ env_abs,
                                                       float* __restrict__ env_rel, float* __restrict__ thr_abs,
                                                       float* __restrict__ thr_rel) {
    const int t = threadIdx.x;
    if (t >= 2 * kGrid) return;
    const bool rel = t >= kGrid;
    const int g = rel ? t - kGrid : t;
    float m = NAN;
    for (long r = 0; r < count; ++r) {
        const float v = rel ? profiles[r].rel_p[g] : profiles[r].abs_p[g];
        if (v == v && !(m >= v)) m = v;
    }
    float* env = rel ? env_rel : env_abs;
    if (env) env[g] = m;
    (rel ? thr_rel : thr_abs)[g] = up32(alpha * (double)m);
}

}  // namespace tao

extern "C" {

int tao_calibrate_thresholds(const tao_error_profile* profiles, long count, double alpha,
                             float* env_abs, float* env_rel, float* thr_abs, float* thr_rel, void* stream) {
    using namespace tao;
    if (count < 1 || !(alpha >= 0.0) || !std::isfinite(alpha)) return TAO_ERR_SHAPE;
    if (!profiles || !thr_abs || !thr_rel) return TAO_ERR_NULL;
    if (!aligned(profiles, 8) || !aligned(env_abs, 4) || !aligned(env_rel, 4) || !aligned(thr_abs, 4) || !aligned(thr_rel, 4))
        return TAO_ERR_ALIGN;
    hipLaunchKernelGGL(calibrate_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, profiles, count, alpha,
                       env_abs, env_rel, thr_abs, thr_rel);
    return launch_status();
}

size_t tao_profile_workspace_bytes(long n) {
    (void)n;
    return (size_t)tao::kMaxPartials *
           (2 * (tao::kBins + tao::kGroups) * sizeof(unsigned int) + sizeof(tao::ErrStats));
}

int tao_profile_errors(const float* claimed, const float* ref, long n, double eps_rel,
                       const float* thr_abs, const float* thr_rel, tao_error_profile* out,
                       void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    if (!out || !ws) return out ? TAO_ERR_WORKSPACE : TAO_ERR_NULL;
    if (n < 0 || !(eps_rel >= 0.0)) return TAO_ERR_SHAPE;       // a negative or NaN eps_rel has no meaning
    if (n > 0 && (!claimed || !ref)) return TAO_ERR_NULL;
    if ((thr_abs == nullptr) != (thr_rel == nullptr)) return TAO_ERR_NULL;
    if (!aligned(claimed, 4) || !aligned(ref, 4) || !aligned(thr_abs, 4) || !aligned(thr_rel, 4) || !aligned(out, 8))
        return TAO_ERR_ALIGN;
    if (!aligned(ws, 256) || ws_bytes < tao_profile_workspace_bytes(n)) return TAO_ERR_WORKSPACE;
    if (n >= (1L << 36)) return TAO_ERR_SHAPE;   // 32-bit per-workgroup counters
    hipStream_t st = (hipStream_t)stream;
    const int vec_ok = aligned(claimed, 16) && aligned(ref, 16);
    long want = (n + (long)kErrThreads * 16 - 1) / ((long)kErrThreads * 16);
    const int nblocks = (int)(want < 1 ? 1 : (want > kMaxPartials ? kMaxPartials : want));
    unsigned int* ws_hist_a = (unsigned int*)ws;
    unsigned int* ws_hist_r = ws_hist_a + (size_t)kMaxPartials * kBins;
    unsigned int* ws_coarse_a = ws_hist_r + (size_t)kMaxPartials * kBins;
    unsigned int* ws_coarse_r = ws_coarse_a + (size_t)kMaxPartials * kGroups;
    ErrStats* ws_stats = (ErrStats*)(ws_coarse_r + (size_t)kMaxPartials * kGroups);
    hipLaunchKernelGGL(errors_pass, dim3(nblocks), dim3(kErrThreads), 0, st, claimed, ref, n, vec_ok, eps_rel,
                       ws_hist_a, ws_hist_r, ws_coarse_a, ws_coarse_r, ws_stats);
    hipLaunchKernelGGL(errors_reduce, dim3(2 * kGroups), dim3(kReduceThreads), 0, st, ws_hist_a, ws_hist_r,
                       ws_coarse_a, ws_coarse_r, nblocks, (unsigned long long)n, out);
    hipLaunchKernelGGL(errors_finalize, dim3(1), dim3(256), 0, st, ws_stats, nblocks, (unsigned long long)n,
                       thr_abs, thr_rel, out);
    return launch_status();
}

}  // extern "C"
