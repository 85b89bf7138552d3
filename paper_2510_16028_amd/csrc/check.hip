// tao_check_and_profile: the leaf check of Sec. 5.4 and the relative-error
// profile of Sec. 5.3 / Sec. 3.2 Eq. (2) as one streaming pass over
// (claimed, ref, tau) plus a small finalising kernel.
//
// Pass 1 (check_pass): grid-stride over 16-byte vectors of the three inputs;
// per element IEEE binary64 arithmetic (no contraction); each workgroup keeps a
// lane-replicated 2048-bin histogram in LDS and writes its partial histogram
// and counters to the workspace -- no global atomics, so the result does not
// depend on scheduling.
// Pass 2 (profile_reduce): one workgroup per 64 bins sums the partials (256-byte
// contiguous reads) into the 64-bit histogram.  Pass 1 also leaves per-workgroup
// counts of each 64-bin group, from which every pass-2 workgroup derives the
// number of elements below its own bins; it can then decide by itself whether a
// nearest-rank percentile falls into one of its bins -- no cross-workgroup
// ordering, fences or atomics.  Workgroup 0 also writes the scalar fields.
#include <atomic>
#include "tao_check.hpp"

namespace tao {

__global__ __launch_bounds__(kCheckThreads) void check_pass(
    const float* __restrict__ claimed, const float* __restrict__ ref, const float* __restrict__ tau,
    long n, int vec_ok, double alpha, double eps_rel,
    unsigned int* __restrict__ ws_hist, unsigned int* __restrict__ ws_coarse,
    BlockStats* __restrict__ ws_stats) {
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
        const float4 c4 = ntload4(reinterpret_cast<const float4*>(claimed) + i);
        const float4 r4 = ntload4(reinterpret_cast<const float4*>(ref) + i);
        const float4 t4 = ntload4(reinterpret_cast<const float4*>(tau) + i);
        check_one(c4.x, r4.x, t4.x, alpha, eps_rel, hist, rep, acc);
        check_one(c4.y, r4.y, t4.y, alpha, eps_rel, hist, rep, acc);
        check_one(c4.z, r4.z, t4.z, alpha, eps_rel, hist, rep, acc);
        check_one(c4.w, r4.w, t4.w, alpha, eps_rel, hist, rep, acc);
    }
    // scalar remainder (everything when the inputs are not 16-byte aligned)
    for (long i = (nvec << 2) + (long)blockIdx.x * kCheckThreads + tid; i < n; i += stride)
        check_one(claimed[i], ref[i], tau[i], alpha, eps_rel, hist, rep, acc);

    flush_block_stats(acc, red, ws_stats);
    flush_histogram(hist, ws_hist + (size_t)blockIdx.x * kBins, ws_coarse + blockIdx.x * kGroups);
}

__global__ __launch_bounds__(kReduceThreads) void profile_reduce(
    const unsigned int* __restrict__ ws_hist, const unsigned int* __restrict__ ws_coarse,
    const BlockStats* __restrict__ ws_stats, int nblocks, unsigned long long n, tao_profile* out) {
    __shared__ unsigned long long smem[kReduceThreads + kReduceWaves];
    __shared__ unsigned long long wv[kReduceWaves], wq[kReduceWaves];
    __shared__ unsigned int wm[kReduceWaves];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    // nearest-rank percentiles p50, p99, p99.9; the three bin and three edge fields of tao_profile
    // are consecutive
    const RankQuery q[3] = {{1, 2}, {99, 100}, {999, 1000}};
    reduce_group<3>(ws_hist, ws_coarse, nblocks, blockIdx.x, n, out->hist, q, &out->p50_bin, &out->p50, smem);
    if (blockIdx.x != 0) return;
    // counters of pass 1 (at most one record per thread)
    unsigned long long v = 0, qn = 0; unsigned int m = 0;
    for (int k = tid; k < nblocks; k += kReduceThreads) {
        v += ws_stats[k].violations; qn += ws_stats[k].nans; m = max(m, ws_stats[k].max_bits);
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) {
        v += __shfl_xor(v, o, kWave); qn += __shfl_xor(qn, o, kWave);
        m = max(m, (unsigned int)__shfl_xor(m, o, kWave));
    }
    if (lane == 0) { wv[wave] = v; wq[wave] = qn; wm[wave] = m; }
    __syncthreads();
    if (tid == 0) {
        v = 0; qn = 0; m = 0;
        for (int w = 0; w < kReduceWaves; ++w) { v += wv[w]; qn += wq[w]; m = max(m, wm[w]); }
        out->n = n;
        out->violations = v;
        out->nan_count = qn;
        out->max_rel = __uint_as_float(m);
        out->accept = (v == 0) ? 1u : 0u;
        out->pad_ = 0;
        if (n == 0) {
            out->p50_bin = out->p99_bin = out->p999_bin = 0;
            out->p50 = out->p99 = out->p999 = bin_upper_edge(0);
        }
    }
}

void launch_profile_reduce(const CheckWorkspace& w, int nblocks, unsigned long long n, tao_profile* out, hipStream_t st) {
    hipLaunchKernelGGL(profile_reduce, dim3(kReduceBlocks), dim3(kReduceThreads), 0, st, w.hist, w.coarse,
                       w.stats, nblocks, n, out);
}

// ---- the entry point that allocates nothing -------------------------------------------------
// Its partial histograms and counters live in this array instead of a caller's workspace: one copy
// per device, held until the process ends.  Host code never uses the array's name as an address
// (on the host it is only a handle): the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[check_workspace_bytes()];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up on the first call there).
static int static_scratch(void** ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return TAO_ERR_LAUNCH; }
    if (dev < 0 || dev >= kMaxDevices) return TAO_ERR_WORKSPACE;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { g_last_hip_error = (int)e; return TAO_ERR_LAUNCH; }
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // (two racing threads store the same address)
    }
    *ptr = p;
    return TAO_OK;
}

}  // namespace tao

extern "C" {

int tao_check_and_profile_static(const float* claimed, const float* ref, const float* tau, long n,
                                 double alpha, double eps_rel, tao_profile* out, void* stream) {
    using namespace tao;
    if (!out) return TAO_ERR_NULL;
    if (n < 0 || n > TAO_STATIC_CHECK_MAX_N || !(eps_rel >= 0.0)) return TAO_ERR_SHAPE;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != TAO_OK) return rc;
    // every workgroup of the pass overwrites its own partial result and the finalising kernel reads
    // only those, so nothing of the previous call's contents has to be cleared
    return tao_check_and_profile(claimed, ref, tau, n, alpha, eps_rel, out, ws, check_workspace_bytes(), stream);
}

size_t tao_check_workspace_bytes(long n) {
    (void)n;
    return tao::check_workspace_bytes();
}

int tao_check_and_profile(const float* claimed, const float* ref, const float* tau, long n,
                          double alpha, double eps_rel, tao_profile* out,
                          void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    if (!out || !ws) return out ? TAO_ERR_WORKSPACE : TAO_ERR_NULL;
    if (n < 0 || !(eps_rel >= 0.0)) return TAO_ERR_SHAPE;       // a negative or NaN eps_rel has no meaning
    if (n > 0 && (!claimed || !ref || !tau)) return TAO_ERR_NULL;
    if (!aligned(claimed, 4) || !aligned(ref, 4) || !aligned(tau, 4) || !aligned(out, 8)) return TAO_ERR_ALIGN;
    if (!aligned(ws, 256) || ws_bytes < tao_check_workspace_bytes(n)) return TAO_ERR_WORKSPACE;
    if (n >= (1L << 36)) return TAO_ERR_SHAPE;   // 32-bit per-workgroup counters
    hipStream_t st = (hipStream_t)stream;
    const int vec_ok = aligned(claimed, 16) && aligned(ref, 16) && aligned(tau, 16);
    // 16 elements (four 16-byte vectors) per thread before another workgroup is worth it
    long want = (n + (long)kCheckThreads * 16 - 1) / ((long)kCheckThreads * 16);
    int nblocks = (int)(want < 1 ? 1 : (want > kMaxCheckBlocks ? kMaxCheckBlocks : want));
    const CheckWorkspace w = carve_check_workspace(ws);
    hipLaunchKernelGGL(check_pass, dim3(nblocks), dim3(kCheckThreads), 0, st, claimed, ref, tau, n,
                       vec_ok, alpha, eps_rel, w.hist, w.coarse, w.stats);
    launch_profile_reduce(w, nblocks, (unsigned long long)n, out, st);
    return launch_status();
}

}  // extern "C"
