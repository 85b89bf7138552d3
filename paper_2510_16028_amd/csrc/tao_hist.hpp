// Histogram machinery shared by tao_check_and_profile and tao_profile_errors: the fixed 2048-bin
// key of a non-negative binary32 error (Sec. 5.3 percentile profiles are taken by nearest rank on
// this histogram), the per-workgroup LDS histogram of the streaming passes, and the second-level
// reduction that also locates nearest-rank percentiles without any cross-workgroup ordering.
#pragma once
#include "tao_device.hpp"
#include "tao.h"

namespace tao {

constexpr int kBins = TAO_NBINS;
constexpr int kReplicas = 4;                 // LDS copies of each bin, selected by lane & 3
constexpr int kMaxPartials = 256;            // pass-1 workgroups (one per CU), one partial each
constexpr int kBinsPerReduceBlock = 64;
constexpr int kGroups = kBins / kBinsPerReduceBlock;                      // 32 coarse groups of 64 bins
constexpr int kReduceThreads = 1024;
constexpr int kReduceSlices = kReduceThreads / kBinsPerReduceBlock;      // 16
constexpr int kPartialsPerThread = kMaxPartials / kReduceSlices;         // 16 independent loads
constexpr int kReduceWaves = kReduceThreads / kWave;

// bin of an error value: bits >> 20 (8 exponent bits, 3 mantissa bits); NaN -> last bin
__device__ __forceinline__ unsigned int error_bin(float e32, bool& is_nan) {
    is_nan = e32 != e32;
    // (errors are non-negative: the entry points reject a negative eps_rel; the minimum keeps a
    // stray sign bit from indexing past the histogram all the same)
    return is_nan ? (unsigned)(kBins - 1) : min(__float_as_uint(e32) >> 20, (unsigned)(kBins - 1));
}

__device__ __forceinline__ float bin_upper_edge(unsigned int b) {
    if (b >= (unsigned)(kBins - 1)) return __uint_as_float(0x7fc00000u);
    if (b >= 2039u) return __uint_as_float(0x7f800000u);
    return __uint_as_float((b + 1u) << 20);
}

// rank = max(1, ceil(n * num / den)); n < 2^36 and num <= 999 keep the product in 64 bits.
__device__ __forceinline__ unsigned long long rank_of(unsigned long long n, unsigned long long num,
                                                       unsigned long long den) {
    unsigned long long r = (n * num + den - 1) / den;
    return r < 1 ? 1 : r;
}

// Flush a lane-replicated LDS histogram (kBins * R counters) of a 1024-thread workgroup to its
// partial histogram `dst[kBins]` and its coarse group counts `coarse[kGroups]`.
template <int R = kReplicas>
__device__ __forceinline__ void flush_histogram(const unsigned int* hist, unsigned int* __restrict__ dst,
                                                unsigned int* __restrict__ coarse) {
    const int tid = threadIdx.x;
    for (int b = tid; b < kBins; b += blockDim.x) {
        unsigned int s = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) s += hist[b * R + r];
        dst[b] = s;
        // a wavefront covers exactly one group of 64 consecutive bins
        unsigned int g = s;
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) g += __shfl_xor(g, o, kWave);
        if ((tid & (kWave - 1)) == 0) coarse[b / kBinsPerReduceBlock] = g;
    }
}

struct RankQuery { unsigned int num, den; };

// Second level, one 1024-thread workgroup per group `grp` of 64 bins: sums the partial histograms
// of `nblocks` pass-1 workgroups (ws_hist[k][kBins], 256-byte contiguous reads, all loads
// independent), writes the 64-bit totals to hist_out, derives the number of elements below its own
// bins from the coarse counts (ws_coarse[k][kGroups]) and, for each of the NQ rank queries, writes
// the bin holding rank max(1, ceil(n num/den)) and its upper edge if that bin is one of its own.
// Every query is answered by exactly one workgroup when n > 0; nothing is written for n == 0.
// smem: kReduceThreads + kReduceWaves 64-bit words.
template <int NQ>
__device__ __forceinline__ void reduce_group(const unsigned int* __restrict__ ws_hist,
                                             const unsigned int* __restrict__ ws_coarse, int nblocks, int grp,
                                             unsigned long long n, uint64_t* __restrict__ hist_out,
                                             const RankQuery* q, unsigned int* __restrict__ bin_out,
                                             float* __restrict__ edge_out, unsigned long long* smem) {
    unsigned long long* part = smem;
    unsigned long long* wsum = smem + kReduceThreads;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int b = tid & (kBinsPerReduceBlock - 1);
    const int slice = tid / kBinsPerReduceBlock;
    const int bin = grp * kBinsPerReduceBlock + b;
    unsigned int vals[kPartialsPerThread];
#pragma unroll
    for (int j = 0; j < kPartialsPerThread; ++j) {
        const int k = slice + kReduceSlices * j;
        vals[j] = (k < nblocks) ? ws_hist[(size_t)k * kBins + bin] : 0u;
    }
    unsigned long long below = 0;
    const int total = nblocks * kGroups;
#pragma unroll
    for (int j = 0; j < (kMaxPartials * kGroups) / kReduceThreads; ++j) {
        const int e = tid + kReduceThreads * j;
        if (e < total && (e % kGroups) < grp) below += ws_coarse[e];
    }
    unsigned long long s = 0;
#pragma unroll
    for (int j = 0; j < kPartialsPerThread; ++j) s += vals[j];
    part[tid] = s;
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) below += __shfl_xor(below, o, kWave);
    if (lane == 0) wsum[wave] = below;
    __syncthreads();
    if (tid < kBinsPerReduceBlock) {            // first wavefront: one lane per bin
        unsigned long long t = 0;
#pragma unroll
        for (int k = 0; k < kReduceSlices; ++k) t += part[k * kBinsPerReduceBlock + tid];
        hist_out[bin] = t;
        unsigned long long before = 0;
#pragma unroll
        for (int w = 0; w < kReduceWaves; ++w) before += wsum[w];
        unsigned long long incl = t;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const unsigned long long up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        const unsigned long long hi = before + incl, lo = hi - t;      // ranks (lo, hi] fall in this bin
        if (n > 0) {
#pragma unroll
            for (int i = 0; i < NQ; ++i) {
                const unsigned long long r = rank_of(n, q[i].num, q[i].den);
                if (lo < r && r <= hi) { bin_out[i] = bin; edge_out[i] = bin_upper_edge(bin); }
            }
        }
    }
    __syncthreads();
}

}  // namespace tao
