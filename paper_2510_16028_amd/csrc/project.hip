// Projections of a tentative perturbation onto the verifier's admissible sets (Sec. 4.4).
//
//   project_clip       (i)  clip(delta, -alpha tau, alpha tau): one streaming pass.
//   project_empirical  (ii) cap the k-th smallest magnitude by the cap curve of Sec. 4.2 at rank
//                      (k - 1/2)/n, after a running maximum over k, and put sign and place back.
//
// (ii) needs every element's rank, i.e. a stable sort of the magnitudes.  The sort is a
// least-significant-digit radix sort of the 31 magnitude bits (a non-negative binary32 orders like
// its bit pattern, NaN above infinity) in four 8-bit passes; the payload is the element's index
// with its sign bit on top.  Per pass: count (digit histogram per tile), scan (of the digit-major
// counter array), scatter (stable rank inside the tile by wave-wide digit matching, elements
// reordered in LDS so that runs of one digit leave as contiguous writes).  The first pass reads
// delta itself (its count kernel copies it to out when the two differ); the last pass writes no sorted array at
// all: the destination of an element IS its rank, so the cap is evaluated there and only the
// elements that exceed their cap are written, straight to out[index] -- the one access of the
// whole path that is random, 4 bytes per 64-byte line, and therefore kept to the elements that
// need it.
//
// The running maximum over ranks needs no scan: the cap curve is piecewise linear in the rank and
// every operation of its formula is monotone under rounding, so inside one segment of the curve
// the computed caps are monotone and the maximum over the ranks up to k is the larger of
// C(first rank of the segment), C(k) and the maxima of the earlier segments (their first and last
// ranks).  A one-wave kernel tabulates those per segment.
#include "tao_device.hpp"
#include "tao_host.hpp"

namespace tao {

constexpr int kSortThreads = 256;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kSortItems = 16;                                // per thread
constexpr int kSortTile = kSortThreads * kSortItems;          // 4096 elements per workgroup
constexpr int kRadix = 256;
constexpr int kScanChunk = kSortThreads * 16;                 // counters per scan workgroup
constexpr int kXcds = 8;
constexpr int kCountCopies = 4;                               // histogram copies per wave in radix_count
constexpr int kCountStride = kRadix + 4;                      // copy c of digit d in LDS bank (d + 4c) % 32

// One segment of the cap curve: ranks whose r lies in (p0, p0 + dp].
struct CapSeg {
    double c0, dc, p0, dp;     // C(r) = c0 + dc * ((r - p0) / dp)
    double head;               // max of the caps of all earlier ranks' segments and of this one's first rank
    double inv_dp;             // ~ 1 / dp, for estimates only
};
struct CapTable {
    CapSeg seg[TAO_NGRID];
    double n;                  // (double)n
    double percent_per_rank;   // ~ 100 / n, for estimates only
};

__device__ __forceinline__ double grid_percent(int j) {      // P = {1, 5, 10, ..., 95, 99, 100}
    return j < 0 ? 0.0 : j == 0 ? 1.0 : j < 20 ? 5.0 * j : j == 20 ? 99.0 : 100.0;
}
__device__ __forceinline__ double rank_percent(double k, double n) { return ((k - 0.5) / n) * 100.0; }

// first knot j with r <= P[j]  (r <= 100 always)
__device__ __forceinline__ int segment_of(double r) {
    int j = (int)(r * 0.2);                                   // near r / 5, then settled by comparisons
    j = j < 0 ? 0 : j > TAO_NGRID - 1 ? TAO_NGRID - 1 : j;
    while (j < TAO_NGRID - 1 && r > grid_percent(j)) ++j;
    while (j > 0 && r <= grid_percent(j - 1)) --j;
    return j;
}
__device__ __forceinline__ double cap_in_segment(const CapSeg& s, double r) {
    return s.c0 + s.dc * ((r - s.p0) / s.dp);
}

// Largest binary32 value <= c, for c >= 0.
__device__ __forceinline__ float down32(double c) {
    float f = (float)c;
    if ((double)f > c) f = __uint_as_float(__float_as_uint(f) - 1u);
    return f;
}

// Fills *tab (global or LDS); called by all threads of a workgroup of at least 64, ends with a barrier.
__device__ __forceinline__ void build_cap_table(const float* __restrict__ thr, double alpha, long n, CapTable* tab) {
    __shared__ double seg_max[TAO_NGRID];
    __shared__ long first_rank[TAO_NGRID + 1];
    const int j = threadIdx.x;
    const double dn = (double)n;
    CapSeg s = {};
    if (j < TAO_NGRID) {
        const double c1 = (double)thr[j] * alpha;
        const double c0 = j == 0 ? 0.0 : (double)thr[j - 1] * alpha;
        s.c0 = c0; s.dc = c1 - c0; s.p0 = grid_percent(j - 1); s.dp = grid_percent(j) - grid_percent(j - 1);
        // smallest rank k in [1, n + 1] with r_k > P[j - 1]  (r_k is nondecreasing in k)
        long lo = 1, hi = n + 1;
        while (lo < hi) {
            const long mid = lo + (hi - lo) / 2;
            if (rank_percent((double)mid, dn) > s.p0) hi = mid; else lo = mid + 1;
        }
        first_rank[j] = lo;
    }
    if (j == TAO_NGRID) first_rank[j] = n + 1;
    __syncthreads();
    double cfirst = 0.0;
    if (j < TAO_NGRID) {
        const long kf = first_rank[j], kl = first_rank[j + 1] - 1;
        double m = 0.0;                                       // caps are non-negative: 0 is neutral
        if (kf <= kl) {
            cfirst = cap_in_segment(s, rank_percent((double)kf, dn));
            m = fmax(cfirst, cap_in_segment(s, rank_percent((double)kl, dn)));
        }
        seg_max[j] = m;
    }
    __syncthreads();
    if (j < TAO_NGRID) {
        double head = cfirst;
        for (int e = 0; e < j; ++e) head = fmax(head, seg_max[e]);
        s.head = head;
        s.inv_dp = 1.0 / s.dp;
        tab->seg[j] = s;
    }
    if (j == 0) { tab->n = dn; tab->percent_per_rank = 100.0 / dn; }
    __syncthreads();
}

__global__ void __launch_bounds__(kWave) cap_table_kernel(const float* __restrict__ thr, double alpha, long n,
                                                          CapTable* __restrict__ tab) {
    build_cap_table(thr, alpha, n, tab);
}

// ---- (i) -------------------------------------------------------------------------------------

__device__ __forceinline__ float clip_one(float d, float t, double alpha) {
    const float a = fabsf(d);
    const double cap = (double)t * alpha;
    const float r = (double)a > cap ? down32(cap) : a;        // NaN compares false and stays
    return copysignf(r, d);
}

__global__ void __launch_bounds__(256) project_clip_kernel(const float* __restrict__ delta, const float* __restrict__ tau,
                                                           double alpha, float* __restrict__ out, long n, int vec_ok) {
    const long stride = (long)gridDim.x * blockDim.x * 4;
    for (long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4; i < n; i += stride) {
        const float4 d = load4<true>(delta, i, n, vec_ok, 0.f);
        const float4 t = load4<true>(tau, i, n, vec_ok, 0.f);
        float4 r;
        r.x = clip_one(d.x, t.x, alpha); r.y = clip_one(d.y, t.y, alpha);
        r.z = clip_one(d.z, t.z, alpha); r.w = clip_one(d.w, t.w, alpha);
        store4(out, i, n, vec_ok, r);
    }
}

// ---- (ii): radix sort passes --------------------------------------------------------------------

// Workgroups are dealt round-robin to the eight XCDs; giving XCD x the x-th contiguous eighth of
// the tiles keeps the counter cache lines that neighbouring tiles share inside one L2.
__device__ __forceinline__ long tile_of_block(long tiles_per_xcd) {
    return (long)(blockIdx.x % kXcds) * tiles_per_xcd + blockIdx.x / kXcds;
}

template <bool FIRST>
__device__ __forceinline__ void load_item(const float* delta, const unsigned* __restrict__ keys,
                                          const unsigned* __restrict__ vals, long e, unsigned& key, unsigned& val) {
    if (FIRST) {
        const unsigned b = __float_as_uint(delta[e]);
        key = b & 0x7fffffffu;
        val = (unsigned)e | (b & 0x80000000u);
    } else {
        key = keys[e];
        val = vals[e];
    }
}

// Digit histogram of every tile: hist[digit * tiles + tile].  Counting does not depend on the
// order inside the tile, so a thread takes four runs of four consecutive keys (16-byte loads, all
// issued before the first is used).  The first pass also copies delta to out on the way.
template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads) radix_count(const float* delta, const unsigned* __restrict__ keys,
                                                            long n, long tiles, long tiles_per_xcd, int shift, int vec_ok,
                                                            unsigned* __restrict__ hist, unsigned* copy_to) {
    __shared__ unsigned cnt[kSortWaves][kCountCopies][kCountStride];
    const long tile = tile_of_block(tiles_per_xcd);
    if (tile >= tiles) return;                                 // whole workgroup
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    for (int d = lane; d < kCountCopies * kCountStride; d += kWave) (&cnt[wave][0][0])[d] = 0;
    __builtin_amdgcn_wave_barrier();
    const unsigned* src = FIRST ? reinterpret_cast<const unsigned*>(delta) : keys;
    const long tile_base = tile * kSortTile;
    unsigned key[kSortItems];
    const bool full = tile_base + kSortTile <= n;
    if (full && vec_ok) {
#pragma unroll
        for (int q = 0; q < kSortItems / 4; ++q) {
            const long e = tile_base + ((long)q * kSortThreads + threadIdx.x) * 4;
            const uint4 v = *reinterpret_cast<const uint4*>(src + e);
            if (FIRST && copy_to) *reinterpret_cast<uint4*>(copy_to + e) = v;
            key[4 * q] = v.x; key[4 * q + 1] = v.y; key[4 * q + 2] = v.z; key[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kSortItems; ++i) {
            const long e = tile_base + (long)i * kSortThreads + threadIdx.x;
            key[i] = e < n ? src[e] : 0u;
            if (FIRST && copy_to && e < n) copy_to[e] = key[i];
        }
    }
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        // element index of key[i] in the scalar layout (the vector layout is only used on full tiles)
        const bool valid = full || tile_base + (long)i * kSortThreads + threadIdx.x < n;
        const unsigned d = ((FIRST ? key[i] & 0x7fffffffu : key[i]) >> shift) & (kRadix - 1);
        // A wave whose valid lanes all hold one digit (the rule in the top byte of narrow data) adds
        // once.  Otherwise LDS atomics, spread over eight copies of the histogram chosen by the lane
        // (a few distinct digits per wave -- exponent bytes, trailing zero bytes of deviations that are
        // differences of nearby values -- would serialise 64 atomics on a handful of addresses); the
        // copies are 260 counters apart, so equal digits of different copies fall into different banks.
        const unsigned long long vmask = __ballot(valid);
        if (vmask == 0) continue;
        const unsigned d0 = __shfl(d, (int)__builtin_ctzll(vmask), kWave);
        if (__ballot(valid && d == d0) == vmask) {
            if (lane == (int)__builtin_ctzll(vmask)) cnt[wave][0][d0] += (unsigned)__popcll(vmask);
        } else if (valid) {
            atomicAdd(&cnt[wave][lane & (kCountCopies - 1)][d], 1u);
        }
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    const int d = threadIdx.x;                                 // kSortThreads == kRadix
    unsigned total = 0;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w)
#pragma unroll
        for (int c = 0; c < kCountCopies; ++c) total += cnt[w][c][d];
    hist[(long)d * tiles + tile] = total;
}

// Exclusive scan of `count` 32-bit counters in three steps (chunk sums, scan of the sums by one
// workgroup, rescan of each chunk with its offset).
__device__ __forceinline__ unsigned block_exclusive_scan(unsigned v, unsigned* wave_tot, unsigned& block_total) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    unsigned inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const unsigned t = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += t;
    }
    if (lane == kWave - 1) wave_tot[wave] = inc;
    __syncthreads();
    unsigned before = 0, all = 0;
    const int nw = blockDim.x / kWave;
    for (int w = 0; w < nw; ++w) { const unsigned t = wave_tot[w]; if (w < wave) before += t; all += t; }
    __syncthreads();
    block_total = all;
    return before + inc - v;
}

__global__ void __launch_bounds__(kSortThreads) scan_chunk_sums(const unsigned* __restrict__ c, long count,
                                                                unsigned* __restrict__ sums) {
    __shared__ unsigned wave_tot[kSortWaves];
    const long base = (long)blockIdx.x * kScanChunk;
    unsigned s = 0;
    for (int i = threadIdx.x; i < kScanChunk; i += kSortThreads) {
        const long e = base + i;
        if (e < count) s += c[e];
    }
    unsigned total;
    block_exclusive_scan(s, wave_tot, total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(1024) scan_spine(unsigned* __restrict__ sums, long chunks) {
    __shared__ unsigned wave_tot[1024 / kWave];
    unsigned carry = 0;
    for (long base = 0; base < chunks; base += 1024) {          // uniform trip count
        const long e = base + threadIdx.x;
        const unsigned v = e < chunks ? sums[e] : 0u;
        unsigned total;
        const unsigned ex = block_exclusive_scan(v, wave_tot, total);
        if (e < chunks) sums[e] = carry + ex;
        carry += total;
    }
}

__global__ void __launch_bounds__(kSortThreads) scan_apply(unsigned* __restrict__ c, long count,
                                                           const unsigned* __restrict__ sums) {
    __shared__ unsigned wave_tot[kSortWaves];
    // thread t owns 16 consecutive counters (the array is 256-byte aligned and chunks start at
    // multiples of 4096 counters): local sequential scan between two block scans
    const long base = (long)blockIdx.x * kScanChunk + (long)threadIdx.x * 16;
    unsigned v[16];
    unsigned s = 0;
    const bool whole = base + 16 <= count;
    if (whole) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 t = *reinterpret_cast<const uint4*>(c + base + 4 * q);
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = base + i < count ? c[base + i] : 0u;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) s += v[i];
    unsigned total;
    unsigned run = block_exclusive_scan(s, wave_tot, total) + sums[blockIdx.x];
#pragma unroll
    for (int i = 0; i < 16; ++i) { const unsigned t = v[i]; v[i] = run; run += t; }
    if (whole) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<uint4*>(c + base + 4 * q) = make_uint4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (base + i < count) c[base + i] = v[i];
    }
}

// LDS of one tile's pass.
struct TileSort {
    unsigned skey[kSortTile];
    unsigned sval[kSortTile];
    unsigned cnt[kSortWaves][kRadix];        // per wave: running count, then the wave's offset in the digit's run
    unsigned tile_excl[kRadix];              // first tile-local position of a digit
    unsigned dest_off[kRadix];               // global destination minus tile-local position
    unsigned wave_tot[kSortWaves];
};

// One stable counting-sort step of a tile on the digit at `shift`: element i of lane l of wave w is
// the tile's element w * 1024 + i * 64 + l (`valid_count` of them exist); on return sh.skey / sh.sval
// hold the tile ordered by digit, equal digits in their old order, and sh.tile_excl the start of
// every digit's run.  All threads of the workgroup call it; it ends with a barrier.
__device__ __forceinline__ void tile_sort_step(TileSort& sh, const unsigned (&key)[kSortItems],
                                               const unsigned (&val)[kSortItems], int valid_count, int shift) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    for (int d = lane; d < kRadix; d += kWave) sh.cnt[wave][d] = 0;
    __builtin_amdgcn_wave_barrier();
    const int first = wave * (kSortItems * kWave) + lane;
    unsigned short rank[kSortItems];
    // Stable rank of every element among those of its wave with the same digit: the elements of a
    // wave are ordered by (i, lane), which is their order in memory.  Eight ballots find the lanes
    // that share a digit; the lowest of them advances the wave's counter.
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const bool valid = first + i * kWave < valid_count;
        const unsigned d = (key[i] >> shift) & (kRadix - 1);
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1u;
            const unsigned long long bal = __ballot(bit);
            same &= bit ? bal : ~bal;
        }
        const unsigned prev = valid ? sh.cnt[wave][d] : 0u;
        const unsigned r = prev + (unsigned)__popcll(same & lanes_below);
        __builtin_amdgcn_wave_barrier();                       // all reads of this round before its writes
        if (valid && (same & lanes_below) == 0) sh.cnt[wave][d] = prev + (unsigned)__popcll(same);
        rank[i] = (unsigned short)r;
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    {   // per digit: offsets of the waves inside the digit's run, the run's place in the tile
        const int d = threadIdx.x;                             // kSortThreads == kRadix
        unsigned run = 0;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) { const unsigned t = sh.cnt[w][d]; sh.cnt[w][d] = run; run += t; }
        unsigned total;
        sh.tile_excl[d] = block_exclusive_scan(run, sh.wave_tot, total);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        if (first + i * kWave < valid_count) {
            const unsigned d = (key[i] >> shift) & (kRadix - 1);
            const unsigned pos = sh.tile_excl[d] + sh.cnt[wave][d] + rank[i];
            if (pos < (unsigned)kSortTile) { sh.skey[pos] = key[i]; sh.sval[pos] = val[i]; }
        }
    }
    __syncthreads();
}

// The element of 0-based rank `rank0` with magnitude bits k and payload v: write its capped value
// if it exceeds its cap (out already holds delta, unless WRITE_ALL).  Most of the work is two
// binary64 divisions; an estimate with reciprocals (error far below the margin used) first sorts
// out the elements that are clearly under their cap.
template <bool WRITE_ALL>
__device__ __forceinline__ void cap_and_store(const CapTable& tab, unsigned rank0, unsigned k, unsigned v, long n,
                                              float* out) {
    const float a = __uint_as_float(k);
    const unsigned idx = v & 0x7fffffffu;
    if ((long)idx >= n) return;                                // cannot happen
    const double kk = (double)rank0 + 0.5;
    const double re = kk * tab.percent_per_rank;
    const CapSeg se = tab.seg[segment_of(re)];
    const double ce = fmax(se.head, se.c0 + se.dc * ((re - se.p0) * se.inv_dp));
    const bool near_knot = fabs(re - se.p0) < 1e-6 || fabs(re - (se.p0 + se.dp)) < 1e-6;
    float star = a;
    if (near_knot || !((double)a < ce - (fabs(se.dc) + ce) * 1e-9)) {
        const double r = rank_percent((double)rank0 + 1.0, tab.n);
        const CapSeg s = tab.seg[segment_of(r)];
        const double cap = fmax(s.head, cap_in_segment(s, r));
        if ((double)a > cap) star = down32(cap);               // NaN compares false and stays
        else if (!WRITE_ALL) return;
    } else if (!WRITE_ALL) {
        return;
    }
    out[idx] = __uint_as_float(__float_as_uint(star) | (v & 0x80000000u));
}

// Scatter pass.  `hist` holds the scanned counters: hist[d * tiles + tile] is the destination of
// the tile's first element with digit d.
template <bool FIRST, bool LAST>
__global__ void __launch_bounds__(kSortThreads) radix_scatter(const float* delta,
                                                              const unsigned* __restrict__ keys_in, const unsigned* __restrict__ vals_in,
                                                              unsigned* __restrict__ keys_out, unsigned* __restrict__ vals_out,
                                                              long n, long tiles, long tiles_per_xcd, int shift,
                                                              const unsigned* __restrict__ hist,
                                                              const CapTable* __restrict__ tab, float* out) {
    __shared__ TileSort sh;
    __shared__ CapTable stab;                                  // LAST: the cap table, read per element
    __shared__ double run_cap[LAST ? kRadix : 1];
    const long tile = tile_of_block(tiles_per_xcd);
    if (tile >= tiles) return;                                 // whole workgroup
    if (LAST) {
        static_assert(sizeof(CapTable) % sizeof(double) == 0 && sizeof(CapTable) / sizeof(double) <= kSortThreads, "one double per thread");
        if (threadIdx.x < sizeof(CapTable) / sizeof(double))
            reinterpret_cast<double*>(&stab)[threadIdx.x] = reinterpret_cast<const double*>(tab)[threadIdx.x];
        // visible after the barriers of the sort step
    }
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const long tile_base = tile * kSortTile;
    const long base = tile_base + (long)wave * (kSortItems * kWave) + lane;
    const long left = n - tile_base;
    const int tile_count = left < kSortTile ? (int)left : kSortTile;

    unsigned key[kSortItems], val[kSortItems];
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const long e = base + (long)i * kWave;
        key[i] = 0xffffffffu; val[i] = 0;
        if (e < n) load_item<FIRST>(delta, keys_in, vals_in, e, key[i], val[i]);
    }
    tile_sort_step(sh, key, val, tile_count, shift);
    {
        const unsigned first_dest = hist[(long)threadIdx.x * tiles + tile];                  // kSortThreads == kRadix
        sh.dest_off[threadIdx.x] = first_dest - sh.tile_excl[threadIdx.x];
        if (LAST) {
            // Caps do not decrease with the rank: the exact cap of the first rank this tile reaches
            // with digit d is a lower bound for all its elements of that digit, and most elements are
            // settled by one comparison with it.
            const double r = rank_percent((double)first_dest + 1.0, stab.n);
            const CapSeg s = stab.seg[segment_of(r)];
            run_cap[threadIdx.x] = (long)first_dest < n ? fmax(s.head, cap_in_segment(s, r)) : 0.0;
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < tile_count; j += kSortThreads) {
        const unsigned k = sh.skey[j], v = sh.sval[j];
        const unsigned d = (k >> shift) & (kRadix - 1);
        const unsigned dest = sh.dest_off[d] + (unsigned)j;
        if ((long)dest >= n) continue;                         // cannot happen with consistent counters
        if (!LAST) {
            keys_out[dest] = k;
            vals_out[dest] = v;
        } else {
            if ((double)__uint_as_float(k) <= run_cap[d]) continue;
            cap_and_store<false>(stab, dest, k, v, n, out);     // dest is the 0-based rank
        }
    }
}

// Tensors of at most one tile: the four passes in LDS by one workgroup, cap table included.
__global__ void __launch_bounds__(kSortThreads) project_one_tile(const float* delta, const float* __restrict__ thr, double alpha,
                                                                 int n, float* out) {
    __shared__ TileSort sh;
    __shared__ CapTable tab;
    build_cap_table(thr, alpha, n, &tab);                      // ends with a barrier
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int first = wave * (kSortItems * kWave) + lane;
    unsigned key[kSortItems], val[kSortItems];
#pragma unroll
    for (int i = 0; i < kSortItems; ++i) {
        const int e = first + i * kWave;
        key[i] = 0xffffffffu; val[i] = 0;
        if (e < n) load_item<true>(delta, nullptr, nullptr, e, key[i], val[i]);
    }
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
        tile_sort_step(sh, key, val, n, 8 * pass);
        if (pass < 3) {
#pragma unroll
            for (int i = 0; i < kSortItems; ++i) {
                const int e = first + i * kWave;
                if (e < n) { key[i] = sh.skey[e]; val[i] = sh.sval[e]; }
            }
            __syncthreads();                                   // before the next step overwrites the tile
        }
    }
    for (int j = threadIdx.x; j < n; j += kSortThreads)
        cap_and_store<true>(tab, (unsigned)j, sh.skey[j], sh.sval[j], n, out);
}

struct ProjectWorkspace {
    CapTable* tab;
    unsigned *hist, *sums, *keys_a, *vals_a, *keys_b, *vals_b;
    long tiles, counters, chunks;
};

inline size_t round256(size_t b) { return (b + 255) / 256 * 256; }

inline size_t carve_project(long n, char* ws, ProjectWorkspace* w) {
    const long tiles = (n + kSortTile - 1) / kSortTile;
    const long counters = tiles * kRadix;
    const long chunks = (counters + kScanChunk - 1) / kScanChunk;
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = ws ? ws + off : nullptr; off += round256(bytes); return p; };
    char* tab = take(sizeof(CapTable));
    char* hist = take((size_t)counters * 4);
    char* sums = take((size_t)chunks * 4);
    char* ka = take((size_t)n * 4); char* va = take((size_t)n * 4);
    char* kb = take((size_t)n * 4); char* vb = take((size_t)n * 4);
    if (w) {
        w->tab = (CapTable*)tab; w->hist = (unsigned*)hist; w->sums = (unsigned*)sums;
        w->keys_a = (unsigned*)ka; w->vals_a = (unsigned*)va; w->keys_b = (unsigned*)kb; w->vals_b = (unsigned*)vb;
        w->tiles = tiles; w->counters = counters; w->chunks = chunks;
    }
    return off;
}

}  // namespace tao

extern "C" {

int tao_project_clip(const float* delta, const float* tau, double alpha, float* out, long n, void* stream) {
    using namespace tao;
    if (n < 0 || !(alpha >= 0.0) || !std::isfinite(alpha)) return TAO_ERR_SHAPE;
    if (n == 0) return TAO_OK;
    if (!delta || !tau || !out) return TAO_ERR_NULL;
    if (!aligned(delta, 4) || !aligned(tau, 4) || !aligned(out, 4)) return TAO_ERR_ALIGN;
    const int vec_ok = aligned(delta, 16) && aligned(tau, 16) && aligned(out, 16);
    long blocks = (n + 1023) / 1024;
    if (blocks > 256L * 32) blocks = 256L * 32;
    hipLaunchKernelGGL(project_clip_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       delta, tau, alpha, out, n, vec_ok);
    return launch_status();
}

size_t tao_project_workspace_bytes(long n) {
    if (n <= 0 || n >= (1L << 31)) return 0;
    return tao::carve_project(n, nullptr, nullptr);
}

int tao_project_empirical(const float* delta, const float* thr_abs, double alpha, float* out, long n,
                          void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    if (n < 0 || n >= (1L << 31) || !(alpha >= 0.0) || !std::isfinite(alpha)) return TAO_ERR_SHAPE;
    if (n == 0) return TAO_OK;
    if (!delta || !thr_abs || !out) return TAO_ERR_NULL;
    if (!aligned(delta, 4) || !aligned(thr_abs, 4) || !aligned(out, 4)) return TAO_ERR_ALIGN;
    if (!ws || !aligned(ws, 256) || ws_bytes < tao_project_workspace_bytes(n)) return TAO_ERR_WORKSPACE;
    if (n <= kSortTile) {
        hipLaunchKernelGGL(project_one_tile, dim3(1), dim3(kSortThreads), 0, (hipStream_t)stream, delta, thr_abs, alpha,
                           (int)n, out);
        return launch_status();
    }
    ProjectWorkspace w;
    carve_project(n, (char*)ws, &w);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(cap_table_kernel, dim3(1), dim3(kWave), 0, st, thr_abs, alpha, n, w.tab);

    const long per_xcd = (w.tiles + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)(per_xcd * kXcds)), blk(kSortThreads);
    const dim3 sgrid((unsigned)w.chunks);
    unsigned* kin = nullptr; unsigned* vin = nullptr;
    unsigned* kout = w.keys_a; unsigned* vout = w.vals_a;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 8 * pass;
        if (pass == 0) hipLaunchKernelGGL((radix_count<true>), grid, blk, 0, st, delta, kin, n, w.tiles, per_xcd, shift,
                                          (int)(aligned(delta, 16) && aligned(out, 16)), w.hist,
                                          out != delta ? reinterpret_cast<unsigned*>(out) : nullptr);
        else           hipLaunchKernelGGL((radix_count<false>), grid, blk, 0, st, delta, kin, n, w.tiles, per_xcd, shift, 1, w.hist, nullptr);
        hipLaunchKernelGGL(scan_chunk_sums, sgrid, blk, 0, st, w.hist, w.counters, w.sums);
        hipLaunchKernelGGL(scan_spine, dim3(1), dim3(1024), 0, st, w.sums, w.chunks);
        hipLaunchKernelGGL(scan_apply, sgrid, blk, 0, st, w.hist, w.counters, w.sums);
        if (pass == 0)
            hipLaunchKernelGGL((radix_scatter<true, false>), grid, blk, 0, st, delta, kin, vin, kout, vout, n, w.tiles, per_xcd,
                               shift, w.hist, w.tab, out);
        else if (pass < 3)
            hipLaunchKernelGGL((radix_scatter<false, false>), grid, blk, 0, st, delta, kin, vin, kout, vout, n, w.tiles, per_xcd,
                               shift, w.hist, w.tab, out);
        else
            hipLaunchKernelGGL((radix_scatter<false, true>), grid, blk, 0, st, delta, kin, vin, kout, vout, n, w.tiles, per_xcd,
                               shift, w.hist, w.tab, out);
        kin = kout; vin = vout;
        kout = kin == w.keys_a ? w.keys_b : w.keys_a;
        vout = vin == w.vals_a ? w.vals_b : w.vals_a;
    }
    return launch_status();
}

}  // extern "C"
