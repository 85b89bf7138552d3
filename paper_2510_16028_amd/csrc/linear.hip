// tao_bound_linear: tau = Gamma(K') (|A| |W|^T + |bias|) on the FP32 matrix cores
// of gfx950 (Sec. 3.1: reductions take gamma_k with the k of the output element;
// App. A.2 Eq. det-sum extended by one rounding per product).
//
// The bound has to be an upper bound of the real-number value and must stay
// within 1e-6 of it, so a plain FP32 accumulation over K (error up to K*u) is
// not usable.  Scheme, per 32 k-steps of an output element:
//   - v_mfma_f32_32x32x2_f32 accumulates eight chains of 2 instructions (4
//     k-steps) from a zero accumulator: 4 roundings per chain;
//   - the eight chain results are added as a binary32 tree of depth 3 on the
//     vector ALU: 3 more roundings;
//   - the tree's root is converted and added to a binary64 running sum.
// Every term is non-negative and passes through at most 7 binary32 roundings, so
// the computed sum S~ satisfies
//   S (1-u)^7 (1-2^-53)^(K/32+1) <= S~ <= S (1+u)^7 (1+2^-53)^(K/32+1)
// under the rounding model of App. A.1.  The epilogue multiplies by the
// reciprocal of the lower factor, by Gamma and by the guard factor and rounds up
// to binary32: exact <= tau <= exact (1 + 16u + ...) < exact (1 + 1e-6).
//
// On this hardware FP32 MFMA and vector-ALU instructions of a SIMD share one
// pipe (neither overlaps the other, from the same or another wavefront), so the
// vector-ALU work per k-step is what the 1e-6 guarantee costs.  The 8 x 4 tree
// is the cheapest member of the family "chain length + tree depth <= 7": seven
// binary32 additions, one conversion and one binary64 addition per 32 k-steps.
// TAO_FLAG_FAST_ACCUM skips all of it (one FP32 chain over K).
//
// Tiling: 128x128 output tile per 512-thread workgroup: eight wavefronts (4 along
// M, 2 along N), each owning two 32x32 MFMA tiles.  K advances in groups of 32;
// |A| and |W| slabs travel global -> registers -> LDS with the sign bit cleared
// on the way in, through four LDS stages with one barrier per two groups; the
// operand registers of the next group are requested from LDS in three pieces
// spread over the current group.
#include <type_traits>
#include "tao_device.hpp"
#include "tao_host.hpp"

namespace tao {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;               // k-steps per group
constexpr int BN = 128;              // output columns per workgroup (both tile shapes)
constexpr int SA = BK + 4;          // LDS row stride (floats) of a k-contiguous slab: 16-byte reads
                                    // of 16 consecutive rows fall in distinct 16-byte bank groups
constexpr int SWT = BN + 2;         // LDS row stride of a [k][n] slab (trans_w): the two k-halves
                                    // of a wavefront (16 rows apart) read disjoint bank halves
constexpr int kLinThreads = 512;    // 8 wavefronts
// Two tile shapes, chosen by the host: WM = 4 wavefronts along M x 2 along N, each owning two
// 32x32 MFMA tiles (128 x 128 outputs per workgroup), or, for problems with too few such tiles to
// fill the chip, WM = 2 x 4 wavefronts of one MFMA tile each (64 x 128 outputs per workgroup).
template <int WM> struct Shape {
    static constexpr int kWN = 8 / WM;                 // wavefronts along N
    static constexpr int kTN = BN / (32 * kWN);        // MFMA tiles per wavefront (along N)
    static constexpr int kBM = 32 * WM;
    static constexpr int kVecA = kBM * BK / 4 / kLinThreads;   // float4 per thread and group
    static constexpr int kVecW = BN * BK / 4 / kLinThreads;
    // one LDS stage holds a kBM x 32 slab of |A| and a 128 x 32 slab of |W|
    static constexpr int kStageFloats = kBM * SA + (BN * SA > BK * SWT ? BN * SA : BK * SWT);
};

struct LinArgs {
    const float* A; const float* W; const float* bias; float* tau;
    long M, N, K, lda, ldw, ldt, strideA, strideW, strideT;
    unsigned tiles_n, tiles_m, ntiles;   // output tiles along N, along M, in all (x batch)
    int vecA, vecW;            // 16-byte global loads allowed
    int fast_ok;               // vecA && vecW && per-thread slab offsets fit in 32 bits
    int all_clean;             // every tile interior and K a multiple of the group size
    double c;                  // Gamma(K'), upper
    double infl;               // reciprocal of the lower rounding factor of the accumulation
    double sabs, sabs0;        // absolute part of the accumulation's rounding error (roundings to subnormal
                               // results), added to a positive sum / to a sum that came out as exactly zero
    double uflow;              // optional absolute underflow term
};

// Convolution as an implicit matrix product: row m = (image, oh, ow) of the patch matrix, column
// k = (r, s, c); the patch matrix is never stored, its slabs are gathered from the channels-last
// input while they are loaded.
struct ConvGeom {
    int H, W, C, OW, S;              // input height, width, channels; output width; filter taps along W
    int sh, sw, ph, pw, dh, dw;      // stride, padding, dilation
    unsigned ohow;                   // output pixels per image
    unsigned xbytes;                 // bytes of the input (range of the buffer descriptor)
    int c_fast;                      // a 32-wide k slab lies inside one tap and 16-byte gathers are allowed
};
struct NoConv {};
template <bool CONV> struct ConvSel { using type = NoConv; };
template <> struct ConvSel<true> { using type = ConvGeom; };
// byte offset no input reaches on the gather path (inputs there are at most 2^31 bytes): a
// buffer load at it is out of range and returns zeros, which is what a padding tap contributes
constexpr unsigned kConvOutside = 0xC0000000u;

__device__ __forceinline__ float4 abs4(float4 v) {
    return make_float4(fabsf(v.x), fabsf(v.y), fabsf(v.z), fabsf(v.w));
}

// Load one float4 of row `r` (global row index, < nrows) at column k (< K), zero beyond the edges.
__device__ __forceinline__ float4 gload(const float* __restrict__ base, long r, long nrows, long ld,
                                        long k, long K, int vec) {
    if (r >= nrows || k >= K) return make_float4(0.f, 0.f, 0.f, 0.f);
    const float* p = base + r * ld + k;
    if (vec && k + 3 < K) return *reinterpret_cast<const float4*>(p);
    float4 v;
    v.x = p[0];
    v.y = (k + 1 < K) ? p[1] : 0.f;
    v.z = (k + 2 < K) ? p[2] : 0.f;
    v.w = (k + 3 < K) ? p[3] : 0.f;
    return v;
}

constexpr int kStages = 4;            // a power of two (stage index = group & 3)

#define TAO_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0)

// CLEAN: every tile is interior and K is a multiple of the group size (decided by the host), so
// every group takes the buffer-load path and the kernel holds no edge-handling code at all; the
// general kernel keeps both paths.  (Separate kernels rather than a branch: with the
// edge-handling loads in the same control flow the compiler's wait-count bookkeeping turns
// conservative and waits for the youngest requests as well, and the scalar registers overflow.)
// PERSIST: a workgroup walks several tiles (short K loops, where the start-up and the epilogue of
// a tile would otherwise stay exposed); without it one workgroup computes one tile and the steady
// loop carries no tile bookkeeping (measured 2 - 3 % faster for long K loops).
// CONV: the A operand is the implicit patch matrix of a convolution (geometry in `cv`).
template <bool TRANS_W, bool FAST, int WM, bool CLEAN, bool PERSIST, bool CONV = false>
__global__ __launch_bounds__(kLinThreads) void absgemm_bound(LinArgs p, typename ConvSel<CONV>::type cv) {
    static_assert(!CONV || (!TRANS_W && !PERSIST), "convolution: k-contiguous filters, one tile per workgroup");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int BM = Shape<WM>::kBM, WN = Shape<WM>::kWN, TN = Shape<WM>::kTN;
    constexpr int kVecA = Shape<WM>::kVecA, kVecW = Shape<WM>::kVecW;
    constexpr int kStageFloats = Shape<WM>::kStageFloats;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int r32 = lane & 31, h = lane >> 5;

    // A workgroup walks the output tiles blockIdx.x, blockIdx.x + gridDim.x, ... (tile index:
    // column tile fastest, then row tile, then batch entry).  Its K loops are concatenated into
    // one stream of 32-k-step groups, so the software pipeline below runs across tile boundaries:
    // the first slabs of the next tile are requested while the current tile still computes, and
    // only the epilogue (the bound of one tile written out) sits between two tiles.
    const unsigned nwg = gridDim.x;
    const unsigned my_tiles = !PERSIST ? 1u : (blockIdx.x < p.ntiles ? (p.ntiles - 1 - blockIdx.x) / nwg + 1 : 0u);
    const long ngroup = (p.K + BK - 1) / BK;
    const long total = (long)my_tiles * ngroup;            // groups of this workgroup
    struct Origin { long m0, n0, z; };
    auto origin = [&](unsigned t) __attribute__((always_inline)) {
        const unsigned x = t % p.tiles_n, yz = t / p.tiles_n;
        Origin o;
        o.n0 = (long)x * BN; o.m0 = (long)(yz % p.tiles_m) * BM; o.z = yz / p.tiles_m;
        return o;
    };

    // global -> register -> LDS mapping.  k-contiguous slab [rows][32]: thread -> rows
    // tid/8 + 64*i, columns 4*(tid%8): eight threads fetch 128 contiguous bytes of a row.
    // [k][n] slab of a transposed W: rows tid/32 + 16*i, columns 4*(tid%32).
    const int ld_row = tid >> 3, ld_k = (tid & 7) * 4;
    const int lt_kr = tid >> 5, lt_n = (tid & 31) * 4;
    const unsigned offA = (unsigned)((ld_row * p.lda + ld_k) * 4);
    const unsigned offW = TRANS_W ? (unsigned)((lt_kr * p.ldw + lt_n) * 4) : (unsigned)((ld_row * p.ldw + ld_k) * 4);
    const long strideAi = 64 * p.lda * 4;                              // bytes between a thread's vectors
    const long strideWi = (TRANS_W ? 16 : 64) * p.ldw * 4;
    const int stA = ld_row * SA + ld_k;                                // + 64*SA*i
    const int stW = BM * SA + (TRANS_W ? lt_kr * SWT + lt_n : ld_row * SA + ld_k);   // + 16*SWT*i or 64*SA*i
    const long slabW = TRANS_W ? (long)BK * p.ldw * 4 : (long)BK * 4;  // bytes per group along K
    // bytes one group's slab spans from its first element (both below 2^31 when fast_ok)
    const long spanA = ((long)(BM - 1) * p.lda + BK) * 4;
    const long spanW = TRANS_W ? ((long)(BK - 1) * p.ldw + BN) * 4 : ((long)(BN - 1) * p.ldw + BK) * 4;

    // Request side of the pipeline: the tile and group of the next slab to request.  Slabs are
    // requested strictly in stream order, one call of load_slab each.
    unsigned l_tile = blockIdx.x;
    long l_g = 0, l_m0 = 0, l_n0 = 0;
    const float* l_A = p.A; const float* l_W = p.W;     // batch entry (edge path)
    const char* l_pa0 = nullptr; const char* l_pw0 = nullptr; // first byte of the tile's first slab
    bool l_interior = false;
    // convolution: the tap (l_r, l_s) and first channel l_c0 of the next slab (gather path), and
    // per patch row of this thread the input coordinates of tap (0, 0), the byte offset of its
    // first element (gather path) and its pixel index (edge path; -1 marks a row beyond M)
    int l_r = 0, l_s = 0, l_c0 = 0;
    int cv_ih0[kVecA], cv_iw0[kVecA];
    unsigned cv_base[kVecA];
    long cv_pix[kVecA];
    auto set_load_tile = [&](unsigned t) __attribute__((always_inline)) {
        const Origin o = origin(t);
        l_m0 = o.m0; l_n0 = o.n0;
        l_A = p.A + o.z * p.strideA; l_W = p.W + o.z * p.strideW;
        l_pa0 = reinterpret_cast<const char*>(l_A + o.m0 * p.lda);
        l_pw0 = reinterpret_cast<const char*>(TRANS_W ? l_W + o.n0 : l_W + o.n0 * p.ldw);
        // Interior tiles of aligned operands take unguarded 16-byte loads
        l_interior = (o.m0 + BM <= p.M) && (o.n0 + BN <= p.N) && p.fast_ok;
        if constexpr (CONV) {
#pragma unroll
            for (int i = 0; i < kVecA; ++i) {
                const long m = o.m0 + ld_row + 64 * i;
                const bool row_ok = m < p.M;
                const unsigned mm = row_ok ? (unsigned)m : 0u;
                const unsigned img = mm / cv.ohow, rem = mm - img * cv.ohow;
                const unsigned oh = rem / (unsigned)cv.OW, ow = rem - oh * (unsigned)cv.OW;
                cv_ih0[i] = (int)oh * cv.sh - cv.ph;
                cv_iw0[i] = (int)ow * cv.sw - cv.pw;
                const long pix = ((long)img * cv.H + cv_ih0[i]) * cv.W + cv_iw0[i];
                cv_pix[i] = pix;
                cv_base[i] = (unsigned)((pix * cv.C + ld_k) * 4);      // modulo 2^32; exact whenever the tap is inside
                if (!row_ok) cv_ih0[i] = -(1 << 30);                   // no tap of such a row is inside
            }
        }
    };
    if (my_tiles > 0) set_load_tile(l_tile);

    // two register sets: the slab requested during group g is written to LDS during group g+2
    float4 ra0[kVecA], rw0[kVecW], ra1[kVecA], rw1[kVecW];
    auto load_slab = [&](float4* ra, float4* rw) __attribute__((always_inline)) {
        const long k0 = l_g * BK;
        if constexpr (CONV) {
            if (CLEAN || (l_interior && k0 + BK <= p.K)) {
                // Gather path: the slab is 32 consecutive channels of one tap, 128 contiguous bytes
                // per patch row; rows whose tap falls into the padding read out of range (zeros).
                const int dr = l_r * cv.dh, ds = l_s * cv.dw;
                const unsigned tap = (unsigned)(((dr * cv.W + ds) * cv.C + l_c0) * 4);
                const __amdgpu_buffer_rsrc_t dx = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.A), 0, (int)cv.xbytes, 0x00020000);
                const char* pw = l_pw0 + l_g * slabW;
                const __amdgpu_buffer_rsrc_t dw = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(pw), 0, (int)spanW, 0x00020000);
#pragma unroll
                for (int i = 0; i < kVecA; ++i) {
                    const bool inside = (unsigned)(cv_ih0[i] + dr) < (unsigned)cv.H && (unsigned)(cv_iw0[i] + ds) < (unsigned)cv.W;
                    const unsigned off = inside ? cv_base[i] + tap : kConvOutside;
                    ra[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(dx, (int)off, 0, 0));
                }
#pragma unroll
                for (int i = 0; i < kVecW; ++i)
                    rw[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(dw, (int)offW, (int)(strideWi * i), 0));
                l_c0 += BK;
                if (l_c0 >= cv.C) { l_c0 = 0; if (++l_s == cv.S) { l_s = 0; ++l_r; } }
            } else {
                // Edge path: element by element, k -> (tap, channel) -> (r, s)
#pragma unroll
                for (int i = 0; i < kVecA; ++i) {
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const long k = k0 + ld_k + j;
                        v[j] = 0.f;
                        if (k < p.K) {
                            const unsigned tp = (unsigned)k / (unsigned)cv.C, ch = (unsigned)k - tp * (unsigned)cv.C;
                            const unsigned r = tp / (unsigned)cv.S, sx = tp - r * (unsigned)cv.S;
                            const int dr = (int)r * cv.dh, ds = (int)sx * cv.dw;
                            if ((unsigned)(cv_ih0[i] + dr) < (unsigned)cv.H && (unsigned)(cv_iw0[i] + ds) < (unsigned)cv.W)
                                v[j] = p.A[(cv_pix[i] + (long)dr * cv.W + ds) * cv.C + ch];
                        }
                    }
                    ra[i] = make_float4(v[0], v[1], v[2], v[3]);
                }
#pragma unroll
                for (int i = 0; i < kVecW; ++i)
                    rw[i] = gload(l_W, l_n0 + ld_row + 64 * i, p.N, p.ldw, k0 + ld_k, p.K, p.vecW);
            }
            ++l_g;
            return;
        }
        if (CLEAN || (l_interior && k0 + BK <= p.K)) {
            // Buffer loads: descriptor (uniform base of this group's slab) in SGPRs, one 32-bit
            // per-thread offset, the vector index as a scalar offset.  Next to FP32 MFMA this
            // form is nearly free, while loads with a 64-bit per-lane address stall the SIMD.
            // (addressed from the tile's base rather than through a running pointer: the compiler
            // then splits the four requests around the LDS writes, measured 1.4 % faster)
            const char* pa = l_pa0 + k0 * 4;
            const char* pw = l_pw0 + l_g * slabW;
            const __amdgpu_buffer_rsrc_t da = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(pa), 0, (int)spanA, 0x00020000);
            const __amdgpu_buffer_rsrc_t dw = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(pw), 0, (int)spanW, 0x00020000);
#pragma unroll
            for (int i = 0; i < kVecA; ++i)
                ra[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(da, (int)offA, (int)(strideAi * i), 0));
#pragma unroll
            for (int i = 0; i < kVecW; ++i)
                rw[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(dw, (int)offW, (int)(strideWi * i), 0));
        } else {
#pragma unroll
            for (int i = 0; i < kVecA; ++i)
                ra[i] = gload(l_A, l_m0 + ld_row + 64 * i, p.M, p.lda, k0 + ld_k, p.K, p.vecA);
#pragma unroll
            for (int i = 0; i < kVecW; ++i)
                rw[i] = TRANS_W ? gload(l_W, k0 + lt_kr + 16 * i, p.K, p.ldw, l_n0 + lt_n, p.N, p.vecW)
                                : gload(l_W, l_n0 + ld_row + 64 * i, p.N, p.ldw, k0 + ld_k, p.K, p.vecW);
        }
        // advance to the next slab of the stream (no memory operation here)
        ++l_g;
        if (PERSIST && l_g == ngroup) {
            l_g = 0; l_tile += nwg;
            if (l_tile < p.ntiles) set_load_tile(l_tile);
        }
    };
    // registers -> LDS stage, sign bits cleared
    auto commit = [&](float* stage, const float4* ra, const float4* rw) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kVecA; ++i) *reinterpret_cast<float4*>(stage + stA + 64 * SA * i) = abs4(ra[i]);
#pragma unroll
        for (int i = 0; i < kVecW; ++i) {
            const float4 w = abs4(rw[i]);
            if (!TRANS_W) {
                *reinterpret_cast<float4*>(stage + stW + 64 * SA * i) = w;
            } else {
                float2* dw = reinterpret_cast<float2*>(stage + stW + 16 * SWT * i);
                dw[0] = make_float2(w.x, w.y); dw[1] = make_float2(w.z, w.w);
            }
        }
    };

    // S: binary64 running sums (tight mode); c0: the single FP32 chain (fast mode)
    double S[TN][16];
    floatx16 c0[TN];
    auto clear_sums = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
#pragma unroll
            for (int v = 0; v < 16; ++v) { S[tj][v] = 0.0; c0[tj][v] = 0.f; }
        }
    };
    clear_sums();
    floatx16 zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) zero[v] = 0.f;

    // The bound of one finished tile: D[i][j] of a 32x32 tile sits in lane (j + 32*((i/4)%2)),
    // register 4*(i/8) + i%4.
    auto epilogue = [&](unsigned t) __attribute__((always_inline)) {
        const Origin o = origin(t);
        float* __restrict__ T = p.tau + o.z * p.strideT;
#pragma unroll
        for (int tj = 0; tj < TN; ++tj) {
            const long col = o.n0 + (wn * TN + tj) * 32 + r32;
            const double ab = (p.bias && col < p.N) ? fabs((double)p.bias[col]) : 0.0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const long row = o.m0 + wm * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < p.M && col < p.N) {
                    const double sv = FAST ? (double)c0[tj][v] : S[tj][v];
                    const double tt = p.c * ((sv + (sv > 0.0 ? p.sabs : p.sabs0)) * p.infl + ab) * kGuard + p.uflow;
                    T[row * p.ldt + col] = up32(tt);
                }
            }
        }
    };
    if (ngroup == 0) {                       // K == 0: tau = Gamma |bias|
        for (unsigned i = 0; i < my_tiles; ++i) epilogue(blockIdx.x + i * nwg);
        return;
    }

    // Operand registers of one group: lane (r32, h) holds k = 16h .. 16h+15 of its A row and of
    // its W row in each tile; MFMA number i of the group multiplies element i of both.
    const int fragA = (wm * 32 + r32) * SA + 16 * h;
    const int fragW = BM * SA + (TRANS_W ? (16 * h) * SWT + wn * 32 * TN + r32 : (wn * 32 * TN + r32) * SA + 16 * h);
    // fb[j]: with two tiles per wavefront the W operands of tile j; with one tile the two
    // buffers alternate between groups (j = parity of the group)
    float fa[16], fb[2][16];
    auto read_a = [&](const float* st) __attribute__((always_inline)) {
        const float4* sa = reinterpret_cast<const float4*>(st + fragA);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 v = sa[j];
            fa[4 * j] = v.x; fa[4 * j + 1] = v.y; fa[4 * j + 2] = v.z; fa[4 * j + 3] = v.w;
        }
    };
    auto read_b = [&](const float* st, int buf) __attribute__((always_inline)) {
        const int tj = TN == 2 ? buf : 0;       // tile whose operands are read
        if (!TRANS_W) {
            const float4* sw = reinterpret_cast<const float4*>(st + fragW + tj * 32 * SA);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 v = sw[j];
                fb[buf][4 * j] = v.x; fb[buf][4 * j + 1] = v.y; fb[buf][4 * j + 2] = v.z; fb[buf][4 * j + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) fb[buf][j] = st[fragW + j * SWT + tj * 32];
        }
    };

    // Four LDS stages and two register sets.  Slab j of the stream (32 k-steps of both operands)
    // is requested from global memory during group j-4, written to stage j%4 at the top of group
    // j-2, and read into operand registers in three pieces: the W operands of tile 1 at the top
    // of group j, the W operands of tile 0 in the middle of group j-1, the A operands at the end
    // of group j-1.  One barrier in the middle of every EVEN group is enough: between the write
    // of a stage (top of group j-2) and its first read (middle of group j-1) lies the barrier of
    // j-2 or of j-1, and between its last read as slab j-4 (top of group j-4) and that write lies
    // the barrier of j-4 or of j-3.  Requests run two groups ahead of the registers' use, which
    // covers the memory latency with a single workgroup per CU.  With one tile per wavefront
    // (64-row workgroup tiles) the W operands of group j are read at the top of group j-1 into
    // the buffer the current group does not use, and the barrier sits at the top of the even
    // groups, right after the LDS write; the same two arguments hold.
    auto stage = [&](long j) __attribute__((always_inline)) { return lds + (int)(j & (kStages - 1)) * kStageFloats; };
    // the MFMA / vector-ALU work of one 32x32 tile over one group: accumulator `acc`, W operands
    // from fb[buf]; `last`: the group's last tile, which requests the next group's A operands
    // as soon as its last MFMA has been issued
    auto tile = [&](int acc, int buf, bool last, bool have_next, long g) __attribute__((always_inline)) {
        if (FAST) {
#pragma unroll
            for (int i = 0; i < 16; ++i) c0[acc] = TAO_MFMA(fa[i], fb[buf][i], c0[acc]);
            if (last && have_next) read_a(stage(g + 1));
            __builtin_amdgcn_sched_barrier(0);
        } else {
            floatx16 x, z;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                // two chains of 4 k-steps from zero, interleaved
                floatx16 pc = TAO_MFMA(fa[4 * c], fb[buf][4 * c], zero);
                floatx16 qc = TAO_MFMA(fa[4 * c + 2], fb[buf][4 * c + 2], zero);
                pc = TAO_MFMA(fa[4 * c + 1], fb[buf][4 * c + 1], pc);
                qc = TAO_MFMA(fa[4 * c + 3], fb[buf][4 * c + 3], qc);
                if (last && c == 3 && have_next) read_a(stage(g + 1));
                if (c == 0) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) x[v] = pc[v] + qc[v];
                } else if (c == 1) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) x[v] = x[v] + (pc[v] + qc[v]);
                } else if (c == 2) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = pc[v] + qc[v];
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) S[acc][v] += (double)(x[v] + (z[v] + (pc[v] + qc[v])));
                }
                // keep the chain pairs and their additions in program order, so that at most
                // two accumulators are live next to x and z
                if (c < 2) asm volatile("" : "+v"(x));
                if (c == 2) asm volatile("" : "+v"(z));
                if (c == 3) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) asm volatile("" : "+v"(S[acc][v]));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // Compute side of the pipeline: tile and group of the group being consumed.
    unsigned c_tile = blockIdx.x;
    long c_g = 0;
    // one group of the stream; (ra, rw) is the register set of the group's parity (`even`)
    auto group = [&](auto steady, auto even_t, long g, float4* ra, float4* rw) __attribute__((always_inline)) {
        // steady (compile time): groups g+1 .. g+4 exist, so nothing below is conditional
        constexpr bool ST = decltype(steady)::value;
        constexpr bool even = decltype(even_t)::value;
        const bool have_next = ST || g + 1 < total;
        if (ST || g + 2 < total) commit(stage(g + 2), ra, rw);
        if (ST || g + 4 < total) load_slab(ra, rw);
        if (TN == 2) {
            read_b(stage(g), 1);                          // W operands of this group's tile 1
            tile(0, 0, false, have_next, g);
            if (even) __syncthreads();
            if (have_next) read_b(stage(g + 1), 0);       // tile 0 of the next group (registers free now)
            tile(1, 1, true, have_next, g);
        } else {
            // one tile per wavefront: the barrier sits at the top of the even groups (after the
            // LDS write), and the W operands of the next group go to the other buffer
            if (even) __syncthreads();
            if (have_next) read_b(stage(g + 1), even ? 1 : 0);
            tile(0, even ? 0 : 1, true, have_next, g);
        }
        if (PERSIST && ++c_g == ngroup) {    // last group of an output tile
            epilogue(c_tile);
            clear_sums();
            c_g = 0; c_tile += nwg;
        }
    };
    {
        long g = 0;
        if (total >= 6) {
            // Steady state: every request, LDS write and LDS read is unconditional, from the
            // prologue on, so the wait counts the compiler derives are exact (one conditional
            // request on any path into the loop makes it wait for all outstanding requests,
            // which halves the distance between a request and its use).
            load_slab(ra0, rw0); load_slab(ra1, rw1);     // one round trip for both
            commit(stage(0), ra0, rw0); commit(stage(1), ra1, rw1);
            load_slab(ra0, rw0);
            load_slab(ra1, rw1);
            __syncthreads();
            read_a(stage(0)); read_b(stage(0), 0);
#pragma unroll 1
            for (; g + 5 < total; g += 2) {
                group(std::true_type(), std::true_type(), g, ra0, rw0);
                group(std::true_type(), std::false_type(), g + 1, ra1, rw1);
            }
        } else {
            if (total > 0) load_slab(ra0, rw0);
            if (total > 1) load_slab(ra1, rw1);
            if (total > 0) commit(stage(0), ra0, rw0);
            if (total > 1) commit(stage(1), ra1, rw1);
            if (total > 2) load_slab(ra0, rw0);
            if (total > 3) load_slab(ra1, rw1);
            __syncthreads();
            if (total > 0) { read_a(stage(0)); read_b(stage(0), 0); }
        }
        // the last groups (all of them when there are fewer than six): conditional copy
#pragma unroll 1
        for (; g < total; g += 2) {
            group(std::false_type(), std::true_type(), g, ra0, rw0);
            if (g + 1 < total) group(std::false_type(), std::false_type(), g + 1, ra1, rw1);
        }
    }
    if (!PERSIST) epilogue(blockIdx.x);
}

template <bool TRANS_W, bool FAST, int WM, bool CLEAN, bool PERSIST>
static hipError_t launch_absgemm(dim3 grid, hipStream_t st, const LinArgs& p) {
    constexpr size_t lds_bytes = (size_t)kStages * Shape<WM>::kStageFloats * sizeof(float);
    static OncePerDevice configured;      // raise the dynamic LDS limit once per instantiation and device
    const hipError_t e = configured.run([] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&absgemm_bound<TRANS_W, FAST, WM, CLEAN, PERSIST>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((absgemm_bound<TRANS_W, FAST, WM, CLEAN, PERSIST>), grid, dim3(kLinThreads), lds_bytes, st, p, NoConv());
    return hipSuccess;
}
template <bool FAST, int WM, bool CLEAN>
static hipError_t launch_conv(dim3 grid, hipStream_t st, const LinArgs& p, const ConvGeom& cv) {
    constexpr size_t lds_bytes = (size_t)kStages * Shape<WM>::kStageFloats * sizeof(float);
    static OncePerDevice configured;
    const hipError_t e = configured.run([] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&absgemm_bound<false, FAST, WM, CLEAN, false, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((absgemm_bound<false, FAST, WM, CLEAN, false, true>), grid, dim3(kLinThreads), lds_bytes, st, p, cv);
    return hipSuccess;
}
template <int WM>
static hipError_t launch_conv_shape(bool fast, bool clean, dim3 grid, hipStream_t st, const LinArgs& p, const ConvGeom& cv) {
    if (clean) return fast ? launch_conv<true, WM, true>(grid, st, p, cv) : launch_conv<false, WM, true>(grid, st, p, cv);
    return fast ? launch_conv<true, WM, false>(grid, st, p, cv) : launch_conv<false, WM, false>(grid, st, p, cv);
}
template <int WM, bool CLEAN, bool PERSIST>
static hipError_t launch_shape(bool trans_w, bool fast, dim3 grid, hipStream_t st, const LinArgs& p) {
    if (trans_w) return fast ? launch_absgemm<true, true, WM, CLEAN, PERSIST>(grid, st, p) : launch_absgemm<true, false, WM, CLEAN, PERSIST>(grid, st, p);
    return fast ? launch_absgemm<false, true, WM, CLEAN, PERSIST>(grid, st, p) : launch_absgemm<false, false, WM, CLEAN, PERSIST>(grid, st, p);
}

// Tile height.  One workgroup occupies a CU, so a launch takes ceil(tiles / CUs) rounds of one
// tile time each; a 64-row tile takes half the time of a 128-row tile plus about 9 % (one MFMA
// tile per wavefront reuses each A operand once instead of twice: measured 86 - 88 against 94 - 96
// TFLOP/s on full rounds).  Take the cheaper shape; up to 64 rows the tall tile is kept.
static bool prefer_64_row_tiles(long M, long tiles_per_row_block, int cus) {
    if (M <= 64) return false;
    const long t128 = tiles_per_row_block * ((M + 127) / 128), t64 = tiles_per_row_block * ((M + 63) / 64);
    const double c128 = (double)((t128 + cus - 1) / cus) * 128.0;
    const double c64 = (double)((t64 + cus - 1) / cus) * 64.0 * 1.09;
    return c64 < c128;
}

// A binary32 rounding whose result is subnormal loses up to 2^-150 absolutely instead of u
// relatively (gradual underflow; the matrix cores keep subnormal values).  An output element sees at
// most 39 roundings per 32 k-steps (32 chain steps and the 7 additions of the tree; K in the
// single-chain mode), each amplified by at most (1 + u)^7 afterwards, so the computed sum is at least
// S lower - sabs with sabs = (1.25 K + 40) 2^-150: the epilogue adds it to every positive sum before
// the inflation.  For sums in the normal range it is far below the 1e-6 budget (K^2 2^-48 of a
// bound of 2^-126).  A sum that comes out as exactly zero is taken as an exact zero (every product
// zero: padding taps, zero operands) -- unless the caller asked for underflow terms, in which case
// it may also be a sum whose every product rounded to zero, and sabs is added there as well.
static double accumulation_abs_term(long K) { return K > 0 ? (1.25 * (double)K + 40.0) * 0x1p-150 : 0.0; }

// ---- matrix-core self test ----------------------------------------------------------------
// out[v*64 + lane] = register v of the accumulator after `steps` chained MFMAs from zero.
__global__ void mfma_probe(const float* __restrict__ a, const float* __restrict__ b, int steps,
                           float* __restrict__ out) {
    const int lane = threadIdx.x;
    floatx16 c;
    for (int v = 0; v < 16; ++v) c[v] = 0.f;
    for (int s = 0; s < steps; ++s)
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s * 64 + lane], b[s * 64 + lane], c, 0, 0, 0);
    for (int v = 0; v < 16; ++v) out[v * 64 + lane] = c[v];
}

}  // namespace tao

extern "C" {

int tao_bound_linear(const float* A, const float* W, const float* bias, float* tau,
                     long M, long N, long K, long lda, long ldw, long ldt, int trans_w,
                     long batch, long strideA, long strideW, long strideT,
                     const tao_fp_model* model, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (M < 0 || N < 0 || K < 0 || batch < 0) return TAO_ERR_SHAPE;
    if (lda < K || ldt < N || ldw < (trans_w ? N : K)) return TAO_ERR_SHAPE;
    if (strideA < 0 || strideW < 0 || strideT < 0) return TAO_ERR_SHAPE;
    if (batch > 1 && strideT < M * ldt - (ldt - N)) return TAO_ERR_SHAPE;   // outputs would overlap
    const long Kp = K + (bias ? 1 : 0);
    const double c = gamma_up(Kp, md);
    if (!(c == c)) return TAO_ERR_K_RANGE;
    if (M == 0 || N == 0 || batch == 0) return TAO_OK;
    if (!tau || (K > 0 && (!A || !W))) return TAO_ERR_NULL;
    if (!aligned(A, 4) || !aligned(W, 4) || !aligned(bias, 4) || !aligned(tau, 4)) return TAO_ERR_ALIGN;

    LinArgs p;
    p.A = A; p.W = W; p.bias = bias; p.tau = tau;
    p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldw = ldw; p.ldt = ldt;
    p.strideA = strideA; p.strideW = strideW; p.strideT = strideT;
    p.vecA = aligned(A, 16) && (lda % 4 == 0) && (strideA % 4 == 0);
    p.vecW = aligned(W, 16) && (ldw % 4 == 0) && (strideW % 4 == 0);
    {   // byte offsets inside one slab must fit in 32 bits for the unguarded load path
        const long spanA = ((long)(128 - 1) * lda + BK) * 4;
        const long spanW = trans_w ? ((long)(BK - 1) * ldw + BN) * 4 : ((long)(BN - 1) * ldw + BK) * 4;
        p.fast_ok = p.vecA && p.vecW && (K % 4 == 0) && spanA < (1L << 31) && spanW < (1L << 31);
    }
    p.c = c;
    const bool fast = (md.flags & TAO_FLAG_FAST_ACCUM) != 0;
    const double u = md.u;
    // lower rounding factor: (1-u)^r (1-2^-53)^f with r roundings in binary32, f in binary64
    const double r32 = fast ? (double)(K > 0 ? K : 1) : 7.0;
    const double f64 = (double)(K / 32 + 2);
    if (!(r32 * u < 0.5)) return TAO_ERR_K_RANGE;
    const double lower = (1.0 - r32 * u) * (1.0 - f64 * 0x1p-53);   // <= (1-u)^r (1-2^-53)^f
    p.infl = widen(1.0 / (lower * (1.0 - 0x1p-52)));
    p.sabs = accumulation_abs_term(K);
    p.sabs0 = (md.flags & TAO_FLAG_UNDERFLOW_TERMS) ? p.sabs : 0.0;
    p.uflow = (md.flags & TAO_FLAG_UNDERFLOW_TERMS) ? (double)Kp * 0x1p-149 : 0.0;

    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus < 1) cus = 256;
    const long tiles_n = (N + BN - 1) / BN;
    const bool small = prefer_64_row_tiles(M, tiles_n * batch, cus);
    const long bm = small ? 64 : 128;
    const long tiles_m = (M + bm - 1) / bm;
    const long ntiles = tiles_n * tiles_m * batch;
    if (ntiles >= (1L << 31)) return TAO_ERR_SHAPE;
    p.tiles_n = (unsigned)tiles_n; p.tiles_m = (unsigned)tiles_m; p.ntiles = (unsigned)ntiles;
    p.all_clean = p.fast_ok && (M % bm == 0) && (N % BN == 0) && (K % BK == 0);
    // One workgroup per CU walks several tiles when every tile is regular and the K loop is short
    // (its pipeline then runs across tile boundaries); otherwise one workgroup per tile.
    const bool persist = p.all_clean && ntiles > cus && K <= 32 * BK;
    dim3 grid((unsigned)(persist ? cus : ntiles));
    hipStream_t st = (hipStream_t)stream;
    const bool tw = trans_w != 0;
    hipError_t e;
    if (persist)          e = small ? launch_shape<2, true, true>(tw, fast, grid, st, p) : launch_shape<4, true, true>(tw, fast, grid, st, p);
    else if (p.all_clean) e = small ? launch_shape<2, true, false>(tw, fast, grid, st, p) : launch_shape<4, true, false>(tw, fast, grid, st, p);
    else                  e = small ? launch_shape<2, false, false>(tw, fast, grid, st, p) : launch_shape<4, false, false>(tw, fast, grid, st, p);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return TAO_ERR_LAUNCH; }
    return launch_status();
}

int tao_bound_conv2d(const float* x, const float* w, const float* bias, float* tau,
                     long batch, long H, long W, long C, long Cout, long R, long S,
                     long stride_h, long stride_w, long pad_h, long pad_w, long dil_h, long dil_w,
                     const tao_fp_model* model, void* stream) {
    using namespace tao;
    tao_fp_model md;
    int rc = resolve_model(model, &md);
    if (rc != TAO_OK) return rc;
    if (batch < 0 || H < 0 || W < 0 || C < 0 || Cout < 0 || R < 1 || S < 1) return TAO_ERR_SHAPE;
    if (stride_h < 1 || stride_w < 1 || dil_h < 1 || dil_w < 1 || pad_h < 0 || pad_w < 0) return TAO_ERR_SHAPE;
    const long lim = 1L << 28;       // each extent, so that coordinate arithmetic stays in 32 bits
    if (H >= lim || W >= lim || C >= lim || R >= lim || S >= lim || Cout >= lim || batch >= lim ||
        stride_h >= lim || stride_w >= lim || dil_h >= lim || dil_w >= lim || pad_h >= lim || pad_w >= lim) return TAO_ERR_SHAPE;
    const long eh = H + 2 * pad_h - dil_h * (R - 1) - 1, ew = W + 2 * pad_w - dil_w * (S - 1) - 1;
    if (eh < 0 || ew < 0) return TAO_ERR_SHAPE;          // filter larger than the padded input
    const long OH = eh / stride_h + 1, OW = ew / stride_w + 1;
    if (dil_h * (R - 1) >= lim || dil_w * (S - 1) >= lim) return TAO_ERR_SHAPE;
    // patch-matrix shape; every index the kernel forms must fit its integer types
    const __int128 M128 = (__int128)batch * OH * OW, K128 = (__int128)R * S * C;
    if (M128 >= (1L << 31) || K128 >= (1L << 31) || OH * OW >= (1L << 31)) return TAO_ERR_SHAPE;
    const long M = (long)M128, K = (long)K128, N = Cout;
    if ((__int128)batch * H * W * C >= ((__int128)1 << 61) || (__int128)M * N >= ((__int128)1 << 61)) return TAO_ERR_SHAPE;
    const long Kp = K + (bias ? 1 : 0);
    const double c = gamma_up(Kp, md);
    if (!(c == c)) return TAO_ERR_K_RANGE;
    if (M == 0 || N == 0) return TAO_OK;
    const long xbytes = batch * H * W * C * 4;
    if (!tau || (K > 0 && !w) || (K > 0 && xbytes > 0 && !x)) return TAO_ERR_NULL;
    if (!aligned(x, 4) || !aligned(w, 4) || !aligned(bias, 4) || !aligned(tau, 4)) return TAO_ERR_ALIGN;

    LinArgs p;
    p.A = x; p.W = w; p.bias = bias; p.tau = tau;
    p.M = M; p.N = N; p.K = K; p.lda = K; p.ldw = K; p.ldt = N;
    p.strideA = 0; p.strideW = 0; p.strideT = 0;
    ConvGeom cv;
    cv.H = (int)H; cv.W = (int)W; cv.C = (int)C; cv.OW = (int)OW; cv.S = (int)S;
    cv.sh = (int)stride_h; cv.sw = (int)stride_w; cv.ph = (int)pad_h; cv.pw = (int)pad_w;
    cv.dh = (int)dil_h; cv.dw = (int)dil_w;
    cv.ohow = (unsigned)(OH * OW);
    // gather path: whole 32-channel slabs inside one tap, 16-byte aligned, input within 2^31 bytes,
    // and the tap offset (dil_h (R-1) W + dil_w (S-1)) C * 4 within 32 bits
    cv.c_fast = (C % BK == 0) && aligned(x, 16) && xbytes <= (1L << 31) &&
                (__int128)(dil_h * (R - 1) * W + dil_w * (S - 1) + 1) * C * 4 < ((__int128)1 << 31);
    cv.xbytes = cv.c_fast ? (unsigned)xbytes : 0u;
    p.vecA = cv.c_fast;
    p.vecW = aligned(w, 16) && (K % 4 == 0);
    p.fast_ok = cv.c_fast && p.vecW && ((long)(BN - 1) * K + BK) * 4 < (1L << 31);
    p.c = c;
    const bool fast = (md.flags & TAO_FLAG_FAST_ACCUM) != 0;
    const double u = md.u;
    const double r32 = fast ? (double)(K > 0 ? K : 1) : 7.0;
    const double f64 = (double)(K / 32 + 2);
    if (!(r32 * u < 0.5)) return TAO_ERR_K_RANGE;
    const double lower = (1.0 - r32 * u) * (1.0 - f64 * 0x1p-53);
    p.infl = widen(1.0 / (lower * (1.0 - 0x1p-52)));
    p.sabs = accumulation_abs_term(K);
    p.sabs0 = (md.flags & TAO_FLAG_UNDERFLOW_TERMS) ? p.sabs : 0.0;
    p.uflow = (md.flags & TAO_FLAG_UNDERFLOW_TERMS) ? (double)Kp * 0x1p-149 : 0.0;

    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus < 1) cus = 256;
    const long tiles_n = (N + BN - 1) / BN;
    const bool small = prefer_64_row_tiles(M, tiles_n, cus);
    const long bm = small ? 64 : 128;
    const long tiles_m = (M + bm - 1) / bm;
    const long ntiles = tiles_n * tiles_m;
    if (ntiles >= (1L << 31)) return TAO_ERR_SHAPE;
    p.tiles_n = (unsigned)tiles_n; p.tiles_m = (unsigned)tiles_m; p.ntiles = (unsigned)ntiles;
    p.all_clean = p.fast_ok && (M % bm == 0) && (N % BN == 0) && (K % BK == 0);
    dim3 grid((unsigned)ntiles);
    hipStream_t st = (hipStream_t)stream;
    const hipError_t e = small ? launch_conv_shape<2>(fast, p.all_clean != 0, grid, st, p, cv)
                               : launch_conv_shape<4>(fast, p.all_clean != 0, grid, st, p, cv);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return TAO_ERR_LAUNCH; }
    return launch_status();
}

int tao_selftest_matrix_core(unsigned* report, void* ws, size_t ws_bytes, void* stream) {
    using namespace tao;
    if (!report) return TAO_ERR_NULL;
    if (!ws || !aligned(ws, 256) || ws_bytes < 8192) return TAO_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int kSteps = 3;
    float ha[kSteps * 64], hb[kSteps * 64], hout[16 * 64];
    float* da = static_cast<float*>(ws);
    float* db = da + kSteps * 64;
    float* dout = db + kSteps * 64;
    auto fail = [&](hipError_t e) { g_last_hip_error = (int)e; return TAO_ERR_LAUNCH; };
    hipError_t e;
    auto run = [&](int steps) -> hipError_t {
        hipError_t r;
        if ((r = hipMemcpyAsync(da, ha, sizeof(ha), hipMemcpyHostToDevice, st)) != hipSuccess) return r;
        if ((r = hipMemcpyAsync(db, hb, sizeof(hb), hipMemcpyHostToDevice, st)) != hipSuccess) return r;
        hipLaunchKernelGGL(mfma_probe, dim3(1), dim3(64), 0, st, da, db, steps, dout);
        if ((r = hipGetLastError()) != hipSuccess) return r;
        if ((r = hipMemcpyAsync(hout, dout, sizeof(hout), hipMemcpyDeviceToHost, st)) != hipSuccess) return r;
        return hipStreamSynchronize(st);
    };
    // operand element (i, k) of A lives in lane i + 32 k; element (k, j) of B in lane j + 32 k
    auto D = [&](int i, int j) { return hout[(4 * (i / 8) + i % 4) * 64 + j + 32 * ((i / 4) % 2)]; };
    unsigned rep = 0;

    // (a) rounding of the accumulation and subnormals: one instruction, D[i][0] = x_i * 1 + y_i * 1
    for (int k = 0; k < kSteps * 64; ++k) { ha[k] = 0.f; hb[k] = 0.f; }
    hb[0] = 1.f;             // B[0][0]
    hb[32] = 1.f;            // B[1][0]
    hb[1] = 0x1p-100f;       // B[0][1]
    ha[0] = 1.f;              ha[32 + 0] = 0x1p-24f;       // tie, even below: stays 1
    ha[1] = 1.f + 0x1p-23f;   ha[32 + 1] = 0x1p-24f;       // tie, even above: 1 + 2^-22
    ha[2] = 1.f;              ha[32 + 2] = 0x1.8p-24f;     // above the tie: 1 + 2^-23
    ha[3] = 0x1p-40f;                                       // times 2^-100: subnormal product
    ha[4] = 0x1p-130f;                                      // subnormal operand
    if ((e = run(1)) != hipSuccess) return fail(e);
    if (D(0, 0) == 1.f && D(1, 0) == 1.f + 0x1p-22f && D(2, 0) == 1.f + 0x1p-23f) rep |= 1u;
    if (D(3, 1) == 0x1p-140f && D(4, 0) == 0x1p-130f) rep |= 2u;

    // (b) three chained instructions on pseudo-random non-negative data vs the exact sum
    unsigned long long lcg = 0x9E3779B97F4A7C15ull;
    auto rnd = [&]() { lcg = lcg * 6364136223846793005ull + 1442695040888963407ull; return (float)((lcg >> 40) + 1) * 0x1p-24f; };
    for (int k = 0; k < kSteps * 64; ++k) { ha[k] = rnd(); hb[k] = rnd() * 4.f; }
    if ((e = run(kSteps)) != hipSuccess) return fail(e);
    bool within = true;
    const double g6 = 6.0 * 0x1p-24 / (1.0 - 6.0 * 0x1p-24);
    for (int i = 0; i < 32 && within; ++i)
        for (int j = 0; j < 32; ++j) {
            double s = 0.0;
            for (int st3 = 0; st3 < kSteps; ++st3)
                for (int kk = 0; kk < 2; ++kk)
                    s += (double)ha[st3 * 64 + i + 32 * kk] * (double)hb[st3 * 64 + j + 32 * kk];
            if (!(std::fabs((double)D(i, j) - s) <= g6 * s)) { within = false; break; }
        }
    if (within) rep |= 4u;
    *report = rep;
    return TAO_OK;
}

}  // extern "C"
