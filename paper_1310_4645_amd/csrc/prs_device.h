// Device-side helpers shared by the gfx950 kernels: cost model, configuration
// decoding and validation, wavefront (64-lane) primitives.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/prs.h"

namespace prs {

constexpr int kWave = 64;

// The dynamically sized LDS allocation of a kernel (one per kernel body).
#ifndef PRS_DYNAMIC_LDS
#define PRS_DYNAMIC_LDS(name) extern __shared__ __align__(256) char name[]
#endif

// ---------------------------------------------------------------- cost types
template <typename T> struct CostTraits;
template <> struct CostTraits<int64_t> {
    static __device__ __forceinline__ int64_t inf() { return INT64_MAX; }
    static __device__ __forceinline__ int64_t bad() { return -1; }
    static __device__ __forceinline__ bool valid(int64_t v) { return v >= 0 && v < (INT64_C(1) << 62); }
    static __device__ __forceinline__ bool fits(double total) { return total < 4.0e18; }       // below 2^62
};
template <> struct CostTraits<double> {
    static __device__ __forceinline__ double inf() { return __builtin_huge_val(); }
    static __device__ __forceinline__ double bad() { return __builtin_nan(""); }
    static __device__ __forceinline__ bool valid(double v) { return v >= 0.0 && v < __builtin_huge_val(); }
    static __device__ __forceinline__ bool fits(double total) { return total < 1.0e300; }
};

// No time of a greedy schedule passes the pipeline's (p-1 + 2(q-1)) rounds of the longest segment (Table I; Theorem 1
// puts uni-greedy below every algorithm that takes the segments in order, and a round of the longest segment covers
// any segment).  A configuration whose bound does not fit the cost type is refused: past it sums would overflow, and
// the largest representable value doubles as "no entry" in the kernels.
template <typename T>
__device__ __forceinline__ bool schedule_fits(int32_t p, int64_t q, T alpha, T beta, T gamma, int64_t sz)
{
    const double round = (static_cast<double>(alpha) + static_cast<double>(beta) * static_cast<double>(sz)) +
                         static_cast<double>(gamma) * static_cast<double>(sz);
    const double rounds = static_cast<double>(p - 1) + 2.0 * static_cast<double>(q - 1);
    return CostTraits<T>::fits(rounds * round);
}

// One configuration after decoding (Section 2: equi-segmentation; Section 5:
// tcomm and tcomp of a segment).  Only two distinct segment sizes occur.
template <typename T> struct Config {
    int32_t p, q;          // processors, segments actually used
    int64_t m, sz, sz_last;
    T alpha, beta, gamma;
    T c_full, g_full, c_last, g_last;
    uint32_t comp;         // composition mode: cut bits of the segmentation with a closing bit at position m-1 (else 0)
    int32_t status;
    __device__ __forceinline__ T c(int j) const { return j == q - 1 ? c_last : c_full; }
    __device__ __forceinline__ T g(int j) const { return j == q - 1 ? g_last : g_full; }
};

// comp_m = 0: configuration i is entry i of the arrays, cut into equal segments from q_req.
// comp_m = M > 0 (Section 8, every segmentation of a short message): configuration i is problem i >> (M-1) of the
// arrays cut by the bit pattern i & (2^(M-1) - 1): bit b set = a segment ends after unit b+1 of the problem's m units
// (m <= M; patterns with bits at or above m-1 are no segmentation of that problem and are marked PRS_CFG_BAD_PARAM).
// Only the uni-greedy completion-time kernel reads compositions.
struct ConfigArrays {
    const int32_t *p, *q_req;
    const int64_t *m;
    const void *alpha, *beta, *gamma;
    int32_t comp_m = 0;
};

// Size of the first segment of a composition (cut bits closed by the bit after the last unit) and the rest of it.
__device__ __forceinline__ int comp_first(uint32_t comp) { return __builtin_ctz(comp) + 1; }
__device__ __forceinline__ uint32_t comp_drop(uint32_t comp, int segments)
{
    for (int s = 0; s < segments && comp != 0; ++s) comp >>= comp_first(comp);
    return comp;
}

template <typename T>
__device__ __forceinline__ Config<T> decode_values(int32_t p, int32_t q_req, int64_t m, T alpha, T beta, T gamma, int32_t p_max,
                                                   int32_t q_max);

template <typename T>
__device__ __forceinline__ Config<T> decode_config(const ConfigArrays &a, int64_t i, int32_t p_max, int32_t q_max)
{
    Config<T> c;
    c.comp = 0;
    if (a.comp_m > 0) {
        const int bits = a.comp_m - 1;
        const uint32_t cuts = static_cast<uint32_t>(i & ((INT64_C(1) << bits) - 1));
        i >>= bits;
        c.p = a.p[i];
        c.m = a.m[i];
        c.alpha = static_cast<const T *>(a.alpha)[i];
        c.beta = static_cast<const T *>(a.beta)[i];
        c.gamma = static_cast<const T *>(a.gamma)[i];
        c.status = PRS_CFG_OK;
        c.q = 1; c.sz = 1; c.sz_last = 1;
        c.c_full = c.g_full = c.c_last = c.g_last = 0;
        if (c.p < 2 || c.m < 1 || c.m > a.comp_m || (cuts >> static_cast<int>(c.m - 1)) != 0 || !CostTraits<T>::valid(c.alpha) ||
            !CostTraits<T>::valid(c.beta) || !CostTraits<T>::valid(c.gamma)) {
            c.status = PRS_CFG_BAD_PARAM;
            return c;
        }
        if (c.p > p_max || a.comp_m > q_max) { c.status = PRS_CFG_TOO_LARGE; return c; }
        c.q = __builtin_popcount(cuts) + 1;
        c.comp = cuts | (1u << static_cast<int>(c.m - 1));
        // the smallest and the largest cost a segment of this problem can have (sizes 1 and m)
        const T c1 = c.alpha + c.beta, cm = c.alpha + c.beta * static_cast<T>(c.m), gm = c.gamma * static_cast<T>(c.m);
        if (!(c1 > 0) || !(cm > 0) || !CostTraits<T>::valid(cm) || !CostTraits<T>::valid(gm)) c.status = PRS_CFG_BAD_PARAM;
        if (!schedule_fits<T>(c.p, c.q, c.alpha, c.beta, c.gamma, c.m)) c.status = PRS_CFG_BAD_PARAM;
        return c;
    }
    return decode_values<T>(a.p[i], a.q_req[i], a.m[i], static_cast<const T *>(a.alpha)[i], static_cast<const T *>(a.beta)[i],
                            static_cast<const T *>(a.gamma)[i], p_max, q_max);
}

// One configuration given by value: equi-segmentation from a segment count (Section 2) and the costs of a full and of
// the last segment (Section 5).
template <typename T>
__device__ __forceinline__ Config<T> decode_values(int32_t p, int32_t q_req, int64_t m, T alpha, T beta, T gamma, int32_t p_max,
                                                   int32_t q_max)
{
    Config<T> c;
    c.comp = 0;
    c.p = p;
    c.m = m;
    c.alpha = alpha;
    c.beta = beta;
    c.gamma = gamma;
    c.status = PRS_CFG_OK;
    c.q = 1; c.sz = 1; c.sz_last = 1;
    c.c_full = c.g_full = c.c_last = c.g_last = 0;
    if (c.p < 2 || q_req < 1 || c.m < 1 || c.m >= (INT64_C(1) << 62) || !CostTraits<T>::valid(c.alpha) ||
        !CostTraits<T>::valid(c.beta) || !CostTraits<T>::valid(c.gamma)) {
        c.status = PRS_CFG_BAD_PARAM;
        return c;
    }
    if (c.p > p_max || q_req > q_max) { c.status = PRS_CFG_TOO_LARGE; return c; }
    c.sz = (c.m + q_req - 1) / q_req;
    const int64_t q = (c.m + c.sz - 1) / c.sz;
    c.q = static_cast<int32_t>(q);
    c.sz_last = c.m - (q - 1) * c.sz;
    // products and sums are separate roundings (the library is built without FMA contraction)
    const T bs = c.beta * static_cast<T>(c.sz);
    c.c_full = c.alpha + bs;
    c.g_full = c.gamma * static_cast<T>(c.sz);
    const T bl = c.beta * static_cast<T>(c.sz_last);
    c.c_last = c.alpha + bl;
    c.g_last = c.gamma * static_cast<T>(c.sz_last);
    if (!(c.c_full > 0) || !(c.c_last > 0) || !CostTraits<T>::valid(c.c_full) || !CostTraits<T>::valid(c.g_full))
        c.status = PRS_CFG_BAD_PARAM;
    if (!schedule_fits<T>(c.p, q, c.alpha, c.beta, c.gamma, c.sz)) c.status = PRS_CFG_BAD_PARAM;
    return c;
}

__device__ __forceinline__ int32_t ceil_log2(int64_t v)
{
    return v <= 1 ? 0 : 64 - __builtin_clzll(static_cast<unsigned long long>(v - 1));
}

// sum that may take stale operands (whose result is then discarded) without signed overflow
template <typename T> __device__ __forceinline__ T wrap_add(T a, T b);
template <> __device__ __forceinline__ int64_t wrap_add<int64_t>(int64_t a, int64_t b)
{
    return static_cast<int64_t>(static_cast<uint64_t>(a) + static_cast<uint64_t>(b));
}
template <> __device__ __forceinline__ double wrap_add<double>(double a, double b) { return a + b; }

// keeps a branch a branch (its body is then not run speculatively on the other path)
#ifndef PRS_KEEP_BRANCH
#define PRS_KEEP_BRANCH() asm volatile("" ::: "memory")
#endif

// Writes base + b for every set bit b of w, in rising order, to out[0], out[1], ...; returns how many.  Four at a
// time while four are left: a 16-byte store costs the memory pipeline what a 4-byte store does.
__device__ __forceinline__ int emit_set_bits(int32_t *out, uint32_t w, int base)
{
    int n = 0;
    while (__builtin_popcount(w) >= 4) {
        int32_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { v[i] = base + __builtin_ctz(w); w &= w - 1; }
        __builtin_memcpy(out + n, v, sizeof(v));
        n += 4;
    }
    while (w) { out[n++] = base + __builtin_ctz(w); w &= w - 1; }
    return n;
}

// ---------------------------------------------------------------- wavefront primitives
__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & (kWave - 1); }

__device__ __forceinline__ uint64_t ballot64(bool pred) { return __ballot(pred ? 1 : 0); }

// number of set bits of `mask` below this lane
__device__ __forceinline__ int rank_below(uint64_t mask)
{
    return static_cast<int>(__builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                                      __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u)));
}

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    const int lane = lane_id();
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int u = __shfl_up(v, o, kWave);
        if (lane >= o) v += u;
    }
    return v;
}

template <typename T> __device__ __forceinline__ T wave_min(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const T u = __shfl_xor(v, o, kWave);
        v = u < v ? u : v;
    }
    return v;
}

// Next index of a work counter, the same value in all 64 lanes.  Every lane issues the atomic (lane 0
// adds one, the others zero) and the result is broadcast with a cross-lane read: no lane-dependent
// branch, so no lane can run ahead of the others into the next loop iteration.
__device__ __forceinline__ int64_t next_ticket(unsigned long long *counter)
{
    const unsigned long long got = atomicAdd(counter, lane_id() == 0 ? 1ULL : 0ULL);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(got));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(got >> 32));
    return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
}

// keep the k lowest set bits of mask (k <= 0: none, k >= popcount: all)
__device__ __forceinline__ uint64_t lowest_bits(uint64_t mask, int k)
{
    // all of them or none: the usual case for all but one word of a set, and a wavefront of such words skips the search
    const uint32_t lo = static_cast<uint32_t>(mask), hi = static_cast<uint32_t>(mask >> 32);
    const int plo = __builtin_popcount(lo), phi = __builtin_popcount(hi);
    if (k <= 0) return 0;
    if (k >= plo + phi) return mask;
    // on the 32-bit half that holds the k-th set bit
    const bool in_lo = k <= plo;
    const uint32_t w = in_lo ? lo : hi;
    int kk = in_lo ? k : k - plo;
    uint32_t pos = 0;                  // after the loop: index of the kk-th set bit of w
#pragma unroll
    for (uint32_t width = 16; width > 0; width >>= 1) {
        const int cnt = __builtin_popcount((w >> pos) & ((1u << width) - 1));
        const bool up = cnt < kk;
        pos += up ? width : 0;
        kk -= up ? cnt : 0;
    }
    const uint32_t part = w & ((2u << pos) - 1);
    const uint64_t some = in_lo ? static_cast<uint64_t>(part) : (static_cast<uint64_t>(part) << 32) | lo;
    return some;
}

__device__ __forceinline__ uint64_t highest_bits(uint64_t mask, int k)
{
    if (k <= 0) return 0;
    const int pc = __popcll(mask);
    if (k >= pc) return mask;
    return mask & ~lowest_bits(mask, pc - k);
}

// ---------------------------------------------------------------- closed forms
// Tables I and III (standard algorithms), Table II / Figure 6 (bounds).
struct TimesOut {
    void *greedy, *binomial, *pipeline, *binary, *revopt;
    double *butterfly, *lower_bound;
    int32_t *q_eff, *cfg_status;
};

// Table III: reversed optimal broadcast (the time bi-greedy meets), (ceil(log2 p) + q - 1) rounds of a full segment
template <typename T> __device__ __forceinline__ T revopt_time(const Config<T> &c)
{
    const T r = (c.alpha + c.beta * static_cast<T>(c.sz)) + c.gamma * static_cast<T>(c.sz);
    return static_cast<T>(static_cast<int64_t>(ceil_log2(c.p)) + c.q - 1) * r;
}

// Table III: butterfly (reduce-scatter by recursive halving, gather by recursive doubling)
template <typename T> __device__ __forceinline__ double butterfly_time(const Config<T> &c)
{
    const double Ld = static_cast<double>(ceil_log2(c.p)), fr = static_cast<double>(c.p - 1) / static_cast<double>(c.p);
    const double md = static_cast<double>(c.m), al = static_cast<double>(c.alpha), be = static_cast<double>(c.beta),
                 ga = static_cast<double>(c.gamma);
    return ((2.0 * Ld) * al + (2.0 * fr) * (be * md)) + fr * (ga * md);
}

template <typename T>
__device__ __forceinline__ void write_closed_forms(const TimesOut &o, int64_t i, const Config<T> &c, int model)
{
    if (c.status != PRS_CFG_OK) {
        const T bad = CostTraits<T>::bad();
        if (o.binomial) static_cast<T *>(o.binomial)[i] = bad;
        if (o.pipeline) static_cast<T *>(o.pipeline)[i] = bad;
        if (o.binary) static_cast<T *>(o.binary)[i] = bad;
        if (o.revopt) static_cast<T *>(o.revopt)[i] = bad;
        if (o.butterfly) o.butterfly[i] = __builtin_nan("");
        if (o.lower_bound) o.lower_bound[i] = __builtin_nan("");
        if (o.q_eff) o.q_eff[i] = -1;
        return;
    }
    const int32_t L = ceil_log2(c.p), N = ceil_log2(static_cast<int64_t>(c.p) + 1);
    const int64_t p = c.p, q = c.q;
    const T r = (c.alpha + c.beta * static_cast<T>(c.sz)) + c.gamma * static_cast<T>(c.sz);
    const T whole = (c.alpha + c.beta * static_cast<T>(c.m)) + c.gamma * static_cast<T>(c.m);
    if (o.binomial) static_cast<T *>(o.binomial)[i] = static_cast<T>(L) * whole;
    if (o.pipeline)
        static_cast<T *>(o.pipeline)[i] = static_cast<T>(model == PRS_UNI ? (p - 1) + 2 * (q - 1) : p + q - 2) * r;
    if (o.binary)
        static_cast<T *>(o.binary)[i] =
            static_cast<T>(model == PRS_UNI ? 2 * static_cast<int64_t>(N - 1) + 4 * (q - 1) : 2 * (N + q - 2)) * r;
    if (o.revopt) static_cast<T *>(o.revopt)[i] = revopt_time<T>(c);
    const double Ld = static_cast<double>(L), fr = static_cast<double>(c.p - 1) / static_cast<double>(c.p);
    const double md = static_cast<double>(c.m), al = static_cast<double>(c.alpha), be = static_cast<double>(c.beta),
                 ga = static_cast<double>(c.gamma);
    if (o.butterfly) o.butterfly[i] = butterfly_time<T>(c);
    if (o.lower_bound) {
        const double bw = (model == PRS_UNI && c.p > 2) ? 2.0 * (md * be) : md * be;
        o.lower_bound[i] = (Ld * al + bw) + fr * (md * ga);
    }
    if (o.q_eff) o.q_eff[i] = c.q;
}

}  // namespace prs
