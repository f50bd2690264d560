// Uni-greedy schedules (Lowery & Langou, Algorithm 1, Section 5) on gfx950.
//
// One 64-lane wavefront runs one configuration.  Algorithm 1 pairs, p-1 times
// per segment, the two processors with the smallest ready times (x, index) at
// t = the larger of the two; the sender leaves with t + tcomm, the receiver
// stays with (t + tcomm) + tcomp.  Within a segment t never decreases, so the
// values that leave (S) and the values that stay (B) are produced in
// non-decreasing order: with the segment's initial states sorted (A), the
// remaining set is at all times the unread tail of A merged with the unread
// tail of B.  The kernel therefore never searches for a minimum.  It takes a
// whole batch of pairs per step: if e2 is the second smallest remaining
// element, nothing produced from now on is smaller than
// bound = (e2 + tcomm) + tcomp, so all remaining elements below bound pair up
// in merged order (1st with 2nd, 3rd with 4th, ...) exactly as the sequential
// rule would pair them.  Lanes rank the batch elements by binary search in the
// other queue and write the results of all pairs of the batch at once.
//
// Ties in fp64 between values produced at different t (equal after rounding)
// can leave equal-valued neighbours of B or S out of index order; this is
// detected after every batch and repaired by one lane.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

template <typename T, bool kSched> struct UniState {
    T *Ax, *Sx, *Bx, *Mx;
    int32_t *Aid, *Sid, *Bid, *Mid;
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

size_t uni_state_bytes(bool sched, int32_t p_max)
{
    const size_t tb = align_up(static_cast<size_t>(p_max) * 8, 256), ib = align_up(static_cast<size_t>(p_max) * 4, 256);
    return sched ? 4 * tb + 4 * ib : 3 * tb;
}

template <typename T, bool kSched>
__device__ __forceinline__ UniState<T, kSched> carve_uni(char *slot, int32_t p_max)
{
    const size_t tb = align_up(static_cast<size_t>(p_max) * 8, 256), ib = align_up(static_cast<size_t>(p_max) * 4, 256);
    UniState<T, kSched> s;
    s.Ax = reinterpret_cast<T *>(slot);
    s.Sx = reinterpret_cast<T *>(slot + tb);
    s.Bx = reinterpret_cast<T *>(slot + 2 * tb);
    s.Mx = nullptr; s.Aid = s.Sid = s.Bid = s.Mid = nullptr;
    if (kSched) {
        s.Mx = reinterpret_cast<T *>(slot + 3 * tb);
        char *q = slot + 4 * tb;
        s.Aid = reinterpret_cast<int32_t *>(q);
        s.Sid = reinterpret_cast<int32_t *>(q + ib);
        s.Bid = reinterpret_cast<int32_t *>(q + 2 * ib);
        s.Mid = reinterpret_cast<int32_t *>(q + 3 * ib);
    }
    return s;
}

// (x, id) order when identities are tracked; plain value order otherwise.
template <typename T, bool kSched>
__device__ __forceinline__ bool key_less(T xa, int32_t ia, T xb, int32_t ib)
{
    if (kSched) return xa < xb || (xa == xb && ia < ib);
    return xa < xb;
}

// Number of leading elements of the sorted range X[lo, hi) that are < bound.
// All 64 lanes take part (64-ary search, uniform arguments and result).
template <typename T> __device__ __forceinline__ int count_less(const T *X, int lo, int hi, T bound)
{
    const int lane = lane_id(), base = lo;
    while (hi > lo) {
        const int len = hi - lo, step = (len + kWave - 1) / kWave;
        const int start = lo + lane * step;
        const int end = start + step < hi ? start + step : hi;
        const bool pred = start < hi && X[end - 1] < bound;
        const int nfull = __popcll(ballot64(pred));
        int lo2 = lo + nfull * step;
        if (lo2 > hi) lo2 = hi;
        if (step == 1) { lo = lo2; break; }
        hi = lo2 + step < hi ? lo2 + step : hi;
        lo = lo2;
    }
    return lo - base;
}

// One lane sorts X/I[lo, hi) by (value, index); only entries with equal values are ever out of place.
template <typename T> __device__ void insertion_sort(T *X, int32_t *I, int lo, int hi)
{
    for (int i = lo + 1; i < hi; ++i) {
        const T x = X[i];
        const int32_t id = I[i];
        int j = i;
        while (j > lo && key_less<T, true>(x, id, X[j - 1], I[j - 1])) { X[j] = X[j - 1]; I[j] = I[j - 1]; --j; }
        X[j] = x; I[j] = id;
    }
}

template <typename T, bool kSched> struct UniOut {
    int32_t *src, *dst, *seg;
    T *tstart;
    int64_t base;
};

// Runs all segments of one configuration; returns the root's final time.
template <typename T, bool kSched>
__device__ T run_uni(const Config<T> &c, UniState<T, kSched> st, const UniOut<T, kSched> &out, int32_t *status)
{
    const int lane = lane_id();
    const int p = c.p;
    for (int i = lane; i < p; i += kWave) {
        st.Ax[i] = 0;
        if (kSched) st.Aid[i] = i;
    }
    __syncthreads();
    T root_time = 0;
    for (int k = 0; k < c.q; ++k) {
        const T cc = c.c(k), gg = c.g(k);
        int ia = 0, ib = 0, jb = 0, ns = 0;
        const int na = p;
        int guard = 0;
        while (ns < p - 1) {
            if (++guard > p + 8) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
            // ---- the two smallest remaining elements (heads of A and B)
            const bool hasA0 = ia < na, hasA1 = ia + 1 < na, hasB0 = ib < jb, hasB1 = ib + 1 < jb;
            const T a0x = hasA0 ? st.Ax[ia] : 0, a1x = hasA1 ? st.Ax[ia + 1] : 0;
            const T b0x = hasB0 ? st.Bx[ib] : 0, b1x = hasB1 ? st.Bx[ib + 1] : 0;
            int32_t a0i = 0, a1i = 0, b0i = 0, b1i = 0;
            if (kSched) {
                a0i = hasA0 ? st.Aid[ia] : 0; a1i = hasA1 ? st.Aid[ia + 1] : 0;
                b0i = hasB0 ? st.Bid[ib] : 0; b1i = hasB1 ? st.Bid[ib + 1] : 0;
            }
            int dA, dB;
            T e2x;
            const bool firstA = hasA0 && (!hasB0 || !key_less<T, kSched>(b0x, b0i, a0x, a0i));
            if (firstA) {
                const bool secondA = hasA1 && (!hasB0 || !key_less<T, kSched>(b0x, b0i, a1x, a1i));
                if (secondA) { dA = 2; dB = 0; e2x = a1x; } else { dA = 1; dB = 1; e2x = b0x; }
            } else {
                const bool secondA = hasA0 && (!hasB1 || !key_less<T, kSched>(b1x, b1i, a0x, a0i));
                if (secondA) { dA = 1; dB = 1; e2x = a0x; } else { dA = 0; dB = 2; e2x = b1x; }
            }
            const T bound = (e2x + cc) + gg;
            // ---- batch = every remaining element below bound (at least the first pair)
            int cntA = count_less(st.Ax, ia, na, bound);
            int cntB = count_less(st.Bx, ib, jb, bound);
            if (cntA + cntB < 2) {
                cntA = dA; cntB = dB;
            } else if ((cntA + cntB) & 1) {        // odd: the largest element waits for the next batch
                bool dropA;
                if (cntA == 0) dropA = false;
                else if (cntB == 0) dropA = true;
                else {
                    const int la = ia + cntA - 1, lb = ib + cntB - 1;
                    dropA = key_less<T, kSched>(st.Bx[lb], kSched ? st.Bid[lb] : 0, st.Ax[la], kSched ? st.Aid[la] : 0);
                }
                if (dropA) --cntA; else --cntB;
            }
            const int npairs = (cntA + cntB) >> 1;
            // ---- merged rank of every batch element; odd ranks close a pair
            for (int a = lane; a < cntA; a += kWave) {
                const T x = st.Ax[ia + a];
                const int32_t id = kSched ? st.Aid[ia + a] : 0;
                int lb = 0, len = cntB;              // elements of B's part that come before (x, id)
                while (len > 0) {
                    const int half = len >> 1, pos = ib + lb + half;
                    if (key_less<T, kSched>(st.Bx[pos], kSched ? st.Bid[pos] : 0, x, id)) { lb += half + 1; len -= half + 1; }
                    else len = half;
                }
                const int r = a + lb;
                if (kSched) { st.Mx[r] = x; st.Mid[r] = id; }
                else if (r & 1) {
                    const T tc = x + cc;
                    st.Sx[ns + (r >> 1)] = tc;
                    st.Bx[jb + (r >> 1)] = tc + gg;
                }
            }
            for (int b = lane; b < cntB; b += kWave) {
                const T x = st.Bx[ib + b];
                const int32_t id = kSched ? st.Bid[ib + b] : 0;
                int lb = 0, len = cntA;              // elements of A's part that come before (x, id); ties: A first
                while (len > 0) {
                    const int half = len >> 1, pos = ia + lb + half;
                    const bool before = kSched ? key_less<T, true>(st.Ax[pos], st.Aid[pos], x, id) : !(x < st.Ax[pos]);
                    if (before) { lb += half + 1; len -= half + 1; }
                    else len = half;
                }
                const int r = b + lb;
                if (kSched) { st.Mx[r] = x; st.Mid[r] = id; }
                else if (r & 1) {
                    const T tc = x + cc;
                    st.Sx[ns + (r >> 1)] = tc;
                    st.Bx[jb + (r >> 1)] = tc + gg;
                }
            }
            __syncthreads();
            if (kSched) {
                for (int kp = lane; kp < npairs; kp += kWave) {
                    const T t = st.Mx[2 * kp + 1];
                    const int32_t g1 = st.Mid[2 * kp], g2 = st.Mid[2 * kp + 1];
                    int32_t s = g1, d = g2;
                    if (g1 == 0) { s = g2; d = 0; }           // the root never sends (Lemma 1 (ii))
                    const T tc = t + cc;
                    // Senders of one run of equal t leave with the same value and must enter S in index
                    // order.  Inside a run they already are, except that the run's first pair may be
                    // led by a processor left over from an earlier, smaller value: rank that one sender
                    // among the others and shift those with smaller index down by one.
                    int rs = 0;
                    for (int len = kp; len > 0;) {             // first pair of this run
                        const int half = len >> 1;
                        if (st.Mx[2 * (rs + half) + 1] < t) { rs += half + 1; len -= half + 1; } else len = half;
                    }
                    int pos = kp;
                    const int32_t f = st.Mid[2 * rs];
                    if (st.Mx[2 * rs] < t && f != 0) {
                        if (kp == rs) {
                            int cnt = 0;
                            for (int len = npairs - rs - 1; len > 0;) {
                                const int half = len >> 1, j = rs + 1 + cnt + half;
                                if (!(t < st.Mx[2 * j + 1]) && st.Mid[2 * j] < f) { cnt += half + 1; len -= half + 1; } else len = half;
                            }
                            pos = rs + cnt;
                        } else if (s < f) {
                            pos = kp - 1;
                        }
                    }
                    st.Sx[ns + pos] = tc; st.Sid[ns + pos] = s;
                    st.Bx[jb + kp] = tc + gg; st.Bid[jb + kp] = d;
                    const int64_t o = out.base + static_cast<int64_t>(k) * (p - 1) + ns + kp;
                    if (out.src) out.src[o] = s;
                    if (out.dst) out.dst[o] = d;
                    if (out.seg) out.seg[o] = k;
                    if (out.tstart) out.tstart[o] = t;
                }
                __syncthreads();
                // values produced at different t that round to the same double can still arrive out of
                // index order: detect (B now, S at the end of the segment) and let one lane repair
                bool bad = false;
                const int live_b = ib + cntB;
                for (int kp = lane; kp < npairs; kp += kWave) {
                    const int bi = jb + kp;
                    if (bi > live_b && key_less<T, true>(st.Bx[bi], st.Bid[bi], st.Bx[bi - 1], st.Bid[bi - 1])) bad = true;
                }
                if (ballot64(bad) != 0) {
                    if (lane == 0) insertion_sort<T>(st.Bx, st.Bid, live_b, jb + npairs);
                    __syncthreads();
                }
            }
            ia += cntA; ib += cntB; ns += npairs; jb += npairs;
        }
        // ---- end of segment: the one element left is the root, last of B; the states of all p
        // processors (S plus the root) become the next segment's sorted A.
        root_time = st.Bx[jb - 1];
        if (!kSched) {
            if (lane == 0) st.Sx[p - 1] = root_time;     // the root holds the maximum
        } else {
            bool bad = false;
            for (int i = lane + 1; i < p - 1; i += kWave)
                if (key_less<T, true>(st.Sx[i], st.Sid[i], st.Sx[i - 1], st.Sid[i - 1])) bad = true;
            if (ballot64(bad) != 0) {
                if (lane == 0) insertion_sort<T>(st.Sx, st.Sid, 0, p - 1);
                __syncthreads();
            }
            // key (root_time, 0) goes before every equal value: shift that tail up by one
            const int pos = count_less(st.Sx, 0, p - 1, root_time);
            const int tail = (p - 1) - pos;
            for (int i = lane; i < tail; i += kWave) { st.Mx[i] = st.Sx[pos + i]; st.Mid[i] = st.Sid[pos + i]; }
            __syncthreads();
            for (int i = lane; i < tail; i += kWave) { st.Sx[pos + 1 + i] = st.Mx[i]; st.Sid[pos + 1 + i] = st.Mid[i]; }
            if (lane == 0) { st.Sx[pos] = root_time; st.Sid[pos] = 0; }
        }
        __syncthreads();
        { T *tx = st.Ax; st.Ax = st.Sx; st.Sx = tx; }
        if (kSched) { int32_t *ti = st.Aid; st.Aid = st.Sid; st.Sid = ti; }
    }
    return root_time;
}

template <typename T, bool kSched, bool kLds>
__global__ __launch_bounds__(kWave) void uni_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model, TimesOut times,
                                                    SchedOut sched, PlanHeader *plan, const int32_t *order, int cls,
                                                    int32_t state_p, char *slots, size_t slot_bytes)
{
    PRS_DYNAMIC_LDS(lds_raw);
    const int lane = lane_id();
    // all per-configuration state in LDS (classes with p <= state_p) or in this block's workspace slot
    char *base = kLds ? lds_raw : slots + static_cast<size_t>(blockIdx.x) * slot_bytes;
    UniState<T, kSched> st = carve_uni<T, kSched>(base, state_p);
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    for (;;) {
        const int64_t ticket = next_ticket(&plan->ticket[cls]);
        if (ticket >= count) break;
        const int64_t i = order[begin + ticket];
        Config<T> c = decode_config<T>(cfg, i, p_max, q_max);
        int32_t status = c.status;
        UniOut<T, kSched> out{sched.src, sched.dst, sched.seg, static_cast<T *>(sched.tstart), 0};
        if (kSched && status == PRS_CFG_OK) {
            out.base = sched.pair_offset[i];
            const int64_t cnt = static_cast<int64_t>(c.p - 1) * c.q;
            if (out.base < 0 || out.base + cnt > sched.pair_capacity) status = PRS_CFG_TOO_LARGE;
        }
        T result = CostTraits<T>::bad();
        if (status == PRS_CFG_OK) result = run_uni<T, kSched>(c, st, out, &status);
        if (lane == 0) {                  // the only lane-dependent branch of the loop body
            if (!kSched) write_closed_forms<T>(times, i, c, model);
            T *tg = static_cast<T *>(kSched ? sched.T_greedy : times.greedy);
            int32_t *cs = kSched ? sched.cfg_status : times.cfg_status;
            if (tg) tg[i] = status == PRS_CFG_OK ? result : CostTraits<T>::bad();
            if (cs) cs[i] = status;
        }
        __syncthreads();                  // the next configuration reuses the state arrays
    }
}

template <typename T, bool kSched>
static hipError_t launch_uni_t(const UniLaunch &L)
{
    if (L.lds_p > 0)
        hipLaunchKernelGGL((uni_kernel<T, kSched, true>), dim3(L.grid), dim3(kWave), L.lds_bytes, L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.sched, L.plan, L.order, L.cls, L.lds_p, L.slots, L.slot_bytes);
    else
        hipLaunchKernelGGL((uni_kernel<T, kSched, false>), dim3(L.grid), dim3(kWave), 0, L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.sched, L.plan, L.order, L.cls, L.slot_p, L.slots, L.slot_bytes);
    return hipGetLastError();
}

hipError_t launch_uni(const UniLaunch &L)
{
    if (L.cost == PRS_COST_I64) return L.want_schedule ? launch_uni_t<int64_t, true>(L) : launch_uni_t<int64_t, false>(L);
    return L.want_schedule ? launch_uni_t<double, true>(L) : launch_uni_t<double, false>(L);
}

}  // namespace prs
