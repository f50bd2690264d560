// Uni-greedy completion times (Lowery & Langou, Algorithm 1, Section 5) on gfx950: segments pipelined
// through the lanes of a wavefront.
//
// Algorithm 1 handles segment k+1 with the final states of segment k as its initial states, but it only
// ever looks at the smallest of them.  The states of segment k leave in non-decreasing order (the start
// time t of its pairs never decreases), so segment k+1 can begin as soon as segment k has produced its
// first values and then follows right behind it.  A configuration is given a group of G lanes
// (G = 1, 4, 16 or 32, chosen from its number of pairs); lane l of the group runs segments l, l+G, l+2G, ...
// and reads the stream written by the lane before it (lane 0 reads the stream the last lane wrote one
// round earlier).  Per iteration every lane whose two smallest remaining values are known performs one
// pair of its segment:
//   remaining values of a segment = unread tail of its input stream A (sorted) merged with the unread
//   tail of B, the values (t + tcomm) + tcomp of its own earlier pairs (sorted as well);
//   the pair takes the two smallest, t = the larger of them; t + tcomm goes to the output stream.
// B is not stored: B[i] = stream[i] + tcomp with the same rounding as (t + tcomm) + tcomp.  The root's
// final state (the largest value of the segment) closes the stream of the segment, so every stream has p
// entries.  A value not yet produced by the previous segment is at least as large as the last one
// produced, so a pair is safe as soon as its larger element does not exceed that value.
//
// How far a segment trails the one before it is the number of its receivers that are still combining
// (the length of B), about p/25 in steady state and up to p/2 in the first segments.  A group much larger
// than p divided by that lag would leave its first lane waiting for the last one at every round, which is
// why light configurations get small groups (and a wavefront then works on several of them).
//
// Streams live in the wavefront's workspace slot (two buffers of p entries per lane, alternating between
// rounds); the last kRing entries of every stream are also kept in LDS, which serves the reads of a
// segment that follows closely.  Entries further back (the first lane of a group reading the last one's
// stream, a long B) are loaded from the workspace one iteration ahead of their use.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kRing = 64;          // stream entries per lane kept in LDS
constexpr int kNear = kRing - 5;   // entries this close behind the writer are read from LDS in the next iteration

// The ring takes 32 KB; asking for 40 KB keeps it to four wavefronts per CU, one per SIMD: a fifth would share a SIMD,
// and the configurations that land on the two sharing wavefronts run at half speed (measured: 11.8 against 12.0 ms).
size_t uni_times_lds_bytes() { return static_cast<size_t>(kRing) * kWave * 8 + 8192; }
size_t uni_times_slot_bytes(int32_t p_cap) { return static_cast<size_t>(kWave) * 2 * static_cast<size_t>(p_cap) * 8; }

// kComp: the segments of a configuration have the sizes its composition gives (Section 8) instead of one size
// and a smaller last one; every lane keeps the part of the composition that starts at its segment.
template <typename T, int G, bool kComp>
__device__ __forceinline__ void uni_times_body(T *ring, const ConfigArrays &cfg, int32_t p_max, int32_t q_max, int model,
                                               const TimesOut &times, PlanHeader *plan, const int32_t *order, int cls, int part,
                                               T *slot, int32_t slot_p)
{
    constexpr int M = kRing - 1;
    const int lane = lane_id(), gl = lane & (G - 1), gbase = lane & ~(G - 1);
    const int prod = gbase | ((gl + G - 1) & (G - 1));
    const uint64_t gmask = (G == 64 ? ~UINT64_C(0) : ((UINT64_C(1) << G) - 1)) << gbase;
    T *mybuf = slot + static_cast<size_t>(lane) * 2 * slot_p;       // [2][slot_p]
    const T *prodbuf = slot + static_cast<size_t>(prod) * 2 * slot_p;
    // part of the class this pass works on: all of it, its giant configurations only, or the rest after those
    int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    unsigned long long *tickets = &plan->ticket[cls];
    if (part == kGiantPart) { count = plan->giant_count; tickets = &plan->ticket_giant; }
    else if (part == kRestPart) { begin += plan->giant_count; count -= plan->giant_count; }
    const T kInf = CostTraits<T>::inf();

    // ---- per-group state (the same in all lanes of a group)
    bool have = false, exhausted = false;
    int64_t ci = 0;
    int p = 2, q = 1;
    T c_full = 0, g_full = 0, c_last = 0, g_last = 0;
    T alpha = 0, beta = 0, gamma = 0;   // kComp only
    uint32_t rest = 0;                  // kComp only: the composition from my segment on (per lane)
    // ---- per-lane state.  Positions count the entries of a stream from the start of the configuration:
    // every finished segment adds p of them.
    int k = 0;                      // segment this lane is running (>= q: none left)
    int par = 0, apar = 0;          // which of the two buffers my segment writes / my input stream is in
    int wtot = 0, segBase = 0;      // entries I have written; the same at the start of my segment
    int apos = 0, astart = 0;       // next entry of my input stream; its first entry
    int bpos = 0;                   // next entry of my own stream whose B value is unread
    T lastS = 0, cc = 0, gg = 0;
    bool farA = false, farB = false, anyFar = false;
    T la0 = 0, la1 = 0, lb0 = 0, lb1 = 0;   // entries loaded from the workspace in the previous iteration

    for (;;) {
        // ---------------------------------------------------------------- fetch a configuration
        if (!have && !exhausted) {
            unsigned long long got = atomicAdd(tickets, gl == 0 ? 1ULL : 0ULL);
            int64_t ticket = static_cast<int64_t>(got);
            if (G > 1) {
                const uint32_t lo = __shfl(static_cast<uint32_t>(got), 0, G), hi = __shfl(static_cast<uint32_t>(got >> 32), 0, G);
                ticket = static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
            }
            if (ticket >= count) {
                exhausted = true;
            } else {
                ci = order[begin + ticket];
                const Config<T> c = decode_config<T>(cfg, ci, p_max, q_max);
                if (gl == 0) {
                    if (!kComp) write_closed_forms<T>(times, ci, c, model);
                    if (times.cfg_status) times.cfg_status[ci] = c.status;
                    if (c.status != PRS_CFG_OK && times.greedy) static_cast<T *>(times.greedy)[ci] = CostTraits<T>::bad();
                }
                if (c.status == PRS_CFG_OK) {
                    have = true;
                    p = c.p; q = c.q;
                    c_full = c.c_full; g_full = c.g_full; c_last = c.c_last; g_last = c.g_last;
                    k = gl; par = 0; apar = gl == 0 ? 1 : 0;
                    wtot = segBase = apos = astart = bpos = 0;
                    lastS = 0; farA = farB = false;
                    cc = k == q - 1 ? c_last : c_full; gg = k == q - 1 ? g_last : g_full;
                    if (kComp) {
                        alpha = c.alpha; beta = c.beta; gamma = c.gamma;
                        rest = comp_drop(c.comp, gl);
                        const T sz = static_cast<T>(rest ? comp_first(rest) : 1);
                        const T bs = beta * sz;                               // each product and sum rounded on its own
                        cc = alpha + bs; gg = gamma * sz;
                    }
                }
            }
        }
        if (ballot64(have) == 0 && ballot64(!exhausted) == 0) break;

        const bool active = have && k < q;

        // ---------------------------------------------------------------- what the neighbours have done so far
        int pw = wtot;
        T plast = lastS;
        if (G > 1) {
            pw = __shfl(wtot, prod, kWave);
            plast = __shfl(lastS, prod, kWave);
        }
        const bool first = k == 0;
        const int aend = astart + p;
        const int availEnd = first ? aend : (pw < aend ? pw : aend);
        // every missing value is >= front (nothing is known before the producer has started this stream)
        const T front = (first || pw >= aend) ? kInf : (pw > astart ? plast : T(0));

        // ---------------------------------------------------------------- heads of A and B
        T a0 = ring[(apos & M) * kWave + prod], a1 = ring[((apos + 1) & M) * kWave + prod];
        T sb0 = ring[(bpos & M) * kWave + lane], sb1 = ring[((bpos + 1) & M) * kWave + lane];
        if (anyFar) {                       // the same in all lanes: only this path waits for the loads below
            PRS_KEEP_BRANCH();
            if (farA) { a0 = la0; a1 = la1; }
            if (farB) { sb0 = lb0; sb1 = lb1; }
        }
        if (first) { a0 = 0; a1 = 0; }
        T b0 = wrap_add<T>(sb0, gg), b1 = wrap_add<T>(sb1, gg);
        if (!(apos < availEnd)) a0 = kInf;
        if (!(apos + 1 < availEnd)) a1 = kInf;
        if (!(bpos < wtot)) b0 = kInf;
        if (!(bpos + 1 < wtot)) b1 = kInf;

        // ---------------------------------------------------------------- the two smallest; e2 is the larger one
        const bool x = a0 <= b0;
        const T u = x ? a1 : a0, v = x ? b0 : b1;
        const bool y = u <= v;
        const T e2 = y ? u : v;
        const int dA = (x ? 1 : 0) + (y ? 1 : 0);
        // (My buffer `par` held my stream of two rounds ago.  Its reader is through with it: I can only have
        // finished the round in between after the first lane of the group finished it, and every lane after the
        // first had to read its producer's whole stream to finish.)
        const bool ok = active && e2 < kInf && e2 <= front;

        // ---------------------------------------------------------------- new state of the lane
        const T tc = wrap_add<T>(e2, cc), tr = wrap_add<T>(tc, gg);           // sender leaves at tc, receiver stays until tr
        const int w0 = wtot, i = wtot - segBase;
        const bool seg_end = ok && i == p - 2;                                // the last receiver is the root
        const bool last_seg = seg_end && k == q - 1;
        T *const wbuf = mybuf + static_cast<size_t>(par) * slot_p;
        if (ok) {
            lastS = tc;
            ++wtot;
            apos += dA; bpos += 2 - dA;
            if (seg_end) {
                lastS = tr;
                ++wtot;
                k += G; par ^= 1;
                segBase = wtot; bpos = wtot;
                astart = gl == 0 ? segBase - p : segBase;                     // the stream my producer writes in its current round
                apar = gl == 0 ? par ^ 1 : par;
                apos = astart;
                cc = k == q - 1 ? c_last : c_full; gg = k == q - 1 ? g_last : g_full;
                if (kComp) {
                    rest = comp_drop(rest, G);
                    const T sz = static_cast<T>(rest ? comp_first(rest) : 1);
                    const T bs = beta * sz;
                    cc = alpha + bs; gg = gamma * sz;
                }
            }
        }
        const bool on = have && k < q;
        const uint64_t on_mask = ballot64(on);
        if ((on_mask & gmask) == 0) have = false;                            // every lane of the group is through: fetch next

        // ---------------------------------------------------------------- entries too far back for LDS: load them now
        // (before this iteration's stores, so that waiting for the loads does not wait for those; what is
        // loaded was written in earlier iterations)
        farA = on && k > 0 && pw - apos > kNear;
        farB = on && w0 - bpos > kNear;
        anyFar = ballot64(farA || farB) != 0;
        if (anyFar) {
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");            // stores of earlier iterations have landed
            if (farA) {
                const int i0 = apos - astart < p ? apos - astart : p - 1, i1 = i0 + 1 < p ? i0 + 1 : p - 1;
                la0 = prodbuf[static_cast<size_t>(apar) * slot_p + i0];
                la1 = prodbuf[static_cast<size_t>(apar) * slot_p + i1];
            }
            if (farB) {
                const int i0 = bpos - segBase;
                lb0 = mybuf[static_cast<size_t>(par) * slot_p + i0];
                lb1 = mybuf[static_cast<size_t>(par) * slot_p + i0 + 1];
            }
        }

        // ---------------------------------------------------------------- this pair's entries
        if (ok) {
            wbuf[i] = tc;
            ring[(w0 & M) * kWave + lane] = tc;
            if (seg_end) {
                wbuf[p - 1] = tr;
                ring[((w0 + 1) & M) * kWave + lane] = tr;
                if (last_seg && times.greedy) static_cast<T *>(times.greedy)[ci] = tr;
            }
        }
    }
}

// One launch for the whole batch: every wavefront works through the classes from the heaviest
// configurations (largest groups) to the lightest, so the long-running ones start first and the light
// ones fill the machine around them.
template <typename T, bool kComp>
__global__ __launch_bounds__(kWave) void uni_times_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model, TimesOut times,
                                                          PlanHeader *plan, const int32_t *order, char *slots, size_t slot_bytes,
                                                          int32_t slot_p)
{
    PRS_DYNAMIC_LDS(lds_raw);
    T *ring = reinterpret_cast<T *>(lds_raw);                    // [kRing][64]
    T *slot = reinterpret_cast<T *>(slots + static_cast<size_t>(blockIdx.x) * slot_bytes);
    // configurations of millions of pairs trail their predecessor segment by thousands of entries: a whole wavefront each
    uni_times_body<T, 64, kComp>(ring, cfg, p_max, q_max, model, times, plan, order, kClasses - 1, kGiantPart, slot, slot_p);
    __syncthreads();
    uni_times_body<T, 32, kComp>(ring, cfg, p_max, q_max, model, times, plan, order, kClasses - 1, kRestPart, slot, slot_p);
    __syncthreads();
    uni_times_body<T, 16, kComp>(ring, cfg, p_max, q_max, model, times, plan, order, 2, kWholeClass, slot, slot_p);
    __syncthreads();
    uni_times_body<T, 4, kComp>(ring, cfg, p_max, q_max, model, times, plan, order, 1, kWholeClass, slot, slot_p);
    __syncthreads();
    uni_times_body<T, 1, kComp>(ring, cfg, p_max, q_max, model, times, plan, order, 0, kWholeClass, slot, slot_p);
}

template <typename T, bool kComp>
static void launch_uni_times_as(const UniLaunch &L)
{
    hipLaunchKernelGGL((uni_times_kernel<T, kComp>), dim3(L.grid), dim3(kWave), uni_times_lds_bytes(), L.stream, L.cfg, L.p_max,
                       L.q_max, L.model, L.times, L.plan, L.order, L.slots, L.slot_bytes, L.slot_p);
}

hipError_t launch_uni_times(const UniLaunch &L)
{
    const bool comp = L.cfg.comp_m > 0;
    if (L.cost == PRS_COST_I64) {
        if (comp) launch_uni_times_as<int64_t, true>(L); else launch_uni_times_as<int64_t, false>(L);
    } else {
        if (comp) launch_uni_times_as<double, true>(L); else launch_uni_times_as<double, false>(L);
    }
    return hipGetLastError();
}

}  // namespace prs
