// Uni-greedy completion times (Lowery & Langou, Algorithm 1, Section 5) on gfx950, one lane per segment.
//
// Algorithm 1 handles segment k+1 with the final states of segment k as its initial states, but it only
// ever looks at the smallest of them.  The states of segment k leave in non-decreasing order (the start
// time t of its pairs never decreases), so segment k+1 can begin as soon as segment k has produced its
// first values and then follows right behind it: the schedule of one configuration is a pipeline of
// segments.  Here the 64 lanes of a wavefront are 64 consecutive segments of one configuration; lane l
// runs segments l, l+64, l+128, ... and reads the stream produced by lane l-1.  Per iteration every lane
// whose two smallest remaining values are known and safe performs one pair of its segment:
//   remaining values of a segment = unread tail of its input stream A (sorted) merged with the unread
//   tail of B, the values (t + tcomm) + tcomp of its own earlier pairs (sorted as well);
//   the pair takes the two smallest, t = the larger of them; t + tcomm goes to the output stream S.
// B is not stored: B[i] = S[i] + tcomp with the same rounding as (t + tcomm) + tcomp.
// A value not yet produced by the previous segment is at least as large as the last one produced, so
// a pair is safe as soon as its larger element does not exceed that value.  The root's final state
// (the maximum) closes each stream.
//
// Streams live in the wavefront's workspace slot (two buffers per lane, alternating between the
// segments a lane runs); the last kRing values of every stream are also kept in LDS, which serves
// nearly all reads.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kRing = 32;          // stream values per lane kept in LDS

size_t uni_pipe_lds_bytes() { return static_cast<size_t>(kRing) * kWave * 8; }
size_t uni_pipe_slot_bytes(int32_t p_cap) { return static_cast<size_t>(kWave) * 2 * static_cast<size_t>(p_cap) * 8; }

template <typename T>
__global__ __launch_bounds__(kWave) void uni_pipe_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model, TimesOut times,
                                                         PlanHeader *plan, const int32_t *order, int cls, char *slots,
                                                         size_t slot_bytes, int32_t slot_p)
{
    PRS_DYNAMIC_LDS(lds_raw);
    T *ring = reinterpret_cast<T *>(lds_raw);                    // [kRing][64]
    const int lane = lane_id();
    const int prod = (lane + kWave - 1) & (kWave - 1), cons = (lane + 1) & (kWave - 1);
    T *slot = reinterpret_cast<T *>(slots + static_cast<size_t>(blockIdx.x) * slot_bytes);
    T *mybuf = slot + static_cast<size_t>(lane) * 2 * slot_p;    // [2][slot_p]
    T *prodbuf = slot + static_cast<size_t>(prod) * 2 * slot_p;
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];

    for (;;) {
        const int64_t ticket = next_ticket(&plan->ticket[cls]);
        if (ticket >= count) break;
        const int64_t ci = order[begin + ticket];
        const Config<T> c = decode_config<T>(cfg, ci, p_max, q_max);
        T final_time = CostTraits<T>::bad();
        if (c.status == PRS_CFG_OK) {
            const int p = c.p, q = c.q;
            // ---- lane state
            int k = lane;                    // segment this lane is running (>= q: none left)
            int par = 0;                     // which of my two stream buffers segment k writes
            int ia = 0, ib = 0, ns = 0;      // read positions in A and B, pairs done
            bool ha0 = false, ha1 = false, hb0 = false, hb1 = false;
            T a0 = 0, a1 = 0, b0 = 0, b1 = 0;             // cached heads of A and B
            T lastS = 0;                     // last value written to my stream in this segment
            T prevRoot = 0;                  // root's final state of the last segment I finished
            int fin = -1;                    // last segment I finished
            int wtot = 0, segBase = 0, prevSegBase = 0;   // values ever written; value of wtot at segment starts
            T cc = c.c(k < q ? k : 0), gg = c.g(k < q ? k : 0);
            T result = 0;
            for (;;) {
                const bool active = k < q;
                if (ballot64(active) == 0) break;
                // ---- what the neighbours have done so far
                const int pk = __shfl(k, prod, kWave), pns = __shfl(ns, prod, kWave), pfin = __shfl(fin, prod, kWave);
                const int pwtot = __shfl(wtot, prod, kWave), pbase = __shfl(segBase, prod, kWave),
                          pprevbase = __shfl(prevSegBase, prod, kWave);
                const T plast = __shfl(lastS, prod, kWave), proot = __shfl(prevRoot, prod, kWave);
                const int cfin = __shfl(fin, cons, kWave);
                // ---- how much of my input stream A is there, and a lower bound for the rest
                int avail = 0;
                bool complete = false;
                T front = 0;                                          // every missing value is >= front
                int abase = 0;                                        // producer's write count at A[0]
                if (active) {
                    if (k == 0 || pfin >= k - 1) { avail = p; complete = true; abase = pk == k - 1 ? pbase : pprevbase; }
                    else if (pk == k - 1) { avail = pns; front = plast; abase = pbase; }
                }
                const int apar = ((k - 1) >> 6) & 1;
                // ---- refill the cached heads; old values come from the workspace, recent ones from LDS
                const bool wa0 = active && !ha0 && ia < avail, wa1 = active && !ha1 && ia + 1 < avail;
                const bool wb0 = active && !hb0 && ib < ns, wb1 = active && !hb1 && ib + 1 < ns;
                const bool ga0 = wa0 && k > 0 && ia < p - 1 && pwtot - (abase + ia) > kRing - 1;
                const bool ga1 = wa1 && k > 0 && ia + 1 < p - 1 && pwtot - (abase + ia + 1) > kRing - 1;
                const bool gb0 = wb0 && wtot - (segBase + ib) > kRing - 1, gb1 = wb1 && wtot - (segBase + ib + 1) > kRing - 1;
                if (ballot64(ga0 || ga1 || gb0 || gb1) != 0)
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");   // stores of earlier iterations have landed
                if (wa0) {
                    if (k == 0) a0 = 0;
                    else if (ia == p - 1) a0 = proot;
                    else if (ga0) a0 = prodbuf[static_cast<size_t>(apar) * slot_p + ia];
                    else a0 = ring[((abase + ia) & (kRing - 1)) * kWave + prod];
                    ha0 = true;
                }
                if (wa1) {
                    if (k == 0) a1 = 0;
                    else if (ia + 1 == p - 1) a1 = proot;
                    else if (ga1) a1 = prodbuf[static_cast<size_t>(apar) * slot_p + ia + 1];
                    else a1 = ring[((abase + ia + 1) & (kRing - 1)) * kWave + prod];
                    ha1 = true;
                }
                if (wb0) {
                    const T s = gb0 ? mybuf[static_cast<size_t>(par) * slot_p + ib] : ring[((segBase + ib) & (kRing - 1)) * kWave + lane];
                    b0 = s + gg;
                    hb0 = true;
                }
                if (wb1) {
                    const T s = gb1 ? mybuf[static_cast<size_t>(par) * slot_p + ib + 1]
                                    : ring[((segBase + ib + 1) & (kRing - 1)) * kWave + lane];
                    b1 = s + gg;
                    hb1 = true;
                }
                // ---- the two smallest remaining values, if known
                bool ok = false;
                int dA = 0, dB = 0;
                T e2 = 0;
                if (ha0 && (!hb0 || !(b0 < a0))) {
                    if (ha1 && (!hb0 || !(b0 < a1))) { dA = 2; e2 = a1; ok = true; }
                    else if (hb0) { dA = 1; dB = 1; e2 = b0; ok = true; }
                } else if (hb0) {
                    if (ha0 && (!hb1 || !(b1 < a0))) { dA = 1; dB = 1; e2 = a0; ok = true; }
                    else if (hb1) { dB = 2; e2 = b1; ok = true; }
                }
                if (ok && !complete && !(e2 <= front)) ok = false;    // a missing value could be smaller
                // my buffer `par` still holds the stream of two rounds ago until its reader is through with it
                if (ns == 0 && k >= 2 * kWave && cfin < k - 2 * kWave + 1) ok = false;
                if (active && ok) {
                    const T tc = e2 + cc, tr = tc + gg;              // sender leaves at tc, receiver stays until tr
                    mybuf[static_cast<size_t>(par) * slot_p + ns] = tc;
                    ring[(wtot & (kRing - 1)) * kWave + lane] = tc;
                    lastS = tc;
                    ++wtot;
                    if (dA == 2) { ia += 2; ha0 = ha1 = false; }
                    else if (dA == 1) { ia += 1; a0 = a1; ha0 = ha1; ha1 = false; }
                    if (dB == 2) { ib += 2; hb0 = hb1 = false; }
                    else if (dB == 1) { ib += 1; b0 = b1; hb0 = hb1; hb1 = false; }
                    ++ns;
                    const int live = ns - ib;                         // the new value of B may be a head already
                    if (live == 1) { b0 = tr; hb0 = true; }
                    else if (live == 2) { b1 = tr; hb1 = true; }
                    if (ns == p - 1) {                                // segment done: the last receiver is the root
                        prevRoot = tr; fin = k; result = tr;
                        k += kWave; par ^= 1;
                        ia = ib = ns = 0; ha0 = ha1 = hb0 = hb1 = false; lastS = 0;
                        prevSegBase = segBase; segBase = wtot;
                        cc = c.c(k < q ? k : 0); gg = c.g(k < q ? k : 0);
                    }
                }
            }
            final_time = __shfl(result, (q - 1) & (kWave - 1), kWave);
        }
        if (lane == 0) {                  // the only lane-dependent branch of the loop body
            write_closed_forms<T>(times, ci, c, model);
            if (times.greedy) static_cast<T *>(times.greedy)[ci] = final_time;
            if (times.cfg_status) times.cfg_status[ci] = c.status;
        }
        __syncthreads();
    }
}

hipError_t launch_uni_pipe(const UniLaunch &L)
{
    if (L.cost == PRS_COST_I64)
        hipLaunchKernelGGL((uni_pipe_kernel<int64_t>), dim3(L.grid), dim3(kWave), uni_pipe_lds_bytes(), L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.plan, L.order, L.cls, L.slots, L.slot_bytes, L.slot_p);
    else
        hipLaunchKernelGGL((uni_pipe_kernel<double>), dim3(L.grid), dim3(kWave), uni_pipe_lds_bytes(), L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.plan, L.order, L.cls, L.slots, L.slot_bytes, L.slot_p);
    return hipGetLastError();
}

}  // namespace prs
