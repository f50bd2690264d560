// Uni-greedy schedules (Lowery & Langou, Algorithm 1, Section 5) on gfx950: the segment pipeline of the
// completion-time kernel with processor identities.  It emits the pairs of every segment in the order of
// Algorithm 1 (ties by processor index, the root never sending) with their start times.
//
// Differences to the value-only pipeline:
//  - stream entries are (value, sender index) and must reach the next segment sorted by both.  Senders
//    of one start time leave with equal values and rising indices, except that the first pair of such a
//    run may be led by a processor left over from a smaller value, and that sums of different start times
//    can round to the same double.  The producer therefore holds back the entry with the largest index of
//    the running value, writes the others in index order (inserting a late smaller index where it
//    belongs), and the next segment only reads entries below the running value: they are final.
//  - the root's final state (largest value, index 0) closes the stream of a segment as in the value pipeline,
//    but it sorts before stream entries of equal value (they occur when tcomp vanishes against the clock),
//    so it goes through the same insertion.
//  - B needs the receiver's index per pair, kept in a per-lane array; its values are still S + tcomp.
//    Equal B values are kept in index order by the same insertion.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kRingS = 32;           // stream entries per lane kept in LDS
constexpr int kNearS = kRingS - 5;   // entries this close behind the writer are read from LDS in the next iteration

constexpr int kStage = 8;            // pairs per lane waiting in LDS for their 16-byte stores

size_t uni_sched_lds_bytes() { return static_cast<size_t>(kRingS) * kWave * 16 + static_cast<size_t>(kWave) * kStage * 16; }
// per lane: stream values [2][p], stream indices [2][p], receiver indices [p]
size_t uni_sched_slot_bytes(int32_t p_cap)
{
    return static_cast<size_t>(kWave) * (2 * static_cast<size_t>(p_cap) * 12 + static_cast<size_t>(p_cap) * 4);
}

template <typename T> __device__ __forceinline__ bool key_less(T xa, int32_t ia, T xb, int32_t ib)
{
    return xa < xb || (xa == xb && ia < ib);
}

// Entries [lo, n) of a per-lane array of processor indices are sorted; the new index wi belongs among them.  Moves
// the larger ones up by one place and returns the place that is now free for wi.  Entry i sits in LDS at
// ring[((ringBase + i) & (kRingS - 1)) * kWave + lane] as long as n + 1 - i <= kRingS (the new entry takes over the
// slot of the one kRingS places back) and in the workspace at buf[i] once i < rows_done; both copies are kept right.
// Four entries are read from LDS at a time: the reads are independent of each other, so a move of up to four places
// costs one LDS round trip.
__device__ __forceinline__ int make_room(int32_t *ring, int32_t *buf, int ringBase, int n, int lo, int rows_done, int32_t wi,
                                         int lane)
{
    constexpr int M = kRingS - 1;
    int at = n;
    for (;;) {
        int32_t m[4];
        bool up[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) m[i] = ring[((ringBase + at - 1 - i) & M) * kWave + lane];
        bool more = true;
        int c = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            more = more && at - 1 - i >= lo && n + 2 - (at - i) <= kRingS && m[i] > wi;
            up[i] = more;
            c += more ? 1 : 0;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (up[i]) {
                ring[((ringBase + at - i) & M) * kWave + lane] = m[i];
                if (at - i < rows_done) buf[at - i] = m[i];
            }
        }
        at -= c;
        if (c < 4) break;
    }
    // entries too old for LDS come from the workspace, eight loads in flight at a time (two runs of equal values
    // that each span hundreds of processors are merged this way, entry by entry of the later one)
    while (at > lo && n + 2 - at > kRingS) {
        int32_t m[8];
        bool up[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) m[i] = buf[at - 1 - i > 0 ? at - 1 - i : 0];
        bool more = true;
        int c = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            more = more && at - 1 - i >= lo && m[i] > wi;
            up[i] = more;
            c += more ? 1 : 0;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (up[i]) {
                if (n + 1 - (at - i) <= kRingS) ring[((ringBase + at - i) & M) * kWave + lane] = m[i];
                if (at - i < rows_done) buf[at - i] = m[i];
            }
        }
        at -= c;
        if (c < 8) break;
    }
    return at;
}

template <typename T, int G>
__device__ __forceinline__ void uni_sched_body(char *lds_raw, const ConfigArrays &cfg, int32_t p_max, int32_t q_max,
                                               const SchedOut &sched, PlanHeader *plan, const int32_t *order, int cls, int part,
                                               char *slot, int32_t slot_p)
{
    constexpr int M = kRingS - 1;
    T *ringX = reinterpret_cast<T *>(lds_raw);                                   // [kRingS][64] stream values
    int32_t *ringI = reinterpret_cast<int32_t *>(ringX + kRingS * kWave);        // [kRingS][64] stream sender indices
    int32_t *ringB = ringI + kRingS * kWave;                                     // [kRingS][64] receiver index per pair
    T *stT = reinterpret_cast<T *>(ringB + kRingS * kWave);                      // [64][kStage] start times of the lane's last pairs
    int32_t *stS = reinterpret_cast<int32_t *>(stT + kWave * kStage);            // [64][kStage] their senders
    int32_t *stD = stS + kWave * kStage;                                         // [64][kStage] their receivers
    const int lane = lane_id(), gl = lane & (G - 1), gbase = lane & ~(G - 1);
    const int prod = gbase | ((gl + G - 1) & (G - 1));
    const uint64_t gmask = (G == 64 ? ~UINT64_C(0) : ((UINT64_C(1) << G) - 1)) << gbase;
    const size_t per_lane = 2 * static_cast<size_t>(slot_p) * 12 + static_cast<size_t>(slot_p) * 4;
    auto bufX = [&](int l, int par) { return reinterpret_cast<T *>(slot + l * per_lane + static_cast<size_t>(par) * slot_p * 8); };
    auto bufI = [&](int l, int par) {
        return reinterpret_cast<int32_t *>(slot + l * per_lane + 2 * static_cast<size_t>(slot_p) * 8 + static_cast<size_t>(par) * slot_p * 4);
    };
    int32_t *bufB = reinterpret_cast<int32_t *>(slot + lane * per_lane + 2 * static_cast<size_t>(slot_p) * 12);
    // part of the class this pass works on: all of it, its giant configurations only, or the rest after those
    int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    unsigned long long *tickets = &plan->ticket[cls];
    if (part == kGiantPart) { count = plan->giant_count; tickets = &plan->ticket_giant; }
    else if (part == kRestPart) { begin += plan->giant_count; count -= plan->giant_count; }
    const T kInf = CostTraits<T>::inf();

    // ---- per-group state (the same in all lanes of a group)
    bool have = false, exhausted = false;
    int64_t ci = 0, out_base = 0;
    int p = 2, q = 1;
    T c_full = 0, g_full = 0, c_last = 0, g_last = 0;
    // ---- per-lane state.  Positions count stream entries from the start of the configuration: every finished
    // segment adds p of them (one per pair and the root's); pair i of a segment shares position i with entry i.
    int k = 0, par = 0, apar = 0;
    int wtot = 0, segBase = 0;      // entries written; the same at the start of my segment
    int ns = 0;                     // pairs done in my segment (entries written + the one held back)
    int runStart = 0;               // first entry of the running value, relative to segBase: entries before it are final
    int apos = 0, astart = 0;       // next entry of my input stream; its first entry
    int bpos = 0;                   // next pair of my segment whose B entry is unread (absolute)
    bool hold = false;
    T holdX = 0; int32_t holdI = 0; // entry of the running value held back (largest index so far)
    T lastS = 0;                    // running value of my stream (0 before the first pair of a segment)
    T lastBx = 0; int brun = 0;     // value of the last B entry pushed, first pair of that value (relative)
    int32_t lastWi = 0, lastBi = 0; // sender of the last stream entry written, receiver of the last B entry
    // Stream entries and receiver indices leave LDS in rows of eight, pairs in rows of four.  Rows are written
    // every fourth iteration of the wavefront, by all lanes at once: done per lane whenever its row fills, the
    // row code would run in almost every iteration for a few lanes each.
    int fW = 0, fB = 0, fO = 0;     // entries / receivers / pairs of my segment that have reached the workspace (multiples of 8, 8 and 4)
    int iter = 0;
    T cc = 0, gg = 0;
    bool farA = false, farB = false, anyFar = false;
    T la0 = 0, la1 = 0, lb0 = 0, lb1 = 0;
    int32_t lai0 = 0, lai1 = 0, lbi0 = 0, lbi1 = 0;

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
                int32_t status = c.status;
                out_base = 0;
                if (status == PRS_CFG_OK) {
                    out_base = sched.pair_offset[ci];
                    const int64_t n_pairs = static_cast<int64_t>(c.p - 1) * c.q;
                    if (out_base < 0 || out_base + n_pairs > sched.pair_capacity) status = PRS_CFG_TOO_LARGE;
                }
                if (gl == 0) {
                    if (sched.cfg_status) sched.cfg_status[ci] = status;
                    if (status != PRS_CFG_OK && sched.T_greedy) static_cast<T *>(sched.T_greedy)[ci] = CostTraits<T>::bad();
                }
                if (status == PRS_CFG_OK) {
                    have = true;
                    p = c.p; q = c.q;
                    c_full = c.c_full; g_full = c.g_full; c_last = c.c_last; g_last = c.g_last;
                    k = gl; par = 0; apar = gl == 0 ? 1 : 0;
                    wtot = segBase = ns = runStart = apos = astart = bpos = brun = 0;
                    fW = fB = fO = 0;
                    hold = false; lastS = 0;
                    farA = farB = false;
                    cc = k == q - 1 ? c_last : c_full; gg = k == q - 1 ? g_last : g_full;
                }
            }
        }
        if (ballot64(have) == 0 && ballot64(!exhausted) == 0) break;

        const bool active = have && k < q;
        const int n1 = p - 1;                                               // entries (pairs) per segment

        // ---------------------------------------------------------------- what my producer has done so far
        int pw = wtot, pfinal = segBase + runStart;
        T plast = lastS;
        if (G > 1) {
            pw = __shfl(wtot, prod, kWave);
            pfinal = __shfl(segBase + runStart, prod, kWave);
            plast = __shfl(lastS, prod, kWave);
        }
        const bool first = k == 0;
        const int aend = astart + p;
        const int availEnd = first ? aend : (pfinal < aend ? pfinal : aend);   // entries below the producer's running value are final
        const bool complete = first || pfinal >= aend;
        // entries not final yet are >= the running value of a producer that is on my stream
        const T front = complete ? kInf : (pfinal >= astart ? plast : T(0));

        // ---------------------------------------------------------------- heads of A and B
        const int r0 = (apos & M) * kWave + prod, r1 = ((apos + 1) & M) * kWave + prod;
        T a0 = ringX[r0], a1 = ringX[r1];
        int32_t a0i = ringI[r0], a1i = ringI[r1];
        T sb0 = ringX[(bpos & M) * kWave + lane], sb1 = ringX[((bpos + 1) & M) * kWave + lane];
        int32_t b0i = ringB[(bpos & M) * kWave + lane], b1i = ringB[((bpos + 1) & M) * kWave + lane];
        if (anyFar) {                       // the same in all lanes: only this path waits for the loads at the end of the loop
            PRS_KEEP_BRANCH();
            if (farA) { a0 = la0; a1 = la1; a0i = lai0; a1i = lai1; }
            if (farB) { sb0 = lb0; sb1 = lb1; b0i = lbi0; b1i = lbi1; }
        }
        if (first) { a0 = 0; a1 = 0; a0i = apos; a1i = apos + 1; }          // first segment: processors 0..p-1 at time 0
        const bool ha0 = apos < availEnd, ha1 = apos + 1 < availEnd;
        // B value i is stream value i; the newest one may still be the held entry of the running value
        if (!(bpos < wtot)) sb0 = lastS;
        if (!(bpos + 1 < wtot)) sb1 = lastS;
        const T b0 = wrap_add<T>(sb0, gg), b1 = wrap_add<T>(sb1, gg);
        const bool hb0 = bpos < segBase + ns, hb1 = bpos + 1 < segBase + ns;

        // ---------------------------------------------------------------- the two smallest keys of A and B
        const bool x = ha0 && !(hb0 && key_less<T>(b0, b0i, a0, a0i));        // the smallest is A's head
        const bool hu = x ? ha1 : ha0, hv = x ? hb0 : hb1;                     // heads after removing it
        const T ux = x ? a1 : a0, vx = x ? b0 : b1;
        const int32_t ui = x ? a1i : a0i, vi = x ? b0i : b1i;
        const bool y = hu && !(hv && key_less<T>(vx, vi, ux, ui));            // the second smallest comes from A
        const int32_t e1i = x ? a0i : b0i;
        const T e2x = y ? ux : vx;
        const int32_t e2i = y ? ui : vi;
        // an entry that is not final yet could come first
        const bool ok = active && (ha0 || hb0) && (hu || hv) && (complete || e2x < front);

        if (ok) {
            const T t = e2x, tc = wrap_add<T>(t, cc), tr = wrap_add<T>(tc, gg);
            int32_t snd = e1i, rcv = e2i;
            if (e1i == 0) { snd = e2i; rcv = 0; }                             // the root never sends (Lemma 1 (ii))
            // ---- the pair waits in the lane's staging rows
            {
                const int slot = lane * kStage + (ns & (kStage - 1));
                stS[slot] = snd; stD[slot] = rcv; stT[slot] = t;
            }
            T *const myX = bufX(lane, par);
            int32_t *const myI = bufI(lane, par);
            int w = wtot - segBase;                                           // entries written in this segment
            // Writes one stream entry.  Entries of the running value are written in rising index order; a
            // smaller index that comes late is inserted (the next segment does not read the running value
            // yet).  Entries that have reached the workspace (the first fW) are corrected there as well; what
            // is read from the workspace is always older than the rows still waiting in LDS.
            // The new entry takes over the LDS slot of the one kRingS places back, so an insertion that
            // reaches that far reads the workspace copy.
            auto put = [&](T wx, int32_t wi, int run_from) {
                int at = w;
                // the usual case: the index is larger than the last one written, nothing to move, nothing to read
                if (lastWi > wi && w > run_from) at = make_room(ringI, myI, segBase, w, run_from, fW, wi, lane);
                ringX[(wtot & M) * kWave + lane] = wx;
                if (w + 1 - at <= kRingS) ringI[((segBase + at) & M) * kWave + lane] = wi;
                if (at < fW) myI[at] = wi;
                if (at == w) lastWi = wi;                                     // index of the last entry written
                ++w; ++wtot;
            };
            // ---- stream entry (tc, snd): keep the largest index of the running value back
            T wx = 0; int32_t wi = 0; bool wr = false;
            if (hold && tc == holdX) {
                if (snd > holdI) { wx = holdX; wi = holdI; holdI = snd; } else { wx = tc; wi = snd; }
                wr = true;
            } else {
                if (hold) { wx = holdX; wi = holdI; wr = true; }
                hold = true; holdX = tc; holdI = snd;
            }
            if (wr) put(wx, wi, runStart);
            if (!(tc == lastS) || ns == 0) runStart = w;                      // entries before the running value are final
            lastS = tc;
            // ---- B entry (tr, rcv) of pair ns; equal values keep rising index order
            if (ns == 0 || !(tr == lastBx)) brun = ns;
            lastBx = tr;
            {
                int at = ns;
                const int ib = bpos - segBase;
                const int lo = brun > ib ? brun : ib;
                if (lastBi > rcv && ns > lo) at = make_room(ringB, bufB, segBase, ns, lo, fB, rcv, lane);
                if (ns + 1 - at <= kRingS) ringB[((segBase + at) & M) * kWave + lane] = rcv;
                if (at < fB) bufB[at] = rcv;
                if (at == ns) lastBi = rcv;                                   // receiver of the last B entry
            }
            // ---- consume
            const int dA = (x ? 1 : 0) + (y ? 1 : 0);
            apos += dA; bpos += 2 - dA;
            ++ns;
            if (ns == n1) {                                                   // segment done: flush, hand over
                put(holdX, holdI, runStart);                                  // the held index is the largest of its value
                hold = false;
                // the root's final state: the largest value, in front of entries of the same value
                if (!(tr == lastS)) runStart = w;
                put(tr, 0, runStart);
                // everything of the segment that still waits in LDS
                for (int j = fW; j < w; ++j) {
                    const int rr = ((segBase + j) & M) * kWave + lane;
                    myX[j] = ringX[rr]; myI[j] = ringI[rr];
                }
                for (int j = fB; j < n1; ++j) bufB[j] = ringB[((segBase + j) & M) * kWave + lane];
                for (int j = fO; j < n1; ++j) {
                    const int slot = lane * kStage + (j & (kStage - 1));
                    const int64_t oj = out_base + static_cast<int64_t>(k) * n1 + j;
                    if (sched.src) sched.src[oj] = stS[slot];
                    if (sched.dst) sched.dst[oj] = stD[slot];
                    if (sched.seg) sched.seg[oj] = k;
                    if (sched.tstart) static_cast<T *>(sched.tstart)[oj] = stT[slot];
                }
                fW = fB = fO = 0;
                if (k == q - 1 && sched.T_greedy) static_cast<T *>(sched.T_greedy)[ci] = tr;
                k += G; par ^= 1;
                segBase = wtot; ns = 0; runStart = 0; brun = 0; bpos = wtot;
                lastS = 0;
                astart = gl == 0 ? segBase - p : segBase;                     // the stream my producer writes in its current round
                apar = gl == 0 ? par ^ 1 : par;
                apos = astart;
                cc = k == q - 1 ? c_last : c_full; gg = k == q - 1 ? g_last : g_full;
            }
        }
        // ---------------------------------------------------------------- full rows leave LDS (every fourth iteration)
        if ((++iter & 3) == 0) {
            T *const myX = bufX(lane, par);
            int32_t *const myI = bufI(lane, par);
            const int w = wtot - segBase;
            // stream entries and receivers in rows of eight (64 bytes of values: whole sectors of a cache line, which
            // the L2 can no longer merge once millions of half-written lines are open)
            if (have && k < q && fW + 8 <= w) {
                T rx8[8]; int32_t ri8[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int rr = ((segBase + fW + j) & M) * kWave + lane;
                    rx8[j] = ringX[rr]; ri8[j] = ringI[rr];
                }
                __builtin_memcpy(myX + fW, rx8, 64);
                __builtin_memcpy(myI + fW, ri8, 32);
                fW += 8;
            }
            if (have && k < q && fB + 8 <= ns) {
                int32_t rb8[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) rb8[j] = ringB[((segBase + fB + j) & M) * kWave + lane];
                __builtin_memcpy(bufB + fB, rb8, 32);
                fB += 8;
            }
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                if (have && k < q && fO + 4 <= ns) {
                    const int row = lane * kStage + (fO & (kStage - 1));
                    const int64_t o4 = out_base + static_cast<int64_t>(k) * n1 + fO;
                    if (sched.src) __builtin_memcpy(sched.src + o4, stS + row, 16);
                    if (sched.dst) __builtin_memcpy(sched.dst + o4, stD + row, 16);
                    if (sched.seg) { const int32_t kk[4] = {k, k, k, k}; __builtin_memcpy(sched.seg + o4, kk, 16); }
                    if (sched.tstart) __builtin_memcpy(static_cast<T *>(sched.tstart) + o4, stT + row, 32);
                    fO += 4;
                }
            }
        }
        const bool on = have && k < q;
        const uint64_t on_mask = ballot64(on);
        if ((on_mask & gmask) == 0) have = false;                            // every lane of the group is through: fetch next

        // ---------------------------------------------------------------- entries too far back for LDS: load them now
        farA = on && k > 0 && pw - apos > kNearS;
        farB = on && segBase + ns - bpos > kNearS;
        anyFar = ballot64(farA || farB) != 0;
        if (anyFar) {
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
            if (farA) {
                const int i0 = apos - astart < p ? apos - astart : p - 1, i1 = i0 + 1 < p ? i0 + 1 : p - 1;
                la0 = bufX(prod, apar)[i0]; lai0 = bufI(prod, apar)[i0];
                la1 = bufX(prod, apar)[i1]; lai1 = bufI(prod, apar)[i1];
            }
            if (farB) {
                const int i0 = bpos - segBase;                                // far: both entries were written long ago
                lb0 = bufX(lane, par)[i0]; lbi0 = bufB[i0];
                lb1 = bufX(lane, par)[i0 + 1]; lbi1 = bufB[i0 + 1];
            }
        }
    }
}

// One launch for the whole batch: every wavefront works through the classes from the heaviest
// configurations (largest groups) to the lightest.
template <typename T>
__global__ __launch_bounds__(kWave) void uni_sched_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, SchedOut sched,
                                                          PlanHeader *plan, const int32_t *order, char *slots, size_t slot_bytes,
                                                          int32_t slot_p)
{
    PRS_DYNAMIC_LDS(lds_raw);
    char *slot = slots + static_cast<size_t>(blockIdx.x) * slot_bytes;
    uni_sched_body<T, 64>(lds_raw, cfg, p_max, q_max, sched, plan, order, kClasses - 1, kGiantPart, slot, slot_p);
    __syncthreads();
    uni_sched_body<T, 32>(lds_raw, cfg, p_max, q_max, sched, plan, order, kClasses - 1, kRestPart, slot, slot_p);
    __syncthreads();
    uni_sched_body<T, 16>(lds_raw, cfg, p_max, q_max, sched, plan, order, 2, kWholeClass, slot, slot_p);
    __syncthreads();
    uni_sched_body<T, 8>(lds_raw, cfg, p_max, q_max, sched, plan, order, 1, kWholeClass, slot, slot_p);
    __syncthreads();
    uni_sched_body<T, 1>(lds_raw, cfg, p_max, q_max, sched, plan, order, 0, kWholeClass, slot, slot_p);
}

hipError_t launch_uni_sched(const UniLaunch &L)
{
    if (L.cost == PRS_COST_I64)
        hipLaunchKernelGGL((uni_sched_kernel<int64_t>), dim3(L.grid), dim3(kWave), uni_sched_lds_bytes(), L.stream, L.cfg, L.p_max,
                           L.q_max, L.sched, L.plan, L.order, L.slots, L.slot_bytes, L.slot_p);
    else
        hipLaunchKernelGGL((uni_sched_kernel<double>), dim3(L.grid), dim3(kWave), uni_sched_lds_bytes(), L.stream, L.cfg, L.p_max,
                           L.q_max, L.sched, L.plan, L.order, L.slots, L.slot_bytes, L.slot_p);
    return hipGetLastError();
}

}  // namespace prs
