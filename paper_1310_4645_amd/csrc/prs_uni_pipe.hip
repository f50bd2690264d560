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
                const int cfin = __shfl(fin, cons, kWave), ck = __shfl(k, cons, kWave), cia = __shfl(ia, cons, kWave);
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
                {
                    // all loads first, then the selects: one wait for the slowest of them
                    T va0 = 0, va1 = 0, vb0 = 0, vb1 = 0;
                    if (ga0) va0 = prodbuf[static_cast<size_t>(apar) * slot_p + ia];
                    if (ga1) va1 = prodbuf[static_cast<size_t>(apar) * slot_p + ia + 1];
                    if (gb0) vb0 = mybuf[static_cast<size_t>(par) * slot_p + ib];
                    if (gb1) vb1 = mybuf[static_cast<size_t>(par) * slot_p + ib + 1];
                    const T ra0 = ring[((abase + ia) & (kRing - 1)) * kWave + prod];
                    const T ra1 = ring[((abase + ia + 1) & (kRing - 1)) * kWave + prod];
                    const T rb0 = ring[((segBase + ib) & (kRing - 1)) * kWave + lane];
                    const T rb1 = ring[((segBase + ib + 1) & (kRing - 1)) * kWave + lane];
                    if (wa0) { a0 = k == 0 ? T(0) : (ia == p - 1 ? proot : (ga0 ? va0 : ra0)); ha0 = true; }
                    if (wa1) { a1 = k == 0 ? T(0) : (ia + 1 == p - 1 ? proot : (ga1 ? va1 : ra1)); ha1 = true; }
                    if (wb0) { b0 = (gb0 ? vb0 : rb0) + gg; hb0 = true; }
                    if (wb1) { b1 = (gb1 ? vb1 : rb1) + gg; hb1 = true; }
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
                // stay within the LDS window of my reader (it then never needs the workspace copy); with two
                // or more values waiting the reader can always go on, so this cannot block for good
                if (k + 1 < q) {
                    const int consumed = ck == k + 1 ? segBase + cia : (ck < k + 1 ? prevSegBase + cia : wtot);
                    if (wtot - consumed >= kRing - 2) ok = false;
                }
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

// ------------------------------------------------------------------------------------------------
// The same pipeline with processor identities: emits the pairs (Section 5, first paragraph) in the
// order of Algorithm 1, ties by processor index, the root never sending.
//
// Differences to the value-only kernel:
//  - stream entries are (value, sender index) and must reach the next segment sorted by both.  Senders
//    of one start time leave with equal values and rising indices, except that the first pair of such a
//    run may be led by a processor left over from a smaller value.  The producer therefore holds back
//    the entry with the largest index of the running value and writes the others; the next segment only
//    reads entries below the running value (they are final), so the order inside the run can still change.
//  - the root's final state (largest value, index 0) is a third source next to A and B: it sorts before
//    stream entries of equal value.
//  - B needs the receiver's index per pair, kept in a per-lane array; its values are still S + tcomp.
//  - sums produced at different times that round to the same double could break the index order inside
//    a run in a way the hold-back does not repair; such a configuration (none in the sweeps) is handed
//    to the batch kernel.
constexpr int kRingS = 16;

size_t uni_pipe_sched_lds_bytes() { return static_cast<size_t>(kRingS) * kWave * 16; }
size_t uni_pipe_sched_slot_bytes(int32_t p_cap)
{
    return static_cast<size_t>(kWave) * (2 * static_cast<size_t>(p_cap) * 12 + static_cast<size_t>(p_cap) * 4);
}

template <typename T> __device__ __forceinline__ bool klt(T xa, int32_t ia, T xb, int32_t ib)
{
    return xa < xb || (xa == xb && ia < ib);
}

template <typename T>
__global__ __launch_bounds__(kWave) void uni_pipe_sched_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, SchedOut sched,
                                                               PlanHeader *plan, const int32_t *order, int cls, int32_t *retry,
                                                               char *slots, size_t slot_bytes, int32_t slot_p)
{
    PRS_DYNAMIC_LDS(lds_raw);
    T *ringX = reinterpret_cast<T *>(lds_raw);                                   // [kRingS][64] stream values
    int32_t *ringI = reinterpret_cast<int32_t *>(ringX + kRingS * kWave);        // [kRingS][64] stream sender indices
    int32_t *ringB = ringI + kRingS * kWave;                                     // [kRingS][64] receiver index per pair
    const int lane = lane_id();
    const int prod = (lane + kWave - 1) & (kWave - 1), cons = (lane + 1) & (kWave - 1);
    char *slot = slots + static_cast<size_t>(blockIdx.x) * slot_bytes;
    const size_t per_lane = 2 * static_cast<size_t>(slot_p) * 12 + static_cast<size_t>(slot_p) * 4;
    auto bufX = [&](int l, int par) { return reinterpret_cast<T *>(slot + l * per_lane + static_cast<size_t>(par) * slot_p * 8); };
    auto bufI = [&](int l, int par) {
        return reinterpret_cast<int32_t *>(slot + l * per_lane + 2 * static_cast<size_t>(slot_p) * 8 + static_cast<size_t>(par) * slot_p * 4);
    };
    int32_t *bufB = reinterpret_cast<int32_t *>(slot + lane * per_lane + 2 * static_cast<size_t>(slot_p) * 12);
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];

    for (;;) {
        const int64_t ticket = next_ticket(&plan->ticket[cls]);
        if (ticket >= count) break;
        const int64_t ci = order[begin + ticket];
        const Config<T> c = decode_config<T>(cfg, ci, p_max, q_max);
        int32_t status = c.status;
        int64_t out_base = 0;
        if (status == PRS_CFG_OK) {
            out_base = sched.pair_offset[ci];
            const int64_t n_pairs = static_cast<int64_t>(c.p - 1) * c.q;
            if (out_base < 0 || out_base + n_pairs > sched.pair_capacity) status = PRS_CFG_TOO_LARGE;
        }
        T final_time = CostTraits<T>::bad();
        bool rerun = false;
        if (status == PRS_CFG_OK) {
            const int p = c.p, q = c.q;
            int k = lane, par = 0;
            int ia = 0, ib = 0, ns = 0;          // stream entries read, B entries read, pairs done
            int w = 0, runStart = 0;             // stream entries written, first entry of the running value
            bool ha0 = false, ha1 = false, hb0 = false, hb1 = false, rootUsed = false;
            T a0 = 0, a1 = 0, b0 = 0, b1 = 0;
            int32_t a0i = 0, a1i = 0, b0i = 0, b1i = 0;
            bool hold = false;                   // entry of the running value held back (largest index so far)
            T holdX = 0; int32_t holdI = 0;
            T lastS = 0;                         // running value of my stream
            T lastBx = 0; int brun = 0;          // value of the last B entry pushed, first pair of that value
            T prevRoot = 0;
            int fin = -1;
            int wtot = 0, segBase = 0, prevSegBase = 0, btot = 0, bsegBase = 0;
            T cc = c.c(k < q ? k : 0), gg = c.g(k < q ? k : 0);
            T result = 0;
            for (;;) {
                const bool active = k < q;
                if (ballot64(active) == 0) break;
                const int pk = __shfl(k, prod, kWave), prun = __shfl(runStart, prod, kWave), pfin = __shfl(fin, prod, kWave);
                const int pwtot = __shfl(wtot, prod, kWave), pbase = __shfl(segBase, prod, kWave),
                          pprevbase = __shfl(prevSegBase, prod, kWave);
                const T plast = __shfl(lastS, prod, kWave), proot = __shfl(prevRoot, prod, kWave);
                const int cfin = __shfl(fin, cons, kWave);
                // stream entries below the producer's running value are final
                int avail = 0;
                bool complete = false;
                T front = 0;
                int abase = 0;
                if (active) {
                    if (k == 0 || pfin >= k - 1) { avail = p - 1; complete = true; abase = pk == k - 1 ? pbase : pprevbase; }
                    else if (pk == k - 1) { avail = prun; front = plast; abase = pbase; }
                }
                const int apar = ((k - 1) >> 6) & 1;
                const bool wa0 = active && !ha0 && ia < avail, wa1 = active && !ha1 && ia + 1 < avail;
                const bool wb0 = active && !hb0 && ib < ns, wb1 = active && !hb1 && ib + 1 < ns;
                // (the producer writes up to two entries per iteration; entries that close to being overwritten are
                // read from the workspace so that the outcome does not depend on lanes running in lockstep)
                const bool ga0 = wa0 && k > 0 && pwtot - (abase + ia) > kRingS - 2;
                const bool ga1 = wa1 && k > 0 && pwtot - (abase + ia + 1) > kRingS - 2;
                // B value i is stream value i (still in a register if not written yet); its index is in ringB / bufB
                const bool gbx0 = wb0 && ib < w && wtot - (segBase + ib) > kRingS - 1;
                const bool gbx1 = wb1 && ib + 1 < w && wtot - (segBase + ib + 1) > kRingS - 1;
                const bool gbi0 = wb0 && btot - (bsegBase + ib) > kRingS - 1, gbi1 = wb1 && btot - (bsegBase + ib + 1) > kRingS - 1;
                if (ballot64(ga0 || ga1 || gbx0 || gbx1 || gbi0 || gbi1) != 0)
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
                {
                    // all loads first, then the selects: one wait for the slowest of them
                    T va0 = 0, va1 = 0, vb0 = 0, vb1 = 0;
                    int32_t ja0 = 0, ja1 = 0, jb0 = 0, jb1 = 0;
                    if (ga0) { va0 = bufX(prod, apar)[ia]; ja0 = bufI(prod, apar)[ia]; }
                    if (ga1) { va1 = bufX(prod, apar)[ia + 1]; ja1 = bufI(prod, apar)[ia + 1]; }
                    if (gbx0) vb0 = bufX(lane, par)[ib];
                    if (gbx1) vb1 = bufX(lane, par)[ib + 1];
                    if (gbi0) jb0 = bufB[ib];
                    if (gbi1) jb1 = bufB[ib + 1];
                    const int r0 = ((abase + ia) & (kRingS - 1)) * kWave + prod, r1 = ((abase + ia + 1) & (kRingS - 1)) * kWave + prod;
                    const T ra0 = ringX[r0], ra1 = ringX[r1];
                    const int32_t ri0 = ringI[r0], ri1 = ringI[r1];
                    const T rb0 = ringX[((segBase + ib) & (kRingS - 1)) * kWave + lane];
                    const T rb1 = ringX[((segBase + ib + 1) & (kRingS - 1)) * kWave + lane];
                    const int32_t rj0 = ringB[((bsegBase + ib) & (kRingS - 1)) * kWave + lane];
                    const int32_t rj1 = ringB[((bsegBase + ib + 1) & (kRingS - 1)) * kWave + lane];
                    if (wa0) {
                        if (k == 0) { a0 = 0; a0i = ia + 1; }             // first segment: processors 1..p-1 at time 0
                        else { a0 = ga0 ? va0 : ra0; a0i = ga0 ? ja0 : ri0; }
                        ha0 = true;
                    }
                    if (wa1) {
                        if (k == 0) { a1 = 0; a1i = ia + 2; }
                        else { a1 = ga1 ? va1 : ra1; a1i = ga1 ? ja1 : ri1; }
                        ha1 = true;
                    }
                    if (wb0) {
                        const T sx = ib < w ? (gbx0 ? vb0 : rb0) : lastS;   // not written yet: the held entry of the running value
                        b0 = sx + gg; b0i = gbi0 ? jb0 : rj0; hb0 = true;
                    }
                    if (wb1) {
                        const T sx = ib + 1 < w ? (gbx1 ? vb1 : rb1) : lastS;
                        b1 = sx + gg; b1i = gbi1 ? jb1 : rj1; hb1 = true;
                    }
                }
                // the root of this segment: at time 0 in the first segment, else the previous segment's root
                const bool hr = active && !rootUsed && (k == 0 || complete);
                const T rx = k == 0 ? 0 : proot;
                // ---- two smallest keys among the heads of A and B and the root
                int s1 = -1, s2 = -1;                  // 0: A, 1: B, 2: root
                T e1x = 0, e2x = 0; int32_t e1i = 0, e2i = 0;
                {
                    T bx = 0; int32_t bi = 0;
                    if (ha0) { s1 = 0; bx = a0; bi = a0i; }
                    if (hb0 && (s1 < 0 || klt<T>(b0, b0i, bx, bi))) { s1 = 1; bx = b0; bi = b0i; }
                    if (hr && (s1 < 0 || klt<T>(rx, 0, bx, bi))) { s1 = 2; bx = rx; bi = 0; }
                    e1x = bx; e1i = bi;
                    // second: heads after removing the first
                    const bool ca = s1 == 0 ? ha1 : ha0, cb = s1 == 1 ? hb1 : hb0, cr = hr && s1 != 2;
                    const T ax = s1 == 0 ? a1 : a0; const int32_t ai = s1 == 0 ? a1i : a0i;
                    const T bbx = s1 == 1 ? b1 : b0; const int32_t bbi = s1 == 1 ? b1i : b0i;
                    T cx = 0; int32_t cid = 0;
                    if (ca) { s2 = 0; cx = ax; cid = ai; }
                    if (cb && (s2 < 0 || klt<T>(bbx, bbi, cx, cid))) { s2 = 1; cx = bbx; cid = bbi; }
                    if (cr && (s2 < 0 || klt<T>(rx, 0, cx, cid))) { s2 = 2; cx = rx; cid = 0; }
                    e2x = cx; e2i = cid;
                }
                bool ok = s1 >= 0 && s2 >= 0;
                if (ok && !complete && !(e2x < front)) ok = false;      // an entry not final yet could come first
                if (ns == 0 && k >= 2 * kWave && cfin < k - 2 * kWave + 1) ok = false;
                if (active && ok) {
                    const T t = e2x, tc = t + cc, tr = tc + gg;
                    bool b_moved = false;
                    int32_t snd = e1i, rcv = e2i;
                    if (e1i == 0) { snd = e2i; rcv = 0; }                 // the root never sends (Lemma 1 (ii))
                    const int64_t o = out_base + static_cast<int64_t>(k) * (p - 1) + ns;
                    if (sched.src) sched.src[o] = snd;
                    if (sched.dst) sched.dst[o] = rcv;
                    if (sched.seg) sched.seg[o] = k;
                    if (sched.tstart) static_cast<T *>(sched.tstart)[o] = t;
                    // ---- stream entry (tc, snd): keep the largest index of the running value back
                    T wx = 0; int32_t wi = 0; bool wr = false;
                    if (hold && tc == holdX) {
                        if (snd > holdI) { wx = holdX; wi = holdI; holdI = snd; } else { wx = tc; wi = snd; }
                        wr = true;
                    } else {
                        if (hold) { wx = holdX; wi = holdI; wr = true; }
                        hold = true; holdX = tc; holdI = snd;
                    }
                    if (wr) {
                        // entries of the running value are written in rising index order; sums of different
                        // times that round to the same value can bring a smaller index late: insert it
                        // (the next segment does not read the running value yet)
                        int at = w;
                        while (at > runStart && bufI(lane, par)[at - 1] > wi) {
                            const int32_t mv = bufI(lane, par)[at - 1];
                            bufI(lane, par)[at] = mv;
                            if (wtot + 1 - (segBase + at) <= kRingS) ringI[((segBase + at) & (kRingS - 1)) * kWave + lane] = mv;
                            --at;
                        }
                        bufX(lane, par)[w] = wx; bufI(lane, par)[at] = wi;
                        ringX[(wtot & (kRingS - 1)) * kWave + lane] = wx;
                        if (wtot + 1 - (segBase + at) <= kRingS) ringI[((segBase + at) & (kRingS - 1)) * kWave + lane] = wi;
                        ++w; ++wtot;
                    }
                    if (!(tc == lastS) || ns == 0) runStart = w;          // entries before the running value are final
                    lastS = tc;
                    // ---- B entry (tr, rcv) of pair ns; equal values keep rising index order (same remark)
                    if (ns == 0 || !(tr == lastBx)) brun = ns;
                    lastBx = tr;
                    {
                        int at = ns;
                        const int lo = brun > ib ? brun : ib;
                        while (at > lo && bufB[at - 1] > rcv) {
                            const int32_t mv = bufB[at - 1];
                            bufB[at] = mv;
                            if (btot + 1 - (bsegBase + at) <= kRingS) ringB[((bsegBase + at) & (kRingS - 1)) * kWave + lane] = mv;
                            --at;
                        }
                        bufB[at] = rcv;
                        if (btot + 1 - (bsegBase + at) <= kRingS) ringB[((bsegBase + at) & (kRingS - 1)) * kWave + lane] = rcv;
                        if (at != ns) { hb0 = hb1 = false; b_moved = true; }   // cached heads may have changed
                        ++btot;
                    }
                    // ---- consume
                    if (s1 == 2 || s2 == 2) rootUsed = true;
                    const int dA = (s1 == 0) + (s2 == 0), dB = (s1 == 1) + (s2 == 1);
                    if (dA == 2) { ia += 2; ha0 = ha1 = false; }
                    else if (dA == 1) { ia += 1; a0 = a1; a0i = a1i; ha0 = ha1; ha1 = false; }
                    if (dB == 2) { ib += 2; hb0 = hb1 = false; }
                    else if (dB == 1) { ib += 1; b0 = b1; b0i = b1i; hb0 = hb1; hb1 = false; }
                    ++ns;
                    const int live = ns - ib;
                    if (!b_moved) {
                        if (live == 1) { b0 = tr; b0i = rcv; hb0 = true; }
                        else if (live == 2) { b1 = tr; b1i = rcv; hb1 = true; }
                    }
                    if (ns == p - 1) {                                    // segment done: flush, hand over
                        bufX(lane, par)[w] = holdX; bufI(lane, par)[w] = holdI;   // the held index is the largest of its value
                        const int r = (wtot & (kRingS - 1)) * kWave + lane;
                        ringX[r] = holdX; ringI[r] = holdI;
                        ++w; ++wtot;
                        hold = false;
                        prevRoot = tr; fin = k; result = tr;
                        k += kWave; par ^= 1;
                        ia = ib = ns = w = runStart = 0;
                        ha0 = ha1 = hb0 = hb1 = rootUsed = false; lastS = 0; brun = 0;
                        prevSegBase = segBase; segBase = wtot; bsegBase = btot;
                        cc = c.c(k < q ? k : 0); gg = c.g(k < q ? k : 0);
                    }
                }
            }
            final_time = __shfl(result, (q - 1) & (kWave - 1), kWave);
        }
        if (lane == 0) {                  // the only lane-dependent branch of the loop body
            if (rerun) {
                retry[atomicAdd(&plan->class_count[kRetryClass], 1)] = static_cast<int32_t>(ci);
            } else {
                if (sched.T_greedy) static_cast<T *>(sched.T_greedy)[ci] = final_time;
                if (sched.cfg_status) sched.cfg_status[ci] = status;
            }
        }
        __syncthreads();
    }
}

hipError_t launch_uni_pipe_sched(const UniLaunch &L, int32_t *retry)
{
    if (L.cost == PRS_COST_I64)
        hipLaunchKernelGGL((uni_pipe_sched_kernel<int64_t>), dim3(L.grid), dim3(kWave), uni_pipe_sched_lds_bytes(), L.stream, L.cfg,
                           L.p_max, L.q_max, L.sched, L.plan, L.order, L.cls, retry, L.slots, L.slot_bytes, L.slot_p);
    else
        hipLaunchKernelGGL((uni_pipe_sched_kernel<double>), dim3(L.grid), dim3(kWave), uni_pipe_sched_lds_bytes(), L.stream, L.cfg,
                           L.p_max, L.q_max, L.sched, L.plan, L.order, L.cls, retry, L.slots, L.slot_bytes, L.slot_p);
    return hipGetLastError();
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
