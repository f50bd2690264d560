// Bi-greedy schedules (Lowery & Langou, Algorithm 2, Section 6.2) on gfx950.
//
// One 64-lane wavefront runs one configuration.  Algorithm 2 walks over time;
// at each time t it visits the segments from the first unfinished one upwards
// and, per segment j, builds three index lists over the processors that still
// hold j and are not excluded by a computation: send port free only, receive
// port free only, both free.  The processors with both ports free are dealt
// to the shorter list (first entries receive, last entries send), the first
// l = min(#send, #recv) entries are paired entry by entry, and the ports and
// the pending computation of the paired processors are updated.
//
// Here every list is a bit set over the processors (64 per machine word), so
// one lane classifies 64 processors with a few logic operations, list lengths
// are population counts, "first k entries" is a rank select inside a word and
// list positions come from wavefront prefix sums.  The unit time step is
// replaced by a jump to the next time a send or receive port frees: no new
// pair can form in between.  Segments in which every processor has sent, and
// visits after the last free send or receive port is used up, are skipped:
// they cannot produce a pair.
//
// A processor's computation interval [C1, C2) always ends when its receive
// port frees, so C2 is not stored separately.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

__host__ __device__ inline size_t bi_align(size_t v) { return (v + 255) / 256 * 256; }

// Small arrays of a configuration: bit sets, list positions, pairing lists, per-segment counters.
struct BiSmall {
    size_t masks, pref, sendList, recvList, rem, total;
    int W;
};

__host__ __device__ inline BiSmall bi_small_layout(int32_t p_cap, int32_t q_cap)
{
    BiSmall L;
    const size_t p = static_cast<size_t>(p_cap), q = static_cast<size_t>(q_cap);
    L.W = static_cast<int>((p + 63) / 64);
    size_t o = 0;
    L.masks = o; o += bi_align(static_cast<size_t>(L.W) * 8 * 7);   // 7 word arrays
    L.pref = o; o += bi_align(static_cast<size_t>(L.W) * 4 * 2);
    L.sendList = o; o += bi_align((p / 2 + 1) * 4);
    L.recvList = o; o += bi_align((p / 2 + 1) * 4);
    L.rem = o; o += bi_align(q * 4);
    L.total = o;
    return L;
}

// Per-processor times and counters: always in the block's workspace slot.
struct BiBig { size_t S, R, C1, nsent, total; };

__host__ __device__ inline BiBig bi_big_layout(int32_t p_cap)
{
    BiBig L;
    const size_t p = static_cast<size_t>(p_cap);
    size_t o = 0;
    L.S = o; o += bi_align(p * 8);
    L.R = o; o += bi_align(p * 8);
    L.C1 = o; o += bi_align(p * 8);
    L.nsent = o; o += bi_align(p * 4);
    L.total = o;
    return L;
}

size_t bi_small_bytes(int32_t p_cap, int32_t q_cap) { return bi_small_layout(p_cap, q_cap).total; }
// The bit sets and list positions alone (the first two arrays of the small layout): what every pass of a visit
// reads and writes.  They can sit in LDS when the lists and counters no longer fit beside them.
size_t bi_masks_bytes(int32_t p_cap) { return bi_small_layout(p_cap, 1).sendList; }
__host__ __device__ inline size_t bi_bitmap_size(int32_t p_cap, int32_t q_cap)
{
    return bi_align(static_cast<size_t>((p_cap + 63) / 64) * static_cast<size_t>(q_cap) * 8);
}
size_t bi_bitmap_bytes(int32_t p_cap, int32_t q_cap) { return bi_bitmap_size(p_cap, q_cap); }
size_t bi_slot_bytes(int32_t p_cap, int32_t q_cap, bool small_in_lds)
{
    return bi_big_layout(p_cap).total + bi_bitmap_size(p_cap, q_cap) + (small_in_lds ? 0 : bi_small_bytes(p_cap, q_cap));
}

struct BiState {
    char *small;         // BiSmall arrays (LDS or slot)
    char *masks;         // the bit sets and list positions of BiSmall, if they are kept apart from the rest (LDS); else null
    char *big;           // BiBig arrays (slot)
    uint64_t *sent;      // [q][W] bitmap (LDS if it fits, else slot)
    int Wcap;            // words per mask array as laid out
    BiSmall sl;
    BiBig bl;
};

template <typename T, bool kSched>
__device__ T run_bi(const Config<T> &c, const BiState &bs, const SchedOut &sched, int64_t out_base, int32_t *status)
{
    const int lane = lane_id();
    const int p = c.p, q = c.q;
    const int W = (p + 63) >> 6;                        // words in use
    T *S = reinterpret_cast<T *>(bs.big + bs.bl.S);
    T *R = reinterpret_cast<T *>(bs.big + bs.bl.R);
    T *C1 = reinterpret_cast<T *>(bs.big + bs.bl.C1);
    int32_t *nsent = reinterpret_cast<int32_t *>(bs.big + bs.bl.nsent);
    char *mbase = bs.masks ? bs.masks : bs.small;       // masks and pref have the same offsets in either place
    uint64_t *mk = reinterpret_cast<uint64_t *>(mbase + bs.sl.masks);
    const int Wc = bs.Wcap;
    uint64_t *sfree = mk, *rfree = mk + Wc, *compF = mk + 2 * Wc, *compL = mk + 3 * Wc;
    uint64_t *sendSet = mk + 4 * Wc, *recvSet = mk + 5 * Wc;
    uint64_t *lateL = mk + 6 * Wc;                      // senders whose send outlasts a transfer of the smaller last segment begun now
    // nsent[i] also carries the kind of i's latest transfers: bit 30 = it last sent the smaller last segment,
    // bit 29 = it last received it
    constexpr int32_t kSentShort = 1 << 30, kRecvShort = 1 << 29, kCount = kRecvShort - 1;
    const bool ragged = c.sz_last != c.sz, guardL = ragged && c.g_last > 0;
    int32_t *prefS = reinterpret_cast<int32_t *>(mbase + bs.sl.pref), *prefR = prefS + Wc;
    int32_t *sendList = reinterpret_cast<int32_t *>(bs.small + bs.sl.sendList);
    int32_t *recvList = reinterpret_cast<int32_t *>(bs.small + bs.sl.recvList);
    int32_t *rem = reinterpret_cast<int32_t *>(bs.small + bs.sl.rem);
    uint64_t *sent = bs.sent;                           // [q][W]

    for (int i = lane; i < p; i += kWave) { S[i] = 0; R[i] = 0; C1[i] = 0; nsent[i] = 0; }
    for (int j = lane; j < q; j += kWave) rem[j] = p - 1;
    for (int64_t k = lane; k < static_cast<int64_t>(q) * W; k += kWave) sent[k] = 0;
    __syncthreads();

    const T kInf = CostTraits<T>::inf();
    T t = 0, Tmax = 0;
    int ndone = 0, segStart = 0;
    int64_t emitted = 0;
    const int64_t max_events = 4 * static_cast<int64_t>(p) * q + 16;
    for (int64_t ev = 0;; ++ev) {
        if (ev > max_events) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
        // ---- port and computation state of every processor at time t, as bit sets
        T minOld = kInf, minLate = kInf;             // next time a port frees / a processor may take in the smaller last segment
        int cs = 0, cr = 0, cu = 0;                  // free send ports, free receive ports, processors with either
        int csAll = 0;                               // free send ports of processors with something left to send
        // (four words of processors per round: their loads are issued together, ahead of the ballots and stores)
        for (int w4 = 0; w4 < W; w4 += 4) {
            T s4[4], r4[4], c4[4];
            int32_t n4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = (w4 + u) * kWave + lane;
                const bool in = i < p;
                s4[u] = in ? S[i] : 0; r4[u] = in ? R[i] : 0; c4[u] = in ? C1[i] : 0;
                n4[u] = in ? nsent[i] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int w = w4 + u;
                const int i = w * kWave + lane;
                const bool in = i < p;
                const T s = s4[u], r = r4[u], c1 = c4[u];
                const int32_t nsnt = n4[u];
                const bool live = in && (i == 0 || (nsnt & kCount) < q);   // still a member of some segment
                const bool sf = live && i != 0 && s <= t;              // the root never sends
                const bool rf = live && r <= t;
                const bool busy = in && c1 <= t && t < r;              // computing now
                const bool pend = in && t < c1;                        // computation scheduled ahead
                // A transfer begun now must not run into that computation.  It was scheduled before t: against a
                // segment of its own size that settles it (comparing the two rounded sums could miss it by one
                // rounding error); against the other size the sums are compared.
                const bool rshort = (nsnt & kRecvShort) != 0;
                const bool cF = busy || (pend && (!rshort || t + c.c_full > c1));
                const bool cL = busy || (pend && (rshort || !ragged || t + c.c_last > c1));
                // Section 2 the other way round: the combine of the smaller last segment, received now, would begin
                // while this processor is still sending a full one; it becomes eligible at s - tcomm(last)
                const bool lt = in && guardL && !(nsnt & kSentShort) && s > t + c.c_last;
                if (in && s > t && s < minOld) minOld = s;
                if (in && r > t && r < minOld) minOld = r;
                if (lt) { const T v = s - c.c_last; if (v > t && v < minLate) minLate = v; }
                const uint64_t bsf = ballot64(sf), brf = ballot64(rf), bcF = ballot64(cF), bcL = ballot64(cL), blt = ballot64(lt);
                if (lane == 0 && w < W) { sfree[w] = bsf; rfree[w] = brf; compF[w] = bcF; compL[w] = bcL; lateL[w] = blt; }
                cs += __popcll(bsf & ~bcL);
                cr += __popcll(brf & ~bcL);
                cu += __popcll((bsf | brf) & ~bcL);
                csAll += __popcll(bsf);
            }
        }
        minOld = wave_min(minOld);
        minLate = wave_min(minLate);
        __syncthreads();
        T minNew = kInf, minNewLate = kInf;
        while (segStart < q && rem[segStart] == 0) ++segStart;
        for (int j = segStart; j < q; ++j) {
            // no further pair can form at this t: a pair needs a free send port and a free receive port on two
            // different processors (a single processor left over with both ports free would otherwise be
            // offered every remaining segment in vain)
            if (cs == 0 || cr == 0 || cu < 2) break;
            int remj = rem[j];
            if (remj == 0) continue;                     // everybody has sent segment j
            const bool last = j == q - 1;
            const T cj = last ? c.c_last : c.c_full, gj = last ? c.g_last : c.g_full;
            // ---- pass A: the three lists of this visit as bit sets, and their lengths
            int ns_ = 0, nr_ = 0, nf_ = 0;
            for (int w0 = 0; w0 < W; w0 += kWave) {
                const int w = w0 + lane;
                if (w < W) {
                    uint64_t valid = ~UINT64_C(0);
                    if (w == W - 1 && (p & 63)) valid = (UINT64_C(1) << (p & 63)) - 1;
                    const uint64_t memb = ~sent[static_cast<size_t>(j) * W + w] & valid;
                    const uint64_t comp = last ? compL[w] : compF[w];
                    const uint64_t sOK = memb & ~comp & sfree[w], rOK = memb & ~comp & rfree[w] & ~(last ? lateL[w] : UINT64_C(0));
                    const uint64_t fr = sOK & rOK, so = sOK ^ fr, ro = rOK ^ fr;
                    ns_ += __popcll(so); nr_ += __popcll(ro); nf_ += __popcll(fr);
                }
            }
            ns_ = wave_sum(ns_); nr_ = wave_sum(nr_); nf_ = wave_sum(nf_);
            // ---- processors with both ports free go to the shorter list
            int toSendLast, toRecvFirst;
            if (ns_ == nr_) {
                toSendLast = toRecvFirst = nf_ / 2;
            } else if (ns_ < nr_) {
                const int y = nr_ - ns_, mm = nf_ < y ? nf_ : y, xx = (nf_ - mm) / 2;
                toSendLast = mm + xx; toRecvFirst = xx;
            } else {
                const int y = ns_ - nr_, mm = nf_ < y ? nf_ : y, xx = (nf_ - mm) / 2;
                toRecvFirst = mm + xx; toSendLast = xx;
            }
            const int sN = ns_ + toSendLast, rN = nr_ + toRecvFirst;
            const int l = sN < rN ? sN : rN;
            if (l == 0) continue;
            // ---- pass B: final send and receive sets (first l of each), word by word with running ranks
            int carryF = 0, carryS = 0, carryR = 0, gone = 0;
            for (int w0 = 0; w0 < W; w0 += kWave) {
                const int w = w0 + lane;
                const bool on = w < W;
                uint64_t fr = 0, so = 0, ro = 0;                          // the three lists of pass A again (nothing has changed)
                if (on) {
                    uint64_t valid = ~UINT64_C(0);
                    if (w == W - 1 && (p & 63)) valid = (UINT64_C(1) << (p & 63)) - 1;
                    const uint64_t memb = ~sent[static_cast<size_t>(j) * W + w] & valid;
                    const uint64_t comp = last ? compL[w] : compF[w];
                    const uint64_t sOK = memb & ~comp & sfree[w], rOK = memb & ~comp & rfree[w] & ~(last ? lateL[w] : UINT64_C(0));
                    fr = sOK & rOK; so = sOK ^ fr; ro = rOK ^ fr;
                }
                const int pf = __popcll(fr);
                const int incF = wave_inclusive_scan(pf);
                const int exF = carryF + incF - pf;                       // free-list rank of this word's first entry
                const uint64_t frR = lowest_bits(fr, toRecvFirst - exF);
                const uint64_t frS = highest_bits(fr, exF + pf - (nf_ - toSendLast));
                uint64_t sset = so | frS, rset = ro | frR;
                const int ps = __popcll(sset), pr = __popcll(rset);
                const int incS = wave_inclusive_scan(ps), incR = wave_inclusive_scan(pr);
                const int exS = carryS + incS - ps, exR = carryR + incR - pr;
                sset = lowest_bits(sset, l - exS);
                rset = lowest_bits(rset, l - exR);
                if (on) {
                    sendSet[w] = sset; recvSet[w] = rset; prefS[w] = exS; prefR[w] = exR;
                    sent[static_cast<size_t>(j) * W + w] |= sset;
                    const uint64_t sf0 = sfree[w], rf0 = rfree[w], open = ~compL[w];
                    sfree[w] = sf0 & ~sset;
                    rfree[w] = rf0 & ~rset;
                    gone += __popcll((sf0 | rf0) & open) - __popcll(((sf0 & ~sset) | (rf0 & ~rset)) & open);
                }
                carryF += __shfl(incF, kWave - 1, kWave);
                carryS += __shfl(incS, kWave - 1, kWave);
                carryR += __shfl(incR, kWave - 1, kWave);
            }
            __syncthreads();
            // ---- pass C: bit sets -> index lists in ascending processor order
            // (every lane looks at one word of 64, and only the words that hold a sender or receiver are expanded:
            // with thousands of processors most words of a visit are empty)
            for (int w0 = 0; w0 < W; w0 += kWave) {
                const int wl = w0 + lane;
                uint64_t some = ballot64(wl < W && (sendSet[wl] | recvSet[wl]) != 0);
                while (some != 0) {
                    const int w = w0 + __builtin_ctzll(some);
                    some &= some - 1;
                    const uint64_t ss = sendSet[w], rs = recvSet[w];
                    if ((ss >> lane) & 1) sendList[prefS[w] + rank_below(ss)] = w * kWave + lane;
                    if ((rs >> lane) & 1) recvList[prefR[w] + rank_below(rs)] = w * kWave + lane;
                }
            }
            __syncthreads();
            // ---- pass D: entry-wise pairing
            const T tc = t + cj, tr = tc + gj;
            if (!(tc > t)) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
            const bool shortNow = last && ragged;
            for (int e = lane; e < l; e += kWave) {
                const int32_t a = sendList[e], b = recvList[e];        // no processor is in both lists of a visit
                S[a] = tc;
                nsent[a] = (((nsent[a] & kCount) + 1) | (nsent[a] & kRecvShort)) | (shortNow ? kSentShort : 0);
                nsent[b] = (nsent[b] & ~kRecvShort) | (shortNow ? kRecvShort : 0);
                R[b] = tr;
                C1[b] = tc;
                if (kSched) {
                    const int64_t o = out_base + emitted + e;
                    if (sched.src) sched.src[o] = a;
                    if (sched.dst) sched.dst[o] = b;
                    if (sched.seg) sched.seg[o] = j;
                    if (sched.tstart) static_cast<T *>(sched.tstart)[o] = t;
                }
            }
            emitted += l;
            if (tc < minNew) minNew = tc;
            if (tr < minNew) minNew = tr;
            if (guardL && !last && tc > t + c.c_last) {           // these senders cannot take the last segment in yet
                for (int w0 = 0; w0 < W; w0 += kWave)
                    if (w0 + lane < W) lateL[w0 + lane] |= sendSet[w0 + lane];
                const T v = tc - c.c_last;
                if (v > t && v < minNewLate) minNewLate = v;
            }
            cs -= l; cr -= l; csAll -= l;
            cu -= wave_sum(gone);
            remj -= l;
            if (lane == 0) rem[j] = remj;
            if (remj == 0) {                              // only the root is left: it finishes after the last arrival
                if (tr > Tmax) Tmax = tr;
                ++ndone;
            }
            __syncthreads();
        }
        if (ndone == q) break;
        T tn = minOld < minNew ? minOld : minNew;
        // The instants at which a sender may take in the last segment count only if a processor with something left to
        // send has a free send port: otherwise nothing can pair before a port frees.
        const T tl = minLate < minNewLate ? minLate : minNewLate;
        if (csAll > 0 && tl < tn) tn = tl;
        if (!(tn < kInf)) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
        t = tn;
    }
    return Tmax;
}

// kPlace: 0 = all arrays of a configuration in its workspace slot, 1 = the small arrays (and, if it fits, the sent
// bitmap) in LDS, 2 = only the bit sets and list positions in LDS (tens of thousands of processors).
template <typename T, bool kSched, int kPlace>
__global__ __launch_bounds__(kWave) void bi_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model, TimesOut times,
                                                   SchedOut sched, PlanHeader *plan, const int32_t *order, int cls,
                                                   int32_t state_p, int32_t state_q, int32_t lds_bitmap_bytes, char *slots,
                                                   size_t slot_bytes)
{
    PRS_DYNAMIC_LDS(lds_raw);
    const int lane = lane_id();
    char *slot = slots + static_cast<size_t>(blockIdx.x) * slot_bytes;
    BiState bs;
    bs.sl = bi_small_layout(state_p, state_q);
    bs.bl = bi_big_layout(state_p);
    bs.Wcap = bs.sl.W;
    bs.big = slot;
    uint64_t *slot_bitmap = reinterpret_cast<uint64_t *>(slot + bs.bl.total);
    constexpr bool kLds = kPlace == 1;
    bs.small = kLds ? lds_raw : slot + bs.bl.total + bi_bitmap_size(state_p, state_q);
    bs.masks = kPlace == 2 ? lds_raw : nullptr;
    uint64_t *lds_bitmap = reinterpret_cast<uint64_t *>(lds_raw + bs.sl.total);
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    for (;;) {
        const int64_t ticket = next_ticket(&plan->ticket[cls]);
        if (ticket >= count) break;
        const int64_t i = order[begin + ticket];
        Config<T> c = decode_config<T>(cfg, i, p_max, q_max);
        int32_t status = c.status;
        int64_t base = 0;
        if (kSched && status == PRS_CFG_OK) {
            base = sched.pair_offset[i];
            const int64_t cnt = static_cast<int64_t>(c.p - 1) * c.q;
            if (base < 0 || base + cnt > sched.pair_capacity) status = PRS_CFG_TOO_LARGE;
        }
        T result = CostTraits<T>::bad();
        if (status == PRS_CFG_OK) {
            const int64_t bitmap_bytes = static_cast<int64_t>((c.p + 63) >> 6) * c.q * 8;
            bs.sent = (kLds && bitmap_bytes <= lds_bitmap_bytes) ? lds_bitmap : slot_bitmap;
            result = run_bi<T, kSched>(c, bs, sched, base, &status);
        }
        __syncthreads();
        if (lane == 0) {                  // the only lane-dependent branch of the loop body
            if (!kSched) write_closed_forms<T>(times, i, c, model);
            T *tg = static_cast<T *>(kSched ? sched.T_greedy : times.greedy);
            int32_t *cs = kSched ? sched.cfg_status : times.cfg_status;
            if (tg) tg[i] = status == PRS_CFG_OK ? result : CostTraits<T>::bad();
            if (cs) cs[i] = status;
        }
        __syncthreads();
    }
}

template <typename T, bool kSched>
static hipError_t launch_bi_t(const BiLaunch &L)
{
    if (L.lds_p > 0)
        hipLaunchKernelGGL((bi_kernel<T, kSched, 1>), dim3(L.grid), dim3(kWave), L.lds_bytes, L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.sched, L.plan, L.order, L.cls, L.slot_p, L.slot_q, L.lds_bitmap_bytes, L.slots,
                           L.slot_bytes);
    else if (L.lds_bytes > 0)                                     // the caller sized it with bi_masks_bytes(slot_p)
        hipLaunchKernelGGL((bi_kernel<T, kSched, 2>), dim3(L.grid), dim3(kWave), L.lds_bytes, L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.sched, L.plan, L.order, L.cls, L.slot_p, L.slot_q, 0, L.slots, L.slot_bytes);
    else
        hipLaunchKernelGGL((bi_kernel<T, kSched, 0>), dim3(L.grid), dim3(kWave), 0, L.stream, L.cfg, L.p_max, L.q_max,
                           L.model, L.times, L.sched, L.plan, L.order, L.cls, L.slot_p, L.slot_q, 0, L.slots, L.slot_bytes);
    return hipGetLastError();
}

hipError_t launch_bi(const BiLaunch &L)
{
    if (L.cost == PRS_COST_I64) return L.want_schedule ? launch_bi_t<int64_t, true>(L) : launch_bi_t<int64_t, false>(L);
    return L.want_schedule ? launch_bi_t<double, true>(L) : launch_bi_t<double, false>(L);
}

}  // namespace prs
