// Bi-greedy schedules (Lowery & Langou, Algorithm 2, Section 6.2) for machines of thousands of processors on
// gfx950: one block of 16 wavefronts per configuration.
//
// The same sequence of set operations as the one-wavefront kernel (every list of Algorithm 2 a bit set over the
// processors, list lengths population counts, "first k entries" a rank select inside a word, list positions from
// prefix sums), with the words of the bit sets and the processors spread over the 1024 threads of a block:
// thread w owns word w of every set, the per-processor times are read 1024 at a time, sums and prefix sums go
// through the wavefronts and then through LDS.  The bit sets of a visit sit in LDS (7 sets of up to 1024 words),
// the per-processor times, the pairing lists, the per-segment counters and the sent bitmap in the block's
// workspace slot.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kBlockThreads = 1024;
constexpr int kBlockWaves = kBlockThreads / kWave;

__host__ __device__ inline size_t bb_align(size_t v) { return (v + 255) / 256 * 256; }

// workspace slot of a block: S, R, C1 (8 B per processor), flags and count of sent segments (4 B), the two pairing
// lists, the per-segment counters, the sent bitmap [q][W]
struct BlockSlot { size_t S, R, C1, nsent, sendList, recvList, rem, sent, total; };

__host__ __device__ inline BlockSlot bi_block_slot(int32_t p_cap, int32_t q_cap)
{
    BlockSlot L;
    const size_t p = static_cast<size_t>(p_cap), q = static_cast<size_t>(q_cap), W = (p + 63) / 64;
    size_t o = 0;
    L.S = o; o += bb_align(p * 8);
    L.R = o; o += bb_align(p * 8);
    L.C1 = o; o += bb_align(p * 8);
    L.nsent = o; o += bb_align(p * 4);
    L.sendList = o; o += bb_align((p / 2 + 1) * 4);
    L.recvList = o; o += bb_align((p / 2 + 1) * 4);
    L.rem = o; o += bb_align(q * 4);
    L.sent = o; o += bb_align(W * q * 8);
    L.total = o;
    return L;
}

size_t bi_block_slot_bytes(int32_t p_cap, int32_t q_cap) { return bi_block_slot(p_cap, q_cap).total; }
// LDS: 7 bit sets and 2 arrays of 16-bit list positions of Wcap words, then the scratch of the block-wide sums
size_t bi_block_lds_bytes(int32_t p_cap)
{
    const size_t W = (static_cast<size_t>(p_cap) + 63) / 64;
    return bb_align(W * 8 * 7) + bb_align(W * 2 * 2) + 1024;
}

struct BlockScratch {
    int32_t *part;       // [3][kBlockWaves] partial sums of the wavefronts
    double *tpart;       // [kBlockWaves] partial minima (bit patterns of T)
};

// sums of three values over the block (the same result in every thread)
__device__ __forceinline__ void block_sum3(const BlockScratch &bs, int &a, int &b, int &c)
{
    const int lane = lane_id(), wave = static_cast<int>(threadIdx.x) >> 6;
    a = wave_sum(a); b = wave_sum(b); c = wave_sum(c);
    __syncthreads();                                             // earlier readers of the scratch are through
    if (lane == 0) { bs.part[wave] = a; bs.part[kBlockWaves + wave] = b; bs.part[2 * kBlockWaves + wave] = c; }
    __syncthreads();
    int sa = 0, sb = 0, sc = 0;
#pragma unroll
    for (int w = 0; w < kBlockWaves; ++w) { sa += bs.part[w]; sb += bs.part[kBlockWaves + w]; sc += bs.part[2 * kBlockWaves + w]; }
    a = sa; b = sb; c = sc;
}

// exclusive prefix sums of two values over the threads of the block, and their totals
__device__ __forceinline__ void block_scan2(const BlockScratch &bs, int a, int b, int &exA, int &exB, int &totA, int &totB)
{
    const int lane = lane_id(), wave = static_cast<int>(threadIdx.x) >> 6;
    const int incA = wave_inclusive_scan(a), incB = wave_inclusive_scan(b);
    __syncthreads();
    if (lane == kWave - 1) { bs.part[wave] = incA; bs.part[kBlockWaves + wave] = incB; }
    __syncthreads();
    int beforeA = 0, beforeB = 0, sa = 0, sb = 0;
#pragma unroll
    for (int w = 0; w < kBlockWaves; ++w) {
        const int va = bs.part[w], vb = bs.part[kBlockWaves + w];
        if (w < wave) { beforeA += va; beforeB += vb; }
        sa += va; sb += vb;
    }
    exA = beforeA + incA - a; exB = beforeB + incB - b;
    totA = sa; totB = sb;
}

template <typename T> __device__ __forceinline__ T block_min(const BlockScratch &bs, T v)
{
    const int lane = lane_id(), wave = static_cast<int>(threadIdx.x) >> 6;
    v = wave_min<T>(v);
    T *tp = reinterpret_cast<T *>(bs.tpart);
    __syncthreads();
    if (lane == 0) tp[wave] = v;
    __syncthreads();
    T m = tp[0];
#pragma unroll
    for (int w = 1; w < kBlockWaves; ++w) { const T u = tp[w]; m = u < m ? u : m; }
    return m;
}

template <typename T, bool kSched>
__device__ T run_bi_block(const Config<T> &c, char *lds, char *slot, const BlockSlot &sl, int Wc, const SchedOut &sched,
                          int64_t out_base, int32_t *status)
{
    const int tid = static_cast<int>(threadIdx.x), lane = lane_id(), wave = tid >> 6;
    const int p = c.p, q = c.q;
    const int W = (p + 63) >> 6;
    T *S = reinterpret_cast<T *>(slot + sl.S);
    T *R = reinterpret_cast<T *>(slot + sl.R);
    T *C1 = reinterpret_cast<T *>(slot + sl.C1);
    int32_t *nsent = reinterpret_cast<int32_t *>(slot + sl.nsent);
    int32_t *sendList = reinterpret_cast<int32_t *>(slot + sl.sendList);
    int32_t *recvList = reinterpret_cast<int32_t *>(slot + sl.recvList);
    int32_t *rem = reinterpret_cast<int32_t *>(slot + sl.rem);
    uint64_t *sent = reinterpret_cast<uint64_t *>(slot + sl.sent);           // [q][W]
    uint64_t *mk = reinterpret_cast<uint64_t *>(lds);
    uint64_t *sfree = mk, *rfree = mk + Wc, *compF = mk + 2 * Wc, *compL = mk + 3 * Wc;
    uint64_t *sendSet = mk + 4 * Wc, *recvSet = mk + 5 * Wc, *lateL = mk + 6 * Wc;
    // list positions of a word's first sender and receiver: below 2^16, a list has at most p/2 <= 32768 entries
    uint16_t *prefS = reinterpret_cast<uint16_t *>(lds + bb_align(static_cast<size_t>(Wc) * 8 * 7)), *prefR = prefS + Wc;
    BlockScratch bs;
    bs.part = reinterpret_cast<int32_t *>(lds + bb_align(static_cast<size_t>(Wc) * 8 * 7) + bb_align(static_cast<size_t>(Wc) * 2 * 2));
    bs.tpart = reinterpret_cast<double *>(bs.part + 3 * kBlockWaves + 16);
    // nsent[i] also carries the kind of i's latest transfers: bit 30 = it last sent the smaller last segment,
    // bit 29 = it last received it
    constexpr int32_t kSentShort = 1 << 30, kRecvShort = 1 << 29, kCount = kRecvShort - 1;
    const bool ragged = c.sz_last != c.sz, guardL = ragged && c.g_last > 0;

    for (int i = tid; i < p; i += kBlockThreads) { S[i] = 0; R[i] = 0; C1[i] = 0; nsent[i] = 0; }
    for (int j = tid; j < q; j += kBlockThreads) rem[j] = p - 1;
    for (int64_t k = tid; k < static_cast<int64_t>(q) * W; k += kBlockThreads) sent[k] = 0;
    __syncthreads();

    const T kInf = CostTraits<T>::inf();
    T t = 0, Tmax = 0;
    int ndone = 0, segStart = 0;
    int64_t emitted = 0;
    bool lateOnly = false;
    const int64_t max_events = 4 * static_cast<int64_t>(p) * q + 16;
    for (int64_t ev = 0;; ++ev) {
        if (ev > max_events) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
        // ---- port and computation state of every processor at time t, as bit sets (wavefront v takes words v, v+16, ...)
        T minOld = kInf, minLate = kInf;             // next time a port frees / a processor may take in the last segment
        int cs = 0, cr = 0, cu = 0;                  // free send ports, free receive ports, processors with either
        int csAll = 0;                               // free send ports of processors with something left to send
        for (int w = wave; w < W; w += kBlockWaves) {
            const int i = w * kWave + lane;
            const bool in = i < p;
            const T s = in ? S[i] : 0, r = in ? R[i] : 0, c1 = in ? C1[i] : 0;
            const int32_t nsnt = in ? nsent[i] : 0;
            const bool live = in && (i == 0 || (nsnt & kCount) < q);   // still a member of some segment
            const bool sf = live && i != 0 && s <= t;              // the root never sends
            const bool rf = live && r <= t;
            const bool busy = in && c1 <= t && t < r;              // computing now
            const bool pend = in && t < c1;                        // computation scheduled ahead
            // A transfer begun now must not run into that computation.  It was scheduled before t: against a segment
            // of its own size that settles it; against the other size the rounded sums are compared.
            const bool rshort = (nsnt & kRecvShort) != 0;
            const bool cF = busy || (pend && (!rshort || t + c.c_full > c1));
            const bool cL = busy || (pend && (rshort || !ragged || t + c.c_last > c1));
            // Section 2 the other way round: the combine of the smaller last segment, received now, would begin while
            // this processor is still sending a full one; it becomes eligible at s - tcomm(last)
            const bool lt = in && guardL && !(nsnt & kSentShort) && s > t + c.c_last;
            if (in && s > t && s < minOld) minOld = s;
            if (in && r > t && r < minOld) minOld = r;
            if (lt) { const T v = s - c.c_last; if (v > t && v < minLate) minLate = v; }
            const uint64_t bsf = ballot64(sf), brf = ballot64(rf), bcF = ballot64(cF), bcL = ballot64(cL), blt = ballot64(lt);
            if (lane == 0) {
                sfree[w] = bsf; rfree[w] = brf; compF[w] = bcF; compL[w] = bcL; lateL[w] = blt;
                cs += __popcll(bsf & ~bcL);
                cr += __popcll(brf & ~bcL);
                cu += __popcll((bsf | brf) & ~bcL);
                csAll += __popcll(bsf);
            }
        }
        minOld = block_min<T>(bs, minOld);
        if (guardL) minLate = block_min<T>(bs, minLate);
        block_sum3(bs, cs, cr, cu);                   // also makes the bit sets visible to every thread
        { int z0 = 0, z1 = 0; block_sum3(bs, csAll, z0, z1); }
        T minNew = kInf, minNewLate = kInf;
        while (segStart < q && rem[segStart] == 0) ++segStart;
        // At a time at which no port frees the candidates of every segment but the last have only become fewer
        // since the event before: only the last segment is visited.
        for (int j = (lateOnly && segStart < q - 1) ? q - 1 : segStart; j < q; ++j) {
            // no further pair can form at this t: a pair needs a free send port and a free receive port on two
            // different processors
            if (cs == 0 || cr == 0 || cu < 2) break;
            int remj = rem[j];
            if (remj == 0) continue;                     // everybody has sent segment j
            const bool last = j == q - 1;
            const T cj = last ? c.c_last : c.c_full, gj = last ? c.g_last : c.g_full;
            // ---- pass A: the three lists of this visit as bit sets (thread w owns word w), and their lengths
            int ns_ = 0, nr_ = 0, nf_ = 0, cand_sent = 0;
            for (int w = tid; w < W; w += kBlockThreads) {
                uint64_t valid = ~UINT64_C(0);
                if (w == W - 1 && (p & 63)) valid = (UINT64_C(1) << (p & 63)) - 1;
                const uint64_t row = sent[static_cast<size_t>(j) * W + w];
                const uint64_t memb = ~row & valid;
                const uint64_t comp = last ? compL[w] : compF[w];
                const uint64_t sOK = memb & ~comp & sfree[w], rOK = memb & ~comp & rfree[w] & ~(last ? lateL[w] : UINT64_C(0));
                const uint64_t fr = sOK & rOK, so = sOK ^ fr, ro = rOK ^ fr;
                ns_ += __popcll(so); nr_ += __popcll(ro); nf_ += __popcll(fr);
                cand_sent += ((sfree[w] | rfree[w]) & ~comp & row & valid) != 0 ? 1 : 0;
            }
            block_sum3(bs, ns_, nr_, nf_);
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
            if (l == 0) {
                // nobody paired although no candidate had already sent j: the candidates of later segments are a
                // subset of these, so none of them can pair at this t either -- except the last segment, whose
                // shorter transfer is kept out by fewer pending computations
                int z0 = 0, z1 = 0;
                block_sum3(bs, cand_sent, z0, z1);
                if (cand_sent == 0) {
                    if (last) break;
                    j = q - 2;                               // go on with the last segment
                }
                continue;
            }
            // ---- pass B: final send and receive sets (first l of each), word by word with running ranks
            int carryF = 0, carryS = 0, carryR = 0, gone = 0;
            for (int w0 = 0; w0 < W; w0 += kBlockThreads) {
                const int w = w0 + tid;
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
                int exF, exDummy, totF, totDummy;
                block_scan2(bs, pf, 0, exF, exDummy, totF, totDummy);
                exF += carryF;                                            // free-list rank of this word's first entry
                const uint64_t frR = lowest_bits(fr, toRecvFirst - exF);
                const uint64_t frS = highest_bits(fr, exF + pf - (nf_ - toSendLast));
                uint64_t sset = so | frS, rset = ro | frR;
                const int ps = __popcll(sset), pr = __popcll(rset);
                int exS, exR, totS, totR;
                block_scan2(bs, ps, pr, exS, exR, totS, totR);
                exS += carryS; exR += carryR;
                sset = lowest_bits(sset, l - exS);
                rset = lowest_bits(rset, l - exR);
                if (on) {
                    sendSet[w] = sset; recvSet[w] = rset;
                    prefS[w] = static_cast<uint16_t>(exS < 65535 ? exS : 65535);       // words past the l-th entry hold nobody
                    prefR[w] = static_cast<uint16_t>(exR < 65535 ? exR : 65535);
                    sent[static_cast<size_t>(j) * W + w] |= sset;
                    const uint64_t sf0 = sfree[w], rf0 = rfree[w], open = ~compL[w];
                    sfree[w] = sf0 & ~sset;
                    rfree[w] = rf0 & ~rset;
                    gone += __popcll((sf0 | rf0) & open) - __popcll(((sf0 & ~sset) | (rf0 & ~rset)) & open);
                }
                carryF += totF; carryS += totS; carryR += totR;
            }
            __syncthreads();
            // ---- pass C: bit sets -> index lists in ascending processor order (a wavefront expands one word at a time,
            // only the words that hold a sender or a receiver)
            for (int w0 = wave * kWave; w0 < W; w0 += kBlockThreads) {
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
            __threadfence_block();
            __syncthreads();
            // ---- pass D: entry-wise pairing
            const T tc = t + cj, tr = tc + gj;
            if (!(tc > t)) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
            const bool shortNow = last && ragged;
            for (int e = tid; e < l; e += kBlockThreads) {
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
                for (int w = tid; w < W; w += kBlockThreads) lateL[w] |= sendSet[w];
                const T v = tc - c.c_last;
                if (v > t && v < minNewLate) minNewLate = v;
            }
            cs -= l; cr -= l; csAll -= l;
            int g0 = 0, g1 = 0;
            block_sum3(bs, gone, g0, g1);
            cu -= gone;
            remj -= l;
            if (tid == 0) rem[j] = remj;
            if (remj == 0) {                              // only the root is left: it finishes after the last arrival
                if (tr > Tmax) Tmax = tr;
                ++ndone;
            }
            __threadfence_block();
            __syncthreads();
        }
        if (ndone == q) break;
        T tn = minOld < minNew ? minOld : minNew;
        const T tl = minLate < minNewLate ? minLate : minNewLate;
        // without a free send port on a processor that still has something to send nothing can pair before a port frees
        lateOnly = csAll > 0 && tl < tn;
        if (lateOnly) tn = tl;
        if (!(tn < kInf)) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }
        t = tn;
        __threadfence_block();
        __syncthreads();                              // the pairs of this event are in S, R, C1 before the next state pass
    }
    return Tmax;
}

template <typename T, bool kSched>
__global__ __launch_bounds__(kBlockThreads) void bi_block_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model,
                                                                 TimesOut times, SchedOut sched, PlanHeader *plan,
                                                                 const int32_t *order, int cls, int32_t state_p, int32_t state_q,
                                                                 char *slots, size_t slot_bytes)
{
    PRS_DYNAMIC_LDS(lds_raw);
    __shared__ long long s_ticket;
    const int tid = static_cast<int>(threadIdx.x);
    char *slot = slots + static_cast<size_t>(blockIdx.x) * slot_bytes;
    const BlockSlot sl = bi_block_slot(state_p, state_q);
    const int Wc = (state_p + 63) >> 6;
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    for (;;) {
        __syncthreads();
        if (tid == 0) s_ticket = static_cast<long long>(atomicAdd(&plan->ticket[cls], 1ULL));
        __syncthreads();
        const int64_t ticket = s_ticket;
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
        if (status == PRS_CFG_OK) result = run_bi_block<T, kSched>(c, lds_raw, slot, sl, Wc, sched, base, &status);
        __syncthreads();
        if (tid == 0) {
            if (!kSched) write_closed_forms<T>(times, i, c, model);
            T *tg = static_cast<T *>(kSched ? sched.T_greedy : times.greedy);
            int32_t *cs = kSched ? sched.cfg_status : times.cfg_status;
            if (tg) tg[i] = status == PRS_CFG_OK ? result : CostTraits<T>::bad();
            if (cs) cs[i] = status;
        }
    }
}

template <typename T, bool kSched>
static hipError_t launch_bi_block_t(const BiLaunch &L)
{
    hipLaunchKernelGGL((bi_block_kernel<T, kSched>), dim3(L.grid), dim3(kBlockThreads), L.lds_bytes, L.stream, L.cfg, L.p_max,
                       L.q_max, L.model, L.times, L.sched, L.plan, L.order, L.cls, L.slot_p, L.slot_q, L.slots, L.slot_bytes);
    return hipGetLastError();
}

hipError_t launch_bi_block(const BiLaunch &L)
{
    if (L.cost == PRS_COST_I64) return L.want_schedule ? launch_bi_block_t<int64_t, true>(L) : launch_bi_block_t<int64_t, false>(L);
    return L.want_schedule ? launch_bi_block_t<double, true>(L) : launch_bi_block_t<double, false>(L);
}

}  // namespace prs
