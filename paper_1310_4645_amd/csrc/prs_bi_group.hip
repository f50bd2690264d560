// Bi-greedy schedules (Lowery & Langou, Algorithm 2, Section 6.2) for p <= 1024 on gfx950:
// several configurations per wavefront.
//
// A configuration is run by LPC adjacent lanes (1, 2, 4, 8 or 16), lane w of the group owning processors
// 64w .. 64w+63 as one machine word; a wavefront carries 64/LPC configurations at once.  Nothing is kept
// per processor:
//  - every send/receive pair scheduled in one visit (time t, segment j) has the same end of send
//    t + tcomm(j) and the same end of combine, so the ports and computations of Algorithm 2 (S, R, C)
//    are a short list of groups (end of send, end of combine, set of senders, set of receivers);
//    a processor's send port is free iff it is in no group whose send still runs, and so on;
//  - the number of segments a processor has sent (needed to drop finished processors from the
//    candidate sets) is a bit-sliced counter: bit b of all 64 counts in one word;
//  - M(i,j) "i has sent j" is one bit-set row per segment in the workspace;
//  - pairing e-th sender with e-th receiver needs no lists: each sender writes its pair record at
//    its rank among the senders, each receiver its own index at its rank among the receivers.
// The visit itself is the same sequence of set operations as in the one-configuration kernel.
// All lanes run one flat loop in which a group either visits the next segment or advances time, so
// groups at different times and segments share the same instructions.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kPlanes = 10;            // bit planes of the sent-segments counter: q <= 1023

// Entries of the list of running groups per configuration.  A configuration that needs more is handed
// to the one-configuration kernel; a launch may lower the limit (never the LDS layout) to force that path.
__host__ __device__ constexpr int bi_group_capacity(int lpc)
{
    return lpc == 1 ? 16 : (lpc == 2 ? 16 : (lpc == 4 ? 22 : (lpc == 8 ? 26 : 28)));
}
int bi_group_list_capacity(int lpc) { return bi_group_capacity(lpc); }

// LDS per wavefront: `cap` list entries, each with the two set words of every lane and the two times of
// every configuration in the wavefront
// (the times twice when lanes share them: see the kernel)
size_t bi_group_lds_bytes(int lpc)
{
    return static_cast<size_t>(bi_group_capacity(lpc)) * (64 * 16 + (64 / lpc) * 16 * (lpc == 1 ? 1 : 2));
}

// Sums and prefix sums over the lanes of a group use data-parallel-primitive moves (a lane reads its source
// operand from another lane of its row of 16: quad_perm inside a quad, row_half_mirror between the two quads of
// half a row, row_ror/row_shr inside the row) instead of LDS permutes: a group is a pair of lanes, a quad, half a
// row or a whole row, and these reductions sit on the dependent path of every visit.
template <int CTRL> __device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);        // lanes without a source read 0
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E;                          // quad_perm:[1,0,3,2], [2,3,0,1]
constexpr int kQuadLane0 = 0x00, kQuadLane1 = 0x55, kQuadLane2 = 0xAA;     // quad_perm broadcasts of lane 0, 1, 2
constexpr int kQuadEven = 0xA0;                                             // quad_perm:[0,0,2,2]: the even lane of each pair
constexpr int kRowHalfMirror = 0x141;                                       // lane i of half a row reads lane 7 - i
constexpr int kRowRor = 0x120, kRowShr = 0x110;                            // + distance 1..15

template <int LPC> __device__ __forceinline__ int group_sum(int v)
{
    if (LPC == 2) {
        v += dpp_move<kQuadXor1>(v);
    } else if (LPC == 4) {
        v += dpp_move<kQuadXor1>(v);
        v += dpp_move<kQuadXor2>(v);
    } else if (LPC == 8) {
        v += dpp_move<kQuadXor1>(v);
        v += dpp_move<kQuadXor2>(v);
        v += dpp_move<kRowHalfMirror>(v);                       // every lane holds its quad's sum: add the other quad's
    } else if (LPC == 16) {
        v += dpp_move<kRowRor + 8>(v);
        v += dpp_move<kRowRor + 4>(v);
        v += dpp_move<kRowRor + 2>(v);
        v += dpp_move<kRowRor + 1>(v);
    }
    return v;
}

// exclusive prefix sum over the LPC lanes of a group
template <int LPC> __device__ __forceinline__ int group_exclusive_scan(int v, int gl)
{
    if (LPC == 2) {
        const int even = dpp_move<kQuadEven>(v);
        return gl == 0 ? 0 : even;
    }
    if (LPC == 4 || LPC == 8) {
        const int a0 = dpp_move<kQuadLane0>(v), a1 = dpp_move<kQuadLane1>(v), a2 = dpp_move<kQuadLane2>(v);
        const int gq = gl & 3;
        int ex = gq == 0 ? 0 : (gq == 1 ? a0 : (gq == 2 ? a0 + a1 : a0 + a1 + a2));
        if (LPC == 8) {
            int quad = v;
            quad += dpp_move<kQuadXor1>(quad);
            quad += dpp_move<kQuadXor2>(quad);
            const int other = dpp_move<kRowHalfMirror>(quad);   // the sum of the other quad of the group
            if (gl & 4) ex += other;
        }
        return ex;
    }
    if (LPC == 16) {
        int inc = v;
        inc += dpp_move<kRowShr + 1>(inc);
        inc += dpp_move<kRowShr + 2>(inc);
        inc += dpp_move<kRowShr + 4>(inc);
        inc += dpp_move<kRowShr + 8>(inc);
        return inc - v;
    }
    (void)gl;
    return 0;
}

constexpr int kNoSegment = 1 << 20;

// How many processors of the group are in `a`, in `b` and in both, each counted up to two per word (enough to tell
// whether two different processors are there): the three counts travel in one sum.
template <int LPC> __device__ __forceinline__ void few_of_each(uint64_t a, uint64_t b, int &na, int &nb, int &nboth)
{
    const int ca = __popcll(a), cb = __popcll(b), cc = __popcll(a & b);
    const int packed = group_sum<LPC>((ca > 2 ? 2 : ca) | ((cb > 2 ? 2 : cb) << 8) | ((cc > 2 ? 2 : cc) << 16));
    na = packed & 255; nb = (packed >> 8) & 255; nboth = packed >> 16;
}

__device__ __forceinline__ void sliced_increment(uint64_t (&plane)[kPlanes], uint64_t who)
{
#pragma unroll
    for (int b = 0; b < kPlanes; ++b) { const uint64_t u = plane[b] & who; plane[b] ^= who; who = u; }
}

template <typename T, bool kSched, int LPC>
__device__ __forceinline__ void bi_group_body(char *lds_raw, int block, const ConfigArrays &cfg, int32_t p_max, int32_t q_max,
                                              int model, const TimesOut &times, const SchedOut &sched, PlanHeader *plan,
                                              const int32_t *order, int cls, int32_t *retry, uint64_t *rows,
                                              size_t rows_per_group, int list_entries)
{
    constexpr int kCap = bi_group_capacity(LPC);
    const int lane = lane_id();
    const int gl = lane & (LPC - 1);                    // lane within the group = word index
    const int group = (block * kWave + lane) / LPC;
    // group list in LDS, entry-major so that the 64 lanes of an entry touch consecutive addresses
    constexpr int kGroups = kWave / LPC;
    const int gw = lane / LPC;                                      // configuration slot within the wavefront
    uint64_t *gSm = reinterpret_cast<uint64_t *>(lds_raw);          // [kCap][64] senders (this lane's word)
    uint64_t *gRm = gSm + kCap * kWave;                             // [kCap][64] receivers
    // The times of an entry are shared by the lanes of a configuration.  Dropping finished entries copies
    // the list into a second buffer instead of compacting in place, so a lane never reads a slot that
    // another lane of its group has already rewritten, whatever the order in which lanes get there.
    constexpr int kBufs = LPC == 1 ? 1 : 2;
    T *gS = reinterpret_cast<T *>(gRm + kCap * kWave);              // [kBufs][kCap][kGroups] end of send
    T *gR = gS + kBufs * kCap * kGroups;                            // [kBufs][kCap][kGroups] end of combine
    int cur = 0;                                                    // buffer in use
    uint64_t *myrows = rows + static_cast<size_t>(group) * rows_per_group;   // [q][LPC] sent bits of this group
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    const T kInf = CostTraits<T>::inf();

    // ---- per-group state (identical in all lanes of a group unless noted)
    bool have = false;          // a configuration is loaded
    bool exhausted = false;     // no more tickets
    int64_t ci = 0;             // configuration index
    Config<T> c;
    int W = 0;
    T t = 0, Tmax = 0, minNew = kInf, minNewLate = kInf, minOld = kInf, minOldLate = kInf;
    int ndone = 0, segStart = 0, j = 0, jhi = -1, ng = 0, status = 0;
    bool need_event = true, overflow = false, idle_visit = false;
    int64_t emitted = 0, out_base = 0, events = 0;
    uint64_t valid = 0, sfree = 0, rfree = 0, compF = 0, compL = 0;   // this lane's word
    uint64_t lateL = 0;         // this lane's word: senders whose send outlasts a transfer of the smaller last segment begun now
    uint32_t shortMask = 0;     // bit s: list entry s carries the smaller last segment
    bool ragged = false, guardL = false;   // the last segment is smaller; and its combine takes time
    uint64_t cnt[kPlanes];      // bit-sliced: segments sent per processor
#pragma unroll
    for (int b = 0; b < kPlanes; ++b) cnt[b] = 0;
    c.p = 2; c.q = 1; c.status = 0; c.c_full = c.c_last = c.g_full = c.g_last = 0;

    for (;;) {
        // ---------------------------------------------------------------- fetch a configuration
        if (!have && !exhausted) {
            unsigned long long got = atomicAdd(&plan->ticket[cls], gl == 0 ? 1ULL : 0ULL);
            const uint32_t lo = __shfl(static_cast<uint32_t>(got), 0, LPC), hi = __shfl(static_cast<uint32_t>(got >> 32), 0, LPC);
            const int64_t ticket = static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
            if (ticket >= count) {
                exhausted = true;
            } else {
                ci = order[begin + ticket];
                c = decode_config<T>(cfg, ci, p_max, q_max);
                status = c.status;
                out_base = 0;
                if (kSched && status == PRS_CFG_OK) {
                    out_base = sched.pair_offset[ci];
                    const int64_t n_pairs = static_cast<int64_t>(c.p - 1) * c.q;
                    if (out_base < 0 || out_base + n_pairs > sched.pair_capacity) status = PRS_CFG_TOO_LARGE;
                }
                have = true;
                W = (c.p + 63) >> 6;
                valid = 0;
                if (gl < W) valid = (gl == W - 1 && (c.p & 63)) ? (UINT64_C(1) << (c.p & 63)) - 1 : ~UINT64_C(0);
                t = 0; Tmax = 0; minNew = kInf; minNewLate = kInf; minOld = kInf; minOldLate = kInf; ndone = 0; segStart = 0; j = 0; jhi = -1; ng = 0; cur = 0;
                shortMask = 0; lateL = 0;
                ragged = c.sz_last != c.sz;
                guardL = ragged && c.g_last > 0;
                need_event = true; overflow = false; idle_visit = false; emitted = 0; events = 0;
#pragma unroll
                for (int b = 0; b < kPlanes; ++b) cnt[b] = 0;
            }
        }
        // wavefront-wide exit: every group out of tickets and idle
        if (ballot64(have) == 0 && ballot64(!exhausted) == 0) break;

        // ---------------------------------------------------------------- finish a configuration
        const bool finished = have && (status != PRS_CFG_OK || ndone == c.q || overflow);
        if (finished) {
            if (gl == 0) {
                if (overflow) {
                    retry[atomicAdd(&plan->class_count[kRetryClass], 1)] = static_cast<int32_t>(ci);   // rerun by the one-configuration kernel
                } else {
                    if (!kSched) write_closed_forms<T>(times, ci, c, model);
                    T *tg = static_cast<T *>(kSched ? sched.T_greedy : times.greedy);
                    int32_t *st = kSched ? sched.cfg_status : times.cfg_status;
                    if (tg) tg[ci] = status == PRS_CFG_OK ? Tmax : CostTraits<T>::bad();
                    if (st) st[ci] = status;
                }
            }
            have = false;
        }
        const bool run = have && !finished;

        // ---------------------------------------------------------------- advance time (Algorithm 2: t <- next port release)
        if (run && need_event) {
            T tn = t;
            bool lateOnly = false;
            if (events > 0) {
                // the earliest end of a send or a combine after t, and the earliest time from which the sender of a
                // full segment may take in the smaller last one (end of its send - tcomm(last)): of the transfers begun
                // since the last event (kept up by the visits) and of the older ones (found when the sets were rebuilt)
                tn = minNew < minOld ? minNew : minOld;
                const T tl = minNewLate < minOldLate ? minNewLate : minOldLate;
                // No port frees at such a time: since the last event the candidates of every segment but the last
                // have only become fewer, so only the last segment is visited -- and if no processor with something
                // left to send has a free send port, nothing can pair before the next port frees: the time is skipped.
                const bool anySender = group_sum<LPC>(sfree != 0 ? 1 : 0) != 0;
                if (anySender && tl < tn) { tn = tl; lateOnly = true; }
                if (!(tn < kInf)) status = PRS_CFG_STALLED;
            }
            if (++events > 4 * static_cast<int64_t>(c.p) * c.q + 16) status = PRS_CFG_STALLED;
            t = tn;
            minNew = kInf; minNewLate = kInf; minOld = kInf; minOldLate = kInf;
            // rebuild the port and computation sets from the groups still running; drop finished groups
            uint64_t sbusy = 0, rbusy = 0, cF = 0, cL = 0, late = 0;
            uint32_t keptShort = 0;
            int keep = 0;
            const int nxt = kBufs == 1 ? 0 : cur ^ 1;
#pragma unroll 4
            for (int s = 0; s < ng; ++s) {
                const T se = gS[(cur * kCap + s) * kGroups + gw], re = gR[(cur * kCap + s) * kGroups + gw];
                const uint64_t sm = gSm[s * kWave + lane], rm = gRm[s * kWave + lane];
                if (re > t || se > t) {
                    if (se > t) sbusy |= sm;
                    if (re > t) rbusy |= rm;
                    const bool busy = se <= t && t < re;                  // receivers are computing
                    const bool pend = t < se;                             // their computation starts at se
                    // A transfer begun now must not run into that computation.  The entry began before t: against
                    // a segment of its own size that settles it (comparing the two rounded sums could miss it by
                    // one rounding error); against the other size the sums are compared.
                    const bool shortEntry = (shortMask >> s) & 1;
                    if (busy || (pend && (!shortEntry || t + c.c_full > se))) cF |= rm;
                    if (busy || (pend && (shortEntry || !ragged || t + c.c_last > se))) cL |= rm;
                    // Section 2 the other way round: the combine of the smaller last segment, received now, would
                    // begin while the sender of a full segment is still sending
                    if (guardL && !shortEntry && se > t + c.c_last) {
                        late |= sm;
                        const T v = se - c.c_last;
                        if (v > t && v < minOldLate) minOldLate = v;
                    }
                    if (se > t && se < minOld) minOld = se;               // the next event among the transfers that go on
                    if (re > t && re < minOld) minOld = re;
                    gS[(nxt * kCap + keep) * kGroups + gw] = se;          // same value from every lane of the group
                    gR[(nxt * kCap + keep) * kGroups + gw] = re;
                    if (keep != s) { gSm[keep * kWave + lane] = sm; gRm[keep * kWave + lane] = rm; }
                    if (shortEntry) keptShort |= 1u << keep;
                    ++keep;
                }
            }
            ng = keep;
            shortMask = keptShort;
            lateL = late;
            cur = nxt;
            // processors that have sent all q segments take part in nothing any more
            uint64_t fin = ~UINT64_C(0);
#pragma unroll
            for (int b = 0; b < kPlanes; ++b) fin &= ((c.q >> b) & 1) ? cnt[b] : ~cnt[b];
            const uint64_t rootbit = gl == 0 ? UINT64_C(1) : 0;
            const uint64_t live = valid & (~fin | rootbit);
            sfree = live & ~rootbit & ~sbusy;                             // the root never sends
            rfree = live & ~rbusy;
            compF = cF; compL = cL;
            j = segStart;
            idle_visit = lateOnly;
            need_event = false;
        }

        // ---------------------------------------------------------------- one visit (t, j)
        const bool visit = run && !need_event && status == PRS_CFG_OK;
        if (visit) {
            // A pair for segment j needs a processor with a free send port and a different one with a free
            // receive port that both still hold j and are not excluded by a computation.  If a visit paired
            // nobody although every candidate still held the segment, no later segment can pair either:
            // its candidates are a subset.  Exclusion by a pending computation depends on tcomm(j),
            // shorter for the last segment only: segments before the last use the full-length exclusion
            // set, the last one its own.  (A per-processor lower bound of the first segment still held, kept
            // as a bit-sliced counter, let a visit jump over segments its candidates had all sent; keeping it
            // up cost more than the visits it saved.)
            {
                int jn = kNoSegment;
                if (!idle_visit) {
                    const uint64_t as = sfree & ~compF, ar = rfree & ~compF;
                    int ns1, nr1, nb1;
                    few_of_each<LPC>(as, ar, ns1, nr1, nb1);
                    const bool pairable = ns1 > 0 && nr1 > 0 && !(ns1 == 1 && nr1 == 1 && nb1 == 1);
                    if (pairable && j < c.q - 1) jn = j;
                }
                if (jn == kNoSegment && j <= c.q - 1) {               // only the last segment is left to try
                    const uint64_t as = sfree & ~compL, ar = rfree & ~compL & ~lateL;
                    int ns1, nr1, nb1;
                    few_of_each<LPC>(as, ar, ns1, nr1, nb1);
                    if (ns1 > 0 && nr1 > 0 && !(ns1 == 1 && nr1 == 1 && nb1 == 1)) jn = c.q - 1;
                }
                j = jn == kNoSegment ? c.q : jn;
                idle_visit = false;
            }
            if (j >= c.q) {
                need_event = true;                                        // nothing more can pair at this t
            } else {
                const bool last = j == c.q - 1;
                uint64_t row = 0;
                if (j <= jhi && gl < W) row = myrows[static_cast<size_t>(j) * LPC + gl];
                const uint64_t rootbit = gl == 0 ? UINT64_C(1) : 0;
                const uint64_t memb = ~row & valid;                       // still hold segment j (root: until done)
                const uint64_t comp = last ? compL : compF;
                const uint64_t sOK = memb & ~comp & sfree, rOK = memb & ~comp & rfree & ~(last ? lateL : UINT64_C(0));
                const uint64_t fr = sOK & rOK, so = sOK ^ fr, ro = rOK ^ fr;
                const int pf = __popcll(fr);
                // counts of up to 1024 processors travel two to a sum
                const int memb_free = group_sum<LPC>(__popcll(memb & ~rootbit) | (pf << 16));
                int remj = memb_free & 0xFFFF;
                const int nf_ = memb_free >> 16;
                if (remj == 0) {                                          // everybody has sent segment j
                    if (j == segStart) ++segStart;
                    ++j;
                } else {
                    const int send_recv = group_sum<LPC>(__popcll(so) | (__popcll(ro) << 16));
                    const int ns_ = send_recv & 0xFFFF, nr_ = send_recv >> 16;
                    int toSendLast, toRecvFirst;                          // free processors go to the shorter list
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
                    if (l > 0) {
                        const int exF = group_exclusive_scan<LPC>(pf, gl);
                        const uint64_t frR = lowest_bits(fr, toRecvFirst - exF);
                        const uint64_t frS = highest_bits(fr, exF + pf - (nf_ - toSendLast));
                        uint64_t sset = so | frS, rset = ro | frR;
                        const int exSR = group_exclusive_scan<LPC>(__popcll(sset) | (__popcll(rset) << 16), gl);
                        const int exS = exSR & 0xFFFF, exR = exSR >> 16;
                        sset = lowest_bits(sset, l - exS);                // first l entries of each list
                        rset = lowest_bits(rset, l - exR);
                        const T cj = last ? c.c_last : c.c_full, gj = last ? c.g_last : c.g_full;
                        const T tc = t + cj, tr = tc + gj;
                        if (!(tc > t)) status = PRS_CFG_STALLED;
                        if (kSched) {                                     // e-th sender pairs with e-th receiver
                            // segment and start time are the same for all pairs of the visit: the lanes of the
                            // group write them side by side, four pairs each
                            for (int e = 4 * gl; e < l; e += 4 * LPC) {
                                const int64_t o = out_base + emitted + e;
                                if (e + 4 <= l) {
                                    const int32_t j4[4] = {j, j, j, j};
                                    const T t4[4] = {t, t, t, t};
                                    if (sched.seg) __builtin_memcpy(sched.seg + o, j4, sizeof(j4));
                                    if (sched.tstart) __builtin_memcpy(static_cast<T *>(sched.tstart) + o, t4, sizeof(t4));
                                } else {
                                    for (int i = 0; e + i < l; ++i) {
                                        if (sched.seg) sched.seg[o + i] = j;
                                        if (sched.tstart) static_cast<T *>(sched.tstart)[o + i] = t;
                                    }
                                }
                            }
                            if (sched.src) {
                                int32_t *const o = sched.src + (out_base + emitted + exS);
                                const int n = emit_set_bits(o, static_cast<uint32_t>(sset), gl * 64);
                                emit_set_bits(o + n, static_cast<uint32_t>(sset >> 32), gl * 64 + 32);
                            }
                            if (sched.dst) {
                                int32_t *const o = sched.dst + (out_base + emitted + exR);
                                const int n = emit_set_bits(o, static_cast<uint32_t>(rset), gl * 64);
                                emit_set_bits(o + n, static_cast<uint32_t>(rset >> 32), gl * 64 + 32);
                            }
                        }
                        emitted += l;
                        row |= sset;
                        sfree &= ~sset;
                        rfree &= ~rset;
                        sliced_increment(cnt, sset);                     // one more sent segment for the senders
                        if (ng < list_entries) {
                            gS[(cur * kCap + ng) * kGroups + gw] = tc; gR[(cur * kCap + ng) * kGroups + gw] = tr;
                            gSm[ng * kWave + lane] = sset; gRm[ng * kWave + lane] = rset;
                            if (last && ragged) shortMask |= 1u << ng;
                            ++ng;
                        } else {
                            overflow = true;
                        }
                        if (tc < minNew) minNew = tc;
                        if (tr < minNew) minNew = tr;
                        if (guardL && !last && tc > t + c.c_last) {      // these senders cannot take the last segment in yet
                            lateL |= sset;
                            const T v = tc - c.c_last;
                            if (v > t && v < minNewLate) minNewLate = v;
                        }
                        remj -= l;
                        if (remj == 0) {                                  // only the root is left: done after the last arrival
                            if (tr > Tmax) Tmax = tr;
                            ++ndone;
                        }
                    }
                    if (gl < W && (l > 0 || j > jhi)) myrows[static_cast<size_t>(j) * LPC + gl] = row;
                    if (j > jhi) {
                        // a jump to the last segment can pass segments nobody has visited: their rows are empty
                        for (int jj = jhi + 1; jj < j; ++jj)
                            if (gl < W) myrows[static_cast<size_t>(jj) * LPC + gl] = 0;
                        jhi = j;
                    }
                    ++j;
                    // nobody paired and no candidate had already sent j
                    idle_visit = l == 0 && group_sum<LPC>(((sfree | rfree) & ~comp & row) != 0 ? 1 : 0) == 0;
                }
            }
        }
    }
}

// One launch runs all group sizes on one resident set of blocks.  The first start[4] blocks begin with the 16-lane
// configurations, the next start[3] with the 8-lane ones and so on, so the longest-running configurations of
// every class start at once; a block whose class has run out of tickets goes on with the others (largest
// groups first).
template <typename T, bool kSched>
__global__ __launch_bounds__(kWave) void bi_group_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model,
                                                         TimesOut times, SchedOut sched, PlanHeader *plan,
                                                         const int32_t *order, int32_t *retry, BiGroupParts parts)
{
    PRS_DYNAMIC_LDS(lds_raw);
    const int b = static_cast<int>(blockIdx.x);
    uint64_t *rows = parts.rows + static_cast<size_t>(b) * parts.rows_per_block;
    int first = 0, upto = 0;
    for (int g = kBiGroupSizes - 1; g >= 0; --g) {
        upto += parts.start[g];
        if (b < upto) { first = g; break; }
    }
    for (int turn = 0; turn < kBiGroupSizes; ++turn) {
        // turn 0: the class this block starts with; then the remaining classes, largest groups first
        int cls = first;
        if (turn > 0) {
            cls = kBiGroupSizes - turn;                      // 4, 3, 2, 1 ...
            if (cls <= first) --cls;                         // ... without the one done in turn 0
        }
        if (!parts.on[cls]) continue;
        switch (cls) {
        case 4:
            bi_group_body<T, kSched, 16>(lds_raw, 0, cfg, p_max, q_max, model, times, sched, plan, order, 4, retry, rows,
                                         parts.rows_per_group[4], parts.list_entries[4]);
            break;
        case 3:
            bi_group_body<T, kSched, 8>(lds_raw, 0, cfg, p_max, q_max, model, times, sched, plan, order, 3, retry, rows,
                                        parts.rows_per_group[3], parts.list_entries[3]);
            break;
        case 2:
            bi_group_body<T, kSched, 4>(lds_raw, 0, cfg, p_max, q_max, model, times, sched, plan, order, 2, retry, rows,
                                        parts.rows_per_group[2], parts.list_entries[2]);
            break;
        case 1:
            bi_group_body<T, kSched, 2>(lds_raw, 0, cfg, p_max, q_max, model, times, sched, plan, order, 1, retry, rows,
                                        parts.rows_per_group[1], parts.list_entries[1]);
            break;
        default:
            bi_group_body<T, kSched, 1>(lds_raw, 0, cfg, p_max, q_max, model, times, sched, plan, order, 0, retry, rows,
                                        parts.rows_per_group[0], parts.list_entries[0]);
            break;
        }
        __syncthreads();
    }
}

template <typename T, bool kSched> static void launch_fused(const BiGroupLaunch &L)
{
    size_t lds = 0;
    int grid = 0;
    for (int k = 0; k < kBiGroupSizes; ++k) {
        if (L.parts.on[k] && bi_group_lds_bytes(1 << k) > lds) lds = bi_group_lds_bytes(1 << k);
        grid += L.parts.start[k];
    }
    hipLaunchKernelGGL((bi_group_kernel<T, kSched>), dim3(grid), dim3(kWave), lds, L.stream, L.cfg, L.p_max, L.q_max, L.model,
                       L.times, L.sched, L.plan, L.order, L.retry, L.parts);
}

hipError_t launch_bi_group(const BiGroupLaunch &L)
{
    int blocks = 0;
    for (int k = 0; k < kBiGroupSizes; ++k) blocks += L.parts.start[k];
    if (blocks == 0) return hipSuccess;
    if (L.cost == PRS_COST_I64) { if (L.want_schedule) launch_fused<int64_t, true>(L); else launch_fused<int64_t, false>(L); }
    else { if (L.want_schedule) launch_fused<double, true>(L); else launch_fused<double, false>(L); }
    return hipGetLastError();
}

}  // namespace prs
