/*
 * TEST INFRASTRUCTURE -- CPU oracle for pipelined-reduction schedules.
 *
 * A plain, slow, single-threaded restatement of what Lowery & Langou,
 * "A Greedy Algorithm for Optimally Pipelining a Reduction", compute:
 * the linear cost model (Section 2), the uni-greedy schedule (Algorithm 1,
 * Section 5), the bi-greedy schedule (Algorithm 2, Section 6.2), the closed
 * forms of the standard algorithms (Tables I-III), an exhaustive search over
 * all in-order unidirectional schedules (what Theorem 1 says uni-greedy
 * attains), and the replay of a schedule on data (Section 4: the receiver
 * combines the received segment into its own).
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * this.  It shares no code with the GPU library and is never a fallback.
 *
 * Readings of the paper taken here (the paper is silent, garbled or at odds
 * with itself at these points):
 *  - Ties in Algorithm 1's ordering P(X) are broken by processor index; g1
 *    sends to g2, except that when g1 is the root the roles swap (Lemma 1).
 *    Completion times do not depend on this choice.
 *  - Equi-segmentation of m into at most q_req segments: size ceil(m/q_req),
 *    the last segment takes the remainder (Section 2, last paragraph).
 *  - Algorithm 2, COMP: a processor is excluded while it computes
 *    (C1 <= t < C2) or when a communication of length tcomm(j) started now
 *    would run into a computation that is already scheduled
 *    (t < C1 < t + tcomm(j)); the printed second clause has no guard.
 *  - Algorithm 2 with a smaller last segment (Section 2 allows one): a
 *    processor does not receive a segment whose combine would begin while
 *    its own, longer send is still running -- Section 2 forbids
 *    communication to overlap computation and the listing only guards the
 *    other direction.  No effect when all segments are equal.
 *  - Algorithm 2, comparisons of t + tcomm(j) with the end of an earlier
 *    transfer of a segment of the same size: decided by the start times.
 *  - Algorithm 2: the root is never a sender (Lemma 1 (ii)); the printed
 *    sendProc does not exclude it.
 *  - Algorithm 2: lists are in ascending processor index (set semantics);
 *    the first l entries of each are paired entry by entry.
 *  - Algorithm 2: "M(i,j) = 0" as "has not sent" is kept as a separate flag.
 *  - Algorithm 2 assumes a unit time step; for real-valued costs t advances
 *    to the next time a port frees or a processor held back by the Section 2
 *    exclusion becomes eligible.  Both advances are implemented and compared
 *    in the tests.
 *  - Table III, bidirectional binary: 2(N+q-2) rounds (see orc_closed_forms).
 *
 * Pins: see tests/test_oracle_*.py.  Parity unpinned: the processor
 * identities of bi-greedy pairs (the paper's figure of its worked example is
 * not available as data); they are checked for validity only.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

int32_t orc_ceil_log2(int64_t v)
{
    int32_t l = 0;
    int64_t pw = 1;
    while (pw < v) { pw <<= 1; ++l; }
    return l;
}

/* Equi-segmentation (Section 2): all segments have size sz except possibly a
 * smaller last one.  From a requested count q_req: sz = ceil(m/q_req), the
 * number of segments actually needed is q = ceil(m/sz) <= q_req. */
void orc_segmentation(int64_t m, int64_t q_req, int64_t *q_eff, int64_t *sz_full, int64_t *sz_last)
{
    const int64_t sz = (m + q_req - 1) / q_req;
    const int64_t q = (m + sz - 1) / sz;
    *q_eff = q;
    *sz_full = sz;
    *sz_last = m - (q - 1) * sz;
}

#define CAT2(a, b) a##b
#define CAT(a, b) CAT2(a, b)
#define FN(name) CAT(name, SUF)

#define T int64_t
#define SUF _i64
#include "greedy_body.inc"
#undef T
#undef SUF

#define T double
#define SUF _f64
#include "greedy_body.inc"
#undef T
#undef SUF

/* Butterfly (Table III, last row) and the sums of the per-term lower bounds
 * (Table II first row; reference line of Figure 6), always in doubles.
 * out[0] = 2 L alpha + 2 (p-1)/p beta m + (p-1)/p gamma m
 * out[1] = L alpha + bw + (p-1)/p gamma m, bw = 2 m beta in the unidirectional
 *          model (m beta for p = 2), m beta in the bidirectional model. */
void orc_butterfly_and_bound(int model, int32_t p, int64_t m, double alpha, double beta, double gamma,
                             double out[2])
{
    const double L = (double)orc_ceil_log2((int64_t)p);
    const double fr = (double)(p - 1) / (double)p;
    const double md = (double)m;
    out[0] = ((2.0 * L) * alpha + (2.0 * fr) * (beta * md)) + fr * (gamma * md);
    const double bw = (model == 0 && p > 2) ? 2.0 * (md * beta) : md * beta;
    out[1] = (L * alpha + bw) + fr * (md * gamma);
}

/* ------------------------------------------------------------------------
 * Exhaustive search (integer costs, tiny p and q).
 *
 * Theorem 1: among unidirectional schedules that handle the segments in order
 * on every processor, uni-greedy finishes first.  This routine enumerates, for
 * each segment, every sequence of p-1 pairings (sender: any non-root
 * processor that has not sent the segment; receiver: any other processor that
 * has not sent it; start at the later of the two ready times), carries the
 * whole set of reachable end-of-segment states to the next segment, and
 * returns the smallest final root time.  States are kept as (root time,
 * sorted times of the others): processors are interchangeable.
 * ---------------------------------------------------------------------- */
typedef struct { int64_t *data; size_t n, cap; int w; } state_set;

static void ss_push(state_set *s, const int64_t *v)
{
    if (s->n == s->cap) {
        s->cap = s->cap ? s->cap * 2 : 1024;
        s->data = (int64_t *)realloc(s->data, s->cap * (size_t)s->w * sizeof(int64_t));
    }
    memcpy(s->data + s->n * (size_t)s->w, v, (size_t)s->w * sizeof(int64_t));
    s->n++;
}

static int g_cmp_w;
static int cmp_state(const void *a, const void *b)
{
    const int64_t *x = (const int64_t *)a, *y = (const int64_t *)b;
    for (int i = 0; i < g_cmp_w; ++i) { if (x[i] < y[i]) return -1; if (x[i] > y[i]) return 1; }
    return 0;
}

static int cmp_i64(const void *a, const void *b)
{
    const int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

static void ss_unique(state_set *s)
{
    if (s->n == 0) return;
    g_cmp_w = s->w;
    qsort(s->data, s->n, (size_t)s->w * sizeof(int64_t), cmp_state);
    size_t o = 1;
    for (size_t i = 1; i < s->n; ++i)
        if (cmp_state(s->data + (o - 1) * (size_t)s->w, s->data + i * (size_t)s->w) != 0) {
            memmove(s->data + o * (size_t)s->w, s->data + i * (size_t)s->w, (size_t)s->w * sizeof(int64_t));
            ++o;
        }
    s->n = o;
}

static void exh_rec(int p, int64_t c, int64_t g, int64_t *x, char *remaining, int left, state_set *out)
{
    if (left == 1) {
        int64_t v[64];
        v[0] = x[0];
        memcpy(v + 1, x + 1, (size_t)(p - 1) * sizeof(int64_t));
        qsort(v + 1, (size_t)(p - 1), sizeof(int64_t), cmp_i64);
        ss_push(out, v);
        return;
    }
    for (int a = 1; a < p; ++a) {
        if (!remaining[a]) continue;
        for (int b = 0; b < p; ++b) {
            if (b == a || !remaining[b]) continue;
            const int64_t xa = x[a], xb = x[b];
            const int64_t t = xa > xb ? xa : xb;
            x[a] = t + c; x[b] = t + c + g; remaining[a] = 0;
            exh_rec(p, c, g, x, remaining, left - 1, out);
            x[a] = xa; x[b] = xb; remaining[a] = 1;
        }
    }
}

/* Returns the optimal in-order completion time, or -1 if p > 63. */
int64_t orc_exhaustive_uni_i64(int32_t p, int32_t q, const int64_t *sizes, int64_t alpha, int64_t beta, int64_t gamma)
{
    if (p > 63) return -1;
    state_set cur = {0, 0, 0, p}, nxt = {0, 0, 0, p};
    int64_t zero[64] = {0};
    ss_push(&cur, zero);
    for (int32_t k = 0; k < q; ++k) {
        const int64_t c = alpha + beta * sizes[k], g = gamma * sizes[k];
        nxt.n = 0;
        for (size_t si = 0; si < cur.n; ++si) {
            int64_t x[64]; char remaining[64];
            memcpy(x, cur.data + si * (size_t)p, (size_t)p * sizeof(int64_t));
            memset(remaining, 1, (size_t)p);
            exh_rec(p, c, g, x, remaining, p, &nxt);
            if (nxt.n > (1u << 22)) ss_unique(&nxt);
        }
        ss_unique(&nxt);
        state_set tmp = cur; cur = nxt; nxt = tmp;
    }
    int64_t best = -1;
    for (size_t si = 0; si < cur.n; ++si) {
        const int64_t v = cur.data[si * (size_t)p];
        if (best < 0 || v < best) best = v;
    }
    free(cur.data); free(nxt.data);
    return best;
}

/* ------------------------------------------------------------------------
 * Replay of a schedule on data (Section 4: the receiver of a pair combines
 * the segment that arrived with its own copy of that segment).
 * buf holds p rows of n_elems values and is updated in place, pair by pair in
 * emission order: buf[dst][segment] = buf[dst][segment] + buf[src][segment].
 * seg_elem_offset[q+1] gives each segment's element range.  The reduction
 * ends up in row 0.
 * ---------------------------------------------------------------------- */
void orc_replay_i32(int32_t p, int64_t n_elems, const int64_t *seg_elem_offset, int64_t n_pairs,
                    const int32_t *src, const int32_t *dst, const int32_t *seg, int32_t *buf)
{
    (void)p;
    for (int64_t e = 0; e < n_pairs; ++e) {
        int32_t *d = buf + (size_t)dst[e] * (size_t)n_elems;
        const int32_t *s = buf + (size_t)src[e] * (size_t)n_elems;
        for (int64_t i = seg_elem_offset[seg[e]]; i < seg_elem_offset[seg[e] + 1]; ++i)
            d[i] = (int32_t)((uint32_t)d[i] + (uint32_t)s[i]);
    }
}

void orc_replay_f32(int32_t p, int64_t n_elems, const int64_t *seg_elem_offset, int64_t n_pairs,
                    const int32_t *src, const int32_t *dst, const int32_t *seg, float *buf)
{
    (void)p;
    for (int64_t e = 0; e < n_pairs; ++e) {
        float *d = buf + (size_t)dst[e] * (size_t)n_elems;
        const float *s = buf + (size_t)src[e] * (size_t)n_elems;
        for (int64_t i = seg_elem_offset[seg[e]]; i < seg_elem_offset[seg[e] + 1]; ++i)
            d[i] = d[i] + s[i];
    }
}
