/*
 * prs.h -- C ABI of the pipelined-reduction-schedule library for AMD gfx950.
 *
 * The library constructs and times reduction schedules on a machine of p
 * homogeneous, fully connected processors under the linear cost model of
 * Lowery & Langou, "A Greedy Algorithm for Optimally Pipelining a Reduction"
 * (Section 2): sending a segment of sz elements keeps the sender busy
 * tcomm = alpha + beta*sz and the receiver tcomm + tcomp, tcomp = gamma*sz;
 * communication and computation never overlap on a processor.  A message of
 * m elements is cut into q segments of equal size, the last possibly smaller.
 * A reduction is a set of (p-1)q send/receive pairs (Section 5, first
 * paragraph); its completion time is the time the root, processor 0,
 * finishes its last combine.
 *
 * Conventions, valid for every entry point:
 *  - "device" pointers address GPU memory of the current HIP device, "host"
 *    pointers ordinary memory.  All buffers are allocated and owned by the
 *    caller; the library allocates no device memory and keeps no state
 *    between calls.  Inputs are never written.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued on it and the call returns without synchronising.
 *  - `workspace` is device scratch of at least prs_workspace_bytes(...)
 *    bytes, 256-byte aligned, private to the call until the stream has
 *    drained it.
 *  - The return value is a prs_status for the call as a whole; when it is
 *    not PRS_OK nothing has been enqueued.  Problems of a single
 *    configuration are reported in its cfg_status entry (prs_cfg_status):
 *    its results are then -1 (integers) or NaN (doubles), its schedule range
 *    is left untouched, and the rest of the batch is unaffected.
 *  - Costs are either all int64_t (integer time units) or all double
 *    (seconds), selected by prs_cost.  Doubles are combined as
 *    tcomm = alpha + (beta*sz), end of send = t + tcomm, end of combine =
 *    (t + tcomm) + tcomp, every operation rounded on its own (no FMA).
 *    Integer overflow is not detected.
 */
#ifndef PRS_H
#define PRS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { PRS_OK = 0, PRS_EINVAL = 1, PRS_ENOSPC = 2, PRS_EDEVICE = 3 } prs_status;
typedef enum { PRS_UNI = 0, PRS_BI = 1 } prs_model;      /* one port / separate send and receive ports (Section 2) */
typedef enum { PRS_COST_I64 = 0, PRS_COST_F64 = 1 } prs_cost;
typedef enum { PRS_I32 = 0, PRS_F32 = 1, PRS_F64 = 2, PRS_I64 = 3 } prs_dtype;
/* combine operation of replay_reduction, OR-ed into its dtype argument */
typedef enum { PRS_OP_SUM = 0, PRS_OP_MAX = 0x100 } prs_op;
typedef enum {
    PRS_CFG_OK = 0,
    PRS_CFG_BAD_PARAM = 1,   /* p < 2, q_req < 1, m < 1, a negative or non-finite cost, tcomm = 0, or a schedule too long for
                                the cost type: (p-1+2(q-1))(alpha+beta s+gamma s), Table I's pipeline time which no greedy
                                time passes, must stay below 4e18 (int64_t) or 1e300 (double) */
    PRS_CFG_TOO_LARGE = 2,   /* p > p_max, q_req > q_max, or the schedule does not fit pair_capacity */
    PRS_CFG_STALLED = 3      /* time could not advance (a cost vanished against the clock in rounding) */
} prs_cfg_status;
typedef enum { PRS_CALL_SIMULATE = 0, PRS_CALL_SCHEDULE = 1, PRS_CALL_REPLAY = 2, PRS_CALL_OFFSETS = 3, PRS_CALL_SEARCH = 4,
               PRS_CALL_UNEQUAL = 5 } prs_call;

/* A batch of n configurations, structure of arrays, DEVICE pointers.
 * q_req is the requested number of segments: the segment size is
 * ceil(m / q_req) and q_eff = ceil(m / size) <= q_req segments are used
 * (Section 2, last paragraph).  alpha, beta, gamma point to int64_t or double
 * according to the prs_cost argument of the call. */
typedef struct prs_configs {
    const int32_t *p;
    const int32_t *q_req;
    const int64_t *m;
    const void *alpha;
    const void *beta;
    const void *gamma;
} prs_configs;

/* Result columns of simulate_completion_batch, DEVICE pointers to n entries
 * each; any of them may be NULL to skip that column.  greedy..revopt have the
 * cost type of the call, butterfly and lower_bound are always double. */
typedef struct prs_times {
    void *greedy;        /* uni-greedy (Algorithm 1) or bi-greedy (Algorithm 2) completion time */
    void *binomial;      /* ceil(log2 p)(alpha + beta m + gamma m)                 Tables I, III */
    void *pipeline;      /* uni (p-1+2(q-1)) r, bi (p+q-2) r, r = alpha+beta sz+gamma sz          */
    void *binary;        /* uni (2(N-1)+4(q-1)) r, bi 2(N+q-2) r, N = ceil(log2(p+1))             */
    void *revopt;        /* reversed optimal broadcast (ceil(log2 p)+q-1) r         Table III    */
    double *butterfly;   /* 2 L alpha + 2 (p-1)/p beta m + (p-1)/p gamma m          Table III    */
    double *lower_bound; /* L alpha + B + (p-1)/p gamma m; B = 2 m beta (uni, p > 2), m beta otherwise
                            (Table II, first row; reference line of Figure 6) */
    int32_t *q_eff;      /* number of segments actually used */
    int32_t *cfg_status; /* prs_cfg_status */
} prs_times;

/* Optional launch tuning of the sweep calls; NULL means the built-in choices.  It changes how
 * configurations are spread over the lanes of a wavefront, never a result; tests use it to push one batch
 * through every code path.
 * uni_group_pairs[k]: a uni-greedy configuration of at most this many send/receive pairs is run by 1 (k=0),
 *   4 (k=1; 8 where schedules are written) or 16 (k=2) lanes, larger ones by 32.  Used if the three are >= 0 and non-decreasing (all zero:
 *   everything on 32 lanes -- also what a zeroed struct selects); otherwise, e.g. with -1, the built-in limits.
 * uni_wave_log2: configurations of at least 2^uni_wave_log2 pairs get a whole wavefront (1..39; else built-in).
 * uni_wide_procs: uni-greedy completion times of machines with at least this many processors are computed by a
 *   whole block per configuration, many pairs of a segment at once (>= 2; else built-in: never, the kernel is
 *   slower than the segment pipeline on every workload measured).
 * bi_list_entries: most entries of the per-configuration list of running transfers in the bi-greedy kernel
 *   for p <= 1024; a configuration that needs more is rerun by the general kernel (1 .. built-in size; else
 *   built-in). */
typedef struct prs_tuning {
    int64_t uni_group_pairs[3];
    int32_t uni_wave_log2;
    int32_t bi_list_entries;
    int32_t uni_wide_procs;
    int32_t reserved;            /* 0 */
} prs_tuning;

/* Bytes of device scratch the given call needs for a batch of n
 * configurations with p <= p_max and q_req <= q_max (for PRS_CALL_REPLAY:
 * n = 1, p_max = p, q_max = q; for PRS_CALL_UNEQUAL: q_max = m_max).  Host
 * function, no GPU work. */
size_t prs_workspace_bytes(int call, int model, int cost, int64_t n, int32_t p_max, int32_t q_max);

/*
 * Completion time of the greedy schedule of every configuration, next to the
 * closed-form times of the standard algorithms it is compared with (Sections
 * 4, 5.2, 6.1).  model = PRS_UNI runs Algorithm 1 (Section 5): per segment,
 * p-1 times, the two processors with the smallest ready times pair up at the
 * larger of the two.  model = PRS_BI runs Algorithm 2 (Section 6.2), its unit
 * time step replaced by a jump to the next time at which a pair can form (a
 * port frees, or a processor may take in the smaller last segment: Section 2
 * lets no combine start while the processor still sends, so with a smaller
 * last segment it receives that segment only from the end of its running
 * send minus tcomm(last) on).
 * cfg, out: host structs holding device pointers.  p_max, q_max: upper bounds
 * on p and q_req in the batch (they size the workspace).
 * Errors: PRS_EINVAL for a NULL struct/array, n < 0, bad enum or bounds;
 * PRS_ENOSPC if workspace_bytes is too small; PRS_EDEVICE if a launch fails.
 */
int simulate_completion_batch(const prs_configs *cfg, int64_t n, int model, int cost,
                              int32_t p_max, int32_t q_max, const prs_times *out,
                              void *workspace, size_t workspace_bytes, void *stream, const prs_tuning *tuning);

/*
 * pair_offset[i] = sum over j < i of (p_j - 1) * q_eff_j, for i = 0..n
 * (invalid configurations count 0): where configuration i's pairs start in
 * the arrays of greedy_schedule_batch.  pair_offset: device, n+1 entries.
 */
int prs_pair_offsets(const prs_configs *cfg, int64_t n, int cost, int32_t p_max, int32_t q_max,
                     int64_t *pair_offset, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The greedy schedule itself (Section 5, Algorithm 1; Section 6.2, Algorithm
 * 2): for configuration i, pairs pair_offset[i] .. pair_offset[i+1]-1 of the
 * device arrays src, dst, seg (int32) and t_start (cost type) receive, in the
 * order the algorithm emits them, the sending processor, the receiving
 * processor, the 0-based segment and the start time of each send/receive
 * pair.  Ties between equal ready times (Algorithm 1) go to the smaller
 * processor index and the first of the two sends unless it is the root.
 * Algorithm 2 emits by time, then segment, then position in its paired lists.
 * Any of src/dst/seg/t_start/T_greedy may be NULL.  A configuration whose
 * range would pass pair_capacity gets PRS_CFG_TOO_LARGE and writes nothing.
 */
int greedy_schedule_batch(const prs_configs *cfg, int64_t n, int model, int cost,
                          int32_t p_max, int32_t q_max,
                          const int64_t *pair_offset, int64_t pair_capacity,
                          int32_t *src, int32_t *dst, int32_t *seg, void *t_start,
                          void *T_greedy, int32_t *cfg_status,
                          void *workspace, size_t workspace_bytes, void *stream, const prs_tuning *tuning);

/*
 * Executes one schedule on data (Section 4: the receiver of a pair combines
 * the segment that arrived with its own copy of it): with buf_i = in + i*stride_elems (i < p, n_elems values each),
 * applying buf_dst[segment] = buf_dst[segment] + buf_src[segment] pair by
 * pair in the order given leaves the reduction in buf_0; that result, with
 * exactly that association of the additions, is written to out (n_elems
 * values).  `in` is not modified.  Segment k covers elements
 * seg_elem_offset[k] .. seg_elem_offset[k+1]-1 (HOST array, q+1 entries,
 * non-decreasing from 0 to n_elems; read before the call returns).
 * src, dst, seg: device, n_pairs = (p-1)q entries, in which every non-root
 * processor sends every segment exactly once, after all it receives of it.
 * dtype: element type PRS_I32, PRS_I64 (wrapping add), PRS_F32 or PRS_F64
 * (IEEE add, no FMA, denormals kept), optionally OR-ed with PRS_OP_MAX: the
 * combine is then buf_dst = max(buf_dst, buf_src) instead of the sum (the
 * paper's reduction is any associative and commutative operation; Section 1),
 * floating point
 * compared in the IEEE total order (-0 below +0, NaNs at the two ends), so
 * that the result is a well-defined element of the inputs.  status: device int32, receives 0, or 1 if the schedule is not a
 * set of q in-trees on p processors, or 2 if a combine tree needs more
 * nested partial sums than the kernel holds (then out is not written).
 * Limits: 2 <= p <= 4096, q <= 65536, (p-1)q < 2^31.
 */
int replay_reduction(int32_t p, int32_t q, const int64_t *seg_elem_offset,
                     const int32_t *src, const int32_t *dst, const int32_t *seg, int64_t n_pairs,
                     const void *in, int64_t stride_elems, int64_t n_elems, int dtype,
                     void *out, int32_t *status,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * replay_reduction for callers that can neither allocate device memory nor
 * bring a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, results and status as
 * replay_reduction, without `workspace`: the tree programs live in a fixed
 * device array of 8 MiB inside the library, one per GPU, taken hold of at the
 * first call on that GPU and kept until the process ends.  The call itself
 * allocates nothing.  Returns PRS_ENOSPC (nothing enqueued) when the schedule
 * needs more than the array holds: 8(q+1) + 4pq + 768 bytes rounded up to
 * multiples of 256, plus 32pq bytes when p > 1536.  All calls on one GPU
 * share that array: two of them must not be in flight at the same time (on
 * different streams, or from different threads); calls that follow each other
 * on one stream are fine.
 */
int replay_reduction_static(int32_t p, int32_t q, const int64_t *seg_elem_offset,
                            const int32_t *src, const int32_t *dst, const int32_t *seg, int64_t n_pairs,
                            const void *in, int64_t stride_elems, int64_t n_elems, int dtype,
                            void *out, int32_t *status, void *stream);

/* Result columns of optimal_segmentation_batch, DEVICE pointers to n entries
 * each, any of them may be NULL.  T_* have the cost type of the call. */
typedef struct prs_best {
    void *T_greedy, *T_pipeline, *T_binary, *T_revopt;      /* smallest completion time over the candidates */
    int32_t *q_greedy, *q_pipeline, *q_binary, *q_revopt;   /* q_req of the first candidate that reaches it */
    int32_t *cfg_status;                                    /* prs_cfg_status of the problem */
} prs_best;

/*
 * Best segmentation per algorithm (Sections 5.2 and 6.1: every algorithm is
 * compared at the segment size that suits it best, found by trying sizes).
 * For each problem (p, m, alpha, beta, gamma) of the batch -- cfg->q_req is
 * not read and may be NULL -- the candidates q_req = 1, 2, 4, ... (powers of
 * two up to q_max) are cut as in simulate_completion_batch and timed with the
 * greedy algorithm of `model`, the pipeline, the binary tree and the reversed
 * optimal broadcast; out receives per algorithm the smallest completion time
 * and the candidate that gives it (the smallest such q_req on ties).
 * Candidates beyond m repeat the unit-size segmentation and never win a tie.
 * Errors as simulate_completion_batch.
 */
int optimal_segmentation_batch(const prs_configs *cfg, int64_t n, int model, int cost,
                               int32_t p_max, int32_t q_max, const prs_best *out,
                               void *workspace, size_t workspace_bytes, void *stream, const prs_tuning *tuning);

/* Result columns of unequal_segmentation_batch, DEVICE pointers, any of them
 * may be NULL.  T_* have the cost type of the call. */
typedef struct prs_unequal {
    void *T_all;            /* n * 2^(m_max-1): time of problem i under cut pattern c at [i * 2^(m_max-1) + c]
                               (the "bad" value -1 / NaN where c is no segmentation of the problem's m) */
    void *T_best;           /* n: smallest time over all 2^(m-1) segmentations */
    uint32_t *cuts_best;    /* n: the numerically smallest cut pattern that reaches it */
    int32_t *n_best;        /* n: how many segmentations reach it */
    void *T_equi;           /* n: smallest time over the equi-segmentations, sizes ceil(m/k), k = 1..m */
    uint32_t *cuts_equi;    /* n: the numerically smallest cut pattern among those */
    int32_t *equi_optimal;  /* n: bit 0: T_equi == T_best; bit 1: an optimal segmentation has equal sizes
                               except a smaller (or equal) last one, whatever that size */
    int32_t *cfg_status;    /* n: prs_cfg_status of the problem */
} prs_unequal;

/*
 * Unequal segmentation (Section 8: the message is fixed to a few units and
 * every way of cutting it into consecutive segments is run through the
 * unidirectional greedy algorithm; "Ratio" = best equi-segmentation time /
 * best time over all segmentations = T_equi / T_best).  Problem i is
 * (p, m, alpha, beta, gamma)[i] with 1 <= m <= m_max <= 24 units; beta and
 * gamma are per unit; cfg->q_req is not read and may be NULL.  A segmentation
 * is a cut pattern of m-1 bits: bit b set = a segment ends after unit b+1, so
 * pattern 0 is the unsegmented message and 2^(m-1)-1 is m unit segments; its
 * segments cost tcomm = alpha + beta*size, tcomp = gamma*size each and run
 * through Algorithm 1 in order.  Equi-segmentations are the ones
 * simulate_completion_batch cuts from a segment count.
 * n * 2^(m_max-1) < 2^31.  Errors as simulate_completion_batch; workspace from
 * prs_workspace_bytes(PRS_CALL_UNEQUAL, PRS_UNI, cost, n, p_max, m_max).
 */
int unequal_segmentation_batch(const prs_configs *cfg, int64_t n, int cost, int32_t p_max, int32_t m_max,
                               const prs_unequal *out, void *workspace, size_t workspace_bytes, void *stream,
                               const prs_tuning *tuning);

/*
 * Butterfly against bi-greedy (Section 6.1, last paragraph and its figure of the parameters for which some
 * message size lets the butterfly win).  For every machine size p[i] (device, n entries) the line is located
 * by bisection over the ratio beta/gamma: gamma = 1, beta = the ratio, latency alpha; at a ratio the butterfly
 * "wins" if for one of the message sizes m = 2^k, k = m_log2_first..m_log2_last, its time (Table III) is
 * below the time of the reversed optimal broadcast -- the time bi-greedy meets, Table III -- at the best of the
 * segment counts 1..min(q_max, m), each cut as in simulate_completion_batch.  Starting from [ratio_lo,
 * ratio_hi] (the caller's bracket: wins at ratio_lo, not at ratio_hi), `steps` times the midpoint
 * lo + (hi - lo)/2 replaces lo if the butterfly wins there, else hi.  ratio_below / ratio_above (device, n
 * doubles, either may be NULL) receive the final lo and hi; cfg_status (device, may be NULL) PRS_CFG_OK, or
 * PRS_CFG_BAD_PARAM for p < 2 (results NaN).  No workspace.
 * Errors: PRS_EINVAL unless 0 <= alpha < 1e300, 0 < ratio_lo < ratio_hi < 1e100, 1 <= q_max <= 2^20,
 * 0 <= m_log2_first <= m_log2_last <= 40, 0 <= steps <= 64, 0 <= n < 2^31.
 */
int butterfly_threshold_batch(const int32_t *p, int64_t n, double alpha, int32_t q_max,
                              int32_t m_log2_first, int32_t m_log2_last,
                              double ratio_lo, double ratio_hi, int32_t steps,
                              double *ratio_below, double *ratio_above, int32_t *cfg_status, void *stream);

/*
 * Measurement helper, no result: `blocks` blocks of 256 lanes each run steps_per_lane dependent steps of the
 * bare arithmetic of Algorithm 1 (Section 5: pick the two smallest of two sorted fronts, add tcomm, add tcomp --
 * two comparisons, two additions) on registers only.  Timed by the caller, blocks * 256 * steps_per_lane steps
 * per launch give the rate the chip reaches on this arithmetic with nothing else in the way: the practical
 * ceiling next to the nominal fp64 rate.  sink: device, one double, never written in practice.
 */
int prs_measure_alu_ceiling(int64_t steps_per_lane, int32_t blocks, double *sink, void *stream);

/* Version of the ABI, bumped on any incompatible change. */
int prs_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PRS_H */
