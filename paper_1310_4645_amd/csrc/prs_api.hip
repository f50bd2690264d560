// C ABI of the library (declared in include/prs.h): argument checks, workspace
// carving and kernel launches.  No device memory is allocated here.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr size_t kHeaderBytes = 256;
constexpr size_t kMaxWorkspace = static_cast<size_t>(16) << 30;   // slots of the global-memory class, at most (if 256 of them fit)

__global__ void clear_words(unsigned long long *w, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) w[i] = 0ULL;
}

hipError_t launch_clear(unsigned long long *words, int count, hipStream_t stream)
{
    hipLaunchKernelGGL(clear_words, dim3((count + 63) / 64), dim3(64), 0, stream, words, count);
    return hipGetLastError();
}

// pair_offset[i] = sum_{j<i} (p_j - 1) q_eff_j; one block, sequential carry over tiles of 1024.
template <typename T>
__global__ __launch_bounds__(1024) void offsets_kernel(ConfigArrays cfg, int64_t n, int32_t p_max, int32_t q_max,
                                                       int64_t *pair_offset)
{
    __shared__ int64_t s_wave[16];
    __shared__ int64_t s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) { s_carry = 0; pair_offset[0] = 0; }
    __syncthreads();
    for (int64_t base = 0; base < n; base += 1024) {
        const int64_t i = base + tid;
        int64_t cnt = 0;
        if (i < n) {
            const Config<T> c = decode_config<T>(cfg, i, p_max, q_max);
            if (c.status == PRS_CFG_OK) cnt = static_cast<int64_t>(c.p - 1) * c.q;
        }
        int64_t inc = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int64_t u = __shfl_up(inc, o, 64);
            if (lane >= o) inc += u;
        }
        if (lane == 63) s_wave[wv] = inc;
        __syncthreads();
        int64_t before = s_carry;
        for (int w = 0; w < wv; ++w) before += s_wave[w];
        if (i < n) pair_offset[i + 1] = before + inc;
        __syncthreads();
        if (tid == 1023) s_carry = before + inc;
        __syncthreads();
    }
}

hipError_t launch_offsets(const OffsetsLaunch &L)
{
    if (L.cost == PRS_COST_I64)
        hipLaunchKernelGGL((offsets_kernel<int64_t>), dim3(1), dim3(1024), 0, L.stream, L.cfg, L.n, L.p_max, L.q_max, L.pair_offset);
    else
        hipLaunchKernelGGL((offsets_kernel<double>), dim3(1), dim3(1024), 0, L.stream, L.cfg, L.n, L.p_max, L.q_max, L.pair_offset);
    return hipGetLastError();
}

// ---- size classes and workspace layout (shared by prs_workspace_bytes and the launches) --------------
//
// A batch is split into four classes, each run by the kernel and the LDS allocation that fit it:
//   uni-greedy (times and schedules): by number of pairs; 1, 4 (schedules: 8), 16 or 32 lanes per configuration, all four
//                                     classes in one launch;
//   bi-greedy:                        1, 2, 4, 8 or 16 lanes per configuration for p <= 64 / 128 / 256 / 512 / 1024 and
//                                     q <= 1023; the general kernel for the rest and for reruns.
enum ClassKind { kUniTimes, kUniSched, kBiGroup, kBiGeneral, kBiBlock, kUniWide };
constexpr size_t kLdsPerCU = 160 * 1024, kLdsPerBlockMax = 64 * 1024, kBitmapLdsMax = 24 * 1024;
constexpr int kCUs = 256, kMaxBlocksPerCU = 24, kGlobalClassGrid = 1024;
constexpr int32_t kGroupQMax = 1023;   // the several-per-wavefront bi-greedy kernel counts sent segments in 10 bit planes
constexpr int kUniGroupSizes = 3;        // group sizes below the largest; the classes between them and the last stay empty
constexpr int64_t kUniWork[kUniGroupSizes] = {1024, 8192, 262144};        // completion times: most pairs of a configuration run by 1, 4, 16 lanes
constexpr int64_t kUniWorkSched[kUniGroupSizes] = {1024, 65536, 262144};  // schedules: by 1, 8, 16 lanes (measured best on the sweep)
// uni-greedy completion times: machines of at least this many processors would get a block per configuration.  Off: measured
// on the large-machine sweep the segment pipeline through the lanes is 2 to 3 times faster (in steady state only a few
// hundred values lie under the bound of a round); the kernel stays reachable through prs_tuning.
constexpr int32_t kUniWideProcs = INT32_MAX;

struct ClassSpec {
    ClassKind kind;
    int lpc;                  // kBiGroup: lanes per configuration
    size_t rows_per_group;    // kBiGroup: words of sent-bit rows per configuration slot
    int32_t p_cap;            // capacity of the per-processor arrays of this class
    int32_t q_cap;            // capacity of its per-segment arrays
    bool lds;                 // state (uni batch) / small arrays and maybe the bitmap (bi general) in LDS
    size_t lds_bytes;
    int32_t lds_bitmap_bytes;
    size_t slot_bytes, slot_offset;
    int grid;
};

struct Layout {
    size_t header, order, retry, total;
    ClassLimits limits;
    ClassSpec cls[kClasses];
    ClassSpec rerun;              // bi-greedy: the one-wavefront kernel for configurations the group kernel hands back
    ClassSpec wide;               // uni-greedy completion times: the block-per-configuration kernel (grid 0: not used)
    bool bi_on[kClasses - 1];     // bi-greedy group classes a configuration can fall into
};

static size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// the one-configuration-per-wavefront bi-greedy kernel: where its arrays go for machines of up to p_cap processors
static void general_spec(ClassSpec &c, int32_t p_cap, int32_t q_cap)
{
    c.kind = kBiGeneral;
    c.p_cap = p_cap;
    c.q_cap = q_cap;
    c.lds = false; c.lds_bytes = 0; c.lds_bitmap_bytes = 0; c.lpc = 0; c.rows_per_group = 0;
    const size_t small = bi_small_bytes(p_cap, q_cap), bitmap = bi_bitmap_bytes(p_cap, q_cap);
    if (small <= kLdsPerBlockMax / 2) {
        c.lds = true;
        c.lds_bitmap_bytes = static_cast<int32_t>(bitmap < kBitmapLdsMax ? bitmap : kBitmapLdsMax);
        c.lds_bytes = small + static_cast<size_t>(c.lds_bitmap_bytes);
    } else if (bi_masks_bytes(p_cap) <= kLdsPerBlockMax) {
        c.lds_bytes = bi_masks_bytes(p_cap);             // bit sets in LDS, lists and counters in the slot
    }
    c.slot_bytes = bi_slot_bytes(p_cap, q_cap, c.lds);
}

static Layout make_layout(int call, int model, int64_t n, int32_t p_max, int32_t q_max, const prs_tuning *tuning = nullptr)
{
    Layout L;
    const bool sched = call == PRS_CALL_SCHEDULE;
    L.header = 0;
    L.order = plan_header_bytes();
    L.retry = L.order + align256(static_cast<size_t>(n < 1 ? 1 : n) * 4);
    size_t off = L.retry + align256(static_cast<size_t>(n < 1 ? 1 : n) * 4);
    // which configurations go where
    const int32_t plim[kClasses - 1] = {64, 128, 256, 512, 1024};
    for (int k = 0; k < kClasses - 1; ++k) L.limits.p[k] = plim[k];
    L.limits.q = kGroupQMax;
    L.limits.by_work = 0;
    for (int k = 0; k < kClasses - 1; ++k) L.limits.work[k] = 0;
    L.limits.giant_log2 = kGiantLog2;
    L.limits.wide_p = 0;
    L.wide.grid = 0; L.wide.slot_bytes = 0; L.wide.slot_offset = 0;
    static const int group_lpc[kClasses - 1] = {1, 2, 4, 8, 16};
    if (model == PRS_UNI) {
        // classes by number of pairs (1, 4 or 8, 16 or 32 lanes per configuration), all run by one launch,
        // described by class 0
        L.limits.by_work = 1;
        for (int k = 0; k < kClasses - 1; ++k) {
            const int g = k < kUniGroupSizes ? k : kUniGroupSizes - 1;
            L.limits.work[k] = sched ? kUniWorkSched[g] : kUniWork[g];
        }
        if (tuning) {                                              // never changes a result, only who runs what
            const int64_t a = tuning->uni_group_pairs[0], b = tuning->uni_group_pairs[1], c3 = tuning->uni_group_pairs[2];
            if (a >= 0 && b >= a && c3 >= b) {
                L.limits.work[0] = a; L.limits.work[1] = b;
                for (int k = 2; k < kClasses - 1; ++k) L.limits.work[k] = c3;
            }
            if (tuning->uni_wave_log2 > 0 && tuning->uni_wave_log2 < kWorkBuckets) L.limits.giant_log2 = tuning->uni_wave_log2;
        }
        for (int k = 0; k < kClasses; ++k) {
            ClassSpec &c = L.cls[k];
            c.q_cap = q_max;
            c.kind = sched ? kUniSched : kUniTimes; c.lpc = 0; c.rows_per_group = 0; c.lds = true; c.lds_bitmap_bytes = 0;
            c.p_cap = (p_max + 15) / 16 * 16;                    // keeps every per-lane array 64-byte aligned
            c.lds_bytes = sched ? uni_sched_lds_bytes() : uni_times_lds_bytes();
            c.slot_bytes = k != 0 ? 0 : (sched ? uni_sched_slot_bytes(c.p_cap) : uni_times_slot_bytes(c.p_cap));
            int64_t g = static_cast<int64_t>(kLdsPerCU / c.lds_bytes) * kCUs;
            while (g > 1 && static_cast<size_t>(g) * c.slot_bytes > kMaxWorkspace) g /= 2;
            c.grid = k == 0 ? static_cast<int>(g) : 0;
            c.slot_offset = off;
            off += align256(static_cast<size_t>(c.grid) * c.slot_bytes);
        }
        // completion times of machines with thousands of processors: a block per configuration
        if (!sched) {
            int32_t wide_p = kUniWideProcs;
            if (tuning && tuning->uni_wide_procs > 0) wide_p = tuning->uni_wide_procs;
            if (p_max >= wide_p) L.limits.wide_p = wide_p;
            {                                                          // its slots are always there: the size of the workspace does not depend on the tuning
                ClassSpec &c = L.wide;
                c.kind = kUniWide; c.p_cap = p_max; c.q_cap = q_max; c.lds = true; c.lds_bytes = uni_wide_lds_bytes();
                c.lds_bitmap_bytes = 0; c.lpc = 0; c.rows_per_group = 0;
                c.slot_bytes = uni_wide_slot_bytes(p_max);
                int64_t g = 2 * kCUs;
                while (g > 1 && static_cast<size_t>(g) * c.slot_bytes > (static_cast<size_t>(1) << 30)) g /= 2;   // at most 1 GiB of the workspace
                if (g > n) g = n < 1 ? 1 : n;
                c.grid = static_cast<int>(g);
                c.slot_offset = off;
                off += align256(static_cast<size_t>(c.grid) * c.slot_bytes);
            }
        }
        L.total = off;
        return L;
    }
    for (int k = 0; k < kClasses; ++k) {
        ClassSpec &c = L.cls[k];
        const bool last = k == kClasses - 1;
        c.p_cap = last ? p_max : (L.limits.p[k] < p_max ? L.limits.p[k] : p_max);
        c.q_cap = q_max;
        c.lds = false; c.lds_bytes = 0; c.lds_bitmap_bytes = 0; c.slot_bytes = 0; c.lpc = 0; c.rows_per_group = 0;
        const bool possible = last || k == 0 || L.limits.p[k - 1] < p_max;   // can a configuration land here?
        if (!last) {
            // several configurations per wavefront; the slot of a wavefront holds the sent-bit rows of its groups
            c.kind = kBiGroup;
            c.lpc = group_lpc[k];
            c.lds = true;
            c.lds_bytes = bi_group_lds_bytes(c.lpc);
            const int32_t q_cap = q_max < kGroupQMax ? q_max : kGroupQMax;
            c.rows_per_group = static_cast<size_t>(q_cap) * c.lpc;
            c.slot_bytes = c.rows_per_group * 8 * (64 / c.lpc);
        } else if (p_max > L.limits.p[kClasses - 2] && bi_block_lds_bytes(c.p_cap) <= kLdsPerBlockMax) {
            // thousands of processors: one block of 16 wavefronts per configuration, bit sets in LDS
            c.kind = kBiBlock;
            c.lds_bytes = bi_block_lds_bytes(c.p_cap);
            c.slot_bytes = bi_block_slot_bytes(c.p_cap, q_max);
        } else {
            // one configuration per wavefront: many segments on a small machine, or more processors than the block
            // kernel's LDS holds
            general_spec(c, c.p_cap, q_max);
        }
        int64_t g;
        if (c.kind == kBiBlock) {
            g = 2 * kCUs;
        } else if (c.lds) {
            int64_t per_cu = static_cast<int64_t>(kLdsPerCU / (c.lds_bytes < 1024 ? 1024 : c.lds_bytes));
            if (per_cu > kMaxBlocksPerCU) per_cu = kMaxBlocksPerCU;
            if (per_cu < 1) per_cu = 1;
            g = per_cu * kCUs;
        } else {
            g = kGlobalClassGrid;
        }
        while (g > 256 && static_cast<size_t>(g) * c.slot_bytes > kMaxWorkspace) g /= 2;   // big slots: fewer resident blocks
        if (g > n) g = n < 1 ? 1 : n;
        if (!possible) g = 0;
        c.grid = static_cast<int>(g);
        if (!last) L.bi_on[k] = possible;
    }
    // the group classes share one resident set of blocks, carried by class 0: as many as the largest LDS
    // allocation of a usable class allows (their slots of sent-bit rows have the same size)
    {
        int g = 0;
        for (int k = 0; k < kClasses - 1; ++k)
            if (L.bi_on[k] && (g == 0 || L.cls[k].grid < g)) g = L.cls[k].grid;
        for (int k = 0; k < kClasses - 1; ++k) L.cls[k].grid = k == 0 ? g : 0;
    }
    for (int k = 0; k < kClasses; ++k) {
        ClassSpec &c = L.cls[k];
        c.slot_offset = off;
        off += align256(static_cast<size_t>(c.grid) * c.slot_bytes);
    }
    // reruns come from the group classes only: at most 1024 processors and 1023 segments
    {
        ClassSpec &c = L.rerun;
        general_spec(c, p_max < L.limits.p[kClasses - 2] ? p_max : L.limits.p[kClasses - 2], q_max < kGroupQMax ? q_max : kGroupQMax);
        int64_t g = kGlobalClassGrid;
        if (c.lds) {
            int64_t per_cu = static_cast<int64_t>(kLdsPerCU / (c.lds_bytes < 1024 ? 1024 : c.lds_bytes));
            if (per_cu > kMaxBlocksPerCU) per_cu = kMaxBlocksPerCU;
            if (per_cu < 1) per_cu = 1;
            g = per_cu * kCUs;
        }
        if (g > n) g = n < 1 ? 1 : n;
        c.grid = static_cast<int>(g);
        c.slot_offset = off;
        off += align256(static_cast<size_t>(c.grid) * c.slot_bytes);
    }
    L.total = off;
    return L;
}

static bool bad_common(const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max)
{
    if (!cfg || n < 0 || n >= (INT64_C(1) << 31) || (model != PRS_UNI && model != PRS_BI) ||
        (cost != PRS_COST_I64 && cost != PRS_COST_F64))
        return true;
    if (p_max < 2 || p_max > (1 << 20) || q_max < 1 || q_max > (1 << 20)) return true;
    if (n > 0 && (!cfg->p || !cfg->q_req || !cfg->m || !cfg->alpha || !cfg->beta || !cfg->gamma)) return true;
    return false;
}

static int run_greedy(int call, const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max,
                      const TimesOut &times, const SchedOut &sched, void *workspace, size_t workspace_bytes, void *stream,
                      const prs_tuning *tuning, int32_t comp_m = 0)
{
    if (comp_m > 0 && (call != PRS_CALL_SIMULATE || model != PRS_UNI)) return PRS_EINVAL;   // compositions: uni-greedy times only
    if (n == 0) return PRS_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PRS_EINVAL;
    const Layout lay = make_layout(call, model, n, p_max, q_max, tuning);
    if (workspace_bytes < lay.total) return PRS_ENOSPC;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    PlanLaunch P;
    P.cfg = ConfigArrays{cfg->p, cfg->q_req, cfg->m, cfg->alpha, cfg->beta, cfg->gamma};
    P.cfg.comp_m = comp_m;
    P.n = n; P.p_max = p_max; P.q_max = q_max; P.cost = cost;
    P.limits = lay.limits;
    P.header = reinterpret_cast<PlanHeader *>(ws + lay.header);
    P.order = reinterpret_cast<int32_t *>(ws + lay.order);
    P.stream = st;
    if (launch_plan(P) != hipSuccess) return PRS_EDEVICE;
    int32_t *retry = reinterpret_cast<int32_t *>(ws + lay.retry);
    auto general = [&](const ClassSpec &c, const int32_t *order, int cls) {          // batch / general kernels
        UniLaunch L;
        L.cfg = P.cfg;
        L.p_max = p_max; L.q_max = q_max; L.model = model; L.cost = cost;
        L.want_schedule = call == PRS_CALL_SCHEDULE;
        L.times = times; L.sched = sched;
        L.plan = P.header; L.order = order; L.cls = cls;
        L.lds_p = c.lds ? c.p_cap : 0;
        L.lds_bitmap_bytes = c.lds_bitmap_bytes;
        L.lds_bytes = c.lds_bytes;
        L.slots = ws + c.slot_offset;
        L.slot_bytes = c.slot_bytes;
        L.slot_p = c.p_cap; L.slot_q = c.q_cap;
        L.grid = c.grid;
        L.stream = st;
        if (c.kind == kUniTimes) return launch_uni_times(L);
        if (c.kind == kUniSched) return launch_uni_sched(L);
        if (c.kind == kBiBlock) return launch_bi_block(L);
        if (c.kind == kUniWide) return launch_uni_wide(L);
        return launch_bi(L);
    };
    // the class with the longest-running configurations first; a class without configurations ends at once
    if (lay.limits.wide_p > 0 && general(lay.wide, P.order, kWideClass) != hipSuccess) return PRS_EDEVICE;
    bool groups_done = false;
    for (int k = kClasses - 1; k >= 0; --k) {
        const ClassSpec &c = lay.cls[k];
        if (c.grid == 0) continue;                       // no configuration can fall in this class
        if (c.kind == kBiGroup) {
            if (groups_done) continue;                   // the group sizes share one launch
            groups_done = true;
            BiGroupLaunch G;
            G.cfg = P.cfg; G.p_max = p_max; G.q_max = q_max; G.model = model; G.cost = cost;
            G.want_schedule = call == PRS_CALL_SCHEDULE;
            G.times = times; G.sched = sched; G.plan = P.header; G.order = P.order;
            G.retry = retry;
            // one resident set of blocks (class 0 carries its size and the sent-bit rows), split between the
            // classes the blocks start with
            const ClassSpec &c0 = lay.cls[0];
            int total = c0.grid, enabled = 0;
            static const int share[kBiGroupSizes] = {2, 2, 3, 6, 7};      // twentieths of the blocks that start with class 0 .. 4 (measured; flat around these)
            for (int g = 0; g < kBiGroupSizes; ++g) {
                G.parts.on[g] = lay.cls[g].kind == kBiGroup && lay.cls[g].lpc > 0 && lay.cls[g].rows_per_group > 0 && lay.bi_on[g];
                G.parts.rows_per_group[g] = lay.cls[g].rows_per_group;
                const int cap = bi_group_list_capacity(lay.cls[g].lpc > 0 ? lay.cls[g].lpc : 1);
                G.parts.list_entries[g] = (tuning && tuning->bi_list_entries > 0 && tuning->bi_list_entries < cap) ? tuning->bi_list_entries : cap;
                if (G.parts.on[g]) enabled += share[g];
            }
            int given = 0;
            for (int g = kBiGroupSizes - 1; g >= 0; --g) {
                G.parts.start[g] = G.parts.on[g] ? total * share[g] / enabled : 0;
                given += G.parts.start[g];
            }
            for (int g = kBiGroupSizes - 1; g >= 0; --g)
                if (G.parts.on[g]) { G.parts.start[g] += total - given; break; }   // rounding remainder
            G.parts.rows = reinterpret_cast<uint64_t *>(ws + c0.slot_offset);
            G.parts.rows_per_block = c0.slot_bytes / 8;
            G.stream = st;
            if (launch_bi_group(G) != hipSuccess) return PRS_EDEVICE;
        } else if (general(c, P.order, k) != hipSuccess) {
            return PRS_EDEVICE;
        }
    }
    // bi-greedy configurations whose list of running groups did not fit go through the general kernel
    if (model == PRS_BI && general(lay.rerun, retry, kRetryClass) != hipSuccess) return PRS_EDEVICE;
    return PRS_OK;
}

// ---- best segmentation per algorithm: candidates q_req = 2^c, c < n_cand, for every problem ----------
template <typename T>
__global__ void search_expand(ConfigArrays in, int64_t n, int n_cand, int32_t *p, int32_t *q_req, int64_t *m, T *alpha, T *beta,
                              T *gamma)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= n * n_cand) return;
    const int64_t i = idx / n_cand;
    const int c = static_cast<int>(idx - i * n_cand);
    p[idx] = in.p[i];
    q_req[idx] = 1 << c;
    m[idx] = in.m[i];
    alpha[idx] = static_cast<const T *>(in.alpha)[i];
    beta[idx] = static_cast<const T *>(in.beta)[i];
    gamma[idx] = static_cast<const T *>(in.gamma)[i];
}

struct BestOut {
    void *T[4];
    int32_t *q[4];
    int32_t *cfg_status;
};

template <typename T>
__global__ void search_pick(int64_t n, int n_cand, const T *greedy, const T *pipeline, const T *binary, const T *revopt,
                            const int32_t *status, BestOut out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const T *col[4] = {greedy, pipeline, binary, revopt};
    const int32_t st = status[i * n_cand];                         // the problem itself: candidate q_req = 1
    if (out.cfg_status) out.cfg_status[i] = st;
    for (int a = 0; a < 4; ++a) {
        T best = CostTraits<T>::bad();
        int32_t best_q = -1;
        if (st == PRS_CFG_OK) {
            for (int c = 0; c < n_cand; ++c) {
                if (status[i * n_cand + c] != PRS_CFG_OK) continue;
                const T v = col[a][i * n_cand + c];
                if (best_q < 0 || v < best) { best = v; best_q = 1 << c; }
            }
        }
        if (out.T[a]) static_cast<T *>(out.T[a])[i] = best;
        if (out.q[a]) out.q[a][i] = best_q;
    }
}

static int search_candidates(int32_t q_max)
{
    int c = 1;
    while ((INT64_C(1) << c) <= q_max) ++c;
    return c;                                                      // 1, 2, ..., 2^(c-1) <= q_max
}

struct SearchLayout {
    int n_cand;
    int64_t n_exp;
    size_t p, q_req, m, alpha, beta, gamma, greedy, pipeline, binary, revopt, status, sim, total;
};

static SearchLayout make_search_layout(int model, int64_t n, int32_t p_max, int32_t q_max)
{
    SearchLayout S;
    S.n_cand = search_candidates(q_max);
    S.n_exp = (n < 1 ? 1 : n) * S.n_cand;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
    const size_t e = static_cast<size_t>(S.n_exp);
    S.p = take(e * 4); S.q_req = take(e * 4); S.m = take(e * 8);
    S.alpha = take(e * 8); S.beta = take(e * 8); S.gamma = take(e * 8);
    S.greedy = take(e * 8); S.pipeline = take(e * 8); S.binary = take(e * 8); S.revopt = take(e * 8);
    S.status = take(e * 4);
    S.sim = off;
    S.total = off + make_layout(PRS_CALL_SIMULATE, model, S.n_exp, p_max, q_max).total;
    return S;
}

// ---- every segmentation of a short message (Section 8) --------------------------------------------
struct UnequalOut {
    void *T_best; uint32_t *cuts_best; int32_t *n_best;
    void *T_equi; uint32_t *cuts_equi; int32_t *equi_optimal; int32_t *cfg_status;
};

// Equal sizes except a last segment that may be smaller: returns that size, or 0 if the composition is not of this kind.
__device__ __forceinline__ int equal_but_last(uint32_t comp)
{
    const int s = comp_first(comp);
    comp >>= s;
    while (comp != 0) {
        const int z = comp_first(comp);
        comp >>= z;
        if (z != s && !(comp == 0 && z < s)) return 0;
    }
    return s;
}

constexpr int kPickThreads = 256;

// One block per problem: minima over its 2^(m-1) times, ties to the smallest cut pattern.
template <typename T>
__global__ __launch_bounds__(kPickThreads) void unequal_pick(ConfigArrays in, int32_t p_max, int32_t m_max, const T *times,
                                                             const int32_t *status, UnequalOut out)
{
    __shared__ T sBest[kPickThreads], sEqui[kPickThreads];
    __shared__ uint32_t sBestC[kPickThreads], sEquiC[kPickThreads];
    const int64_t i = blockIdx.x;
    const int tid = static_cast<int>(threadIdx.x);
    const int bits = m_max - 1;
    const int64_t base = i << bits;
    const int64_t m = in.m[i];
    const int32_t st = status[base];                               // pattern 0 is a segmentation of every valid problem
    if (st != PRS_CFG_OK) {
        if (tid == 0) {
            if (out.cfg_status) out.cfg_status[i] = st;
            if (out.T_best) static_cast<T *>(out.T_best)[i] = CostTraits<T>::bad();
            if (out.T_equi) static_cast<T *>(out.T_equi)[i] = CostTraits<T>::bad();
            if (out.cuts_best) out.cuts_best[i] = 0;
            if (out.cuts_equi) out.cuts_equi[i] = 0;
            if (out.n_best) out.n_best[i] = 0;
            if (out.equi_optimal) out.equi_optimal[i] = 0;
        }
        return;
    }
    const uint32_t n_comp = 1u << static_cast<int>(m - 1);
    const uint32_t closing = 1u << static_cast<int>(m - 1);
    const T kInf = CostTraits<T>::inf();
    T best = kInf, equi = kInf;
    uint32_t best_c = 0, equi_c = 0;
    for (uint32_t c = tid; c < n_comp; c += kPickThreads) {        // rising patterns: the first minimum is the smallest pattern
        const T v = times[base + c];
        if (v < best) { best = v; best_c = c; }
        const int s = equal_but_last(c | closing);
        // an equi-segmentation cut from a count k has size ceil(m/k): s is such a size iff ceil(m / ceil(m/s)) == s
        if (s > 0) {
            const int64_t k = (m + s - 1) / s;
            if ((m + k - 1) / k == s && v < equi) { equi = v; equi_c = c; }
        }
    }
    sBest[tid] = best; sBestC[tid] = best_c; sEqui[tid] = equi; sEquiC[tid] = equi_c;
    __syncthreads();
    for (int t = 0; t < kPickThreads; ++t) {                        // every thread folds the whole table: all end with the same minima
        const T b = sBest[t];
        if (b < best || (b == best && sBestC[t] < best_c)) { best = b; best_c = sBestC[t]; }
        const T e = sEqui[t];
        if (e < equi || (e == equi && sEquiC[t] < equi_c)) { equi = e; equi_c = sEquiC[t]; }
    }
    // second pass: how many segmentations reach the minimum, and whether one of them has equal sizes but the last
    int cnt = 0, wide = 0;
    for (uint32_t c = tid; c < n_comp; c += kPickThreads) {
        if (times[base + c] == best) {
            ++cnt;
            if (equal_but_last(c | closing) > 0) wide = 1;
        }
    }
    __shared__ int sCnt[kPickThreads], sWide[kPickThreads];
    sCnt[tid] = cnt; sWide[tid] = wide;
    __syncthreads();
    if (tid == 0) {
        int total = 0, any_wide = 0;
        for (int t = 0; t < kPickThreads; ++t) { total += sCnt[t]; any_wide |= sWide[t]; }
        if (out.cfg_status) out.cfg_status[i] = PRS_CFG_OK;
        if (out.T_best) static_cast<T *>(out.T_best)[i] = best;
        if (out.cuts_best) out.cuts_best[i] = best_c;
        if (out.n_best) out.n_best[i] = total;
        if (out.T_equi) static_cast<T *>(out.T_equi)[i] = equi;
        if (out.cuts_equi) out.cuts_equi[i] = equi_c;
        if (out.equi_optimal) out.equi_optimal[i] = (equi == best ? 1 : 0) | (any_wide ? 2 : 0);
    }
}

struct UnequalLayout {
    int64_t n_exp;
    size_t times, status, sim, total;
};

static UnequalLayout make_unequal_layout(int64_t n, int32_t p_max, int32_t m_max)
{
    UnequalLayout U;
    U.n_exp = (n < 1 ? 1 : n) << (m_max - 1);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
    U.times = take(static_cast<size_t>(U.n_exp) * 8);
    U.status = take(static_cast<size_t>(U.n_exp) * 4);
    U.sim = off;
    U.total = off + make_layout(PRS_CALL_SIMULATE, PRS_UNI, U.n_exp, p_max, m_max).total;
    return U;
}

constexpr int kUnequalMaxM = 24;

}  // namespace prs

using namespace prs;

extern "C" {

int prs_abi_version(void) { return 2; }

size_t prs_workspace_bytes(int call, int model, int cost, int64_t n, int32_t p_max, int32_t q_max)
{
    (void)cost;
    if (n < 0 || p_max < 2 || q_max < 1) return 0;
    if (call == PRS_CALL_REPLAY) return replay_workspace_bytes(p_max, q_max);
    if (call == PRS_CALL_OFFSETS) return kHeaderBytes;
    if (call == PRS_CALL_SEARCH) return make_search_layout(model, n, p_max, q_max).total;
    if (call == PRS_CALL_UNEQUAL) {
        if (q_max > kUnequalMaxM || (n << (q_max - 1)) >= (INT64_C(1) << 31)) return 0;
        return make_unequal_layout(n, p_max, q_max).total;
    }
    if (call != PRS_CALL_SIMULATE && call != PRS_CALL_SCHEDULE) return 0;
    return make_layout(call, model, n, p_max, q_max).total;
}

int simulate_completion_batch(const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max,
                              const prs_times *out, void *workspace, size_t workspace_bytes, void *stream,
                              const prs_tuning *tuning)
{
    if (bad_common(cfg, n, model, cost, p_max, q_max) || !out) return PRS_EINVAL;
    TimesOut t{out->greedy, out->binomial, out->pipeline, out->binary, out->revopt,
               out->butterfly, out->lower_bound, out->q_eff, out->cfg_status};
    SchedOut s{};
    return run_greedy(PRS_CALL_SIMULATE, cfg, n, model, cost, p_max, q_max, t, s, workspace, workspace_bytes, stream, tuning);
}

int optimal_segmentation_batch(const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max,
                               const prs_best *out, void *workspace, size_t workspace_bytes, void *stream,
                               const prs_tuning *tuning)
{
    if (!cfg || !out || n < 0 || n >= (INT64_C(1) << 26) || (model != PRS_UNI && model != PRS_BI) ||
        (cost != PRS_COST_I64 && cost != PRS_COST_F64) || p_max < 2 || p_max > (1 << 20) || q_max < 1 || q_max > (1 << 20))
        return PRS_EINVAL;
    if (n > 0 && (!cfg->p || !cfg->m || !cfg->alpha || !cfg->beta || !cfg->gamma)) return PRS_EINVAL;
    if (n == 0) return PRS_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PRS_EINVAL;
    const SearchLayout S = make_search_layout(model, n, p_max, q_max);
    if (workspace_bytes < S.total) return PRS_ENOSPC;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const ConfigArrays in{cfg->p, nullptr, cfg->m, cfg->alpha, cfg->beta, cfg->gamma};
    int32_t *ep = reinterpret_cast<int32_t *>(ws + S.p), *eq = reinterpret_cast<int32_t *>(ws + S.q_req);
    int64_t *em = reinterpret_cast<int64_t *>(ws + S.m);
    const int64_t n_exp = n * S.n_cand;
    const unsigned blocks = static_cast<unsigned>((n_exp + 255) / 256);
    if (cost == PRS_COST_I64)
        hipLaunchKernelGGL((search_expand<int64_t>), dim3(blocks), dim3(256), 0, st, in, n, S.n_cand, ep, eq, em,
                           reinterpret_cast<int64_t *>(ws + S.alpha), reinterpret_cast<int64_t *>(ws + S.beta),
                           reinterpret_cast<int64_t *>(ws + S.gamma));
    else
        hipLaunchKernelGGL((search_expand<double>), dim3(blocks), dim3(256), 0, st, in, n, S.n_cand, ep, eq, em,
                           reinterpret_cast<double *>(ws + S.alpha), reinterpret_cast<double *>(ws + S.beta),
                           reinterpret_cast<double *>(ws + S.gamma));
    if (hipGetLastError() != hipSuccess) return PRS_EDEVICE;
    const prs_configs exp_cfg{ep, eq, em, ws + S.alpha, ws + S.beta, ws + S.gamma};
    TimesOut t{ws + S.greedy, nullptr, ws + S.pipeline, ws + S.binary, ws + S.revopt, nullptr, nullptr, nullptr,
               reinterpret_cast<int32_t *>(ws + S.status)};
    SchedOut s{};
    const int rc = run_greedy(PRS_CALL_SIMULATE, &exp_cfg, n_exp, model, cost, p_max, q_max, t, s, ws + S.sim,
                              workspace_bytes - S.sim, stream, tuning);
    if (rc != PRS_OK) return rc;
    BestOut b{{out->T_greedy, out->T_pipeline, out->T_binary, out->T_revopt},
              {out->q_greedy, out->q_pipeline, out->q_binary, out->q_revopt}, out->cfg_status};
    const unsigned pblocks = static_cast<unsigned>((n + 255) / 256);
    if (cost == PRS_COST_I64)
        hipLaunchKernelGGL((search_pick<int64_t>), dim3(pblocks), dim3(256), 0, st, n, S.n_cand,
                           reinterpret_cast<const int64_t *>(ws + S.greedy), reinterpret_cast<const int64_t *>(ws + S.pipeline),
                           reinterpret_cast<const int64_t *>(ws + S.binary), reinterpret_cast<const int64_t *>(ws + S.revopt),
                           reinterpret_cast<const int32_t *>(ws + S.status), b);
    else
        hipLaunchKernelGGL((search_pick<double>), dim3(pblocks), dim3(256), 0, st, n, S.n_cand,
                           reinterpret_cast<const double *>(ws + S.greedy), reinterpret_cast<const double *>(ws + S.pipeline),
                           reinterpret_cast<const double *>(ws + S.binary), reinterpret_cast<const double *>(ws + S.revopt),
                           reinterpret_cast<const int32_t *>(ws + S.status), b);
    return hipGetLastError() == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

int unequal_segmentation_batch(const prs_configs *cfg, int64_t n, int cost, int32_t p_max, int32_t m_max,
                               const prs_unequal *out, void *workspace, size_t workspace_bytes, void *stream,
                               const prs_tuning *tuning)
{
    if (!cfg || !out || n < 0 || (cost != PRS_COST_I64 && cost != PRS_COST_F64) || p_max < 2 || p_max > (1 << 20) ||
        m_max < 1 || m_max > kUnequalMaxM || (n << (m_max - 1)) >= (INT64_C(1) << 31))
        return PRS_EINVAL;
    if (n > 0 && (!cfg->p || !cfg->m || !cfg->alpha || !cfg->beta || !cfg->gamma)) return PRS_EINVAL;
    if (n == 0) return PRS_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PRS_EINVAL;
    const UnequalLayout U = make_unequal_layout(n, p_max, m_max);
    if (workspace_bytes < U.total) return PRS_ENOSPC;
    char *ws = static_cast<char *>(workspace);
    void *all = out->T_all ? out->T_all : static_cast<void *>(ws + U.times);
    int32_t *status = reinterpret_cast<int32_t *>(ws + U.status);
    const prs_configs problems{cfg->p, nullptr, cfg->m, cfg->alpha, cfg->beta, cfg->gamma};
    TimesOut t{all, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, status};
    SchedOut s{};
    const int rc = run_greedy(PRS_CALL_SIMULATE, &problems, U.n_exp, PRS_UNI, cost, p_max, m_max, t, s, ws + U.sim,
                              workspace_bytes - U.sim, stream, tuning, m_max);
    if (rc != PRS_OK) return rc;
    const ConfigArrays in{cfg->p, nullptr, cfg->m, cfg->alpha, cfg->beta, cfg->gamma};
    const UnequalOut u{out->T_best, out->cuts_best, out->n_best, out->T_equi, out->cuts_equi, out->equi_optimal, out->cfg_status};
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (cost == PRS_COST_I64)
        hipLaunchKernelGGL((unequal_pick<int64_t>), dim3(static_cast<unsigned>(n)), dim3(kPickThreads), 0, st, in, p_max, m_max,
                           static_cast<const int64_t *>(all), status, u);
    else
        hipLaunchKernelGGL((unequal_pick<double>), dim3(static_cast<unsigned>(n)), dim3(kPickThreads), 0, st, in, p_max, m_max,
                           static_cast<const double *>(all), status, u);
    return hipGetLastError() == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

int butterfly_threshold_batch(const int32_t *p, int64_t n, double alpha, int32_t q_max, int32_t m_log2_first,
                              int32_t m_log2_last, double ratio_lo, double ratio_hi, int32_t steps, double *ratio_below,
                              double *ratio_above, int32_t *cfg_status, void *stream)
{
    if (n < 0 || n >= (INT64_C(1) << 31) || (n > 0 && !p) || q_max < 1 || q_max > (1 << 20) || m_log2_first < 0 ||
        m_log2_last < m_log2_first || m_log2_last > 40 || steps < 0 || steps > 64)
        return PRS_EINVAL;
    if (!(alpha >= 0.0) || !(alpha < 1e300) || !(ratio_lo > 0.0) || !(ratio_hi > ratio_lo) || !(ratio_hi < 1e100)) return PRS_EINVAL;
    if (n == 0) return PRS_OK;
    ThresholdLaunch L{p, n, alpha, q_max, m_log2_first, m_log2_last, ratio_lo, ratio_hi, steps, ratio_below, ratio_above,
                      cfg_status, static_cast<hipStream_t>(stream)};
    return launch_threshold(L) == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

int prs_measure_alu_ceiling(int64_t steps_per_lane, int32_t blocks, double *sink, void *stream)
{
    if (steps_per_lane < 0 || blocks < 1 || blocks > (1 << 20) || !sink) return PRS_EINVAL;
    return launch_alu_ceiling(steps_per_lane, blocks, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

int prs_pair_offsets(const prs_configs *cfg, int64_t n, int cost, int32_t p_max, int32_t q_max, int64_t *pair_offset,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    (void)workspace; (void)workspace_bytes;
    if (bad_common(cfg, n, PRS_UNI, cost, p_max, q_max) || !pair_offset) return PRS_EINVAL;
    OffsetsLaunch L{ConfigArrays{cfg->p, cfg->q_req, cfg->m, cfg->alpha, cfg->beta, cfg->gamma}, n, p_max, q_max, cost,
                    pair_offset, static_cast<hipStream_t>(stream)};
    return launch_offsets(L) == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

int greedy_schedule_batch(const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max,
                          const int64_t *pair_offset, int64_t pair_capacity, int32_t *src, int32_t *dst, int32_t *seg,
                          void *t_start, void *T_greedy, int32_t *cfg_status, void *workspace, size_t workspace_bytes,
                          void *stream, const prs_tuning *tuning)
{
    if (bad_common(cfg, n, model, cost, p_max, q_max) || pair_capacity < 0 || (n > 0 && !pair_offset)) return PRS_EINVAL;
    TimesOut t{};
    SchedOut s{pair_offset, pair_capacity, src, dst, seg, t_start, T_greedy, cfg_status};
    return run_greedy(PRS_CALL_SCHEDULE, cfg, n, model, cost, p_max, q_max, t, s, workspace, workspace_bytes, stream, tuning);
}

// argument checks shared by the two replay entry points
static int replay_bad_arguments(int32_t p, int32_t q, const int64_t *seg_elem_offset, const int32_t *src, const int32_t *dst,
                                const int32_t *seg, int64_t n_pairs, const void *in, int64_t stride_elems, int64_t n_elems,
                                int dtype, const void *out)
{
    if (p < 2 || p > 4096 || q < 1 || q > 65536 || !seg_elem_offset || !src || !dst || !seg || !in || !out) return PRS_EINVAL;
    if (n_pairs != static_cast<int64_t>(p - 1) * q || n_pairs >= (INT64_C(1) << 31)) return PRS_EINVAL;
    const int elem = dtype & 0xFF, op = dtype & ~0xFF;
    if ((elem != PRS_I32 && elem != PRS_F32 && elem != PRS_F64 && elem != PRS_I64) || (op != PRS_OP_SUM && op != PRS_OP_MAX))
        return PRS_EINVAL;
    if (n_elems < 0 || stride_elems < n_elems) return PRS_EINVAL;
    if (seg_elem_offset[0] != 0 || seg_elem_offset[q] != n_elems) return PRS_EINVAL;
    for (int k = 0; k < q; ++k)
        if (seg_elem_offset[k + 1] < seg_elem_offset[k]) return PRS_EINVAL;
    return PRS_OK;
}

int replay_reduction_static(int32_t p, int32_t q, const int64_t *seg_elem_offset, const int32_t *src, const int32_t *dst,
                            const int32_t *seg, int64_t n_pairs, const void *in, int64_t stride_elems, int64_t n_elems,
                            int dtype, void *out, int32_t *status, void *stream)
{
    const int bad = replay_bad_arguments(p, q, seg_elem_offset, src, dst, seg, n_pairs, in, stride_elems, n_elems, dtype, out);
    if (bad != PRS_OK) return bad;
    if (replay_scratch_bytes(p, q) > kReplayStaticBytes) return PRS_ENOSPC;       // too many processors x segments for the fixed array
    void *ws = nullptr;
    if (replay_static_scratch(&ws) != hipSuccess) return PRS_EDEVICE;
    ReplayLaunch L{p, q, seg_elem_offset, src, dst, seg, n_pairs, in, stride_elems, n_elems, dtype & 0xFF, dtype & ~0xFF, out, status,
                   static_cast<char *>(ws), static_cast<hipStream_t>(stream)};
    return launch_replay(L) == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

int replay_reduction(int32_t p, int32_t q, const int64_t *seg_elem_offset, const int32_t *src, const int32_t *dst,
                     const int32_t *seg, int64_t n_pairs, const void *in, int64_t stride_elems, int64_t n_elems, int dtype,
                     void *out, int32_t *status, void *workspace, size_t workspace_bytes, void *stream)
{
    if (p < 2 || p > 4096 || q < 1 || q > 65536 || !seg_elem_offset || !src || !dst || !seg || !in || !out) return PRS_EINVAL;
    if (n_pairs != static_cast<int64_t>(p - 1) * q || n_pairs >= (INT64_C(1) << 31)) return PRS_EINVAL;
    const int elem = dtype & 0xFF, op = dtype & ~0xFF;
    if ((elem != PRS_I32 && elem != PRS_F32 && elem != PRS_F64 && elem != PRS_I64) || (op != PRS_OP_SUM && op != PRS_OP_MAX))
        return PRS_EINVAL;
    if (n_elems < 0 || stride_elems < n_elems) return PRS_EINVAL;
    if (seg_elem_offset[0] != 0 || seg_elem_offset[q] != n_elems) return PRS_EINVAL;
    for (int k = 0; k < q; ++k)
        if (seg_elem_offset[k + 1] < seg_elem_offset[k]) return PRS_EINVAL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PRS_EINVAL;
    if (workspace_bytes < replay_workspace_bytes(p, q)) return PRS_ENOSPC;
    ReplayLaunch L{p, q, seg_elem_offset, src, dst, seg, n_pairs, in, stride_elems, n_elems, elem, op, out, status,
                   static_cast<char *>(workspace), static_cast<hipStream_t>(stream)};
    return launch_replay(L) == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

}  // extern "C"
