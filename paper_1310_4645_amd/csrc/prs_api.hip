// C ABI of the library (declared in include/prs.h): argument checks, workspace
// carving and kernel launches.  No device memory is allocated here.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr size_t kHeaderBytes = 256;       // ticket counter at the start of the workspace
constexpr int kMaxGrid = 4096;             // wavefront-sized blocks resident at once, at most
constexpr size_t kMaxWorkspace = static_cast<size_t>(16) << 30;   // what prs_workspace_bytes asks for, at most (if 512 slots fit)

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

static int grid_for(int64_t n, size_t slot, size_t workspace_bytes)
{
    int64_t g = n < kMaxGrid ? n : kMaxGrid;
    if (g < 1) g = 1;
    if (workspace_bytes > kHeaderBytes && slot > 0) {
        const int64_t fit = static_cast<int64_t>((workspace_bytes - kHeaderBytes) / slot);
        if (fit < g) g = fit;
    } else {
        g = 0;
    }
    return static_cast<int>(g);
}

static size_t slot_bytes_for(int call, int model, int32_t p_max, int32_t q_max)
{
    if (model == PRS_UNI) return uni_slot_bytes(call == PRS_CALL_SCHEDULE, p_max);
    return bi_slot_bytes(p_max, q_max);
}

static bool bad_common(const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max)
{
    if (!cfg || n < 0 || (model != PRS_UNI && model != PRS_BI) || (cost != PRS_COST_I64 && cost != PRS_COST_F64)) return true;
    if (p_max < 2 || p_max > (1 << 20) || q_max < 1 || q_max > (1 << 20)) return true;
    if (n > 0 && (!cfg->p || !cfg->q_req || !cfg->m || !cfg->alpha || !cfg->beta || !cfg->gamma)) return true;
    return false;
}

static int run_greedy(int call, const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max,
                      const TimesOut &times, const SchedOut &sched, void *workspace, size_t workspace_bytes, void *stream)
{
    if (n == 0) return PRS_OK;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PRS_EINVAL;
    const size_t slot = slot_bytes_for(call, model, p_max, q_max);
    const int grid = grid_for(n, slot, workspace_bytes);
    if (grid < 1) return PRS_ENOSPC;
    UniLaunch L;
    L.cfg = ConfigArrays{cfg->p, cfg->q_req, cfg->m, cfg->alpha, cfg->beta, cfg->gamma};
    L.n = n; L.p_max = p_max; L.q_max = q_max; L.model = model; L.cost = cost;
    L.want_schedule = call == PRS_CALL_SCHEDULE;
    L.times = times; L.sched = sched;
    L.slots = static_cast<char *>(workspace) + kHeaderBytes;
    L.slot_bytes = slot;
    L.ticket = static_cast<unsigned long long *>(workspace);
    L.grid = grid;
    L.stream = static_cast<hipStream_t>(stream);
    if (launch_clear(L.ticket, 4, L.stream) != hipSuccess) return PRS_EDEVICE;
    const hipError_t err = model == PRS_UNI ? launch_uni(L) : launch_bi(L);
    return err == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

}  // namespace prs

using namespace prs;

extern "C" {

int prs_abi_version(void) { return 1; }

size_t prs_workspace_bytes(int call, int model, int cost, int64_t n, int32_t p_max, int32_t q_max)
{
    (void)cost;
    if (n < 0 || p_max < 2 || q_max < 1) return 0;
    if (call == PRS_CALL_REPLAY) return replay_workspace_bytes(p_max, q_max);
    if (call == PRS_CALL_OFFSETS) return kHeaderBytes;
    if (call != PRS_CALL_SIMULATE && call != PRS_CALL_SCHEDULE) return 0;
    int64_t g = n < kMaxGrid ? (n < 1 ? 1 : n) : kMaxGrid;
    const size_t slot = slot_bytes_for(call, model, p_max, q_max);
    while (g > 512 && static_cast<size_t>(g) * slot > kMaxWorkspace) g /= 2;   // fewer resident configurations when each is big
    return kHeaderBytes + static_cast<size_t>(g) * slot;
}

int simulate_completion_batch(const prs_configs *cfg, int64_t n, int model, int cost, int32_t p_max, int32_t q_max,
                              const prs_times *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (bad_common(cfg, n, model, cost, p_max, q_max) || !out) return PRS_EINVAL;
    TimesOut t{out->greedy, out->binomial, out->pipeline, out->binary, out->revopt,
               out->butterfly, out->lower_bound, out->q_eff, out->cfg_status};
    SchedOut s{};
    return run_greedy(PRS_CALL_SIMULATE, cfg, n, model, cost, p_max, q_max, t, s, workspace, workspace_bytes, stream);
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
                          void *stream)
{
    if (bad_common(cfg, n, model, cost, p_max, q_max) || pair_capacity < 0 || (n > 0 && !pair_offset)) return PRS_EINVAL;
    TimesOut t{};
    SchedOut s{pair_offset, pair_capacity, src, dst, seg, t_start, T_greedy, cfg_status};
    return run_greedy(PRS_CALL_SCHEDULE, cfg, n, model, cost, p_max, q_max, t, s, workspace, workspace_bytes, stream);
}

int replay_reduction(int32_t p, int32_t q, const int64_t *seg_elem_offset, const int32_t *src, const int32_t *dst,
                     const int32_t *seg, int64_t n_pairs, const void *in, int64_t stride_elems, int64_t n_elems, int dtype,
                     void *out, int32_t *status, void *workspace, size_t workspace_bytes, void *stream)
{
    if (p < 2 || p > 4096 || q < 1 || q > 65536 || !seg_elem_offset || !src || !dst || !seg || !in || !out) return PRS_EINVAL;
    if (n_pairs != static_cast<int64_t>(p - 1) * q || n_pairs >= (INT64_C(1) << 31)) return PRS_EINVAL;
    if (dtype != PRS_I32 && dtype != PRS_F32) return PRS_EINVAL;
    if (n_elems < 0 || stride_elems < n_elems) return PRS_EINVAL;
    if (seg_elem_offset[0] != 0 || seg_elem_offset[q] != n_elems) return PRS_EINVAL;
    for (int k = 0; k < q; ++k)
        if (seg_elem_offset[k + 1] < seg_elem_offset[k]) return PRS_EINVAL;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return PRS_EINVAL;
    if (workspace_bytes < replay_workspace_bytes(p, q)) return PRS_ENOSPC;
    ReplayLaunch L{p, q, seg_elem_offset, src, dst, seg, n_pairs, in, stride_elems, n_elems, dtype, out, status,
                   static_cast<char *>(workspace), static_cast<hipStream_t>(stream)};
    return launch_replay(L) == hipSuccess ? PRS_OK : PRS_EDEVICE;
}

}  // extern "C"
