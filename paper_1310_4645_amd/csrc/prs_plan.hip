#include "prs_plan.h"

namespace prs {

template <typename T>
__device__ __forceinline__ int plan_bucket(const ConfigArrays &cfg, int64_t i, int32_t p_max, int32_t q_max,
                                           const ClassLimits &lim)
{
    const Config<T> c = decode_config<T>(cfg, i, p_max, q_max);
    if (c.status != PRS_CFG_OK) return kWorkBuckets - 1;                 // nothing to do: lightest bucket of class 0
    const int64_t work = static_cast<int64_t>(c.p - 1) * c.q;
    int cls = kClasses - 1;
    if (lim.by_work) {
        for (int k = kClasses - 2; k >= 0; --k)
            if (work <= lim.work[k]) cls = k;
        if (lim.wide_p > 0 && c.p >= lim.wide_p && cfg.comp_m == 0) cls = kWideClass;
    } else {
        for (int k = kClasses - 2; k >= 0; --k)
            if (c.p <= lim.p[k] && c.q <= lim.q) cls = k;
    }
    int lg = 63 - __builtin_clzll(static_cast<unsigned long long>(work) | 1ULL);
    if (lg > kWorkBuckets - 1) lg = kWorkBuckets - 1;
    return cls * kWorkBuckets + (kWorkBuckets - 1 - lg);
}

__global__ void plan_clear(PlanHeader *h)
{
    const int i = threadIdx.x;
    if (i < kClasses + 1) { h->ticket[i] = 0ULL; h->class_begin[i] = 0; h->class_count[i] = 0; }
    if (i == 0) { h->giant_count = 0; h->ticket_giant = 0ULL; }
    for (int k = i; k < kPlanClasses * kWorkBuckets; k += blockDim.x) { h->hist[k] = 0; h->start[k] = 0; h->cursor[k] = 0; }
}

constexpr int kPlanThreads = 256;
constexpr int kPlanBins = kPlanClasses * kWorkBuckets;

// Both passes count inside the block first (LDS) and touch the global counters once per block and bin: with one
// global atomic per configuration, a batch of millions spends its time queueing on a few dozen addresses.
template <typename T>
__global__ __launch_bounds__(kPlanThreads) void plan_hist(ConfigArrays cfg, int64_t n, int32_t p_max, int32_t q_max, ClassLimits lim,
                                                          PlanHeader *h)
{
    __shared__ int32_t local[kPlanBins];
    const int tid = static_cast<int>(threadIdx.x);
    for (int k = tid; k < kPlanBins; k += kPlanThreads) local[k] = 0;
    __syncthreads();
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kPlanThreads + tid;
    if (i < n) atomicAdd(&local[plan_bucket<T>(cfg, i, p_max, q_max, lim)], 1);
    __syncthreads();
    for (int k = tid; k < kPlanBins; k += kPlanThreads)
        if (local[k] != 0) atomicAdd(&h->hist[k], local[k]);
}

// n_classes: kClasses, or kPlanClasses when the batch has a class of wide machines (otherwise that slot is the
// retry list of bi-greedy, which starts empty at position 0 of an array of its own)
__global__ void plan_scan(PlanHeader *h, int32_t giant_log2, int n_classes)
{
    if (threadIdx.x != 0) return;
    int32_t run = 0;
    for (int c = 0; c < n_classes; ++c) {
        h->class_begin[c] = run;
        for (int b = 0; b < kWorkBuckets; ++b) {
            h->start[c * kWorkBuckets + b] = run;
            run += h->hist[c * kWorkBuckets + b];
        }
        h->class_count[c] = run - h->class_begin[c];
    }
    int32_t giants = 0;                                   // buckets are ordered heaviest first: bucket b holds floor(log2) = kWorkBuckets-1-b
    for (int b = 0; b <= kWorkBuckets - 1 - giant_log2; ++b) giants += h->hist[(kClasses - 1) * kWorkBuckets + b];
    h->giant_count = giants;
}

template <typename T>
__global__ __launch_bounds__(kPlanThreads) void plan_scatter(ConfigArrays cfg, int64_t n, int32_t p_max, int32_t q_max, ClassLimits lim,
                                                             PlanHeader *h, int32_t *order)
{
    __shared__ int32_t local[kPlanBins];                             // configurations of this block per bin, then the bin's first slot
    const int tid = static_cast<int>(threadIdx.x);
    for (int k = tid; k < kPlanBins; k += kPlanThreads) local[k] = 0;
    __syncthreads();
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kPlanThreads + tid;
    int b = 0, rank = 0;
    if (i < n) {
        b = plan_bucket<T>(cfg, i, p_max, q_max, lim);
        rank = atomicAdd(&local[b], 1);
    }
    __syncthreads();
    for (int k = tid; k < kPlanBins; k += kPlanThreads)
        if (local[k] != 0) local[k] = h->start[k] + atomicAdd(&h->cursor[k], local[k]);
    __syncthreads();
    if (i < n) order[local[b] + rank] = static_cast<int32_t>(i);
}

hipError_t launch_plan(const PlanLaunch &L)
{
    const unsigned blocks = static_cast<unsigned>((L.n + kPlanThreads - 1) / kPlanThreads);
    hipLaunchKernelGGL(plan_clear, dim3(1), dim3(256), 0, L.stream, L.header);
    if (L.cost == PRS_COST_I64) {
        hipLaunchKernelGGL((plan_hist<int64_t>), dim3(blocks), dim3(kPlanThreads), 0, L.stream, L.cfg, L.n, L.p_max, L.q_max, L.limits, L.header);
        hipLaunchKernelGGL(plan_scan, dim3(1), dim3(64), 0, L.stream, L.header, L.limits.giant_log2, (L.limits.by_work && L.limits.wide_p > 0) ? kPlanClasses : kClasses);
        hipLaunchKernelGGL((plan_scatter<int64_t>), dim3(blocks), dim3(kPlanThreads), 0, L.stream, L.cfg, L.n, L.p_max, L.q_max, L.limits, L.header, L.order);
    } else {
        hipLaunchKernelGGL((plan_hist<double>), dim3(blocks), dim3(kPlanThreads), 0, L.stream, L.cfg, L.n, L.p_max, L.q_max, L.limits, L.header);
        hipLaunchKernelGGL(plan_scan, dim3(1), dim3(64), 0, L.stream, L.header, L.limits.giant_log2, (L.limits.by_work && L.limits.wide_p > 0) ? kPlanClasses : kClasses);
        hipLaunchKernelGGL((plan_scatter<double>), dim3(blocks), dim3(kPlanThreads), 0, L.stream, L.cfg, L.n, L.p_max, L.q_max, L.limits, L.header, L.order);
    }
    return hipGetLastError();
}

}  // namespace prs
