// Butterfly against bi-greedy (Lowery & Langou, Section 6.1, last paragraph and its figure) on gfx950.
//
// For a machine of p processors the section asks below which ratio beta/gamma some message size lets the butterfly
// (recursive halving and doubling, Table III) finish before the reversed optimal broadcast, whose time bi-greedy
// meets, at the best of the allowed segment counts.  Both times are the closed forms of Table III, so the line is
// found by bisection over the ratio: gamma = 1, beta = the ratio, message sizes 2^k, every segment count
// 1..min(q_max, m) cut as Section 2 says.  One block per machine; the threads share the (message size, segment
// count) grid of a step, the smallest broadcast time per message size is kept in LDS as the bit pattern of the
// (non-negative) double, which orders like the value.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kThresholdThreads = 256;
constexpr int kThresholdSizes = 64;          // message sizes 2^0 .. 2^62 at most

__global__ __launch_bounds__(kThresholdThreads) void butterfly_threshold_kernel(ThresholdLaunch L)
{
    __shared__ unsigned long long best[kThresholdSizes];       // per message size: smallest broadcast-based time (bits)
    __shared__ int wins;
    const int tid = static_cast<int>(threadIdx.x);
    const int64_t i = blockIdx.x;
    const int32_t p = L.p[i];
    if (p < 2) {
        if (tid == 0) {
            if (L.ratio_below) L.ratio_below[i] = __builtin_nan("");
            if (L.ratio_above) L.ratio_above[i] = __builtin_nan("");
            if (L.cfg_status) L.cfg_status[i] = PRS_CFG_BAD_PARAM;
        }
        return;
    }
    const int n_sizes = L.m_log2_last - L.m_log2_first + 1;
    double lo = L.ratio_lo, hi = L.ratio_hi;
    for (int step = 0; step < L.steps; ++step) {
        const double mid = lo + (hi - lo) * 0.5;
        for (int k = tid; k < n_sizes; k += kThresholdThreads) best[k] = ~0ULL;
        if (tid == 0) wins = 0;
        __syncthreads();
        for (int k = 0; k < n_sizes; ++k) {
            const int64_t m = INT64_C(1) << (L.m_log2_first + k);
            const int64_t counts = m < L.q_max ? m : L.q_max;
            double mine = __builtin_huge_val();
            for (int64_t q_req = 1 + tid; q_req <= counts; q_req += kThresholdThreads) {
                const Config<double> c = decode_values<double>(p, static_cast<int32_t>(q_req), m, L.alpha, mid, 1.0, p, L.q_max);
                const double t = revopt_time<double>(c);
                if (c.status == PRS_CFG_OK && t < mine) mine = t;
            }
            if (mine < __builtin_huge_val()) atomicMin(&best[k], static_cast<unsigned long long>(__double_as_longlong(mine)));
        }
        __syncthreads();
        for (int k = tid; k < n_sizes; k += kThresholdThreads) {
            const int64_t m = INT64_C(1) << (L.m_log2_first + k);
            const Config<double> c = decode_values<double>(p, 1, m, L.alpha, mid, 1.0, p, L.q_max);
            if (best[k] != ~0ULL && butterfly_time<double>(c) < __longlong_as_double(static_cast<long long>(best[k]))) wins = 1;
        }
        __syncthreads();
        if (wins) lo = mid; else hi = mid;                      // the same decision in every thread
        __syncthreads();
    }
    if (tid == 0) {
        if (L.ratio_below) L.ratio_below[i] = lo;
        if (L.ratio_above) L.ratio_above[i] = hi;
        if (L.cfg_status) L.cfg_status[i] = PRS_CFG_OK;
    }
}

hipError_t launch_threshold(const ThresholdLaunch &L)
{
    hipLaunchKernelGGL(butterfly_threshold_kernel, dim3(static_cast<unsigned>(L.n)), dim3(kThresholdThreads), 0, L.stream, L);
    return hipGetLastError();
}

}  // namespace prs
