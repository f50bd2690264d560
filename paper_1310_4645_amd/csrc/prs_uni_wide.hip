// Uni-greedy completion times (Lowery & Langou, Algorithm 1, Section 5) for machines of thousands of processors on
// gfx950: one block of 16 wavefronts per configuration, many pairs of a segment at once.
//
// A step of Algorithm 1 takes the two smallest ready times of the remaining set; the sender leaves with
// t + tcomm, the receiver comes back with (t + tcomm) + tcomp, t the larger of the two.  The remaining set is the
// unread tail of the segment's sorted input stream A merged with the unread tail of B, the values of the receivers of
// earlier pairs (sorted as well, t never decreases).  No value a later pair puts into B can be smaller than
// bound = (t_next + tcomm) + tcomp, t_next the start of the next pair.  So every remaining value up to that bound is
// paired exactly as Algorithm 1 would pair it, one after the other, whatever the pairs before it produce: the
// merged sequence of those values is cut into consecutive pairs, and all of them are computed in one go.  On a
// machine of tens of thousands of processors a thousand pairs fit under the bound.
//
// Per round the block loads the next 1024 values of A and of B into LDS, takes the values up to
// min(bound, last loaded value of a stream that has more) -- a prefix of the merged order --, thread i finds the
// (2i+1)-th of them by a merge-path search and writes pair i's two results.  Values only: which processor sends
// does not enter any time.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kWideThreads = 1024;
constexpr int kWideWaves = kWideThreads / kWave;
constexpr int kWideTile = kWideThreads;          // values of A and of B looked at per round

size_t uni_wide_slot_bytes(int32_t p_cap) { return 3 * ((static_cast<size_t>(p_cap) * 8 + 255) / 256 * 256); }
size_t uni_wide_lds_bytes() { return static_cast<size_t>(kWideTile) * 8 * 2 + 256; }

// number of X among the first k values of the merge of X[0..nx) and Y[0..ny) (sorted; X first among equals)
template <typename T> __device__ __forceinline__ int merge_rank(const T *X, int nx, const T *Y, int ny, int k)
{
    int lo = k - ny > 0 ? k - ny : 0, hi = k < nx ? k : nx;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (X[mid] <= Y[k - 1 - mid]) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <typename T>
__device__ T run_uni_wide(const Config<T> &c, char *lds, T *bufA, T *bufOut, T *bufB, int32_t *status)
{
    const int tid = static_cast<int>(threadIdx.x), lane = lane_id(), wave = tid >> 6;
    T *tA = reinterpret_cast<T *>(lds), *tB = tA + kWideTile;
    int32_t *part = reinterpret_cast<int32_t *>(tB + kWideTile);         // [2][kWideWaves]
    const int p = c.p, q = c.q;
    const T kInf = CostTraits<T>::inf();
    T *A = bufA, *Out = bufOut, *B = bufB;
    for (int i = tid; i < p; i += kWideThreads) A[i] = 0;
    __threadfence_block();
    __syncthreads();
    T result = 0;
    for (int k = 0; k < q; ++k) {
        const T cc = c.c(k), gg = c.g(k);
        int a = 0, b = 0, nB = 0;                       // values of A and B consumed; pairs done = values of B produced
        while (nB < p - 1) {
            const int lenA = p - a, lenB = nB - b;
            const int nA = lenA < kWideTile ? lenA : kWideTile, nBt = lenB < kWideTile ? lenB : kWideTile;
            const T va = tid < nA ? A[a + tid] : kInf, vb = tid < nBt ? B[b + tid] : kInf;
            tA[tid] = va; tB[tid] = vb;
            __syncthreads();
            // start of the next pair: the second smallest remaining value
            const T a0 = tA[0], a1 = tA[1], b0 = tB[0], b1 = tB[1];
            const bool x = a0 <= b0;
            const T u = x ? a1 : a0, v = x ? b0 : b1;
            const T t2 = u <= v ? u : v;
            T limit = wrap_add<T>(wrap_add<T>(t2, cc), gg);
            if (nA < lenA) { const T e = tA[nA - 1]; limit = e < limit ? e : limit; }      // more of A than loaded
            if (nBt < lenB) { const T e = tB[nBt - 1]; limit = e < limit ? e : limit; }
            // how many loaded values lie under the limit (both streams are sorted: a count per stream)
            int cntA = wave_sum(va <= limit ? 1 : 0), cntB = wave_sum(vb <= limit ? 1 : 0);
            if (lane == 0) { part[wave] = cntA; part[kWideWaves + wave] = cntB; }
            __syncthreads();
            cntA = 0; cntB = 0;
#pragma unroll
            for (int w = 0; w < kWideWaves; ++w) { cntA += part[w]; cntB += part[kWideWaves + w]; }
            const int np = (cntA + cntB) >> 1;          // at least one: the two smallest are under the limit
            if (np == 0) { *status = PRS_CFG_STALLED; return CostTraits<T>::bad(); }   // (never with finite times; ends the loop for all threads alike)
            if (tid < np) {
                const int kk = 2 * tid + 1;              // the later value of pair tid starts it
                const int ia = merge_rank<T>(tA, cntA, tB, cntB, kk), ib = kk - ia;
                const bool fromA = ia < cntA && (ib >= cntB || tA[ia] <= tB[ib]);
                const T t = fromA ? tA[ia] : tB[ib];
                const T ts = wrap_add<T>(t, cc), tr = wrap_add<T>(ts, gg);
                Out[nB + tid] = ts;                     // the sender leaves the segment
                B[nB + tid] = tr;                       // the receiver stays
            }
            const int ca = merge_rank<T>(tA, cntA, tB, cntB, 2 * np);
            a += ca; b += 2 * np - ca; nB += np;
            __threadfence_block();
            __syncthreads();
        }
        // the root is what remains: the receiver of the last pair, the largest value
        if (tid == 0) Out[p - 1] = B[p - 2];
        __threadfence_block();
        __syncthreads();
        result = Out[p - 1];
        T *sw = A; A = Out; Out = sw;
    }
    return result;
}

template <typename T>
__global__ __launch_bounds__(kWideThreads) void uni_wide_kernel(ConfigArrays cfg, int32_t p_max, int32_t q_max, int model,
                                                                TimesOut times, PlanHeader *plan, const int32_t *order, int cls,
                                                                char *slots, size_t slot_bytes)
{
    PRS_DYNAMIC_LDS(lds_raw);
    __shared__ long long s_ticket;
    const int tid = static_cast<int>(threadIdx.x);
    char *slot = slots + static_cast<size_t>(blockIdx.x) * slot_bytes;
    const size_t third = slot_bytes / 3;
    const int32_t count = plan->class_count[cls], begin = plan->class_begin[cls];
    for (;;) {
        __syncthreads();
        if (tid == 0) s_ticket = static_cast<long long>(atomicAdd(&plan->ticket[cls], 1ULL));
        __syncthreads();
        const int64_t ticket = s_ticket;
        if (ticket >= count) break;
        const int64_t i = order[begin + ticket];
        const Config<T> c = decode_config<T>(cfg, i, p_max, q_max);
        T result = CostTraits<T>::bad();
        int32_t status = c.status;
        if (status == PRS_CFG_OK)
            result = run_uni_wide<T>(c, lds_raw, reinterpret_cast<T *>(slot), reinterpret_cast<T *>(slot + third),
                                     reinterpret_cast<T *>(slot + 2 * third), &status);
        if (tid == 0) {
            write_closed_forms<T>(times, i, c, model);
            if (times.cfg_status) times.cfg_status[i] = status;
            if (times.greedy) static_cast<T *>(times.greedy)[i] = status == PRS_CFG_OK ? result : CostTraits<T>::bad();
        }
    }
}

hipError_t launch_uni_wide(const UniLaunch &L)
{
    if (L.grid <= 0) return hipSuccess;
    if (L.cost == PRS_COST_I64)
        hipLaunchKernelGGL((uni_wide_kernel<int64_t>), dim3(L.grid), dim3(kWideThreads), uni_wide_lds_bytes(), L.stream, L.cfg, L.p_max,
                           L.q_max, L.model, L.times, L.plan, L.order, L.cls, L.slots, L.slot_bytes);
    else
        hipLaunchKernelGGL((uni_wide_kernel<double>), dim3(L.grid), dim3(kWideThreads), uni_wide_lds_bytes(), L.stream, L.cfg, L.p_max,
                           L.q_max, L.model, L.times, L.plan, L.order, L.cls, L.slots, L.slot_bytes);
    return hipGetLastError();
}

}  // namespace prs
