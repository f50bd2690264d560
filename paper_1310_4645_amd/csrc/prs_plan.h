// Work plan of a batch: configurations grouped into classes (by size or by number of pairs, so that each
// class gets the kernel variant and group size that fit it) and, inside a class, ordered from most to least work, so the
// longest-running configurations start first.  Built on the device by three small kernels; no host sync.
#pragma once

#include "prs_device.h"

namespace prs {

constexpr int kClasses = 6;          // bi-greedy: five group sizes and the general kernel; uni-greedy uses 0, 1, 2 and the last
constexpr int kWorkBuckets = 40;     // floor(log2(work)) buckets, heaviest first
constexpr int kRetryClass = kClasses; // pseudo class: configurations handed back to the general kernel
constexpr int kWideClass = kClasses;  // uni-greedy completion times: machines large enough for a block of their own
constexpr int kPlanClasses = kClasses + 1;

struct PlanHeader {
    unsigned long long ticket[kClasses + 1];
    int32_t class_begin[kClasses + 1];
    int32_t class_count[kClasses + 1];
    int32_t hist[kPlanClasses * kWorkBuckets];
    int32_t start[kPlanClasses * kWorkBuckets];
    int32_t cursor[kPlanClasses * kWorkBuckets];
    // The heaviest configurations of the last class (at least 2^giant_log2 pairs) come first in its order; the
    // uni-greedy kernels run them on whole wavefronts and draw them from a ticket counter of their own.
    int32_t giant_count;
    unsigned long long ticket_giant;
};
constexpr int kGiantLog2 = 23;
enum ClassPart { kWholeClass = 0, kGiantPart = 1, kRestPart = 2 };

// By size (by_work == 0): class k holds p <= limits.p[k]; the last class the rest and every configuration
// with more than q segments.
// By work (by_work != 0): class k holds the configurations with at most work[k] pairs, the last class the rest.
struct ClassLimits {
    int32_t p[kClasses - 1];
    int32_t q;
    int32_t by_work;
    int64_t work[kClasses - 1];
    int32_t giant_log2;          // configurations of the last class with at least 2^giant_log2 pairs are "giant"
    int32_t wide_p;              // by_work only: machines of at least this many processors form the class kWideClass (0: none)
};

struct PlanLaunch {
    ConfigArrays cfg;
    int64_t n;
    int32_t p_max, q_max;
    int cost;
    ClassLimits limits;
    PlanHeader *header;
    int32_t *order;
    hipStream_t stream;
};

hipError_t launch_plan(const PlanLaunch &L);

__host__ __device__ inline size_t plan_header_bytes() { return (sizeof(PlanHeader) + 255) / 256 * 256; }

}  // namespace prs
