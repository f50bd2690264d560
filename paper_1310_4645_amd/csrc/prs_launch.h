// Host-side launch descriptors shared by the API file and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "prs_device.h"
#include "prs_plan.h"

namespace prs {

struct SchedOut {
    const int64_t *pair_offset;
    int64_t pair_capacity;
    int32_t *src, *dst, *seg;
    void *tstart;
    void *T_greedy;
    int32_t *cfg_status;
};

// One launch = one size class of the plan.  lds_p > 0: per-configuration state lives in LDS arrays sized
// for lds_p processors (uni) / the small arrays and, if it fits lds_bitmap_bytes, the sent bitmap (bi);
// slots then hold only what stays in global memory.  slot_p/slot_q size the slot arrays.
struct UniLaunch {
    ConfigArrays cfg;
    int32_t p_max, q_max;
    int model, cost;
    bool want_schedule;
    TimesOut times;
    SchedOut sched;
    PlanHeader *plan;
    const int32_t *order;
    int cls;
    int32_t lds_p;
    int32_t lds_bitmap_bytes;
    size_t lds_bytes;
    char *slots;
    size_t slot_bytes;
    int32_t slot_p, slot_q;
    int grid;
    hipStream_t stream;
};

typedef UniLaunch BiLaunch;   // same fields; slots sized by bi_slot_bytes

size_t bi_small_bytes(int32_t p_cap, int32_t q_cap);               // masks, lists, per-segment counters
size_t bi_bitmap_bytes(int32_t p_cap, int32_t q_cap);              // sent bitmap
size_t bi_masks_bytes(int32_t p_cap);                              // the bit sets and list positions among the small arrays
size_t bi_slot_bytes(int32_t p_cap, int32_t q_cap, bool small_in_lds);   // what a bi-greedy block keeps in global memory
// Several configurations per wavefront (p <= 1024, q <= 1023): 1, 2, 4, 8 or 16 lanes per configuration
// (plan classes 0, 1, 2), all three in one launch of one resident set of blocks.  start[k] blocks begin with
// class k (so the longest-running configurations of every class start at once); every block then goes on
// with the other classes until all tickets are gone.
constexpr int kBiGroupSizes = kClasses - 1;   // 1, 2, 4, 8, 16 lanes per configuration
struct BiGroupParts {
    int start[kBiGroupSizes];
    bool on[kBiGroupSizes];
    uint64_t *rows;               // sent-bit rows: one slot of rows_per_block words per block
    size_t rows_per_block;
    size_t rows_per_group[kBiGroupSizes];
    int list_entries[kBiGroupSizes];          // entries of the list of running transfers a configuration may use (<= the LDS layout's)
};
struct BiGroupLaunch {
    ConfigArrays cfg;
    int32_t p_max, q_max;
    int model, cost;
    bool want_schedule;
    TimesOut times;
    SchedOut sched;
    PlanHeader *plan;
    const int32_t *order;
    int32_t *retry;
    BiGroupParts parts;
    hipStream_t stream;
};
size_t bi_group_lds_bytes(int lpc);
int bi_group_list_capacity(int lpc);
hipError_t launch_bi_group(const BiGroupLaunch &L);
// uni-greedy: all classes of a batch in one launch
size_t uni_times_lds_bytes();
size_t uni_times_slot_bytes(int32_t p_cap);
hipError_t launch_uni_times(const UniLaunch &L);
size_t uni_sched_lds_bytes();
size_t uni_sched_slot_bytes(int32_t p_cap);
hipError_t launch_uni_sched(const UniLaunch &L);
// uni-greedy completion times of machines with thousands of processors: one block per configuration
size_t uni_wide_slot_bytes(int32_t p_cap);
size_t uni_wide_lds_bytes();
hipError_t launch_uni_wide(const UniLaunch &L);
hipError_t launch_bi(const BiLaunch &L);
// one block of 16 wavefronts per configuration: thousands of processors
size_t bi_block_slot_bytes(int32_t p_cap, int32_t q_cap);
size_t bi_block_lds_bytes(int32_t p_cap);
hipError_t launch_bi_block(const BiLaunch &L);

struct ReplayLaunch {
    int32_t p, q;
    const int64_t *seg_elem_offset;
    const int32_t *src, *dst, *seg;
    int64_t n_pairs;
    const void *in;
    int64_t stride_elems, n_elems;
    int dtype, op;
    void *out;
    int32_t *status;
    char *workspace;
    hipStream_t stream;
};
size_t replay_workspace_bytes(int32_t p, int32_t q);
hipError_t launch_replay(const ReplayLaunch &L);
// replay without a caller's workspace: a fixed device array per GPU
constexpr size_t kReplayStaticBytes = static_cast<size_t>(8) << 20;
size_t replay_scratch_bytes(int32_t p, int32_t q);          // what a replay touches of its scratch memory
hipError_t replay_static_scratch(void **ptr);                // address of the current device's array

struct ThresholdLaunch {
    const int32_t *p;
    int64_t n;
    double alpha;
    int32_t q_max, m_log2_first, m_log2_last;
    double ratio_lo, ratio_hi;
    int32_t steps;
    double *ratio_below, *ratio_above;
    int32_t *cfg_status;
    hipStream_t stream;
};
hipError_t launch_threshold(const ThresholdLaunch &L);

hipError_t launch_alu_ceiling(int64_t steps, int32_t blocks, double *sink, hipStream_t stream);

struct OffsetsLaunch {
    ConfigArrays cfg;
    int64_t n;
    int32_t p_max, q_max;
    int cost;
    int64_t *pair_offset;
    hipStream_t stream;
};
hipError_t launch_offsets(const OffsetsLaunch &L);
hipError_t launch_clear(unsigned long long *words, int count, hipStream_t stream);

}  // namespace prs
