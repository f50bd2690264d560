// Replay of a reduction schedule on data (Lowery & Langou, Section 4: the
// receiver of a pair combines the received segment into its own) on gfx950.
//
// Applying the pairs one after the other would move every partial result
// through memory once per pair.  Instead, per segment the pairs form an
// in-tree rooted at processor 0; the value the root ends with is
//     e(i) = (((own_i + e(c_1)) + e(c_2)) + ... )          c_k = k-th sender to i
// evaluated recursively.  A small kernel turns each segment's tree into a
// linear program over the p input buffers (each read exactly once), and the
// streaming kernel evaluates that program per element with a short stack of
// partial sums held in registers.  Because a + b == b + a bit for bit, the
// first child's subtree is evaluated in place before own_i is added, so only
// later children that have children of their own need a stack slot.
//
// Program entry for position k of segment s: prog[s*p + k] =
//     processor | push << 20 | npop << 21
// "load the processor's element; if push, save the running sum and start a new
// one from the loaded value, else add it to the running sum; then npop times
// add the running sum into the last saved one".
#include <mutex>

#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

constexpr int kReplayThreads = 128;
constexpr int kBuildThreads = 256;
constexpr int kStackDepth = 24;      // saved partial sums per element
constexpr int kPrefetch = 8;         // rows per group of loads; two groups are in flight per lane

struct ReplayWs {
    int64_t *offsets;      // q+1
    uint32_t *prog;        // q*p
    int32_t *tmp;          // q * 8 * p scratch of the builder
    int32_t *flags;        // [0] invalid, [1] too deep, [2] saved partial sums needed at once
};

__host__ __device__ inline size_t rp_align(size_t v) { return (v + 255) / 256 * 256; }

// The builder's work arrays (eight of p entries per segment) sit in LDS up to this many processors, beyond it in
// the scratch memory.
constexpr int32_t kBuildLdsProcs = 48 * 1024 / (8 * 4);

size_t replay_workspace_bytes(int32_t p, int32_t q)
{
    const size_t P = static_cast<size_t>(p), Q = static_cast<size_t>(q);
    return rp_align((Q + 1) * 8) + rp_align(Q * P * 4) + 256 + rp_align(Q * P * 4 * 8);
}

// What a replay really touches of its scratch memory: the builder's arrays only for machines too large for LDS.
size_t replay_scratch_bytes(int32_t p, int32_t q)
{
    const size_t P = static_cast<size_t>(p), Q = static_cast<size_t>(q);
    return rp_align((Q + 1) * 8) + rp_align(Q * P * 4) + 256 + (p > kBuildLdsProcs ? rp_align(Q * P * 4 * 8) : 0);
}

static ReplayWs carve_replay(char *ws, int32_t p, int32_t q)
{
    const size_t P = static_cast<size_t>(p), Q = static_cast<size_t>(q);
    ReplayWs w;
    w.offsets = reinterpret_cast<int64_t *>(ws); ws += rp_align((Q + 1) * 8);
    w.prog = reinterpret_cast<uint32_t *>(ws); ws += rp_align(Q * P * 4);
    w.flags = reinterpret_cast<int32_t *>(ws); ws += 256;
    w.tmp = reinterpret_cast<int32_t *>(ws);
    return w;
}

// Scratch memory for callers that cannot allocate: one array per GPU, held from the first use on that GPU until the
// process ends.  The name `scratch` is only a handle on the host; kernels get the address hipGetSymbolAddress
// returns for the current device.
static __device__ __align__(256) unsigned char scratch[kReplayStaticBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

hipError_t replay_static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

__global__ void replay_clear_flags(int32_t *flags) { if (threadIdx.x < 3) flags[threadIdx.x] = 0; }

// Segment offsets travel as kernel arguments, a chunk at a time: no host-to-device copy is enqueued.
constexpr int kOffsetChunk = 256;
struct OffsetChunk { int64_t v[kOffsetChunk]; };
__global__ void replay_store_offsets(OffsetChunk chunk, int base, int count, int64_t *dst)
{
    const int i = threadIdx.x;
    if (i < count) dst[base + i] = chunk.v[i];
}

// One block per segment: tree of the segment's pairs -> linear program.  The eight work arrays of p entries
// sit in LDS when they fit (kLds), else in the workspace.
template <bool kLds>
__global__ __launch_bounds__(kBuildThreads) void replay_build(int32_t p, int32_t q, const int32_t *src, const int32_t *dst,
                                                              const int32_t *seg, int64_t n_pairs, uint32_t *prog,
                                                              int32_t *tmp, int32_t *flags)
{
    PRS_DYNAMIC_LDS(lds_raw);
    const int k = blockIdx.x, tid = threadIdx.x;
    int32_t *base = kLds ? reinterpret_cast<int32_t *>(lds_raw) : tmp + static_cast<size_t>(k) * 8 * p;
    int32_t *parent = base, *ord = base + p, *ci = base + 2 * p, *nchild = base + 3 * p, *size = base + 4 * p,
            *offStart = base + 5 * p, *fchild = base + 6 * p, *start = base + 7 * p;
    __shared__ int s_bad, s_count, s_deep;
    if (tid == 0) { s_bad = 0; s_count = 0; s_deep = 0; }
    for (int i = tid; i < p; i += kBuildThreads) { parent[i] = -1; ord[i] = -1; nchild[i] = 0; size[i] = 1; fchild[i] = -1; }
    __syncthreads();
    // 1. who sends to whom, and when (position in emission order)
    //    A schedule written segment by segment has the p - 1 pairs of segment k in a row, at k (p - 1): if all of
    //    those carry this block's segment (and the schedule has q (p - 1) pairs, so that every block can find its
    //    own there and none is left over), only they are read.  Otherwise the block reads the segment index of
    //    every pair and keeps its own, eight loads in flight per thread.
    int64_t scan_from = 0, scan_to = n_pairs;
    if (n_pairs == static_cast<int64_t>(q) * (p - 1)) {
        const int64_t lo = static_cast<int64_t>(k) * (p - 1);
        for (int64_t e = lo + tid; e < lo + p - 1; e += kBuildThreads)
            if (seg[e] == k) atomicAdd(&s_deep, 1);
        __syncthreads();
        if (s_deep == p - 1) { scan_from = lo; scan_to = lo + p - 1; }
        __syncthreads();
        if (tid == 0) s_deep = 0;
        __syncthreads();
    }
    constexpr int kAhead = 8;
    for (int64_t e0 = scan_from + tid; e0 < scan_to; e0 += static_cast<int64_t>(kBuildThreads) * kAhead) {
        int32_t sg[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int64_t e = e0 + static_cast<int64_t>(u) * kBuildThreads;
            sg[u] = e < scan_to ? seg[e] : k + 1;                              // past the end: some other segment
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int64_t e = e0 + static_cast<int64_t>(u) * kBuildThreads;
            if (sg[u] != k) { if (e < scan_to && (sg[u] < 0 || sg[u] >= q)) s_bad = 1; continue; }
            const int32_t s = src[e], d = dst[e];
            if (s <= 0 || s >= p || d < 0 || d >= p || s == d) { s_bad = 1; continue; }
            if (atomicCAS(&parent[s], -1, d) != -1) { s_bad = 1; continue; }      // sends the segment twice
            ord[s] = static_cast<int32_t>(e);
            atomicAdd(&nchild[d], 1);
            atomicAdd(&s_count, 1);
        }
    }
    __syncthreads();
    if (s_count != p - 1) s_bad = 1;
    __syncthreads();
    // 2. position among the senders to the same receiver; a processor sends after all it receives.  Every processor
    //    looks at every other one: a wavefront loads 64 entries at a time, one per lane, and hands them round
    //    lane by lane (a lane's register is read by all others), so the inner loop touches no memory.
    const int lane = tid & (kWave - 1);
    for (int i0 = 0; i0 < p; i0 += kBuildThreads) {
        const int i = i0 + tid;
        const bool sender = i > 0 && i < p && parent[i] >= 0;
        const int32_t par = sender ? parent[i] : -3, oi = sender ? ord[i] : 0;
        int32_t c = 0;
        bool late_child = false;
        for (int s0 = 0; s0 < p; s0 += kWave) {
            const int sl = s0 + lane;
            const int32_t pv = sl < p ? parent[sl] : -2, ov = sl < p ? ord[sl] : 0;
#pragma unroll
            for (int u = 0; u < kWave; ++u) {
                const int32_t ps = __builtin_amdgcn_readlane(pv, u), os = __builtin_amdgcn_readlane(ov, u);
                c += (ps == par && os < oi) ? 1 : 0;
                late_child = late_child || (ps == i && os > oi);
            }
        }
        if (i < p) {
            if (sender && late_child) s_bad = 1;
            ci[i] = sender ? c : 0;
            if (sender && c == 0) fchild[par] = i;
        }
    }
    __syncthreads();
    if (s_bad) { if (tid == 0) flags[0] = 1; return; }
    // 3. subtree sizes: every processor counts itself into each of its ancestors (ord grows along
    //    the way to the root, so the walk ends)
    for (int i = tid; i < p; i += kBuildThreads)
        for (int a = parent[i], hops = 0; a >= 0 && hops < p; a = parent[a], ++hops) atomicAdd(&size[a], 1);
    __syncthreads();
    // 4. where a child's part starts relative to its parent's part: the first child starts with
    //    the parent; later ones after the first child's part, the parent itself and the earlier siblings
    for (int i0 = 0; i0 < p; i0 += kBuildThreads) {
        const int i = i0 + tid;
        const bool later = i > 0 && i < p && ci[i] > 0;
        const int32_t par = later ? parent[i] : -3, me = later ? ci[i] : 0;
        int32_t off = 0;
        for (int s0 = 0; s0 < p; s0 += kWave) {
            const int sl = s0 + lane;
            const bool has = sl >= 1 && sl < p;
            const int32_t pv = has ? parent[sl] : -2, cv = has ? ci[sl] : 0, zv = has ? size[sl] : 0;
#pragma unroll
            for (int u = 0; u < kWave; ++u) {
                const int32_t ps = __builtin_amdgcn_readlane(pv, u), cs = __builtin_amdgcn_readlane(cv, u),
                              zs = __builtin_amdgcn_readlane(zv, u);
                off += (ps == par && cs < me) ? zs : 0;
            }
        }
        if (i < p) offStart[i] = later ? off + 1 : 0;
    }
    __syncthreads();
    for (int i = tid; i < p; i += kBuildThreads) {
        int32_t st = 0;
        for (int a = i, hops = 0; a > 0 && hops < p; a = parent[a], ++hops) st += offStart[a];
        start[i] = st;
    }
    __syncthreads();
    // 5. one program entry per processor
    int deepest = 0;
    for (int i = tid; i < p; i += kBuildThreads) {
        const int32_t pos = start[i] + (nchild[i] > 0 ? size[fchild[i]] : 0);
        int push = 0;
        if (nchild[i] == 0) {                       // a leaf that opens the part of a saved subtree (or of the root)
            int a = i;
            for (int hops = 0; a != 0 && ci[a] == 0 && hops < p; ++hops) a = parent[a];
            push = (a == 0 || a != i) ? 1 : 0;
        }
        int npop = 0, depth = 0;
        for (int a = i, hops = 0; a > 0 && hops < p; a = parent[a], ++hops) {
            const bool saved = ci[a] > 0 && nchild[a] > 0;
            if (saved) {
                ++depth;
                if (start[a] + size[a] - 1 == pos) ++npop;
            }
        }
        if (depth > deepest) deepest = depth;
        prog[static_cast<size_t>(k) * p + pos] = static_cast<uint32_t>(i) | (static_cast<uint32_t>(push) << 20) |
                                                 (static_cast<uint32_t>(npop) << 21);
    }
    // one update of the global flags per block: thousands of atomic operations on one address would queue up
    atomicMax(&s_deep, deepest + 1);
    __syncthreads();
    if (tid == 0) {
        if (s_deep > kStackDepth) flags[1] = 1;
        atomicMax(&flags[2], s_deep);
    }
}

// The combine operation of a replay.  Sum: wrapping for integers, one IEEE addition (no FMA) for floating point.
// Max: the larger operand; floating point is compared in the IEEE total order (-NaN < -inf < ... < -0 < +0 < ... <
// +inf < +NaN), which is a comparison of the bit patterns as sign-magnitude integers, so the result does not
// depend on the order of the operands either.
template <typename E> struct Bits;
template <> struct Bits<float> { using I = int32_t; };
template <> struct Bits<double> { using I = int64_t; };

template <typename E> __device__ __forceinline__ E total_max(E a, E b)
{
    using I = typename Bits<E>::I;
    constexpr I kMag = static_cast<I>(~(static_cast<I>(1) << (sizeof(I) * 8 - 1)));     // all bits but the sign
    I ia, ib;
    __builtin_memcpy(&ia, &a, sizeof(E));
    __builtin_memcpy(&ib, &b, sizeof(E));
    const I ka = ia < 0 ? static_cast<I>(ia ^ kMag) : ia, kb = ib < 0 ? static_cast<I>(ib ^ kMag) : ib;
    return ka < kb ? b : a;
}

template <typename E, int OP> struct Combine;
template <> struct Combine<int32_t, PRS_OP_SUM> {
    static __device__ __forceinline__ int32_t identity() { return 0; }
    static __device__ __forceinline__ int32_t apply(int32_t a, int32_t b) { return static_cast<int32_t>(static_cast<uint32_t>(a) + static_cast<uint32_t>(b)); }
};
template <> struct Combine<int64_t, PRS_OP_SUM> {
    static __device__ __forceinline__ int64_t identity() { return 0; }
    static __device__ __forceinline__ int64_t apply(int64_t a, int64_t b) { return static_cast<int64_t>(static_cast<uint64_t>(a) + static_cast<uint64_t>(b)); }
};
template <> struct Combine<float, PRS_OP_SUM> {
    static __device__ __forceinline__ float identity() { return 0.0f; }
    static __device__ __forceinline__ float apply(float a, float b) { return a + b; }
};
template <> struct Combine<double, PRS_OP_SUM> {
    static __device__ __forceinline__ double identity() { return 0.0; }
    static __device__ __forceinline__ double apply(double a, double b) { return a + b; }
};
template <> struct Combine<int32_t, PRS_OP_MAX> {
    static __device__ __forceinline__ int32_t identity() { return INT32_MIN; }
    static __device__ __forceinline__ int32_t apply(int32_t a, int32_t b) { return a < b ? b : a; }
};
template <> struct Combine<int64_t, PRS_OP_MAX> {
    static __device__ __forceinline__ int64_t identity() { return INT64_MIN; }
    static __device__ __forceinline__ int64_t apply(int64_t a, int64_t b) { return a < b ? b : a; }
};
template <> struct Combine<float, PRS_OP_MAX> {
    static __device__ __forceinline__ float identity() { return __builtin_bit_cast(float, 0xFFFFFFFFu); }        // least in the total order
    static __device__ __forceinline__ float apply(float a, float b) { return total_max<float>(a, b); }
};
template <> struct Combine<double, PRS_OP_MAX> {
    static __device__ __forceinline__ double identity() { return __builtin_bit_cast(double, ~UINT64_C(0)); }
    static __device__ __forceinline__ double apply(double a, double b) { return total_max<double>(a, b); }
};

template <typename E, int VEC> struct Acc {
    E v[VEC];
};

template <typename E, int VEC>
__device__ __forceinline__ Acc<E, VEC> load_elems(const E *ptr, int nvalid)
{
    Acc<E, VEC> a;
    if (VEC * sizeof(E) == 16 && nvalid == VEC) {
        // every input element is read once: a streaming load, which leaves the caches to the tree programs
        typedef float row16 __attribute__((ext_vector_type(4)));
        const row16 f = __builtin_nontemporal_load(reinterpret_cast<const row16 *>(ptr));
        const E *fe = reinterpret_cast<const E *>(&f);
#pragma unroll
        for (int i = 0; i < VEC; ++i) a.v[i] = fe[i];
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) a.v[i] = i < nvalid ? ptr[i] : E(0);    // elements past the end are never stored
    }
    return a;
}

template <typename E, int VEC>
__device__ __forceinline__ void store_elems(E *ptr, const Acc<E, VEC> &a, int nvalid)
{
    if (VEC * sizeof(E) == 16 && nvalid == VEC) {
        float4 f;
        E *fe = reinterpret_cast<E *>(&f);
#pragma unroll
        for (int i = 0; i < VEC; ++i) fe[i] = a.v[i];
        *reinterpret_cast<float4 *>(ptr) = f;
    } else {
        for (int i = 0; i < nvalid; ++i) ptr[i] = a.v[i];
    }
}

// One thread reduces VEC neighbouring elements of a segment by running the segment's program: p entries
// (row | push << 20 | pops << 21), the same for every thread of a block.  The partial sums a push saves sit
// in LDS ([depth][thread], 16 bytes per thread and level), so the registers are free for the loads: two
// groups of kPrefetch rows are in flight while the group before them is added up.  The LDS allocation fixes
// the depth D (8, 16 or 24 levels, the fewer the more blocks fit on a CU); every variant is launched and only
// the one that fits the schedule's trees (flags[2], found by replay_build) runs.
template <typename E, int VEC, int OP>
__device__ __forceinline__ void replay_step(Acc<E, VEC> &acc, int &sp, E *stk, uint32_t ent, const Acc<E, VEC> &val)
{
    if ((ent >> 20) & 1u) {
        E *slot = stk + static_cast<size_t>(sp) * kReplayThreads * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i) slot[i] = acc.v[i];
        ++sp;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = val.v[i];
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = Combine<E, OP>::apply(acc.v[i], val.v[i]);
    }
    for (int np = static_cast<int>(ent >> 21); np > 0; --np) {
        --sp;
        const E *slot = stk + static_cast<size_t>(sp) * kReplayThreads * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = Combine<E, OP>::apply(slot[i], acc.v[i]);   // saved partial result, then the finished subtree
    }
}

template <typename E, int VEC, int D, int OP>
__global__ __launch_bounds__(kReplayThreads) void replay_kernel(int32_t p, const int64_t *__restrict__ offsets,
                                                                const uint32_t *__restrict__ prog, const E *__restrict__ in,
                                                                int64_t stride, E *__restrict__ out,
                                                                const int32_t *__restrict__ flags)
{
    PRS_DYNAMIC_LDS(lds_raw);
    if (flags[0] | flags[1]) return;
    const int need = flags[2];
    if (need > D || need <= D - 8) return;                     // another depth variant takes this schedule
    // Workgroups go to the eight XCDs in turn (workgroup b to XCD b mod 8): the tiles are renumbered so that each
    // XCD streams one contiguous eighth of the (segment, chunk) tiles instead of every eighth 2 KB chunk.
    const unsigned tiles = gridDim.x * gridDim.y, b = blockIdx.y * gridDim.x + blockIdx.x;
    const unsigned xcd = b & 7u, each = tiles >> 3, extra = tiles & 7u;
    const unsigned tile = xcd * each + (xcd < extra ? xcd : extra) + (b >> 3);
    const int k = static_cast<int>(tile / gridDim.x);
    const int64_t lo = offsets[k], hi = offsets[k + 1];
    const int64_t b0 = lo + static_cast<int64_t>(tile % gridDim.x) * kReplayThreads * VEC;
    if (b0 >= hi) return;
    const int64_t e0 = b0 + static_cast<int64_t>(threadIdx.x) * VEC;
    const uint32_t *pg = prog + static_cast<size_t>(k) * p;
    Acc<E, VEC> acc;
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc.v[i] = Combine<E, OP>::identity();
    E *const stk = reinterpret_cast<E *>(lds_raw) + static_cast<size_t>(threadIdx.x) * VEC;   // this thread's column of the LDS stack
    int sp = 0;
    const bool full = b0 + static_cast<int64_t>(kReplayThreads) * VEC <= hi;   // every thread of the block has VEC elements
    if (full) {
        // entries past the end of the program repeat the last row (loaded, not used): the loads stay
        // unconditional, so that waiting for one group does not wait for the next
        auto row = [&](int idx) { return pg[idx < p ? idx : p - 1]; };
        uint32_t entA[kPrefetch], entB[kPrefetch];
        Acc<E, VEC> valA[kPrefetch], valB[kPrefetch];
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) entA[u] = row(u);
#pragma unroll
        for (int u = 0; u < kPrefetch; ++u) valA[u] = load_elems<E, VEC>(in + static_cast<int64_t>(entA[u] & 0xFFFFFu) * stride + e0, VEC);
        for (int base = 0; base < p; base += 2 * kPrefetch) {
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) entB[u] = row(base + kPrefetch + u);
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) valB[u] = load_elems<E, VEC>(in + static_cast<int64_t>(entB[u] & 0xFFFFFu) * stride + e0, VEC);
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u)
                if (base + u < p) replay_step<E, VEC, OP>(acc, sp, stk, entA[u], valA[u]);
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) entA[u] = row(base + 2 * kPrefetch + u);
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u) valA[u] = load_elems<E, VEC>(in + static_cast<int64_t>(entA[u] & 0xFFFFFu) * stride + e0, VEC);
#pragma unroll
            for (int u = 0; u < kPrefetch; ++u)
                if (base + kPrefetch + u < p) replay_step<E, VEC, OP>(acc, sp, stk, entB[u], valB[u]);
        }
        store_elems<E, VEC>(out + e0, acc, VEC);
    } else if (e0 < hi) {
        // ragged end of a segment: plain loop
        const int nvalid = hi - e0 >= VEC ? VEC : static_cast<int>(hi - e0);
        for (int idx = 0; idx < p; ++idx) {
            const uint32_t ent = pg[idx];
            replay_step<E, VEC, OP>(acc, sp, stk, ent, load_elems<E, VEC>(in + static_cast<int64_t>(ent & 0xFFFFFu) * stride + e0, nvalid));
        }
        store_elems<E, VEC>(out + e0, acc, nvalid);
    }
}

__global__ void replay_write_status(const int32_t *flags, int32_t *status)
{
    if (threadIdx.x == 0 && status) *status = flags[0] ? 1 : (flags[1] ? 2 : 0);
}

static size_t replay_lds_bytes(int vec, int depth, size_t elem) { return static_cast<size_t>(depth) * kReplayThreads * vec * elem; }

template <typename E, int VEC, int OP>
static void launch_replay_depths(const ReplayLaunch &L, const ReplayWs &w, int64_t max_len)
{
    const E *in = static_cast<const E *>(L.in);
    E *out = static_cast<E *>(L.out);
    const int64_t groups = (max_len + VEC - 1) / VEC;
    dim3 grid(static_cast<unsigned>((groups + kReplayThreads - 1) / kReplayThreads), static_cast<unsigned>(L.q));
    hipLaunchKernelGGL((replay_kernel<E, VEC, 8, OP>), grid, dim3(kReplayThreads), replay_lds_bytes(VEC, 8, sizeof(E)), L.stream, L.p,
                       w.offsets, w.prog, in, L.stride_elems, out, w.flags);
    hipLaunchKernelGGL((replay_kernel<E, VEC, 16, OP>), grid, dim3(kReplayThreads), replay_lds_bytes(VEC, 16, sizeof(E)), L.stream, L.p,
                       w.offsets, w.prog, in, L.stride_elems, out, w.flags);
    hipLaunchKernelGGL((replay_kernel<E, VEC, 24, OP>), grid, dim3(kReplayThreads), replay_lds_bytes(VEC, 24, sizeof(E)), L.stream, L.p,
                       w.offsets, w.prog, in, L.stride_elems, out, w.flags);
}

template <typename E>
static hipError_t launch_replay_t(const ReplayLaunch &L, const ReplayWs &w, int64_t max_len, bool vec_ok)
{
    constexpr int kVec = 16 / sizeof(E);                           // 16 bytes per lane and row
    if (max_len > 0) {
        if (L.op == PRS_OP_MAX) {
            if (vec_ok) launch_replay_depths<E, kVec, PRS_OP_MAX>(L, w, max_len); else launch_replay_depths<E, 1, PRS_OP_MAX>(L, w, max_len);
        } else {
            if (vec_ok) launch_replay_depths<E, kVec, PRS_OP_SUM>(L, w, max_len); else launch_replay_depths<E, 1, PRS_OP_SUM>(L, w, max_len);
        }
    }
    return hipGetLastError();
}

// L.seg_elem_offset is a host array here (validated by the caller).
hipError_t launch_replay(const ReplayLaunch &L)
{
    const ReplayWs w = carve_replay(L.workspace, L.p, L.q);
    int64_t max_len = 0;
    const int vec = (L.dtype == PRS_F64 || L.dtype == PRS_I64) ? 2 : 4;       // elements in 16 bytes
    bool vec_ok = (L.stride_elems % vec == 0) && (reinterpret_cast<uintptr_t>(L.in) % 16 == 0) &&
                  (reinterpret_cast<uintptr_t>(L.out) % 16 == 0);
    for (int k = 0; k < L.q; ++k) {
        const int64_t len = L.seg_elem_offset[k + 1] - L.seg_elem_offset[k];
        if (len > max_len) max_len = len;
        if (L.seg_elem_offset[k] % vec != 0) vec_ok = false;
    }
    hipError_t err = hipSuccess;
    for (int base = 0; base < L.q + 1; base += kOffsetChunk) {
        OffsetChunk chunk;
        const int count = L.q + 1 - base < kOffsetChunk ? L.q + 1 - base : kOffsetChunk;
        for (int i = 0; i < count; ++i) chunk.v[i] = L.seg_elem_offset[base + i];
        hipLaunchKernelGGL(replay_store_offsets, dim3(1), dim3(kOffsetChunk), 0, L.stream, chunk, base, count, w.offsets);
    }
    hipLaunchKernelGGL(replay_clear_flags, dim3(1), dim3(64), 0, L.stream, w.flags);
    const size_t build_lds = static_cast<size_t>(L.p) * 8 * 4;
    if (L.p <= kBuildLdsProcs)
        hipLaunchKernelGGL(replay_build<true>, dim3(static_cast<unsigned>(L.q)), dim3(kBuildThreads), build_lds, L.stream, L.p, L.q,
                           L.src, L.dst, L.seg, L.n_pairs, w.prog, w.tmp, w.flags);
    else
        hipLaunchKernelGGL(replay_build<false>, dim3(static_cast<unsigned>(L.q)), dim3(kBuildThreads), 0, L.stream, L.p, L.q,
                           L.src, L.dst, L.seg, L.n_pairs, w.prog, w.tmp, w.flags);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    switch (L.dtype) {
    case PRS_F32: err = launch_replay_t<float>(L, w, max_len, vec_ok); break;
    case PRS_F64: err = launch_replay_t<double>(L, w, max_len, vec_ok); break;
    case PRS_I64: err = launch_replay_t<int64_t>(L, w, max_len, vec_ok); break;
    default: err = launch_replay_t<int32_t>(L, w, max_len, vec_ok); break;
    }
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(replay_write_status, dim3(1), dim3(64), 0, L.stream, w.flags, L.status);
    return hipGetLastError();
}

}  // namespace prs
