// Measurement helper: what the chip reaches on the bare arithmetic of one step of Algorithm 1 (Lowery & Langou,
// Section 5) when nothing else is in the way -- no streams, no LDS, no memory: every lane keeps the four heads of
// two sorted fronts in registers, picks the two smallest (two comparisons with their selects), adds tcomm and tcomp
// (two additions) and feeds the results back as new heads.  The steps of a lane depend on each other, as in the
// real kernels; the grid fills every SIMD with several wavefronts.  This is the practical ceiling the sweep kernels
// are compared with next to the chip's nominal fp64 rate.
#include "prs_device.h"
#include "prs_launch.h"

namespace prs {

__global__ __launch_bounds__(256) void alu_ceiling_kernel(int64_t steps, double c, double g, double *sink)
{
    const int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    double a0 = static_cast<double>(id & 7), a1 = a0 + 1.0, b0 = a0 + 0.5, b1 = a0 + 2.5;
    for (int64_t s = 0; s < steps; ++s) {
        const bool x = a0 <= b0;                       // the smallest of the two fronts
        const double u = x ? a1 : a0, v = x ? b0 : b1;
        const bool y = u <= v;                         // the second smallest
        const double t = y ? u : v;
        const double tc = t + c, tr = tc + g;          // the sender leaves at tc, the receiver stays until tr
        a0 = x ? (y ? tc : a1) : (y ? a1 : a0);        // consumed heads are replaced by the new values
        a1 = a0 + c;
        b0 = x ? (y ? b0 : b1) : (y ? b1 : tr);
        b1 = b0 + g;
    }
    if (a0 + a1 + b0 + b1 == -1.0) sink[0] = a0;       // never true: keeps the loop alive
}

hipError_t launch_alu_ceiling(int64_t steps, int32_t blocks, double *sink, hipStream_t stream)
{
    hipLaunchKernelGGL(alu_ceiling_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream, steps, 1.25, 0.5, sink);
    return hipGetLastError();
}

}  // namespace prs
