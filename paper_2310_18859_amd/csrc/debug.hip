// Debug helpers (sida_set_debug): a check that the ids a layer was run with are the ids it was
// planned with, and a poison pattern for slots that are about to be reloaded.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

// One workgroup: expert e's device-side count against the plan's.  A mismatch latches layer + 1
// into *flag (host memory the device can write).
__global__ __launch_bounds__(256) void check_counts(const int32_t *__restrict__ counts, const CountTable want, int E,
                                                    int layer, int32_t *flag)
{
    const int e = threadIdx.x;
    if (e < E && counts[e] != want.n[e]) atomicExch(flag, layer + 1);
}

// Fills the listed slots with bf16 quiet NaNs (0x7FC0), 16 bytes per lane.
__global__ __launch_bounds__(256) void poison_slots(const CopyTable tbl, size_t vecs)
{
    uint4 *dst = static_cast<uint4 *>(tbl.dst[blockIdx.y]);
    const uint4 nan4 = make_uint4(0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u, 0x7FC07FC0u);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < vecs; i += (size_t)gridDim.x * 256) dst[i] = nan4;
}

}  // namespace

int launch_check_counts(const int32_t *counts, const CountTable &want, int32_t E, int32_t layer, int32_t *flag_dev,
                        hipStream_t st)
{
    hipLaunchKernelGGL(check_counts, dim3(1), dim3(256), 0, st, counts, want, E, layer, flag_dev);
    return (int)hipGetLastError();
}

int launch_poison_slots(const CopyTable &tbl, size_t expert_bytes, hipStream_t st)
{
    if (tbl.n <= 0) return 0;
    hipLaunchKernelGGL(poison_slots, dim3(64, tbl.n), dim3(256), 0, st, tbl, expert_bytes / 16);
    return (int)hipGetLastError();
}

}  // namespace sida
