// Expert prefetch by kernel: copies the missing experts of one wave from pinned host memory into
// their pool slots (Section 3.1: the activated experts are loaded ahead of the forward pass).
//
// One hipMemcpyAsync per expert pays a fixed cost per copy: with 9.4 MB experts the copy engine
// reaches about 45 GB/s where a single large copy reaches 57 GB/s.  A kernel that reads the pinned
// blocks over the host link itself has no per-expert cost; a few hundred KB in flight saturate the
// link (56-57 GB/s measured), one launch per wave.  The kernel uses
// no LDS and few registers, so its workgroups share compute units with the grouped GEMMs.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

constexpr int kInFlight = 4;          // 16-byte loads in flight per lane
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_experts(const CopyTable tbl, size_t vecs_per_expert)
{
    const u32x4 *__restrict__ src = static_cast<const u32x4 *>(tbl.src[blockIdx.y]);
    u32x4 *__restrict__ dst = static_cast<u32x4 *>(tbl.dst[blockIdx.y]);
    const size_t step = 256 * kInFlight, stride = (size_t)gridDim.x * step;
    size_t base = (size_t)blockIdx.x * step + threadIdx.x;
    // whole steps: all loads first, then the stores
    for (; base + step - threadIdx.x <= vecs_per_expert; base += stride) {
        u32x4 v[kInFlight];
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) v[i] = src[base + (size_t)i * 256];
        // plain stores: a wave's experts (150 MB at the bench workload) stay in the 256 MB Infinity
        // Cache until the wave's GEMMs read them; with non-temporal stores GEMM 1 of a wave was
        // 40 % slower
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) dst[base + (size_t)i * 256] = v[i];
    }
    // the last, partial step of the expert (taken by the workgroup whose turn it is)
    for (int i = 0; i < kInFlight; ++i)
        if (base + (size_t)i * 256 < vecs_per_expert && base - threadIdx.x < vecs_per_expert)
            dst[base + (size_t)i * 256] = src[base + (size_t)i * 256];
}

}  // namespace

int launch_expert_copy(const CopyTable &tbl, size_t expert_bytes, hipStream_t st)
{
    if (tbl.n <= 0) return 0;
    // Few workgroups: 16 with 4 x 16 bytes in flight per lane keep the link full (56 GB/s), and the
    // fewer host-link reads are outstanding in the L2s, the less the GEMMs that run beside the copy
    // are slowed (GEMM 1 of a wave: 35 us with 16 workgroups, 41 with 32, 45 with 64).
    int per = (16 + tbl.n - 1) / tbl.n;
    per = per < 1 ? 1 : per > 16 ? 16 : per;
    hipLaunchKernelGGL(copy_experts, dim3(per, tbl.n), dim3(256), 0, st, tbl, expert_bytes / 16);
    return (int)hipGetLastError();
}

}  // namespace sida
