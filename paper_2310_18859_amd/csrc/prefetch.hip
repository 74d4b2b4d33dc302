// Expert prefetch by kernel: copies the missing experts of one wave from pinned host memory into
// their pool slots (Section 3.1: the activated experts are loaded ahead of the forward pass).
//
// One hipMemcpyAsync per expert pays a fixed cost per copy: with 9.4 MB experts the copy engine
// reaches about 45 GB/s where a single large copy reaches 57 GB/s.  A kernel that reads the pinned
// blocks over the host link itself has no per-expert cost: 32 or more workgroups with 8 x 16 bytes
// in flight per lane saturate the link (57 GB/s measured), one launch per wave.  The kernel uses
// no LDS and few registers, so its workgroups share compute units with the grouped GEMMs.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

constexpr int kInFlight = 8;          // 16-byte loads in flight per lane
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_experts(const CopyTable tbl, size_t vecs_per_expert)
{
    const u32x4 *__restrict__ src = static_cast<const u32x4 *>(tbl.src[blockIdx.y]);
    u32x4 *__restrict__ dst = static_cast<u32x4 *>(tbl.dst[blockIdx.y]);
    const size_t stride = (size_t)gridDim.x * 256 * kInFlight;
    for (size_t base = (size_t)blockIdx.x * 256 * kInFlight + threadIdx.x; base < vecs_per_expert; base += stride) {
        u32x4 v[kInFlight];
#pragma unroll
        for (int i = 0; i < kInFlight; ++i)
            if (base + (size_t)i * 256 < vecs_per_expert) v[i] = src[base + (size_t)i * 256];
        // plain stores: a wave's experts (150 MB at the bench workload) stay in the 256 MB Infinity
        // Cache until the wave's GEMMs read them; with non-temporal stores GEMM 1 of a wave was
        // 40 % slower
#pragma unroll
        for (int i = 0; i < kInFlight; ++i)
            if (base + (size_t)i * 256 < vecs_per_expert) dst[base + (size_t)i * 256] = v[i];
    }
}

}  // namespace

int launch_expert_copy(const CopyTable &tbl, size_t expert_bytes, hipStream_t st)
{
    if (tbl.n <= 0) return 0;
    // at least 64 workgroups in total, at most 16 per expert
    int per = (64 + tbl.n - 1) / tbl.n;
    per = per < 1 ? 1 : per > 16 ? 16 : per;
    hipLaunchKernelGGL(copy_experts, dim3(per, tbl.n), dim3(256), 0, st, tbl, expert_bytes / 16);
    return (int)hipGetLastError();
}

}  // namespace sida
