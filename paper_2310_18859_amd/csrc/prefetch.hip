// Expert prefetch: brings the missing experts of one wave from pinned host memory into their pool
// slots (Section 3.1: the activated experts are loaded ahead of the forward pass), in the slot
// layout the grouped FFN reads (kernels.h).
//
// One hipMemcpyAsync per expert pays a fixed cost per copy: with 9.4 MB experts the copy engine
// reaches about 45 GB/s where a single large copy reaches 57 GB/s.  A kernel that reads the pinned
// blocks over the host link itself has no per-expert cost; a few hundred KB in flight saturate the
// link (56-57 GB/s measured), one launch per wave, and it writes the slot layout directly.  The
// kernel runs on a few compute units of its own (sida_streams_create): a grouped GEMM that shares
// a compute unit with lanes waiting on host-link reads is slowed by them.
// With the copy engine the host block lands in the slot as it is and a second, in-place kernel
// re-orders it.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

constexpr int kInFlight = 4;          // 16-byte loads in flight per lane
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Piece i of an expert's host block (16 bytes; W_in's pieces first, row-major) -> its piece index
// in the slot.  kpr = pieces per row of the matrix the piece belongs to.
__device__ __forceinline__ size_t slot_piece(size_t i, size_t pieces_in, int kpr_in, int kpr_out)
{
    const bool second = i >= pieces_in;
    const size_t j = second ? i - pieces_in : i;
    const size_t kpr = second ? kpr_out : kpr_in;
    const size_t r = j / kpr, p = j - r * kpr;
    return (second ? pieces_in : 0) + ((r >> 5) * kpr + p) * 32 + (r & 31);
}

// Reads are linear over the host block (consecutive lanes, consecutive 16 bytes); the writes of a
// wavefront scatter over the stripe, 16 bytes each, and the eight rows that share a 128-byte line
// of the slot are written within a few steps of the same workgroup.
__global__ __launch_bounds__(256) void copy_experts(const CopyTable tbl, size_t pieces_in, size_t pieces, int kpr_in,
                                                    int kpr_out)
{
    const u32x4 *__restrict__ src = static_cast<const u32x4 *>(tbl.src[blockIdx.y]);
    u32x4 *__restrict__ dst = static_cast<u32x4 *>(tbl.dst[blockIdx.y]);
    const size_t step = 256 * kInFlight, stride = (size_t)gridDim.x * step;
    for (size_t base = (size_t)blockIdx.x * step + threadIdx.x; base - threadIdx.x < pieces; base += stride) {
        u32x4 v[kInFlight];
        // all loads first, then the stores.  Plain stores: a wave's experts (150 MB at the bench
        // workload) stay in the 256 MB Infinity Cache until the wave's GEMMs read them
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) {                 // unconditional loads (past the end: the last piece again)
            const size_t j = base + (size_t)i * 256;
            v[i] = src[j < pieces ? j : pieces - 1];
        }
#pragma unroll
        for (int i = 0; i < kInFlight; ++i)
            if (base + (size_t)i * 256 < pieces) dst[slot_piece(base + (size_t)i * 256, pieces_in, kpr_in, kpr_out)] = v[i];
    }
}

// In-place re-ordering of slots that hold plain copies of host blocks: one workgroup per stripe of
// 32 rows (the same bytes in both layouts).  Every thread reads its pieces, the workgroup waits
// for all reads, then every thread writes: nothing is overwritten before it was read.
constexpr int kRelayoutThreads = 1024;
constexpr int kRelayoutPieces = 32 * (kMaxRelayoutK / 8) / kRelayoutThreads;   // per thread, at most

__global__ __launch_bounds__(kRelayoutThreads) void relayout_slots(const CopyTable tbl, int stripes_in, int kpr_in,
                                                                   int kpr_out, size_t pieces_in)
{
    u32x4 *slot = static_cast<u32x4 *>(tbl.dst[blockIdx.y]);
    const bool second = (int)blockIdx.x >= stripes_in;
    const int stripe = second ? blockIdx.x - stripes_in : blockIdx.x;
    const int kpr = second ? kpr_out : kpr_in;
    u32x4 *base = slot + (second ? pieces_in : 0) + (size_t)stripe * 32 * kpr;
    const int n = 32 * kpr;                                   // pieces of the stripe
    u32x4 v[kRelayoutPieces];
#pragma unroll
    for (int i = 0; i < kRelayoutPieces; ++i) {
        const int j = i * kRelayoutThreads + threadIdx.x;     // row-major piece (r, p) = (j / kpr, j % kpr)
        v[i] = base[j < n ? j : n - 1];                       // unconditional loads
    }
    __syncthreads();                                          // waits for this thread's loads, then for everyone's
#pragma unroll
    for (int i = 0; i < kRelayoutPieces; ++i) {
        const int j = i * kRelayoutThreads + threadIdx.x;
        if (j < n) {
            const int r = j / kpr, p = j - r * kpr;
            base[p * 32 + r] = v[i];
        }
    }
}

}  // namespace

int launch_expert_copy(const CopyTable &tbl, int32_t d, int32_t F, hipStream_t st)
{
    if (tbl.n <= 0) return 0;
    // Few workgroups: 16 with 4 x 16 bytes in flight per lane keep the link full (56 GB/s), and the
    // fewer host-link reads are outstanding in the L2s, the less the GEMMs that run beside the copy
    // are slowed (GEMM 1 of a wave: 35 us with 16 workgroups, 41 with 32, 45 with 64).
    int per = (16 + tbl.n - 1) / tbl.n;
    per = per < 1 ? 1 : per > 16 ? 16 : per;
    const size_t pieces_in = (size_t)F * d / 8;
    hipLaunchKernelGGL(copy_experts, dim3(per, tbl.n), dim3(256), 0, st, tbl, pieces_in, 2 * pieces_in, d / 8, F / 8);
    return (int)hipGetLastError();
}

int launch_slot_relayout(const CopyTable &tbl, int32_t d, int32_t F, hipStream_t st)
{
    if (tbl.n <= 0) return 0;
    if (d > kMaxRelayoutK || F > kMaxRelayoutK) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(relayout_slots, dim3(F / 32 + d / 32, tbl.n), dim3(kRelayoutThreads), 0, st, tbl, F / 32, d / 8, F / 8,
                       (size_t)F * d / 8);
    return (int)hipGetLastError();
}

}  // namespace sida
