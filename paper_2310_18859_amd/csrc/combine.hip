// K-c: gate-weighted scatter-combine.  The alpha factors of Eq. 1 (Section 2.1), applied while
// the expert outputs go back from expert order to token order:
//     y[t,:] = sum_{j<k} alpha[t*k+j] * y_perm[inv[t*k+j],:]        (k = 1 for Switch routing)
// Products and sum in fp32, terms in the order j = 0..k-1, one rounding to bf16 (nearest even).
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

// 16-byte accesses (8 bf16 values).  A workgroup takes kCombineRows consecutive token rows: their
// source rows and gate values go to LDS first, then the rows' pieces are dealt to the 256 threads
// as one flat range, so that no lane idles whatever the row length (96 pieces at d = 768).
constexpr int kCombineRows = 8;
__global__ __launch_bounds__(256) void combine_rows(const bf16x8 *__restrict__ y_perm,
                                                    const int32_t *__restrict__ inv,
                                                    const float *__restrict__ alpha, int n_tokens,
                                                    int vec_per_row, bf16x8 *__restrict__ y, int k)
{
    __shared__ int src_row[kCombineRows * 8];                 // k <= 8 entries per token
    __shared__ float gate[kCombineRows * 8];
    const int t0 = blockIdx.x * kCombineRows;
    const int rows = min(kCombineRows, n_tokens - t0);
    if ((int)threadIdx.x < rows * k) {
        src_row[threadIdx.x] = inv[(size_t)t0 * k + threadIdx.x];
        gate[threadIdx.x] = alpha[(size_t)t0 * k + threadIdx.x];
    }
    __syncthreads();
    const int n = rows * vec_per_row;                         // pieces of this workgroup
    bf16x8 *dst = y + (size_t)t0 * vec_per_row;               // its token rows are one contiguous range
    for (int p = threadIdx.x; p < n; p += 256) {
        const int r = p / vec_per_row, i = p - r * vec_per_row;
        float acc[8];
        {
            const float a = gate[r * k];
            const bf16x8 v = y_perm[(size_t)src_row[r * k] * vec_per_row + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = a * (float)v[j];
        }
        for (int s = 1; s < k; ++s) {
            const float a = gate[r * k + s];
            const bf16x8 v = y_perm[(size_t)src_row[r * k + s] * vec_per_row + i];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += a * (float)v[j];
        }
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = (__bf16)acc[j];
        dst[p] = o;
    }
}

}  // namespace

int launch_combine(const void *y_perm, const int32_t *inv, const float *alpha, int32_t T, int32_t d,
                   void *y, hipStream_t st, const LaunchEvents *ev, int32_t k)
{
    const int n_tokens = T / k;
    hipExtLaunchKernelGGL(combine_rows, dim3((n_tokens + kCombineRows - 1) / kCombineRows), dim3(256), 0, st, ev ? ev->start : nullptr,
                          ev ? ev->stop : nullptr, 0, (const bf16x8 *)y_perm, inv, alpha, n_tokens, d / 8,
                          (bf16x8 *)y, k);
    return (int)hipGetLastError();
}

}  // namespace sida
