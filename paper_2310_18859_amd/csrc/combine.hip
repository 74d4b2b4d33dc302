// K-c: gate-weighted scatter-combine.  The alpha factor of Eq. 1 (Section 2.1), applied while
// the expert outputs go back from expert order to token order:
//     y[t,:] = alpha[t] * y_perm[inv[t],:]
// The product is taken in fp32 and rounded to bf16 once (round to nearest even).
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

// One wavefront per token row; 16-byte accesses (8 bf16 values).
__global__ __launch_bounds__(256) void combine_rows(const bf16x8 *__restrict__ y_perm,
                                                    const int32_t *__restrict__ inv,
                                                    const float *__restrict__ alpha, int T, int vec_per_row,
                                                    bf16x8 *__restrict__ y)
{
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = threadIdx.x & 63;
    const float a = alpha[t];
    const bf16x8 *src = y_perm + (size_t)inv[t] * vec_per_row;
    bf16x8 *dst = y + (size_t)t * vec_per_row;
    for (int i = lane; i < vec_per_row; i += 64) {
        const bf16x8 v = src[i];
        bf16x8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = (__bf16)(a * (float)v[j]);
        dst[i] = o;
    }
}

}  // namespace

int launch_combine(const void *y_perm, const int32_t *inv, const float *alpha, int32_t T, int32_t d,
                   void *y, hipStream_t st, const LaunchEvents *ev)
{
    hipExtLaunchKernelGGL(combine_rows, dim3((T + 3) / 4), dim3(256), 0, st, ev ? ev->start : nullptr,
                          ev ? ev->stop : nullptr, 0, (const bf16x8 *)y_perm, inv, alpha, T, d / 8, (bf16x8 *)y);
    return (int)hipGetLastError();
}

}  // namespace sida
