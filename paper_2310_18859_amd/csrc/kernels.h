// Launchers of the HIP kernels.  Each returns the hipError_t of its launch (as int).
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace sida {

// Experts of one wave in the order their tiles are scheduled (largest first), passed to the
// grouped GEMM kernels by value as a kernel argument.
struct WaveTable {
    int32_t n;                 // experts in the wave
    int32_t m_tiles;           // sum over the wave's experts of ceil(count / tile rows)
    int16_t slot[256];         // pool slot of entry i
    uint8_t expert[256];       // expert id of entry i
};

// K-a: stable counting sort of T tokens by expert id.
//   ids int32[T] -> counts[E], offsets[E+1], perm[T], inv[T];  block_hist is scratch [n_chunks*E].
int launch_sort(const int32_t *ids, int32_t T, int32_t E, int32_t *counts, int32_t *offsets,
                int32_t *block_hist, int32_t *perm, int32_t *inv, hipStream_t st);
// K-a: x_perm[r,:] = x[perm[r],:], rows of d bf16 values.
int launch_gather(const void *x, const int32_t *perm, int32_t T, int32_t d, void *x_perm, hipStream_t st);
// K-b: h = relu(x_perm W_in^T) then y_perm = h W_out^T for the experts in tbl.
int launch_ffn_gemm1(const void *x_perm, void *h, const char *pool, size_t expert_bytes,
                     const int32_t *offsets, const WaveTable &tbl, int32_t d, int32_t F, hipStream_t st);
int launch_ffn_gemm2(const void *h, void *y_perm, const char *pool, size_t expert_bytes,
                     const int32_t *offsets, const WaveTable &tbl, int32_t d, int32_t F, hipStream_t st);
// K-c: y[t,:] = alpha[t] * y_perm[inv[t],:].
int launch_combine(const void *y_perm, const int32_t *inv, const float *alpha, int32_t T, int32_t d,
                   void *y, hipStream_t st);

constexpr int kGemmTileM = 128;   // token rows per GEMM tile (WaveTable::m_tiles is counted in these)

}  // namespace sida
