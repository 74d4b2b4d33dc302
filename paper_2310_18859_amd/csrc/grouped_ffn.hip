// K-b: grouped expert FFN on bf16 MFMA (gfx950).
//
// For every expert e of a wave, with its tokens in rows [offsets[e], offsets[e+1]) of x_perm:
//     h      = relu(x_perm_e * W_in[e]^T)      (GEMM 1, [rows, d] x [F, d]^T, ReLU, bf16 out)
//     y_perm = h * W_out[e]^T                  (GEMM 2, [rows, F] x [d, F]^T, bf16 out)
// which is the expert MLP f_i of Eq. 1 (Section 2.1) invoked only for experts that have tokens
// (Section 2.2).  Expert weights are read from the pool slot named by the wave table.
//
// Both GEMMs are "NT": activations [M,K] and weights [N,K] are K-contiguous, so every MFMA
// operand fragment (8 consecutive K values of one row) is one 16-byte access.
//
// Tiling: one workgroup (4 wavefronts, 2x2) computes a 128 (tokens) x 128 (weight rows) tile,
// K in steps of 64 through double-buffered LDS; each wavefront owns 64x64 = 2x2 MFMA 32x32x16
// tiles, fp32 accumulators.  The weight rows are fed as the MFMA's first operand and the token
// rows as the second, so a lane ends up with 4 consecutive output columns of one token row and
// stores them as one 8-byte piece.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = kGemmTileM;   // token rows per tile
constexpr int BN = 128;          // weight rows (output columns) per tile
constexpr int BK = 64;           // K step
constexpr int LDK = BK + 8;      // LDS row pitch in elements: 144 B keeps 16-byte reads conflict-free
constexpr int kStageElems = (BM + BN) * LDK;
constexpr int kLdsBytes = 2 * kStageElems * 2;

template <bool RELU>
__global__ __launch_bounds__(256) void grouped_gemm_nt(const __bf16 *__restrict__ A, __bf16 *__restrict__ C,
                                                       const char *__restrict__ pool, size_t expert_bytes,
                                                       size_t w_off, const int32_t *__restrict__ offsets,
                                                       const WaveTable tbl, int N, int K)
{
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    __bf16 *lds = reinterpret_cast<__bf16 *>(lds_raw);
    __shared__ int s_info[3];
    __shared__ int s_wsum[4];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int n_tiles_n = N / BN;
    const int nt = blockIdx.x % n_tiles_n;
    const int mt = blockIdx.x / n_tiles_n;

    // ---- which expert does token tile `mt` belong to?  thread i owns wave-table entry i ----
    int my_off = 0, my_cnt = 0, my_tiles = 0;
    if (tid < tbl.n) {
        const int e = tbl.expert[tid];
        my_off = offsets[e];
        my_cnt = offsets[e + 1] - my_off;
        my_tiles = (my_cnt + BM - 1) / BM;
    }
    int incl = my_tiles;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (tid < 3) s_info[tid] = 0;
    if (lane == 63) s_wsum[wv] = incl;
    __syncthreads();
    for (int i = 0; i < wv; ++i) incl += s_wsum[i];
    const int excl = incl - my_tiles;
    if (mt >= excl && mt < incl) {
        const int local = mt - excl;
        s_info[0] = tbl.slot[tid];
        s_info[1] = my_off + local * BM;
        s_info[2] = min(BM, my_cnt - local * BM);
    }
    __syncthreads();
    const int rows = s_info[2];
    if (rows <= 0) return;                                   // grid larger than the work: nothing to do
    const int row0 = s_info[1];
    const __bf16 *Wt = reinterpret_cast<const __bf16 *>(pool + (size_t)s_info[0] * expert_bytes + w_off) +
                       (size_t)nt * BN * K;
    const __bf16 *At = A + (size_t)row0 * K;

    // ---- global -> LDS staging: 4 + 4 16-byte pieces per thread per K step ----
    const int kc = (tid & 7) * 8;                            // K offset of this thread's pieces
    int a_row[4], b_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (tid >> 3) + 32 * i;
        a_row[i] = min(r, rows - 1);                         // rows past the end re-read the last valid row
        b_row[i] = r;
    }
    bf16x8 ga[4], gb[4];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ga[i] = *reinterpret_cast<const bf16x8 *>(At + (size_t)a_row[i] * K + k0 + kc);
            gb[i] = *reinterpret_cast<const bf16x8 *>(Wt + (size_t)b_row[i] * K + k0 + kc);
        }
    };
    auto store_lds = [&](int buf) {
        __bf16 *sa = lds + buf * kStageElems;
        __bf16 *sb = sa + BM * LDK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = (tid >> 3) + 32 * i;
            *reinterpret_cast<bf16x8 *>(sa + r * LDK + kc) = ga[i];
            *reinterpret_cast<bf16x8 *>(sb + r * LDK + kc) = gb[i];
        }
    };

    const int wm = wv & 1, wn = wv >> 1;                     // wavefront position in the 2x2 grid
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_global((kt + 1) * BK);
        const __bf16 *sa = lds + buf * kStageElems + (wm * 64 + frag_row) * LDK + frag_k;
        const __bf16 *sb = lds + buf * kStageElems + BM * LDK + (wn * 64 + frag_row) * LDK + frag_k;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 xf[2], wf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                xf[i] = *reinterpret_cast<const bf16x8 *>(sa + i * 32 * LDK + kk);
                wf[i] = *reinterpret_cast<const bf16x8 *>(sb + i * 32 * LDK + kk);
            }
#pragma unroll
            for (int in = 0; in < 2; ++in)
#pragma unroll
                for (int im = 0; im < 2; ++im)
                    acc[in][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[in], xf[im], acc[in][im], 0, 0, 0);
        }
        if (kt + 1 < nk) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds D[n][m] with m = lane&31 and n = 8*(r/4) + 4*(lane>>5) + r%4 ----
    const int half = lane >> 5;
#pragma unroll
    for (int im = 0; im < 2; ++im) {
        const int m = wm * 64 + im * 32 + frag_row;
        if (m >= rows) continue;
        __bf16 *crow = C + (size_t)(row0 + m) * N + (size_t)nt * BN + wn * 64;
#pragma unroll
        for (int in = 0; in < 2; ++in)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float v = acc[in][im][q * 4 + j];
                    if (RELU) v = v > 0.f ? v : 0.f;
                    o[j] = (__bf16)v;
                }
                *reinterpret_cast<bf16x4 *>(crow + in * 32 + q * 8 + half * 4) = o;
            }
    }
}

template <bool RELU>
int launch(const void *A, void *C, const char *pool, size_t expert_bytes, size_t w_off, const int32_t *offsets,
           const WaveTable &tbl, int N, int K, hipStream_t st)
{
    static bool attr_set = false;                            // per kernel instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&grouped_gemm_nt<RELU>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    if (tbl.m_tiles <= 0) return 0;
    const unsigned grid = (unsigned)tbl.m_tiles * (unsigned)(N / BN);
    hipLaunchKernelGGL(grouped_gemm_nt<RELU>, dim3(grid), dim3(256), kLdsBytes, st, (const __bf16 *)A, (__bf16 *)C,
                       pool, expert_bytes, w_off, offsets, tbl, N, K);
    return (int)hipGetLastError();
}

}  // namespace

int launch_ffn_gemm1(const void *x_perm, void *h, const char *pool, size_t expert_bytes, const int32_t *offsets,
                     const WaveTable &tbl, int32_t d, int32_t F, hipStream_t st)
{
    return launch<true>(x_perm, h, pool, expert_bytes, 0, offsets, tbl, F, d, st);
}

int launch_ffn_gemm2(const void *h, void *y_perm, const char *pool, size_t expert_bytes, const int32_t *offsets,
                     const WaveTable &tbl, int32_t d, int32_t F, hipStream_t st)
{
    return launch<false>(h, y_perm, pool, expert_bytes, (size_t)F * (size_t)d * 2, offsets, tbl, d, F, st);
}

}  // namespace sida
