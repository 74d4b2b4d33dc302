// The hash function of the hash-building thread (Section 3.4.2): predicts, for every token of a
// sequence and every MoE layer, the experts to activate and their scaling factors, from the token
// embeddings alone - a fully connected layer that compresses the embedding, a 2-layer LSTM, an
// attention layer over the LSTM's output sequence whose weights go through SparseMax, a residual
// connection, and one linear head per MoE layer (Algorithm 1, right column: k <- h_l(X)[s]).
// Readings where the paper gives no detail: compressed width = LSTM hidden width C; standard LSTM
// cell (gates input, forget, cell, output), zero initial state; dot-product scores without scaling;
// the residual adds the token's own compressed embedding; alpha = SoftMax probability of the
// expert within its layer's head; the k largest are kept, ties to the lower expert id.
//
// A lightweight network (a few MFLOP per token): plain fp32 kernels, one launch per stage (the
// dense stages are fp32 contractions; the fp32 matrix-core rate of this chip equals its vector
// rate, and bf16 inputs would move the predicted probabilities by more than the parity bound).  The
// recurrent part keeps a gate row of W_hh in the registers of each of the 4C threads of a
// sequence's workgroup and the state in LDS; SparseMax finds its threshold by bisection on
// sum(max(s - tau, 0)) = 1 and then takes the closed form on the support that bisection found.
#include <hip/hip_runtime.h>

#include <cfloat>
#include <mutex>

#include "kernels.h"

namespace sida {

namespace {

// Scratch of sida_hash_forward_static: the intermediates of one call (8*C floats per token) live
// here instead of in a caller's workspace.  Every GPU the library runs on holds its own copy of
// the array, at its own address, until the process ends.  In host code the array's name is only a
// stand-in for the symbol: the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[kHashStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float *g_scratch_ptr[kMaxDevices] = {};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

__device__ __forceinline__ float sigmoidf_(float v) { return 1.f / (1.f + __expf(-v)); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// The three dense stages (compress, gate pre-activations, heads) take kTokenBlock tokens per
// workgroup: a thread owns one output unit, reads its weight row once and applies it to every
// token of the block (the tokens' inputs sit in LDS and are read as broadcasts), so a weight matrix
// is fetched once per block instead of once per token.  Each (token, unit) sum runs in index order.
constexpr int kTokenBlock = 8;

// c0[n, j] = b_in[j] + sum_i x[n, i] * w_in[j, i].  One workgroup of C threads per block of TB tokens.
template <int C, int TB>
__global__ __launch_bounds__(C) void hash_compress(const __bf16 *__restrict__ x, const float *__restrict__ w_in,
                                                   const float *__restrict__ b_in, int d, int n_tokens,
                                                   float *__restrict__ c0)
{
    extern __shared__ __attribute__((aligned(16))) float xs[];                              // [TB][d] the tokens' embeddings, fp32
    const int n0 = blockIdx.x * TB, j = threadIdx.x;
    const int nb = min(TB, n_tokens - n0);
    for (int i = j; i < TB * d; i += C) {
        const int tb = i / d;
        xs[i] = tb < nb ? (float)x[(size_t)n0 * d + i] : 0.f;
    }
    __syncthreads();
    const float4 *w = reinterpret_cast<const float4 *>(w_in + (size_t)j * d);
    float acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = b_in[j];
    for (int i = 0; i < d / 4; ++i) {
        const float4 wv = w[i];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const float4 xv = *reinterpret_cast<const float4 *>(xs + tb * d + 4 * i);
            acc[tb] += xv.x * wv.x;
            acc[tb] += xv.y * wv.y;
            acc[tb] += xv.z * wv.z;
            acc[tb] += xv.w * wv.w;
        }
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
        if (tb < nb) c0[(size_t)(n0 + tb) * C + j] = acc[tb];
}

// pre[n, g] = b_ih[g] + b_hh[g] + sum_i in[n, i] * w_ih[g, i].  One workgroup of 4C threads per block of TB tokens.
template <int C, int TB>
__global__ __launch_bounds__(4 * C) void hash_gates_in(const float *__restrict__ in, const float *__restrict__ w_ih,
                                                       const float *__restrict__ b_ih, const float *__restrict__ b_hh,
                                                       int n_tokens, float *__restrict__ pre)
{
    __shared__ __attribute__((aligned(16))) float row[TB][C];
    const int n0 = blockIdx.x * TB, g = threadIdx.x;
    const int nb = min(TB, n_tokens - n0);
    for (int i = g; i < TB * C; i += 4 * C) (&row[0][0])[i] = i / C < nb ? in[(size_t)n0 * C + i] : 0.f;
    __syncthreads();
    const float4 *w = reinterpret_cast<const float4 *>(w_ih + (size_t)g * C);
    float acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = b_ih[g] + b_hh[g];
#pragma unroll 4
    for (int i = 0; i < C / 4; ++i) {
        const float4 wv = w[i];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const float4 xv = *reinterpret_cast<const float4 *>(&row[tb][4 * i]);
            acc[tb] += xv.x * wv.x;
            acc[tb] += xv.y * wv.y;
            acc[tb] += xv.z * wv.z;
            acc[tb] += xv.w * wv.w;
        }
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
        if (tb < nb) pre[(size_t)(n0 + tb) * 4 * C + g] = acc[tb];
}

// The recurrence of one LSTM layer.  One workgroup of 4C threads per sequence: thread g owns gate
// row g of W_hh (in registers) and, for g < C, the cell state of unit g.
template <int C>
__global__ __launch_bounds__(4 * C) void hash_lstm(const float *__restrict__ pre, const float *__restrict__ w_hh, int T,
                                                   float *__restrict__ out)
{
    __shared__ float h[C];
    __shared__ float gates[4 * C];
    const int b = blockIdx.x, g = threadIdx.x;
    float w[C];
#pragma unroll
    for (int i = 0; i < C; ++i) w[i] = w_hh[(size_t)g * C + i];
    if (g < C) h[g] = 0.f;
    float cell = 0.f;
    __syncthreads();
    for (int t = 0; t < T; ++t) {
        const size_t n = (size_t)b * T + t;
        float acc = pre[n * 4 * C + g];
#pragma unroll
        for (int i = 0; i < C; ++i) acc += w[i] * h[i];
        gates[g] = (g >= 2 * C && g < 3 * C) ? tanhf(acc) : sigmoidf_(acc);
        __syncthreads();
        if (g < C) {
            cell = gates[C + g] * cell + gates[g] * gates[2 * C + g];
            const float hv = gates[3 * C + g] * tanhf(cell);
            h[g] = hv;
            out[n * C + g] = hv;
        }
        __syncthreads();
    }
}

// Sparse attention + residual for one query token: r[t] = c0[t] + sum_u sparsemax_u(h2[t] . h2[u]) h2[u].
// One wavefront per token; scores of the sequence in LDS.
template <int C>
__global__ __launch_bounds__(64) void hash_attention(const float *__restrict__ h2, const float *__restrict__ c0, int T,
                                                     float *__restrict__ r)
{
    extern __shared__ float s[];                               // [T] scores, then weights
    __shared__ float q[C];
    const int n = blockIdx.x, lane = threadIdx.x;
    const int seq0 = (n / T) * T;                              // first token of this sequence
    for (int i = lane; i < C; i += 64) q[i] = h2[(size_t)n * C + i];
    __syncthreads();
    float mx = -FLT_MAX;
    for (int u = lane; u < T; u += 64) {
        const float *k = h2 + (size_t)(seq0 + u) * C;
        float acc = 0.f;
#pragma unroll 8
        for (int i = 0; i < C; ++i) acc += q[i] * k[i];
        s[u] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    __syncthreads();
    // threshold: sum_u max(s_u - tau, 0) is 1 somewhere in [max - 1, max]
    float lo = mx - 1.f, hi = mx;
    for (int it = 0; it < 30; ++it) {
        const float tau = 0.5f * (lo + hi);
        float part = 0.f;
        for (int u = lane; u < T; u += 64) part += fmaxf(s[u] - tau, 0.f);
        if (wave_sum(part) >= 1.f) lo = tau;
        else hi = tau;
    }
    // closed form on the support the bisection found
    float sum_s = 0.f, cnt = 0.f;
    for (int u = lane; u < T; u += 64)
        if (s[u] > lo) {
            sum_s += s[u];
            cnt += 1.f;
        }
    sum_s = wave_sum(sum_s);
    cnt = wave_sum(cnt);
    const float tau = cnt > 0.f ? (sum_s - 1.f) / cnt : lo;
    for (int u = lane; u < T; u += 64) s[u] = fmaxf(s[u] - tau, 0.f);
    __syncthreads();
    for (int i = lane; i < C; i += 64) {
        float acc = c0[(size_t)n * C + i];
        for (int u = 0; u < T; ++u) {
            const float p = s[u];                              // same address for every lane: a broadcast
            if (p > 0.f) acc += p * h2[(size_t)(seq0 + u) * C + i];
        }
        r[(size_t)n * C + i] = acc;
    }
}

// Heads: per MoE layer l the E logits of a token, their SoftMax, and the k most probable experts.
// One workgroup of 256 threads per block of TB tokens; wavefront w takes the (token, layer) pairs
// w, w+4, ...
template <int C, int TB>
__global__ __launch_bounds__(256) void hash_heads(const float *__restrict__ r, const float *__restrict__ w_out,
                                                  const float *__restrict__ b_out, int L, int E, int top_k,
                                                  int n_tokens, int32_t *__restrict__ ids, float *__restrict__ alpha)
{
    extern __shared__ __attribute__((aligned(16))) float logit[];                           // [TB][L*E]
    __shared__ __attribute__((aligned(16))) float row[TB][C];
    const int n0 = blockIdx.x * TB, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nb = min(TB, n_tokens - n0);
    const int LE = L * E;
    for (int i = tid; i < TB * C; i += 256) (&row[0][0])[i] = i / C < nb ? r[(size_t)n0 * C + i] : 0.f;
    __syncthreads();
    for (int o = tid; o < LE; o += 256) {
        const float4 *w = reinterpret_cast<const float4 *>(w_out + (size_t)o * C);
        float acc[TB];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[tb] = b_out[o];
#pragma unroll 4
        for (int i = 0; i < C / 4; ++i) {
            const float4 wv4 = w[i];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const float4 xv = *reinterpret_cast<const float4 *>(&row[tb][4 * i]);
                acc[tb] += xv.x * wv4.x;
                acc[tb] += xv.y * wv4.y;
                acc[tb] += xv.z * wv4.z;
                acc[tb] += xv.w * wv4.w;
            }
        }
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) logit[tb * LE + o] = acc[tb];
    }
    __syncthreads();
    for (int pair = wv; pair < nb * L; pair += 4) {
        const int tb = pair / L, l = pair % L, n = n0 + tb;
        float *z = logit + tb * LE + l * E;
        float mx = -FLT_MAX;
        for (int e = lane; e < E; e += 64) mx = fmaxf(mx, z[e]);
        mx = wave_max(mx);
        float sum = 0.f;
        for (int e = lane; e < E; e += 64) sum += __expf(z[e] - mx);
        sum = wave_sum(sum);
        for (int j = 0; j < top_k; ++j) {
            // largest remaining logit, ties to the lower expert id
            float best = -FLT_MAX;
            int arg = E;
            for (int e = lane; e < E; e += 64)
                if (z[e] > best) {
                    best = z[e];
                    arg = e;
                }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ob = __shfl_xor(best, o, 64);
                const int oa = __shfl_xor(arg, o, 64);
                if (ob > best || (ob == best && oa < arg)) {
                    best = ob;
                    arg = oa;
                }
            }
            if (lane == 0) {
                const size_t at = ((size_t)l * n_tokens + n) * top_k + j;
                ids[at] = arg < E ? arg : 0;
                alpha[at] = __expf(best - mx) / sum;
            }
            if (arg < E && lane == (arg & 63)) z[arg] = -FLT_MAX;          // taken
            __builtin_amdgcn_wave_barrier();
        }
    }
}

template <int C>
int run(const HashShape &sh, const float *p, const void *x, int n_seq, int T, int32_t *ids, float *alpha, float *ws,
        hipStream_t st)
{
    const int N = n_seq * T, d = sh.d_model;
    // parameters, packed in this order
    const float *w_in = p, *b_in = w_in + (size_t)C * d;
    const float *w_ih1 = b_in + C, *w_hh1 = w_ih1 + 4 * C * C, *b_ih1 = w_hh1 + 4 * C * C, *b_hh1 = b_ih1 + 4 * C;
    const float *w_ih2 = b_hh1 + 4 * C, *w_hh2 = w_ih2 + 4 * C * C, *b_ih2 = w_hh2 + 4 * C * C, *b_hh2 = b_ih2 + 4 * C;
    const float *w_out = b_hh2 + 4 * C, *b_out = w_out + (size_t)sh.L * sh.E * C;
    // workspace
    float *c0 = ws, *pre = c0 + (size_t)N * C, *h1 = pre + (size_t)N * 4 * C, *h2 = h1 + (size_t)N * C,
          *r = h2 + (size_t)N * C;
    // Tokens per workgroup of the dense stages: 8 when that still gives every compute unit several
    // workgroups, fewer for short batches (one 128-token sequence: 1, as many workgroups as tokens),
    // and never more than fit 48 KiB of LDS.
    constexpr size_t kLdsCap = 48 * 1024;
    const int want = N >= 4096 ? kTokenBlock : N >= 1024 ? 2 : 1;
    auto block_for = [&](size_t bytes_per_token) {
        int tb = want;
        while (tb > 1 && tb * bytes_per_token > kLdsCap) tb = tb == kTokenBlock ? 2 : 1;
        return tb;
    };
    auto blocks = [&](int tb) { return dim3((N + tb - 1) / tb); };
    const size_t x_bytes = d * sizeof(float), le_bytes = (size_t)sh.L * sh.E * sizeof(float);
    const __bf16 *xb = (const __bf16 *)x;
    switch (block_for(x_bytes)) {
        case kTokenBlock: hipLaunchKernelGGL((hash_compress<C, kTokenBlock>), blocks(kTokenBlock), dim3(C), kTokenBlock * x_bytes, st, xb, w_in, b_in, d, N, c0); break;
        case 2: hipLaunchKernelGGL((hash_compress<C, 2>), blocks(2), dim3(C), 2 * x_bytes, st, xb, w_in, b_in, d, N, c0); break;
        default: hipLaunchKernelGGL((hash_compress<C, 1>), blocks(1), dim3(C), x_bytes, st, xb, w_in, b_in, d, N, c0); break;
    }
    auto gates = [&](const float *in, const float *w_ih, const float *b_ih, const float *b_hh) {
        switch (want) {
            case kTokenBlock: hipLaunchKernelGGL((hash_gates_in<C, kTokenBlock>), blocks(kTokenBlock), dim3(4 * C), 0, st, in, w_ih, b_ih, b_hh, N, pre); break;
            case 2: hipLaunchKernelGGL((hash_gates_in<C, 2>), blocks(2), dim3(4 * C), 0, st, in, w_ih, b_ih, b_hh, N, pre); break;
            default: hipLaunchKernelGGL((hash_gates_in<C, 1>), blocks(1), dim3(4 * C), 0, st, in, w_ih, b_ih, b_hh, N, pre); break;
        }
    };
    gates(c0, w_ih1, b_ih1, b_hh1);
    hipLaunchKernelGGL(hash_lstm<C>, dim3(n_seq), dim3(4 * C), 0, st, pre, w_hh1, T, h1);
    gates(h1, w_ih2, b_ih2, b_hh2);
    hipLaunchKernelGGL(hash_lstm<C>, dim3(n_seq), dim3(4 * C), 0, st, pre, w_hh2, T, h2);
    hipLaunchKernelGGL(hash_attention<C>, dim3(N), dim3(64), T * sizeof(float), st, h2, c0, T, r);
    switch (block_for(le_bytes)) {
        case kTokenBlock: hipLaunchKernelGGL((hash_heads<C, kTokenBlock>), blocks(kTokenBlock), dim3(256), kTokenBlock * le_bytes, st, r, w_out, b_out, sh.L, sh.E, sh.top_k, N, ids, alpha); break;
        case 2: hipLaunchKernelGGL((hash_heads<C, 2>), blocks(2), dim3(256), 2 * le_bytes, st, r, w_out, b_out, sh.L, sh.E, sh.top_k, N, ids, alpha); break;
        default: hipLaunchKernelGGL((hash_heads<C, 1>), blocks(1), dim3(256), le_bytes, st, r, w_out, b_out, sh.L, sh.E, sh.top_k, N, ids, alpha); break;
    }
    return (int)hipGetLastError();
}

}  // namespace

int hash_static_scratch(float **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // the current device's copy of the array
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_scratch_ptr[dev];
    return 0;
}

int launch_hash_forward(const HashShape &sh, const float *params, const void *x, int32_t n_seq, int32_t seq_len,
                        int32_t *ids, float *alpha, float *ws, hipStream_t st)
{
    if (sh.C == 64) return run<64>(sh, params, x, n_seq, seq_len, ids, alpha, ws, st);
    return run<128>(sh, params, x, n_seq, seq_len, ids, alpha, ws, st);
}

}  // namespace sida
