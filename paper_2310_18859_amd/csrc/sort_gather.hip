// K-a: token -> expert stable counting sort and permute-gather.
//
// Any implementation that invokes only the experts that have tokens (Section 2.3) must bring the
// rows of one expert together.  The order is fixed as (expert id, token index) so that the result
// is unique: perm[offsets[e] + j] is the j-th smallest token index routed to expert e.
//
// By size of the call: one workgroup (sort_one, up to 4096 tokens), one launch of independent
// workgroups (sort_chunks, up to 65536 tokens), or three small launches (one workgroup doing the
// whole sort was measured at 20 us for 16384 tokens: the ballot ranking is VALU-bound on a single
// compute unit):
//   sort_hist   one wavefront per chunk of 256 tokens: LDS histogram of the chunk
//   sort_scan   one workgroup: per-expert totals, exclusive scan over experts (offsets), the
//               first output row of every (chunk, expert) pair, and the grouped FFN's token-tile
//               descriptors
//   sort_rank   one wavefront per chunk: rank of a token among equal ids = (tokens of that id in
//               earlier chunks) + (earlier rounds of this chunk) + (lower lanes of this round, by
//               wavefront ballots over the 8 id bits)
// plus the row gather (gather_rows, 16-byte accesses) when it is not folded into the first GEMM.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace sida {

namespace {

constexpr int kChunk = 256;      // tokens per wavefront (4 rounds of 64)
constexpr int kMaxE = 256;

__device__ __forceinline__ int clamp_id(int k, int E) { return k < 0 ? 0 : (k >= E ? E - 1 : k); }

__global__ __launch_bounds__(64) void sort_hist(const int32_t *__restrict__ ids, int T, int E,
                                                int32_t *__restrict__ block_hist)
{
    __shared__ int hist[kMaxE];
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) hist[e] = 0;
    __syncthreads();
    const int base = blockIdx.x * kChunk;
#pragma unroll
    for (int r = 0; r < kChunk / 64; ++r) {
        const int t = base + r * 64 + lane;
        if (t < T) atomicAdd(&hist[clamp_id(ids[t], E)], 1);
    }
    __syncthreads();
    for (int e = lane; e < E; e += 64) block_hist[(size_t)blockIdx.x * E + e] = hist[e];
}

// One workgroup of 1024 threads: thread (p, e) owns expert e over quarter p of the chunks, so the
// walks over the chunks are short and their loads are issued 8 at a time.  Also expands the
// layer's expert table into the token-tile descriptors of the grouped FFN (thread i: entry i).
__global__ __launch_bounds__(1024) void sort_scan(int32_t *__restrict__ block_hist, int n_chunks, int E, int T,
                                                  int32_t *__restrict__ counts, int32_t *__restrict__ offsets,
                                                  const LayerTable tbl, TileDesc *__restrict__ tiles, int max_tiles)
{
    __shared__ int part[4][kMaxE];
    __shared__ int s_off[kMaxE + 1];
    __shared__ int s_wsum[4];
    const int tid = threadIdx.x, e = tid & 255, p = tid >> 8;
    const int per = (n_chunks + 3) / 4;
    const int b0 = p * per, b1 = min(n_chunks, b0 + per);

    int sum = 0;
    if (e < E)
        for (int b = b0; b < b1; b += 8) {
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = b + i < b1 ? block_hist[(size_t)(b + i) * E + e] : 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) sum += v[i];
        }
    part[p][e] = sum;
    __syncthreads();

    const int lane = tid & 63, wv = tid >> 6;
    int total = 0, incl = 0;
    if (tid < 256) {
        total = part[0][e] + part[1][e] + part[2][e] + part[3][e];
        if (e >= E) total = 0;
        incl = total;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wsum[wv] = incl;
    }
    __syncthreads();
    if (tid < 256) {
        for (int i = 0; i < wv; ++i) incl += s_wsum[i];
        const int excl = incl - total;
        if (e < E) {
            counts[e] = total;
            offsets[e] = excl;
            s_off[e] = excl;
            if (e == E - 1) {
                offsets[E] = T;
                s_off[E] = T;
            }
        }
    }
    __syncthreads();

    // first output row of (chunk b, expert e) for this thread's chunks
    if (e < E) {
        int run = s_off[e];
        for (int q = 0; q < p; ++q) run += part[q][e];
        for (int b = b0; b < b1; b += 8) {
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = b + i < b1 ? block_hist[(size_t)(b + i) * E + e] : 0;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (b + i < b1) {
                    block_hist[(size_t)(b + i) * E + e] = run;
                    run += v[i];
                }
        }
    }

    if (tbl.n > 0) {
        int ex = 0, slot = 0, off = 0, cnt = 0, n_t = 0;
        if (tid < tbl.n) {
            ex = tbl.expert[tid];
            slot = tbl.slot[tid];
            off = s_off[ex];
            cnt = s_off[ex + 1] - off;
            n_t = (cnt + tbl.tile_m - 1) / tbl.tile_m;
        }
        __syncthreads();                                        // s_wsum is reused
        int inc2 = n_t;
        if (tid < 256) {
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(inc2, o, 64);
                if (lane >= o) inc2 += v;
            }
            if (lane == 63) s_wsum[wv] = inc2;
        }
        __syncthreads();
        if (tid < 256) {
            for (int i = 0; i < wv; ++i) inc2 += s_wsum[i];
            int at = inc2 - n_t;
            for (int k = 0; k < n_t && at < max_tiles; ++k, ++at) {
                TileDesc td;
                td.slot = slot;
                td.row0 = off + k * tbl.tile_m;
                td.rows = min(tbl.tile_m, cnt - k * tbl.tile_m);
                td.expert = ex;
                tiles[at] = td;
            }
        }
    }
}

__global__ __launch_bounds__(64) void sort_rank(const int32_t *__restrict__ ids, int T, int E,
                                                const int32_t *__restrict__ block_base,
                                                int32_t *__restrict__ perm, int32_t *__restrict__ inv,
                                                const float *__restrict__ alpha, float *__restrict__ gate_perm)
{
    __shared__ int next_row[kMaxE];
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) next_row[e] = block_base[(size_t)blockIdx.x * E + e];
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
    const int base = blockIdx.x * kChunk;
#pragma unroll
    for (int r = 0; r < kChunk / 64; ++r) {
        const int t = base + r * 64 + lane;
        const bool live = t < T;
        const int k = live ? clamp_id(ids[t], E) : 0;
        // lanes of this round that hold the same id
        unsigned long long same = __ballot(live);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const unsigned long long b = __ballot((k >> bit) & 1);
            same &= ((k >> bit) & 1) ? b : ~b;
        }
        if (live) {
            const int ahead = __popcll(same & below);
            const int row = next_row[k] + ahead;
            perm[row] = t;
            inv[t] = row;
            if (alpha) gate_perm[row] = alpha[t];
        }
        __syncthreads();               // every lane has read next_row before anyone advances it
        if (live && (same & below) == 0) next_row[k] += __popcll(same);
        __syncthreads();
    }
}

// The whole sort in one workgroup for layer calls of up to 4096 tokens (from one or two sequences
// per batch, the paper's serving regime, upwards): wavefront w owns chunks w*CPW .. w*CPW+CPW-1,
// the per-chunk histograms and bases live in LDS, and the three launches above shrink to one.
// Same results.  NWV wavefronts x CPW chunks of 256 tokens.  Measured: 9 us up to 2048 tokens and
// 10 us (14 us when the gate values move along) at 4096 against 17-19 us for the three launches; at
// 8192 tokens (16 x 2 chunks) 15 us and 24 us, the latter slower than the three launches.
constexpr int kOneT = 4096;      // most tokens the single-workgroup sort takes

template <int NWV, int CPW>
__global__ __launch_bounds__(NWV * 64) void sort_one(const int32_t *__restrict__ ids, int T, int E,
                                                     int32_t *__restrict__ counts, int32_t *__restrict__ offsets,
                                                     int32_t *__restrict__ perm, int32_t *__restrict__ inv,
                                                     const float *__restrict__ alpha, float *__restrict__ gate_perm,
                                                     const LayerTable tbl, TileDesc *__restrict__ tiles, int max_tiles)
{
    constexpr int NCH = NWV * CPW;
    __shared__ int hist[NCH][kMaxE];               // per-chunk histogram, then first output row of (chunk, expert)
    __shared__ int s_off[kMaxE + 1];
    __shared__ int s_wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    for (int i = tid; i < NCH * kMaxE; i += NWV * 64) (&hist[0][0])[i] = 0;
    __syncthreads();

    int my_id[CPW][kChunk / 64];
#pragma unroll
    for (int j = 0; j < CPW; ++j)
#pragma unroll
        for (int r = 0; r < kChunk / 64; ++r) {
            const int t = (wv * CPW + j) * kChunk + r * 64 + lane;
            my_id[j][r] = t < T ? clamp_id(ids[t], E) : -1;
            if (my_id[j][r] >= 0) atomicAdd(&hist[wv * CPW + j][my_id[j][r]], 1);
        }
    __syncthreads();

    // expert totals -> offsets (threads 0..255: one expert each), then the bases of every chunk
    int total = 0, incl = 0;
    if (tid < 256) {
        if (tid < E)
            for (int c = 0; c < NCH; ++c) total += hist[c][tid];
        incl = total;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o, 64);
            if (lane >= o) incl += v;
        }
        if (lane == 63) s_wsum[wv] = incl;
    }
    __syncthreads();
    if (tid < 256) {
        for (int i = 0; i < wv; ++i) incl += s_wsum[i];
        const int excl = incl - total;
        if (tid < E) {
            counts[tid] = total;
            offsets[tid] = excl;
            s_off[tid] = excl;
            if (tid == E - 1) {
                offsets[E] = T;
                s_off[E] = T;
            }
            int run = excl;
            for (int c = 0; c < NCH; ++c) {
                const int v = hist[c][tid];
                hist[c][tid] = run;
                run += v;
            }
        }
    }
    __syncthreads();

    // token tiles of the grouped FFN (as in sort_scan)
    if (tbl.n > 0) {
        int ex = 0, slot = 0, off = 0, cnt = 0, n_t = 0;
        if (tid < tbl.n) {
            ex = tbl.expert[tid];
            slot = tbl.slot[tid];
            off = s_off[ex];
            cnt = s_off[ex + 1] - off;
            n_t = (cnt + tbl.tile_m - 1) / tbl.tile_m;
        }
        int inc2 = n_t;
        if (tid < 256) {
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int v = __shfl_up(inc2, o, 64);
                if (lane >= o) inc2 += v;
            }
        }
        __syncthreads();                                        // s_wsum is reused
        if (tid < 256 && lane == 63) s_wsum[wv] = inc2;
        __syncthreads();
        if (tid < 256) {
            for (int i = 0; i < wv; ++i) inc2 += s_wsum[i];
            int at = inc2 - n_t;
            for (int k = 0; k < n_t && at < max_tiles; ++k, ++at) {
                TileDesc td;
                td.slot = slot;
                td.row0 = off + k * tbl.tile_m;
                td.rows = min(tbl.tile_m, cnt - k * tbl.tile_m);
                td.expert = ex;
                tiles[at] = td;
            }
        }
    }

    // ranks: wavefront w walks its chunks in rounds of 64 tokens (LDS accesses of one wavefront
    // execute in program order, so the reads of a round precede its updates)
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        int *next_row = hist[wv * CPW + j];
#pragma unroll
        for (int r = 0; r < kChunk / 64; ++r) {
            const int t = (wv * CPW + j) * kChunk + r * 64 + lane;
            const bool live = my_id[j][r] >= 0;
            const int k = live ? my_id[j][r] : 0;
            unsigned long long same = __ballot(live);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const unsigned long long b = __ballot((k >> bit) & 1);
                same &= ((k >> bit) & 1) ? b : ~b;
            }
            int row = 0;
            if (live) row = next_row[k] + __popcll(same & below);
            __builtin_amdgcn_wave_barrier();
            if (live && (same & below) == 0) next_row[k] += __popcll(same);
            __builtin_amdgcn_wave_barrier();
            if (live) {
                perm[row] = t;
                inv[t] = row;
                if (alpha) gate_perm[row] = alpha[t];
            }
        }
    }
}

// The whole sort in ONE launch for calls between kOneT and kChunksT tokens, without any exchange
// between workgroups: workgroup c (one per chunk of kFineChunk tokens) histograms ALL ids itself - those
// before its chunk and the rest separately, 64 KiB of L2-resident ids at 16384 tokens - which gives
// it the expert totals (hence the offsets) and the number of tokens of every expert in earlier
// chunks, i.e. the first output row of each of its (chunk, expert) pairs; its first wavefront
// then ranks the chunk's tokens as sort_rank does.  Workgroup 0 also writes counts, offsets and the
// token tiles.  Same results as the three launches (17 us at 16384 tokens) in about half the time.
constexpr int kChunksT = 65536;
constexpr int kFineChunk = 128;                    // two ranking rounds per workgroup
constexpr int kIdLoads = 8;                        // 16-byte id loads in flight per thread
__global__ __launch_bounds__(256) void sort_chunks(const int32_t *__restrict__ ids, int T, int E,
                                                   int32_t *__restrict__ counts, int32_t *__restrict__ offsets,
                                                   int32_t *__restrict__ perm, int32_t *__restrict__ inv,
                                                   const float *__restrict__ alpha, float *__restrict__ gate_perm,
                                                   const LayerTable tbl, TileDesc *__restrict__ tiles, int max_tiles)
{
    __shared__ int s_rest[kMaxE];                  // tokens per expert from this chunk on
    __shared__ int s_before[kMaxE];                // ... in earlier chunks, then the next output row
    __shared__ int s_off[kMaxE + 1];
    __shared__ int s_wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int my0 = blockIdx.x * kFineChunk;
    s_rest[tid] = 0;
    s_before[tid] = 0;
    __syncthreads();
    // four ids per load, kIdLoads loads in flight per thread
    const int n4 = T >> 2;
    const int4 *ids4 = reinterpret_cast<const int4 *>(ids);
    for (int base = tid; base < n4; base += 256 * kIdLoads) {
        int4 v[kIdLoads];
#pragma unroll
        for (int u = 0; u < kIdLoads; ++u) v[u] = ids4[min(base + u * 256, n4 - 1)];   // unconditional loads
#pragma unroll
        for (int u = 0; u < kIdLoads; ++u)
            if (base + u * 256 < n4) {
                int *h = (base + u * 256) * 4 < my0 ? s_before : s_rest;   // chunks start at multiples of 4
                atomicAdd(&h[clamp_id(v[u].x, E)], 1);
                atomicAdd(&h[clamp_id(v[u].y, E)], 1);
                atomicAdd(&h[clamp_id(v[u].z, E)], 1);
                atomicAdd(&h[clamp_id(v[u].w, E)], 1);
            }
    }
    if (tid < (T & 3)) {                           // the last T % 4 ids
        const int t = (n4 << 2) + tid;
        atomicAdd(&(t < my0 ? s_before : s_rest)[clamp_id(ids[t], E)], 1);
    }
    __syncthreads();

    // expert totals -> offsets (thread e: expert e), then this chunk's first row per expert
    const int before = s_before[tid];
    int total = tid < E ? before + s_rest[tid] : 0, incl = total;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) s_wsum[wv] = incl;
    __syncthreads();
    for (int i = 0; i < wv; ++i) incl += s_wsum[i];
    const int excl = incl - total;
    if (tid < E) {
        s_off[tid] = excl;
        if (tid == E - 1) s_off[E] = T;
        s_before[tid] = excl + before;             // next output row of (this chunk, expert tid)
        if (blockIdx.x == 0) {
            counts[tid] = total;
            offsets[tid] = excl;
            if (tid == E - 1) offsets[E] = T;
        }
    }
    __syncthreads();

    // token tiles of the grouped FFN (as in sort_scan), by workgroup 0
    if (blockIdx.x == 0 && tbl.n > 0) {
        int ex = 0, slot = 0, off = 0, cnt = 0, n_t = 0;
        if (tid < tbl.n) {
            ex = tbl.expert[tid];
            slot = tbl.slot[tid];
            off = s_off[ex];
            cnt = s_off[ex + 1] - off;
            n_t = (cnt + tbl.tile_m - 1) / tbl.tile_m;
        }
        int inc2 = n_t;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(inc2, o, 64);
            if (lane >= o) inc2 += v;
        }
        __syncthreads();                           // s_wsum is reused
        if (lane == 63) s_wsum[wv] = inc2;
        __syncthreads();
        for (int i = 0; i < wv; ++i) inc2 += s_wsum[i];
        int at = inc2 - n_t;
        for (int k = 0; k < n_t && at < max_tiles; ++k, ++at) {
            TileDesc td;
            td.slot = slot;
            td.row0 = off + k * tbl.tile_m;
            td.rows = min(tbl.tile_m, cnt - k * tbl.tile_m);
            td.expert = ex;
            tiles[at] = td;
        }
    }

    // ranks: the first wavefront walks the chunk in rounds of 64 tokens (LDS accesses of one
    // wavefront execute in program order, so the reads of a round precede its updates)
    if (wv != 0) return;
    int *next_row = s_before;
    const unsigned long long below = (1ull << lane) - 1ull;
    int my_id[kFineChunk / 64];
#pragma unroll
    for (int r = 0; r < kFineChunk / 64; ++r) {
        const int t = my0 + r * 64 + lane;
        my_id[r] = t < T ? clamp_id(ids[t], E) : -1;
    }
#pragma unroll
    for (int r = 0; r < kFineChunk / 64; ++r) {
        const int t = my0 + r * 64 + lane;
        const bool live = my_id[r] >= 0;
        const int k = live ? my_id[r] : 0;
        unsigned long long same = __ballot(live);
#pragma unroll
        for (int bit = 0; bit < 8; ++bit) {
            const unsigned long long b = __ballot((k >> bit) & 1);
            same &= ((k >> bit) & 1) ? b : ~b;
        }
        int row = 0;
        if (live) row = next_row[k] + __popcll(same & below);
        __builtin_amdgcn_wave_barrier();
        if (live && (same & below) == 0) next_row[k] += __popcll(same);
        __builtin_amdgcn_wave_barrier();
        if (live) {
            perm[row] = t;
            inv[t] = row;
            if (alpha) gate_perm[row] = alpha[t];
        }
    }
}

// Rows of d*2 bytes moved as 16-byte pieces.  A workgroup takes kGatherRows consecutive output rows:
// their source rows go to LDS first, then the rows' pieces are dealt to the 256 threads as one flat
// range (no lane idles whatever the row length - 96 pieces at d = 768), kGatherUnroll independent
// loads in flight per thread.
constexpr int kGatherRows = 8, kGatherUnroll = 4;
__global__ __launch_bounds__(256) void gather_rows(const uint4 *__restrict__ x, const int32_t *__restrict__ perm,
                                                   int T, int vec_per_row, uint4 *__restrict__ x_perm, int k)
{
    __shared__ int src_row[kGatherRows];
    const int row0 = blockIdx.x * kGatherRows;
    const int rows = min(kGatherRows, T - row0);
    if ((int)threadIdx.x < rows) {
        const int t = perm[row0 + threadIdx.x];
        src_row[threadIdx.x] = k == 1 ? t : t / k;            // row r belongs to token perm[r] / k
    }
    __syncthreads();
    const int n = rows * vec_per_row;                         // pieces of this workgroup
    uint4 *dst = x_perm + (size_t)row0 * vec_per_row;         // its output rows are one contiguous range
    for (int base = threadIdx.x; base < n; base += 256 * kGatherUnroll) {
        uint4 v[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u) {             // unconditional loads (past the end: the last piece again)
            const int j = min(base + u * 256, n - 1);
            const int r = j / vec_per_row, i = j - r * vec_per_row;
            v[u] = x[(size_t)src_row[r] * vec_per_row + i];
        }
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (base + u * 256 < n) dst[base + u * 256] = v[u];
    }
}

}  // namespace

int launch_sort(const int32_t *ids, int32_t T, int32_t E, int32_t *counts, int32_t *offsets,
                int32_t *block_hist, int32_t *perm, int32_t *inv, const LayerTable *tbl, TileDesc *tiles,
                int32_t max_tiles, hipStream_t st, const float *alpha, float *gate_perm)
{
    const int n_chunks = (T + kChunk - 1) / kChunk;
    LayerTable none;
    none.n = 0;
    none.tile_m = kGemmTileM;
    if (T <= kOneT) {
        const LayerTable &t = tbl ? *tbl : none;
        float *gp = alpha ? gate_perm : nullptr;
        if (T <= 8 * kChunk)
            hipLaunchKernelGGL((sort_one<8, 1>), dim3(1), dim3(512), 0, st, ids, T, E, counts, offsets, perm, inv, alpha, gp, t,
                               tiles, max_tiles);
        else
            hipLaunchKernelGGL((sort_one<16, 1>), dim3(1), dim3(1024), 0, st, ids, T, E, counts, offsets, perm, inv, alpha, gp,
                               t, tiles, max_tiles);
        return (int)hipGetLastError();
    }
    if (T <= kChunksT && (reinterpret_cast<uintptr_t>(ids) & 15u) == 0) {   // ids are read 16 bytes at a time
        hipLaunchKernelGGL(sort_chunks, dim3((T + kFineChunk - 1) / kFineChunk), dim3(256), 0, st, ids, T, E, counts, offsets, perm, inv, alpha,
                           alpha ? gate_perm : nullptr, tbl ? *tbl : none, tiles, max_tiles);
        return (int)hipGetLastError();
    }
    hipLaunchKernelGGL(sort_hist, dim3(n_chunks), dim3(64), 0, st, ids, T, E, block_hist);
    hipLaunchKernelGGL(sort_scan, dim3(1), dim3(1024), 0, st, block_hist, n_chunks, E, T, counts, offsets,
                       tbl ? *tbl : none, tiles, max_tiles);
    hipLaunchKernelGGL(sort_rank, dim3(n_chunks), dim3(64), 0, st, ids, T, E, block_hist, perm, inv, alpha,
                       alpha ? gate_perm : nullptr);
    return (int)hipGetLastError();
}

int launch_gather(const void *x, const int32_t *perm, int32_t T, int32_t d, void *x_perm, hipStream_t st,
                  const LaunchEvents *ev, int32_t k)
{
    const int vec_per_row = d / 8;
    hipExtLaunchKernelGGL(gather_rows, dim3((T + kGatherRows - 1) / kGatherRows), dim3(256), 0, st, ev ? ev->start : nullptr,
                          ev ? ev->stop : nullptr, 0, (const uint4 *)x, perm, T, vec_per_row, (uint4 *)x_perm, k);
    return (int)hipGetLastError();
}

}  // namespace sida
