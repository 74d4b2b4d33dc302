// K-b: grouped expert FFN on bf16 MFMA (gfx950).
//
// For every expert e of a wave, with its tokens in rows [offsets[e], offsets[e+1]) of x_perm:
//     h      = relu(x_perm_e * W_in[e]^T)      (GEMM 1, [rows, d] x [F, d]^T, ReLU, bf16 out)
//     y_perm = h * W_out[e]^T                  (GEMM 2, [rows, F] x [d, F]^T, bf16 out)
// which is the expert MLP f_i of Eq. 1 (Section 2.1) invoked only for experts that have tokens
// (Section 2.3).  Expert weights are read from the pool slot named by the wave table.
//
// Both GEMMs are "NT": activations [M,K] and weights [N,K] are K-contiguous, so every MFMA
// operand fragment (8 consecutive K values of one row) is one 16-byte access.
//
// The layer is bound by streaming each activated expert's weights from HBM once, so the kernel
// is built to keep many bytes in flight per compute unit: tiles go global -> LDS directly
// (global_load_lds, no register staging) through a ring of STAGES buffers, STAGES-1 K-steps
// ahead of the MFMAs, with one workgroup barrier per K-step.
//
// Tiling: one workgroup of WM x WN wavefronts computes a BM (tokens) x BN (weight rows) tile, K in
// steps of BK; each wavefront owns (BM/WM) x (BN/WN) as MFMA 32x32x16 tiles, fp32 accumulators.
// Eight wavefronts per compute unit are needed to pull enough bytes per clock out of L2 with
// direct-to-LDS loads (four reach about half of that).  The weight rows are the MFMA's first
// operand and the token rows the second, so a lane ends up with 4 consecutive output columns of
// one token row; finished tiles are turned around through LDS so that the global stores are
// 16 bytes per lane and consecutive lanes cover whole row segments.
//
// LDS tile layout (BK = 64): row r of a tile is 128 bytes; its 16-byte piece c is stored at piece
// position c ^ (r & 7).  A direct-to-LDS load writes lane i's 16 bytes at offset 16*i of the
// instruction's 1 KB window (8 rows), so lane i fetches global piece (i%8) ^ (i/8) of row i/8;
// the MFMA fragment reads (32 rows, same logical piece) then touch 8 different positions per
// 8 rows and are bank-conflict free without padding.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <mutex>
#include <unordered_map>

#include "kernels.h"
#include "tile_order.h"

namespace sida {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;


template <int N>
__device__ __forceinline__ void wait_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void load_to_lds(const void *gsrc, void *lds_dst)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gsrc,
                                     (__attribute__((address_space(3))) void *)lds_dst, 16, 0, 0);
}

// One dword per lane: lane i's word lands at offset 4*i of the 256-byte window at lds_dst.
__device__ __forceinline__ void load_word_to_lds(const void *gsrc, void *lds_dst)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gsrc,
                                     (__attribute__((address_space(3))) void *)lds_dst, 4, 0, 0);
}

// Persistent workgroups: one per compute unit, each walks its tiles t = b, b+G, ...
//
// (tile, K-step) is ONE stream of stages: the loads run STAGES-1 stages ahead of the MFMAs, also
// across tile boundaries.  The K loop of a tile is cut in two: while its first nk-(STAGES-1) steps
// are multiplied the loads still fetch this tile, during the last STAGES-1 steps they already
// fetch the next one.  Per step a wavefront executes: one s_waitcnt, one s_barrier, LOADS direct
// loads with running pointers, the LDS fragment reads and the MFMAs - no tile bookkeeping.
//
// BM x BN is the output tile (tokens x weight rows), WM x WN the wavefront grid (8 wavefronts).
//
// FUSE selects what the token rows are addressed through:
//   kPlain    A rows and C rows are the tile's rows row0 .. row0+rows-1 (x_perm -> h -> y_perm);
//   kGather   A is x in token order: row r of the tile is read from x[perm[row0 + r]] (GEMM 1
//             without a separate gather pass);
//   kScatter  C is y in token order: row r of the tile is scaled by gate_perm[row0 + r] (fp32
//             product of the bf16-rounded result, one more rounding to bf16 - the arithmetic of
//             the separate combine pass) and written to y[perm[row0 + r]] (GEMM 2 without a
//             separate combine pass; top-1 routing writes every y row exactly once).
// The row maps are fetched into a small private LDS buffer per wavefront with the same direct
// loads as the tiles (no register-returning vector loads, which would make every use wait for
// all older tile loads): kExtra more operations per tile in the wait counts.
enum { kPlain = 0, kGather = 1, kScatter = 2 };

template <int BM, int BN, int BK, int WM, int WN, int STAGES, bool RELU, int FUSE>
__global__ __launch_bounds__(WM * WN * 64) void grouped_gemm_nt(const __bf16 *__restrict__ A, __bf16 *__restrict__ C,
                                                               const char *__restrict__ pool, size_t expert_bytes,
                                                               size_t w_off, const TileDesc *__restrict__ tiles,
                                                               int m_tiles, int m_tall, int nw, int N, int K,
                                                               char *__restrict__ sink,
                                                               const int32_t *__restrict__ perm,
                                                               const float *__restrict__ gate_perm, int top_k)
{
    constexpr int NW = WM * WN;
    constexpr int kRowBytes = BK * 2;                         // a tile row in LDS: BK bf16 (128 or 64 bytes)
    constexpr int PPR = kRowBytes / 16;                       // 16-byte pieces per row
    constexpr int RPL = 64 / PPR;                             // rows filled by one direct load (1 KiB)
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    constexpr int kRingBytes = STAGES * kStageBytes;
    constexpr int LOADS = (BM + BN) / (RPL * NW);             // direct loads per thread per K-step
    constexpr int kSideBytes = FUSE == kPlain ? 0 : 512;      // per wavefront: row maps of a tile
    constexpr int kExtra = FUSE == kPlain ? 0 : 2;            // direct loads per thread per tile for them
    static_assert(FUSE == kPlain || ((BM == 128 || BM == 64) && WM == 2), "row maps are laid out for tiles of up to 128 rows, two wavefront rows");
    static_assert(BK == 64 || BK == 32, "K step");
    constexpr int MI = BM / (32 * WM);                        // 32-row MFMA blocks per wavefront along tokens
    constexpr int NI = BN / (32 * WN);                        //   ... along weight rows
    constexpr int KS = BK / 16;                               // MFMA K sub-steps per stage
    constexpr int STORES = MI * NI * 2;                       // result stores per thread per tile (16 bytes each)
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && (BM + BN) % (RPL * NW) == 0 && BM % RPL == 0, "tile");
    static_assert(STAGES >= 2 && (STAGES - 2) * LOADS + STORES + kExtra <= 63, "vmcnt range");
    static_assert(NW * 64 * 16 <= kGemmSinkBytes, "sink size");

    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_tiles_n = N / BN;
    const int total = m_tiles * n_tiles_n;
    const int G = gridDim.x;
    if ((int)blockIdx.x >= total) return;
    const int n = (total - (int)blockIdx.x + G - 1) / G;      // tiles of this workgroup
    const int nk = K / BK;                                    // the launcher guarantees nk >= STAGES - 1

    // ---- load side.  A stage is BM token rows followed by BN weight rows; direct load number i of
    // a stage fills rows RPL*i .. RPL*i+RPL-1 (1 KiB): lane l covers row l/PPR of that window and
    // stores at piece position l%PPR.  Swizzle: piece c of row r is stored at position c ^ (r & 7)
    // for 128-byte rows and at c ^ ((r >> 2) & 3) for 64-byte rows; both make the 32-row fragment
    // reads conflict free.  Wavefront w issues loads w*LOADS .. w*LOADS+LOADS-1 of every stage.
    const int sub_row = lane / PPR;
    const int piece = (lane % PPR) ^ (BK == 64 ? sub_row : (sub_row >> 2) & 3);   // logical piece this lane fetches
    struct Coord {
        int row0, rows, nt;
    };
    auto locate = [&](int i, Coord *c) {                      // i-th tile of this workgroup; returns its pool slot
        int mt, nt;
        map_tile((int)blockIdx.x + i * G, m_tiles, m_tall, n_tiles_n, nw, &mt, &nt);
        const TileDesc td = tiles[mt];                        // uniform address: a scalar load
        *c = Coord{td.row0, td.rows, nt};
        return td.slot;
    };
    char *side = lds + kRingBytes + wv * kSideBytes;          // this wavefront's row maps (FUSE != kPlain)
    // kGather: perm[row0 .. row0+127] of a tile (rows past its end repeat the last one) -> side[0..127]
    auto fetch_rows_in = [&](const Coord &c) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            load_word_to_lds(perm + c.row0 + min(i * 64 + lane, c.rows - 1), side + i * 256);
    };
    auto point = [&](const Coord &c, int slot, const char *(&p)[LOADS]) {
        const char *Wt = pool + (size_t)slot * expert_bytes + w_off + (size_t)c.nt * BN * K * 2;
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int r = (wv * LOADS + j) * RPL + sub_row;   // row in the stage
            const int ra = min(r, c.rows - 1);                // rows past the end re-read the last one
            int src = c.row0 + ra;
            if (FUSE == kGather) {                            // row ra of the tile is one of token src / top_k
                src = reinterpret_cast<const int *>(side)[ra];
                if (top_k != 1) src /= top_k;
            }
            p[j] = r < BM ? reinterpret_cast<const char *>(A) + (size_t)src * K * 2 + piece * 16
                          : Wt + (size_t)(r - BM) * K * 2 + piece * 16;
        }
    };
    int wr_off = 0;                                           // ring offset of the stage filled next
    auto issue = [&](const char *(&p)[LOADS]) {               // next K-step of the tile p points into
        char *dst = lds + wr_off + wv * LOADS * 1024;
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            load_to_lds(p[j], dst + j * 1024);
            p[j] += kRowBytes;
        }
        wr_off = wr_off + kStageBytes == kRingBytes ? 0 : wr_off + kStageBytes;
    };

    // ---- compute side ----
    const int wm = wv % WM, wn = wv / WM;                     // wavefront position in the WM x WN grid
    const int frag_row = lane & 31, half = lane >> 5;
    const int sw = BK == 64 ? (frag_row & 7) : ((frag_row >> 2) & 3);
    int x_at[MI][KS], w_at[NI][KS];                           // fragment offsets inside a stage
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int pos = ((ks * 2 + half) ^ sw) * 16;
#pragma unroll
        for (int i = 0; i < MI; ++i) x_at[i][ks] = (wm * (BM / WM) + i * 32 + frag_row) * kRowBytes + pos;
#pragma unroll
        for (int i = 0; i < NI; ++i) w_at[i][ks] = BM * kRowBytes + (wn * (BN / WN) + i * 32 + frag_row) * kRowBytes + pos;
    }
    f32x16 acc[NI][MI];
    auto clear = [&]() {
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < MI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    };
    int rd_off = 0;                                           // ring offset of the stage multiplied next
    auto multiply_stage = [&]() {
        const char *st = lds + rd_off;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 xf[MI], wf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) xf[i] = *reinterpret_cast<const bf16x8 *>(st + x_at[i][ks]);
#pragma unroll
            for (int i = 0; i < NI; ++i) wf[i] = *reinterpret_cast<const bf16x8 *>(st + w_at[i][ks]);
#pragma unroll
            for (int in = 0; in < NI; ++in)
#pragma unroll
                for (int im = 0; im < MI; ++im)
                    acc[in][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[in], xf[im], acc[in][im], 0, 0, 0);
        }
        rd_off = rd_off + kStageBytes == kRingBytes ? 0 : rd_off + kStageBytes;
    };
    // Result stores.  A lane holds D[n][m] with m = lane&31 and n = 8*(r/4) + 4*(lane>>5) + r%4, i.e.
    // 8-byte runs of 32 different token rows.  Each wavefront turns its 32-row blocks around through
    // a private piece of the stage that was multiplied last (free until the next K-step refills it)
    // and then stores 16 bytes per lane, consecutive lanes covering whole output-row segments.
    // Every thread issues all its stores (the waits count them): rows past the end of the tile go
    // to a scratch sink instead of C.
    constexpr int kOutCols = NI * 32;                         // output columns of a wavefront
    constexpr int kOutPitch = kOutCols * 2 + 16;              // staging row pitch in bytes
    constexpr int LPR = kOutCols * 2 / 16;                    // lanes per output-row segment
    constexpr int RPI = 64 / LPR;                             // rows per store instruction
    static_assert(STORES == MI * (32 / RPI), "store count");
    static_assert(NW * 32 * kOutPitch <= kStageBytes, "staging fits in a stage");
    // kScatter: this wavefront's BM/WM rows of the tile: perm -> side[0..63], gate_perm -> side[64..127]
    auto fetch_rows_out = [&](const Coord &c) {
        const int r = c.row0 + min(wm * (BM / WM) + lane, c.rows - 1);
        load_word_to_lds(perm + r, side);
        load_word_to_lds(gate_perm + r, side + 256);
    };
    auto store_tile = [&](const Coord &c) {
        __builtin_amdgcn_s_barrier();                         // everyone is done reading the last stage
        char *stg = lds + (rd_off == 0 ? kRingBytes - kStageBytes : rd_off - kStageBytes) + wv * (32 * kOutPitch);
        const int seg = lane % LPR, srow = lane / LPR;
#pragma unroll
        for (int im = 0; im < MI; ++im) {
            float gate = 1.f;
            if (FUSE == kScatter) gate = reinterpret_cast<const float *>(side + 256)[im * 32 + frag_row];
#pragma unroll
            for (int in = 0; in < NI; ++in)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float v = acc[in][im][q * 4 + j];
                        if (RELU) v = v > 0.f ? v : 0.f;
                        o[j] = (__bf16)v;
                        if (FUSE == kScatter) o[j] = (__bf16)(gate * (float)o[j]);
                    }
                    *reinterpret_cast<bf16x4 *>(stg + frag_row * kOutPitch + (in * 32 + q * 8 + half * 4) * 2) = o;
                }
            // LDS operations of one wavefront execute in order: no barrier between its writes and reads
#pragma unroll
            for (int i = 0; i < 32 / RPI; ++i) {
                const int r = i * RPI + srow;
                const int m = wm * (BM / WM) + im * 32 + r;
                const bf16x8 v = *reinterpret_cast<const bf16x8 *>(stg + r * kOutPitch + seg * 16);
                const int out_row = FUSE == kScatter ? reinterpret_cast<const int *>(side)[im * 32 + r] : c.row0 + m;
                __bf16 *dst = m < c.rows ? C + (size_t)out_row * N + (size_t)c.nt * BN + wn * (BN / WN) + seg * 8
                                         : reinterpret_cast<__bf16 *>(sink) + (size_t)tid * 8;
                *reinterpret_cast<bf16x8 *>(dst) = v;
            }
        }
    };

    const char *cur[LOADS];                                   // running load pointers
    Coord cc, nc;
    int slot = locate(0, &cc);
    nc = cc;
    if (FUSE == kGather) {                                    // the first tile's row map is needed at once
        fetch_rows_in(cc);
        wait_loads<0>();
    }
    point(cc, slot, cur);
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) issue(cur);          // K-steps 0 .. STAGES-2 of the first tile
    clear();

    for (int t = 0; t < n; ++t) {
        const bool has_next = t + 1 < n;
        int next_slot = 0;
        if (has_next) next_slot = locate(t + 1, &nc);         // used only after the first part of the K loop
        // row maps: of the next tile's token rows (read by point() below), or of this tile's result
        // rows (read by store_tile()); issued by every thread on every tile so that the waits can
        // count them.  The previous reads of the buffer are behind this wavefront.
        if (FUSE == kGather) fetch_rows_in(nc);
        if (FUSE == kScatter) fetch_rows_out(cc);
        // ---- K-steps whose loads still belong to this tile.  For the first STAGES-1 steps after a
        // tile's result stores those may be outstanding too (vector memory operations of a
        // wavefront complete in issue order, stores included).
        for (int k = 0; k <= nk - STAGES; ++k) {
            if (t > 0 && k < STAGES - 1) wait_loads<(STAGES - 2) * LOADS + STORES + kExtra>();
            else wait_loads<(STAGES - 2) * LOADS>();
            __builtin_amdgcn_s_barrier();                     // everyone's pieces of this stage are in LDS, and
                                                              // everyone is done reading the stage refilled next
            issue(cur);
            multiply_stage();
        }
        // ---- last STAGES-1 K-steps: the loads already fetch the next tile
        if (has_next) {
            // the row map of the next tile is in LDS once a wait of step STAGES-1 or later has passed
            if (FUSE == kGather && nk < 2 * STAGES - 1) wait_loads<0>();
            point(nc, next_slot, cur);                        // all loads of this tile have been issued
#pragma unroll
            for (int k = 0; k < STAGES - 1; ++k) {
                if (t > 0 && nk - (STAGES - 1) + k < STAGES - 1) wait_loads<(STAGES - 2) * LOADS + STORES + kExtra>();
                else wait_loads<(STAGES - 2) * LOADS>();
                __builtin_amdgcn_s_barrier();
                issue(cur);
                multiply_stage();
            }
        } else {
#pragma unroll
            for (int k = 0; k < STAGES - 1; ++k) {            // the stream ends: nothing more to fetch
                wait_loads<0>();
                __builtin_amdgcn_s_barrier();
                multiply_stage();
            }
        }
        if (FUSE == kScatter && has_next && nk < STAGES) wait_loads<0>();   // as above, for this tile's row maps
        store_tile(cc);
        clear();
        cc = nc;
    }
}

// Compute units the stream's kernels may run on (streams can be created with a compute-unit mask,
// see sida_streams_create), rounded down to a multiple of the 8 XCDs; cached per stream.
std::mutex g_cu_mu;
std::unordered_map<hipStream_t, int> g_cu_cache;

int persistent_grid(hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_cu_mu);
    auto &cache = g_cu_cache;
    auto it = cache.find(st);
    if (it != cache.end()) return it->second;
    int dev = 0, total = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        total = prop.multiProcessorCount;
    int cus = total;
    uint32_t mask[16] = {};
    if (hipExtStreamGetCUMask(st, 16, mask) == hipSuccess) {
        int bits = 0;
        for (int i = 0; i < 16; ++i) bits += __builtin_popcount(mask[i]);
        if (bits > 0 && bits < total) cus = bits;
    } else {
        (void)hipGetLastError();
    }
    cus = cus >= 8 ? cus / 8 * 8 : 8;
    cache[st] = cus;
    return cus;
}

// Measured on the Switch-base-128 workload: a K step of 32 with a deeper ring (more bytes in
// flight, 64-byte row segments) is slower than 64, and a fifth stage for 128 x 128 tiles changes
// nothing.
template <int BM, int BN, int BK, int WM, int WN, int STAGES, bool RELU, int FUSE>
int launch_as(const void *A, void *C, const char *pool, size_t expert_bytes, size_t w_off, const TileDesc *tiles,
              int32_t m_tiles, int32_t m_tall, int N, int K, void *sink, const int32_t *perm, const float *gate_perm,
              int top_k, hipStream_t st, const LaunchEvents *ev)
{
    constexpr int kLdsBytes = STAGES * (BM + BN) * BK * 2 + (FUSE == kPlain ? 0 : WM * WN * 512);
    static_assert(kLdsBytes <= 160 * 1024, "LDS");
    static bool attr_set = false;                            // per kernel instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&grouped_gemm_nt<BM, BN, BK, WM, WN, STAGES, RELU, FUSE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    if (m_tiles <= 0) {                                      // nothing to launch: keep the events usable
        if (ev) {
            (void)hipEventRecord(ev->start, st);
            (void)hipEventRecord(ev->stop, st);
        }
        return 0;
    }
    const int n_tiles_n = N / BN;
    const int nw = tile_block_width(n_tiles_n);
    const int total = m_tiles * n_tiles_n;
    const int cus = persistent_grid(st);
    const int grid = total < cus ? (total + 7) / 8 * 8 : cus;   // multiple of 8 XCDs
    hipExtLaunchKernelGGL((grouped_gemm_nt<BM, BN, BK, WM, WN, STAGES, RELU, FUSE>), dim3(grid), dim3(WM * WN * 64), kLdsBytes,
                          st, ev ? ev->start : nullptr, ev ? ev->stop : nullptr, 0, (const __bf16 *)A, (__bf16 *)C, pool,
                          expert_bytes, w_off, tiles, m_tiles, m_tall, nw, N, K, (char *)sink, perm, gate_perm, top_k);
    return (int)hipGetLastError();
}

// GEMM 1 gathers when a row map is given, GEMM 2 scatters.
template <int BM, int BN, int BK, int WM, int WN, int STAGES, bool RELU>
int launch(const void *A, void *C, const char *pool, size_t expert_bytes, size_t w_off, const TileDesc *tiles,
           int32_t m_tiles, int32_t m_tall, int N, int K, void *sink, const int32_t *perm, const float *gate_perm,
           int top_k, hipStream_t st, const LaunchEvents *ev)
{
    if (!perm)
        return launch_as<BM, BN, BK, WM, WN, STAGES, RELU, kPlain>(A, C, pool, expert_bytes, w_off, tiles, m_tiles, m_tall, N,
                                                                   K, sink, nullptr, nullptr, 1, st, ev);
    return launch_as<BM, BN, BK, WM, WN, STAGES, RELU, RELU ? kGather : kScatter>(A, C, pool, expert_bytes, w_off, tiles,
                                                                                  m_tiles, m_tall, N, K, sink, perm,
                                                                                  gate_perm, top_k, st, ev);
}

// Tile width of a launch: the shape whose busiest compute unit moves the fewest tile bytes through
// its LDS, rounds of tiles times rows per K-step; a tie goes to the wide tile, which re-reads the
// token rows half as often.  For GEMM 2 (K = d_ff, four times fewer and longer tiles) the wide tile
// is charged 9/8 of its rows: measured on the resident Switch shapes, 128-wide tiles are 5 % and
// 2 % faster there at 100 and 205 token tiles (model 768 : 768 and 1280 : 1152) and 10 % and 8 %
// slower at 420 and 330 (2560 : 1920, 2816 : 2304).
bool wide_tiles_pay(int32_t m_tiles, int32_t N, int32_t tile_m, bool gemm2, hipStream_t st)
{
    const int64_t cus = persistent_grid(st);
    const int64_t narrow = ((int64_t)m_tiles * (N / 128) + cus - 1) / cus * (tile_m + 128);
    const int64_t wide = ((int64_t)m_tiles * (N / 256) + cus - 1) / cus * (tile_m + 256);
    return (gemm2 ? wide * 9 : wide * 8) <= narrow * 8;
}

// One GEMM of the pair: BM = token rows per tile (64 or 128), wide or narrow tiles by the launch's
// size, ring depth by the length of the K loop (a tile's K loop needs at least STAGES-1 steps of 64).
template <int BM, bool RELU>
int launch_shape(const void *A, void *C, const char *pool, size_t expert_bytes, size_t w_off, const TileDesc *tiles,
                 int32_t m_tiles, int32_t m_tall, int N, int K, void *sink, const int32_t *perm, const float *gate_perm,
                 int top_k, hipStream_t st, const LaunchEvents *ev)
{
    // N and K are multiples of 256 for every Switch shape; other widths fall back to 128-wide tiles
    if (N % 256 == 0 && K >= 128 && wide_tiles_pay(m_tiles, N, BM, !RELU, st))
        return launch<BM, 256, 64, 2, 4, 3, RELU>(A, C, pool, expert_bytes, w_off, tiles, m_tiles, m_tall, N, K, sink, perm,
                                                  gate_perm, top_k, st, ev);
    if (K < 192)
        return launch<BM, 128, 64, 2, 4, 3, RELU>(A, C, pool, expert_bytes, w_off, tiles, m_tiles, m_tall, N, K, sink, perm,
                                                  gate_perm, top_k, st, ev);
    return launch<BM, 128, 64, 2, 4, 4, RELU>(A, C, pool, expert_bytes, w_off, tiles, m_tiles, m_tall, N, K, sink, perm,
                                              gate_perm, top_k, st, ev);
}

}  // namespace

void forget_stream(hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_cu_mu);
    g_cu_cache.erase(st);
}

int launch_ffn_gemm1(const void *x_perm, void *h, const char *pool, size_t expert_bytes, const TileDesc *tiles,
                     int32_t m_tiles, int32_t m_tall, int32_t d, int32_t F, void *sink, hipStream_t st,
                     const LaunchEvents *ev, const int32_t *perm, int32_t top_k, int32_t tile_m)
{
    if (tile_m == kGemmTileSmall)
        return launch_shape<kGemmTileSmall, true>(x_perm, h, pool, expert_bytes, 0, tiles, m_tiles, m_tall, F, d, sink, perm,
                                                  nullptr, top_k, st, ev);
    return launch_shape<kGemmTileM, true>(x_perm, h, pool, expert_bytes, 0, tiles, m_tiles, m_tall, F, d, sink, perm, nullptr,
                                          top_k, st, ev);
}

int launch_ffn_gemm2(const void *h, void *y_perm, const char *pool, size_t expert_bytes, const TileDesc *tiles,
                     int32_t m_tiles, int32_t m_tall, int32_t d, int32_t F, void *sink, hipStream_t st,
                     const LaunchEvents *ev, const int32_t *perm, const float *gate_perm, int32_t tile_m)
{
    const size_t w_out = (size_t)F * (size_t)d * 2;          // W_out follows W_in in an expert's block
    // scattering is only defined for one expert per token: top_k = 1
    if (tile_m == kGemmTileSmall)
        return launch_shape<kGemmTileSmall, false>(h, y_perm, pool, expert_bytes, w_out, tiles, m_tiles, m_tall, d, F, sink, perm,
                                                   gate_perm, 1, st, ev);
    return launch_shape<kGemmTileM, false>(h, y_perm, pool, expert_bytes, w_out, tiles, m_tiles, m_tall, d, F, sink, perm,
                                           gate_perm, 1, st, ev);
}

// ---- token-tile descriptors ----------------------------------------------------------------
namespace {

// One workgroup; thread i owns table entry i.
__global__ __launch_bounds__(256) void build_tiles(const LayerTable tbl, const int32_t *__restrict__ offsets,
                                                   TileDesc *__restrict__ tiles, int max_tiles)
{
    __shared__ int s_wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int e = 0, slot = 0, off = 0, cnt = 0, n_t = 0;
    if (tid < tbl.n) {
        e = tbl.expert[tid];
        slot = tbl.slot[tid];
        off = offsets[e];
        cnt = offsets[e + 1] - off;
        n_t = (cnt + tbl.tile_m - 1) / tbl.tile_m;
    }
    int incl = n_t;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) s_wsum[wv] = incl;
    __syncthreads();
    for (int i = 0; i < wv; ++i) incl += s_wsum[i];
    int at = incl - n_t;
    for (int k = 0; k < n_t && at < max_tiles; ++k, ++at) {
        TileDesc t;
        t.slot = slot;
        t.row0 = off + k * tbl.tile_m;
        t.rows = min(tbl.tile_m, cnt - k * tbl.tile_m);
        t.expert = e;
        tiles[at] = t;
    }
}

}  // namespace

int launch_build_tiles(const LayerTable &tbl, const int32_t *offsets, TileDesc *tiles, int32_t max_tiles,
                       hipStream_t st)
{
    hipLaunchKernelGGL(build_tiles, dim3(1), dim3(256), 0, st, tbl, offsets, tiles, max_tiles);
    return (int)hipGetLastError();
}

}  // namespace sida
