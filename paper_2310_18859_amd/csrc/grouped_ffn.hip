// K-b: grouped expert FFN on bf16 MFMA (gfx950).
//
// For every expert e of a wave, with its tokens in rows [offsets[e], offsets[e+1]) of x_perm:
//     h      = relu(x_perm_e * W_in[e]^T)      (GEMM 1, [rows, d] x [F, d]^T, ReLU, bf16 out)
//     y_perm = h * W_out[e]^T                  (GEMM 2, [rows, F] x [d, F]^T, bf16 out)
// which is the expert MLP f_i of Eq. 1 (Section 2.1) invoked only for experts that have tokens
// (Section 2.3).  Expert weights are read from the pool slot named by the wave table.
//
// Operand paths.  The two operands of a tile take different routes into the matrix cores:
//  * weights go global -> registers.  A pool slot holds an expert in MFMA-fragment order (see
//    kernels.h, "slot layout"): the 32 weight rows x 16 K values one 32x32x16 MFMA takes as its
//    first operand are 1 KiB of consecutive memory, lane l's 16 bytes at offset 16*l, so a
//    wavefront fetches a fragment with one fully coalesced 16-byte-per-lane load and nothing of
//    the weights passes through LDS.  Every weight fragment is used by exactly one wavefront;
//  * token rows go global -> LDS directly (buffer_load ... lds, no register staging) through a
//    ring of NB+1 stages of BM rows x 64 K values and are read as fragments by all wavefronts.
// Both run NB K-steps ahead of the MFMAs, across tile boundaries too: the weights in NB rotating
// register buffers (a buffer is refilled right after the MFMAs that consumed it), the tokens in
// the ring.  All loads use buffer descriptors (32-bit offsets; reads past a descriptor's end
// return zeros instead of faulting) - and, deliberately, no FLAT-encoded LDS loads: with those in
// flight the compiler must wait for ALL outstanding loads at every use of a loaded register.
//
// Tiling: a workgroup of NWV = 4 wavefronts computes BM tokens x (NWV*NS*32) weight rows; wavefront w
// owns NS stripes of 32 weight rows and all BM token rows, i.e. NS x BM/32 accumulator blocks of
// 32x32 (fp32).  Two workgroups share a compute unit (8 wavefronts, two per SIMD), so that one's
// result stores and tile switch overlap the other's MFMAs.  One LDS fragment read feeds NS MFMAs.
// Launches with few tiles use workgroups of NWV = 2 wavefronts, three per compute unit.
//
// LDS token tile layout: row r of a stage is 128 bytes; its 16-byte piece c is stored at piece
// position c ^ (r & 7).  A direct-to-LDS load writes lane i's 16 bytes at offset 16*i of the
// instruction's 1 KiB window (8 rows), so lane i fetches global piece (i%8) ^ (i/8) of row i/8; the
// fragment reads (32 rows, same logical piece) then touch 8 different positions per 8 rows and are
// bank-conflict free without padding.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstddef>
#include <mutex>
#include <unordered_map>

#include "kernels.h"
#include "tile_order.h"

namespace sida {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

// Waits until at most N of this wavefront's vector memory operations are outstanding (they
// complete in issue order).  Operations the kernel issues beyond the ones a count is derived
// from only make a wait stricter, never too weak.
template <int N>
__device__ __forceinline__ void wait_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Raw buffer descriptor over [base, base + bytes).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
// 16 bytes per lane straight into LDS: lane i's piece lands at lds_dst + 16*i.
__device__ __forceinline__ void load_to_lds(__amdgpu_buffer_rsrc_t r, int voffset, int soffset, void *lds_dst)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)lds_dst, 16, voffset, soffset, 0, 0);
}
// One dword per lane into LDS: lane i's word lands at lds_dst + 4*i.
__device__ __forceinline__ void load_word_to_lds(__amdgpu_buffer_rsrc_t r, int voffset, void *lds_dst)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)lds_dst, 4, voffset, 0, 0, 0);
}
// STREAM: the non-temporal cache policy, for data that is read once (it is not kept in L2 at the
// expense of data that is read again).
template <bool STREAM>
__device__ __forceinline__ bf16x8 load_frag(__amdgpu_buffer_rsrc_t r, int voffset, int soffset)
{
    return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, voffset, soffset, STREAM ? 2 : 0));
}

// FUSE selects what the token rows are addressed through:
//   kPlain    A rows and C rows are the tile's rows row0 .. row0+rows-1 (x_perm -> h -> y_perm);
//   kGather   A is x in token order: row r of the tile is read from x[perm[row0 + r] / top_k]
//             (GEMM 1 without a separate gather pass);
//   kScatter  C is y in token order: row r of the tile is scaled by gate_perm[row0 + r] (fp32
//             product of the bf16-rounded result, one more rounding to bf16 - the arithmetic of
//             the separate combine pass) and written to y[perm[row0 + r]] (GEMM 2 without a
//             separate combine pass; top-1 routing writes every y row exactly once).
// The row maps are fetched into a small private LDS buffer per wavefront with direct loads, a
// whole tile ahead of their use, so that no register-returning load has to be waited for.
enum { kPlain = 0, kGather = 1, kScatter = 2 };

constexpr int kWaves = 4;        // wavefronts per workgroup

struct GemmArgs {
    const __bf16 *A;             // token rows [a_rows, K]
    __bf16 *C;                   // results [.., N]
    const char *pool;
    size_t expert_bytes, w_off;  // W_in at offset 0 of a slot, W_out behind it
    const TileDesc *tiles;
    int m_tiles, m_tall, gm, nw, N, K;      // gm x nw: block of the tile order (tile_order.h)
    uint32_t a_bytes;            // bytes of A
    char *sink;
    const int32_t *perm;         // fused modes: row maps, `map_len` entries
    const float *gate_perm;
    int map_len, top_k;
    bool stream_once;            // weights of experts with a single token tile take the streaming cache policy
};

// Persistent workgroups: two per compute unit, each walks its tiles t = b, b+G, ...
//
// (tile, K-step) is ONE stream of steps: the loads run NB steps ahead of the MFMAs (K/64 is a
// multiple of NB), also across
// tile boundaries (the last NB steps of a tile already fetch the next one; a workgroup's last tile
// fetches its own first steps once more, unused, so that the loop has no data-dependent branch).
// Per step a wavefront executes: one s_waitcnt, one s_barrier, its share of the token loads, and
// per 16 K values BM/32 LDS fragment reads, NS*BM/32 MFMAs and NS weight-fragment loads.
template <int BM, int NS, int NB, bool RELU, int FUSE, int NWV>
__global__ __launch_bounds__(NWV * 64, NWV == kWaves ? 2 : 3) void grouped_gemm_nt(const GemmArgs g)
{
    constexpr int BN = NWV * NS * 32;
    constexpr int TS = NB + 1;                                  // token ring stages
    constexpr int kStageBytes = BM * 128;
    constexpr int kRingBytes = TS * kStageBytes;
    constexpr int QN = BM / 8;                                  // direct loads (1 KiB = 8 rows) per stage
    constexpr int TL = QN / NWV;                                // ... per wavefront
    constexpr int MI = BM / 32;
    constexpr int KS = 4;                                       // MFMA K sub-steps per K-step of 64
    constexpr int kOutCols = NS * 32;                           // output columns of a wavefront
    constexpr int kOutPitch = kOutCols * 2 + 16;                // staging row pitch in bytes
    constexpr int LPR = kOutCols * 2 / 16;                      // lanes per output-row segment
    constexpr int RPI = 64 / LPR;                               // rows per store instruction
    constexpr int STORES = MI * (32 / RPI);                     // result stores per thread per tile
    constexpr int kStepOps = TL + KS * NS;                      // loads per thread per K-step
    constexpr int kBase = (NB - 1) * kStepOps;                  // at the start of a K-step, everything issued NB steps ago must have landed
    constexpr int kStage = NWV * 32 * kOutPitch;                // result staging, 32 rows per wavefront
    constexpr int kSide = FUSE == kPlain ? 0 : (FUSE == kGather ? 256 : 2 * BM * 4);   // row maps, per wavefront
    static_assert(QN % NWV == 0 && TL * 8 <= 64, "token loads per wavefront");
    static_assert(kBase + STORES + 4 <= 63, "vmcnt range");
    static_assert(NWV * 64 * 16 <= kGemmSinkBytes / 2, "sink size");
    static_assert(kRingBytes + kStage + NWV * kSide <= (NWV == kWaves ? 80 : 53) * 1024, "two (three) workgroups per compute unit");

    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    char *stg = lds + kRingBytes + wv * (32 * kOutPitch);
    char *side = lds + kRingBytes + kStage + wv * kSide;        // this wavefront's row maps (FUSE != kPlain)
    const int N = g.N, K = g.K;
    const int n_tiles_n = N / BN;
    const int total = g.m_tiles * n_tiles_n;
    const int G = gridDim.x, wg = blockIdx.x;
    if (wg >= total) return;
    const int n = (total - wg + G - 1) / G;                     // tiles of this workgroup
    const int nkk = K / (64 * NB);
    const int stripe_bytes = 32 * K * 2;
    // results of rows past a tile's end go to a scratch sink (every thread issues all its stores,
    // the waits count them); the two workgroups of a compute unit may share it
    __bf16 *const sink = reinterpret_cast<__bf16 *>(g.sink) + (size_t)tid * 8;

    struct Coord {
        int row0, rows, nt;
        bool once;                                              // the expert's only token tile: its weights are read once
    };
    auto locate = [&](int i, Coord *c) {                        // i-th tile of this workgroup; returns its pool slot
        int mt, nt;
        map_tile(wg + i * G, g.m_tiles, g.m_tall, n_tiles_n, g.gm, g.nw, &mt, &nt);
        // The descriptors were written by an earlier launch: read through the constant address space, a
        // scalar load.  (As a vector load its result is waited for with vmcnt(0), which also waits for
        // every prefetched tile load in flight - once per tile.)  The values are uniform, so descriptors
        // and offsets built from them stay in scalar registers.
        static_assert(sizeof(TileDesc) == 16 && offsetof(TileDesc, slot) == 0 && offsetof(TileDesc, row0) == 4 &&
                      offsetof(TileDesc, rows) == 8, "a tile descriptor is read as four ints");
        typedef const __attribute__((address_space(4))) i32x4 *ConstTiles;
        const i32x4 td = ((ConstTiles)(uintptr_t)g.tiles)[mt];  // slot, row0, rows, expert
        *c = Coord{td.y, td.z, nt, g.stream_once && mt >= g.m_tall};
        return td.x;
    };

    // ---- load side.  Direct load q of a stage fills token rows 8q .. 8q+7 (1 KiB): lane l covers
    // row l/8 of that window and stores at piece position l%8, so it fetches logical piece
    // (l%8) ^ (row & 7).  Wavefront w issues loads w*TL .. w*TL+TL-1 of every stage, i.e. token
    // rows 8*TL*w .. 8*TL*(w+1)-1, and the NS*4 fragments of its own weight stripes.
    const int sub_row = lane >> 3;
    const int piece = (lane & 7) ^ sub_row;
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(g.A, g.a_bytes);
    const __amdgpu_buffer_rsrc_t map_rsrc = make_rsrc(g.perm, FUSE == kPlain ? 0u : (uint32_t)g.map_len * 4u);
    const __amdgpu_buffer_rsrc_t gate_rsrc = make_rsrc(g.gate_perm, FUSE == kScatter ? (uint32_t)g.map_len * 4u : 0u);
    __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(g.pool, 0);
    int tok_v[TL], w_v[NS];                                     // per-lane byte offsets
    int tok_s = 0, w_s = 0;                                     // running K offsets (uniform)
    bool w_once = false;                                        // cache policy of the weight loads (uniform)
    // kGather: perm of this wavefront's 8*TL token rows of a tile (rows past its end repeat the last one) -> side
    auto fetch_rows_in = [&](const Coord &c) {
        load_word_to_lds(map_rsrc, (c.row0 + min(wv * TL * 8 + (lane & (TL * 8 - 1)), c.rows - 1)) * 4, side);
    };
    auto point = [&](const Coord &c, int slot) {
#pragma unroll
        for (int j = 0; j < TL; ++j) {
            const int r = (wv * TL + j) * 8 + sub_row;          // row in the tile
            const int ra = min(r, c.rows - 1);                  // rows past the end re-read the last one
            int src = c.row0 + ra;
            if (FUSE == kGather) {                              // row ra of the tile is one of token src / top_k
                src = reinterpret_cast<const int *>(side)[j * 8 + sub_row];
                if (g.top_k != 1) src /= g.top_k;
            }
            tok_v[j] = src * K * 2 + piece * 16;
        }
        w_rsrc = make_rsrc(g.pool + (size_t)slot * g.expert_bytes + g.w_off, (uint32_t)N * (uint32_t)K * 2u);
#pragma unroll
        for (int s = 0; s < NS; ++s) w_v[s] = (c.nt * (BN / 32) + wv * NS + s) * stripe_bytes + lane * 16;
        tok_s = 0;
        w_s = 0;
        w_once = c.once;
    };
    int wr_off = 0;                                             // ring offset of the stage filled next
    auto issue_tokens = [&]() {
#pragma unroll
        for (int j = 0; j < TL; ++j) load_to_lds(a_rsrc, tok_v[j], tok_s, lds + wr_off + (wv * TL + j) * 1024);
        tok_s += 128;
        wr_off = wr_off + kStageBytes == kRingBytes ? 0 : wr_off + kStageBytes;
    };
    bf16x8 w[NB][KS][NS];                                       // weight fragments of NB K-steps
    // The weight fragments of one K-step into buffer b.  Weights of an expert with one token tile are
    // read by this tile's workgroups only: streamed past L2's replacement, they leave the token tiles
    // and the many-token experts' weights in place.  (A uniform branch around two equal sets of loads.)
    auto issue_weights = [&](bf16x8 (&wb)[KS][NS]) {
        if (w_once) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int s = 0; s < NS; ++s) wb[ks][s] = load_frag<true>(w_rsrc, w_v[s], w_s + ks * 1024);
        } else {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int s = 0; s < NS; ++s) wb[ks][s] = load_frag<false>(w_rsrc, w_v[s], w_s + ks * 1024);
        }
        w_s += 4096;
    };

    // ---- compute side
    const int frag_row = lane & 31, half = lane >> 5;
    int x_at[KS];                                               // fragment offsets inside a stage
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) x_at[ks] = frag_row * 128 + (((ks * 2 + half) ^ (frag_row & 7)) * 16);
    f32x16 acc[NS][MI];
    auto clear = [&]() {
#pragma unroll
        for (int i = 0; i < NS; ++i)
#pragma unroll
            for (int j = 0; j < MI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    };
    int rd_off = 0;                                             // ring offset of the stage multiplied next

    // Result stores.  A lane holds D[n][m] with m = lane&31 and n = 8*(r/4) + 4*(lane>>5) + r%4, i.e.
    // 8-byte runs of 32 different token rows.  Each wavefront turns its 32-row blocks around through
    // its private staging area and then stores 16 bytes per lane, consecutive lanes covering whole
    // output-row segments (LDS operations of one wavefront execute in order: no barrier between
    // its writes and reads).
    // kScatter: perm and gate_perm of the tile's BM rows -> side[0 .. BM), side[BM .. 2 BM)
    auto fetch_rows_out = [&](const Coord &c) {
#pragma unroll
        for (int i = 0; i < BM / 64; ++i) {
            const int r = (c.row0 + min(i * 64 + lane, c.rows - 1)) * 4;
            load_word_to_lds(map_rsrc, r, side + i * 256);
            load_word_to_lds(gate_rsrc, r, side + BM * 4 + i * 256);
        }
    };
    auto store_tile = [&](const Coord &c) {
        const int seg = lane % LPR, srow = lane / LPR;
#pragma unroll
        for (int im = 0; im < MI; ++im) {
            float gate = 1.f;
            if (FUSE == kScatter) gate = reinterpret_cast<const float *>(side + BM * 4)[im * 32 + frag_row];
#pragma unroll
            for (int in = 0; in < NS; ++in)
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
#pragma unroll
            for (int i = 0; i < 32 / RPI; ++i) {
                const int r = i * RPI + srow;
                const int m = im * 32 + r;
                const bf16x8 v = *reinterpret_cast<const bf16x8 *>(stg + r * kOutPitch + seg * 16);
                const int out_row = FUSE == kScatter ? reinterpret_cast<const int *>(side)[m] : c.row0 + m;
                __bf16 *dst = m < c.rows ? g.C + (size_t)out_row * N + (size_t)c.nt * BN + wv * kOutCols + seg * 8 : sink;
                *reinterpret_cast<bf16x8 *>(dst) = v;
            }
        }
    };

    Coord cc, nc;
    int slot = locate(0, &cc);
    nc = cc;
    if (FUSE == kGather) {                                      // the first tile's row map is needed at once
        fetch_rows_in(cc);
        wait_loads<0>();
    }
    point(cc, slot);
#pragma unroll
    for (int b = 0; b < NB; ++b) {                              // K-steps 0 .. NB-1 of the first tile
        issue_tokens();
        issue_weights(w[b]);
    }
    clear();

    for (int t = 0; t < n; ++t) {
        int next_slot = slot;
        if (t + 1 < n) next_slot = locate(t + 1, &nc);          // used from the last NB steps of this tile on
        // row maps: of the next tile's token rows (read by point() below), or of this tile's result
        // rows (read by store_tile()); the previous reads of the buffer are behind this wavefront
        if (FUSE == kGather) fetch_rows_in(nc);
        if (FUSE == kScatter) fetch_rows_out(cc);
        const int live = (cc.rows + 31) >> 5;                   // 32-row blocks of this tile that hold tokens
#pragma clang loop unroll(disable)
        for (int kk = 0; kk < nkk; ++kk) {
            if (kk == nkk - 1) {                                // all loads of this tile have been issued
                if (FUSE == kGather && nkk == 1) wait_loads<0>();   // else a wait of an earlier step covered the row map
                point(nc, next_slot);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                // result stores of the previous tile may still be outstanding during a tile's first steps
                if (t > 0 && kk == 0) wait_loads<kBase + STORES>();
                else wait_loads<kBase>();
                __builtin_amdgcn_s_barrier();                   // everyone's token rows of this step are in LDS, and
                                                                // everyone is done reading the stage refilled next
                issue_tokens();
                const char *st = lds + rd_off;
                // 32-row blocks of tokens past the tile's end are neither read nor multiplied
#pragma unroll
                for (int im = 0; im < MI; ++im)
                    if (im == 0 || im < live) {
                        bf16x8 xf[KS];
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) xf[ks] = *reinterpret_cast<const bf16x8 *>(st + im * 4096 + x_at[ks]);
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                            for (int s = 0; s < NS; ++s)
                                acc[s][im] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[b][ks][s], xf[ks], acc[s][im], 0, 0, 0);
                    }
                issue_weights(w[b]);
                rd_off = rd_off + kStageBytes == kRingBytes ? 0 : rd_off + kStageBytes;
            }
        }
        if (FUSE == kScatter && nkk == 1) wait_loads<0>();      // as above, for this tile's row maps
        store_tile(cc);
        clear();
        cc = nc;
        slot = next_slot;
    }
    wait_loads<0>();                                            // the last prefetches still write LDS
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

// One GEMM of the pair as one launch: BM token rows per tile, 4*NS*32 weight rows, NB K-steps ahead.
template <int BM, int NS, int NB, bool RELU, int FUSE, int NWV = kWaves>
int launch_as(const GemmArgs &a, hipStream_t st, const LaunchEvents *ev)
{
    constexpr int kLdsBytes = (NB + 1) * BM * 128 + NWV * 32 * (NS * 64 + 16) +
                              NWV * (FUSE == kPlain ? 0 : (FUSE == kGather ? 256 : 2 * BM * 4));
    static bool attr_set = false;                            // per kernel instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&grouped_gemm_nt<BM, NS, NB, RELU, FUSE, NWV>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    GemmArgs g = a;
    // Weights that only one token tile reads are streamed past L2's replacement - when there are
    // more of them than stay in the 256 MB Infinity Cache from one pass to the next anyway
    // (measured: a 128-token batch over 52 experts, second GEMM 47 -> 43.5 us; 8 experts that are
    // read again and again, 12 -> 14 us).
    g.stream_once = (int64_t)(a.m_tiles - a.m_tall) * a.N * a.K * 2 > (int64_t)128 << 20;
    const int n_tiles_n = a.N / (NWV * NS * 32);
    g.gm = tile_group_height(a.m_tiles, a.m_tall, a.K > a.N);
    g.nw = tile_block_width(n_tiles_n, g.gm);
    const int total = a.m_tiles * n_tiles_n;
    const int cap = (NWV == kWaves ? 2 : 3) * persistent_grid(st);   // workgroups per compute unit
    const int grid = total < cap ? (total + 7) / 8 * 8 : cap;   // multiple of 8 XCDs
    hipExtLaunchKernelGGL((grouped_gemm_nt<BM, NS, NB, RELU, FUSE, NWV>), dim3(grid), dim3(NWV * 64), kLdsBytes, st,
                          ev ? ev->start : nullptr, ev ? ev->stop : nullptr, 0, g);
    return (int)hipGetLastError();
}

// Tile shape of a launch.  BM = 64 or 128 token rows as the layer's descriptors say.  Weight rows per
// tile: 256 (two stripes per wavefront, one LDS fragment read per two MFMAs) when the matrix has a
// multiple of 256 rows - every Switch shape has - unless 128-row tiles, twice as many at a little
// more than half the time each (fitted: 5/8), need fewer rounds over the persistent grid's
// workgroup slots: tiles are dealt to the workgroups in turn, so a launch takes as long as its
// workgroup with the most tiles.  A launch that leaves
// workgroup slots idle streams every tile's weights through few registers per compute unit, so
// narrow 64-row tiles also fetch four K-steps ahead instead of two where the K loop allows it (with
// 128-row tiles a five-stage token ring would not leave room for two workgroups per compute unit,
// and the loads of a wavefront complete in order, so the ring has to be as deep as the weights).
template <int BM, bool RELU, int FUSE>
int launch_width(const GemmArgs &a, hipStream_t st, const LaunchEvents *ev)
{
    const int64_t slots = 2 * (int64_t)persistent_grid(st);
    const int64_t t_wide = (int64_t)a.m_tiles * (a.N / 256);
    bool wide = a.N % 256 == 0 && (t_wide + slots - 1) / slots * 8 <= (2 * t_wide + slots - 1) / slots * 5;
    // Wide tiles for at most three quarters of the workgroup slots, over mostly single-tile experts:
    // the launch is a stream of weights, and twice as many narrower tiles keep more of it in flight
    // (64 experts, 8192 tokens, second GEMM: 95 -> 87 us; 128 experts, 512 tokens: 92 -> 81 us; with
    // wide tiles for 0.8 of the slots the narrow ones are 6 % slower, and many-token experts prefer
    // the wide tile at any count).
    if (wide && 4 * t_wide <= 3 * slots && 2 * a.m_tall <= a.m_tiles) wide = false;
    if (wide) return launch_as<BM, 2, 2, RELU, FUSE>(a, st, ev);
    if constexpr (BM == kGemmTileSmall) {
        // 128-wide tiles for at most three quarters of the workgroup slots, and few tokens per tile:
        // workgroups of two wavefronts (64 weight rows), three per compute unit, put twice as many
        // weight streams in flight.  (A 128-token batch's second GEMM, 312 tiles: 53 -> 47 us.  With
        // tiles for 0.8 of the slots and more, or with full token tiles, fetching the token rows twice
        // as often costs more than the streams gain.)
        const int64_t rows = a.a_bytes / (2 * (int64_t)a.K);
        if (4 * (int64_t)a.m_tiles * (a.N / 128) <= 3 * slots && rows <= 32 * (int64_t)a.m_tiles) {
            if (a.K % 256 == 0) return launch_as<BM, 1, 4, RELU, FUSE, 2>(a, st, ev);
            return launch_as<BM, 1, 2, RELU, FUSE, 2>(a, st, ev);
        }
        if (a.K % 256 == 0) return launch_as<BM, 1, 4, RELU, FUSE>(a, st, ev);
    }
    return launch_as<BM, 1, 2, RELU, FUSE>(a, st, ev);
}

template <bool RELU, int FUSE>
int launch_shape(const GemmArgs &a, int tile_m, hipStream_t st, const LaunchEvents *ev)
{
    if (a.m_tiles <= 0) {                                    // nothing to launch: keep the events usable
        if (ev) {
            (void)hipEventRecord(ev->start, st);
            (void)hipEventRecord(ev->stop, st);
        }
        return 0;
    }
    if (tile_m == kGemmTileSmall) return launch_width<kGemmTileSmall, RELU, FUSE>(a, st, ev);
    return launch_width<kGemmTileM, RELU, FUSE>(a, st, ev);
}

}  // namespace

void forget_stream(hipStream_t st)
{
    std::lock_guard<std::mutex> lk(g_cu_mu);
    g_cu_cache.erase(st);
}

int launch_ffn_gemm1(const void *x_perm, void *h, const char *pool, size_t expert_bytes, const TileDesc *tiles,
                     int32_t m_tiles, int32_t m_tall, int32_t d, int32_t F, void *sink, hipStream_t st,
                     const LaunchEvents *ev, int32_t a_rows, const int32_t *perm, int32_t map_len, int32_t top_k,
                     int32_t tile_m)
{
    GemmArgs a{};
    a.A = (const __bf16 *)x_perm;
    a.C = (__bf16 *)h;
    a.pool = pool;
    a.expert_bytes = expert_bytes;
    a.w_off = 0;
    a.tiles = tiles;
    a.m_tiles = m_tiles;
    a.m_tall = m_tall;
    a.N = F;
    a.K = d;
    a.a_bytes = (uint32_t)((size_t)a_rows * d * 2);
    a.sink = (char *)sink;
    a.perm = perm;
    a.map_len = map_len;
    a.top_k = top_k;
    return perm ? launch_shape<true, kGather>(a, tile_m, st, ev) : launch_shape<true, kPlain>(a, tile_m, st, ev);
}

int launch_ffn_gemm2(const void *h, void *y_perm, const char *pool, size_t expert_bytes, const TileDesc *tiles,
                     int32_t m_tiles, int32_t m_tall, int32_t d, int32_t F, void *sink, hipStream_t st,
                     const LaunchEvents *ev, int32_t a_rows, const int32_t *perm, const float *gate_perm, int32_t tile_m)
{
    GemmArgs a{};
    a.A = (const __bf16 *)h;
    a.C = (__bf16 *)y_perm;
    a.pool = pool;
    a.expert_bytes = expert_bytes;
    a.w_off = (size_t)F * (size_t)d * 2;                     // W_out follows W_in in a slot
    a.tiles = tiles;
    a.m_tiles = m_tiles;
    a.m_tall = m_tall;
    a.N = d;
    a.K = F;
    a.a_bytes = (uint32_t)((size_t)a_rows * F * 2);
    a.sink = (char *)sink + kGemmSinkBytes / 2;              // GEMM 1 and GEMM 2 of concurrent streams do not share
    a.perm = perm;
    a.gate_perm = gate_perm;
    a.map_len = a_rows;
    a.top_k = 1;                                             // scattering is only defined for one expert per token
    return perm ? launch_shape<false, kScatter>(a, tile_m, st, ev) : launch_shape<false, kPlain>(a, tile_m, st, ev);
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
