// Launchers of the HIP kernels.  Each returns the hipError_t of its launch (as int).
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace sida {

// The activated experts of one layer in the order their token tiles are scheduled: wave by wave,
// inside a wave the expert with the most tokens first (so the long experts do not end up as the
// tail of a launch).  Passed by value to the kernel that expands it into token-tile descriptors.
struct LayerTable {
    int32_t n;                 // activated experts
    int32_t tile_m;            // token rows per tile of this layer's grouped GEMMs: 64 or 128
    int16_t slot[256];         // pool slot of entry i
    uint8_t expert[256];       // expert id of entry i
};

// One token tile of the grouped GEMMs: up to tile_m (64 or 128) consecutive rows of one expert.
struct TileDesc {
    int32_t slot;              // pool slot holding the expert's weights
    int32_t row0;              // first row in x_perm / h / y_perm
    int32_t rows;              // 1..tile_m
    int32_t expert;
};

// Optional timing of a single-kernel launch: the two events are attached to the kernel's own
// dispatch, so their elapsed time is the kernel's execution time without the gaps a pair of
// hipEventRecord calls around the launch would add.  NULL = not timed.
struct LaunchEvents {
    hipEvent_t start, stop;
};

// K-a: stable counting sort of T tokens by expert id.
//   ids int32[T] -> counts[E], offsets[E+1], perm[T], inv[T];  block_hist is scratch [n_chunks*E].
// When tbl is given (may be NULL) it is also expanded into token tiles, see launch_build_tiles.
// With alpha (may be NULL) the gate values are moved along: gate_perm[r] = alpha[perm[r]].
int launch_sort(const int32_t *ids, int32_t T, int32_t E, int32_t *counts, int32_t *offsets,
                int32_t *block_hist, int32_t *perm, int32_t *inv, const LayerTable *tbl, TileDesc *tiles,
                int32_t max_tiles, hipStream_t st, const float *alpha = nullptr, float *gate_perm = nullptr);
// K-a: x_perm[r,:] = x[perm[r] / k,:], rows of d bf16 values; T = rows of x_perm (k per token).
int launch_gather(const void *x, const int32_t *perm, int32_t T, int32_t d, void *x_perm, hipStream_t st,
                  const LaunchEvents *ev = nullptr, int32_t k = 1);
// K-b: h = relu(x_perm W_in^T) then y_perm = h W_out^T for the experts in tbl.
// tiles[0 .. m_tiles) are the token tiles of the experts to compute (see launch_build_tiles); the
// first m_tall of them belong to experts with more than one tile; tile_m = rows per tile (64 when
// most experts of the layer have at most 64 tokens, 128 otherwise).
// sink: kGemmSinkBytes of device scratch that absorbs the stores of rows past a tile's end.
// With a row map (perm, and for GEMM 2 gate_perm) the gather / combine passes are folded in:
// GEMM 1 then reads row r from x[perm[r] / k] (x_perm = x in token order, k rows per token), GEMM 2 writes
// bf16(gate_perm[r] * result row r) to y[perm[r]] (y_perm = y in token order).
// a_rows: rows of the token operand (x_perm / h, or x when gathering), map_len: entries of perm.
// The experts are read from their pool slots in the slot layout below.
int launch_ffn_gemm1(const void *x_perm, void *h, const char *pool, size_t expert_bytes,
                     const TileDesc *tiles, int32_t m_tiles, int32_t m_tall, int32_t d, int32_t F, void *sink,
                     hipStream_t st, const LaunchEvents *ev, int32_t a_rows, const int32_t *perm = nullptr,
                     int32_t map_len = 0, int32_t k = 1, int32_t tile_m = 128);
int launch_ffn_gemm2(const void *h, void *y_perm, const char *pool, size_t expert_bytes,
                     const TileDesc *tiles, int32_t m_tiles, int32_t m_tall, int32_t d, int32_t F, void *sink,
                     hipStream_t st, const LaunchEvents *ev, int32_t a_rows, const int32_t *perm = nullptr,
                     const float *gate_perm = nullptr, int32_t tile_m = 128);

// Slot layout.  The host block of an expert is W_in [F, d] then W_out [d, F], row-major (the ABI);
// a pool slot holds the same two matrices, each in MFMA-fragment order: a matrix [R, K] is cut
// into stripes of 32 rows, and the 16-byte piece p (K values 8p .. 8p+7) of row r is stored at
//     ((r / 32) * (K / 8) + p) * 512 + (r % 32) * 16
// bytes from the matrix's start - a 32 x (K/8) matrix of pieces per stripe, transposed.  The 32
// rows x 16 K values a 32x32x16 MFMA takes as one operand (pieces 2j and 2j+1 of a stripe) are
// then 1 KiB of consecutive memory with lane l's 16 bytes at offset 16*l.  A stripe occupies the
// same bytes in both layouts, so a slot can be re-ordered in place, stripe by stripe.
inline size_t slot_piece_offset(size_t r, size_t p, size_t K) { return ((r / 32) * (K / 8) + p) * 512 + (r % 32) * 16; }
// Re-orders, in place, the n slots listed in tbl.dst from host-block order to slot order (after a
// plain copy of the host block into the slot).  d, F <= kMaxRelayoutK (a stripe is held in the
// registers of one workgroup).
constexpr int kMaxRelayoutK = 4096;
// A stream is about to be destroyed: drop what is cached about it (its handle may be reused).
void forget_stream(hipStream_t st);
// Expands tbl into token tiles: entry i gets ceil(count_i / tbl.tile_m) consecutive descriptors,
// entries in table order; counts come from `offsets` (device).  At most max_tiles are written.
int launch_build_tiles(const LayerTable &tbl, const int32_t *offsets, TileDesc *tiles, int32_t max_tiles,
                       hipStream_t st);
// K-c: y[t,:] = sum_{j<k} alpha[t*k+j] * y_perm[inv[t*k+j],:]; T = rows of y_perm (k per token).
int launch_combine(const void *y_perm, const int32_t *inv, const float *alpha, int32_t T, int32_t d,
                   void *y, hipStream_t st, const LaunchEvents *ev = nullptr, int32_t k = 1);

// Prefetch by kernel: up to kCopyBatch experts per launch, src = pinned host block (device-visible
// address), dst = pool slot.  expert_bytes is a multiple of 16.
constexpr int kCopyBatch = 64;
struct CopyTable {
    int32_t n;
    const void *src[kCopyBatch];
    void *dst[kCopyBatch];
};
// Copies the listed experts host -> slot, re-ordering them into the slot layout on the way.
int launch_expert_copy(const CopyTable &tbl, int32_t d, int32_t F, hipStream_t st);
int launch_slot_relayout(const CopyTable &tbl, int32_t d, int32_t F, hipStream_t st);

// Debug helpers (debug.hip).  check: latches layer + 1 into *flag_dev (device-visible host memory)
// when a device-side count differs from the plan's; poison: fills the listed slots with bf16 NaNs.
struct CountTable {
    int32_t n[256];
};
int launch_check_counts(const int32_t *counts, const CountTable &want, int32_t E, int32_t layer, int32_t *flag_dev,
                        hipStream_t st);
int launch_poison_slots(const CopyTable &tbl, size_t expert_bytes, hipStream_t st);

// The hash function (hash_fn.hip).  C is 64 or 128; ws holds 8*C floats per token.
struct HashShape {
    int32_t d_model, C, L, E, top_k;
};
int launch_hash_forward(const HashShape &sh, const float *params, const void *x, int32_t n_seq, int32_t seq_len,
                        int32_t *ids, float *alpha, float *ws, hipStream_t st);
// Device address of the current device's statically allocated hash-function scratch
// (kHashStaticScratchBytes bytes, 256-byte aligned); looked up once per device.  Returns a hipError_t.
constexpr size_t kHashStaticScratchBytes = size_t(16) << 20;
int hash_static_scratch(float **out);

constexpr int kGemmSinkBytes = 64 * 1024;
constexpr int kGemmTileM = 128;   // token rows per GEMM tile of large launches
constexpr int kGemmTileSmall = 64; // ... of small launches

}  // namespace sida
