// Internal definitions shared by the host-side sources of the library.
#pragma once
#include <hip/hip_runtime_api.h>

#include <condition_variable>
#include <cstdint>
#include <deque>
#include <mutex>
#include <vector>

#include "sida_moe.h"

namespace sida {

constexpr int kEventRing = 512;        // waves whose events can be outstanding at once
constexpr int kSortChunk = 256;        // tokens handled by one wavefront of the sort kernels
constexpr int kProfRing = 8192;        // profiled launches between two sida_profile_read calls

struct ProfRec {
    hipEvent_t start, stop;
    int klass;
};

// One queued hash table (Section 3.1): the expert ids of every MoE layer for one batch.
struct QueuedTable {
    int64_t tag = 0;
    int32_t T = 0;
    std::vector<int32_t> ids;          // [L][T]
    std::vector<int32_t> keys;         // activated keys layer*E+e, layer by layer, first-appearance order
    std::vector<int32_t> key_begin;    // [L+1] range of layer l inside keys
};

}  // namespace sida

struct sida_ctx {
    sida_config cfg{};
    size_t expert_bytes = 0;

    // bound resources (caller-owned)
    char *pool = nullptr;
    size_t pool_bytes = 0;
    std::vector<const void *> host_blocks;
    std::vector<const void *> host_blocks_dev;   // device-visible addresses of the blocks, empty if any is not pinned
    int32_t prefetch_mode = SIDA_PREFETCH_AUTO;

    // residency bookkeeping (Algorithm 1 + FIFO)
    std::vector<int32_t> slot_key;     // [S] key held by each slot, -1 empty
    std::vector<int32_t> key_slot;     // [L*E] slot holding the key, -1 absent
    std::vector<int32_t> last_use;     // [S] global wave that last computes from the slot
    int32_t cursor = 0;                // first-in-first-out: the slot overwritten next
    int32_t policy = SIDA_POLICY_FIFO;
    int32_t lookahead = 0;             // queued batches a popped batch may look ahead at
    int64_t clock = 0;                 // counts loads and hits
    std::vector<int64_t> loaded_at;    // [S] clock of the load that filled the slot
    std::vector<int64_t> touched_at;   // [S] clock of the slot's last load or hit
    std::vector<int64_t> next_use;     // [L*E] scratch of the planner
    std::vector<int32_t> wave_mark;    // [S] scratch of the planner: slots of the wave being assembled
    int32_t next_wave = 0;             // next global wave index to hand out
    uint32_t epoch = 1;

    // enqueue progress
    int32_t prefetched_upto = 0;       // global waves < this have their copies enqueued
    int32_t forwarded_upto = 0;        // global waves < this have their compute enqueued
    std::vector<hipEvent_t> ev_ready;  // ring: copies of wave g done
    std::vector<hipEvent_t> ev_done;   // ring: compute of wave g done
    std::vector<uint8_t> ready_recorded;  // ring: wave g recorded a ready event (it had misses)
    bool events_made = false;

    bool fused = true;                 // gather / combine folded into the grouped GEMMs (the default)
    int32_t top_k = 1;                 // experts per token (rows of a layer call = tokens * top_k)

    // kernel timing
    bool profiling = false;
    std::vector<sida::ProfRec> prof_pool;
    size_t prof_used = 0;
    double prof_ms[SIDA_K_COUNT] = {};
    int64_t prof_n[SIDA_K_COUNT] = {};

    // hash-table queue between the hash-building thread (push) and the inference thread (pop)
    std::mutex q_mu;
    std::condition_variable q_cv;
    std::deque<sida::QueuedTable> queue;
    bool q_closed = false;

    // debug switches (sida_set_debug)
    int32_t debug = 0;
    int32_t *debug_flag = nullptr;     // pinned host word the check kernel latches a mismatch into
    int32_t *debug_flag_dev = nullptr; // its device-visible address

    int last_hip = 0;
};

namespace sida {

// Host planner (plan.cpp).
int plan_layer(sida_ctx *c, int32_t layer, const int32_t *ids, int32_t T, const int32_t *future,
               int64_t n_future, sida_plan *out);

}  // namespace sida
