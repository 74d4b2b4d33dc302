// Host side of the C ABI: context, pool binding, expert prefetch, layer forward.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstring>
#include <new>

#include "ctx.h"
#include "kernels.h"
#include "tile_order.h"

using namespace sida;

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define HIP_TRY(ctx, expr)                           \
    do {                                             \
        hipError_t err__ = (expr);                   \
        if (err__ != hipSuccess) {                   \
            (ctx)->last_hip = (int)err__;            \
            return SIDA_EHIP;                        \
        }                                            \
    } while (0)

int make_events(sida_ctx *c)
{
    if (c->events_made) return SIDA_OK;
    c->ev_ready.assign(kEventRing, nullptr);
    c->ev_done.assign(kEventRing, nullptr);
    c->ready_recorded.assign(kEventRing, 0);
    for (int i = 0; i < kEventRing; ++i) {
        hipError_t e = hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_done[i], hipEventDisableTiming);
        if (e != hipSuccess) {                                // give back what was made: a later call starts over
            for (int j = 0; j <= i; ++j) {
                if (c->ev_ready[j]) (void)hipEventDestroy(c->ev_ready[j]);
                if (c->ev_done[j]) (void)hipEventDestroy(c->ev_done[j]);
            }
            c->ev_ready.clear();
            c->ev_done.clear();
            c->last_hip = (int)e;
            return SIDA_EHIP;
        }
    }
    c->events_made = true;
    return SIDA_OK;
}

// Upper bound of token tiles of a layer: every expert may end in a partial tile.
size_t max_tiles(const sida_config &cfg, int32_t T) { return (size_t)T / kGemmTileSmall + (size_t)cfg.E + 1; }

void layout(const sida_config &cfg, int32_t T, sida_ws_layout *o)
{
    const size_t n_chunks = ((size_t)T + kSortChunk - 1) / kSortChunk;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    o->counts = take(sizeof(int32_t) * (size_t)cfg.E);
    o->offsets = take(sizeof(int32_t) * ((size_t)cfg.E + 1));
    o->block_hist = take(sizeof(int32_t) * std::max<size_t>(1, n_chunks) * (size_t)cfg.E);
    o->perm = take(sizeof(int32_t) * (size_t)T);
    o->inv = take(sizeof(int32_t) * (size_t)T);
    o->x_perm = take(2 * (size_t)T * (size_t)cfg.d_model);
    o->h = take(2 * (size_t)T * (size_t)cfg.d_ff);
    o->y_perm = take(2 * (size_t)T * (size_t)cfg.d_model);
    o->tiles = take(sizeof(TileDesc) * max_tiles(cfg, T));
    o->sink = take(kGemmSinkBytes);
    o->gate_perm = take(sizeof(float) * (size_t)T);
    o->total = off;
}

struct Ws {
    int32_t *counts, *offsets, *block_hist, *perm, *inv;
    void *x_perm, *h, *y_perm;
    TileDesc *tiles;
    int32_t max_tiles;
    void *sink;
    float *gate_perm;
};

Ws carve(const sida_config &cfg, int32_t T, void *base)
{
    sida_ws_layout l;
    layout(cfg, T, &l);
    char *b = static_cast<char *>(base);
    return Ws{(int32_t *)(b + l.counts), (int32_t *)(b + l.offsets), (int32_t *)(b + l.block_hist),
              (int32_t *)(b + l.perm),   (int32_t *)(b + l.inv),     b + l.x_perm,
              b + l.h,                   b + l.y_perm,               (TileDesc *)(b + l.tiles),
              (int32_t)max_tiles(cfg, T), b + l.sink, (float *)(b + l.gate_perm)};
}

int check_plan(const sida_ctx *c, const sida_plan *p)
{
    if (!c || !p) return SIDA_EINVAL;
    if (p->epoch != c->epoch) return SIDA_ESTATE;
    if (p->E != c->cfg.E || p->layer < 0 || p->layer >= c->cfg.L || p->T < 0 || p->T > c->cfg.max_T) return SIDA_EINVAL;
    if (p->n_waves < 0 || p->n_active < 0 || p->n_active > c->cfg.E) return SIDA_EINVAL;
    if (p->n_waves > 0 && (p->first_wave < 0 || p->first_wave + p->n_waves > c->next_wave)) return SIDA_ESTATE;
    return SIDA_OK;
}

// A layer whose device-side token counts differed from its plan's was seen (SIDA_DEBUG_CHECK_IDS).
bool ids_mismatch_latched(const sida_ctx *c) { return c->debug_flag && *static_cast<volatile int32_t *>(c->debug_flag) != 0; }

int check_ws(const sida_ctx *c, int32_t T, const void *ws, size_t bytes)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SIDA_EINVAL;
    sida_ws_layout l;
    layout(c->cfg, T, &l);
    return bytes < l.total ? SIDA_ENOSPC : SIDA_OK;
}

// ---- kernel timing -------------------------------------------------------------------------
struct Timed {
    sida_ctx *c;
    hipStream_t st;
    ProfRec *rec = nullptr;
    Timed(sida_ctx *ctx, int klass, hipStream_t s) : c(ctx), st(s)
    {
        if (!c->profiling) return;
        if (c->prof_used == c->prof_pool.size()) {
            if (c->prof_pool.size() >= (size_t)kProfRing) return;     // ring full: launch goes untimed
            ProfRec r{};
            if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return;
            c->prof_pool.push_back(r);
        }
        rec = &c->prof_pool[c->prof_used++];
        rec->klass = klass;
        (void)hipEventRecord(rec->start, st);
    }
    ~Timed()
    {
        if (rec) (void)hipEventRecord(rec->stop, st);
    }
};

// Timing record of a class that is one kernel: the events ride on the kernel's own dispatch.
struct TimedKernel {
    LaunchEvents ev{};
    bool on = false;
    TimedKernel(sida_ctx *c, int klass)
    {
        if (!c->profiling) return;
        if (c->prof_used == c->prof_pool.size()) {
            if (c->prof_pool.size() >= (size_t)kProfRing) return;
            ProfRec r{};
            if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return;
            c->prof_pool.push_back(r);
        }
        ProfRec *rec = &c->prof_pool[c->prof_used++];
        rec->klass = klass;
        ev.start = rec->start;
        ev.stop = rec->stop;
        on = true;
    }
    const LaunchEvents *get() const { return on ? &ev : nullptr; }
};

// Tile schedule of a layer: the activated experts wave by wave, inside a wave most tokens first,
// and for every local wave the range of token tiles it owns in the expanded descriptor array.
struct LayerSchedule {
    LayerTable tbl;
    int32_t tile_begin[SIDA_MAX_E];
    int32_t m_tiles[SIDA_MAX_E];
    int32_t m_tall[SIDA_MAX_E];       // leading tiles of the wave that belong to experts with more than one tile
};

// Token rows per tile for a layer.  A grouped GEMM is bound by the rows its tiles pull through LDS:
// a tile of tile_m token rows and 256 weight rows costs tile_m + 256 rows per K-step whether or not
// all its token rows exist.  64-row tiles pay when most experts have at most 64 tokens, i.e. when
// halving the tile height adds few tiles: tiles(64) * 320 <= tiles(128) * 384.  (Measured on the
// Switch-base-128 shape: 64-row tiles are 8-10 % faster at 8-16 tokens per expert, even at 64, and
// 6 % slower at 128 tokens per expert.)
int32_t choose_tile_m(const sida_plan *p)
{
    // A layer that is cut into waves launches a few experts at a time: small launches, hidden
    // behind the copies; 64-row tiles give them more (and deeper-fetching) tiles.
    if (p->n_waves > 1) return kGemmTileSmall;
    int64_t t64 = 0, t128 = 0;
    for (int32_t i = 0; i < p->n_active; ++i) {
        const int32_t n = p->counts[p->order[i]];
        t64 += (n + kGemmTileSmall - 1) / kGemmTileSmall;
        t128 += (n + kGemmTileM - 1) / kGemmTileM;
    }
    return 5 * t64 <= 6 * t128 ? kGemmTileSmall : kGemmTileM;
}

void build_schedule(const sida_plan *p, int32_t tile_m, LayerSchedule *s)
{
    int32_t idx[SIDA_MAX_E];
    for (int32_t i = 0; i < p->n_active; ++i) idx[i] = p->order[i];     // already grouped by wave
    std::stable_sort(idx, idx + p->n_active, [&](int32_t a, int32_t b) {
        if (p->wave[a] != p->wave[b]) return p->wave[a] < p->wave[b];
        return p->counts[a] > p->counts[b];
    });
    s->tbl.n = p->n_active;
    s->tbl.tile_m = tile_m;
    for (int32_t w = 0; w < p->n_waves; ++w) s->tile_begin[w] = s->m_tiles[w] = s->m_tall[w] = 0;
    int32_t at = 0, cur = -1;
    for (int32_t i = 0; i < p->n_active; ++i) {
        const int32_t e = idx[i];
        s->tbl.expert[i] = (uint8_t)e;
        s->tbl.slot[i] = (int16_t)p->slot[e];
        const int32_t w = p->wave[e] - p->first_wave;
        if (w != cur) {
            s->tile_begin[w] = at;
            cur = w;
        }
        const int32_t n_t = (p->counts[e] + tile_m - 1) / tile_m;
        s->m_tiles[w] += n_t;
        if (n_t > 1) s->m_tall[w] += n_t;                            // sorted by count: these come first
        at += n_t;
    }
}

// Copies of local wave w (global g).  Caller has checked order and dependencies.
int enqueue_prefetch(sida_ctx *c, const sida_plan *p, int32_t w, hipStream_t copy)
{
    const int32_t g = p->first_wave + w;
    const int ring = g % kEventRing;
    int32_t misses = 0;
    for (int32_t i = 0; i < p->n_active; ++i) {
        const int32_t e = p->order[i];
        if (p->wave[e] == g && p->hit[e] == 0) ++misses;
    }
    c->ready_recorded[ring] = 0;
    if (misses) {
        if (g >= kEventRing) HIP_TRY(c, hipEventSynchronize(c->ev_ready[ring]));   // slot of wave g - ring
        const int32_t dep = p->wave_dep[w];
        if (dep >= 0) HIP_TRY(c, hipStreamWaitEvent(copy, c->ev_done[dep % kEventRing], 0));
        {
            Timed tm(c, SIDA_K_COPY, copy);
            const bool by_kernel = c->prefetch_mode != SIDA_PREFETCH_COPY_ENGINE && !c->host_blocks_dev.empty();
            // by kernel: the copy writes the slot layout itself; by copy engine: the host block lands
            // as it is and the slots are re-ordered in place afterwards
            auto flush = [&](const CopyTable &t) {
                return by_kernel ? launch_expert_copy(t, c->cfg.d_model, c->cfg.d_ff, copy)
                                 : launch_slot_relayout(t, c->cfg.d_model, c->cfg.d_ff, copy);
            };
            if (c->debug & SIDA_DEBUG_POISON_SLOTS) {           // after the wait above: the slots' last readers are done
                CopyTable pt;
                pt.n = 0;
                for (int32_t i = 0; i < p->n_active; ++i) {
                    const int32_t e = p->order[i];
                    if (p->wave[e] != g || p->hit[e] != 0) continue;
                    pt.src[pt.n] = nullptr;
                    pt.dst[pt.n] = c->pool + (size_t)p->slot[e] * c->expert_bytes;
                    if (++pt.n == kCopyBatch) {
                        HIP_TRY(c, (hipError_t)launch_poison_slots(pt, c->expert_bytes, copy));
                        pt.n = 0;
                    }
                }
                HIP_TRY(c, (hipError_t)launch_poison_slots(pt, c->expert_bytes, copy));
            }
            CopyTable tbl;
            tbl.n = 0;
            for (int32_t i = 0; i < p->n_active; ++i) {
                const int32_t e = p->order[i];
                if (p->wave[e] != g || p->hit[e] != 0) continue;
                const size_t key = (size_t)p->layer * c->cfg.E + e;
                char *dst = c->pool + (size_t)p->slot[e] * c->expert_bytes;
                if (!by_kernel)
                    HIP_TRY(c, hipMemcpyAsync(dst, c->host_blocks[key], c->expert_bytes, hipMemcpyHostToDevice, copy));
                tbl.src[tbl.n] = by_kernel ? c->host_blocks_dev[key] : nullptr;
                tbl.dst[tbl.n] = dst;
                if (++tbl.n == kCopyBatch) {
                    HIP_TRY(c, (hipError_t)flush(tbl));
                    tbl.n = 0;
                }
            }
            if (tbl.n) HIP_TRY(c, (hipError_t)flush(tbl));
        }
        HIP_TRY(c, hipEventRecord(c->ev_ready[ring], copy));
        c->ready_recorded[ring] = 1;
    }
    c->prefetched_upto = g + 1;
    return SIDA_OK;
}

int prefetch_allowed(const sida_ctx *c, const sida_plan *p, int32_t w)
{
    const int32_t g = p->first_wave + w;
    if (g != c->prefetched_upto) return SIDA_ESTATE;
    if (p->wave_dep[w] >= c->forwarded_upto) return SIDA_ESTATE;
    return SIDA_OK;
}

// alpha != NULL: the fused path - the gate values are moved along with the sort and the gather
// pass is left to GEMM 1.
int launch_dispatch(sida_ctx *c, const void *x, const int32_t *ids, int32_t T, const Ws &ws, const LayerTable *tbl,
                    hipStream_t st, const float *alpha = nullptr)
{
    {
        Timed tm(c, SIDA_K_SORT, st);
        HIP_TRY(c, (hipError_t)launch_sort(ids, T, c->cfg.E, ws.counts, ws.offsets, ws.block_hist, ws.perm, ws.inv, tbl,
                                           ws.tiles, ws.max_tiles, st, alpha, ws.gate_perm));
    }
    if (!alpha) {
        TimedKernel tk(c, SIDA_K_GATHER);
        HIP_TRY(c, (hipError_t)launch_gather(x, ws.perm, T, c->cfg.d_model, ws.x_perm, st, tk.get(), c->top_k));
    }
    return SIDA_OK;
}

int launch_tiles(sida_ctx *c, const LayerSchedule &s, const Ws &ws, hipStream_t st)
{
    Timed tm(c, SIDA_K_SORT, st);
    HIP_TRY(c, (hipError_t)launch_build_tiles(s.tbl, ws.offsets, ws.tiles, ws.max_tiles, st));
    return SIDA_OK;
}

// x, y != NULL: the fused path - GEMM 1 reads x through perm, GEMM 2 scales by the gate and writes y.
int launch_wave_ffn(sida_ctx *c, const LayerSchedule &s, int32_t w, const Ws &ws, int32_t T, hipStream_t st,
                    const void *x = nullptr, void *y = nullptr)
{
    const TileDesc *tiles = ws.tiles + s.tile_begin[w];
    {
        TimedKernel tk(c, SIDA_K_GEMM1);
        HIP_TRY(c, (hipError_t)launch_ffn_gemm1(x ? x : ws.x_perm, ws.h, c->pool, c->expert_bytes, tiles, s.m_tiles[w],
                                                s.m_tall[w], c->cfg.d_model, c->cfg.d_ff, ws.sink, st, tk.get(),
                                                x ? T / c->top_k : T, x ? ws.perm : nullptr, T, c->top_k, s.tbl.tile_m));
    }
    {
        TimedKernel tk(c, SIDA_K_GEMM2);
        HIP_TRY(c, (hipError_t)launch_ffn_gemm2(ws.h, y ? y : ws.y_perm, c->pool, c->expert_bytes, tiles, s.m_tiles[w],
                                                s.m_tall[w], c->cfg.d_model, c->cfg.d_ff, ws.sink, st, tk.get(), T,
                                                y ? ws.perm : nullptr, y ? ws.gate_perm : nullptr, s.tbl.tile_m));
    }
    return SIDA_OK;
}

struct LayerArgs {
    const sida_plan *plan;
    const void *x;
    const int32_t *ids;
    const float *alpha;
    void *y;
};

int check_layer_args(const sida_ctx *c, const LayerArgs &a)
{
    int rc = check_plan(c, a.plan);
    if (rc) return rc;
    if (a.plan->T > 0 && (!a.x || !a.ids || !a.alpha || !a.y)) return SIDA_EINVAL;
    if (a.plan->T % c->top_k) return SIDA_EINVAL;               // k (token, expert) pairs per token
    return SIDA_OK;
}

// Forwards `n` consecutive layers.  The copy stream is kept one wave ahead of the compute
// whenever the next wave's dependency has already been enqueued.
int forward_layers(sida_ctx *c, int32_t n, const LayerArgs *layers, void *ws_dev, size_t ws_bytes,
                   hipStream_t compute, hipStream_t copy)
{
    if (!c->pool || c->host_blocks.empty()) return SIDA_ESTATE;
    if (ids_mismatch_latched(c)) return SIDA_ESTATE;
    int32_t expect = c->forwarded_upto;
    for (int32_t i = 0; i < n; ++i) {
        int rc = check_layer_args(c, layers[i]);
        if (rc) return rc;
        const sida_plan *p = layers[i].plan;
        if (p->n_waves == 0) continue;
        if (p->first_wave != expect) return SIDA_ESTATE;           // layers out of planned order
        expect += p->n_waves;
        rc = check_ws(c, p->T, ws_dev, ws_bytes);
        if (rc) return rc;
    }
    int rc = make_events(c);
    if (rc) return rc;

    // flat list of (layer, local wave) still to forward, to find "the next wave" across layers
    auto next_of = [&](int32_t li, int32_t w, int32_t *nli, int32_t *nw) {
        ++w;
        while (li < n && w >= layers[li].plan->n_waves) {
            ++li;
            w = 0;
        }
        *nli = li;
        *nw = w;
        return li < n;
    };
    auto try_prefetch = [&](int32_t li, int32_t w) -> int {
        const sida_plan *p = layers[li].plan;
        const int32_t g = p->first_wave + w;
        if (g < c->prefetched_upto) return SIDA_OK;                // done earlier (by the caller)
        if (prefetch_allowed(c, p, w) != SIDA_OK) return 1;        // not yet possible
        return enqueue_prefetch(c, p, w, copy);
    };

    for (int32_t li = 0; li < n; ++li) {
        const LayerArgs &a = layers[li];
        const sida_plan *p = a.plan;
        if (p->n_waves == 0) continue;
        const Ws ws = carve(c->cfg, p->T, ws_dev);
        LayerSchedule sched;
        build_schedule(p, choose_tile_m(p), &sched);
        const bool fused = c->fused;
        rc = launch_dispatch(c, a.x, a.ids, p->T, ws, &sched.tbl, compute,      // also expands sched.tbl into tiles
                             fused ? a.alpha : nullptr);
        if (rc) return rc;
        if (c->debug & SIDA_DEBUG_CHECK_IDS) {                 // the sort's counts against the plan's
            CountTable want;
            std::memcpy(want.n, p->counts, sizeof want.n);
            HIP_TRY(c, (hipError_t)launch_check_counts(ws.counts, want, c->cfg.E, p->layer, c->debug_flag_dev, compute));
        }
        for (int32_t w = 0; w < p->n_waves; ++w) {
            const int32_t g = p->first_wave + w;
            rc = try_prefetch(li, w);
            if (rc < 0) return rc;
            if (rc > 0) return SIDA_ESTATE;                        // cannot happen: wave_dep < g
            int32_t nli, nw;
            if (next_of(li, w, &nli, &nw)) {
                rc = try_prefetch(nli, nw);                        // look one wave ahead
                if (rc < 0) return rc;
            }
            const int ring = g % kEventRing;
            if (c->ready_recorded[ring]) HIP_TRY(c, hipStreamWaitEvent(compute, c->ev_ready[ring], 0));
            // with several experts per token a y row is a sum over tiles: only the gather is folded in
            rc = launch_wave_ffn(c, sched, w, ws, p->T, compute, fused ? a.x : nullptr,
                                 fused && c->top_k == 1 ? a.y : nullptr);
            if (rc) return rc;
            if (g >= kEventRing) HIP_TRY(c, hipEventSynchronize(c->ev_done[ring]));
            HIP_TRY(c, hipEventRecord(c->ev_done[ring], compute));
            c->forwarded_upto = g + 1;
        }
        if (!fused || c->top_k > 1) {
            TimedKernel tk(c, SIDA_K_COMBINE);
            HIP_TRY(c, (hipError_t)launch_combine(ws.y_perm, ws.inv, a.alpha, p->T, c->cfg.d_model, a.y, compute, tk.get(),
                                                  c->top_k));
        }
    }
    return SIDA_OK;
}

}  // namespace

extern "C" {

int sida_create(const sida_config *cfg, sida_ctx **out)
{
    if (!cfg || !out) return SIDA_EINVAL;
    *out = nullptr;
    if (cfg->L < 1 || cfg->E < 1 || cfg->E > SIDA_MAX_E || cfg->S < 1 || cfg->S > 32767 || cfg->W < 1 ||
        cfg->W > cfg->S || cfg->W > SIDA_MAX_E || cfg->max_T < 0 || cfg->d_model < 128 || cfg->d_ff < 128 ||
        cfg->d_model % 128 || cfg->d_ff % 128 || cfg->d_model > kMaxRelayoutK || cfg->d_ff > kMaxRelayoutK)
        return SIDA_EINVAL;
    // the kernels address activation rows with 32-bit byte offsets
    if ((int64_t)cfg->max_T * std::max(cfg->d_model, cfg->d_ff) * 2 > INT32_MAX) return SIDA_EINVAL;
    if ((int64_t)cfg->L * cfg->E > INT32_MAX) return SIDA_EINVAL;
    sida_ctx *c = new (std::nothrow) sida_ctx;
    if (!c) return SIDA_ENOMEM;
    try {
        c->cfg = *cfg;
        c->expert_bytes = (size_t)4 * cfg->d_model * cfg->d_ff;
        c->slot_key.assign(cfg->S, -1);
        c->last_use.assign(cfg->S, -1);
        c->loaded_at.assign(cfg->S, -1);
        c->touched_at.assign(cfg->S, -1);
        c->key_slot.assign((size_t)cfg->L * cfg->E, -1);
        c->next_use.reserve((size_t)cfg->L * cfg->E);
        c->wave_mark.assign(cfg->S, -1);
    } catch (const std::bad_alloc &) {
        delete c;
        return SIDA_ENOMEM;
    }
    *out = c;
    return SIDA_OK;
}

void sida_destroy(sida_ctx *c)
{
    if (!c) return;
    if (c->events_made)
        for (int i = 0; i < kEventRing; ++i) {
            if (c->ev_ready[i]) (void)hipEventDestroy(c->ev_ready[i]);
            if (c->ev_done[i]) (void)hipEventDestroy(c->ev_done[i]);
        }
    for (auto &r : c->prof_pool) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    if (c->debug_flag) (void)hipHostFree(c->debug_flag);
    delete c;
}

const char *sida_strerror(int code)
{
    switch (code) {
        case SIDA_OK: return "ok";
        case SIDA_EINVAL: return "invalid argument";
        case SIDA_EAGAIN: return "hash-table queue empty (timed out)";
        case SIDA_ECLOSED: return "hash-table queue closed";
        case SIDA_ENOSPC: return "workspace or pool too small";
        case SIDA_ESTATE: return "call not valid in this state (unbound pool/weights, stale plan or wrong order)";
        case SIDA_EHIP: return "HIP call failed";
        case SIDA_ENOMEM: return "out of host memory";
        default: return "unknown status";
    }
}

int sida_last_hip_error(const sida_ctx *c) { return c ? c->last_hip : 0; }

size_t sida_expert_bytes(const sida_ctx *c) { return c ? c->expert_bytes : 0; }

size_t sida_slot_offset(const sida_ctx *c, int32_t which, int32_t row, int32_t col)
{
    if (!c || which < 0 || which > 1 || row < 0 || col < 0) return (size_t)-1;
    const size_t R = which == 0 ? c->cfg.d_ff : c->cfg.d_model, K = which == 0 ? c->cfg.d_model : c->cfg.d_ff;
    if ((size_t)row >= R || (size_t)col >= K) return (size_t)-1;
    return (which == 0 ? 0 : R * K * 2) + slot_piece_offset(row, col / 8, K) + (size_t)(col % 8) * 2;
}

size_t sida_workspace_bytes(const sida_ctx *c, int32_t T)
{
    if (!c || T < 0 || T > c->cfg.max_T) return 0;
    sida_ws_layout l;
    layout(c->cfg, T, &l);
    return l.total;
}

int sida_workspace_layout(const sida_ctx *c, int32_t T, sida_ws_layout *out)
{
    if (!c || !out || T < 0 || T > c->cfg.max_T) return SIDA_EINVAL;
    layout(c->cfg, T, out);
    return SIDA_OK;
}

int sida_bind_pool(sida_ctx *c, void *pool_dev, size_t bytes)
{
    if (!c || !pool_dev || (reinterpret_cast<uintptr_t>(pool_dev) & 255u)) return SIDA_EINVAL;
    if (bytes < (size_t)c->cfg.S * c->expert_bytes) return SIDA_ENOSPC;
    c->pool = static_cast<char *>(pool_dev);
    c->pool_bytes = bytes;
    return SIDA_OK;
}

int sida_bind_host_weights(sida_ctx *c, const void *const *host_blocks)
{
    if (!c || !host_blocks) return SIDA_EINVAL;
    const size_t n = (size_t)c->cfg.L * c->cfg.E;
    for (size_t i = 0; i < n; ++i)
        if (!host_blocks[i]) return SIDA_EINVAL;
    try {
        c->host_blocks.assign(host_blocks, host_blocks + n);
        // Blocks in pinned (page-locked, device-mapped) memory can be read by a kernel; anything
        // else is left to hipMemcpyAsync, which stages pageable memory itself.
        c->host_blocks_dev.assign(n, nullptr);
        bool all_pinned = true;
        for (size_t i = 0; i < n && all_pinned; ++i) {
            hipPointerAttribute_t at{};
            if (hipPointerGetAttributes(&at, host_blocks[i]) != hipSuccess || at.type != hipMemoryTypeHost ||
                !at.devicePointer) {
                (void)hipGetLastError();                         // not an error of this call
                all_pinned = false;
                break;
            }
            c->host_blocks_dev[i] = at.devicePointer;
        }
        if (!all_pinned) c->host_blocks_dev.clear();
    } catch (const std::bad_alloc &) {
        return SIDA_ENOMEM;
    }
    return SIDA_OK;
}

int sida_streams_create(int32_t copy_cus, void **compute_stream, void **copy_stream)
{
    if (!compute_stream || !copy_stream || copy_cus < 0) return SIDA_EINVAL;
    *compute_stream = *copy_stream = nullptr;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return SIDA_EHIP;
    const int total = prop.multiProcessorCount;
    if (copy_cus > 0 && (copy_cus % 8 || copy_cus > total / 2 || total > 512)) return SIDA_EINVAL;
    hipStream_t cs = nullptr, ps = nullptr;
    if (copy_cus == 0) {
        if (hipStreamCreateWithFlags(&cs, hipStreamNonBlocking) != hipSuccess) return SIDA_EHIP;
        if (hipStreamCreateWithFlags(&ps, hipStreamNonBlocking) != hipSuccess) {
            (void)hipStreamDestroy(cs);
            return SIDA_EHIP;
        }
    } else {
        // mask bit i is compute unit i / 8 of XCD i % 8: the first copy_cus bits are copy_cus / 8
        // compute units of every XCD
        uint32_t copy_mask[16] = {}, comp_mask[16] = {};
        for (int i = 0; i < total; ++i) (i < copy_cus ? copy_mask : comp_mask)[i >> 5] |= 1u << (i & 31);
        const int words = (total + 31) / 32;
        if (hipExtStreamCreateWithCUMask(&cs, words, comp_mask) != hipSuccess) return SIDA_EHIP;
        if (hipExtStreamCreateWithCUMask(&ps, words, copy_mask) != hipSuccess) {
            (void)hipStreamDestroy(cs);
            return SIDA_EHIP;
        }
    }
    *compute_stream = cs;
    *copy_stream = ps;
    return SIDA_OK;
}

int sida_streams_destroy(void *compute_stream, void *copy_stream)
{
    int rc = SIDA_OK;
    forget_stream(static_cast<hipStream_t>(compute_stream));
    forget_stream(static_cast<hipStream_t>(copy_stream));
    if (compute_stream && hipStreamDestroy(static_cast<hipStream_t>(compute_stream)) != hipSuccess) rc = SIDA_EHIP;
    if (copy_stream && hipStreamDestroy(static_cast<hipStream_t>(copy_stream)) != hipSuccess) rc = SIDA_EHIP;
    return rc;
}

int sida_set_prefetch_mode(sida_ctx *c, int32_t mode)
{
    if (!c || mode < SIDA_PREFETCH_AUTO || mode > SIDA_PREFETCH_KERNEL) return SIDA_EINVAL;
    if (mode == SIDA_PREFETCH_KERNEL && c->host_blocks_dev.empty()) return SIDA_ESTATE;
    c->prefetch_mode = mode;
    return SIDA_OK;
}

int sida_pool_reset(sida_ctx *c)
{
    if (!c) return SIDA_EINVAL;
    std::fill(c->slot_key.begin(), c->slot_key.end(), -1);
    std::fill(c->last_use.begin(), c->last_use.end(), -1);
    std::fill(c->key_slot.begin(), c->key_slot.end(), -1);
    std::fill(c->ready_recorded.begin(), c->ready_recorded.end(), 0);
    std::fill(c->loaded_at.begin(), c->loaded_at.end(), -1);
    std::fill(c->touched_at.begin(), c->touched_at.end(), -1);
    c->clock = 0;
    c->cursor = 0;
    c->next_wave = 0;
    c->prefetched_upto = 0;
    c->forwarded_upto = 0;
    ++c->epoch;
    if (c->debug_flag) *c->debug_flag = 0;
    return SIDA_OK;
}

int sida_pool_state(const sida_ctx *c, int32_t *slot_key, int32_t *cursor, int32_t *next_wave)
{
    if (!c) return SIDA_EINVAL;
    if (slot_key) std::memcpy(slot_key, c->slot_key.data(), sizeof(int32_t) * c->slot_key.size());
    if (cursor) *cursor = c->cursor;
    if (next_wave) *next_wave = c->next_wave;
    return SIDA_OK;
}

int sida_moe_plan(sida_ctx *c, int32_t layer, const int32_t *ids_host, int32_t T, sida_plan *out)
{
    if (!c || !out || layer < 0 || layer >= c->cfg.L || T < 0 || T > c->cfg.max_T || (T > 0 && !ids_host))
        return SIDA_EINVAL;
    if (c->next_wave > INT32_MAX - 2 * SIDA_MAX_E) return SIDA_ESTATE;   // wave counter exhausted: reset the pool
    try {
        return plan_layer(c, layer, ids_host, T, nullptr, 0, out);
    } catch (const std::bad_alloc &) {
        return SIDA_ENOMEM;
    }
}

int sida_moe_plan_lookahead(sida_ctx *c, int32_t layer, const int32_t *ids_host, int32_t T,
                            const int32_t *future_keys, int64_t n_future, sida_plan *out)
{
    if (!c || !out || layer < 0 || layer >= c->cfg.L || T < 0 || T > c->cfg.max_T || (T > 0 && !ids_host) ||
        n_future < 0 || (n_future > 0 && !future_keys))
        return SIDA_EINVAL;
    if (c->next_wave > INT32_MAX - 2 * SIDA_MAX_E) return SIDA_ESTATE;
    try {
        return plan_layer(c, layer, ids_host, T, future_keys, n_future, out);
    } catch (const std::bad_alloc &) {
        return SIDA_ENOMEM;
    }
}

int sida_set_top_k(sida_ctx *c, int32_t k)
{
    if (!c || k < 1 || k > SIDA_MAX_TOP_K) return SIDA_EINVAL;
    c->top_k = k;
    return SIDA_OK;
}

int sida_set_fusion(sida_ctx *c, int32_t on)
{
    if (!c) return SIDA_EINVAL;
    c->fused = on != 0;
    return SIDA_OK;
}

int sida_set_debug(sida_ctx *c, int32_t flags)
{
    if (!c || (flags & ~(SIDA_DEBUG_CHECK_IDS | SIDA_DEBUG_POISON_SLOTS))) return SIDA_EINVAL;
    if ((flags & SIDA_DEBUG_CHECK_IDS) && !c->debug_flag) {    // one pinned word the check kernel can write
        void *p = nullptr, *d = nullptr;
        HIP_TRY(c, hipHostMalloc(&p, 64, hipHostMallocMapped));
        if (hipHostGetDevicePointer(&d, p, 0) != hipSuccess) {
            (void)hipHostFree(p);
            c->last_hip = (int)hipGetLastError();
            return SIDA_EHIP;
        }
        c->debug_flag = static_cast<int32_t *>(p);
        c->debug_flag_dev = static_cast<int32_t *>(d);
    }
    if (c->debug_flag) *c->debug_flag = 0;
    c->debug = flags;
    return SIDA_OK;
}

int sida_debug_mismatch_layer(const sida_ctx *c)
{
    if (!c) return SIDA_EINVAL;
    return c->debug_flag ? *static_cast<volatile int32_t *>(c->debug_flag) - 1 : -1;
}

int sida_set_policy(sida_ctx *c, int32_t policy, int32_t lookahead_batches)
{
    if (!c || policy < SIDA_POLICY_FIFO || policy > SIDA_POLICY_BELADY || lookahead_batches < 0 ||
        lookahead_batches > SIDA_QUEUE_CAPACITY)
        return SIDA_EINVAL;
    for (int32_t k : c->slot_key)
        if (k >= 0) return SIDA_ESTATE;              // ages of resident experts would be meaningless
    c->policy = policy;
    c->lookahead = lookahead_batches;
    return SIDA_OK;
}

// ---- hash-table queue ------------------------------------------------------------------------
int sida_queue_push(sida_ctx *c, int64_t tag, const int32_t *ids_host, int32_t T)
{
    if (!c || T < 0 || T > c->cfg.max_T || (T > 0 && !ids_host)) return SIDA_EINVAL;
    const int32_t L = c->cfg.L, E = c->cfg.E;
    QueuedTable q;
    try {
        q.tag = tag;
        q.T = T;
        q.ids.assign(ids_host, ids_host + (size_t)L * T);
        q.key_begin.assign(L + 1, 0);
        std::vector<uint8_t> seen(E);
        for (int32_t l = 0; l < L; ++l) {
            std::fill(seen.begin(), seen.end(), 0);
            for (int32_t t = 0; t < T; ++t) {
                const int32_t k = q.ids[(size_t)l * T + t];
                if (k < 0 || k >= E) return SIDA_EINVAL;
                if (!seen[k]) {
                    seen[k] = 1;
                    q.keys.push_back(l * E + k);
                }
            }
            q.key_begin[l + 1] = (int32_t)q.keys.size();
        }
        std::lock_guard<std::mutex> lk(c->q_mu);
        if (c->q_closed) return SIDA_ECLOSED;
        if (c->queue.size() >= (size_t)SIDA_QUEUE_CAPACITY) return SIDA_ENOSPC;
        c->queue.push_back(std::move(q));
    } catch (const std::bad_alloc &) {
        return SIDA_ENOMEM;
    }
    c->q_cv.notify_one();
    return SIDA_OK;
}

int sida_queue_close(sida_ctx *c)
{
    if (!c) return SIDA_EINVAL;
    {
        std::lock_guard<std::mutex> lk(c->q_mu);
        c->q_closed = true;
    }
    c->q_cv.notify_all();
    return SIDA_OK;
}

int sida_queue_size(sida_ctx *c)
{
    if (!c) return SIDA_EINVAL;
    std::lock_guard<std::mutex> lk(c->q_mu);
    return (int)c->queue.size();
}

int sida_queue_pop_plan(sida_ctx *c, int32_t timeout_ms, int64_t *tag, int32_t *T, sida_plan *plans)
{
    if (!c || !plans || timeout_ms < 0) return SIDA_EINVAL;
    const int32_t L = c->cfg.L;
    if (c->next_wave > INT32_MAX - 2 * SIDA_MAX_E * L) return SIDA_ESTATE;
    QueuedTable q;
    std::vector<int32_t> behind;                      // activated keys of the batches still queued
    std::vector<int32_t> future;
    try {
        std::unique_lock<std::mutex> lk(c->q_mu);
        if (!c->q_cv.wait_for(lk, std::chrono::milliseconds(timeout_ms),
                              [&] { return !c->queue.empty() || c->q_closed; }))
            return SIDA_EAGAIN;                       // the inference thread stays idle (Section 3.1)
        if (c->queue.empty()) return SIDA_ECLOSED;
        // Everything that allocates happens while the table is still queued: a failure leaves
        // the queue and the pool bookkeeping as they were.
        if (c->policy == SIDA_POLICY_BELADY) {
            int32_t n = 0;
            for (auto it = c->queue.begin() + 1; it != c->queue.end(); ++it) {
                if (n++ == c->lookahead) break;
                behind.insert(behind.end(), it->keys.begin(), it->keys.end());
            }
        }
        future.reserve(c->queue.front().keys.size() + behind.size());
        q = std::move(c->queue.front());              // moving a QueuedTable does not allocate
        c->queue.pop_front();
    } catch (const std::bad_alloc &) {
        return SIDA_ENOMEM;
    }
    for (int32_t l = 0; l < L; ++l) {                 // within the reserved capacity: no allocation
        future.assign(q.keys.begin() + q.key_begin[l + 1], q.keys.end());   // later layers of this batch
        future.insert(future.end(), behind.begin(), behind.end());
        const int rc = plan_layer(c, l, q.ids.data() + (size_t)l * q.T, q.T, future.data(), (int64_t)future.size(),
                                  &plans[l]);
        if (rc != SIDA_OK) return rc;                 // cannot happen: ids were checked when pushed, and the
                                                      // planner allocates nothing
    }
    if (tag) *tag = q.tag;
    if (T) *T = q.T;
    return SIDA_OK;
}

int sida_expert_prefetch(sida_ctx *c, const sida_plan *plan, int32_t wave, void *copy_stream)
{
    int rc = check_plan(c, plan);
    if (rc) return rc;
    if (wave < 0 || wave >= plan->n_waves) return SIDA_EINVAL;
    if (!c->pool || c->host_blocks.empty()) return SIDA_ESTATE;
    if (ids_mismatch_latched(c)) return SIDA_ESTATE;
    if (plan->first_wave + wave < c->prefetched_upto) return SIDA_OK;
    rc = prefetch_allowed(c, plan, wave);
    if (rc) return rc;
    rc = make_events(c);
    if (rc) return rc;
    return enqueue_prefetch(c, plan, wave, static_cast<hipStream_t>(copy_stream));
}

int sida_moe_layer_forward(sida_ctx *c, const sida_plan *plan, const void *x_dev, const int32_t *ids_dev,
                           const float *alpha_dev, void *y_dev, void *workspace_dev, size_t workspace_bytes,
                           void *compute_stream, void *copy_stream)
{
    if (!c || !plan) return SIDA_EINVAL;
    LayerArgs a{plan, x_dev, ids_dev, alpha_dev, y_dev};
    return forward_layers(c, 1, &a, workspace_dev, workspace_bytes, static_cast<hipStream_t>(compute_stream),
                          static_cast<hipStream_t>(copy_stream));
}

int sida_run_layers(sida_ctx *c, int32_t n, const sida_plan *const *plans, const void *const *x_dev,
                    const int32_t *const *ids_dev, const float *const *alpha_dev, void *const *y_dev,
                    void *workspace_dev, size_t workspace_bytes, void *compute_stream, void *copy_stream)
{
    if (!c || n < 0 || (n > 0 && (!plans || !x_dev || !ids_dev || !alpha_dev || !y_dev))) return SIDA_EINVAL;
    std::vector<LayerArgs> v;
    try {
        v.reserve(n);
    } catch (const std::bad_alloc &) {
        return SIDA_ENOMEM;
    }
    for (int32_t i = 0; i < n; ++i) {
        if (!plans[i]) return SIDA_EINVAL;
        v.push_back(LayerArgs{plans[i], x_dev[i], ids_dev[i], alpha_dev[i], y_dev[i]});
    }
    return forward_layers(c, n, v.data(), workspace_dev, workspace_bytes, static_cast<hipStream_t>(compute_stream),
                          static_cast<hipStream_t>(copy_stream));
}

int sida_dispatch(sida_ctx *c, const void *x_dev, const int32_t *ids_dev, int32_t T, void *workspace_dev,
                  size_t workspace_bytes, void *stream)
{
    if (!c || T < 0 || T > c->cfg.max_T || T % c->top_k) return SIDA_EINVAL;
    if (T == 0) return SIDA_OK;
    if (!x_dev || !ids_dev) return SIDA_EINVAL;
    int rc = check_ws(c, T, workspace_dev, workspace_bytes);
    if (rc) return rc;
    return launch_dispatch(c, x_dev, ids_dev, T, carve(c->cfg, T, workspace_dev), nullptr, static_cast<hipStream_t>(stream));
}

int sida_grouped_ffn(sida_ctx *c, const sida_plan *plan, int32_t wave, void *workspace_dev, size_t workspace_bytes,
                     void *stream)
{
    int rc = check_plan(c, plan);
    if (rc) return rc;
    if (wave < 0 || wave >= plan->n_waves) return SIDA_EINVAL;
    if (!c->pool) return SIDA_ESTATE;
    rc = check_ws(c, plan->T, workspace_dev, workspace_bytes);
    if (rc) return rc;
    LayerSchedule sched;
    build_schedule(plan, choose_tile_m(plan), &sched);
    const Ws ws = carve(c->cfg, plan->T, workspace_dev);
    rc = launch_tiles(c, sched, ws, static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_wave_ffn(c, sched, wave, ws, plan->T, static_cast<hipStream_t>(stream));
}

int sida_combine(sida_ctx *c, const float *alpha_dev, int32_t T, void *y_dev, void *workspace_dev,
                 size_t workspace_bytes, void *stream)
{
    if (!c || T < 0 || T > c->cfg.max_T || T % c->top_k) return SIDA_EINVAL;
    if (T == 0) return SIDA_OK;
    if (!alpha_dev || !y_dev) return SIDA_EINVAL;
    int rc = check_ws(c, T, workspace_dev, workspace_bytes);
    if (rc) return rc;
    const Ws ws = carve(c->cfg, T, workspace_dev);
    hipStream_t st = static_cast<hipStream_t>(stream);
    TimedKernel tk(c, SIDA_K_COMBINE);
    HIP_TRY(c, (hipError_t)launch_combine(ws.y_perm, ws.inv, alpha_dev, T, c->cfg.d_model, y_dev, st, tk.get(), c->top_k));
    return SIDA_OK;
}

// ---- hash function ---------------------------------------------------------------------------
namespace {
bool hash_cfg_ok(const sida_hash_config *h)
{
    return h && (h->C == 64 || h->C == 128) && h->d_model >= 8 && h->d_model <= 8192 && h->d_model % 8 == 0 && h->L >= 1 && h->E >= 1 &&
           h->E <= SIDA_MAX_E && (int64_t)h->L * h->E <= 8192 && h->top_k >= 1 && h->top_k <= SIDA_MAX_TOP_K &&
           h->top_k <= h->E && h->max_seq_len >= 1 && h->max_seq_len <= 4096;
}
}  // namespace

size_t sida_hash_param_count(const sida_hash_config *h)
{
    if (!hash_cfg_ok(h)) return 0;
    const size_t C = h->C;
    return C * h->d_model + C + 2 * (2 * 4 * C * C + 2 * 4 * C) + (size_t)h->L * h->E * C + (size_t)h->L * h->E;
}

size_t sida_hash_workspace_bytes(const sida_hash_config *h, int32_t n_tokens)
{
    if (!hash_cfg_ok(h) || n_tokens < 0) return 0;
    return sizeof(float) * 8 * (size_t)h->C * (size_t)n_tokens + 256;
}

int sida_hash_forward(const sida_hash_config *h, const float *params_dev, const void *x_dev, int32_t n_seq,
                      int32_t seq_len, int32_t *ids_dev, float *alpha_dev, void *workspace_dev, size_t workspace_bytes,
                      void *stream)
{
    if (!hash_cfg_ok(h) || n_seq < 0 || seq_len < 0 || seq_len > h->max_seq_len) return SIDA_EINVAL;
    if ((int64_t)n_seq * seq_len > INT32_MAX / 8) return SIDA_EINVAL;
    if (n_seq == 0 || seq_len == 0) return SIDA_OK;
    if (!params_dev || !x_dev || !ids_dev || !alpha_dev || !workspace_dev) return SIDA_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace_dev) & 255u) return SIDA_EINVAL;
    if (workspace_bytes < sida_hash_workspace_bytes(h, n_seq * seq_len)) return SIDA_ENOSPC;
    const HashShape sh{h->d_model, h->C, h->L, h->E, h->top_k};
    const int rc = launch_hash_forward(sh, params_dev, x_dev, n_seq, seq_len, ids_dev, alpha_dev,
                                       static_cast<float *>(workspace_dev), static_cast<hipStream_t>(stream));
    return rc == 0 ? SIDA_OK : SIDA_EHIP;
}

int sida_hash_forward_static(const sida_hash_config *h, const float *params_dev, const void *x_dev, int32_t n_seq,
                             int32_t seq_len, int32_t *ids_dev, float *alpha_dev, void *stream)
{
    static_assert(kHashStaticScratchBytes == SIDA_HASH_STATIC_SCRATCH_BYTES, "header and library agree on the limit");
    if (!hash_cfg_ok(h) || n_seq < 0 || seq_len < 0 || seq_len > h->max_seq_len) return SIDA_EINVAL;
    if ((int64_t)n_seq * seq_len > INT32_MAX / 8) return SIDA_EINVAL;
    if (n_seq == 0 || seq_len == 0) return SIDA_OK;
    if (!params_dev || !x_dev || !ids_dev || !alpha_dev) return SIDA_EINVAL;
    if (sida_hash_workspace_bytes(h, n_seq * seq_len) > kHashStaticScratchBytes) return SIDA_ENOSPC;
    float *ws = nullptr;
    if (hash_static_scratch(&ws) != 0) return SIDA_EHIP;
    const HashShape sh{h->d_model, h->C, h->L, h->E, h->top_k};
    // every intermediate is written before it is read: nothing in the scratch has to start at zero
    const int rc = launch_hash_forward(sh, params_dev, x_dev, n_seq, seq_len, ids_dev, alpha_dev, ws,
                                       static_cast<hipStream_t>(stream));
    return rc == 0 ? SIDA_OK : SIDA_EHIP;
}

int sida_tile_order(int32_t m_tiles, int32_t m_tall, int32_t n_tiles_n, int32_t long_rows, int32_t *token_tile,
                    int32_t *weight_tile)
{
    if (m_tiles < 0 || m_tall < 0 || m_tall > m_tiles || n_tiles_n < 1 || !token_tile || !weight_tile) return SIDA_EINVAL;
    if ((int64_t)m_tiles * n_tiles_n > INT32_MAX) return SIDA_EINVAL;
    const int gm = tile_group_height(m_tiles, m_tall, long_rows != 0), nw = tile_block_width(n_tiles_n, gm);
    for (int32_t t = 0; t < m_tiles * n_tiles_n; ++t) {
        int mt, nt;
        map_tile(t, m_tiles, m_tall, n_tiles_n, gm, nw, &mt, &nt);
        token_tile[t] = mt;
        weight_tile[t] = nt;
    }
    return SIDA_OK;
}

int sida_profile_enable(sida_ctx *c, int32_t on)
{
    if (!c) return SIDA_EINVAL;
    c->profiling = on != 0;
    return SIDA_OK;
}

int sida_profile_read(sida_ctx *c, double *ms, int64_t *launches, int32_t reset)
{
    if (!c) return SIDA_EINVAL;
    for (size_t i = 0; i < c->prof_used; ++i) {
        ProfRec &r = c->prof_pool[i];
        HIP_TRY(c, hipEventSynchronize(r.stop));
        float t = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&t, r.start, r.stop));
        c->prof_ms[r.klass] += t;
        c->prof_n[r.klass] += 1;
    }
    c->prof_used = 0;
    for (int k = 0; k < SIDA_K_COUNT; ++k) {
        if (ms) ms[k] = c->prof_ms[k];
        if (launches) launches[k] = c->prof_n[k];
        if (reset) {
            c->prof_ms[k] = 0;
            c->prof_n[k] = 0;
        }
    }
    return SIDA_OK;
}

}  // extern "C"
