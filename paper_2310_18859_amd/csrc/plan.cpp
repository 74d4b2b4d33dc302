// Host-side residency planner: Algorithm 1's inference-thread loop (check every token's expert,
// load it when it is not on the GPU) under the FIFO memory budget of Section 3.1 / Section 4.3.
// Integers only; no HIP calls.
#include <cstring>

#include "ctx.h"

namespace sida {

int plan_layer(sida_ctx *c, int32_t layer, const int32_t *ids, int32_t T, sida_plan *out)
{
    const int32_t E = c->cfg.E, S = c->cfg.S, W = c->cfg.W;

    sida_plan p;
    std::memset(&p, 0, sizeof p);
    p.layer = layer;
    p.T = T;
    p.E = E;
    p.epoch = c->epoch;
    p.first_wave = -1;
    for (int e = 0; e < SIDA_MAX_E; ++e) {
        p.slot[e] = p.wave[e] = p.hit[e] = p.evicted_key[e] = -1;
        p.order[e] = -1;
        p.wave_dep[e] = -1;
    }

    // One pass over the tokens: histogram, and the experts in order of first appearance.
    for (int32_t t = 0; t < T; ++t) {
        const int32_t k = ids[t];
        if (k < 0 || k >= E) return SIDA_EINVAL;
        if (p.counts[k]++ == 0) p.order[p.n_active++] = k;
    }
    for (int e = 0; e < E; ++e) p.offsets[e + 1] = p.offsets[e] + p.counts[e];
    if (p.n_active == 0) {
        *out = p;
        return SIDA_OK;
    }

    // Everything below works on the context's vectors directly; nothing can fail from here on.
    int32_t g = c->next_wave;
    p.first_wave = g;
    int32_t in_wave = 0;              // experts already placed in wave g
    std::vector<int32_t> used(S, -1); // used[s] == g  <=>  slot s belongs to the current wave
    int32_t dep = -1;
    auto close_wave = [&]() {
        p.wave_dep[g - p.first_wave] = dep;
        ++g;
        in_wave = 0;
        dep = -1;
    };

    for (int32_t i = 0; i < p.n_active; ++i) {
        const int32_t e = p.order[i];
        const int32_t key = layer * E + e;
        int32_t s = c->key_slot[key];
        if (s >= 0) {                               // resident: nothing to copy, age unchanged
            if (in_wave == W) close_wave();
            p.hit[e] = 1;
        } else {                                    // not resident: overwrite the oldest load
            if (in_wave == W || used[c->cursor] == g) close_wave();
            s = c->cursor;
            const int32_t old = c->slot_key[s];
            p.evicted_key[e] = old;
            if (old >= 0) c->key_slot[old] = -1;
            c->slot_key[s] = key;
            c->key_slot[key] = s;
            c->cursor = (s + 1 == S) ? 0 : s + 1;
            if (c->last_use[s] > dep) dep = c->last_use[s];
            p.hit[e] = 0;
            ++p.n_miss;
        }
        p.slot[e] = s;
        p.wave[e] = g;
        used[s] = g;
        c->last_use[s] = g;
        ++in_wave;
    }
    close_wave();                                   // a layer never shares a wave with the next
    p.n_waves = g - p.first_wave;
    c->next_wave = g;
    *out = p;
    return SIDA_OK;
}

}  // namespace sida
