// Host-side residency planner: Algorithm 1's inference-thread loop (check every token's expert,
// load it when it is not on the GPU) under the memory budget of Section 3.1 / Section 4.3, with
// first-in-first-out replacement as in the paper or one of the other strategies its footnote
// allows (least recently used; farthest next use in the future the hash-table queue exposes).
// Integers only; no HIP calls.
#include <cstring>

#include "ctx.h"

namespace sida {

namespace {

constexpr int64_t kNever = int64_t(1) << 60;

}  // namespace

int plan_layer(sida_ctx *c, int32_t layer, const int32_t *ids, int32_t T, const int32_t *future,
               int64_t n_future, sida_plan *out)
{
    const int32_t E = c->cfg.E, S = c->cfg.S, W = c->cfg.W;
    const int32_t n_keys = c->cfg.L * E;

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
    for (int64_t j = 0; j < n_future; ++j)
        if (future[j] < 0 || future[j] >= n_keys) return SIDA_EINVAL;
    for (int e = 0; e < E; ++e) p.offsets[e + 1] = p.offsets[e] + p.counts[e];
    if (p.n_active == 0) {
        *out = p;
        return SIDA_OK;
    }

    // Farthest-next-use replacement: position of every key's next use.  The experts of this layer
    // that are still to be placed come first (in placement order), then the caller's future.
    const bool belady = c->policy == SIDA_POLICY_BELADY;
    std::vector<int64_t> &later = c->next_use;        // [L*E] first position in `future`
    int32_t place[SIDA_MAX_E];                        // position of expert e in this layer's order
    if (belady) {
        later.assign((size_t)n_keys, kNever);
        for (int64_t j = n_future - 1; j >= 0; --j) later[future[j]] = j;
        for (int e = 0; e < E; ++e) place[e] = -1;
        for (int32_t i = 0; i < p.n_active; ++i) place[p.order[i]] = i;
    }
    auto next_use = [&](int32_t key, int32_t i) -> int64_t {
        if (key / E == layer && place[key % E] > i) return place[key % E] - i;
        return later[key] == kNever ? kNever : p.n_active + later[key];
    };

    // Everything below works on the context's vectors directly and allocates nothing: it cannot fail.
    int32_t g = c->next_wave;
    p.first_wave = g;
    int32_t in_wave = 0;              // experts already placed in wave g
    std::vector<int32_t> &used = c->wave_mark;   // [S], sized when the context was made:
    std::fill(used.begin(), used.end(), -1);     // used[s] == g  <=>  slot s belongs to the current wave
    int32_t dep = -1;
    auto close_wave = [&]() {
        p.wave_dep[g - p.first_wave] = dep;
        ++g;
        in_wave = 0;
        dep = -1;
    };
    // Slot to overwrite for expert number i of the layer (policies other than first-in-first-out):
    // an empty slot if there is one, else by policy; never a slot of the wave being assembled.
    auto victim = [&](int32_t i) {
        int32_t best = -1;
        for (int32_t s = 0; s < S; ++s) {
            if (used[s] == g) continue;
            if (c->slot_key[s] < 0) return s;
            if (best < 0) {
                best = s;
                continue;
            }
            if (belady) {
                const int64_t a = next_use(c->slot_key[s], i), b = next_use(c->slot_key[best], i);
                if (a > b || (a == b && c->loaded_at[s] < c->loaded_at[best])) best = s;
            } else if (c->touched_at[s] < c->touched_at[best]) {
                best = s;
            }
        }
        return best;
    };

    for (int32_t i = 0; i < p.n_active; ++i) {
        const int32_t e = p.order[i];
        const int32_t key = layer * E + e;
        int32_t s = c->key_slot[key];
        if (s >= 0) {                               // resident: nothing to copy
            if (in_wave == W) close_wave();
            p.hit[e] = 1;
        } else {                                    // not resident: overwrite a slot
            if (c->policy == SIDA_POLICY_FIFO) {    // the oldest load (a hit does not renew an age)
                if (in_wave == W || used[c->cursor] == g) close_wave();
                s = c->cursor;
                c->cursor = (s + 1 == S) ? 0 : s + 1;
            } else {
                if (in_wave == W) close_wave();
                s = victim(i);
                if (s < 0) {                        // every slot belongs to this wave
                    close_wave();
                    s = victim(i);
                }
            }
            const int32_t old = c->slot_key[s];
            p.evicted_key[e] = old;
            if (old >= 0) c->key_slot[old] = -1;
            c->slot_key[s] = key;
            c->key_slot[key] = s;
            c->loaded_at[s] = c->clock;
            if (c->last_use[s] > dep) dep = c->last_use[s];
            p.hit[e] = 0;
            ++p.n_miss;
        }
        c->touched_at[s] = c->clock++;
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
