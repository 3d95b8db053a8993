// Host-side tick scheduler (declared in flowcache_sched.h): a small state machine, no GPU
// calls.  Unit i is active at ticks [i*stagger, i*stagger + steps); the unit that takes its
// last step at a tick is committed after it, which moves the clean length along the two
// cache phases of App. C.1 (append while it fits the budget, compress to the budget after).
#include <cstring>

#include "flowcache_sched.h"

namespace {

constexpr uint32_t kMagic = 0x46435348u;   // "FCSH"

struct State {
    uint32_t magic;
    fc_sched_config cfg;
    int32_t window;
    int64_t tick;
    int64_t total;
    int32_t L_clean;
};

inline State* as_state(void* p) { return reinterpret_cast<State*>(p); }
inline const State* as_state(const void* p) { return reinterpret_cast<const State*>(p); }

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

size_t flowcache_sched_state_bytes(void) { return sizeof(State); }

int flowcache_sched_init(void* state, size_t state_bytes, const fc_sched_config* cfg) {
    if (!state || !cfg || state_bytes < sizeof(State)) return FC_INVALID_ARGUMENT;
    const fc_sched_config& c = *cfg;
    if (c.n_units < 1 || c.steps < 1 || c.stagger < 1 || c.stagger > c.steps || c.L_c < 1 ||
        c.budget < 0 || c.prefix_tokens < 0 || c.prefix_tokens > c.budget)
        return FC_INVALID_ARGUMENT;
    const int need = (c.steps + c.stagger - 1) / c.stagger;   // units that can overlap in time
    const int window = c.window == 0 ? need : c.window;
    if (window < need || window > FC_MAX_ACTIVE) return FC_INVALID_ARGUMENT;
    const int64_t cap = (int64_t)c.budget + c.L_c + (int64_t)window * c.L_c;
    if (cap > INT32_MAX) return FC_INVALID_ARGUMENT;
    State* s = as_state(state);
    std::memset(s, 0, sizeof(State));
    s->magic = kMagic;
    s->cfg = c;
    s->window = window;
    s->tick = 0;
    s->total = (int64_t)(c.n_units - 1) * c.stagger + c.steps;
    s->L_clean = c.prefix_tokens;
    return FC_OK;
}

int64_t flowcache_sched_capacity(const void* state) {
    const State* s = as_state(state);
    if (!s || s->magic != kMagic) return 0;
    return (int64_t)s->cfg.budget + s->cfg.L_c + (int64_t)s->window * s->cfg.L_c;
}

int64_t flowcache_sched_total_ticks(const void* state) {
    const State* s = as_state(state);
    if (!s || s->magic != kMagic) return 0;
    return s->total;
}

int flowcache_sched_next(void* state, fc_tick* out) {
    State* s = as_state(state);
    if (!s || !out || s->magic != kMagic) return FC_INVALID_ARGUMENT;
    if (s->tick >= s->total) return FC_SCHED_DONE;
    const fc_sched_config& c = s->cfg;
    const int64_t t = s->tick;
    fc_tick k;
    std::memset(&k, 0, sizeof(k));
    k.tick = (int32_t)t;
    // oldest unit still running: the first i with i*stagger + steps > t
    int64_t first = (t - c.steps + c.stagger) / c.stagger;   // ceil((t - steps + 1) / stagger)
    if (t - c.steps + 1 <= 0) first = 0;
    int64_t last = t / c.stagger;                             // newest unit already started
    if (last > c.n_units - 1) last = c.n_units - 1;
    const int32_t ring_base = c.budget + c.L_c;
    int A = 0;
    for (int64_t i = first; i <= last; ++i, ++A) {
        k.unit[A] = (int32_t)i;
        k.step_idx[A] = (int32_t)(t - i * c.stagger);
        k.active_off[A] = ring_base + (int32_t)(i % s->window) * c.L_c;
    }
    k.A = A;
    k.L_clean = s->L_clean;
    k.commit_unit = -1;
    k.L_clean_after = s->L_clean;
    if (A > 0 && k.step_idx[0] == c.steps - 1) {   // the oldest unit finishes with this tick
        k.commit_unit = k.unit[0];
        k.commit_src_off = k.active_off[0];
        k.commit_dst_off = s->L_clean;
        k.merged_len = s->L_clean + c.L_c;
        k.compress = k.merged_len > c.budget ? 1 : 0;
        k.L_clean_after = k.compress ? c.budget : k.merged_len;
    }
    s->L_clean = k.L_clean_after;
    s->tick = t + 1;
    *out = k;
    return FC_OK;
}

}  // extern "C"
#pragma GCC visibility pop
