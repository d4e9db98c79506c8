// Host-side pieces around the verification kernel: the runtime guard that refines the profile-selected strategy
// during the early verification steps (Section 6.3, Algorithm 1) and the flattening of a draft tree into the
// verifier batch in BFS (siblings adjacent) or DFS (parent/child adjacent) order (Section 4.1).  No GPU work.
#pragma once
#include <cstring>
#include <vector>

#include "../../include/ssv_nsa.h"

namespace ssv {

inline void guard_restart_strategy(ssv_guard_state* s) {
    s->has_ema = 0;
    s->ema = 0.0;
    s->steps_on_active = 0;
    s->below_streak = 0;
}

inline int guard_init(ssv_guard_state* s, const ssv_guard_config* cfg, const double* expected, const uint8_t* valid, int n) {
    if (!s || !cfg || !expected || n < 1 || n > SSV_GUARD_MAX_CANDIDATES) return SSV_EINVAL;
    if (!(cfg->alpha > 0.0 && cfg->alpha <= 1.0) || !(cfg->ratio >= 0.0) || cfg->warmup_steps < 0 || cfg->patience < 1 ||
        cfg->max_transitions < 0 || cfg->early_steps < 0)
        return SSV_EINVAL;
    std::memset(s, 0, sizeof(*s));
    s->cfg = *cfg;
    s->n_candidates = n;
    s->active = -1;
    for (int i = 0; i < n; ++i) {
        s->expected[i] = expected[i];
        s->valid[i] = valid ? (valid[i] != 0) : 1;
        if (s->active < 0 && s->valid[i]) s->active = i;      // preselection: the best-ranked valid strategy
    }
    if (s->active < 0) return SSV_EINVAL;
    s->explored[s->active] = 1;
    guard_restart_strategy(s);
    return SSV_OK;
}

inline int guard_observe(ssv_guard_state* s, double accepted, double latency) {
    if (!s || s->n_candidates < 1 || s->active < 0 || s->active >= s->n_candidates) return SSV_EINVAL;
    const ssv_guard_config& c = s->cfg;
    s->total_steps += 1;
    s->sum_accepted[s->active] += accepted;
    s->sum_latency[s->active] += latency;
    const bool in_window = c.early_steps == 0 || s->total_steps <= c.early_steps;
    if (s->settled || !in_window) return s->active;
    s->steps_on_active += 1;
    s->ema = s->has_ema ? c.alpha * accepted + (1.0 - c.alpha) * s->ema : accepted;
    s->has_ema = 1;
    if (s->steps_on_active <= c.warmup_steps) return s->active;
    s->below_streak = (s->ema < c.ratio * s->expected[s->active]) ? s->below_streak + 1 : 0;
    if (s->below_streak < c.patience) return s->active;
    int next = -1;
    if (s->transitions < c.max_transitions)
        for (int i = s->active + 1; i < s->n_candidates; ++i)
            if (s->valid[i]) { next = i; break; }
    if (next >= 0) {
        s->active = next;
        s->explored[next] = 1;
        s->transitions += 1;
        guard_restart_strategy(s);
    } else {
        // the mismatch persists and no move is left: settle on the best strategy explored in this run
        int best = s->active;
        double best_rate = -1.0;
        for (int i = 0; i < s->n_candidates; ++i)
            if (s->explored[i] && s->sum_latency[i] > 0.0) {
                const double rate = s->sum_accepted[i] / s->sum_latency[i];
                if (rate > best_rate) { best = i; best_rate = rate; }
            }
        s->active = best;
        s->settled = 1;
    }
    return s->active;
}

inline int tree_flatten(const int32_t* parents, int n, int order, int32_t* perm, int32_t* new_parents) {
    if (!parents || !perm || !new_parents || n < 0 || (order != SSV_TREE_BFS && order != SSV_TREE_DFS)) return SSV_EINVAL;
    for (int i = 0; i < n; ++i)
        if (parents[i] < -1 || parents[i] >= i) return SSV_EINVAL;
    // children lists in original order: first child and next sibling (index n stands for the root -1)
    std::vector<int32_t> first(n + 1, -1), last(n + 1, -1), next(n, -1);
    for (int i = 0; i < n; ++i) {
        const int p = parents[i] < 0 ? n : parents[i];
        if (first[p] < 0) first[p] = i; else next[last[p]] = i;
        last[p] = i;
    }
    int out = 0;
    if (order == SSV_TREE_BFS) {
        // perm doubles as the queue: nodes are appended level by level
        for (int c = first[n]; c >= 0; c = next[c]) perm[out++] = c;
        for (int head = 0; head < out; ++head)
            for (int c = first[perm[head]]; c >= 0; c = next[c]) perm[out++] = c;
    } else {
        // pre-order without recursion: after a node comes its first child, else the next sibling of the nearest
        // ancestor-or-self that has one
        int node = first[n];
        while (node >= 0) {
            perm[out++] = node;
            if (first[node] >= 0) { node = first[node]; continue; }
            while (node >= 0 && next[node] < 0) node = parents[node];
            if (node >= 0) node = next[node];
        }
    }
    if (out != n) return SSV_EINVAL;
    std::vector<int32_t> new_of(n);
    for (int i = 0; i < n; ++i) new_of[perm[i]] = i;
    for (int i = 0; i < n; ++i) new_parents[i] = parents[perm[i]] < 0 ? -1 : new_of[parents[perm[i]]];
    return SSV_OK;
}

}  // namespace ssv
