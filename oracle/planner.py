"""TEST INFRASTRUCTURE: plain Python statement of the host-side pieces around the verification kernel:
the runtime guard that refines the profile-selected strategy (Section 6.3, Algorithm 1) and the
flattening of a draft tree into the verifier batch in BFS or DFS order (Section 4.1).
Only tests may import it; it shares nothing with the library.

Guard, as the paper states it: smooth the accepted-token counts A_t with coefficient alpha; after a
warm-up, if the smoothed value stays below ratio x (profiled expectation of the active strategy) for
`patience` consecutive steps, move to the next-ranked valid strategy of the profile; at most
`max_transitions` moves per request; if the mismatch persists after the last move, settle on the best
strategy explored in this run.  Constants of the paper: alpha 0.40, warm-up 8, ratio 0.85, patience 5, two moves.

Readings where the paper is silent: the smoothed value starts at the first observation of a strategy;
warm-up steps update it but are not counted; a move restarts smoothing, warm-up and the count for the new
strategy; "best explored" is the largest accepted tokens per unit latency (sum A / sum T) over the steps each
explored strategy ran, ties to the better-ranked; refinement stops after `early_steps` steps (0 = never)
and once settled.
"""
from __future__ import annotations

from dataclasses import dataclass


@dataclass
class GuardConfig:
    alpha: float = 0.40
    ratio: float = 0.85
    warmup_steps: int = 8
    patience: int = 5
    max_transitions: int = 2
    early_steps: int = 0


def guard_trace(cfg: GuardConfig, expected, valid, observations):
    """Active strategy index after every observation (A_t, T_t); expected[i] = profiled E[A] of candidate i,
    candidates ranked best first; valid[i] = whether candidate i may be used."""
    n = len(expected)
    ranked = [i for i in range(n) if valid is None or valid[i]]
    assert ranked, "no valid strategy"
    pos = 0                      # position in `ranked`
    active = ranked[pos]
    ema, steps_on_active, below, transitions, settled = None, 0, 0, 0, False
    total = 0
    sums = {active: [0.0, 0.0]}
    out = []
    for A, T in observations:
        total += 1
        sums[active][0] += A
        sums[active][1] += T
        if not settled and (cfg.early_steps == 0 or total <= cfg.early_steps):
            steps_on_active += 1
            ema = A if ema is None else cfg.alpha * A + (1.0 - cfg.alpha) * ema
            if steps_on_active > cfg.warmup_steps:
                below = below + 1 if ema < cfg.ratio * expected[active] else 0
                if below >= cfg.patience:
                    if transitions < cfg.max_transitions and pos + 1 < len(ranked):
                        pos += 1
                        transitions += 1
                        active = ranked[pos]
                        sums.setdefault(active, [0.0, 0.0])
                        ema, steps_on_active, below = None, 0, 0
                    else:
                        best, best_rate = None, -1.0
                        for cand in ranked:          # rank order: ties go to the better-ranked
                            if cand in sums and sums[cand][1] > 0 and sums[cand][0] / sums[cand][1] > best_rate:
                                best, best_rate = cand, sums[cand][0] / sums[cand][1]
                        active = best if best is not None else active
                        settled = True
        out.append(active)
    return out


def flatten_tree(parents, order: str):
    """Reorder a draft tree (parents[i] in {-1, 0..i-1}; -1 = child of the last committed token) into the
    flattened verifier batch.  BFS: level by level, so siblings are adjacent; DFS: pre-order, so a node is
    followed by its first child's subtree.  Children keep their original relative order.
    Returns (perm, new_parents): perm[new] = old index; new_parents in the new numbering."""
    n = len(parents)
    children = {i: [] for i in range(-1, n)}
    for i, p in enumerate(parents):
        assert -1 <= p < i
        children[p].append(i)
    perm = []
    if order == "bfs":
        frontier = list(children[-1])
        while frontier:
            perm.extend(frontier)
            frontier = [c for node in frontier for c in children[node]]
    elif order == "dfs":
        def visit(node):
            perm.append(node)
            for c in children[node]:
                visit(c)
        for root in children[-1]:
            visit(root)
    else:
        raise ValueError(order)
    new_of = {old: new for new, old in enumerate(perm)}
    new_parents = [-1 if parents[old] < 0 else new_of[parents[old]] for old in perm]
    return perm, new_parents
