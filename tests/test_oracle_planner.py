"""Pins of the planner-guard and tree-flattening oracle (CPU only): hand-worked traces from the constants the
paper states, closed forms of the smoothing, and structural properties of the two traversal orders."""
import json
import os

import numpy as np
import pytest

import ssv_inputs as si
from oracle import planner as op

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")


def paper_cfg(**over):
    with open(GOLDEN) as f:
        g = json.load(f)["runtime_guard"]
    cfg = op.GuardConfig(alpha=g["alpha"], ratio=g["ratio"], warmup_steps=g["warmup_steps"], patience=g["patience"],
                         max_transitions=g["max_transitions"])
    for k, v in over.items():
        setattr(cfg, k, v)
    return cfg


def test_defaults_are_the_papers_constants():
    assert op.GuardConfig() == paper_cfg()


def test_constant_shortfall_switches_after_warmup_plus_patience():
    # expectation 4.0 -> threshold 3.4; a constant 3.0 keeps the smoothed value at 3.0: steps 1-8 warm up,
    # steps 9-13 are the five consecutive misses, so step 13 is the first one on the next strategy
    trace = op.guard_trace(paper_cfg(), [4.0, 3.9, 3.8], None, [(3.0, 1.0)] * 30)
    assert trace[:12] == [0] * 12 and trace[12] == 1
    # the second strategy needs its own 13 steps (steps 14..26): step 26 moves to the third
    assert trace[12:25] == [1] * 13 and trace[25] == 2
    # just above the threshold nothing ever happens
    assert set(op.guard_trace(paper_cfg(), [4.0, 3.9], None, [(3.41, 1.0)] * 60)) == {0}


def test_smoothed_value_follows_the_geometric_closed_form():
    # A_1 = 10, then 0 forever: smoothed value = 10 * 0.6^(t-1); expectation 1.0 -> below 0.85 from t = 6 on
    # (10 * 0.6^5 = 0.78), but counting starts after the warm-up: misses at steps 9..13
    trace = op.guard_trace(paper_cfg(), [1.0, 1.0], None, [(10.0, 1.0)] + [(0.0, 1.0)] * 20)
    assert trace.index(1) == 12
    # with a 2-step warm-up the count starts at step 3 but the value is still high there:
    # 10 * 0.6^(t-1) < 0.85 first at t = 6, so misses are steps 6..10
    trace = op.guard_trace(paper_cfg(warmup_steps=2), [1.0, 1.0], None, [(10.0, 1.0)] + [(0.0, 1.0)] * 20)
    assert trace.index(1) == 9
    # a single good step among the misses restarts the count (smoothed value jumps above the threshold)
    obs = [(3.0, 1.0)] * 11 + [(9.0, 1.0)] + [(3.0, 1.0)] * 30
    trace = op.guard_trace(paper_cfg(), [4.0, 4.0], None, obs)
    # after the 9.0 the smoothed value is 5.4, then 3 + 2.4 * 0.6^k: below 3.4 from k = 4 (0.311) on -> steps 16..20
    assert trace.index(1) == 19


def test_at_most_two_transitions_then_the_best_explored_strategy():
    # every strategy disappoints; latencies make the second one the best accepted-tokens-per-time of the run
    exp = [4.0, 4.0, 4.0, 4.0]
    obs = [(3.0, 1.0)] * 13 + [(3.0, 0.5)] * 13 + [(3.0, 2.0)] * 30
    trace = op.guard_trace(paper_cfg(), exp, None, obs)
    assert trace[12] == 1 and trace[25] == 2
    assert max(trace) == 2                      # never a third move
    assert trace[38] == 1 and set(trace[38:]) == {1}   # settled on the best explored one
    # invalid candidates are skipped by both the initial choice and the moves
    trace = op.guard_trace(paper_cfg(), exp, [False, True, False, True], [(3.0, 1.0)] * 14)
    assert trace[0] == 1 and trace[12] == 3
    # nothing left to move to: settle where we are
    trace = op.guard_trace(paper_cfg(), [4.0], None, [(3.0, 1.0)] * 40)
    assert set(trace) == {0}


def test_refinement_window_closes():
    trace = op.guard_trace(paper_cfg(early_steps=12), [4.0, 4.0], None, [(3.0, 1.0)] * 40)
    assert set(trace) == {0}
    trace = op.guard_trace(paper_cfg(early_steps=13), [4.0, 4.0], None, [(3.0, 1.0)] * 40)
    assert trace[12] == 1 and set(trace[13:]) == {1}


# ----------------------------------------------------------------------------- tree flattening
def depths(parents):
    d = []
    for i, p in enumerate(parents):
        d.append(0 if p < 0 else d[p] + 1)
    return d


def canonical_paths(parents):
    """Root-to-node paths as tuples of sibling ranks: identifies a node independently of the numbering."""
    kids, path = {}, []
    for i, p in enumerate(parents):
        rank = kids.setdefault(p, 0)
        kids[p] = rank + 1
        path.append((rank,) if p < 0 else path[p] + (rank,))
    return path


def test_hand_worked_tree():
    #        -1
    #      0     3
    #    1  2      4
    #              5
    parents = [-1, 0, 0, -1, 3, 4]
    perm, new_par = op.flatten_tree(parents, "bfs")
    assert perm == [0, 3, 1, 2, 4, 5] and new_par == [-1, -1, 0, 0, 1, 4]
    perm, new_par = op.flatten_tree(parents, "dfs")
    assert perm == [0, 1, 2, 3, 4, 5] and new_par == parents


@pytest.mark.parametrize("seed", range(6))
def test_orders_have_their_defining_properties(seed):
    rng = np.random.default_rng(seed)
    n = 40
    parents = [-1] + [int(rng.integers(-1, i)) for i in range(1, n)]
    paths = canonical_paths(parents)
    for order in ("bfs", "dfs"):
        perm, new_par = op.flatten_tree(parents, order)
        assert sorted(perm) == list(range(n))
        assert all(-1 <= p < i for i, p in enumerate(new_par))            # still topological
        new_paths = canonical_paths(new_par)
        assert [paths[old] for old in perm] == new_paths                   # same tree, children in the same order
        d = depths(new_par)
        if order == "bfs":
            assert d == sorted(d)                                          # level by level
            assert new_paths == sorted(new_paths, key=lambda t: (len(t), t))
        else:
            assert new_paths == sorted(new_paths)                          # pre-order = lexicographic order of paths
            for i, p in enumerate(new_par):                                # every subtree is one contiguous run
                if i + 1 < n and new_par[i + 1] not in (-1,) and new_par[i + 1] != i:
                    assert new_par[i + 1] < i
    # the two orders are re-flattenings of each other
    pb, parb = op.flatten_tree(parents, "bfs")
    _, pard = op.flatten_tree(parents, "dfs")
    assert op.flatten_tree(parb, "dfs")[1] == pard


def test_agrees_with_the_seeded_tree_generator():
    for fan in ((4, 3, 2), (2, 2, 2, 2), (3, 1, 2)):
        bfs, dfs = si.tree_parents(fan, "bfs").tolist(), si.tree_parents(fan, "dfs").tolist()
        assert op.flatten_tree(bfs, "dfs")[1] == dfs
        assert op.flatten_tree(dfs, "bfs")[1] == bfs
        assert op.flatten_tree(bfs, "bfs")[0] == list(range(len(bfs)))
