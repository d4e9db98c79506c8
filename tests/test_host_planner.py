"""The library's host-side guard and tree flattening (C ABI, no GPU needed) against the Python oracle."""
import ctypes

import numpy as np
import pytest

from oracle import planner as op
from paper_2605_19893_amd import binding as B


def library_trace(cfg, expected, valid, observations):
    c = B.ssv_guard_default_config()
    c.alpha, c.ratio, c.warmup_steps, c.patience = cfg.alpha, cfg.ratio, cfg.warmup_steps, cfg.patience
    c.max_transitions, c.early_steps = cfg.max_transitions, cfg.early_steps
    state = B.ssv_guard_init(c, expected, valid)
    return [B.ssv_guard_observe(state, a, t) for a, t in observations], state


def test_default_config_holds_the_papers_constants():
    c = B.ssv_guard_default_config()
    d = op.GuardConfig()
    assert (c.alpha, c.ratio, c.warmup_steps, c.patience, c.max_transitions, c.early_steps) == \
           (d.alpha, d.ratio, d.warmup_steps, d.patience, d.max_transitions, d.early_steps)
    assert ctypes.sizeof(B.SsvGuardConfig) == 32 and ctypes.sizeof(B.SsvGuardState) == 32 + 8 * 4 + 8 + 16 * 8 + 32 + 2 * 16 * 8


@pytest.mark.parametrize("seed", range(12))
def test_guard_matches_the_oracle_on_random_requests(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 13))
    expected = np.sort(rng.uniform(2.0, 5.0, n))[::-1].tolist()
    valid = (rng.random(n) < 0.8).tolist()
    if not any(valid):
        valid[int(rng.integers(0, n))] = True
    cfg = op.GuardConfig(alpha=float(rng.choice([0.4, 0.25, 1.0])), ratio=float(rng.choice([0.85, 0.6])),
                         warmup_steps=int(rng.integers(0, 10)), patience=int(rng.integers(1, 7)),
                         max_transitions=int(rng.integers(0, 4)), early_steps=int(rng.choice([0, 0, 40])))
    # acceptance drifts below the expectation for a while, in steps of 1/8 (no near-ties with the thresholds)
    obs = [(float(rng.integers(8, 40)) / 8.0, float(rng.integers(1, 9)) / 4.0) for _ in range(120)]
    want = op.guard_trace(cfg, expected, valid, obs)
    got, state = library_trace(cfg, expected, valid, obs)
    assert got == want
    assert state.total_steps == 120 and state.transitions <= cfg.max_transitions


def test_guard_paper_constants_trace():
    got, state = library_trace(op.GuardConfig(), [4.0, 3.9, 3.8, 3.7], None, [(3.0, 1.0)] * 13 + [(3.0, 0.5)] * 13 + [(3.0, 2.0)] * 30)
    assert got[11] == 0 and got[12] == 1 and got[25] == 2 and got[37] == 2 and got[38] == 1 and got[-1] == 1
    assert state.settled == 1 and state.transitions == 2


def test_guard_rejects_bad_arguments():
    c = B.ssv_guard_default_config()
    with pytest.raises(B.SsvError):
        B.ssv_guard_init(c, [1.0] * 17)
    with pytest.raises(B.SsvError):
        B.ssv_guard_init(c, [])
    with pytest.raises(B.SsvError):
        B.ssv_guard_init(c, [1.0, 2.0], [False, False])
    c.alpha = 0.0
    with pytest.raises(B.SsvError):
        B.ssv_guard_init(c, [1.0])


@pytest.mark.parametrize("seed", range(8))
def test_tree_flatten_matches_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 65))
    parents = [-1] + [int(rng.integers(-1, i)) for i in range(1, n)]
    for order, name in ((B.SSV_TREE_BFS, "bfs"), (B.SSV_TREE_DFS, "dfs")):
        perm, newp = B.ssv_tree_flatten(parents, order)
        want_perm, want_newp = op.flatten_tree(parents, name)
        assert perm == want_perm and newp == want_newp


def test_tree_flatten_edge_cases():
    assert B.ssv_tree_flatten([], B.SSV_TREE_BFS) == ([], [])
    assert B.ssv_tree_flatten([-1], B.SSV_TREE_DFS) == ([0], [-1])
    chain = [-1, 0, 1, 2, 3]
    assert B.ssv_tree_flatten(chain, B.SSV_TREE_BFS) == (list(range(5)), chain)
    for bad in ([0], [-1, 1], [-1, -2], [-1, 5]):
        with pytest.raises(B.SsvError):
            B.ssv_tree_flatten(bad, B.SSV_TREE_BFS)
    with pytest.raises(B.SsvError):
        B.ssv_tree_flatten([-1, 0], 7)
