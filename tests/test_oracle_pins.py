"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test fixes one part of the oracle to a definition, closed form, invariant or
brute-force result, chosen so that a dropped term, wrong sign/index or transposed
operand in oracle/nsa_verify_oracle.c fails at least one of them.
"""
import json
import os

import numpy as np
import pytest

import ssv_inputs as si
from brute_force import brute_force_verify, dense_tree_attention

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")
TINY = si.NsaParams(l=8, d=4, l_sel=16, n_sel=4, w=8)


def tiny_case(seed, L=75, T=5, H=4, H_kv=2, d_k=8, d_v=6, nsa=TINY, dtype="f32", parents=None, B=1, **kw):
    seq = [L + 7 * b for b in range(B)]
    return si.make_case("tiny", dtype, B, T, H, H_kv, d_k, d_v, nsa, seq, seed, rho=kw.pop("rho", 0.3),
                        parents=parents, workers=1, **kw)


# ----------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed,L,T,n_sel,w,dtype", [
    (1, 40, 3, 3, 8, "f32"), (2, 75, 5, 4, 32, "f32"), (3, 130, 4, 4, 8, "bf16"),
    (4, 300, 5, 5, 32, "f32"), (5, 16, 5, 4, 8, "f32"), (6, 3, 4, 3, 8, "f32"), (7, 64, 1, 4, 16, "bf16"),
])
def test_matches_brute_force_chain(oracle, seed, L, T, n_sel, w, dtype):
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=n_sel, w=w)
    case = tiny_case(seed, L=L, T=T, nsa=nsa, dtype=dtype, B=2)
    r = oracle.nsa_verify(case, branches=True, want_imp=True)
    out, sel, br, imps = brute_force_verify(case)
    assert np.array_equal(sel, r.sel_idx)
    np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.stack([r.o_cmp, r.o_slc, r.o_win]), br, rtol=0, atol=1e-12)
    for (b, i, g), imp in imps.items():
        np.testing.assert_allclose(r.imp[b, i, g, :len(imp)], imp, rtol=0, atol=1e-12)


@pytest.mark.parametrize("order", ["bfs", "dfs"])
@pytest.mark.parametrize("fanouts,L", [((2, 2), 70), ((3, 1, 2), 129), ((1, 1, 1, 1), 50)])
def test_matches_brute_force_tree(oracle, order, fanouts, L):
    par = si.tree_parents(fanouts, order)
    case = tiny_case(11, L=L, T=len(par), parents=par, B=2)
    r = oracle.nsa_verify(case, branches=True)
    out, sel, br, _ = brute_force_verify(case)
    assert np.array_equal(sel, r.sel_idx)
    np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.stack([r.o_cmp, r.o_slc, r.o_win]), br, rtol=0, atol=1e-12)


def test_ragged_n_query_and_other_ratios(oracle):
    nsa = si.NsaParams(l=12, d=4, l_sel=8, n_sel=5, w=10, n_init=2, n_local=1)  # l/d = 3, l'/d = 2
    case = si.make_case("ragged", "f32", 3, 6, 6, 2, 8, 4, nsa, [50, 9, 121], 21, rho=0.5, n_query=[6, 2, 4],
                        workers=1)
    r = oracle.nsa_verify(case, branches=True)
    out, sel, br, _ = brute_force_verify(case)
    assert np.array_equal(sel, r.sel_idx)
    np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)
    assert np.all(r.out[1, 2:] == 0) and np.all(r.sel_idx[1, 2:] == -1)


# ----------------------------------------------------------------------------- invariant 1
@pytest.mark.parametrize("parents", [None, si.tree_parents((2, 2), "bfs"), si.tree_parents((2, 2), "dfs")])
def test_selected_and_window_reduce_to_dense_attention(oracle, parents):
    """Top-n >= number of blocks and window >= context: each raw-KV branch equals textbook
    causal (tree-masked) softmax attention."""
    T = 5 if parents is None else len(parents)
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=16, w=4096)
    case = tiny_case(31, L=90, T=T, nsa=nsa, parents=parents, B=2)
    r = oracle.nsa_verify(case, branches=True)
    dense = dense_tree_attention(case)
    np.testing.assert_allclose(r.o_slc, dense, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r.o_win, dense, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- invariant 2
def _decode_case(case, b, i, anc_path):
    """The T=1 autoregressive decode problem of query i: committed tokens are the prefix
    followed by i's proper ancestors (root first), the query is the only draft token."""
    L = int(case.seq_lens[b])
    m = len(anc_path) - 1
    nsa = case.nsa
    one = si.make_case("decode", case.dtype, 1, 1, case.H, case.H_kv, case.d_k, case.d_v, nsa, [L + m], 1, workers=1)
    slots = list(range(L)) + [L + t for t in anc_path]
    for src, dst in ((case.k, one.k), (case.v, one.v)):
        dst[0, :, :L + m + 1] = src[b][:, slots]
    one.q[0, 0] = case.q[b, i]
    one.gates[0, 0] = case.gates[b, i]
    nc = si.n_cmp_blocks(L + m + 1, nsa.l, nsa.d)
    one.n_cmp[0] = nc
    for h in range(case.H_kv):
        for src, dst in ((one.k, one.k_cmp), (one.v, one.v_cmp)):
            x = si.to_f32(src[0, h], case.dtype)
            dst[0, h, :nc] = si.to_storage(si._pool_slice(x, nc, nsa.l, nsa.d), case.dtype)
    return one


@pytest.mark.parametrize("L,T", [(75, 6), (61, 5), (128, 4)])
def test_each_chain_query_equals_single_query_decode(oracle, L, T):
    """Exact merged-schedule semantics (Section 4.2): every verifier query's output and indices
    equal running that query alone as an autoregressive decode step at its position."""
    case = tiny_case(41, L=L, T=T, B=2)
    r = oracle.nsa_verify(case)
    for b in range(case.B):
        for i in range(T):
            one = _decode_case(case, b, i, list(range(i + 1)))
            r1 = oracle.nsa_verify(one)
            assert np.array_equal(r1.sel_idx[0, 0], r.sel_idx[b, i])
            np.testing.assert_allclose(r1.out[0, 0], r.out[b, i], rtol=0, atol=1e-12)


def test_tree_query_equals_decode_on_its_path(oracle):
    """Trees, under the stated preconditions (all draft slots inside one selection block whose
    index does not change along the path, compressed cache built over the prefix only)."""
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=4, w=8)
    for order in ("bfs", "dfs"):
        par = si.tree_parents((2, 2, 1), order)
        case = tiny_case(43, L=96, T=len(par), parents=par, nsa=nsa)
        r = oracle.nsa_verify(case)
        for i in range(len(par)):
            path, t = [], i
            while t >= 0:
                path.append(t)
                t = int(par[t])
            path = path[::-1]
            one = _decode_case(case, 0, i, path)
            one.n_cmp[0] = case.n_cmp[0]          # deferred commit: compressed cache covers the prefix only
            one.k_cmp[0, :, :case.n_cmp[0]] = case.k_cmp[0, :, :case.n_cmp[0]]
            one.v_cmp[0, :, :case.n_cmp[0]] = case.v_cmp[0, :, :case.n_cmp[0]]
            r1 = oracle.nsa_verify(one)
            assert np.array_equal(r1.sel_idx[0, 0], r.sel_idx[0, i])
            np.testing.assert_allclose(r1.out[0, 0], r.out[0, i], rtol=0, atol=1e-12)


def test_tree_result_independent_of_flattening_order(oracle):
    """Same preconditions: all 20 draft slots lie in one selection block (l' = 32, L = 5 * 32)."""
    nsa = si.NsaParams(l=8, d=4, l_sel=32, n_sel=4, w=8)
    fan = (2, 3, 2)
    pb, pd = si.tree_parents(fan, "bfs"), si.tree_parents(fan, "dfs")
    cb = tiny_case(47, L=160, T=len(pb), parents=pb, nsa=nsa)
    # node identity = path of child ranks; map DFS index -> BFS index

    def paths(par):
        kids, out = {}, []
        for i, p in enumerate(par):
            rank = kids.setdefault(int(p), 0)
            kids[int(p)] = rank + 1
            out.append((out[p] if p >= 0 else ()) + (rank,))
        return out

    path_b, path_d = paths(pb), paths(pd)
    d2b = [path_b.index(pth) for pth in path_d]
    cd = tiny_case(47, L=160, T=len(pd), parents=pd, nsa=nsa)
    L = 160
    for arr_d, arr_b in ((cd.k, cb.k), (cd.v, cb.v)):
        arr_d[0, :, L:L + len(pd)] = arr_b[0, :, [L + t for t in d2b]].transpose(1, 0, 2)
    cd.q[0] = cb.q[0, d2b]
    cd.gates[0] = cb.gates[0, d2b]
    rb, rd = oracle.nsa_verify(cb), oracle.nsa_verify(cd)
    np.testing.assert_allclose(rd.out[0], rb.out[0, d2b], rtol=0, atol=1e-12)
    assert np.array_equal(rd.sel_idx[0], rb.sel_idx[0, d2b])


# ----------------------------------------------------------------------------- compressed branch
def test_compressed_branch_is_softmax_attention_over_visible_rows(oracle):
    case = tiny_case(51, L=77, T=4)
    r = oracle.nsa_verify(case, branches=True, want_p=True)
    nsa = case.nsa
    kc = case.k_cmp.astype(np.float64)
    vc = case.v_cmp.astype(np.float64)
    for i in range(4):
        n_vis = si.n_cmp_blocks(77 + i + 1, nsa.l, nsa.d)     # chain: complete blocks within pos(i)+1 tokens
        for h in range(case.H):
            g = h // case.H_g
            s = (kc[0, g, :n_vis] @ case.q[0, i, h].astype(np.float64)) / np.sqrt(case.d_k)
            p = np.exp(s - s.max())
            p /= p.sum()
            np.testing.assert_allclose(r.p_cmp[0, i, h, :n_vis], p, rtol=0, atol=1e-14)
            assert np.all(r.p_cmp[0, i, h, n_vis:] == 0)
            np.testing.assert_allclose(r.o_cmp[0, i, h], p @ vc[0, g, :n_vis], rtol=0, atol=1e-13)


def test_constant_keys_give_uniform_probabilities_and_mean_value(oracle):
    case = tiny_case(53, L=64, T=3)
    case.k_cmp[...] = 0.25
    r = oracle.nsa_verify(case, branches=True, want_p=True)
    for i in range(3):
        n_vis = si.n_cmp_blocks(64 + i + 1, case.nsa.l, case.nsa.d)
        np.testing.assert_allclose(r.p_cmp[0, i, :, :n_vis], 1.0 / n_vis, rtol=0, atol=1e-15)
        for h in range(case.H):
            mean = case.v_cmp[0, h // case.H_g, :n_vis].astype(np.float64).mean(axis=0)
            np.testing.assert_allclose(r.o_cmp[0, i, h], mean, rtol=0, atol=1e-14)


def test_no_visible_compressed_block_gives_zero(oracle):
    case = tiny_case(55, L=3, T=4)      # fewer than l = 8 visible tokens for every query
    r = oracle.nsa_verify(case, branches=True)
    assert np.all(r.o_cmp == 0)
    assert np.all(np.isfinite(r.out))


# ----------------------------------------------------------------------------- importance
@pytest.mark.parametrize("nsa", [TINY, si.NsaParams(l=12, d=4, l_sel=8, n_sel=5, w=10),
                                 si.NsaParams(l=32, d=16, l_sel=64, n_sel=4, w=16)])
def test_importance_sums_to_heads_times_l_over_d(oracle, nsa):
    """Every visible compression block covers l/d stride-d chunks, each inside a candidate
    selection block, and each head's probabilities sum to one."""
    case = tiny_case(61, L=333, T=4, nsa=nsa, H=6, H_kv=2)
    r = oracle.nsa_verify(case, want_imp=True)
    np.testing.assert_allclose(r.imp.sum(axis=-1), case.H_g * nsa.l / nsa.d, rtol=0, atol=1e-12)


def test_one_hot_probability_lands_on_the_overlapped_blocks(oracle):
    """A single dominant compression block c feeds only the selection blocks it overlaps:
    with l=32, d=16, l'=64 it covers chunks c and c+1, i.e. block c//4 twice, or blocks
    c//4 and c//4+1 once each when c % 4 == 3."""
    nsa = si.NsaParams(l=32, d=16, l_sel=64, n_sel=4, w=16)
    for c_star in (9, 11):
        case = tiny_case(63, L=512, T=1, H=2, H_kv=1, d_k=8, nsa=nsa)
        case.q[...] = 1.0
        case.k_cmp[...] = 0.0
        case.k_cmp[0, 0, c_star] = 40.0
        r = oracle.nsa_verify(case, want_imp=True)
        imp = r.imp[0, 0, 0]
        expect = np.zeros_like(imp)
        if c_star % 4 == 3:
            expect[c_star // 4] = expect[c_star // 4 + 1] = case.H_g
        else:
            expect[c_star // 4] = 2 * case.H_g
        np.testing.assert_allclose(imp, expect, rtol=0, atol=1e-9)


def test_head_permutation_inside_a_group_keeps_indices(oracle):
    case = tiny_case(65, L=200, T=4, H=8, H_kv=2)
    r = oracle.nsa_verify(case)
    perm = np.array([2, 0, 3, 1, 7, 6, 4, 5])
    case.q[...] = case.q[:, :, perm]
    case.gates[...] = case.gates[:, :, perm]
    r2 = oracle.nsa_verify(case)
    assert np.array_equal(r.sel_idx, r2.sel_idx)
    np.testing.assert_allclose(r2.out, r.out[:, :, perm], rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- selection
def test_planted_needles_are_selected(oracle):
    """Keys of a few blocks aligned with the (shared) query direction dominate the compressed
    scores, so exactly those blocks are selected next to the forced ones."""
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=6, w=8)
    case = tiny_case(71, L=400, T=3, H=4, H_kv=2, d_k=8, nsa=nsa)
    u = np.zeros(8, np.float32)
    u[0] = 1.0
    case.q[...] = 3.0 * u
    rng = np.random.default_rng(5)
    case.k[...] = (0.05 * rng.standard_normal(case.k.shape)).astype(np.float32)
    needles = [3, 11, 17]
    for j in needles:
        case.k[:, :, 16 * j:16 * j + 16] = 6.0 * u
    for h in range(case.H_kv):
        nc = int(case.n_cmp[0])
        case.k_cmp[0, h, :nc] = si._pool_slice(case.k[0, h], nc, nsa.l, nsa.d)
    r = oracle.nsa_verify(case)
    for i in range(3):
        J = (400 + i) // 16
        assert sorted(r.sel_idx[0, i, 0].tolist()) == sorted([0] + needles + [J - 1, J])
        assert r.gap[0, i, 0] > 0.1


def test_forced_blocks_and_adjacent_overlap_lower_bound(oracle):
    with open(GOLDEN) as f:
        gold = json.load(f)
    std = gold["nsa_standard"]
    assert (si.STD_NSA.l, si.STD_NSA.d, si.STD_NSA.l_sel, si.STD_NSA.n_sel, si.STD_NSA.w) == \
           (std["l"], std["d"], std["l_sel"], std["n_sel"], std["w"])
    assert (si.STD_NSA.n_init, si.STD_NSA.n_local) == (gold["forced_blocks"]["n_init"], gold["forced_blocks"]["n_local"])
    case = si.make_case("std", "f32", 1, 6, 4, 1, 16, 8, si.STD_NSA, [4096 + 5], 73, rho=0.0, workers=1)
    r = oracle.nsa_verify(case)
    for i in range(6):
        J = (4101 + i) // 64
        s = set(r.sel_idx[0, i, 0].tolist())
        assert {0, J - 1, J} <= s and len(s) == 16
        if i:
            assert len(s & set(r.sel_idx[0, i - 1, 0].tolist())) >= gold["min_adjacent_overlap_s"]


def test_fewer_candidates_than_n_selects_all_and_pads(oracle):
    case = tiny_case(75, L=20, T=3, nsa=si.NsaParams(l=8, d=4, l_sel=16, n_sel=6, w=8))
    r = oracle.nsa_verify(case)
    assert r.sel_idx[0, 0, 0].tolist() == [0, 1, -1, -1, -1, -1]
    assert np.all(np.isinf(r.gap))


def test_ties_go_to_the_smaller_index(oracle):
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=5, w=8)
    case = tiny_case(77, L=200, T=1, nsa=nsa)
    case.k_cmp[...] = 0.0                      # uniform p: interior blocks tie exactly
    r = oracle.nsa_verify(case, want_imp=True)
    J = 200 // 16
    imp = r.imp[0, 0, 0]
    assert np.all(imp[1:J - 1] == imp[1])      # block 0 lacks the c = -1 term, interior blocks are equal
    assert r.sel_idx[0, 0, 0].tolist() == [0, 1, 2, J - 1, J]
    assert r.gap[0, 0, 0] == 0.0


# ----------------------------------------------------------------------------- gates, reuse
def test_gates_select_and_scale_branches(oracle):
    case = tiny_case(81, L=90, T=3)
    r = oracle.nsa_verify(case, branches=True)
    for idx, branch in enumerate((r.o_cmp, r.o_slc, r.o_win)):
        case.gates[...] = 0.0
        case.gates[..., idx] = 1.0
        np.testing.assert_allclose(oracle.nsa_verify(case).out, branch, rtol=0, atol=0)
    case.gates[...] = 0.0
    assert np.all(oracle.nsa_verify(case).out == 0)
    case.gates[...] = [0.5, 0.25, 2.0]
    np.testing.assert_allclose(oracle.nsa_verify(case).out, 0.5 * r.o_cmp + 0.25 * r.o_slc + 2.0 * r.o_win,
                               rtol=0, atol=1e-13)


def test_reuse_mode(oracle):
    case = tiny_case(83, L=150, T=4)
    r = oracle.nsa_verify(case)
    again = oracle.nsa_verify(case, sel_idx=r.sel_idx)
    np.testing.assert_allclose(again.out, r.out, rtol=0, atol=0)
    # negative, repeated, out-of-range entries are ignored; order does not matter
    messy = r.sel_idx[..., ::-1].copy()
    wide = np.concatenate([messy, messy[..., :1], np.full_like(messy[..., :1], 10 ** 6)], axis=-1)
    case6 = tiny_case(83, L=150, T=4, nsa=si.NsaParams(l=8, d=4, l_sel=16, n_sel=6, w=8))
    r6 = oracle.nsa_verify(case6, sel_idx=wide)
    np.testing.assert_allclose(r6.out, r.out, rtol=0, atol=0)
    out_bf, _, _, _ = brute_force_verify(case6, sel_idx=wide)
    np.testing.assert_allclose(r6.out, out_bf, rtol=0, atol=1e-12)
    # blocks beyond the query's own block contribute nothing: all their tokens are invisible
    far = r.sel_idx.copy()
    far[:, 0, :, 0] = (150 + 3) // 16 + 0      # block of the last draft slot, not visible to query 0
    if (150 + 3) // 16 > 150 // 16:
        base = far.copy()
        base[:, 0, :, 0] = -1
        np.testing.assert_allclose(oracle.nsa_verify(case, sel_idx=far).out,
                                   oracle.nsa_verify(case, sel_idx=base).out, rtol=0, atol=0)


def test_window_is_exactly_w_positions_including_self(oracle):
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=4, w=5)
    case = tiny_case(85, L=50, T=3, nsa=nsa, H=2, H_kv=1)
    r = oracle.nsa_verify(case, branches=True)
    k, v, q = (a.astype(np.float64) for a in (case.k, case.v, case.q))
    for i in range(3):
        pos = 50 + i
        idx = np.arange(pos - 4, pos + 1)
        for h in range(2):
            s = (k[0, 0, idx] @ q[0, i, h]) / np.sqrt(case.d_k)
            p = np.exp(s - s.max())
            p /= p.sum()
            np.testing.assert_allclose(r.o_win[0, i, h], p @ v[0, 0, idx], rtol=0, atol=1e-13)


def test_query_mask_computes_only_requested_rows(oracle):
    case = tiny_case(87, L=90, T=4, B=2)
    full = oracle.nsa_verify(case)
    mask = np.zeros((2, 4), np.uint8)
    mask[1, 2] = 1
    part = oracle.nsa_verify(case, query_mask=mask)
    np.testing.assert_allclose(part.out[1, 2], full.out[1, 2], rtol=0, atol=0)
    assert np.all(part.out[0] == 0) and np.all(part.sel_idx[0] == -1)


def test_bf16_inputs_are_read_exactly(oracle):
    case = tiny_case(89, L=70, T=2, dtype="bf16")
    as_f32 = si.make_case("x", "f32", 1, 2, 4, 2, 8, 6, TINY, [70], 89, rho=0.3, workers=1)
    for name in ("q", "k", "v", "k_cmp", "v_cmp"):
        getattr(as_f32, name)[...] = si.bf16_bits_to_f32(getattr(case, name))
    as_f32.gates[...] = case.gates
    np.testing.assert_allclose(oracle.nsa_verify(case).out, oracle.nsa_verify(as_f32).out, rtol=0, atol=0)


def test_more_than_64_verifier_queries_match_brute_force(oracle):
    """Draft budgets beyond one machine word of ancestor bits: a 70-token chain and a 78-node tree."""
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=4, w=24)
    chain = tiny_case(91, L=90, T=70, nsa=nsa, H=2, H_kv=1)
    r = oracle.nsa_verify(chain, branches=True)
    out, sel, br, _ = brute_force_verify(chain)
    assert np.array_equal(sel, r.sel_idx)
    np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)
    par = si.tree_parents((2, 2, 3, 2), "dfs")       # 2 + 4 + 12 + 24 = 42 ... extended below
    par = np.concatenate([par, par[:36] + np.where(par[:36] >= 0, len(par), 0)]).astype(np.int32)   # a second copy of a subtree
    tree = tiny_case(93, L=75, T=len(par), nsa=nsa, H=2, H_kv=1, parents=par)
    r = oracle.nsa_verify(tree, branches=True)
    out, sel, br, _ = brute_force_verify(tree)
    assert len(par) > 64 and np.array_equal(sel, r.sel_idx)
    np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)
