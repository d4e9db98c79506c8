"""Pins of the oracle's approximate shared-index variant (Section 4.3) against brute force, the exact
variant and the cases where the approximation vanishes (CPU only)."""
import numpy as np
import pytest

import ssv_inputs as si
from brute_force import brute_force_verify, tree_info
from test_oracle_pins import TINY, tiny_case


def brute_force_shared(case, C):
    """Independent restatement: exact brute-force selection, the deepest (then latest) member of every run of
    C queries lends its set to the whole run, brute-force attention with those sets."""
    _, sel_exact, _, _ = brute_force_verify(case)
    shared = np.full_like(sel_exact, -1)
    for b in range(case.B):
        Tq = int(case.n_query[b])
        parents = case.parents[b] if case.parents is not None else si.chain_parents(case.T)
        depth, _ = tree_info(parents, Tq)
        for start in range(0, Tq, C):
            stop = min(start + C, Tq)
            rep = start
            for i in range(start, stop):
                if depth[i] >= depth[rep]:
                    rep = i
            shared[b, start:stop] = sel_exact[b, rep]
    out, _, branches, _ = brute_force_verify(case, sel_idx=shared)
    return out, shared, branches


@pytest.mark.parametrize("C", [2, 3, 4])
@pytest.mark.parametrize("L,T,dtype", [(75, 5, "f32"), (130, 7, "bf16"), (12, 4, "f32")])
def test_shared_matches_brute_force_chain(oracle, C, L, T, dtype):
    case = tiny_case(31, L=L, T=T, dtype=dtype, B=2)
    r = oracle.nsa_verify_shared(case, C, branches=True)
    out, shared, br = brute_force_shared(case, C)
    assert np.array_equal(r.sel_idx, shared)
    np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.stack([r.o_cmp, r.o_slc, r.o_win]), br, rtol=0, atol=1e-12)


@pytest.mark.parametrize("order", ["bfs", "dfs"])
def test_shared_matches_brute_force_tree(oracle, order):
    par = si.tree_parents((3, 2, 1), order)
    case = tiny_case(33, L=70, T=len(par), parents=par, B=2, n_query=[len(par), len(par) - 4])
    for C in (2, 4, 5):
        r = oracle.nsa_verify_shared(case, C, branches=True)
        out, shared, br = brute_force_shared(case, C)
        assert np.array_equal(r.sel_idx, shared)
        np.testing.assert_allclose(r.out, out, rtol=0, atol=1e-12)


def test_group_of_one_is_the_exact_variant(oracle):
    case = tiny_case(35, L=200, T=6, B=2)
    exact = oracle.nsa_verify(case)
    shared = oracle.nsa_verify_shared(case, 1)
    assert np.array_equal(exact.sel_idx, shared.sel_idx)
    assert np.array_equal(exact.out, shared.out)


def test_representative_is_exact_and_only_the_selected_branch_changes(oracle):
    case = tiny_case(37, L=300, T=8, B=1, rho=0.0)
    exact = oracle.nsa_verify(case, branches=True)
    shared = oracle.nsa_verify_shared(case, 4, branches=True)
    rep = oracle.group_representatives(case, 4)
    assert rep[0].tolist() == [3, 3, 3, 3, 7, 7, 7, 7]
    for i in (3, 7):
        assert np.array_equal(shared.out[0, i], exact.out[0, i])
        assert np.array_equal(shared.sel_idx[0, i], exact.sel_idx[0, i])
    assert np.array_equal(shared.o_cmp, exact.o_cmp) and np.array_equal(shared.o_win, exact.o_win)
    # with independent queries (rho = 0) some member does lose its own blocks
    assert np.any(shared.sel_idx != exact.sel_idx) and np.any(shared.o_slc != exact.o_slc)
    for i in range(8):
        assert np.array_equal(shared.sel_idx[0, i], exact.sel_idx[0, rep[0, i]])


def test_identical_queries_in_one_block_make_the_variant_exact(oracle):
    """All members of a group score alike (same query vector), sit in the same selection block and see no
    further compressed block: their exact sets coincide, so sharing changes nothing."""
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=4, w=8)
    case = tiny_case(39, L=130, T=4, nsa=nsa, B=1)       # slots 130..133: one selection block (128..143)
    case.q[0, :] = case.q[0, 0]
    case.n_cmp[0] = si.n_cmp_blocks(130, nsa.l, nsa.d)      # deferred commit: no block reaches into the drafts
    exact = oracle.nsa_verify(case)
    assert all(np.array_equal(exact.sel_idx[0, i], exact.sel_idx[0, 0]) for i in range(4))
    shared = oracle.nsa_verify_shared(case, 4)
    assert np.array_equal(shared.sel_idx, exact.sel_idx)
    assert np.array_equal(shared.out, exact.out)


def test_representatives_in_a_tree_prefer_depth_then_order(oracle):
    par = np.array([-1, 0, 0, -1, 3, 4], np.int32)      # depths 0 1 1 0 1 2
    case = tiny_case(41, L=60, T=6, parents=par, B=1)
    assert oracle.group_representatives(case, 3)[0].tolist() == [2, 2, 2, 5, 5, 5]
    assert oracle.group_representatives(case, 4)[0].tolist() == [2, 2, 2, 2, 5, 5]
    assert oracle.group_representatives(case, 2)[0].tolist() == [1, 1, 2, 2, 5, 5]
    case.n_query[0] = 4
    assert oracle.group_representatives(case, 3)[0].tolist() == [2, 2, 2, 3, -1, -1]
