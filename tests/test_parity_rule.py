"""The comparison rule itself (CPU only): a GPU index set that differs from the oracle's is accepted only
when every swapped block lies within 1e-4 of the oracle's selection boundary, in the oracle's importance."""
from types import SimpleNamespace

import numpy as np
import pytest

import ssv_inputs as si
from parity import AMBIGUOUS_GAP, check, compare, swap_margins


def _fake(imp_row, want, L=64 * 9 + 5, n_sel=6):
    """One sequence, one query, one KV group with a hand-made importance row over blocks 0..J (J = 9)."""
    nsa = si.NsaParams(l=32, d=16, l_sel=64, n_sel=n_sel, w=64)
    case = SimpleNamespace(B=1, T=1, H_kv=1, nsa=nsa, seq_lens=np.array([L]), n_query=np.array([1]))
    imp = np.zeros((1, 1, 1, 12))
    imp[0, 0, 0, :len(imp_row)] = imp_row
    sel = np.full((1, 1, 1, n_sel), -1, np.int32)
    sel[0, 0, 0, :len(want)] = want
    return case, SimpleNamespace(imp=imp, sel_idx=sel)


# blocks 0, 8, 9 are forced (initial + two local); three free picks among 1..7
IMP = np.array([9., .50, .40, .30, .29995, .10, .05, .01, 9., 9.])


def test_swap_inside_the_band_is_accepted_and_measured():
    case, ref = _fake(IMP, [0, 1, 2, 3, 8, 9])
    gpu = ref.sel_idx.copy()
    gpu[0, 0, 0] = [0, 1, 2, 4, 8, 9]                     # 4 instead of 3: 5e-5 apart
    differ = np.ones((1, 1, 1), bool)
    worst, n_viol = swap_margins(case, None, ref, gpu, differ)
    assert n_viol == 0 and worst == pytest.approx(5e-5, abs=1e-12)


@pytest.mark.parametrize("bad,margin", [([0, 1, 2, 5, 8, 9], 0.2), ([0, 1, 3, 4, 8, 9], 0.10005), ([0, 2, 3, 7, 8, 9], 0.29)])
def test_clearly_worse_block_is_rejected(bad, margin):
    case, ref = _fake(IMP, [0, 1, 2, 3, 8, 9])
    gpu = ref.sel_idx.copy()
    gpu[0, 0, 0] = bad
    worst, n_viol = swap_margins(case, None, ref, gpu, np.ones((1, 1, 1), bool))
    assert n_viol >= 1 and worst == pytest.approx(margin, abs=1e-9) and worst > AMBIGUOUS_GAP


def test_compare_fails_a_wrong_selection_even_when_the_oracle_gap_is_small(oracle):
    """End to end on a real tiny batch: the oracle's own result with one clearly worse block swapped in must fail
    `check`, whatever the oracle's boundary gap is (the old rule let it through when the gap was below 1e-4)."""
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=5, w=8)
    case = si.make_case("rule", "f32", 1, 3, 4, 2, 8, 6, nsa, [300], 77, rho=0.3, workers=1)
    ref = oracle.nsa_verify(case, want_imp=True)
    ref.gap[...] = 0.0                                     # pretend every unit is ambiguous
    good_out = ref.out
    check(case, compare(case, oracle, ref, good_out, ref.sel_idx.copy()))
    b, i, g = 0, 1, 1
    J = (300 + i) // 16
    row = ref.imp[b, i, g, :J + 1]
    chosen = set(ref.sel_idx[b, i, g].tolist())
    free = [j for j in chosen if j not in (0, J - 1, J)]
    worst_block = min((j for j in range(J + 1) if j not in chosen), key=lambda j: row[j])
    victim = max(free, key=lambda j: row[j])
    assert row[victim] - row[worst_block] > 10 * AMBIGUOUS_GAP
    bad = ref.sel_idx.copy()
    bad[b, i, g] = sorted((chosen - {victim}) | {worst_block})
    rep = compare(case, oracle, ref, oracle.nsa_verify(case, sel_idx=bad).out, bad)
    assert rep.n_mismatch == 1 and rep.n_mismatch_strict == 0 and rep.n_swap_violations >= 1
    with pytest.raises(AssertionError):
        check(case, rep)
