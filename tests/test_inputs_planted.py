"""The planted index sets of the paper's kernel workload (CPU only): exact adjacent overlap, valid selections."""
import numpy as np
import pytest

import ssv_inputs as si


@pytest.mark.parametrize("s", [3, 6, 10, 16])
@pytest.mark.parametrize("L,T", [(8192, 4), (8190, 64), (65536 - 20, 64)])
def test_adjacent_queries_share_exactly_s_blocks(s, L, T):
    if s == 16 and T > 4:
        pytest.skip("a chain that crosses a block boundary cannot share all 16 blocks: the new local block is new")
    case = si.make_case("planted", "bf16", 1, T, 8, 4, 8, 8, si.STD_NSA, [L], 5, rho=0.0, workers=1)
    sel = si.planted_overlap_indices(case, s, seed=11)
    assert sel.shape == (1, T, 4, 16) and sel.dtype == np.int32
    for g in range(4):
        for i in range(T):
            row = sel[0, i, g]
            J = (L + i) // 64
            assert np.all(np.diff(row) > 0) and row.min() >= 0 and row.max() == J
            assert {0, J - 1, J} <= set(row.tolist())
            if i:
                assert len(set(row.tolist()) & set(sel[0, i - 1, g].tolist())) == s
    assert not np.array_equal(sel[0, :, 0], sel[0, :, 1])       # KV groups draw their own sets
    assert np.array_equal(sel, si.planted_overlap_indices(case, s, seed=11))      # seeded


def test_short_context_and_impossible_overlap():
    case = si.make_case("planted_short", "bf16", 1, 3, 8, 4, 8, 8, si.STD_NSA, [200], 5, rho=0.0, workers=1)
    sel = si.planted_overlap_indices(case, 4, seed=1)            # J = 3: all four blocks selected by everyone
    assert np.all(sel[0, :, :, :4] == np.arange(4)) and np.all(sel[0, :, :, 4:] == -1)
    case = si.make_case("planted_bad", "bf16", 1, 3, 8, 4, 8, 8, si.STD_NSA, [8192], 5, rho=0.0, workers=1)
    with pytest.raises(AssertionError):
        si.planted_overlap_indices(case, 2, seed=1)              # below the three mandatory blocks
