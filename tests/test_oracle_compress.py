"""Pins of the compression oracle (CPU only): block geometry, closed forms, a library routine, brute force."""
import json
import os

import numpy as np
import pytest
from scipy.ndimage import uniform_filter1d

import ssv_inputs as si
from oracle import compress as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")


def test_block_counts_at_the_standard_configuration():
    with open(GOLDEN) as f:
        nsa = json.load(f)["nsa_standard"]
    l, d = nsa["l"], nsa["d"]
    assert (l, d) == (32, 16)
    assert [oc.n_cmp_rows(L, l, d) for L in (0, 31, 32, 47, 48, 32768, 65536, 131072)] == [0, 0, 1, 1, 2, 2047, 4095, 8191]
    # brute force: count the blocks [c*d, c*d+l) that fit
    for L in range(0, 200):
        assert oc.n_cmp_rows(L, 12, 4) == sum(1 for c in range(L) if c * 4 + 12 <= L)


def test_constant_and_linear_rows_have_closed_form_means():
    S, D = 200, 5
    const = np.full((S, D), 3.25)
    first, vals, mean = oc.compress(const, 0, S, 32, 16, "f32")
    assert first == 0 and vals.shape == (oc.n_cmp_rows(S, 32, 16), D) and np.all(vals == 3.25)
    ramp = np.arange(S, dtype=np.float64)[:, None] * np.array([1.0, -2.0, 0.5, 0.0, 4.0])
    _, _, mean = oc.compress(ramp, 0, S, 32, 16, "f32")
    mid = (16 * np.arange(mean.shape[0]) + 15.5)[:, None] * np.array([1.0, -2.0, 0.5, 0.0, 4.0])   # mean of c*d .. c*d+l-1
    np.testing.assert_allclose(mean, mid, rtol=0, atol=1e-12)


@pytest.mark.parametrize("l,d", [(32, 16), (8, 4), (12, 4), (16, 16)])
def test_equals_a_strided_moving_average(l, d):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((333, 7))
    _, _, mean = oc.compress(x, 0, 333, l, d, "f32")
    # library routine: centred uniform filter of width l, sampled at the block centres
    filt = uniform_filter1d(x, size=l, axis=0, mode="constant", origin=0)
    centres = np.arange(mean.shape[0]) * d + l // 2
    np.testing.assert_allclose(mean, filt[centres], rtol=0, atol=1e-12)


def test_incremental_updates_tile_the_full_build_and_defer_uncommitted_tokens():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((300, 4))
    _, full, _ = oc.compress(x, 0, 300, 32, 16, "bf16")
    got = np.zeros_like(full)
    L = 0
    for step in (31, 1, 15, 1, 100, 7, 0, 9, 136):
        first, vals, _ = oc.compress(x, L, L + step, 32, 16, "bf16")
        # nothing is produced from slots at or beyond the committed length
        assert first * 16 + (32 if len(vals) else 0) <= L + step or len(vals) == 0
        assert all((first + j) * 16 + 32 <= L + step for j in range(len(vals)))
        got[first:first + len(vals)] = vals
        L += step
    assert L == 300 and np.array_equal(got, full)
    # changing an uncommitted slot changes nothing
    y = x.copy()
    y[250:] = 99.0
    _, part_x, _ = oc.compress(x, 0, 250, 32, 16, "bf16")
    _, part_y, _ = oc.compress(y, 0, 250, 32, 16, "bf16")
    assert np.array_equal(part_x, part_y)


def test_rounding_to_bf16_is_nearest_even_and_matches_the_input_helpers():
    # exactly representable values stay; halves go to the even neighbour
    assert oc.round_to_storage(np.array([1.0, -0.15625, 3.0e-5 * 0 + 258.0]), "bf16").tolist() == [1.0, -0.15625, 258.0]
    ulp = 2.0 ** -7          # spacing of bf16 in [1, 2)
    x = np.array([1 + 0.5 * ulp, 1 + 1.5 * ulp, 1 + 0.5 * ulp + 1e-9, -(1 + 2.5 * ulp)])
    assert oc.round_to_storage(x, "bf16").tolist() == [1.0, 1 + 2 * ulp, 1 + ulp, -(1 + 2 * ulp)]
    # on values that are exact in fp32 it agrees with the generators' fp32 -> bf16 conversion
    v = np.random.default_rng(9).standard_normal(10000).astype(np.float32)
    want = si.bf16_bits_to_f32(si.f32_to_bf16_bits(v)).astype(np.float64)
    assert np.array_equal(oc.round_to_storage(v.astype(np.float64), "bf16"), want)


def test_matches_the_pooled_caches_of_the_seeded_batches():
    """The generators' k_cmp / v_cmp (fp32 mean, one rounding) agree with the fp64 oracle to one rounding step."""
    case = si.make_case("pool", "bf16", 2, 3, 4, 2, 16, 8, si.NsaParams(l=32, d=16, l_sel=64, n_sel=4, w=64), [200, 133], 3)
    for b in range(2):
        for h in range(2):
            L = int(case.seq_lens[b]) + 3
            _, vals, mean = oc.compress(si.bf16_bits_to_f32(case.k[b, h]).astype(np.float64), 0, L, 32, 16, "bf16")
            have = si.bf16_bits_to_f32(case.k_cmp[b, h, :len(vals)]).astype(np.float64)
            assert len(vals) == case.n_cmp[b]
            assert np.all(np.abs(have - mean) <= np.abs(mean) * 2.0 ** -8 + 1e-30)
            assert np.mean(have == vals) > 0.999
