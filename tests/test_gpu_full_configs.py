"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration
bench.py times (default group size and split plan).  The fp64 oracle is fast enough (seconds on the
host cores) to check EVERY output element and EVERY index set at these sizes, so no sampling is
needed; inputs are the seeded synthetic stand-ins described in ssv_inputs.py."""
import numpy as np
import pytest

import ssv_inputs as si
from parity import check, compare

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2605_19893_amd import device_case
    return device_case


def _refresh_then_reuse(dev_mod, oracle, case):
    from paper_2605_19893_amd import SSV_REUSE
    ref = oracle.nsa_verify(case)
    dev = dev_mod.DeviceCase(case)
    print(f"[run] {case.name} plan={dev.plan.as_dict()}", flush=True)
    dev.run()
    out, sel = dev.results()
    rep = compare(case, oracle, ref, out, sel)
    check(case, rep)
    # reuse with the indices just produced must reproduce the refresh output (same kernels, same order)
    dev.set_mode(SSV_REUSE)
    dev.run()
    out2, _ = dev.results()
    ref2 = oracle.nsa_verify(case, sel_idx=sel)
    check(case, compare(case, oracle, ref2, out2, sel, reuse_sel=sel))
    return dev, ref, out, sel


def test_config0_tiny_fp32(dev_mod, oracle):
    _, ref, _, sel = _refresh_then_reuse(dev_mod, oracle, si.config0())
    assert np.array_equal(sel, ref.sel_idx)


@pytest.mark.parametrize("rho", [0.0, 0.5, 0.9])
def test_config1_b1_32k(dev_mod, oracle, rho):
    _refresh_then_reuse(dev_mod, oracle, si.config1(rho))


def test_config2_batched_64k(dev_mod, oracle):
    _refresh_then_reuse(dev_mod, oracle, si.config2())


@pytest.mark.parametrize("order", ["bfs", "dfs"])
def test_config3_tree_128k(dev_mod, oracle, order):
    _refresh_then_reuse(dev_mod, oracle, si.config3(order))


def test_config4_mixed_lengths_two_steps(dev_mod, oracle):
    from paper_2605_19893_amd import SSV_REUSE
    step1 = si.config4()
    _, _, _, sel1 = _refresh_then_reuse(dev_mod, oracle, step1)
    step2 = si.advance_case(step1)
    del step1
    # step 2, recomputing the indices
    _refresh_then_reuse(dev_mod, oracle, step2)
    # step 2, reusing the indices of step 1 (query i inherits the set of query i)
    ref = oracle.nsa_verify(step2, sel_idx=sel1)
    dev = dev_mod.DeviceCase(step2, mode=SSV_REUSE)
    dev.set_sel_idx(sel1)
    dev.run()
    out, _ = dev.results()
    check(step2, compare(step2, oracle, ref, out, sel1, reuse_sel=sel1))


@pytest.mark.parametrize("make,C", [(lambda: si.config1(0.5), 4), (lambda: si.config3("dfs"), 4), (lambda: si.config2(), 2)])
def test_shared_index_variant_full_size(dev_mod, oracle, make, C):
    """Approximate shared-index variant (Section 4.3; C = 4 in the paper) at benchmark sizes."""
    from paper_2605_19893_amd import SSV_REFRESH_SHARED
    case = make()
    ref = oracle.nsa_verify_shared(case, C)
    routed_by = oracle.group_representatives(case, C)
    dev = dev_mod.DeviceCase(case, mode=SSV_REFRESH_SHARED, group_size=C)
    print(f"[run] {case.name} shared-index C={C} plan={dev.plan.as_dict()}", flush=True)
    dev.run()
    out, sel = dev.results()
    check(case, compare(case, oracle, ref, out, sel, routed_by=routed_by))


def test_config4_lengths_chains_of_8_work_table(dev_mod, oracle):
    """The mixed lengths of configuration 4 with chains of 8 (128 rows per KV head: the streaming kernel scans): a
    scan long enough for the automatic plan to start the call with the work-table kernel; every element and index
    set, refresh and reuse, and the shared-index variant."""
    from paper_2605_19893_amd import SSV_REFRESH_SHARED
    case = si.config4(T=8)
    dev, _, _, _ = _refresh_then_reuse(dev_mod, oracle, case)
    assert dev.plan.scan_matrix == 0
    ref = oracle.nsa_verify_shared(case, 4)
    dev = dev_mod.DeviceCase(case, mode=SSV_REFRESH_SHARED, group_size=4)
    assert dev.plan.n_launches == 5      # table kernel, scan + window, importance, selected branch (with the selection), combine
    dev.run()
    out, sel = dev.results()
    check(case, compare(case, oracle, ref, out, sel, routed_by=oracle.group_representatives(case, 4)))
