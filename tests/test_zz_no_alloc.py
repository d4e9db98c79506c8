"""ssv_nsa_verify_static, the entry point for callers that cannot allocate: same results as ssv_nsa_verify on a
caller-owned workspace, on two calls in a row that share the library's fixed scratch array (the second on a
smaller problem, so that it runs over what the first left behind), in every mode; problems that need more
scratch than the array holds are refused before anything is enqueued."""
import numpy as np
import pytest

import ssv_inputs as si

pytestmark = pytest.mark.gpu


def _both_ways(case, mode, sel=None, **dev_kw):
    """(out, sel) through ssv_nsa_verify on a workspace of the caller's and through ssv_nsa_verify_static."""
    import torch
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    dev = DeviceCase(case, mode=mode, **dev_kw)
    assert 0 < B.ssv_nsa_workspace_bytes(dev.params) <= B.SSV_STATIC_SCRATCH_BYTES
    if sel is not None:
        dev.set_sel_idx(sel)
    dev.run()
    want_out, want_sel = dev.results()
    dev.out.fill_(3.0)
    if mode != B.SSV_REUSE:
        dev.sel_idx.fill_(-5)
    print(f"[run] {case.name} mode={mode} static scratch, needs {B.ssv_nsa_workspace_bytes(dev.params)} bytes", flush=True)
    B.ssv_nsa_verify_static(dev.q, dev.k, dev.v, dev.k_cmp, dev.v_cmp, dev.gates, dev.seq_lens, dev.n_cmp, dev.n_query,
                            dev.parents, dev.params, dev.out, dev.sel_idx, torch.cuda.current_stream().cuda_stream)
    got_out, got_sel = dev.results()
    return want_out, want_sel, got_out, got_sel


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2605_19893_amd import binding as B
    from parity import check, compare
    par = si.tree_parents((3, 2), "bfs")
    big = si.make_case("static_big", "bf16", 2, len(par), 64, 4, 192, 128, si.STD_NSA, [6000, 3100], 401, rho=0.5, parents=par)
    small = si.make_case("static_small", "bf16", 1, 3, 64, 4, 192, 128, si.STD_NSA, [1500], 403, rho=0.5, n_query=[2])
    for mode in (B.SSV_REFRESH, B.SSV_REFRESH_SHARED):
        sels = []
        for case in (big, small):         # two calls in a row on the same array, the second smaller
            want_out, want_sel, got_out, got_sel = _both_ways(case, mode)
            assert np.array_equal(got_sel, want_sel)
            assert np.array_equal(got_out, want_out)      # same kernels, same order: bit-identical
            sels.append(got_sel)
        if mode == B.SSV_REFRESH:
            for case, sel in zip((big, small), sels):
                check(case, compare(case, oracle, oracle.nsa_verify(case), *_both_ways(case, mode)[2:]))
                want_out, _, got_out, _ = _both_ways(case, B.SSV_REUSE, sel=sel)
                assert np.array_equal(got_out, want_out)
    # the unfused execution keeps its branch outputs in the same array
    for case in (big, small):
        want_out, want_sel, got_out, got_sel = _both_ways(case, B.SSV_REFRESH, exec=B.SSV_EXEC_UNFUSED)
        assert np.array_equal(got_sel, want_sel) and np.array_equal(got_out, want_out)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    case = si.make_case("static_too_big", "bf16", 24, 16, 64, 4, 192, 128, si.STD_NSA, [300] * 24, 405, rho=0.5)
    dev = DeviceCase(case)
    assert B.ssv_nsa_workspace_bytes(dev.params) > B.SSV_STATIC_SCRATCH_BYTES
    dev.out.fill_(3.0)
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_verify_static(dev.q, dev.k, dev.v, dev.k_cmp, dev.v_cmp, dev.gates, dev.seq_lens, dev.n_cmp, dev.n_query,
                                dev.parents, dev.params, dev.out, dev.sel_idx, torch.cuda.current_stream().cuda_stream)
    assert e.value.code == B.SSV_ESTATIC
    torch.cuda.synchronize()
    assert torch.all(dev.out == 3.0)      # nothing was enqueued
