"""Several verification rounds end to end on the GPU, the way a serving loop would drive the library:
compressed cache kept up to date incrementally from committed tokens only (draft tokens enter it when they are
accepted), a refresh call followed by a reuse call on the same indices (two layers of one step), acceptance of a
prefix of the chain, and the planner's runtime guard fed with the accepted counts.  Every call is checked against
the oracles on the same data."""
import dataclasses

import numpy as np
import pytest

import ssv_inputs as si
from oracle import compress as oc
from oracle import planner as op
from parity import check, compare

pytestmark = pytest.mark.gpu


def test_verification_rounds_with_deferred_commit(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_2605_19893_amd as P
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase, _to_device

    T, rounds = 8, 4
    nsa = si.STD_NSA
    start = np.array([2040, 1531], np.int32)
    case = si.make_case("rounds", "bf16", 2, T, 32, 2, 192, 128, nsa, start, 145, rho=0.6)
    # the device container is sized for the longest state any round can reach
    roomy = si.make_case("rounds_capacity", "bf16", 2, T, 32, 2, 192, 128, nsa, start + T * rounds, 146, rho=0.0)
    dev = DeviceCase(roomy)
    dev.k_cmp.zero_()
    dev.v_cmp.zero_()
    del roomy
    stream = torch.cuda.current_stream().cuda_stream
    # a guard with a short warm-up and patience, so that the four rounds take it through two moves: the profiled
    # expectations of the first two strategies are far above anything a chain of 8 can accept
    gcfg = B.ssv_guard_default_config()
    gcfg.warmup_steps, gcfg.patience = 1, 1
    expected = [20.0, 19.0, 0.1]
    guard = B.ssv_guard_init(gcfg, expected)
    observations, strategies = [], []
    committed_before = np.zeros(2, np.int32)
    rng = np.random.default_rng(7)
    for r in range(rounds):
        L = case.seq_lens.astype(np.int32)
        # upload this round's state: committed rows (unchanged from the previous round), the new draft rows, queries, gates
        S = case.k.shape[2]
        dev.case = case
        dev.k[:, :, :S].copy_(_to_device(case.k, "bf16", dev.device))
        dev.v[:, :, :S].copy_(_to_device(case.v, "bf16", dev.device))
        dev.set_queries(case.q)
        dev.gates.copy_(torch.from_numpy(case.gates).to(dev.device))
        dev.seq_lens.copy_(torch.from_numpy(L).to(dev.device))
        # 1. compressed cache: only blocks made of committed tokens, built incrementally
        cp = P.make_cmp_params(B=case.B, H_kv=case.H_kv, d_k=case.d_k, d_v=case.d_v, l=nsa.l, d=nsa.d, dtype=P.SSV_BF16,
                               max_new_rows=dev.k_cmp.shape[2], kv_capacity=dev.k.shape[2], cmp_capacity=dev.k_cmp.shape[2],
                               k_stride=dev.k.stride()[:3], v_stride=dev.v.stride()[:3], kc_stride=dev.k_cmp.stride()[:3],
                               vc_stride=dev.v_cmp.stride()[:3])
        P.ssv_nsa_compress(dev.k, dev.v, dev.k_cmp, dev.v_cmp, torch.from_numpy(committed_before).to(dev.device),
                           dev.seq_lens, dev.n_cmp, cp, stream)
        n_cmp = dev.n_cmp.cpu().numpy()
        assert n_cmp.tolist() == [oc.n_cmp_rows(int(x), nsa.l, nsa.d) for x in L]
        kc_host = dev.k_cmp.view(torch.int16).cpu().numpy().view(np.uint16)
        vc_host = dev.v_cmp.view(torch.int16).cpu().numpy().view(np.uint16)
        for b in range(case.B):
            _, want, _ = oc.compress(si.bf16_bits_to_f32(case.k[b, 1]).astype(np.float64), 0, int(L[b]), nsa.l, nsa.d, "bf16")
            got = si.bf16_bits_to_f32(kc_host[b, 1, :n_cmp[b]]).astype(np.float64)
            assert np.mean(got == want) > 0.999 and np.abs(got - want).max() < 0.02
        # the oracle sees exactly what the verification kernel sees
        mirror = dataclasses.replace(case, name=f"rounds_{r}", n_cmp=n_cmp.astype(np.int32), k_cmp=kc_host.copy(),
                                     v_cmp=vc_host.copy())
        # 2. first layer: refresh; second layer: reuse of the same indices
        dev.set_mode(P.SSV_REFRESH)
        dev.run()
        out, sel = dev.results()
        ref = oracle.nsa_verify(mirror)
        check(mirror, compare(mirror, oracle, ref, out, sel))
        dev.set_mode(P.SSV_REUSE)
        dev.run()
        out2, _ = dev.results()
        check(mirror, compare(mirror, oracle, oracle.nsa_verify(mirror, sel_idx=sel), out2, sel, reuse_sel=sel))
        # 3. acceptance of a prefix of the chain; the guard sees the counts
        accept = rng.integers(0, T + 1, size=2).astype(np.int32)
        observations.append((float(accept.mean()), 1.0 + 0.25 * r))
        strategies.append(B.ssv_guard_observe(guard, *observations[-1]))
        committed_before = L.copy()
        case = si.advance_case(case, step=r + 10, accept=accept)
    assert guard.total_steps == rounds and guard.transitions == 2
    want = op.guard_trace(op.GuardConfig(warmup_steps=1, patience=1), expected, None, observations)
    assert strategies == want == [0, 1, 1, 2]
