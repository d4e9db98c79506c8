"""GPU parity of the compressed-cache construction (ssv_nsa_compress) against the fp64 oracle.

Bar: the oracle's mean is exact to fp64; the kernel accumulates in fp32 and rounds once, so every element must
lie within half a unit in the last place of the storage type (plus the fp32 accumulation error) of the exact
mean, and all but a vanishing fraction must equal the oracle's own rounding bit for bit."""
import numpy as np
import pytest

import ssv_inputs as si
from oracle import compress as oc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    return torch


def _device(arr, dtype, torch):
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(arr).cuda()


def _host(t, dtype):
    import torch
    return t.float().cpu().numpy().astype(np.float64) if dtype == "bf16" else t.cpu().numpy().astype(np.float64)


def run_compress(torch, dtype, B, H_kv, d_k, d_v, l, d, S, before, after, seed, max_new_rows=None, cmp_cap=None, sentinel=7.0):
    import paper_2605_19893_amd as P
    rng = np.random.default_rng(seed)
    k32 = rng.standard_normal((B, H_kv, S, d_k), dtype=np.float32)
    v32 = rng.standard_normal((B, H_kv, S, d_v), dtype=np.float32) * 3.0
    k_st, v_st = si.to_storage(k32, dtype), si.to_storage(v32, dtype)
    kf, vf = si.to_f32(k_st, dtype).astype(np.float64), si.to_f32(v_st, dtype).astype(np.float64)
    cap = oc.n_cmp_rows(S, l, d) + 1 if cmp_cap is None else cmp_cap
    k, v = _device(k_st, dtype, torch), _device(v_st, dtype, torch)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    kc = torch.full((B, H_kv, cap, d_k), sentinel, dtype=tdt, device="cuda")
    vc = torch.full((B, H_kv, cap, d_v), sentinel, dtype=tdt, device="cuda")
    aft = torch.tensor(after, dtype=torch.int32, device="cuda")
    bef = None if before is None else torch.tensor(before, dtype=torch.int32, device="cuda")
    n_cmp = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    before_l = [0] * B if before is None else list(before)
    if max_new_rows is None:
        max_new_rows = max(1, max(oc.n_cmp_rows(a, l, d) - oc.n_cmp_rows(b0, l, d) for a, b0 in zip(after, before_l)))
    p = P.make_cmp_params(B=B, H_kv=H_kv, d_k=d_k, d_v=d_v, l=l, d=d, dtype=P.SSV_BF16 if dtype == "bf16" else P.SSV_F32,
                          max_new_rows=max_new_rows, kv_capacity=S, cmp_capacity=cap, k_stride=k.stride()[:3],
                          v_stride=v.stride()[:3], kc_stride=kc.stride()[:3], vc_stride=vc.stride()[:3])
    print(f"[run] compress {dtype} B={B} H_kv={H_kv} d=({d_k},{d_v}) l={l} d={d} S={S} before={before} after={after} "
          f"max_new_rows={max_new_rows} cap={cap}", flush=True)
    P.ssv_nsa_compress(k, v, kc, vc, bef, aft, n_cmp, p, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got_n = n_cmp.cpu().numpy()
    kc_h, vc_h = _host(kc, dtype), _host(vc, dtype)
    sig_bits = 8 if dtype == "bf16" else 24
    exact = total = 0
    for b in range(B):
        La = min(after[b], S)
        lo = min(oc.n_cmp_rows(before_l[b], l, d), cap)
        hi = min(oc.n_cmp_rows(La, l, d), cap, lo + max_new_rows)
        assert got_n[b] == hi, (b, got_n[b], hi)
        for h in range(H_kv):
            for raw, have in ((kf[b, h], kc_h[b, h]), (vf[b, h], vc_h[b, h])):
                first, want, mean = oc.compress(raw, before_l[b], La, l, d, dtype)
                want, mean = want[:max(0, hi - lo)], mean[:max(0, hi - lo)]
                got = have[lo:hi]
                # half an ulp of the storage type around the exact mean, plus the fp32 accumulation error
                spacing = np.ldexp(1.0, np.frexp(mean)[1] - sig_bits)      # of the storage type around each mean
                tol = 0.5 * spacing + 1e-6 * np.abs(raw).max()
                assert np.all(np.abs(got - mean) <= tol), (b, h, float(np.abs(got - mean).max()))
                exact += int(np.sum(got == want))
                total += want.size
                # rows outside [lo, hi) are untouched
                assert np.all(have[:lo] == sentinel) and np.all(have[hi:] == sentinel)
    if total:
        print(f"[parity] compress: {total} elements, {total - exact} differ from the oracle's rounding", flush=True)
        if dtype == "bf16":
            assert exact >= total * (1 - 1e-3)
    return kc, vc, got_n


def test_full_build_standard_shapes(torch_mod):
    run_compress(torch_mod, "bf16", 2, 4, 192, 128, 32, 16, 5000, None, [4999, 2077], 1)


def test_full_build_fp32_and_other_ratios(torch_mod):
    run_compress(torch_mod, "f32", 3, 1, 64, 64, 32, 16, 700, None, [700, 31, 32], 2)
    run_compress(torch_mod, "f32", 1, 2, 64, 32, 12, 4, 333, None, [330], 3)
    run_compress(torch_mod, "bf16", 1, 2, 64, 64, 16, 16, 1000, None, [999], 4)
    run_compress(torch_mod, "bf16", 1, 1, 128, 128, 64, 8, 600, None, [600], 5)


def test_incremental_updates_and_deferred_commit(torch_mod):
    """Verification rounds: 0..16 accepted tokens at a time; only rows whose tokens are all committed appear."""
    before = [4096, 1000, 31, 47, 640]
    after = [4112, 1003, 32, 47, 700]
    run_compress(torch_mod, "bf16", 5, 4, 192, 128, 32, 16, 4200, before, after, 6)


def test_rollback_capacity_and_row_bound(torch_mod):
    # committed length shrinks: nothing is written, the row count follows
    run_compress(torch_mod, "bf16", 2, 2, 64, 64, 32, 16, 600, [500, 100], [300, 90], 7)
    # more rows than the compressed cache holds; committed length beyond the raw cache; fewer rows allowed than due
    run_compress(torch_mod, "bf16", 1, 2, 64, 64, 32, 16, 600, None, [600], 8, cmp_cap=20)
    run_compress(torch_mod, "bf16", 1, 2, 64, 64, 32, 16, 600, None, [10 ** 6], 9)
    run_compress(torch_mod, "bf16", 2, 2, 64, 64, 32, 16, 600, [0, 320], [600, 600], 10, max_new_rows=5)


def test_compressed_cache_feeds_the_verification_path(torch_mod, oracle):
    """Build k_cmp / v_cmp on the GPU from the raw cache of a seeded batch and verify with them: indices and outputs
    must match the oracle run on the SAME compressed rows (read back), and those rows match the compression oracle."""
    import paper_2605_19893_amd as P
    from paper_2605_19893_amd.device_case import DeviceCase
    from parity import check, compare
    torch = torch_mod
    case = si.make_case("cmp_feed", "bf16", 2, 6, 32, 2, 192, 128, si.STD_NSA, [3000, 2500], 133, rho=0.5)
    dev = DeviceCase(case)
    dev.k_cmp.fill_(0)
    dev.v_cmp.fill_(0)
    committed = torch.tensor((case.seq_lens + case.n_query).astype(np.int32), device="cuda")   # chain: pooled over prefix + drafts
    p = P.make_cmp_params(B=case.B, H_kv=case.H_kv, d_k=case.d_k, d_v=case.d_v, l=32, d=16, dtype=P.SSV_BF16,
                          max_new_rows=case.k_cmp.shape[2], kv_capacity=case.k.shape[2], cmp_capacity=case.k_cmp.shape[2],
                          k_stride=dev.k.stride()[:3], v_stride=dev.v.stride()[:3], kc_stride=dev.k_cmp.stride()[:3],
                          vc_stride=dev.v_cmp.stride()[:3])
    P.ssv_nsa_compress(dev.k, dev.v, dev.k_cmp, dev.v_cmp, None, committed, dev.n_cmp, p, torch.cuda.current_stream().cuda_stream)
    dev.run()
    out, sel = dev.results()
    assert np.array_equal(dev.n_cmp.cpu().numpy(), case.n_cmp)
    case.k_cmp[...] = dev.k_cmp.view(torch.int16).cpu().numpy().view(np.uint16)
    case.v_cmp[...] = dev.v_cmp.view(torch.int16).cpu().numpy().view(np.uint16)
    ref = oracle.nsa_verify(case)
    check(case, compare(case, oracle, ref, out, sel))
