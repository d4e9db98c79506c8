"""GPU parity over seeded random small problems: shapes, lengths, trees, ragged query counts, groupings and
modes drawn from a fixed list of seeds, so that slice counts of one, two and three tiles, partial row tiles, every
GQA ratio and both homes of the top-n selection all occur.  Each case is one the oracle finishes in a second or two."""
import numpy as np
import pytest

import ssv_inputs as si
from parity import check, compare

pytestmark = pytest.mark.gpu

SHAPES = [  # dtype, H, H_kv, d_k, d_v
    ("bf16", 64, 4, 192, 128), ("bf16", 32, 4, 192, 128), ("bf16", 16, 4, 128, 128), ("bf16", 8, 4, 64, 64),
    ("bf16", 4, 4, 64, 64), ("f32", 16, 1, 64, 64), ("f32", 4, 2, 64, 64), ("f32", 3, 3, 64, 64),
]


def random_parents(rng, T):
    """A random forest over the draft tokens: parents[i] in {-1, 0..i-1}."""
    return np.asarray([-1 if i == 0 or rng.random() < 0.2 else int(rng.integers(0, i)) for i in range(T)], np.int32)


def draw_case(seed):
    rng = np.random.default_rng(seed)
    dtype, H, H_kv, d_k, d_v = SHAPES[int(rng.integers(len(SHAPES)))]
    B = int(rng.integers(1, 4))
    T = int(rng.choice([1, 2, 3, 5, 8, 13, 21]))
    if rng.random() < 0.5:
        nsa = si.STD_NSA
    else:
        nsa = si.NsaParams(l=32, d=16, l_sel=64, n_sel=int(rng.choice([3, 4, 8, 16])), w=int(rng.choice([1, 64, 100, 512])))
    lens = [int(rng.integers(1, 7000)) if rng.random() < 0.8 else int(rng.integers(1, 200)) for _ in range(B)]
    n_query = [int(rng.integers(0, T + 1)) if rng.random() < 0.3 else T for _ in range(B)]
    parents = None
    if rng.random() < 0.5 and T > 1:
        parents = np.stack([random_parents(rng, T) for _ in range(B)])
    case = si.make_case(f"sweep_{seed}", dtype, B, T, H, H_kv, d_k, d_v, nsa, lens, 9000 + seed, rho=float(rng.random()),
                        parents=parents, n_query=n_query, poison_pad=bool(rng.random() < 0.5), workers=4)
    H_g = H // H_kv
    c_max = max(1, min(T, 64, 128 // H_g))
    group = int(rng.integers(0, c_max + 1))
    scan_group = int(rng.integers(0, c_max + 1))
    share = int(rng.integers(1, T + 1))
    return case, group, scan_group, share, bool(rng.random() < 0.5)


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_problem(seed, oracle):
    from paper_2605_19893_amd import SSV_REFRESH, SSV_REUSE, SSV_REFRESH_SHARED
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    case, group, scan_group, share, fused = draw_case(seed)
    ref = oracle.nsa_verify(case)
    dev = DeviceCase(case, group_size=group, topn_home=B.SSV_TOPN_IN_SLC if fused else B.SSV_TOPN_SEPARATE,
                     max_slice_tiles=(0, 2, 5)[seed % 3])
    dev.set_group_size(group, SSV_REFRESH, scan_group_size=scan_group)
    print(f"[run] {case.name} B={case.B} T={case.T} H={case.H}/{case.H_kv} L={case.seq_lens.tolist()} nq={case.n_query.tolist()} "
          f"tree={case.parents is not None} fused_topn={fused} plan={dev.plan.as_dict()}", flush=True)
    dev.run()
    out, sel = dev.results()
    check(case, compare(case, oracle, ref, out, sel))
    dev.set_mode(SSV_REUSE)
    dev.run()
    out2, _ = dev.results()
    check(case, compare(case, oracle, oracle.nsa_verify(case, sel_idx=sel), out2, sel, reuse_sel=sel))
    dev.set_group_size(share, SSV_REFRESH_SHARED, scan_group_size=scan_group)
    dev.run()
    out3, sel3 = dev.results()
    check(case, compare(case, oracle, oracle.nsa_verify_shared(case, share), out3, sel3,
                        routed_by=oracle.group_representatives(case, share)))


@pytest.mark.parametrize("seed", list(range(100, 116)))
def test_random_problem_scan_variants(seed, oracle):
    """The same random problems through the other homes of the compressed scan: the streaming kernel with its slices
    from the work table, and (bf16) the matrix-core kernel, whose split is the balanced one whenever the lengths of the
    batch differ in their tile counts; refresh, reuse and the shared-index variant."""
    from paper_2605_19893_amd import SSV_REFRESH, SSV_REUSE, SSV_REFRESH_SHARED
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    case, _, _, share, fused = draw_case(seed)
    kernels = [B.SSV_SCAN_STREAM_TABLE] + ([B.SSV_SCAN_MATRIX] if case.dtype == "bf16" else [])
    ref = oracle.nsa_verify(case)
    ref_shared = oracle.nsa_verify_shared(case, share)
    for kern in kernels:
        dev = DeviceCase(case, scan_kernel=kern, topn_home=B.SSV_TOPN_IN_SLC if fused else B.SSV_TOPN_SEPARATE)
        print(f"[run] {case.name} scan_kernel={kern} B={case.B} T={case.T} H={case.H}/{case.H_kv} L={case.seq_lens.tolist()} "
              f"nq={case.n_query.tolist()} tree={case.parents is not None} plan={dev.plan.as_dict()}", flush=True)
        dev.run()
        out, sel = dev.results()
        check(case, compare(case, oracle, ref, out, sel))
        dev.set_mode(SSV_REUSE)
        dev.run()
        out2, _ = dev.results()
        check(case, compare(case, oracle, oracle.nsa_verify(case, sel_idx=sel), out2, sel, reuse_sel=sel))
        dev.set_group_size(share, SSV_REFRESH_SHARED)
        dev.run()
        out3, sel3 = dev.results()
        check(case, compare(case, oracle, ref_shared, out3, sel3, routed_by=oracle.group_representatives(case, share)))
