"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle, element by element on
the same seeded inputs.  Sizes here are ones the oracle finishes in seconds while still spanning
several 64-row tiles, several splits and ragged tails."""
import numpy as np
import pytest

import ssv_inputs as si
from parity import check, compare

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    from paper_2605_19893_amd import device_case
    return device_case


def run_refresh(dev_mod, oracle, case, group_size=0, **dev_kw):
    ref = oracle.nsa_verify(case)
    dev = dev_mod.DeviceCase(case, group_size=group_size, **dev_kw)
    print(f"[run] {case.name} refresh C={dev.plan.C} plan={dev.plan.as_dict()}", flush=True)
    dev.run()
    out, sel = dev.results()
    rep = compare(case, oracle, ref, out, sel)
    check(case, rep)
    return dev, ref, out, sel


def run_reuse(dev_mod, oracle, case, sel, group_size=0, dev=None):
    from paper_2605_19893_amd import SSV_REUSE
    ref = oracle.nsa_verify(case, sel_idx=sel)
    if dev is None:
        dev = dev_mod.DeviceCase(case, group_size=group_size)
    dev.set_mode(SSV_REUSE)
    dev.set_sel_idx(sel)
    print(f"[run] {case.name} reuse C={dev.plan.C}", flush=True)
    dev.run()
    out, _ = dev.results()
    rep = compare(case, oracle, ref, out, sel, reuse_sel=sel)
    check(case, rep)
    return out


def run_shared(dev_mod, oracle, case, C, **dev_kw):
    """Approximate shared-index variant with groups of C queries, then reuse of the indices it wrote."""
    from paper_2605_19893_amd import SSV_REFRESH_SHARED
    ref = oracle.nsa_verify_shared(case, C)
    rep = oracle.group_representatives(case, C)
    dev = dev_mod.DeviceCase(case, mode=SSV_REFRESH_SHARED, group_size=C, **dev_kw)
    assert dev.plan.share_group == C
    print(f"[run] {case.name} shared-index C={C} plan={dev.plan.as_dict()}", flush=True)
    dev.run()
    out, sel = dev.results()
    check(case, compare(case, oracle, ref, out, sel, routed_by=rep))
    for b in range(case.B):
        for i in range(int(case.n_query[b])):
            assert np.array_equal(sel[b, i], sel[b, rep[b, i]]), (b, i)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)
    return out, sel


def test_config0_fp32(dev_mod, oracle):
    case = si.config0()
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    assert np.array_equal(sel, ref.sel_idx)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


@pytest.mark.parametrize("group_size", [0, 1, 3, 5])
def test_bf16_ragged_tiles_and_splits(dev_mod, oracle, group_size):
    """Two sequences of different, non-aligned lengths; 5 queries: group sizes from 1 query per workgroup up
    to all 5 (80 rows: two row tiles per wave)."""
    case = si.make_case("bf16_ragged", "bf16", 2, 5, 32, 2, 192, 128, si.STD_NSA, [3001, 1237], 101, rho=0.5,
                        poison_pad=True)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case, group_size=group_size)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


def test_f32_chain_crossing_block_boundaries(dev_mod, oracle):
    """L chosen so that the draft tokens cross a selection-block and a compression-window boundary."""
    nsa = si.NsaParams(l=32, d=16, l_sel=64, n_sel=6, w=100)
    case = si.make_case("f32_cross", "f32", 3, 7, 8, 2, 64, 64, nsa, [1021, 2045, 636], 103, rho=0.3, poison_pad=True)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    assert np.array_equal(sel, ref.sel_idx)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


@pytest.mark.parametrize("order", ["bfs", "dfs"])
def test_tree_masks(dev_mod, oracle, order):
    par = si.tree_parents((3, 2, 2), order)   # 3 + 6 + 12 = 21 queries
    case = si.make_case(f"tree_{order}", "bf16", 2, len(par), 32, 2, 192, 128, si.STD_NSA, [2048, 1500], 105,
                        rho=0.6, parents=par)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


def test_tree_compressed_over_drafts_and_explicit_chain_parents(dev_mod, oracle):
    """A chain given by explicit parent indices equals the NULL-parents fast path; a tree whose
    compressed cache covers draft slots exercises the contiguous-extent visibility rule."""
    chain = si.make_case("chain_explicit", "bf16", 1, 6, 16, 1, 192, 128, si.STD_NSA, [1008], 107, rho=0.5,
                         parents=si.chain_parents(6))
    _, _, out_a, sel_a = run_refresh(dev_mod, oracle, chain)
    chain.parents = None
    _, _, out_b, sel_b = run_refresh(dev_mod, oracle, chain)
    assert np.array_equal(out_a, out_b) and np.array_equal(sel_a, sel_b)
    par = si.tree_parents((2, 2), "dfs")
    tree = si.make_case("tree_cmp_drafts", "f32", 1, len(par), 4, 1, 64, 64,
                        si.NsaParams(l=32, d=16, l_sel=64, n_sel=5, w=64), [1010], 109, rho=0.5, parents=par,
                        cmp_over_drafts=True)
    run_refresh(dev_mod, oracle, tree)


@pytest.mark.parametrize("H,H_kv", [(32, 8), (16, 2), (4, 2), (3, 3)])
def test_gqa_group_sizes_paper_kernel_shape(dev_mod, oracle, H, H_kv):
    """Head dim 64 as in the paper's kernel benchmark (32 query heads / 8 KV heads there); H_g = 4, 8, 2, 1."""
    case = si.make_case(f"hg{H // H_kv}", "bf16", 2, 9, H, H_kv, 64, 64, si.STD_NSA, [1500, 2111], 111, rho=0.5)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


def test_short_contexts_and_ragged_query_counts(dev_mod, oracle):
    """Contexts shorter than one compression window / fewer blocks than n; sequences with fewer queries."""
    case = si.make_case("short", "f32", 4, 5, 4, 1, 64, 64, si.NsaParams(l=32, d=16, l_sel=64, n_sel=4, w=40),
                        [3, 40, 130, 700], 113, rho=0.2, n_query=[5, 1, 3, 4], poison_pad=True)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    assert np.array_equal(sel, ref.sel_idx)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


def test_reuse_ignores_bad_entries(dev_mod, oracle):
    case = si.make_case("reuse_messy", "bf16", 1, 4, 16, 1, 192, 128, si.STD_NSA, [4000], 115, rho=0.5)
    ref = oracle.nsa_verify(case)
    messy = ref.sel_idx[..., ::-1].copy()
    messy[0, 0, 0, 3] = messy[0, 0, 0, 4]     # duplicate
    messy[0, 1, 0, 5] = 10 ** 6               # out of range
    messy[0, 2, 0, 7] = -5                    # negative
    messy[0, 3, 0, 2] = (4000 + 3) // 64      # the last block: legal, partially visible
    run_reuse(dev_mod, oracle, case, messy)


def test_planted_needles_are_selected_exactly(dev_mod, oracle):
    """Well-separated importances: indices must be bit-exact and far from the ambiguity band."""
    case = si.make_case("needles", "bf16", 1, 4, 16, 1, 192, 128, si.STD_NSA, [8192], 117, rho=0.95)
    qdir = si.bf16_bits_to_f32(case.q[0, 0]).mean(axis=0)
    qdir /= np.linalg.norm(qdir)
    needles = [5, 17, 40, 41, 77, 90, 100, 101, 110, 111, 120, 121, 125]
    kf = si.bf16_bits_to_f32(case.k)
    for j in needles:
        kf[0, 0, 64 * j:64 * j + 64] = 2.0 * qdir
    case.k[...] = si.f32_to_bf16_bits(kf)
    nc = int(case.n_cmp[0])
    case.k_cmp[0, 0, :nc] = si.f32_to_bf16_bits(si._pool_slice(si.bf16_bits_to_f32(case.k[0, 0]), nc, 32, 16))
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    assert np.all(ref.gap > 1e-3)
    assert np.array_equal(sel, ref.sel_idx)
    assert sorted(sel[0, 0, 0].tolist()) == sorted([0] + needles + [127, 128])


def test_gates_one_hot_isolate_each_branch(dev_mod, oracle):
    case = si.make_case("gates", "bf16", 1, 3, 16, 1, 192, 128, si.STD_NSA, [2500], 119, rho=0.5)
    for idx in range(3):
        case.gates[...] = 0.0
        case.gates[..., idx] = 1.0
        run_refresh(dev_mod, oracle, case)


def test_runs_are_bitwise_reproducible(dev_mod, oracle):
    case = si.make_case("repro", "bf16", 2, 8, 64, 4, 192, 128, si.STD_NSA, [5000, 4100], 121, rho=0.5)
    dev = dev_mod.DeviceCase(case)
    dev.run()
    out1, sel1 = dev.results()
    dev.workspace.fill_(0x7F)      # stale scratch contents must not matter
    dev.run()
    out2, sel2 = dev.results()
    assert np.array_equal(out1, out2) and np.array_equal(sel1, sel2)


@pytest.mark.parametrize("C", [1, 2, 4])
def test_shared_index_variant_chain(dev_mod, oracle, C):
    """Section 4.3: the last query of every run of C routes for the run; T = 7 leaves a short last group."""
    case = si.make_case("shared_chain", "bf16", 2, 7, 32, 2, 192, 128, si.STD_NSA, [3001, 2040], 123, rho=0.3,
                        poison_pad=True)
    out, sel = run_shared(dev_mod, oracle, case, C)
    if C == 1:
        dev, ref, out_exact, sel_exact = run_refresh(dev_mod, oracle, case)
        assert np.array_equal(sel, sel_exact) and np.array_equal(out, out_exact)


@pytest.mark.parametrize("order", ["bfs", "dfs"])
def test_shared_index_variant_tree_and_ragged(dev_mod, oracle, order):
    par = si.tree_parents((3, 2, 2), order)
    case = si.make_case(f"shared_tree_{order}", "bf16", 3, len(par), 16, 1, 192, 128, si.STD_NSA, [2048, 1500, 777],
                        125, rho=0.6, parents=par, n_query=[len(par), 9, 1])
    run_shared(dev_mod, oracle, case, 4)


def test_shared_index_variant_small_heads_many_groups(dev_mod, oracle):
    """H_g = 4, T = 33, C = 2: 17 representatives packed 16 to a routing workgroup; fp32 at head dim 64."""
    case = si.make_case("shared_hg4", "f32", 1, 33, 8, 2, 64, 64, si.NsaParams(l=32, d=16, l_sel=64, n_sel=6, w=100),
                        [1990], 127, rho=0.4)
    run_shared(dev_mod, oracle, case, 2)


@pytest.mark.parametrize("gamma,C", [(64, 1), (64, 2), (64, 0), (4, 1), (4, 2)])
def test_paper_kernel_workload_shape(dev_mod, oracle, gamma, C):
    """32 query heads / 8 KV heads of dimension 64 and draft lengths 4 and 64 (the paper's isolated-kernel
    setting, Section 7): per-query execution (C = 1), the paper's exact variant (C = 2), default grouping."""
    case = si.make_case(f"kw_g{gamma}", "bf16", 1, gamma, 32, 8, 64, 64, si.STD_NSA, [8192 + 37], 129, rho=0.6)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case, group_size=C)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)


def test_group_size_can_change_on_a_live_case(dev_mod, oracle):
    case = si.make_case("regroup", "bf16", 1, 12, 32, 8, 64, 64, si.STD_NSA, [4000], 131, rho=0.5)
    ref = oracle.nsa_verify(case)
    dev = dev_mod.DeviceCase(case, group_size=1)
    outs = []
    for C in (1, 3, 0, 12):
        dev.set_group_size(C)
        dev.run()
        out, sel = dev.results()
        check(case, compare(case, oracle, ref, out, sel))
        outs.append(sel)
    assert all(np.array_equal(outs[0], s) for s in outs[1:])


@pytest.mark.parametrize("shape", ["chain", "tree_bfs", "tree_dfs"])
def test_scan_launch_with_its_own_grouping(dev_mod, oracle, shape):
    """The compressed and window scans grouped differently from the selected branch (larger, smaller, ragged last
    group, two row tiles per wave), in refresh, reuse and shared-index mode: the partial states of the two launches
    meet per output row, so every combination gives the oracle's result and the same indices."""
    from paper_2605_19893_amd import SSV_REFRESH, SSV_REUSE, SSV_REFRESH_SHARED
    if shape == "chain":
        case = si.make_case("scan_groups_chain", "bf16", 2, 11, 64, 4, 192, 128, si.STD_NSA, [5000, 2300], 171, rho=0.6,
                            n_query=[11, 7], poison_pad=True)
    else:
        par = si.tree_parents((3, 2, 2), shape[5:])   # 21 queries
        case = si.make_case(f"scan_groups_{shape}", "bf16", 2, len(par), 32, 2, 192, 128, si.STD_NSA, [4100, 1500], 173,
                            rho=0.6, parents=par)
    ref = oracle.nsa_verify(case)
    dev = dev_mod.DeviceCase(case)
    sels = []
    H_g = case.H // case.H_kv
    for C, C_scan in ((0, 128 // H_g), (2, 8), (4, 3), (3, 5), (8, 1)):
        dev.set_group_size(C, SSV_REFRESH, scan_group_size=C_scan)
        assert dev.plan.C_scan == C_scan and dev.plan.n_qg_scan == -(-case.T // C_scan)
        print(f"[run] {case.name} refresh plan={dev.plan.as_dict()}", flush=True)
        dev.run()
        out, sel = dev.results()
        check(case, compare(case, oracle, ref, out, sel))
        sels.append(sel)
        dev.set_mode(SSV_REUSE)     # two launches here as well
        dev.run()
        out2, _ = dev.results()
        check(case, compare(case, oracle, oracle.nsa_verify(case, sel_idx=sel), out2, sel, reuse_sel=sel))
    assert all(np.array_equal(sels[0], s) for s in sels[1:])
    G = 3
    dev.set_group_size(G, SSV_REFRESH_SHARED, scan_group_size=128 // H_g)
    dev.run()
    out, sel = dev.results()
    check(case, compare(case, oracle, oracle.nsa_verify_shared(case, G), out, sel, routed_by=oracle.group_representatives(case, G)))


@pytest.mark.parametrize("where", ["separate_launch", "inside_selected_launch"])
def test_both_homes_of_the_top_n_selection(dev_mod, oracle, where):
    """The top-n selection runs inside the selected-branch launch (one wavefront per query) when that launch
    leaves CUs idle, else as a launch of its own; both are forced here on the same cases through the topn_home
    parameter: chain with ragged query counts, tree, shared-index variant, massive ties, a geometry other than
    the standard one, fp32."""
    from paper_2605_19893_amd import binding as B
    home = B.SSV_TOPN_SEPARATE if where == "separate_launch" else B.SSV_TOPN_IN_SLC
    case = si.make_case("topn_home_chain", "bf16", 2, 11, 64, 4, 192, 128, si.STD_NSA, [5000, 2300], 181, rho=0.6,
                        n_query=[11, 7], poison_pad=True)
    for C in (0, 8, 3):
        dev, ref, out, sel = run_refresh(dev_mod, oracle, case, group_size=C, topn_home=home)
        assert dev.plan.topn_in_slc == (where == "inside_selected_launch")
    run_reuse(dev_mod, oracle, case, sel, dev=dev)
    par = si.tree_parents((3, 2, 2), "dfs")
    case = si.make_case("topn_home_tree", "bf16", 2, len(par), 32, 2, 192, 128, si.STD_NSA, [4100, 1500], 183, rho=0.6,
                        parents=par)
    run_refresh(dev_mod, oracle, case, topn_home=home)
    run_shared(dev_mod, oracle, case, 3, topn_home=home)
    # every key equal: all importances tie, the smallest indices win (the list of candidates overflows)
    case = si.make_case("topn_home_ties", "f32", 1, 3, 4, 2, 64, 64, si.STD_NSA, [40000], 185, rho=0.0)
    case.k[:] = 0.25
    case.k_cmp[:] = 0.25
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case, topn_home=home)
    assert np.array_equal(sel, ref.sel_idx)
    # l = 64, d = 16, l' = 64: seven compressed columns per block (the general form of the importance sum)
    nsa = si.NsaParams(l=64, d=16, l_sel=64, n_sel=8, w=128)
    case = si.make_case("topn_home_geometry", "f32", 2, 5, 8, 2, 64, 64, nsa, [3000, 1111], 187, rho=0.4)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case, topn_home=home)
    assert np.array_equal(sel, ref.sel_idx)


def test_library_flattening_reorders_a_tree_without_changing_results(dev_mod, oracle):
    """A BFS-ordered draft tree re-flattened to DFS with ssv_tree_flatten (Section 4.1): queries, gates and draft
    K/V rows are permuted with the returned order; every node keeps its output and index set.  All 21 draft slots
    lie in one selection block and no compressed block reaches into the drafts, so slot order is immaterial."""
    from paper_2605_19893_amd import binding as B
    import copy
    par = si.tree_parents((3, 2, 2), "bfs")
    T, L = len(par), 2048
    bfs = si.make_case("flatten_bfs", "bf16", 1, T, 32, 2, 192, 128, si.STD_NSA, [L], 135, rho=0.6, parents=par)
    perm, new_par = B.ssv_tree_flatten(par.tolist(), B.SSV_TREE_DFS)
    assert new_par == si.tree_parents((3, 2, 2), "dfs").tolist()
    dfs = copy.deepcopy(bfs)
    dfs.name = "flatten_dfs"
    dfs.parents = np.asarray(new_par, np.int32)[None, :].copy()
    dfs.q[0] = bfs.q[0, perm]
    dfs.gates[0] = bfs.gates[0, perm]
    for arr_d, arr_b in ((dfs.k, bfs.k), (dfs.v, bfs.v)):
        arr_d[0, :, L:L + T] = arr_b[0, :, [L + t for t in perm]].transpose(1, 0, 2)
    _, _, out_b, sel_b = run_refresh(dev_mod, oracle, bfs)
    _, _, out_d, sel_d = run_refresh(dev_mod, oracle, dfs)
    assert np.array_equal(sel_d[0], sel_b[0, perm])
    assert np.abs(out_d[0] - out_b[0, perm]).max() <= 2e-2


def test_lengths_beyond_the_host_bounds_are_clamped(dev_mod, oracle):
    """seq_lens / n_cmp entries larger than max_seq_len / max_n_cmp (what every buffer was sized with) are clamped on
    the device instead of taking loads past the caches: the longest sequence then behaves as declared."""
    import torch
    case = si.make_case("clamp", "bf16", 2, 4, 32, 2, 192, 128, si.STD_NSA, [3000, 1200], 143, rho=0.5)
    ref = oracle.nsa_verify(case)
    dev = dev_mod.DeviceCase(case)
    dev.seq_lens.copy_(torch.tensor([10 ** 6, 1200], dtype=torch.int32))
    dev.n_cmp.copy_(torch.tensor([2 ** 30, int(case.n_cmp[1])], dtype=torch.int32))
    dev.run()
    out, sel = dev.results()
    check(case, compare(case, oracle, ref, out, sel))
    dev.seq_lens.copy_(torch.tensor([-5, 1200], dtype=torch.int32))      # negative: an empty context
    dev.n_cmp.copy_(torch.tensor([-1, int(case.n_cmp[1])], dtype=torch.int32))
    dev.run()
    out2, sel2 = dev.results()
    assert np.all(np.isfinite(out2)) and np.array_equal(out2[1], out[1]) and np.array_equal(sel2[1], sel[1])


def test_massive_ties_take_the_smallest_indices(dev_mod, oracle):
    """Identical keys everywhere: uniform compressed probabilities, every interior block has the same importance,
    and the tie rule (smaller index wins) decides the whole selection; more than 512 tied candidates also drive
    the top-n kernel through its serial path."""
    case = si.make_case("ties", "bf16", 1, 3, 16, 1, 192, 128, si.STD_NSA, [40000], 147, rho=0.2)
    row = case.k[0, 0, 5].copy()
    case.k[0, 0, :] = row
    case.k_cmp[0, 0, :] = row          # the mean of identical rows
    ref = oracle.nsa_verify(case)
    J = 40000 // 64
    for i in range(3):
        assert ref.sel_idx[0, i, 0].tolist() == list(range(14)) + [J - 1, J]
    dev = dev_mod.DeviceCase(case)
    dev.run()
    out, sel = dev.results()
    assert np.array_equal(sel, ref.sel_idx)
    check(case, compare(case, oracle, ref, out, sel))


@pytest.mark.parametrize("shape", ["chain_hg4", "chain_hg16", "tree_bfs", "tree_dfs"])
def test_up_to_128_verifier_queries(dev_mod, oracle, shape):
    """Draft budgets above 64 tokens (the paper goes to 128): ancestor sets span two machine words and the draft
    slots span up to three key tiles."""
    if shape == "chain_hg4":
        case = si.make_case("t128_chain", "bf16", 2, 128, 32, 8, 64, 64, si.STD_NSA, [4000 + 21, 2999], 149, rho=0.5,
                            n_query=[128, 97])
    elif shape == "chain_hg16":
        case = si.make_case("t100_chain", "bf16", 1, 100, 16, 1, 192, 128, si.STD_NSA, [3000 + 40], 151, rho=0.5)
    else:
        par = si.tree_parents((4, 3, 3, 2), shape[5:])      # 4 + 12 + 36 + 72 = 124 nodes
        case = si.make_case(f"t124_{shape}", "bf16", 2, len(par), 32, 8, 64, 64, si.STD_NSA, [4096 - 30, 2048 + 7], 153,
                            rho=0.6, parents=par, n_query=[len(par), 70])
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)
    if shape == "tree_dfs":
        run_shared(dev_mod, oracle, case, 4)


@pytest.mark.parametrize("scan_kernel", [0, 2, 3])
def test_calls_can_be_captured_in_a_hip_graph(dev_mod, oracle, scan_kernel):
    """A refresh call and a reuse call recorded into a HIP graph and replayed: the library allocates nothing,
    never synchronises and clears no memory with memset nodes, so every replay (with eager work and synchronisation
    in between) must reproduce the eager result bit for bit.  The scratch is filled with a byte pattern between
    replays: every slot, table and counter a call reads it has written itself.  With the automatic scan, the
    matrix-core scan (its balanced split: the lengths differ) and the streaming scan from its work table."""
    import torch
    from paper_2605_19893_amd import SSV_REFRESH, SSV_REUSE
    case = si.make_case("graph", "bf16", 3, 6, 32, 2, 192, 128, si.STD_NSA, [3001, 2222, 150], 155, rho=0.5, n_query=[6, 4, 6])
    ref = oracle.nsa_verify(case)
    dev = dev_mod.DeviceCase(case, scan_kernel=scan_kernel)
    dev.run()
    out_eager, sel_eager = dev.results()
    check(case, compare(case, oracle, ref, out_eager, sel_eager))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dev.run()                       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            dev.run()
    torch.cuda.synchronize()
    for replay in range(3):
        dev.out.zero_()
        dev.sel_idx.fill_(-7)
        dev.workspace.fill_(0x55)       # eager work between replays; stale scratch must not matter
        torch.cuda.synchronize()
        graph.replay()
        out, sel = dev.results()
        assert np.array_equal(out, out_eager) and np.array_equal(sel, sel_eager), replay
    # reuse mode, captured separately (its launch sequence differs)
    dev.set_mode(SSV_REUSE)
    dev.set_sel_idx(sel_eager)
    dev.run()
    out_reuse, _ = dev.results()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph2, stream=side):
            dev.run()
    torch.cuda.synchronize()
    for replay in range(2):
        dev.out.zero_()
        dev.workspace.fill_(0x55)
        torch.cuda.synchronize()
        graph2.replay()
        out, _ = dev.results()
        assert np.array_equal(out, out_reuse), replay


# ----------------------------------------------------------------------------- unfused execution, strided q / out
@pytest.mark.parametrize("shape", ["std_chain", "tree_small_heads", "fp32"])
def test_unfused_per_query_execution_matches_the_oracle(dev_mod, oracle, shape):
    """SSV_EXEC_UNFUSED (every query on its own, one launch per branch, branch outputs through scratch in the
    storage type, separate gate kernel) computes the same function: refresh and reuse against the oracle, and the
    indices equal to the fused execution's bit for bit (the routing kernels are the same)."""
    from paper_2605_19893_amd import binding as B
    if shape == "std_chain":
        case = si.make_case("unfused_chain", "bf16", 2, 9, 64, 4, 192, 128, si.STD_NSA, [5000, 2300], 301, rho=0.6,
                            n_query=[9, 5], poison_pad=True)
    elif shape == "tree_small_heads":
        par = si.tree_parents((3, 2, 2), "bfs")
        case = si.make_case("unfused_tree", "bf16", 2, len(par), 32, 8, 64, 64, si.STD_NSA, [4100, 700], 303, rho=0.5,
                            parents=par)
    else:
        case = si.make_case("unfused_f32", "f32", 1, 5, 8, 2, 64, 64, si.STD_NSA, [3000], 305, rho=0.4)
    dev_f, ref, out_f, sel_f = run_refresh(dev_mod, oracle, case)
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case, exec=B.SSV_EXEC_UNFUSED)
    assert dev.plan.C == 1 and dev.plan.n_launches == 9
    assert np.array_equal(sel, sel_f)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)
    assert dev.plan.n_launches == 7
    # per-kernel timing entry point covers the additional launches
    ms = []
    dev.run(kernel_ms=ms)
    assert len(ms) == B.SSV_NUM_TIMINGS and all(ms[k] > 0 for k in (B.SSV_K_STREAM_A, B.SSV_K_STREAM_B, B.SSV_K_STREAM_W,
                                                                   B.SSV_K_OUT_CMP, B.SSV_K_OUT_SLC, B.SSV_K_OUT_WIN, B.SSV_K_COMBINE))


@pytest.mark.parametrize("exec_name", ["fused", "unfused"])
def test_strided_queries_and_output(dev_mod, oracle, exec_name):
    """q and out addressed through (batch, query, head) strides: head-major buffers with padded rows; the padding
    of the output buffer is left untouched."""
    import torch
    from paper_2605_19893_amd import binding as B
    ex = B.SSV_EXEC_UNFUSED if exec_name == "unfused" else B.SSV_EXEC_FUSED
    par = si.tree_parents((2, 3), "dfs")
    case = si.make_case("strided", "bf16", 2, len(par), 64, 4, 192, 128, si.STD_NSA, [3000, 4500], 311, rho=0.5, parents=par,
                        n_query=[len(par), 5])
    dev, ref, out, sel = run_refresh(dev_mod, oracle, case, exec=ex, strided_q_out=True)
    assert dev.params.q_stride[2] == case.T * (case.d_k + 8) and dev.params.out_stride[1] == case.d_v + 8
    assert torch.all(dev.out_buf[..., case.d_v:] == 7.0)
    run_reuse(dev_mod, oracle, case, sel, dev=dev)
    dev.set_group_size(0 if ex else 3, B.SSV_REFRESH)
    dev.run()
    out2, sel2 = dev.results()
    check(case, compare(case, oracle, ref, out2, sel2))


@pytest.mark.parametrize("imp_rows", [128, 256])
def test_wide_importance_pass(dev_mod, oracle, imp_rows):
    """The importance pass with 128 or 256 rows per workgroup (row blocks of one workgroup share every strip of
    k_cmp through the ring in LDS) selects exactly what the 64-row pass selects: chains with ragged query counts and
    several tiles per slice, a tree, every heads-per-group class, the shared-index variant, fp32."""
    from paper_2605_19893_amd import binding as B
    cases = [
        si.make_case("wide_imp_chain", "bf16", 2, 19, 64, 4, 192, 128, si.STD_NSA, [9000, 2300], 501, rho=0.6, n_query=[19, 11],
                     poison_pad=True),
        si.make_case("wide_imp_tree", "bf16", 2, len(si.tree_parents((4, 3, 2), "bfs")), 32, 2, 192, 128, si.STD_NSA, [4100, 12000], 503,
                     rho=0.6, parents=si.tree_parents((4, 3, 2), "bfs")),
        si.make_case("wide_imp_hg4", "bf16", 1, 64, 32, 8, 64, 64, si.STD_NSA, [7000], 505, rho=0.3),
        si.make_case("wide_imp_hg8", "bf16", 2, 30, 16, 2, 128, 128, si.STD_NSA, [3000, 5000], 507, rho=0.3, n_query=[30, 17]),
        si.make_case("wide_imp_hg2", "bf16", 1, 100, 4, 2, 64, 64, si.STD_NSA, [2500], 509, rho=0.3),
        si.make_case("wide_imp_hg1", "f32", 1, 128, 2, 2, 64, 64, si.STD_NSA, [1800], 511, rho=0.3),
    ]
    for case in cases:
        dev, ref, out, sel = run_refresh(dev_mod, oracle, case, imp_rows=64)
        assert dev.plan.imp_rows == 64
        dev_w, ref, out_w, sel_w = run_refresh(dev_mod, oracle, case, imp_rows=imp_rows)
        assert dev_w.plan.imp_rows in (128, 256) and dev_w.plan.imp_rows <= imp_rows
        assert np.array_equal(sel_w, sel), case.name            # the same sums in the same order
        assert np.array_equal(out_w, out), case.name
    run_shared(dev_mod, oracle, cases[0], 2, imp_rows=imp_rows)
    run_shared(dev_mod, oracle, cases[1], 3, imp_rows=imp_rows)


def test_matrix_core_scan(dev_mod, oracle):
    """The compressed scan in the matrix-core kernel (256 rows per workgroup, the window branch moved into the
    selected-branch launch) against the oracle: chains with ragged query counts and several tiles per slice, a row count
    that fills one workgroup partly and one that needs three, a tree (per-row visibility limits in the last tiles),
    every heads-per-group class, a sequence with fewer compressed rows than one tile and one with none, the
    shared-index variant, reuse mode, and an explicit scan grouping."""
    from paper_2605_19893_amd import binding as B
    tree = si.tree_parents((4, 3, 2), "bfs")
    cases = [
        si.make_case("mscan_chain", "bf16", 2, 19, 64, 4, 192, 128, si.STD_NSA, [9000, 2300], 601, rho=0.6, n_query=[19, 11],
                     poison_pad=True),
        si.make_case("mscan_tree", "bf16", 2, len(tree), 32, 2, 192, 128, si.STD_NSA, [4100, 12000], 603, rho=0.6, parents=tree),
        si.make_case("mscan_hg4", "bf16", 1, 64, 32, 8, 64, 64, si.STD_NSA, [7000], 605, rho=0.3),
        si.make_case("mscan_hg8", "bf16", 2, 30, 16, 2, 128, 128, si.STD_NSA, [3000, 5000], 607, rho=0.3, n_query=[30, 17]),
        si.make_case("mscan_hg2", "bf16", 1, 100, 4, 2, 64, 64, si.STD_NSA, [2500], 609, rho=0.3),
        si.make_case("mscan_short", "bf16", 3, 6, 32, 2, 192, 128, si.STD_NSA, [700, 20, 1100], 611, rho=0.3, n_query=[6, 6, 2]),
    ]
    for case in cases:
        dev, ref, out, sel = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_MATRIX)
        assert dev.plan.scan_matrix == 1 and dev.plan.C_scan * (case.H // case.H_kv) <= 256
        run_reuse(dev_mod, oracle, case, sel, dev=dev)
        assert dev.plan.scan_matrix == 1
        dev_s, _, out_s, sel_s = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_STREAM)
        assert dev_s.plan.scan_matrix == 0
        assert np.array_equal(sel_s, sel), case.name            # the routing sees the same statistics up to rounding
        if len(set(case.seq_lens.tolist())) > 1:
            # sequences of different lengths took the balanced split (ranges over the whole batch); without the hint
            # of the average length the same batch takes even slices per group: the same selections, outputs to tolerance
            dev_e, _, out_e, sel_e = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_MATRIX, avg_seq_len=0)
            assert dev_e.plan.scan_matrix == 1
            assert np.array_equal(sel_e, sel), case.name
    run_shared(dev_mod, oracle, cases[0], 2, scan_kernel=B.SSV_SCAN_MATRIX)
    run_shared(dev_mod, oracle, cases[1], 3, scan_kernel=B.SSV_SCAN_MATRIX)
    # explicit scan grouping: 5 queries (80 rows) per workgroup of the scan, 2 per workgroup of the other branches
    dev = dev_mod.DeviceCase(cases[0], scan_kernel=B.SSV_SCAN_MATRIX)
    dev.set_group_size(2, B.SSV_REFRESH, scan_group_size=5)
    assert dev.plan.scan_matrix == 1 and dev.plan.C_scan == 5 and dev.plan.C == 2
    dev.run()
    out, sel = dev.results()
    check(cases[0], compare(cases[0], oracle, oracle.nsa_verify(cases[0]), out, sel))


def test_matrix_core_scan_balanced_split(dev_mod, oracle):
    """The matrix-core scan's split for batches of mixed lengths: the tiles of all (sequence, KV head) pairs laid end to
    end and cut into equal ranges, a workgroup finishing one pair's state and starting the next.  Batches whose lengths
    span two orders of magnitude, sequences without queries, without compressed rows and shorter than one tile between
    long ones, a batch without any query, an odd batch size, three query groups walking the same ranges (a tree of 40 nodes), ranges much longer
    than the short sequences (a workgroup crosses several pairs) and much shorter than the long ones (a pair is cut into
    many slices), against the oracle in refresh and reuse mode."""
    from paper_2605_19893_amd import binding as B
    tree = si.tree_parents((4, 3, 2), "bfs")
    cases = [
        si.make_case("bal_chain16", "bf16", 7, 16, 64, 4, 192, 128, si.STD_NSA, [300, 26000, 40, 5200, 900, 13000, 2100], 701, rho=0.6,
                     n_query=[16, 16, 5, 0, 16, 9, 16], poison_pad=True),
        si.make_case("bal_tree40", "bf16", 3, len(tree), 32, 2, 192, 128, si.STD_NSA, [1500, 21000, 6400], 703, rho=0.6, parents=tree),
        si.make_case("bal_many_short", "bf16", 12, 16, 32, 2, 128, 128, si.STD_NSA,
                     [260, 700, 330, 18000, 512, 96, 1300, 450, 15, 2000, 640, 800], 705, rho=0.4),
        si.make_case("bal_hg4", "bf16", 3, 64, 32, 8, 64, 64, si.STD_NSA, [9000, 400, 3100], 707, rho=0.3, n_query=[64, 40, 64]),
        si.make_case("bal_no_queries", "bf16", 2, 16, 32, 2, 192, 128, si.STD_NSA, [3000, 500], 709, rho=0.3, n_query=[0, 0]),
    ]
    for case in cases:
        dev, ref, out, sel = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_MATRIX)
        assert dev.plan.scan_matrix == 1 and dev.plan.n_cmp_chunks >= 2
        run_reuse(dev_mod, oracle, case, sel, dev=dev)
        # the importance pass took its slices from the work table the scan wrote; with 256 rows per workgroup too
        dev_w, _, out_w, sel_w = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_MATRIX, imp_rows=256)
        assert np.array_equal(sel_w, sel), case.name
        # the hint only sizes the slots: far below the true average (more slots than ranges cut), far above it (few slots:
        # the kernel lengthens its ranges so that no pair needs more, and a range crosses several short pairs), equal
        # to the maximum (even slices per group)
        mx = int(case.seq_lens.max())
        for hint in (mx // 16 + 1, int(mx * 0.9), mx):
            dev_h, _, out_h, sel_h = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_MATRIX, avg_seq_len=hint)
            assert np.array_equal(sel_h, sel), (case.name, hint)


def test_matrix_core_scan_large_batches(dev_mod, oracle):
    """Batches beyond what the balanced split's tables take: 300 sequences (more than half the importance pass's work
    table holds: that pass cuts every sequence the same way) and 1100 sequences (more than the scan's prefix array
    holds: even slices per sequence), mixed lengths, against the oracle."""
    from paper_2605_19893_amd import binding as B
    rng = np.random.default_rng(907)
    for nb in (300, 1100):
        lens = rng.integers(20, 700, size=nb).tolist()
        lens[3] = 5000
        case = si.make_case(f"mscan_b{nb}", "bf16", nb, 3, 4, 2, 64, 64, si.STD_NSA, lens, 909 + nb, rho=0.3,
                            n_query=rng.integers(0, 4, size=nb).tolist())
        dev, ref, out, sel = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_MATRIX)
        assert dev.plan.scan_matrix == 1
        run_reuse(dev_mod, oracle, case, sel, dev=dev)


def test_streaming_scan_work_table(dev_mod, oracle):
    """The streaming kernel's compressed scan with its slices from the work table that a one-workgroup kernel builds
    from the device-resident lengths (mixed-length batches): lengths over two orders of magnitude, sequences without
    queries, without compressed rows and shorter than one tile, a tree, 128-row scan groups, fp32, refresh, reuse (all
    branches in one launch) and the shared-index variant, against the oracle and against the even slices' selections."""
    from paper_2605_19893_amd import binding as B
    tree = si.tree_parents((3, 2), "bfs")
    cases = [
        si.make_case("tab_chain", "bf16", 7, 8, 64, 4, 192, 128, si.STD_NSA, [300, 26000, 40, 5200, 900, 13000, 2100], 901, rho=0.6,
                     n_query=[8, 8, 5, 0, 8, 3, 8], poison_pad=True),
        si.make_case("tab_tree", "bf16", 3, len(tree), 32, 2, 192, 128, si.STD_NSA, [1500, 21000, 6400], 903, rho=0.6, parents=tree),
        si.make_case("tab_many", "bf16", 12, 4, 32, 2, 128, 128, si.STD_NSA, [260, 700, 330, 18000, 512, 96, 1300, 450, 15, 2000, 640, 800],
                     905, rho=0.4),
        si.make_case("tab_f32", "f32", 3, 4, 8, 2, 64, 64, si.STD_NSA, [3000, 200, 1200], 907, rho=0.5),
        si.make_case("tab_none", "bf16", 2, 4, 32, 2, 192, 128, si.STD_NSA, [3000, 500], 909, rho=0.3, n_query=[0, 0]),
    ]
    for case in cases:
        dev, ref, out, sel = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_STREAM_TABLE)
        assert dev.plan.scan_matrix == 0
        launches = dev.plan.n_launches
        run_reuse(dev_mod, oracle, case, sel, dev=dev)
        dev_e, _, out_e, sel_e = run_refresh(dev_mod, oracle, case, scan_kernel=B.SSV_SCAN_STREAM)
        assert dev_e.plan.n_launches == launches - 1      # (the table kernel)
        assert np.array_equal(sel_e, sel), case.name
        # 128-row groups in the scan launch
        dev_g = dev_mod.DeviceCase(case, scan_kernel=B.SSV_SCAN_STREAM_TABLE)
        C = dev_g.plan.C
        if 2 * C <= case.T:
            dev_g.set_group_size(C, B.SSV_REFRESH, scan_group_size=2 * C)
            dev_g.run()
            out_g, sel_g = dev_g.results()
            check(case, compare(case, oracle, ref, out_g, sel_g))
    run_shared(dev_mod, oracle, cases[0], 2, scan_kernel=B.SSV_SCAN_STREAM_TABLE)
