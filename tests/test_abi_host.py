"""Host-side checks of the C ABI (no GPU, no compute calls): the library loads, exports every symbol the
header declares, validates its arguments before touching the device, and plans launches sensibly."""
import ctypes
import os
import re

import pytest

from paper_2605_19893_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def std_params(**over):
    kw = dict(B=1, T=8, H=64, H_kv=4, d_k=192, d_v=128, l=32, d=16, l_sel=64, n_sel=16, w=512, dtype=B.SSV_BF16,
              mode=B.SSV_REFRESH, max_seq_len=32768, max_n_cmp=2047,
              k_stride=(4 * 32832 * 192, 32832 * 192, 192), v_stride=(4 * 32832 * 128, 32832 * 128, 128),
              kc_stride=(4 * 2047 * 192, 2047 * 192, 192), vc_stride=(4 * 2047 * 128, 2047 * 128, 128))
    kw.update(over)
    return B.make_params(**kw)


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    with open(os.path.join(ROOT, "include", "ssv_nsa.h")) as f:
        header = f.read()
    declared = set(re.findall(r"\b(ssv_(?:nsa|guard|tree)_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.ssv_nsa_version() >= 1


def test_struct_layout_matches_header():
    # 21 four-byte fields (+ 4 bytes of padding), 18 int64 strides, 5 four-byte fields (+ padding); 18 ints and an int64 in the plan
    assert ctypes.sizeof(B.SsvNsaParams) == 22 * 4 + 18 * 8 + 6 * 4
    assert ctypes.sizeof(B.SsvNsaPlan) == 18 * 4 + 8
    with open(os.path.join(ROOT, "include", "ssv_nsa.h")) as f:
        header = f.read()
    # every field of the two structs appears in the header in the binding's order
    for struct, cls in (("ssv_nsa_params", B.SsvNsaParams), ("ssv_nsa_plan", B.SsvNsaPlan)):
        body = header[header.index("typedef struct " + struct):header.index("} " + struct + ";")]
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        names = re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*(?:\[\d+\])?\s*[,;]", body)
        assert names == [n for n, _ in cls._fields_], (struct, names)


def test_error_strings():
    assert B.strerror(B.SSV_OK) == "ok"
    for code in (B.SSV_EINVAL, B.SSV_EUNSUPPORTED, B.SSV_EWORKSPACE, B.SSV_ELAUNCH, B.SSV_ESTATIC):
        assert B.strerror(code) and B.strerror(code) != "unknown error"
    assert B.kernel_name(0).startswith("k_stream") and B.kernel_name(99) == ""


def test_supported_shapes():
    assert B.ssv_nsa_supported(B.SSV_BF16, 192, 128)
    assert B.ssv_nsa_supported(B.SSV_F32, 64, 64)
    assert B.ssv_nsa_supported(B.SSV_BF16, 64, 64)
    assert not B.ssv_nsa_supported(B.SSV_F32, 192, 128)


@pytest.mark.parametrize("over,code", [
    (dict(B=0), B.SSV_EINVAL), (dict(H=63), B.SSV_EINVAL), (dict(l=32, d=12), B.SSV_EINVAL),
    (dict(n_sel=2), B.SSV_EINVAL), (dict(dtype=7), B.SSV_EINVAL), (dict(mode=3), B.SSV_EINVAL),
    (dict(w=0), B.SSV_EINVAL), (dict(avg_seq_len=40000), B.SSV_EINVAL), (dict(group_size=9), B.SSV_EINVAL), (dict(scale=-1.0), B.SSV_EINVAL),
    (dict(k_stride=(1, 1, 100)), B.SSV_EINVAL), (dict(k_stride=(4 * 32832 * 192, 32832 * 192, 196)), B.SSV_EINVAL),
    (dict(mode=B.SSV_REFRESH_SHARED, group_size=9), B.SSV_EINVAL),
    (dict(exec=2), B.SSV_EINVAL), (dict(topn_home=3), B.SSV_EINVAL), (dict(max_slice_tiles=1), B.SSV_EINVAL),
    (dict(max_slice_tiles=65), B.SSV_EINVAL), (dict(imp_rows=100), B.SSV_EINVAL), (dict(exec=B.SSV_EXEC_UNFUSED, group_size=2), B.SSV_EINVAL),
    (dict(exec=B.SSV_EXEC_UNFUSED, mode=B.SSV_REFRESH_SHARED), B.SSV_EINVAL),
    (dict(q_stride=(8 * 64 * 192, 64 * 192, 100)), B.SSV_EINVAL), (dict(out_stride=(8 * 64 * 128, 64 * 128, 130)), B.SSV_EINVAL),
    # the merged schedule of 32 queries x 32 blocks does not fit the LDS next to the tiles of d_k = 192
    (dict(T=32, H=16, H_kv=4, n_sel=32, group_size=32), B.SSV_EUNSUPPORTED),
    (dict(T=129), B.SSV_EUNSUPPORTED), (dict(H=96, H_kv=4), B.SSV_EUNSUPPORTED), (dict(l_sel=128), B.SSV_EUNSUPPORTED),
    (dict(d_k=96), B.SSV_EUNSUPPORTED), (dict(n_sel=40), B.SSV_EUNSUPPORTED),
    (dict(max_seq_len=2 ** 21), B.SSV_EUNSUPPORTED),
    # rows of one (sequence, KV head) spread over 2 GiB or more: beyond the 32-bit offsets of the K loads
    (dict(max_seq_len=2 ** 19, k_stride=(4 * 2 ** 20 * 2048, 2 ** 20 * 2048, 2048)), B.SSV_EUNSUPPORTED),
    (dict(max_n_cmp=2 ** 15, kc_stride=(4 * 2 ** 15 * 2 ** 15, 2 ** 15 * 2 ** 15, 2 ** 15)), B.SSV_EUNSUPPORTED),
])
def test_bad_parameters_are_rejected_without_a_launch(over, code):
    p = std_params(**over)
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_plan_query(p)
    assert e.value.code == code
    assert B.ssv_nsa_workspace_bytes(p) == 0
    fake = 4096   # non-null, aligned: validation of p happens before any pointer is used
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_verify(fake, fake, fake, fake, fake, fake, fake, fake, None, None, p, fake, fake, fake, 1 << 40, 0)
    assert e.value.code == code


def test_null_misaligned_and_workspace_errors():
    p = std_params()
    need = B.ssv_nsa_workspace_bytes(p)
    assert need > 0
    a = 4096
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_verify(None, a, a, a, a, a, a, a, None, None, p, a, a, a, need, 0)
    assert e.value.code == B.SSV_EINVAL
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_verify(a, a + 2, a, a, a, a, a, a, None, None, p, a, a, a, need, 0)
    assert e.value.code == B.SSV_EINVAL
    for ws, nbytes in ((None, need), (a + 16, need), (a, need - 1)):
        with pytest.raises(B.SsvError) as e:
            B.ssv_nsa_verify(a, a, a, a, a, a, a, a, None, None, p, a, a, ws, nbytes, 0)
        assert e.value.code == B.SSV_EWORKSPACE


def test_plan_fills_the_chip_and_respects_limits():
    cfgs = {
        "cfg1": std_params(),
        "cfg2": std_params(B=16, T=4, max_seq_len=65536, max_n_cmp=4095),
        "cfg3": std_params(B=4, T=40, max_seq_len=131072, max_n_cmp=8191),
        "cfg4": std_params(B=32, T=16, max_seq_len=131072, max_n_cmp=8191),
    }
    for name, p in cfgs.items():
        pl = B.ssv_nsa_plan_query(p)
        H_g = p.H // p.H_kv
        assert pl.C * H_g == pl.rows_per_wg <= 64 and pl.C * pl.n_qg >= p.T
        assert pl.n_slots == pl.n_cmp_chunks + pl.n_win_splits + pl.n_slc_splits
        assert pl.n_cmp_chunks * pl.tiles_per_chunk * 64 >= p.max_n_cmp
        assert pl.max_sched_entries == pl.C * p.n_sel
        # scan launch: larger, balanced groups only where the scans keep the chip busy for several rounds; the
        # matrix-core scan (groups of up to 256 rows, one workgroup per CU) where a KV head has the rows for it
        assert pl.scan_matrix == {"cfg1": 0, "cfg2": 0, "cfg3": 1, "cfg4": 1}[name]
        assert pl.C_scan * pl.n_qg_scan >= p.T and pl.C <= pl.C_scan <= (256 if pl.scan_matrix else 128) // H_g
        assert (pl.C_scan, pl.n_qg_scan) == {"cfg1": (4, 2), "cfg2": (4, 1), "cfg3": (14, 3), "cfg4": (16, 1)}[name]
        units = p.B * p.H_kv * pl.n_qg_scan
        if pl.scan_matrix:
            wgs = units * pl.n_cmp_chunks
            # one round of one workgroup per CU, or several rounds of slices of at most 32 tiles
            assert 128 < wgs <= 256 or (wgs > 256 and pl.tiles_per_chunk <= 32), (name, wgs)
            assert pl.n_launches == (5 if name == "cfg4" else 4)
            # behind the matrix-core scan the window shares the selected-branch launch: in one round of workgroups the
            # parts of a group are cut over window tiles and schedule entries together (a slot of either branch per
            # part), in several rounds each branch has slices of its own
            assert (pl.n_win_splits, pl.n_slc_splits) == {"cfg3": (3, 3), "cfg4": (1, 2)}[name]
        else:
            wgs = units * (pl.n_cmp_chunks + pl.n_win_splits)
            # either one resident round (at most 2 workgroups per CU) or several rounds of slices of at most 32 tiles
            assert wgs >= min(256, units * ((p.max_n_cmp + 63) // 64) // 2), (name, wgs)
            assert wgs <= 512 or pl.tiles_per_chunk <= 32, (name, wgs)
        assert pl.workspace_bytes == B.ssv_nsa_workspace_bytes(p) and pl.workspace_bytes % 256 == 0
    p = std_params(group_size=2)
    pl = B.ssv_nsa_plan_query(p)
    assert (pl.C, pl.n_qg, pl.rows_per_wg) == (2, 4, 32)
    pl = B.ssv_nsa_plan_query(std_params(group_size=8))
    assert (pl.C, pl.n_qg, pl.rows_per_wg) == (8, 1, 128)
    # an explicit group size applies to both launches
    pl = B.ssv_nsa_plan_query(std_params(B=4, T=40, max_seq_len=131072, max_n_cmp=8191, group_size=2))
    assert (pl.C, pl.C_scan, pl.n_qg_scan) == (2, 2, 20)
    pl = B.ssv_nsa_plan_query(std_params(group_size=2, scan_group_size=8))
    assert (pl.C, pl.n_qg, pl.C_scan, pl.n_qg_scan) == (2, 4, 8, 1)
    pl = B.ssv_nsa_plan_query(std_params(scan_group_size=3))
    assert (pl.C, pl.n_qg, pl.C_scan, pl.n_qg_scan) == (4, 2, 3, 3)
    for bad in (-1, 9):
        with pytest.raises(B.SsvError) as e:
            B.ssv_nsa_plan_query(std_params(scan_group_size=bad))
        assert e.value.code == B.SSV_EINVAL
    # 12 queries: one group of 192 rows in the matrix-core scan; two balanced groups of 6 in the streaming kernel
    pl = B.ssv_nsa_plan_query(std_params(B=32, T=12, max_seq_len=131072, max_n_cmp=8191))
    assert (pl.C, pl.n_qg, pl.C_scan, pl.n_qg_scan, pl.scan_matrix) == (4, 3, 12, 1, 1)
    pl = B.ssv_nsa_plan_query(std_params(B=32, T=12, max_seq_len=131072, max_n_cmp=8191, scan_kernel=B.SSV_SCAN_STREAM))
    assert (pl.C, pl.n_qg, pl.C_scan, pl.n_qg_scan, pl.scan_matrix) == (4, 3, 6, 2, 0)
    # a long streaming scan of a mixed-length batch (the mean well below the maximum) starts with the work-table kernel:
    # one launch more, slots sized for the longest sequence's share of one round; a uniform batch does not
    mixed = std_params(B=32, T=8, max_seq_len=131072, max_n_cmp=8191, avg_seq_len=40000)
    pl = B.ssv_nsa_plan_query(mixed)
    pl_u = B.ssv_nsa_plan_query(std_params(B=32, T=8, max_seq_len=131072, max_n_cmp=8191))
    assert pl.scan_matrix == 0 and pl_u.scan_matrix == 0 and pl.n_launches == pl_u.n_launches + 1
    assert 2 <= pl.n_cmp_chunks <= 16 and pl.workspace_bytes == B.ssv_nsa_workspace_bytes(mixed)
    pl = B.ssv_nsa_plan_query(std_params(scan_kernel=B.SSV_SCAN_STREAM_TABLE))
    assert pl.scan_matrix == 0 and pl.n_launches == 5
    # the matrix-core scan on request: any bf16 problem of the fused execution; its groups hold up to 256 rows
    pl = B.ssv_nsa_plan_query(std_params(scan_kernel=B.SSV_SCAN_MATRIX))
    assert (pl.scan_matrix, pl.C_scan, pl.n_qg_scan, pl.n_launches) == (1, 8, 1, 4)
    pl = B.ssv_nsa_plan_query(std_params(scan_kernel=B.SSV_SCAN_MATRIX, scan_group_size=3, mode=B.SSV_REUSE))
    assert (pl.scan_matrix, pl.C_scan, pl.n_qg_scan, pl.n_launches) == (1, 3, 3, 3)
    for bad in (dict(scan_kernel=4), dict(scan_kernel=B.SSV_SCAN_STREAM_TABLE, exec=B.SSV_EXEC_UNFUSED), dict(scan_kernel=B.SSV_SCAN_MATRIX, exec=B.SSV_EXEC_UNFUSED),
                dict(scan_kernel=B.SSV_SCAN_MATRIX, dtype=B.SSV_F32, d_k=64, d_v=64), dict(scan_kernel=B.SSV_SCAN_MATRIX, scan_group_size=17)):
        with pytest.raises(B.SsvError) as e:
            B.ssv_nsa_plan_query(std_params(**bad))
        assert e.value.code == B.SSV_EINVAL, bad


def test_static_scratch_entry_point_checks_before_touching_the_device():
    fake = 4096
    big = std_params(B=16, T=4, max_seq_len=65536, max_n_cmp=4095)
    assert B.ssv_nsa_workspace_bytes(big) > B.SSV_STATIC_SCRATCH_BYTES
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_verify_static(fake, fake, fake, fake, fake, fake, fake, fake, None, None, big, fake, fake, 0)
    assert e.value.code == B.SSV_ESTATIC and "static" in B.strerror(B.SSV_ESTATIC)
    with pytest.raises(B.SsvError) as e:      # parameter errors come first, as in the other entry points
        B.ssv_nsa_verify_static(fake, fake, fake, fake, fake, fake, fake, fake, None, None, std_params(H=63), fake, fake, 0)
    assert e.value.code == B.SSV_EINVAL
    assert 0 < B.ssv_nsa_workspace_bytes(std_params()) <= B.SSV_STATIC_SCRATCH_BYTES      # the 32K single-sequence shape fits


def test_plan_reflects_the_execution_choices():
    auto = B.ssv_nsa_plan_query(std_params())
    assert auto.topn_in_slc == 1 and auto.n_launches == 4 and auto.n_imp_chunks >= 1      # cfg1: selection inside launch B
    sep = B.ssv_nsa_plan_query(std_params(topn_home=B.SSV_TOPN_SEPARATE))
    assert sep.topn_in_slc == 0 and sep.n_launches == 5
    assert B.ssv_nsa_plan_query(std_params(B=16, T=4, max_seq_len=65536, max_n_cmp=4095)).topn_in_slc == 1   # 512 workgroups: still inside
    big = std_params(B=32, T=16, max_seq_len=131072, max_n_cmp=8191)
    assert B.ssv_nsa_plan_query(big).topn_in_slc == 0
    big.topn_home = B.SSV_TOPN_IN_SLC
    assert B.ssv_nsa_plan_query(big).topn_in_slc == 1
    reuse = B.ssv_nsa_plan_query(std_params(mode=B.SSV_REUSE))
    assert reuse.topn_in_slc == 0 and reuse.n_imp_chunks == 0 and reuse.n_launches == 2
    # several rounds of workgroups: the slice bound applies
    long_default = B.ssv_nsa_plan_query(std_params(B=32, T=16, max_seq_len=131072, max_n_cmp=8191))
    long_12 = B.ssv_nsa_plan_query(std_params(B=32, T=16, max_seq_len=131072, max_n_cmp=8191, max_slice_tiles=12))
    assert long_default.tiles_per_chunk <= 32 and long_12.tiles_per_chunk <= 12 and long_12.n_cmp_chunks > long_default.n_cmp_chunks
    # importance pass: 64 rows per workgroup for small problems, wider where a KV head has the rows and the pass is long
    assert auto.imp_rows == 64 and reuse.imp_rows == 0
    assert B.ssv_nsa_plan_query(std_params(B=4, T=40, max_seq_len=131072, max_n_cmp=8191)).imp_rows == 256
    assert B.ssv_nsa_plan_query(std_params(B=32, T=16, max_seq_len=131072, max_n_cmp=8191)).imp_rows == 256
    assert B.ssv_nsa_plan_query(std_params(B=32, T=8, max_seq_len=131072, max_n_cmp=8191)).imp_rows == 128
    assert B.ssv_nsa_plan_query(std_params(B=16, T=4, max_seq_len=65536, max_n_cmp=4095)).imp_rows == 64
    assert B.ssv_nsa_plan_query(std_params(imp_rows=256)).imp_rows == 128      # 8 queries x 16 heads fill two blocks
    assert B.ssv_nsa_plan_query(std_params(B=4, T=40, max_seq_len=131072, max_n_cmp=8191, imp_rows=64)).imp_rows == 64
    # unfused execution: every query on its own, one launch per branch plus their merges and the gate kernel
    un = B.ssv_nsa_plan_query(std_params(exec=B.SSV_EXEC_UNFUSED))
    assert (un.C, un.n_qg, un.C_scan, un.n_qg_scan, un.topn_in_slc, un.n_launches) == (1, 8, 1, 8, 0, 9)
    assert B.ssv_nsa_plan_query(std_params(exec=B.SSV_EXEC_UNFUSED, mode=B.SSV_REUSE)).n_launches == 7
    rows = 8 * 64
    assert un.workspace_bytes >= 3 * rows * 128 * 2 + un.n_slots * rows * 130 * 4


def test_plan_workspace_and_verify_agree():
    """One set of checks serves the three entry points: whatever the plan query accepts, the workspace query sizes
    and verify accepts (up to its pointer checks), and the reverse."""
    fake = 4096
    grid = [dict(), dict(T=32, H=16, H_kv=4, n_sel=32, group_size=32), dict(T=32, H=16, H_kv=4, n_sel=32, group_size=16),
            dict(T=64, H=8, H_kv=4, n_sel=32, group_size=64), dict(T=64, H=8, H_kv=4, n_sel=16, group_size=64),
            dict(d_k=64, d_v=64, T=64, H=8, H_kv=4, n_sel=32, group_size=64), dict(exec=B.SSV_EXEC_UNFUSED)]
    seen = set()
    for over in grid:
        p = std_params(**over)
        try:
            B.ssv_nsa_plan_query(p)
            plan_rc = B.SSV_OK
        except B.SsvError as e:
            plan_rc = e.code
        need = B.ssv_nsa_workspace_bytes(p)
        assert (need > 0) == (plan_rc == B.SSV_OK)
        with pytest.raises(B.SsvError) as e:      # a null query pointer: the first check after the parameters
            B.ssv_nsa_verify(None, fake, fake, fake, fake, fake, fake, fake, None, None, p, fake, fake, fake, 1 << 40, 0)
        assert e.value.code == (B.SSV_EINVAL if plan_rc == B.SSV_OK else plan_rc), over
        seen.add(plan_rc)
    assert seen == {B.SSV_OK, B.SSV_EUNSUPPORTED}


def test_shared_index_plan_keeps_the_automatic_grouping():
    p = std_params(mode=B.SSV_REFRESH_SHARED, group_size=2)
    plan = B.ssv_nsa_plan_query(p)
    auto = B.ssv_nsa_plan_query(std_params())
    assert plan.share_group == 2 and plan.C == auto.C and auto.share_group == 0
    assert B.ssv_nsa_plan_query(std_params(mode=B.SSV_REFRESH_SHARED)).share_group == auto.C
    # T = 8 queries may share one set even though a workgroup holds only 4 of them
    assert B.ssv_nsa_plan_query(std_params(mode=B.SSV_REFRESH_SHARED, group_size=8)).share_group == 8


def cmp_params(**over):
    kw = dict(B=2, H_kv=4, d_k=192, d_v=128, l=32, d=16, dtype=B.SSV_BF16, max_new_rows=8, kv_capacity=4096,
              cmp_capacity=256, k_stride=(4 * 4096 * 192, 4096 * 192, 192), v_stride=(4 * 4096 * 128, 4096 * 128, 128),
              kc_stride=(4 * 256 * 192, 256 * 192, 192), vc_stride=(4 * 256 * 128, 256 * 128, 128))
    kw.update(over)
    return B.make_cmp_params(**kw)


@pytest.mark.parametrize("over,code", [
    (dict(B=0), B.SSV_EINVAL), (dict(l=32, d=12), B.SSV_EINVAL), (dict(dtype=5), B.SSV_EINVAL),
    (dict(max_new_rows=0), B.SSV_EINVAL), (dict(cmp_capacity=0), B.SSV_EINVAL), (dict(d_k=100), B.SSV_EINVAL),
    (dict(k_stride=(1, 1, 100)), B.SSV_EINVAL), (dict(l=2048, d=16), B.SSV_EUNSUPPORTED), (dict(d_k=2048, k_stride=(4 * 4096 * 2048, 4096 * 2048, 2048), kc_stride=(4 * 256 * 2048, 256 * 2048, 2048)), B.SSV_EUNSUPPORTED),
])
def test_compress_rejects_bad_parameters_without_a_launch(over, code):
    assert ctypes.sizeof(B.SsvCmpParams) == 10 * 4 + 12 * 8
    fake = 4096
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_compress(fake, fake, fake, fake, None, fake, fake, cmp_params(**over), 0)
    assert e.value.code == code
    with pytest.raises(B.SsvError) as e:
        B.ssv_nsa_compress(fake, fake, fake, None, None, fake, fake, cmp_params(), 0)
    assert e.value.code == B.SSV_EINVAL
