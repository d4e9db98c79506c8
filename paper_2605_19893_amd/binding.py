"""Thin ctypes binding of libssv_nsa.so (include/ssv_nsa.h): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI.  PyTorch appears here only as the
owner of device memory and of the stream; nothing in this module computes on tensors.  There is
no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssv_nsa.so")

SSV_OK, SSV_EINVAL, SSV_EUNSUPPORTED, SSV_EWORKSPACE, SSV_ELAUNCH, SSV_ESTATIC = 0, -1, -2, -3, -4, -5
SSV_STATIC_SCRATCH_BYTES = 32 << 20
SSV_F32, SSV_BF16 = 0, 1
SSV_REFRESH, SSV_REUSE, SSV_REFRESH_SHARED = 0, 1, 2
SSV_MAX_T = 128
(SSV_K_STREAM_A, SSV_K_IMPORTANCE, SSV_K_TOPN, SSV_K_STREAM_B, SSV_K_COMBINE, SSV_K_STREAM_W, SSV_K_OUT_CMP, SSV_K_OUT_SLC,
 SSV_K_OUT_WIN) = range(9)
SSV_NUM_KERNELS = 9
SSV_T_EVENT_PAIR, SSV_NUM_TIMINGS = 9, 10
SSV_EXEC_FUSED, SSV_EXEC_UNFUSED = 0, 1
SSV_TOPN_AUTO, SSV_TOPN_SEPARATE, SSV_TOPN_IN_SLC = 0, 1, 2
SSV_SCAN_AUTO, SSV_SCAN_STREAM, SSV_SCAN_MATRIX, SSV_SCAN_STREAM_TABLE = 0, 1, 2, 3

EXPORTS = ("ssv_nsa_verify", "ssv_nsa_verify_static", "ssv_nsa_verify_timed", "ssv_nsa_plan_query", "ssv_nsa_workspace_bytes",
           "ssv_nsa_supported", "ssv_nsa_strerror", "ssv_nsa_kernel_name", "ssv_nsa_version", "ssv_nsa_compress",
           "ssv_guard_default_config", "ssv_guard_init", "ssv_guard_observe", "ssv_tree_flatten")
SSV_GUARD_MAX_CANDIDATES = 16
SSV_TREE_BFS, SSV_TREE_DFS = 0, 1


class SsvNsaParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "T", "H", "H_kv", "d_k", "d_v", "l", "d", "l_sel", "n_sel", "w", "n_init", "n_local",
                 "dtype", "mode", "group_size")] + \
               [("scale", ctypes.c_float), ("max_seq_len", ctypes.c_int32), ("max_n_cmp", ctypes.c_int32),
                ("avg_seq_len", ctypes.c_int32), ("scan_group_size", ctypes.c_int32)] + \
               [(n, ctypes.c_int64 * 3) for n in ("k_stride", "v_stride", "kc_stride", "vc_stride", "q_stride", "out_stride")] + \
               [(n, ctypes.c_int32) for n in ("exec", "topn_home", "max_slice_tiles", "imp_rows", "scan_kernel")]


class SsvCmpParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "H_kv", "d_k", "d_v", "l", "d", "dtype", "max_new_rows", "kv_capacity", "cmp_capacity")] + \
               [(n, ctypes.c_int64 * 3) for n in ("k_stride", "v_stride", "kc_stride", "vc_stride")]


class SsvGuardConfig(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("ratio", ctypes.c_double), ("warmup_steps", ctypes.c_int32),
                ("patience", ctypes.c_int32), ("max_transitions", ctypes.c_int32), ("early_steps", ctypes.c_int32)]


class SsvGuardState(ctypes.Structure):
    _fields_ = [("cfg", SsvGuardConfig)] + \
               [(n, ctypes.c_int32) for n in ("n_candidates", "active", "transitions", "settled", "total_steps",
                                              "steps_on_active", "below_streak", "has_ema")] + \
               [("ema", ctypes.c_double), ("expected", ctypes.c_double * SSV_GUARD_MAX_CANDIDATES),
                ("valid", ctypes.c_uint8 * SSV_GUARD_MAX_CANDIDATES), ("explored", ctypes.c_uint8 * SSV_GUARD_MAX_CANDIDATES),
                ("sum_accepted", ctypes.c_double * SSV_GUARD_MAX_CANDIDATES),
                ("sum_latency", ctypes.c_double * SSV_GUARD_MAX_CANDIDATES)]


class SsvNsaPlan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("C", "n_qg", "rows_per_wg", "n_cmp_chunks", "tiles_per_chunk", "n_win_splits", "n_slc_splits",
                 "min_tiles_per_split", "n_slots", "max_sched_entries", "share_group", "C_scan", "n_qg_scan", "topn_in_slc",
                 "n_imp_chunks", "imp_rows", "n_launches", "scan_matrix")] + [("workspace_bytes", ctypes.c_int64)]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class SsvError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (code {code})")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built HIP library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run __graft_entry__.build() (hipcc, gfx950) first")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        common = [vp] * 5 + [vp, i32p, i32p, i32p, i32p, ctypes.POINTER(SsvNsaParams), vp, i32p, vp, ctypes.c_size_t, vp]
        lib.ssv_nsa_verify.restype = ctypes.c_int
        lib.ssv_nsa_verify.argtypes = common
        lib.ssv_nsa_verify_static.restype = ctypes.c_int
        lib.ssv_nsa_verify_static.argtypes = common[:13] + [vp]
        lib.ssv_nsa_verify_timed.restype = ctypes.c_int
        lib.ssv_nsa_verify_timed.argtypes = common + [ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
        lib.ssv_nsa_plan_query.restype = ctypes.c_int
        lib.ssv_nsa_plan_query.argtypes = [ctypes.POINTER(SsvNsaParams), ctypes.POINTER(SsvNsaPlan)]
        lib.ssv_nsa_workspace_bytes.restype = ctypes.c_size_t
        lib.ssv_nsa_workspace_bytes.argtypes = [ctypes.POINTER(SsvNsaParams)]
        lib.ssv_nsa_supported.restype = ctypes.c_int
        lib.ssv_nsa_supported.argtypes = [ctypes.c_int32] * 3
        lib.ssv_nsa_strerror.restype = ctypes.c_char_p
        lib.ssv_nsa_strerror.argtypes = [ctypes.c_int]
        lib.ssv_nsa_kernel_name.restype = ctypes.c_char_p
        lib.ssv_nsa_kernel_name.argtypes = [ctypes.c_int]
        lib.ssv_nsa_version.restype = ctypes.c_int
        lib.ssv_guard_default_config.restype = None
        lib.ssv_guard_default_config.argtypes = [ctypes.POINTER(SsvGuardConfig)]
        lib.ssv_guard_init.restype = ctypes.c_int
        lib.ssv_guard_init.argtypes = [ctypes.POINTER(SsvGuardState), ctypes.POINTER(SsvGuardConfig),
                                       ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint8), ctypes.c_int32]
        lib.ssv_guard_observe.restype = ctypes.c_int
        lib.ssv_guard_observe.argtypes = [ctypes.POINTER(SsvGuardState), ctypes.c_double, ctypes.c_double]
        lib.ssv_tree_flatten.restype = ctypes.c_int
        lib.ssv_tree_flatten.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, ctypes.c_int32,
                                         ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
        lib.ssv_nsa_compress.restype = ctypes.c_int
        lib.ssv_nsa_compress.argtypes = [vp] * 4 + [i32p] * 3 + [ctypes.POINTER(SsvCmpParams), vp]
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load_library().ssv_nsa_strerror(code).decode()


def kernel_name(idx: int) -> str:
    return load_library().ssv_nsa_kernel_name(idx).decode()


def make_params(*, B, T, H, H_kv, d_k, d_v, l, d, l_sel, n_sel, w, n_init=1, n_local=2, dtype=SSV_BF16,
                mode=SSV_REFRESH, group_size=0, scale=0.0, max_seq_len, max_n_cmp, avg_seq_len=0, scan_group_size=0, k_stride, v_stride, kc_stride,
                vc_stride, q_stride=(0, 0, 0), out_stride=(0, 0, 0), exec=SSV_EXEC_FUSED, topn_home=SSV_TOPN_AUTO,
                max_slice_tiles=0, imp_rows=0, scan_kernel=SSV_SCAN_AUTO) -> SsvNsaParams:
    p = SsvNsaParams(B=B, T=T, H=H, H_kv=H_kv, d_k=d_k, d_v=d_v, l=l, d=d, l_sel=l_sel, n_sel=n_sel, w=w,
                     n_init=n_init, n_local=n_local, dtype=dtype, mode=mode, group_size=group_size, scale=scale,
                     max_seq_len=max_seq_len, max_n_cmp=max_n_cmp, avg_seq_len=avg_seq_len, scan_group_size=scan_group_size,
                     exec=exec, topn_home=topn_home, max_slice_tiles=max_slice_tiles, imp_rows=imp_rows,
                     scan_kernel=scan_kernel)
    for name, st in (("k_stride", k_stride), ("v_stride", v_stride), ("kc_stride", kc_stride), ("vc_stride", vc_stride),
                     ("q_stride", q_stride), ("out_stride", out_stride)):
        setattr(p, name, (ctypes.c_int64 * 3)(*[int(x) for x in st]))
    return p


def ssv_nsa_plan_query(p: SsvNsaParams) -> SsvNsaPlan:
    plan = SsvNsaPlan()
    rc = load_library().ssv_nsa_plan_query(ctypes.byref(p), ctypes.byref(plan))
    if rc != SSV_OK:
        raise SsvError(rc, "ssv_nsa_plan_query")
    return plan


def ssv_nsa_workspace_bytes(p: SsvNsaParams) -> int:
    return int(load_library().ssv_nsa_workspace_bytes(ctypes.byref(p)))


def ssv_nsa_supported(dtype: int, d_k: int, d_v: int) -> bool:
    return bool(load_library().ssv_nsa_supported(dtype, d_k, d_v))


def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or a raw integer address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def ssv_nsa_verify(q, k, v, k_cmp, v_cmp, gates, seq_lens, n_cmp, n_query, tree_parents, p: SsvNsaParams, out, sel_idx,
                   workspace, workspace_bytes: int, stream: int, kernel_ms=None, repeats: int = 1) -> None:
    """Enqueue one verification call on `stream` (a hipStream_t as an integer).

    Tensors are device tensors (or integer device addresses); `p` describes shapes and strides.
    With kernel_ms (a list), the timed entry point is used: every kernel runs `repeats` times back to
    back, the stream is synchronised, and the average per-kernel durations (ms) are appended to the list.
    """
    lib = load_library()
    args = [_ptr(q), _ptr(k), _ptr(v), _ptr(k_cmp), _ptr(v_cmp), _ptr(gates), _ptr(seq_lens), _ptr(n_cmp),
            _ptr(n_query), _ptr(tree_parents), ctypes.byref(p), _ptr(out), _ptr(sel_idx), _ptr(workspace),
            ctypes.c_size_t(int(workspace_bytes)), ctypes.c_void_p(int(stream))]
    if kernel_ms is None:
        rc = lib.ssv_nsa_verify(*args)
    else:
        ms = (ctypes.c_float * SSV_NUM_TIMINGS)()
        rc = lib.ssv_nsa_verify_timed(*args, int(repeats), ms)
        kernel_ms.extend(float(x) for x in ms)
    if rc != SSV_OK:
        raise SsvError(rc, "ssv_nsa_verify")


def ssv_nsa_verify_static(q, k, v, k_cmp, v_cmp, gates, seq_lens, n_cmp, n_query, tree_parents, p: SsvNsaParams, out, sel_idx,
                          stream: int) -> None:
    """ssv_nsa_verify on the library's own fixed scratch array: no workspace argument, nothing allocated."""
    rc = load_library().ssv_nsa_verify_static(_ptr(q), _ptr(k), _ptr(v), _ptr(k_cmp), _ptr(v_cmp), _ptr(gates), _ptr(seq_lens),
                                              _ptr(n_cmp), _ptr(n_query), _ptr(tree_parents), ctypes.byref(p), _ptr(out),
                                              _ptr(sel_idx), ctypes.c_void_p(int(stream)))
    if rc != SSV_OK:
        raise SsvError(rc, "ssv_nsa_verify_static")


def make_cmp_params(*, B, H_kv, d_k, d_v, l, d, dtype, max_new_rows, kv_capacity, cmp_capacity, k_stride, v_stride,
                    kc_stride, vc_stride) -> SsvCmpParams:
    p = SsvCmpParams(B=B, H_kv=H_kv, d_k=d_k, d_v=d_v, l=l, d=d, dtype=dtype, max_new_rows=max_new_rows,
                     kv_capacity=kv_capacity, cmp_capacity=cmp_capacity)
    for name, st in (("k_stride", k_stride), ("v_stride", v_stride), ("kc_stride", kc_stride), ("vc_stride", vc_stride)):
        setattr(p, name, (ctypes.c_int64 * 3)(*[int(x) for x in st]))
    return p


def ssv_nsa_compress(k, v, k_cmp, v_cmp, committed_before, committed_after, n_cmp, p: SsvCmpParams, stream: int) -> None:
    """Enqueue the construction of the compressed rows that become complete between two committed lengths."""
    rc = load_library().ssv_nsa_compress(_ptr(k), _ptr(v), _ptr(k_cmp), _ptr(v_cmp), _ptr(committed_before),
                                         _ptr(committed_after), _ptr(n_cmp), ctypes.byref(p), ctypes.c_void_p(int(stream)))
    if rc != SSV_OK:
        raise SsvError(rc, "ssv_nsa_compress")


def ssv_guard_default_config() -> SsvGuardConfig:
    cfg = SsvGuardConfig()
    load_library().ssv_guard_default_config(ctypes.byref(cfg))
    return cfg


def ssv_guard_init(cfg: SsvGuardConfig, expected, valid=None) -> SsvGuardState:
    n = len(expected)
    state = SsvGuardState()
    exp = (ctypes.c_double * max(n, 1))(*[float(x) for x in expected])
    val = None if valid is None else (ctypes.c_uint8 * max(n, 1))(*[1 if x else 0 for x in valid])
    rc = load_library().ssv_guard_init(ctypes.byref(state), ctypes.byref(cfg), exp, val, n)
    if rc != SSV_OK:
        raise SsvError(rc, "ssv_guard_init")
    return state


def ssv_guard_observe(state: SsvGuardState, accepted_tokens: float, step_latency: float) -> int:
    rc = load_library().ssv_guard_observe(ctypes.byref(state), float(accepted_tokens), float(step_latency))
    if rc < 0:
        raise SsvError(rc, "ssv_guard_observe")
    return rc


def ssv_tree_flatten(parents, order: int):
    """(perm, new_parents) as Python lists; perm[new] = old."""
    n = len(parents)
    par = (ctypes.c_int32 * max(n, 1))(*[int(x) for x in parents])
    perm, newp = (ctypes.c_int32 * max(n, 1))(), (ctypes.c_int32 * max(n, 1))()
    rc = load_library().ssv_tree_flatten(par, n, order, perm, newp)
    if rc != SSV_OK:
        raise SsvError(rc, "ssv_tree_flatten")
    return list(perm)[:n], list(newp)[:n]
