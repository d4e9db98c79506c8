"""TEST INFRASTRUCTURE: ctypes front end of the fp64 CPU oracle (nsa_verify_oracle.c).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It shares nothing with the HIP library and does not import it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nsa_verify_oracle.c")
_LIB = os.path.join(_HERE, "libnsa_verify_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP) into oracle/libnsa_verify_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "T", "H", "H_kv", "d_k", "d_v", "l", "d", "l_sel", "n_sel", "w", "n_init", "n_local",
                 "dtype", "reuse", "n_threads")] + \
               [("S_cap", ctypes.c_int64), ("NC_cap", ctypes.c_int64), ("NS_cap", ctypes.c_int64),
                ("scale", ctypes.c_double)]


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.ssv_oracle_nsa_verify.restype = ctypes.c_int
        _lib.ssv_oracle_nsa_verify.argtypes = [ctypes.c_void_p] * 20
        _lib.ssv_oracle_threads.restype = ctypes.c_int
    return _lib


def default_threads() -> int:
    return int(_load().ssv_oracle_threads())


@dataclass
class OracleResult:
    out: np.ndarray                 # float64 [B, T, H, d_v]
    sel_idx: np.ndarray             # int32 [B, T, H_kv, n_sel]
    gap: Optional[np.ndarray]       # float64 [B, T, H_kv] (refresh mode only)
    o_cmp: Optional[np.ndarray] = None
    o_slc: Optional[np.ndarray] = None
    o_win: Optional[np.ndarray] = None
    imp: Optional[np.ndarray] = None      # float64 [B, T, H_kv, NS_cap]
    p_cmp: Optional[np.ndarray] = None    # float64 [B, T, H, NC_cap]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def nsa_verify(case, *, sel_idx: Optional[np.ndarray] = None, scale: float = 0.0, branches: bool = False,
               want_imp: bool = False, want_p: bool = False, query_mask: Optional[np.ndarray] = None,
               n_threads: int = 0) -> OracleResult:
    """Run the oracle on a batch (any object with the fields of ssv_inputs.VerifyCase).

    sel_idx given  -> reuse mode (indices are an input);  None -> they are computed.
    """
    lib = _load()
    nsa = case.nsa
    B, T, H, H_kv = case.B, case.T, case.H, case.H_kv
    reuse = sel_idx is not None
    if reuse:
        sel = np.ascontiguousarray(sel_idx, dtype=np.int32).reshape(B, T, H_kv, nsa.n_sel).copy()
    else:
        sel = np.full((B, T, H_kv, nsa.n_sel), -1, np.int32)
    NS_cap = (int(case.seq_lens.max()) + T) // nsa.l_sel + 1
    prm = _Params(B=B, T=T, H=H, H_kv=H_kv, d_k=case.d_k, d_v=case.d_v, l=nsa.l, d=nsa.d, l_sel=nsa.l_sel,
                  n_sel=nsa.n_sel, w=nsa.w, n_init=nsa.n_init, n_local=nsa.n_local,
                  dtype=0 if case.dtype == "f32" else 1, reuse=int(reuse), n_threads=int(n_threads),
                  S_cap=case.k.shape[2], NC_cap=case.k_cmp.shape[2], NS_cap=NS_cap, scale=float(scale))
    arrays = [np.ascontiguousarray(a) for a in (case.q, case.k, case.v, case.k_cmp, case.v_cmp)]
    gates = np.ascontiguousarray(case.gates, dtype=np.float32)
    seq = np.ascontiguousarray(case.seq_lens, dtype=np.int32)
    ncmp = np.ascontiguousarray(case.n_cmp, dtype=np.int32)
    nq = np.ascontiguousarray(case.n_query, dtype=np.int32)
    par = None if case.parents is None else np.ascontiguousarray(case.parents, dtype=np.int32)
    out = np.zeros((B, T, H, case.d_v), np.float64)
    gap = None if reuse else np.full((B, T, H_kv), np.inf, np.float64)
    oc = np.zeros_like(out) if branches else None
    os_ = np.zeros_like(out) if branches else None
    ow = np.zeros_like(out) if branches else None
    imp = np.zeros((B, T, H_kv, NS_cap), np.float64) if want_imp else None
    pc = np.zeros((B, T, H, case.k_cmp.shape[2]), np.float64) if want_p else None
    qm = None if query_mask is None else np.ascontiguousarray(query_mask, dtype=np.uint8).reshape(B, T)
    rc = lib.ssv_oracle_nsa_verify(ctypes.byref(prm), *[_ptr(a) for a in arrays], _ptr(gates), _ptr(seq),
                                   _ptr(ncmp), _ptr(nq), _ptr(par), _ptr(sel), _ptr(out), _ptr(gap), _ptr(oc),
                                   _ptr(os_), _ptr(ow), _ptr(imp), _ptr(pc), _ptr(qm))
    if rc != 0:
        raise ValueError(f"oracle rejected its arguments (code {rc})")
    return OracleResult(out=out, sel_idx=sel, gap=gap, o_cmp=oc, o_slc=os_, o_win=ow, imp=imp, p_cmp=pc)


def group_representatives(case, C: int) -> np.ndarray:
    """Representative verifier query of every group of C consecutive queries (flattened order), [B, T] int32.

    Approximate shared-index variant (Section 4.3): the representative is the member with the longest
    prefix, i.e. the largest position L + depth; among equally deep members (a tree) the last one in
    flattened order.  In a linear chain that is the last query of the group.  Entry [b, i] is the
    representative of i's group, -1 for i >= n_query[b].
    """
    B, T = case.B, case.T
    rep = np.full((B, T), -1, np.int32)
    for b in range(B):
        Tq = int(case.n_query[b])
        depth = np.zeros(Tq, np.int64)
        for i in range(Tq):
            par = i - 1 if case.parents is None else int(case.parents[b, i])
            depth[i] = 0 if par < 0 else depth[par] + 1
        for g0 in range(0, Tq, C):
            members = range(g0, min(g0 + C, Tq))
            best = max(members, key=lambda i: (depth[i], i))
            rep[b, g0:min(g0 + C, Tq)] = best
    return rep


def nsa_verify_shared(case, C: int, *, scale: float = 0.0, branches: bool = False, n_threads: int = 0) -> OracleResult:
    """Approximate shared-index variant (Section 4.3), as its three steps: (1) one representative per group of
    C queries; (2) the selected block set is computed for the representative alone (exact selection of
    that query); (3) every query of the group attends to that set, under its own visibility, position and
    window (the compressed and window branches are those of the exact variant).  sel_idx and gap of the
    result hold the representative's set and boundary gap in every member's row.
    """
    rep = group_representatives(case, C)
    B, T = case.B, case.T
    mask = np.zeros((B, T), np.uint8)
    for b in range(B):
        for i in range(int(case.n_query[b])):
            mask[b, rep[b, i]] = 1
    routed = nsa_verify(case, scale=scale, query_mask=mask, n_threads=n_threads)
    sel = np.full_like(routed.sel_idx, -1)
    gap = np.full_like(routed.gap, np.inf)
    for b in range(B):
        for i in range(int(case.n_query[b])):
            sel[b, i] = routed.sel_idx[b, rep[b, i]]
            gap[b, i] = routed.gap[b, rep[b, i]]
    res = nsa_verify(case, sel_idx=sel, scale=scale, branches=branches, n_threads=n_threads)
    res.gap = gap
    return res
