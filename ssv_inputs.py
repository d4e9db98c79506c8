"""Seeded synthetic inputs for NSA speculative verification.

This module only draws random numbers, rounds them to the storage dtype and lays them
out in memory.  It contains none of the attention arithmetic: both the CPU oracle and
the HIP path receive the arrays produced here, and neither of them is imported here.

The workloads stand in for the trained-model KV caches and draft traces that the
paper measures on (Section 7, evaluation setup): Gaussian Q/K/V, verifier queries with
a controlled cross-query correlation rho (which controls the overlap of the selected
blocks of adjacent queries, the quantity the paper's kernel benchmark varies), linear
draft chains and draft trees given by parent indices.

Array layout (C order):
  q      [B, T, H, d_k]
  k      [B, H_kv, S_cap, d_k]      slot s < L: committed token s; slot L+i: draft token i
  v      [B, H_kv, S_cap, d_v]
  k_cmp  [B, H_kv, NC_cap, d_k]     mean over slots [c*d, c*d+l) of k (a stand-in for the
  v_cmp  [B, H_kv, NC_cap, d_v]     learned compression map; an input of the hot path)
  gates  [B, T, H, 3] float32       (cmp, slc, win)
bf16 arrays are numpy uint16 holding the bit patterns; f32 arrays are float32.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Optional

import numpy as np

BASE_SEED = 20260519


# --------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    return x if dtype == "f32" else bf16_bits_to_f32(x)


def storage_np_dtype(dtype: str):
    return np.float32 if dtype == "f32" else np.uint16


# --------------------------------------------------------------------------- containers
@dataclass
class NsaParams:
    l: int = 32          # compression block length
    d: int = 16          # compression stride
    l_sel: int = 64      # selection block size l'
    n_sel: int = 16      # selected blocks per query (forced ones included)
    w: int = 512         # sliding window
    n_init: int = 1      # forced leading blocks
    n_local: int = 2     # forced blocks ending at the query's own block


@dataclass
class VerifyCase:
    name: str
    dtype: str
    B: int
    T: int
    H: int
    H_kv: int
    d_k: int
    d_v: int
    nsa: NsaParams
    seq_lens: np.ndarray            # int32 [B]
    n_query: np.ndarray             # int32 [B]
    n_cmp: np.ndarray               # int32 [B]
    parents: Optional[np.ndarray]   # int32 [B, T] or None (= linear chain)
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    k_cmp: np.ndarray
    v_cmp: np.ndarray
    gates: np.ndarray
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def S_cap(self) -> int:
        return self.k.shape[2]

    @property
    def NC_cap(self) -> int:
        return self.k_cmp.shape[2]

    @property
    def H_g(self) -> int:
        return self.H // self.H_kv

    def total_queries(self) -> int:
        return int(self.n_query.sum())


def n_cmp_blocks(x: int, l: int, d: int) -> int:
    """Number of complete compression windows inside the first x slots."""
    return 0 if x < l else (x - l) // d + 1


# --------------------------------------------------------------------------- trees
def chain_parents(T: int) -> np.ndarray:
    return np.arange(-1, T - 1, dtype=np.int32)


def tree_parents(fanouts, order: str = "bfs") -> np.ndarray:
    """Parent indices of a uniform draft tree (fanouts[0] children of the last committed
    token, each with fanouts[1] children, ...), flattened breadth-first or depth-first.
    Parents always precede their children in both orders."""
    if order == "bfs":
        par, level = [], [-1]
        for f in fanouts:
            nxt = []
            for p in level:
                for _ in range(f):
                    par.append(p)
                    nxt.append(len(par) - 1)
            level = nxt
        return np.asarray(par, dtype=np.int32)
    if order == "dfs":
        par = []

        def rec(p, depth):
            if depth == len(fanouts):
                return
            for _ in range(fanouts[depth]):
                par.append(p)
                rec(len(par) - 1, depth + 1)

        rec(-1, 0)
        return np.asarray(par, dtype=np.int32)
    raise ValueError(order)


def node_depths(parents: np.ndarray) -> np.ndarray:
    dep = np.zeros(len(parents), dtype=np.int32)
    for i, p in enumerate(parents):
        dep[i] = 0 if p < 0 else dep[p] + 1
    return dep


def root_branch(parents: np.ndarray) -> np.ndarray:
    """Index of the depth-0 ancestor (the root subtree) of every node."""
    br = np.zeros(len(parents), dtype=np.int32)
    nroot = 0
    for i, p in enumerate(parents):
        if p < 0:
            br[i] = nroot
            nroot += 1
        else:
            br[i] = br[p]
    return br


# --------------------------------------------------------------------------- generation
def _rng(seed: int, *tags: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *tags])))


def _pool_slice(x_f32: np.ndarray, n_blocks: int, l: int, d: int) -> np.ndarray:
    """Mean over windows [c*d, c*d+l) of the rows of x (rows, dim), c < n_blocks."""
    dim = x_f32.shape[1]
    if n_blocks <= 0:
        return np.zeros((0, dim), np.float32)
    if l % d == 0:
        per = l // d
        nchunk = n_blocks + per - 1
        chunks = x_f32[: nchunk * d].reshape(nchunk, d, dim).sum(axis=1, dtype=np.float64)
        acc = chunks[:n_blocks].copy()
        for m in range(1, per):
            acc += chunks[m:m + n_blocks]
    else:
        acc = np.stack([x_f32[c * d:c * d + l].sum(axis=0, dtype=np.float64) for c in range(n_blocks)])
    return (acc / l).astype(np.float32)


def _fill_kv(case: VerifyCase, seed: int, heavy_frac: float = 0.0, heavy_scale: float = 4.0,
             slot_from: Optional[np.ndarray] = None, workers: int = 8,
             needle_blocks: Optional[dict] = None, poison_pad: bool = False) -> None:
    """Draw K, V ~ N(0,1) for the slots [slot_from[b], L_b + T) of each sequence, round to the
    storage dtype, and (re)pool k_cmp / v_cmp for every complete window.  Slots below
    slot_from[b] keep their current contents (used when a serving step appends tokens)."""
    B, H_kv, nsa = case.B, case.H_kv, case.nsa
    if slot_from is None:
        slot_from = np.zeros(B, dtype=np.int64)
    heavy = {}
    if heavy_frac > 0:
        for b in range(B):
            used = int(case.seq_lens[b]) + case.T
            heavy[b] = _rng(seed, 7, b).random(used) < heavy_frac

    def work(item):
        b, h = item
        used = int(case.seq_lens[b]) + case.T
        s0 = int(slot_from[b])
        for name, arr, cmp_arr, dim, tag in (("k", case.k, case.k_cmp, case.d_k, 1),
                                             ("v", case.v, case.v_cmp, case.d_v, 2)):
            x = _rng(seed, tag, b, h).standard_normal((used - s0, dim), dtype=np.float32)
            if name == "k" and heavy_frac > 0:
                x[heavy[b][s0:used]] *= heavy_scale
            if name == "k" and needle_blocks and b in needle_blocks:
                for blk, gain in needle_blocks[b]:
                    lo, hi = blk * nsa.l_sel - s0, (blk + 1) * nsa.l_sel - s0
                    if hi > 0:
                        x[max(lo, 0):hi] *= gain
            arr[b, h, s0:used] = to_storage(x, case.dtype)
            if poison_pad and used < arr.shape[2]:
                arr[b, h, used:] = np.nan if case.dtype == "f32" else 0x7FC0
            nc = int(case.n_cmp[b])
            full = to_f32(arr[b, h, : (nc - 1) * nsa.d + nsa.l] if nc > 0 else arr[b, h, :0], case.dtype)
            cmp_arr[b, h, :nc] = to_storage(_pool_slice(full, nc, nsa.l, nsa.d), case.dtype)
            if poison_pad and nc < cmp_arr.shape[2]:
                cmp_arr[b, h, nc:] = np.nan if case.dtype == "f32" else 0x7FC0

    items = [(b, h) for b in range(B) for h in range(H_kv)]
    if workers > 1 and len(items) > 1:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(work, items))
    else:
        for it in items:
            work(it)


def make_case(name: str, dtype: str, B: int, T: int, H: int, H_kv: int, d_k: int, d_v: int,
              nsa: NsaParams, seq_lens, seed: int, rho=0.0, parents: Optional[np.ndarray] = None,
              n_query=None, cmp_over_drafts: Optional[bool] = None, heavy_frac: float = 0.0,
              needle_blocks: Optional[dict] = None, poison_pad: bool = False,
              workers: int = 8) -> VerifyCase:
    """Build one verification batch.

    rho: scalar, or array [B, T] of per-query correlations with the per-(sequence, head)
         shared query direction: q_i = sqrt(rho) q_shared + sqrt(1-rho) eps_i.
    parents: int32 [T] or [B, T]; None = linear chain (parents[i] = i-1).
    cmp_over_drafts: pool compressed blocks over committed + draft slots (default for
         chains, where it equals what autoregressive decoding would have built) or over
         the committed prefix only (default for trees: deferred commit).
    """
    seq_lens = np.asarray(seq_lens, dtype=np.int32).reshape(B)
    n_query = np.full(B, T, np.int32) if n_query is None else np.asarray(n_query, np.int32).reshape(B)
    if parents is not None:
        parents = np.asarray(parents, dtype=np.int32)
        if parents.ndim == 1:
            parents = np.broadcast_to(parents, (B, T)).copy()
    is_chain = parents is None or all(np.array_equal(parents[b], chain_parents(T)) for b in range(B))
    if cmp_over_drafts is None:
        cmp_over_drafts = is_chain
    n_cmp = np.asarray([n_cmp_blocks(int(seq_lens[b]) + (int(n_query[b]) if cmp_over_drafts else 0), nsa.l, nsa.d)
                        for b in range(B)], dtype=np.int32)
    max_used = int(seq_lens.max()) + T
    S_cap = -(-max_used // nsa.l_sel) * nsa.l_sel
    NC_cap = max(1, n_cmp_blocks(max_used, nsa.l, nsa.d))
    st = storage_np_dtype(dtype)
    case = VerifyCase(
        name=name, dtype=dtype, B=B, T=T, H=H, H_kv=H_kv, d_k=d_k, d_v=d_v, nsa=nsa,
        seq_lens=seq_lens, n_query=n_query, n_cmp=n_cmp, parents=parents,
        q=np.zeros((B, T, H, d_k), st), k=np.zeros((B, H_kv, S_cap, d_k), st),
        v=np.zeros((B, H_kv, S_cap, d_v), st), k_cmp=np.zeros((B, H_kv, NC_cap, d_k), st),
        v_cmp=np.zeros((B, H_kv, NC_cap, d_v), st), gates=np.zeros((B, T, H, 3), np.float32), seed=seed)
    _fill_kv(case, seed, heavy_frac=heavy_frac, workers=workers, needle_blocks=needle_blocks,
             poison_pad=poison_pad)
    _fill_queries(case, seed, rho)
    return case


def _fill_queries(case: VerifyCase, seed: int, rho) -> None:
    B, T, H, d_k = case.B, case.T, case.H, case.d_k
    rho = np.broadcast_to(np.asarray(rho, dtype=np.float32), (B, T)).reshape(B, T, 1, 1)
    g = _rng(seed, 3)
    q_shared = g.standard_normal((B, 1, H, d_k), dtype=np.float32)
    eps = g.standard_normal((B, T, H, d_k), dtype=np.float32)
    case.q[...] = to_storage(np.sqrt(rho) * q_shared + np.sqrt(1.0 - rho) * eps, case.dtype)
    case.gates[...] = _rng(seed, 4).random((B, T, H, 3), dtype=np.float32)
    case.extra["rho"] = rho.reshape(B, T).copy()


# --------------------------------------------------------------------------- named configs
STD_NSA = NsaParams(l=32, d=16, l_sel=64, n_sel=16, w=512)
TREE_FANOUTS = (4, 3, 2)   # 4 + 12 + 24 = 40 verifier queries


def config_seed(idx: int, step: int = 0) -> int:
    return BASE_SEED + idx + 1000 * step


def config0(seed: Optional[int] = None) -> VerifyCase:
    """Tiny fp32 case: B=1, L=2048, 4 query heads / 1 KV head, d=64, chain of 4."""
    return make_case("cfg0_tiny_f32", "f32", 1, 4, 4, 1, 64, 64,
                     NsaParams(l=32, d=16, l_sel=64, n_sel=4, w=128), [2048],
                     config_seed(0) if seed is None else seed)


def config1(rho: float = 0.5, L: int = 32768, seed: Optional[int] = None, T: int = 8) -> VerifyCase:
    """27B-style layer, bf16: B=1, 64 query heads / 4 KV heads, d_k=192, d_v=128, chain of 8."""
    return make_case(f"cfg1_b1_L{L}_T{T}_rho{rho}", "bf16", 1, T, 64, 4, 192, 128, STD_NSA, [L],
                     config_seed(1) if seed is None else seed, rho=rho)


def config2(B: int = 16, L: int = 65536, seed: Optional[int] = None) -> VerifyCase:
    """Batched verification, bf16: chains of 4, rho=0.7, 5 % of key positions scaled x4."""
    return make_case(f"cfg2_b{B}_L{L}_T4", "bf16", B, 4, 64, 4, 192, 128, STD_NSA, [L] * B,
                     config_seed(2) if seed is None else seed, rho=0.7, heavy_frac=0.05)


def config3(order: str = "bfs", B: int = 4, L: int = 131072, seed: Optional[int] = None) -> VerifyCase:
    """Tree verification, bf16: 40-node draft tree, rho drawn per root subtree ~ U(0.3, 0.95)."""
    seed = config_seed(3) if seed is None else seed
    par = tree_parents(TREE_FANOUTS, order)
    T = len(par)
    br = root_branch(par)
    rho_branch = _rng(seed, 5).uniform(0.3, 0.95, size=(B, TREE_FANOUTS[0])).astype(np.float32)
    rho = rho_branch[:, br]
    return make_case(f"cfg3_tree_{order}_b{B}_L{L}", "bf16", B, T, 64, 4, 192, 128, STD_NSA, [L] * B,
                     seed, rho=rho, parents=par)


def config4_lengths(B: int, seed: int, lo: int = 4096, hi: int = 131072) -> np.ndarray:
    u = _rng(seed, 6).uniform(math.log(lo), math.log(hi), size=B)
    return (np.round(np.exp(u) / 64.0).astype(np.int64) * 64).astype(np.int32)


def config4(B: int = 32, seed: Optional[int] = None, lo: int = 4096, hi: int = 131072, T: int = 16) -> VerifyCase:
    """Mixed-length serving batch, bf16: contexts log-uniform in [lo, hi] rounded to 64, chains of 16."""
    seed = config_seed(4) if seed is None else seed
    return make_case(f"cfg4_mixed_b{B}", "bf16", B, T, 64, 4, 192, 128, STD_NSA,
                     config4_lengths(B, seed, lo, hi), seed, rho=0.7)


def advance_case(case: VerifyCase, step: int = 1, accept: Optional[np.ndarray] = None) -> VerifyCase:
    """Second serving step: sequence b accepts a_b ~ U{0..T} draft tokens (their K/V stay in
    place as committed tokens), fresh draft K/V are drawn for the slots from the new length on,
    new queries and gates are drawn, and the compressed cache is re-pooled."""
    seed = case.seed + 1000 * step
    B, T = case.B, case.T
    if accept is None:
        accept = _rng(seed, 8).integers(0, T + 1, size=B)
    accept = np.asarray(accept, dtype=np.int32)
    new_len = (case.seq_lens + accept).astype(np.int32)
    max_used = int(new_len.max()) + T
    nsa = case.nsa
    S_cap = max(case.S_cap, -(-max_used // nsa.l_sel) * nsa.l_sel)
    NC_cap = max(case.NC_cap, n_cmp_blocks(max_used, nsa.l, nsa.d))

    def grow(a, cap):
        if a.shape[2] == cap:
            return a.copy()
        out = np.zeros(a.shape[:2] + (cap,) + a.shape[3:], a.dtype)
        out[:, :, : a.shape[2]] = a
        return out

    nxt = replace(case, name=case.name + f"_step{step + 1}", seq_lens=new_len,
                  n_cmp=np.asarray([n_cmp_blocks(int(new_len[b]) + T, nsa.l, nsa.d) for b in range(B)], np.int32),
                  q=np.zeros_like(case.q), gates=np.zeros_like(case.gates),
                  k=grow(case.k, S_cap), v=grow(case.v, S_cap),
                  k_cmp=grow(case.k_cmp, NC_cap), v_cmp=grow(case.v_cmp, NC_cap), seed=seed, extra={})
    _fill_kv(nxt, seed, slot_from=new_len.astype(np.int64))
    _fill_queries(nxt, seed, 0.7)
    nxt.extra["accept"] = accept
    return nxt


def planted_overlap_indices(case: VerifyCase, s: int, seed: int) -> np.ndarray:
    """Index sets for reuse-mode calls with a controlled overlap (the knob of the paper's kernel benchmark, Section
    7.3): along every chain, consecutive verifier queries share exactly `s` selected blocks, the mandatory initial
    and local blocks included (so s >= 3 at the standard parameters).  Sets are valid selections: ascending, no
    block beyond the query's own, forced blocks present.  [B, T, H_kv, n_sel] int32, -1 padded.  Chains only."""
    assert case.parents is None, "planted overlaps are defined along linear chains"
    nsa = case.nsa
    sel = np.full((case.B, case.T, case.H_kv, nsa.n_sel), -1, np.int32)
    for b in range(case.B):
        L, Tq = int(case.seq_lens[b]), int(case.n_query[b])
        for g in range(case.H_kv):
            rng = _rng(seed, 77, b, g)
            prev = None
            for i in range(Tq):
                J = (L + i) // nsa.l_sel
                forced = {j for j in range(nsa.n_init) if j <= J} | {j for j in range(J - nsa.n_local + 1, J + 1) if j >= 0}
                n_eff = min(nsa.n_sel, J + 1)
                n_free = n_eff - len(forced)
                pool = [j for j in range(J + 1) if j not in forced]
                if prev is None:
                    chosen = set(rng.choice(pool, size=n_free, replace=False).tolist()) if n_free else set()
                else:
                    keep_from = sorted(prev - forced)
                    n_keep = s - len(forced & prev)
                    fresh_pool = [j for j in pool if j not in prev]
                    assert 0 <= n_keep <= min(len(keep_from), n_free) and n_free - n_keep <= len(fresh_pool), \
                        f"overlap {s} cannot be planted at L={L}, query {i}"
                    kept = set(rng.choice(keep_from, size=n_keep, replace=False).tolist()) if n_keep else set()
                    fresh = set(rng.choice(fresh_pool, size=n_free - n_keep, replace=False).tolist()) if n_free > n_keep else set()
                    chosen = kept | fresh
                cur = forced | chosen
                row = sorted(cur)
                sel[b, i, g, :len(row)] = row
                prev = cur
    return sel
