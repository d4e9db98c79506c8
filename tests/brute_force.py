"""Brute-force NSA verification by definition, for tiny inputs only (test helper).

Written independently of oracle/: dense score vectors over every slot plus boolean masks,
a scatter formulation of the block importance, and Python sorting for the selection.
"""
from __future__ import annotations

import numpy as np

import ssv_inputs as si


def _softmax_masked(scores: np.ndarray, mask: np.ndarray) -> np.ndarray:
    p = np.zeros_like(scores)
    if mask.any():
        z = scores[mask] - scores[mask].max()
        e = np.exp(z)
        p[mask] = e / e.sum()
    return p


def tree_info(parents, Tq):
    depth = [0] * Tq
    anc = [set() for _ in range(Tq)]
    for i in range(Tq):
        p = int(parents[i])
        depth[i] = 0 if p < 0 else depth[p] + 1
        anc[i] = {i} | (anc[p] if p >= 0 else set())
    return depth, anc


def brute_force_verify(case, sel_idx=None, scale=None):
    nsa = case.nsa
    B, T, H, H_kv, H_g = case.B, case.T, case.H, case.H_kv, case.H_g
    f = lambda a: si.to_f32(a, case.dtype).astype(np.float64)
    q, k, v, kc, vc = f(case.q), f(case.k), f(case.v), f(case.k_cmp), f(case.v_cmp)
    scale = 1.0 / np.sqrt(case.d_k) if scale is None else scale
    out = np.zeros((B, T, H, case.d_v))
    branches = np.zeros((3, B, T, H, case.d_v))
    sel_out = np.full((B, T, H_kv, nsa.n_sel), -1, np.int32)
    imps = {}
    a, bq = nsa.l_sel // nsa.d, nsa.l // nsa.d
    for b in range(B):
        L, Tq = int(case.seq_lens[b]), int(case.n_query[b])
        parents = case.parents[b] if case.parents is not None else si.chain_parents(T)
        depth, anc = tree_info(parents, Tq)
        n_slots = L + Tq
        kpos = np.array([s if s < L else L + depth[s - L] for s in range(n_slots)])
        for i in range(Tq):
            vis = np.array([s < L or (s - L) in anc[i] for s in range(n_slots)])
            lead = 0
            while lead < Tq and lead in anc[i]:
                lead += 1
            E = L + lead
            cvis = np.array([c * nsa.d + nsa.l <= E for c in range(int(case.n_cmp[b]))], dtype=bool)
            J = (L + i) // nsa.l_sel
            pos = L + depth[i]
            for g in range(H_kv):
                imp = np.zeros(J + 2 + len(cvis))
                o_cmp = {}
                for h in range(g * H_g, (g + 1) * H_g):
                    sc = scale * (kc[b, g, :len(cvis)] @ q[b, i, h])
                    p = _softmax_masked(sc, cvis)
                    o_cmp[h] = p @ vc[b, g, :len(cvis)]
                    for c in np.nonzero(cvis)[0]:
                        for x in range(c, c + bq):     # stride-d chunks covered by compression block c
                            imp[x // a] += p[c]
                assert np.all(imp[J + 1:] == 0)
                imp = imp[:J + 1]
                imps[(b, i, g)] = imp
                if sel_idx is None:
                    forced = sorted({j for j in range(nsa.n_init) if j <= J} |
                                    {j for j in range(J - nsa.n_local + 1, J + 1) if j >= 0})
                    n_eff = min(nsa.n_sel, J + 1)
                    free = sorted((j for j in range(J + 1) if j not in forced), key=lambda j: (-imp[j], j))
                    chosen = sorted(forced + free[:n_eff - len(forced)])
                    sel_out[b, i, g, :len(chosen)] = chosen
                else:
                    n_blk = -(-n_slots // nsa.l_sel)
                    chosen = sorted({int(x) for x in sel_idx[b, i, g] if 0 <= x < n_blk})
                    sel_out[b, i, g] = sel_idx[b, i, g]
                in_sel = np.isin(np.arange(n_slots) // nsa.l_sel, chosen) & vis
                in_win = vis & (kpos > pos - nsa.w) & (kpos <= pos)
                for h in range(g * H_g, (g + 1) * H_g):
                    sc = scale * (k[b, g, :n_slots] @ q[b, i, h])
                    o_slc = _softmax_masked(sc, in_sel) @ v[b, g, :n_slots]
                    o_win = _softmax_masked(sc, in_win) @ v[b, g, :n_slots]
                    gt = case.gates[b, i, h].astype(np.float64)
                    branches[0, b, i, h], branches[1, b, i, h], branches[2, b, i, h] = o_cmp[h], o_slc, o_win
                    out[b, i, h] = gt[0] * o_cmp[h] + gt[1] * o_slc + gt[2] * o_win
    return out, sel_out, branches, imps


def dense_tree_attention(case, scale=None):
    """Textbook softmax attention of every verifier query over all the slots it may see
    (committed prefix + itself + its ancestors)."""
    B, T, H, H_g = case.B, case.T, case.H, case.H_g
    f = lambda a: si.to_f32(a, case.dtype).astype(np.float64)
    q, k, v = f(case.q), f(case.k), f(case.v)
    scale = 1.0 / np.sqrt(case.d_k) if scale is None else scale
    out = np.zeros((B, T, H, case.d_v))
    for b in range(B):
        L, Tq = int(case.seq_lens[b]), int(case.n_query[b])
        parents = case.parents[b] if case.parents is not None else si.chain_parents(T)
        _, anc = tree_info(parents, Tq)
        for i in range(Tq):
            idx = np.array(list(range(L)) + sorted(L + t for t in anc[i]))
            for h in range(H):
                g = h // H_g
                s = scale * (k[b, g, idx] @ q[b, i, h])
                e = np.exp(s - s.max())
                out[b, i, h] = (e / e.sum()) @ v[b, g, idx]
    return out
