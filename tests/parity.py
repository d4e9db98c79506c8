"""Comparison rule between the HIP path and the oracle (test helper).

Selected indices must match the oracle as sets per (sequence, query, KV group), except where the
oracle's own decision is ambiguous: its boundary gap (smallest chosen free importance minus largest
unchosen one) is below 1e-4.  Such cases are counted and reported, and their outputs are still
checked: the oracle is re-run in reuse mode with the indices the GPU produced.
A differing set is accepted only if the blocks it swapped lie inside that band: every block the GPU
chose and the oracle did not must have an oracle importance of at least (smallest chosen free
importance - 1e-4), and every block the oracle chose and the GPU did not at most (largest unchosen
importance + 1e-4).  The worst margin by which a swapped block sits on the wrong side of the
oracle's boundary is reported.
Outputs must agree within max-abs 2e-2 for bf16 inputs (fp32 accumulation) and 1e-4 for fp32.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

TOL = {"bf16": 2e-2, "f32": 1e-4}
AMBIGUOUS_GAP = 1e-4


@dataclass
class ParityReport:
    n_units: int
    n_mismatch: int          # (b, i, g) whose index set differs from the oracle's
    n_mismatch_strict: int   # of those, how many the ambiguity rule does not cover (must be 0)
    n_ambiguous: int         # (b, i, g) whose oracle gap is below 1e-4, matched or not
    max_gap_at_mismatch: float
    max_abs_err: float
    worst_swap_margin: float = 0.0   # largest oracle-importance distance of a swapped block from the oracle's boundary
    n_swap_violations: int = 0       # swapped blocks further than 1e-4 from the boundary (must be 0)

    def line(self) -> str:
        return (f"units={self.n_units} idx_mismatch={self.n_mismatch} (uncovered={self.n_mismatch_strict}, "
                f"max oracle gap there={self.max_gap_at_mismatch:.2e}, worst swap margin={self.worst_swap_margin:.2e}, "
                f"swaps beyond 1e-4={self.n_swap_violations}) ambiguous_units={self.n_ambiguous} "
                f"max_abs_err={self.max_abs_err:.3e}")


def compare(case, oracle_mod, ref, gpu_out: np.ndarray, gpu_sel: np.ndarray, reuse_sel=None, routed_by=None) -> ParityReport:
    """ref: oracle result in the same mode; reuse_sel: indices given to both sides in reuse mode;
    routed_by [B, T]: in the shared-index variant, the query whose selection each row holds."""
    B, T, H_kv = case.B, case.T, case.H_kv
    active = np.arange(T)[None, :] < case.n_query[:, None]
    n_units = int(active.sum()) * H_kv
    n_mis = n_strict = n_amb = 0
    max_gap = worst_margin = 0.0
    n_viol = 0
    expected = ref.out
    if reuse_sel is None:
        gs, rs = np.sort(gpu_sel, axis=-1), np.sort(ref.sel_idx, axis=-1)
        differ = np.any(gs != rs, axis=-1) & active[:, :, None]
        amb = (ref.gap < AMBIGUOUS_GAP) & active[:, :, None]
        n_mis, n_amb = int(differ.sum()), int(amb.sum())
        n_strict = int((differ & ~amb).sum())
        if n_mis:
            max_gap = float(ref.gap[differ].max())
            expected = oracle_mod.nsa_verify(case, sel_idx=gpu_sel).out
            worst_margin, n_viol = swap_margins(case, oracle_mod, ref, gpu_sel, differ, routed_by)
        # every produced set must be valid in itself: ascending, unique, -1 padded, forced blocks present
        for b, i, g in zip(*np.nonzero(np.broadcast_to(active[:, :, None], differ.shape))):
            row = gpu_sel[b, i, g]
            chosen = row[row >= 0]
            assert np.all(np.diff(chosen) > 0) and np.all(row[len(chosen):] == -1), (b, i, g, row)
            J = (int(case.seq_lens[b]) + (i if routed_by is None else int(routed_by[b, i]))) // case.nsa.l_sel
            assert len(chosen) == min(case.nsa.n_sel, J + 1) and chosen.max() <= J, (b, i, g, row)
            forced = {j for j in range(case.nsa.n_init) if j <= J} | \
                     {j for j in range(J - case.nsa.n_local + 1, J + 1) if j >= 0}
            assert forced <= set(chosen.tolist()), (b, i, g, row)
        assert np.all(gpu_sel[~active] == -1)
    err = np.abs(gpu_out - expected)
    assert np.all(np.isfinite(gpu_out))
    assert np.all(gpu_out[~active] == 0)
    return ParityReport(n_units, n_mis, n_strict, n_amb, max_gap, float(err.max()), worst_margin, n_viol)


def swap_margins(case, oracle_mod, ref, gpu_sel, differ, routed_by=None):
    """For every unit whose index set differs from the oracle's: how far, in the oracle's own fp64 importance,
    each swapped block lies on the wrong side of the oracle's selection boundary.  Returns (worst margin,
    number of swapped blocks beyond the 1e-4 band)."""
    B, T = case.B, case.T
    imp = ref.imp
    if imp is None:      # importance of the routed queries of the differing units only
        mask = np.zeros((B, T), np.uint8)
        for b, i, g in zip(*np.nonzero(differ)):
            mask[b, i if routed_by is None else int(routed_by[b, i])] = 1
        imp = oracle_mod.nsa_verify(case, want_imp=True, query_mask=mask).imp
    worst, n_viol = 0.0, 0
    nsa = case.nsa
    for b, i, g in zip(*np.nonzero(differ)):
        r = i if routed_by is None else int(routed_by[b, i])
        J = (int(case.seq_lens[b]) + r) // nsa.l_sel
        row = imp[b, r, g, :J + 1]
        forced = {j for j in range(nsa.n_init) if j <= J} | {j for j in range(J - nsa.n_local + 1, J + 1) if j >= 0}
        want = {int(j) for j in ref.sel_idx[b, i, g] if j >= 0}
        got = {int(j) for j in gpu_sel[b, i, g] if j >= 0}
        free = sorted(want - forced)
        unchosen = [j for j in range(J + 1) if j not in want]
        assert free and unchosen, (b, i, g)      # a set can only differ where a free choice existed
        min_chosen = min(row[j] for j in free)
        max_unchosen = max(row[j] for j in unchosen)
        margins = [min_chosen - row[j] for j in got - want] + [row[j] - max_unchosen for j in want - got]
        worst = max(worst, float(max(margins)))
        n_viol += sum(1 for m in margins if m > AMBIGUOUS_GAP)
    return worst, n_viol


def check(case, report: ParityReport) -> None:
    print(f"[parity] {case.name}: {report.line()}", flush=True)
    assert report.n_mismatch_strict == 0, report.line()
    assert report.n_swap_violations == 0, report.line()
    assert report.max_abs_err <= TOL[case.dtype], report.line()
