#!/usr/bin/env python3
"""Benchmark of the NSA speculative-verification hot path on one MI355X.

A "step" is one ssv_nsa_verify call in refresh mode: the whole hot path (compressed scan, block
importance, top-n selection, merged selected-block + sliding-window attention, gated combine) over
one batch of seeded synthetic inputs that are already resident in HBM.  The default run measures the
four benchmark configurations the metric's context range spans: cfg1 (B=1, 32K context, 8 verifier
queries: the latency row), cfg2 (B=16, 64K, 4 queries: the bandwidth-bound batch and the headline),
cfg3 (B=4, 128K, a 40-node draft tree) and cfg4 (B=32, mixed 4K-128K, 16 queries), every one with its
parity check against the fp64 oracle, per-call statistics, per-kernel durations and both roofline
fractions per kernel (HBM bytes and MFMA flops of the method against the chip's peaks).  One JSON line
is printed.

Cold numbers rotate over enough copies of the inputs that the bytes touched between two uses of a copy
exceed 512 MB, twice the 256 MB last-level cache; warm numbers reuse one copy.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
COLD_FOOTPRINT_BYTES = 512e6


def method_work(case, sel_idx, C, C_scan=None):
    """Bytes the method itself must move and flops it must do for one call.  Bytes: compressed rows once per KV
    head; raw KV tokens of the union of selected blocks and windows once per group of C queries (windows: per
    group of C_scan queries); q, out, gates, indices.  Flops: 2 (d_k + d_v) per (query head, visible key) of each
    branch, 2 d_k per (query head, compressed row) for the normalised importance pass."""
    import ssv_inputs as si
    es = 2 if case.dtype == "bf16" else 4
    nsa = case.nsa
    C_scan = C if C_scan is None else C_scan
    row_b = (case.d_k + case.d_v) * es
    H_g = case.H // case.H_kv
    cmp_b = slc_b = win_b = union_b = 0
    cmp_keys = slc_keys = win_keys = 0      # (query, KV group, visible key) triples
    for b in range(case.B):
        L, Tq = int(case.seq_lens[b]), int(case.n_query[b])
        par = case.parents[b] if case.parents is not None else si.chain_parents(case.T)
        depth = si.node_depths(par[:Tq])
        anc = []
        for i in range(Tq):
            a, t = set(), i
            while t >= 0:
                a.add(t)
                t = int(par[t])
            anc.append(a)
        ncv = 0
        for i in range(Tq):
            lead = 0
            while lead < Tq and lead in anc[i]:
                lead += 1
            ncv_i = min(int(case.n_cmp[b]), si.n_cmp_blocks(L + lead, nsa.l, nsa.d))
            cmp_keys += ncv_i * case.H_kv
            ncv = max(ncv, ncv_i)
        cmp_b += case.H_kv * ncv * row_b

        def window_mask(i):
            win = np.zeros(L + Tq, bool)
            pos = L + int(depth[i])
            win[max(0, pos - nsa.w + 1):L] = True
            for t in anc[i]:
                if pos - nsa.w < L + int(depth[t]) <= pos:
                    win[L + t] = True
            return win

        wins = [window_mask(i) for i in range(Tq)]
        win_keys += sum(int(w.sum()) for w in wins) * case.H_kv
        for q0 in range(0, Tq, C_scan):
            u = np.zeros(L + Tq, bool)
            for i in range(q0, min(Tq, q0 + C_scan)):
                u |= wins[i]
            win_b += int(u.sum()) * row_b * case.H_kv
        for g in range(case.H_kv):
            for q0 in range(0, Tq, C):
                grp = range(q0, min(Tq, q0 + C))
                slc = np.zeros(L + Tq, bool)
                win = np.zeros(L + Tq, bool)
                for i in grp:
                    mine = np.zeros(L + Tq, bool)
                    vis_draft = np.zeros(Tq, bool)
                    vis_draft[list(anc[i])] = True
                    for j in sel_idx[b, i, g]:
                        if j < 0:
                            continue
                        lo, hi = j * nsa.l_sel, min((j + 1) * nsa.l_sel, L + Tq)
                        mine[lo:min(hi, L)] = True
                        if hi > L:
                            s = np.arange(max(lo, L), hi)
                            mine[s] |= vis_draft[s - L]
                    slc_keys += int(mine.sum())
                    slc |= mine
                    win |= wins[i]
                slc_b += int(slc.sum()) * row_b
                union_b += int((slc | win).sum()) * row_b
    tq = int(case.n_query.sum())
    io_b = tq * case.H * (case.d_k + case.d_v) * es + tq * case.H * 3 * 4 + tq * case.H_kv * nsa.n_sel * 4
    f = 2 * H_g
    return {"bytes": {"compressed": cmp_b, "selected_union": slc_b, "window_union": win_b, "raw_union": union_b,
                      "q_out_gates_idx": io_b, "total": cmp_b + union_b + io_b},
            "flops": {"compressed": f * cmp_keys * (case.d_k + case.d_v), "importance": f * cmp_keys * case.d_k,
                      "selected": f * slc_keys * (case.d_k + case.d_v), "window": f * win_keys * (case.d_k + case.d_v)}}


def time_calls(torch, devs, steps, warmup, per_call=False):
    """Warm up, then time exactly `steps` calls (rotating over devs) between synchronisations: one event pair
    around all of them gives the mean (ms per call), next to the host's wall clock.  With per_call, a second pass
    of `steps` calls records an event after every call and returns the spacings of consecutive events (ms): the
    distribution of the per-call time.  Every event costs the stream a few microseconds of its own (the empty
    event pair the library reports), so that pass is kept apart from the mean."""
    n = len(devs)
    for s in range(warmup):
        devs[s % n].run()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for s in range(steps):
        devs[s % n].run()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    mean_ms = ev0.elapsed_time(ev1) / steps
    spacing = None
    if per_call:
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        marks[0].record()
        for s in range(steps):
            devs[s % n].run()
            marks[s + 1].record()
        torch.cuda.synchronize()
        spacing = np.array([marks[s].elapsed_time(marks[s + 1]) for s in range(steps)])
    return mean_ms, wall_ms / steps, spacing


def time_graph_replays(torch, devs, steps, warmup):
    """The same calls recorded once into HIP graphs (one per input copy) and replayed: what a serving loop that
    captures its verification step would see."""
    side = torch.cuda.Stream()
    graphs = []
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for d in devs:
            d.run()
        side.synchronize()
        for d in devs:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                d.run()
            graphs.append(g)
    torch.cuda.synchronize()
    n = len(graphs)
    for s in range(warmup):
        graphs[s % n].replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for s in range(steps):
        graphs[s % n].replay()
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / steps


def kernel_breakdown(devs, rounds, repeats=1):
    """Launch duration (ms) of every kernel, measured with HIP events inside the library on the call's stream.
    repeats == 1: one launch per kernel with start/stop events bound to the launch (the dispatch's own begin and
    end, what a kernel trace reports), rotating over the input copies (cold caches); returns the mean and the
    median over the rounds.  repeats > 1: that many back-to-back launches per event pair on one copy."""
    from paper_2605_19893_amd import binding as B
    rows = []
    n = max(rounds, len(devs))
    for r in range(n):
        ms = []
        devs[r % len(devs)].run(kernel_ms=ms, repeats=repeats)
        rows.append(ms)
    rows = np.asarray(rows)
    assert rows.shape[1] == B.SSV_NUM_TIMINGS
    return rows.mean(axis=0), np.median(rows, axis=0)


def read_traffic(tag):
    """HBM bytes per launch from the committed rocprofv3 counter summary (profiles/hbm_traffic_<tag>.txt):
    lines 'kernel_index: fetch_bytes write_bytes', already scaled by the copy-kernel calibration."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{tag}.txt")
    out = {}
    if os.path.exists(path):
        with open(path) as f:
            for line in f:
                if line.startswith("kernel_index"):
                    parts = line.split()
                    out[int(parts[1].rstrip(":"))] = int(parts[2]) + int(parts[3])
    return out


def kernel_roofs(B, work, dtype, refresh_ms, plan):
    """Per kernel of the refresh path: the method's bytes and flops of that launch, the time each would take at the
    chip's peaks (HBM 8 TB/s; dense MFMA 2.5 PFLOP/s bf16), which of the two binds, and the measured fraction.
    With the matrix-core scan (plan.scan_matrix) the window branch runs in the selected-branch launch."""
    by, fl = work["bytes"], work["flops"]
    win_in_b = bool(plan.scan_matrix)
    per_kernel = {
        B.SSV_K_STREAM_A: (by["compressed"] + (0 if win_in_b else by["window_union"]), fl["compressed"] + (0 if win_in_b else fl["window"])),
        B.SSV_K_IMPORTANCE: (work["kcmp_bytes"], fl["importance"]),
        B.SSV_K_STREAM_B: (by["selected_union"] + (by["window_union"] if win_in_b else 0), fl["selected"] + (fl["window"] if win_in_b else 0)),
    }
    peak_fl = MFMA_PEAK_TFLOPS[dtype] * 1e12
    rows = {}
    for k, (nbytes, nflops) in per_kernel.items():
        ms = float(refresh_ms[k])
        if ms <= 0:
            continue
        t_hbm, t_mfma = nbytes / (HBM_PEAK_GBS * 1e9), nflops / peak_fl
        name = B.kernel_name(k)
        if plan.scan_matrix and k == B.SSV_K_STREAM_A:
            name = "k_scan32 (compressed scan on the 32x32x16 matrix instruction)"
        if plan.scan_matrix and k == B.SSV_K_STREAM_B:
            name = "k_stream (window + selected blocks, merged schedule)"
        rows[k] = {"kernel": name, "us": ms * 1e3, "method_bytes": int(nbytes), "method_flops": int(nflops),
                   "hbm_frac": t_hbm / (ms * 1e-3), "mfma_frac": t_mfma / (ms * 1e-3),
                   "bound": "hbm" if t_hbm >= t_mfma else "mfma"}
    return rows


COLD_ONLY = False   # --cold-only: profiling runs in which every launch of the trace sees cold inputs
EXTRAS = False      # --extras: warm-cache, graph-replay and back-to-back figures as well


def copies_for(case, total_bytes, cap_bytes=24e9):
    """Input copies to rotate over so that the bytes touched between two uses of a copy exceed 512 MB."""
    kv = case.k.nbytes + case.v.nbytes + case.k_cmp.nbytes + case.v_cmp.nbytes
    want = int(np.ceil(COLD_FOOTPRINT_BYTES / max(total_bytes, 1)))
    return int(max(1, min(want, cap_bytes // kv)))


def measure_workload(torch, oracle, case, name, tag, steps, warmup, parity=True, group_size=0):
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    res = {"workload": name, "tag": tag}
    t0 = time.perf_counter()
    ref = oracle.nsa_verify(case)
    res["oracle_s"] = time.perf_counter() - t0
    dev0 = DeviceCase(case, group_size=group_size)
    dev0.run()
    out, sel = dev0.results()
    if parity:
        from parity import compare
        rep = compare(case, oracle, ref, out, sel)
        res["parity"] = {"idx_mismatch": rep.n_mismatch, "idx_mismatch_outside_ambiguity": rep.n_mismatch_strict,
                         "swapped_blocks_beyond_1e-4_of_the_boundary": rep.n_swap_violations,
                         "worst_swap_margin": rep.worst_swap_margin,
                         "ambiguous_units": rep.n_ambiguous, "units": rep.n_units, "max_abs_err": rep.max_abs_err}
        assert rep.n_mismatch_strict == 0 and rep.n_swap_violations == 0, rep.line()
    # (with the matrix-core scan the window branch runs in the selected-branch launch, in that launch's groups)
    work = method_work(case, ref.sel_idx, dev0.plan.C, dev0.plan.C if dev0.plan.scan_matrix else dev0.plan.C_scan)
    work["kcmp_bytes"] = work["bytes"]["compressed"] * case.d_k // (case.d_k + case.d_v)
    ab = work["bytes"]
    res["algorithmic_bytes"] = ab
    res["method_flops"] = work["flops"]
    n_copies = copies_for(case, ab["total"])
    devs = [dev0] + [DeviceCase(case, group_size=group_size) for _ in range(n_copies - 1)]
    res["cold_rotation"] = {"input_copies": n_copies, "bytes_touched_between_reuses_of_a_copy": int(n_copies * ab["total"])}
    tokens = int(case.n_query.sum())
    out_modes = {}
    raw = {}
    for mode, mname in ((B.SSV_REFRESH, "refresh"), (B.SSV_REUSE, "reuse")):
        for d in devs:
            d.set_mode(mode)
            if mode == B.SSV_REUSE:
                d.set_sel_idx(ref.sel_idx)
        cold_ms, cold_wall, per_call = time_calls(torch, devs, steps, warmup, per_call=True)
        kmean, kmed = kernel_breakdown(devs, 8, 1)
        raw[mname] = kmed
        nk = B.SSV_NUM_KERNELS
        m = {
            "plan": devs[0].plan.as_dict(),
            "us_per_call_cold": cold_ms * 1e3, "us_per_call_cold_wallclock": cold_wall * 1e3,
            # distribution over calls, from one event after every call: each includes that event's own cost
            "us_per_call_cold_median": float(np.median(per_call)) * 1e3,
            "us_per_call_cold_p10": float(np.percentile(per_call, 10)) * 1e3,
            "us_per_call_cold_p90": float(np.percentile(per_call, 90)) * 1e3,
            "per_call_event_cost_us": float(max(np.median(per_call) - cold_ms, 0.0)) * 1e3,
            "timed_calls": int(steps),
            "tokens_per_s_cold": tokens / (cold_ms * 1e-3),
            "algorithmic_GBs_cold": ab["total"] / (cold_ms * 1e-3) / 1e9,
            "hbm_frac_whole_call_cold": ab["total"] / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "kernel_us_cold_single_launch_median": {B.kernel_name(i): float(kmed[i] * 1e3) for i in range(nk) if kmed[i] > 0},
            "kernel_us_cold_single_launch_mean": {B.kernel_name(i): float(kmean[i] * 1e3) for i in range(nk) if kmean[i] > 0},
            "event_pair_overhead_us": float(kmed[B.SSV_T_EVENT_PAIR] * 1e3),
        }
        if EXTRAS and not COLD_ONLY:
            warm_ms, _, _ = time_calls(torch, devs[:1], steps, warmup)
            m["us_per_call_warm"] = warm_ms * 1e3
            m["us_per_call_cold_graph_replay"] = time_graph_replays(torch, devs, steps, warmup) * 1e3
            krep, _ = kernel_breakdown(devs[:1], 2, 20)
            m["kernel_us_20_back_to_back_launches"] = {B.kernel_name(i): float(krep[i] * 1e3) for i in range(nk) if krep[i] > 0}
        out_modes[mname] = m
    res["modes"] = out_modes
    # both roofs per kernel of the refresh path, and the roofline object of the longest one
    for d in devs:
        d.set_mode(B.SSV_REFRESH)
    roofs = kernel_roofs(B, work, case.dtype, raw["refresh"], devs[0].plan)
    res["kernel_roofs_refresh"] = list(roofs.values())
    dom = max(roofs, key=lambda k: roofs[k]["us"])
    r = roofs[dom]
    traffic = read_traffic(tag).get(dom)
    if r["bound"] == "hbm":
        achieved, peak, unit = r["method_bytes"] / (r["us"] * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
    else:
        achieved, peak, unit = r["method_flops"] / (r["us"] * 1e-6) / 1e12, MFMA_PEAK_TFLOPS[case.dtype], "TFLOP/s"
    res["roofline"] = {"bound": r["bound"], "kernel": r["kernel"], "achieved": achieved, "peak": peak, "unit": unit,
                       "frac": achieved / peak, "traffic": traffic,
                       "algorithmic_bytes_per_launch": r["method_bytes"], "method_flops_per_launch": r["method_flops"],
                       "avg_launch_us": r["us"], "hbm_frac": r["hbm_frac"], "mfma_frac": r["mfma_frac"]}
    del devs, dev0
    torch.cuda.empty_cache()
    return res, ref


def shared_index_study(torch, oracle, si, T, rhos, C, steps, warmup):
    """Approximate shared-index variant (Section 4.3) against the exact merged schedule on the cfg1 shape with
    groups of C queries: time per call, bytes of selected blocks loaded, and how far the outputs move (fp64
    oracle of each variant), as a function of the cross-query correlation rho."""
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import compare
    rows = []
    for rho in rhos:
        case = si.config1(rho, T=T)
        exact, shared = oracle.nsa_verify(case), oracle.nsa_verify_shared(case, C)
        routed_by = oracle.group_representatives(case, C)
        dev_out = np.abs(shared.out - exact.out)
        row = {"rho": rho, "T": T, "C": C,
               "output_deviation_max_abs": float(dev_out.max()),
               "output_deviation_rms": float(np.sqrt((dev_out ** 2).mean())),
               "output_rms": float(np.sqrt((exact.out ** 2).mean())),
               "index_sets_changed": int(np.any(np.sort(shared.sel_idx, -1) != np.sort(exact.sel_idx, -1), axis=-1).sum()),
               "index_sets": int(case.n_query.sum()) * case.H_kv}
        for mode, mname, ref in ((B.SSV_REFRESH, "exact", exact), (B.SSV_REFRESH_SHARED, "shared", shared)):
            ab = method_work(case, ref.sel_idx, C)["bytes"]
            devs = [DeviceCase(case, mode=mode, group_size=C) for _ in range(copies_for(case, ab["total"]))]
            devs[0].run()
            out, sel = devs[0].results()
            rep = compare(case, oracle, ref, out, sel, routed_by=routed_by if mode == B.SSV_REFRESH_SHARED else None)
            cold_ms, _, _ = time_calls(torch, devs, steps, warmup)
            row[mname] = {"us_per_call_cold": cold_ms * 1e3, "selected_union_bytes": ab["selected_union"],
                          "algorithmic_bytes_total": ab["total"],
                          "parity_max_abs_err": rep.max_abs_err, "idx_mismatch_outside_ambiguity": rep.n_mismatch_strict}
            del devs
            torch.cuda.empty_cache()
        rows.append(row)
    return rows


def mean_adjacent_overlap(sel, n_query):
    """Mean of |I_i and I_(i-1)| over consecutive chain queries and KV groups (the paper's overlap s, Section 7.3)."""
    tot = cnt = 0
    for b in range(sel.shape[0]):
        for i in range(1, int(n_query[b])):
            for g in range(sel.shape[2]):
                a, c = sel[b, i, g], sel[b, i - 1, g]
                tot += len(set(a[a >= 0].tolist()) & set(c[c >= 0].tolist()))
                cnt += 1
    return tot / max(cnt, 1)


def kernel_workload_study(torch, oracle, si, steps, warmup, contexts=(8192, 16384, 32768, 65536), gammas=(4, 64),
                          overlaps=(3, 6, 10)):
    """The paper's isolated-kernel workload (Section 7 setup and Section 7.3): batch 1, 32 query heads / 8 KV heads,
    head dimension 64, bf16, standard NSA parameters, draft length gamma in {4, 64} (a linear chain), context
    N in {8K..64K}.  Reuse-mode calls run on PLANTED index sets in which consecutive queries share exactly
    s in {3, 6, 10} blocks (the mandatory initial and local blocks included), the paper's overlap knob; refresh-mode
    calls construct their own indices from the synthetic data (uncorrelated queries: s close to the lower bound).
    Executions: unfused per-query (one launch per branch and query, branch outputs through HBM, gate kernel: the
    structure of the original NSA kernels), fused per-query (C = 1), the paper's exact variant (C = 2), this
    build's default grouping (64 rows: C = min(gamma, 16)), and the approximate shared-index variant (C = 4)."""
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import compare
    rows = []
    for N in contexts:
        for gamma in gammas:
            case = si.make_case(f"kernel_workload_N{N}_g{gamma}", "bf16", 1, gamma, 32, 8, 64, 64, si.STD_NSA, [N],
                                si.config_seed(5), rho=0.0)
            kv_bytes = case.k.nbytes + case.v.nbytes + case.k_cmp.nbytes + case.v_cmp.nbytes
            n_copies = int(min(32, max(2, -(-600_000_000 // kv_bytes))))
            devs = [DeviceCase(case) for _ in range(n_copies)]
            exact = oracle.nsa_verify(case)
            shared = oracle.nsa_verify_shared(case, 4)
            routed_by = oracle.group_representatives(case, 4)
            # (name, exec, mode of the refresh call, group size)
            variants = (("unfused_per_query", B.SSV_EXEC_UNFUSED, B.SSV_REFRESH, 0),
                        ("fused_per_query", B.SSV_EXEC_FUSED, B.SSV_REFRESH, 1),
                        ("fused_exact_C2", B.SSV_EXEC_FUSED, B.SSV_REFRESH, 2),
                        ("fused_default_C", B.SSV_EXEC_FUSED, B.SSV_REFRESH, 0),
                        ("fused_shared_C4", B.SSV_EXEC_FUSED, B.SSV_REFRESH_SHARED, 4))
            row = {"N": N, "gamma": gamma, "input_copies": n_copies,
                   "refresh_mean_adjacent_overlap": mean_adjacent_overlap(exact.sel_idx, case.n_query), "refresh_us": {}, "C": {}}
            worst = 0.0
            for vname, ex, mode, C in variants:
                ref = shared if mode == B.SSV_REFRESH_SHARED else exact
                for d in devs:
                    d.params.exec = ex
                    d.set_group_size(C, mode)
                devs[0].run()
                out, sel = devs[0].results()
                rep = compare(case, oracle, ref, out, sel, routed_by=routed_by if mode == B.SSV_REFRESH_SHARED else None)
                assert rep.n_mismatch_strict == 0 and rep.n_swap_violations == 0, (vname, rep.line())
                worst = max(worst, rep.max_abs_err)
                t, _, _ = time_calls(torch, devs, steps, warmup)
                row["refresh_us"][vname] = t * 1e3
                row["C"][vname] = int(devs[0].plan.C)
            row["reuse_us"] = {}
            for s in overlaps:
                planted = si.planted_overlap_indices(case, s, seed=si.config_seed(5) + s)
                want = oracle.nsa_verify(case, sel_idx=planted).out
                rs = {}
                for vname, ex, mode, C in variants:
                    if mode == B.SSV_REFRESH_SHARED:
                        continue          # with the indices given, the shared variant is the default grouping
                    for d in devs:
                        d.params.exec = ex
                        d.set_group_size(C, B.SSV_REUSE)
                        d.set_sel_idx(planted)
                    devs[0].run()
                    out, _ = devs[0].results()
                    err = float(np.abs(out - want).max())
                    assert err <= 2e-2, (vname, s, err)
                    worst = max(worst, err)
                    t, _, _ = time_calls(torch, devs, steps, warmup)
                    rs[vname] = t * 1e3
                row["reuse_us"][f"s={s}"] = rs
            base = row["refresh_us"]["unfused_per_query"]
            row["ratios"] = {
                "fused_over_unfused_refresh_per_query": base / row["refresh_us"]["fused_per_query"],
                "grouped_over_per_query_refresh": row["refresh_us"]["fused_per_query"] / row["refresh_us"]["fused_default_C"],
                "default_over_unfused_refresh": base / row["refresh_us"]["fused_default_C"],
                "shared_C4_over_unfused_refresh": base / row["refresh_us"]["fused_shared_C4"],
                "index_construction_share_of_refresh": 1.0 - row["reuse_us"]["s=3"]["fused_default_C"] / row["refresh_us"]["fused_default_C"],
            }
            for s in overlaps:
                rs = row["reuse_us"][f"s={s}"]
                row["ratios"][f"s={s}"] = {
                    "reuse_fused_over_refresh_unfused_per_query": base / rs["fused_per_query"],
                    "reuse_default_over_refresh_unfused": base / rs["fused_default_C"],
                    "reuse_fused_over_reuse_unfused_per_query": rs["unfused_per_query"] / rs["fused_per_query"],
                    "reuse_grouped_over_per_query": rs["fused_per_query"] / rs["fused_default_C"],
                    "reuse_exact_C2_over_per_query": rs["fused_per_query"] / rs["fused_exact_C2"],
                }
            row["parity_max_abs_err"] = worst
            rows.append(row)
            print(f"[kernel workload] N={N} gamma={gamma}: refresh " +
                  " ".join(f"{v}={t:.0f}" for v, t in row["refresh_us"].items()) + " | reuse s=6 " +
                  " ".join(f"{v}={t:.0f}" for v, t in row["reuse_us"].get("s=6", {}).items()) + " us",
                  file=sys.stderr, flush=True)
            del devs
            torch.cuda.empty_cache()
    return rows


def compress_study(torch, si, steps, warmup):
    """Compressed-cache construction (ssv_nsa_compress): a from-scratch build at the cfg2 shape (the prefill-sized
    case, HBM-bound: every raw K/V row is read once) and an incremental update after a verification round at the
    cfg4 shape (0..16 newly committed tokens per sequence: latency-bound).  Sampled rows are checked against the
    fp64 compression oracle."""
    import paper_2605_19893_amd as P
    from oracle import compress as oc
    res = {}
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(si.config_seed(6))
    for name, B_, L in (("full_build_cfg2_shape", 16, 65536), ("incremental_cfg4_shape", 32, None)):
        H_kv, d_k, d_v, l, d = 4, 192, 128, 32, 16
        if L is None:
            before = si.config4_lengths(B_, si.config_seed(4)).astype(np.int32)
            after = before + rng.integers(0, 17, B_).astype(np.int32)
        else:
            before, after = np.zeros(B_, np.int32), np.full(B_, L, np.int32)
        S = int(after.max())
        cap = oc.n_cmp_rows(S, l, d)
        k = torch.randn((B_, H_kv, S, d_k), dtype=torch.bfloat16, device="cuda")
        v = torch.randn((B_, H_kv, S, d_v), dtype=torch.bfloat16, device="cuda")
        kc = torch.zeros((B_, H_kv, cap, d_k), dtype=torch.bfloat16, device="cuda")
        vc = torch.zeros((B_, H_kv, cap, d_v), dtype=torch.bfloat16, device="cuda")
        n_cmp = torch.zeros(B_, dtype=torch.int32, device="cuda")
        bef_d, aft_d = torch.from_numpy(before).cuda(), torch.from_numpy(after).cuda()
        new_rows = [oc.n_cmp_rows(int(a), l, d) - oc.n_cmp_rows(int(b0), l, d) for a, b0 in zip(after, before)]
        p = P.make_cmp_params(B=B_, H_kv=H_kv, d_k=d_k, d_v=d_v, l=l, d=d, dtype=P.SSV_BF16, max_new_rows=max(1, max(new_rows)),
                              kv_capacity=S, cmp_capacity=cap, k_stride=k.stride()[:3], v_stride=v.stride()[:3],
                              kc_stride=kc.stride()[:3], vc_stride=vc.stride()[:3])
        call = lambda: P.ssv_nsa_compress(k, v, kc, vc, bef_d, aft_d, n_cmp, p, stream)
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(steps):
            call()
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / steps
        # algorithmic bytes: every raw row under a new compressed row once, every new compressed row once
        raw_rows = sum((n - 1) * d + l for n in new_rows if n > 0)
        nbytes = H_kv * (d_k + d_v) * 2 * (raw_rows + sum(new_rows))
        # sampled parity against the oracle
        worst_ulps, checked = 0.0, 0
        for _ in range(48):
            b = int(rng.integers(0, B_))
            if new_rows[b] <= 0:
                continue
            h = int(rng.integers(0, H_kv))
            c = oc.n_cmp_rows(int(before[b]), l, d) + int(rng.integers(0, new_rows[b]))
            for src, dst in ((k, kc), (v, vc)):
                raw = src[b, h, c * d:c * d + l].float().cpu().numpy().astype(np.float64)
                _, want, mean = oc.compress(raw, 0, l, l, d, "bf16")
                got = dst[b, h, c].float().cpu().numpy().astype(np.float64)
                spacing = np.ldexp(1.0, np.frexp(mean[0])[1] - 8)
                worst_ulps = max(worst_ulps, float((np.abs(got - mean[0]) / spacing).max()))
                checked += got.size
        assert worst_ulps <= 0.5 + 1e-3, worst_ulps
        assert np.array_equal(n_cmp.cpu().numpy(), [oc.n_cmp_rows(int(a), l, d) for a in after])
        res[name] = {"B": B_, "new_compressed_rows_per_head": int(sum(new_rows)), "us_per_call": ms * 1e3,
                     "algorithmic_bytes": int(nbytes), "achieved_GBs": nbytes / (ms * 1e-3) / 1e9,
                     "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "parity_sampled_elements": checked, "parity_max_error_in_storage_ulps": worst_ulps}
        del k, v, kc, vc
        torch.cuda.empty_cache()
    return res


def cpu_baseline(oracle, case, label, budget_s=12.0, also_single_thread=None):
    """The oracle as it stands, timed on this machine's host cores on the same workload: whole calls repeated until the
    budget is used; also the time of one call on a single thread of another (small) workload."""
    threads = oracle.default_threads()
    cores = len(os.sched_getaffinity(0))
    tokens = int(case.n_query.sum())
    t0 = time.perf_counter()
    reps = 0
    while True:
        oracle.nsa_verify(case)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= 2000:
            break
    res = {"value": tokens * reps / el, "unit": "tokens/s", "cores": threads, "host_cores_available": cores, "kind": "oracle",
           "sample": f"the full {label} workload ({tokens} verifier queries x all heads), {reps} call(s), "
                     f"{el:.1f} s of wall time on {threads} OpenMP threads ({cores} cores in the process's affinity mask)",
           "ms_per_call": el / reps * 1e3}
    if also_single_thread is not None:
        c1, l1 = also_single_thread
        t0 = time.perf_counter()
        oracle.nsa_verify(c1, n_threads=1)
        el1 = time.perf_counter() - t0
        oracle.nsa_verify(c1, n_threads=threads)      # (the thread count is sticky in the OpenMP runtime: restore it)
        res["single_thread"] = {"workload": l1, "ms_per_call": el1 * 1e3, "tokens_per_s": int(c1.n_query.sum()) / el1}
    return res


LABELS = {
    "cfg1": "cfg1: B=1 L=32768 T=8 chain rho={rho} H=64/4 d_k=192 d_v=128 l=32 d=16 l'=64 n=16 w=512",
    "cfg2": "cfg2: B=16 L=65536 T=4 chain rho=0.7, 5% keys x4, H=64/4 d_k=192 d_v=128 l=32 d=16 l'=64 n=16 w=512",
    "cfg3": "cfg3: B=4 L=131072 T=40 tree (4,3,2) BFS order, same heads and NSA parameters",
    "cfg4": "cfg4: B=32 L log-uniform 4K..128K T=16 chain rho=0.7, same heads and NSA parameters",
    "cfg4-t8": "cfg4-t8: the lengths of cfg4 with chains of 8 (128 rows per KV head: the streaming kernel scans, from its work table)",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="timed calls of the headline workload (the others: 100)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--rho", type=float, default=0.5)
    ap.add_argument("--no-extra", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true", help="warm-cache, graph-replay and back-to-back figures as well")
    ap.add_argument("--cold-only", action="store_true",
                    help="kept for the profiling commands: every launch of a trace runs on cold inputs (the default now)")
    ap.add_argument("--only", default="", help="measure only this workload (cfg1, cfg2, cfg3 or cfg4; for profiling runs; cfg4-t8: the lengths of cfg4 "
                    "with chains of 8), "
                    "'shared': the shared-index study alone, at T = 8 and T = 32, or 'kernel-workload': the full grid of the "
                    "paper's isolated-kernel workload (32/8 heads of dimension 64, draft lengths 4 and 64, contexts 8K-64K), "
                    "or 'compress': the compressed-cache construction kernel")
    ap.add_argument("--group-size", type=int, default=0, help="verifier queries per workgroup (0 = library default)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="kept for the profiling commands: the plain 1 GiB device-to-device copy (a known-size reference for HBM "
                         "byte counters) runs in every invocation")
    args = ap.parse_args()
    global COLD_ONLY, EXTRAS
    COLD_ONLY, EXTRAS = args.cold_only, args.extras
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(sequences and KV heads are independent: more GPUs would each take a share of them, with no exchange)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU: there is no CPU fallback for the product path", file=sys.stderr)
        sys.exit(2)
    import oracle
    import ssv_inputs as si

    torch.cuda.set_device(0)
    # a plain 1 GiB device-to-device copy: the known-size reference for the HBM byte counters, and the copy
    # bandwidth of this machine (read + write bytes over time) to set next to the 8 TB/s peak
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(3):
        dst.copy_(src)       # reads 1 GiB, writes 1 GiB per copy
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 3 * 2 * (1 << 30) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()

    if args.only == "compress":
        print(json.dumps({"compressed_cache_construction": compress_study(torch, si, max(20, args.steps // 10), 5),
                          "device_copy_GBs": copy_gbs}))
        return
    if args.only == "kernel-workload":
        rows = kernel_workload_study(torch, oracle, si, max(50, args.steps // 2), max(5, args.warmup // 2))
        print(json.dumps({"paper_kernel_workload": rows}))
        return
    if args.only == "shared":
        rows = shared_index_study(torch, oracle, si, 8, (0.0, 0.5, 0.9), 4, max(50, args.steps // 2), args.warmup)
        rows += shared_index_study(torch, oracle, si, 32, (0.0, 0.5, 0.9), 4, max(50, args.steps // 2), args.warmup)
        print(json.dumps({"approx_shared_index_variant": rows}))
        return

    makers = {"cfg1": lambda: si.config1(args.rho), "cfg2": si.config2, "cfg3": lambda: si.config3("bfs"), "cfg4": si.config4}
    if args.only == "cfg4-t8":      # (not one of the named configurations: measured on request only)
        makers["cfg4-t8"] = lambda: si.config4(T=8)
    headline = args.only if args.only in makers else "cfg2"
    order = [headline] if (args.only or args.no_extra) else [headline] + [t for t in makers if t != headline]
    results = {}
    base = None
    for tag in order:
        t0 = time.perf_counter()
        case = makers[tag]()
        label = LABELS[tag].format(rho=args.rho)
        steps = args.steps if tag == headline else max(100, args.steps // 2)
        res, _ = measure_workload(torch, oracle, case, label, tag, steps, args.warmup, group_size=args.group_size)
        if tag == headline and not args.no_cpu_baseline:
            # the oracle on the headline workload, bounded to about a dozen seconds; one thread on the 32K workload
            small = case if tag == "cfg1" else si.config1(args.rho)
            base = cpu_baseline(oracle, case, tag, also_single_thread=(small, "cfg1 (B=1, 32K context, 8 verifier queries)"))
        res["wall_s_including_input_generation_and_oracle"] = time.perf_counter() - t0
        results[tag] = res
        print(f"[bench] {tag}: refresh {res['modes']['refresh']['us_per_call_cold']:.1f} us, reuse "
              f"{res['modes']['reuse']['us_per_call_cold']:.1f} us per call", file=sys.stderr, flush=True)
        del case
    main_res = results[headline]
    extra = {}
    if not args.only and not args.no_extra:
        extra["approx_shared_index_variant"] = shared_index_study(torch, oracle, si, 8, (0.0, 0.9), 4, 100, args.warmup)
        # the paper's kernel workload, reduced grid (the full one: --only kernel-workload)
        extra["paper_kernel_workload_reduced_grid"] = kernel_workload_study(torch, oracle, si, 100, 10, contexts=(8192, 65536),
                                                                           gammas=(4, 64), overlaps=(3, 6, 10))

    refresh = main_res["modes"]["refresh"]
    line = {
        "metric": "verified query-tokens/s, NSA verify attention (refresh path: routing + selected/window/compressed + gates)",
        "value": refresh["tokens_per_s_cold"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": refresh["us_per_call_cold"] / 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": main_res["workload"], "mode": "refresh", "cache": "cold (rotating input copies)",
                   "plan": refresh["plan"]},
        "roofline": main_res["roofline"],
        "cpu_baseline": base,
        "us_per_call": refresh["us_per_call_cold"],
        "us_per_call_median_p10_p90_with_an_event_per_call": [refresh["us_per_call_cold_median"], refresh["us_per_call_cold_p10"],
                                                              refresh["us_per_call_cold_p90"]],
        "hbm_frac_whole_call": refresh["hbm_frac_whole_call_cold"],
        "algorithmic_bytes": main_res["algorithmic_bytes"],
        "parity": main_res.get("parity"),
        "kernel_roofs_refresh": main_res["kernel_roofs_refresh"],
        "modes": main_res["modes"],
        "cold_rotation": main_res["cold_rotation"],
        "other_workloads": [results[t] for t in order if t != headline],
        "device_copy_GBs": copy_gbs,
    }
    line.update(extra)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
