#!/usr/bin/env python3
"""Benchmark of the NSA speculative-verification hot path on one MI355X.

A "step" is one ssv_nsa_verify call in refresh mode: the whole hot path (compressed scan, block
importance, top-n selection, merged selected-block + sliding-window attention, gated combine) over
one batch of seeded synthetic inputs that are already resident in HBM.  The headline workload is
benchmark configuration 1 (B=1, 32K context, 8 verifier queries, 64/4 heads, d_k=192, d_v=128, bf16);
configuration 2 (B=16, 64K, 4 queries), the bandwidth-bound one, is measured in the same run and
reported under "other_workloads".  One JSON line is printed.

Cold numbers rotate over several copies of the inputs so that every call reads memory the previous
calls have pushed out of the 256 MB last-level cache; warm numbers reuse one copy.
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


def algorithmic_bytes(case, sel_idx, C):
    """Bytes the method itself must move for one call (compressed rows once per KV head; raw KV tokens
    of the union of selected blocks and windows once per group of C queries; q, out, gates, indices)."""
    import ssv_inputs as si
    es = 2 if case.dtype == "bf16" else 4
    nsa = case.nsa
    row_b = (case.d_k + case.d_v) * es
    cmp_b = slc_b = win_b = union_b = 0
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
            ncv = max(ncv, min(int(case.n_cmp[b]), si.n_cmp_blocks(L + lead, nsa.l, nsa.d)))
        cmp_b += case.H_kv * ncv * row_b
        for g in range(case.H_kv):
            for q0 in range(0, Tq, C):
                grp = range(q0, min(Tq, q0 + C))
                slc = np.zeros(L + Tq, bool)
                win = np.zeros(L + Tq, bool)
                for i in grp:
                    vis_draft = np.zeros(Tq, bool)
                    vis_draft[list(anc[i])] = True
                    for j in sel_idx[b, i, g]:
                        if j < 0:
                            continue
                        lo, hi = j * nsa.l_sel, min((j + 1) * nsa.l_sel, L + Tq)
                        slc[lo:min(hi, L)] = True
                        if hi > L:
                            s = np.arange(max(lo, L), hi)
                            slc[s] |= vis_draft[s - L]
                    pos = L + int(depth[i])
                    win[max(0, pos - nsa.w + 1):L] = True
                    for t in anc[i]:
                        if pos - nsa.w < L + int(depth[t]) <= pos:
                            win[L + t] = True
                slc_b += int(slc.sum()) * row_b
                win_b += int(win.sum()) * row_b
                union_b += int((slc | win).sum()) * row_b
    tq = int(case.n_query.sum())
    io_b = tq * case.H * (case.d_k + case.d_v) * es + tq * case.H * 3 * 4 + tq * case.H_kv * nsa.n_sel * 4
    return {"compressed": cmp_b, "selected_union": slc_b, "window_union": win_b, "raw_union": union_b,
            "q_out_gates_idx": io_b, "total": cmp_b + union_b + io_b}


def time_calls(torch, devs, steps, warmup):
    """Warm up, then time exactly `steps` calls (rotating over devs) between synchronisations."""
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
    return ev0.elapsed_time(ev1) / steps, wall_ms / steps


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
    t0 = time.perf_counter()
    ev0.record()
    for s in range(steps):
        graphs[s % n].replay()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return ev0.elapsed_time(ev1) / steps, wall_ms / steps


def kernel_breakdown(devs, rounds, repeats):
    """Average launch duration (ms) of every kernel, measured with HIP events inside the library on the call's
    stream.  repeats == 1: one launch per kernel with start/stop events bound to the launch (the dispatch's own
    begin and end, what a kernel trace reports), rotating over the input copies (cold caches).  repeats > 1: that
    many back-to-back launches per event pair on one copy (the event overhead amortises, but inputs of small
    workloads stay cache-resident)."""
    from paper_2605_19893_amd import binding as B
    acc = np.zeros(B.SSV_NUM_TIMINGS)
    n = rounds * len(devs)
    for r in range(n):
        ms = []
        devs[r % len(devs)].run(kernel_ms=ms, repeats=repeats)
        acc += np.asarray(ms)
    return acc / n


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


COLD_ONLY = False   # --cold-only: profiling runs in which every launch of the trace sees cold inputs


def measure_workload(torch, oracle, case, name, tag, steps, warmup, n_copies, parity=True, group_size=0):
    from paper_2605_19893_amd import binding as B
    from paper_2605_19893_amd.device_case import DeviceCase
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    devs = [DeviceCase(case, group_size=group_size) for _ in range(n_copies)]
    res = {"workload": name}
    ref = oracle.nsa_verify(case)
    devs[0].run()
    out, sel = devs[0].results()
    if parity:
        from parity import compare
        rep = compare(case, oracle, ref, out, sel)
        res["parity"] = {"idx_mismatch": rep.n_mismatch, "idx_mismatch_outside_ambiguity": rep.n_mismatch_strict,
                         "ambiguous_units": rep.n_ambiguous, "units": rep.n_units, "max_abs_err": rep.max_abs_err}
    ab = algorithmic_bytes(case, ref.sel_idx, devs[0].plan.C)
    res["algorithmic_bytes"] = ab
    tokens = int(case.n_query.sum())
    out_modes = {}
    raw = {}
    for mode, mname in ((B.SSV_REFRESH, "refresh"), (B.SSV_REUSE, "reuse")):
        for d in devs:
            d.set_mode(mode)
            if mode == B.SSV_REUSE:
                d.set_sel_idx(ref.sel_idx)
        cold_ms, cold_wall = time_calls(torch, devs, steps, warmup)
        nan = float("nan")
        warm_ms, _ = (nan, nan) if COLD_ONLY else time_calls(torch, devs[:1], steps, warmup)
        graph_ms, graph_wall = (nan, nan) if COLD_ONLY else time_graph_replays(torch, devs, steps, warmup)
        kms = kernel_breakdown(devs, 8, 1)
        kms_rep = np.zeros_like(kms) if COLD_ONLY else kernel_breakdown(devs[:1], 2, 20)
        raw[mname] = kms
        nk = B.SSV_NUM_KERNELS
        out_modes[mname] = {k_: (None if isinstance(v_, float) and v_ != v_ else v_) for k_, v_ in {
            "plan": devs[0].plan.as_dict(),
            "us_per_call_cold": cold_ms * 1e3, "us_per_call_warm": warm_ms * 1e3, "us_per_call_cold_wallclock": cold_wall * 1e3,
            "us_per_call_cold_graph_replay": graph_ms * 1e3, "us_per_call_cold_graph_replay_wallclock": graph_wall * 1e3,
            "tokens_per_s_cold": tokens / (cold_ms * 1e-3), "tokens_per_s_warm": tokens / (warm_ms * 1e-3),
            "algorithmic_GBs_cold": ab["total"] / (cold_ms * 1e-3) / 1e9,
            "hbm_frac_whole_call_cold": ab["total"] / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "kernel_us_cold_single_launch": {B.kernel_name(i): float(kms[i] * 1e3) for i in range(nk) if kms[i] > 0},
            "event_pair_overhead_us": float(kms[B.SSV_T_EVENT_PAIR] * 1e3),
            "kernel_us_20_back_to_back_launches": {B.kernel_name(i): float(kms_rep[i] * 1e3) for i in range(nk) if kms_rep[i] > 0},
        }.items()}
    res["modes"] = out_modes
    # roofline of the dominant kernel of the refresh path: algorithmic bytes of that launch over its average
    # duration (one launch with its own start/stop events, cold inputs)
    kms = raw["refresh"]
    dom = int(np.argmax(kms[:B.SSV_NUM_KERNELS]))
    kbytes = {B.SSV_K_STREAM_A: ab["compressed"] + ab["window_union"],
              B.SSV_K_IMPORTANCE: ab["compressed"] * case.d_k // (case.d_k + case.d_v),
              B.SSV_K_STREAM_B: ab["selected_union"]}.get(dom, 0)
    dur_ms = max(kms[dom], 1e-6)
    achieved = kbytes / (dur_ms * 1e-3) / 1e9
    res["roofline"] = {"bound": "hbm", "kernel": B.kernel_name(dom), "achieved": achieved, "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(tag).get(dom),
                       "algorithmic_bytes_per_launch": int(kbytes), "avg_launch_us": float(dur_ms * 1e3)}
    del devs
    torch.cuda.empty_cache()
    return res, ref


def shared_index_study(torch, oracle, si, T, rhos, C, steps, warmup, n_copies=8):
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
            devs = [DeviceCase(case, mode=mode, group_size=C) for _ in range(n_copies)]
            devs[0].run()
            out, sel = devs[0].results()
            rep = compare(case, oracle, ref, out, sel, routed_by=routed_by if mode == B.SSV_REFRESH_SHARED else None)
            cold_ms, _ = time_calls(torch, devs, steps, warmup)
            kms = kernel_breakdown(devs[:1], 2, 20)
            ab = algorithmic_bytes(case, ref.sel_idx, C)
            row[mname] = {"us_per_call_cold": cold_ms * 1e3, "selected_union_bytes": ab["selected_union"],
                          "algorithmic_bytes_total": ab["total"],
                          "parity_max_abs_err": rep.max_abs_err, "idx_mismatch_outside_ambiguity": rep.n_mismatch_strict,
                          "kernel_us_20_back_to_back_launches": {B.kernel_name(i): float(kms[i] * 1e3)
                                                                  for i in range(B.SSV_NUM_KERNELS) if kms[i] > 0}}
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
    N in {8K..64K}.  The adjacent-query overlap s is steered through the correlation rho of the synthetic
    queries (rho = 0 for the lower bound s ~ 3; bisection on the oracle's indices for s ~ 6 and 10), so that
    refresh and reuse calls see the same, data-driven index sets.  Variants: per-query execution (C = 1), the
    paper's exact variant (C = 2), this build's default grouping (64 rows: C = min(gamma, 16)), and the
    approximate shared-index variant (C = 4), each with index construction (refresh) and without (reuse)."""
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
            for target in overlaps:
                lo, hi, rho = 0.0, 1.0, 0.0
                if target > 3:
                    for _ in range(9):      # overlap grows with rho
                        rho = 0.5 * (lo + hi)
                        si._fill_queries(case, case.seed, rho)
                        if mean_adjacent_overlap(oracle.nsa_verify(case).sel_idx, case.n_query) < target:
                            lo = rho
                        else:
                            hi = rho
                si._fill_queries(case, case.seed, rho)
                exact = oracle.nsa_verify(case)
                shared = oracle.nsa_verify_shared(case, 4)
                routed_by = oracle.group_representatives(case, 4)
                for d in devs:
                    d.set_queries(case.q)
                row = {"N": N, "gamma": gamma, "target_overlap": target, "rho": rho,
                       "mean_adjacent_overlap": mean_adjacent_overlap(exact.sel_idx, case.n_query), "input_copies": n_copies}
                variants = (("per_query", B.SSV_REFRESH, 1, exact), ("exact_C2", B.SSV_REFRESH, 2, exact),
                            ("exact_default_C", B.SSV_REFRESH, 0, exact), ("shared_C4", B.SSV_REFRESH_SHARED, 4, shared))
                worst = 0.0
                for vname, mode, C, ref in variants:
                    for d in devs:
                        d.set_group_size(C, mode)
                    devs[0].run()
                    out, sel = devs[0].results()
                    rep = compare(case, oracle, ref, out, sel, routed_by=routed_by if mode == B.SSV_REFRESH_SHARED else None)
                    assert rep.n_mismatch_strict == 0, (vname, rep.line())
                    worst = max(worst, rep.max_abs_err)
                    t_refresh, _ = time_calls(torch, devs, steps, warmup)
                    for d in devs:      # indices are an input now: the shared sets need no particular grouping
                        d.set_group_size(0 if mode == B.SSV_REFRESH_SHARED else C, B.SSV_REUSE)
                        d.set_sel_idx(ref.sel_idx)
                    devs[0].run()
                    out2, _ = devs[0].results()
                    worst = max(worst, float(np.abs(out2 - ref.out).max()))
                    t_reuse, _ = time_calls(torch, devs, steps, warmup)
                    row[vname] = {"C": int(devs[0].plan.C), "share_group": C if mode == B.SSV_REFRESH_SHARED else 0, "refresh_us": t_refresh * 1e3, "reuse_us": t_reuse * 1e3}
                base = row["per_query"]["refresh_us"]
                row["speedup_over_per_query_refresh"] = {f"{v}_{m}": base / row[v][f"{m}_us"]
                                                         for v in ("per_query", "exact_C2", "exact_default_C", "shared_C4")
                                                         for m in ("refresh", "reuse")}
                row["index_construction_share_of_refresh"] = 1.0 - row["exact_default_C"]["reuse_us"] / row["exact_default_C"]["refresh_us"]
                row["parity_max_abs_err"] = worst
                rows.append(row)
                print(f"[kernel workload] N={N} gamma={gamma} s~{row['mean_adjacent_overlap']:.1f}: " +
                      " ".join(f"{v}={row[v]['refresh_us']:.0f}/{row[v]['reuse_us']:.0f}us" for v, *_ in variants),
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
        kh, vh = None, None
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


def cpu_baseline(oracle, case, budget_s=12.0):
    """The oracle as it stands, timed on this machine's host cores on the same workload."""
    threads = oracle.default_threads()
    tokens = int(case.n_query.sum())
    t0 = time.perf_counter()
    reps = 0
    while True:
        oracle.nsa_verify(case)
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s or reps >= 2000:
            break
    return {"value": tokens * reps / el, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"the full headline workload ({tokens} verifier queries x all heads), {reps} repetitions, "
                      f"{el:.1f} s of wall time on {threads} OpenMP threads", "ms_per_call": el / reps * 1e3}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--rho", type=float, default=0.5)
    ap.add_argument("--no-extra", action="store_true", help="skip the configuration-2 measurement")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cold-only", action="store_true",
                    help="skip the warm-input, back-to-back and graph-replay measurements (for kernel traces: every "
                         "launch then runs on cold inputs, like the timed calls)")
    ap.add_argument("--only", default="", help="measure only this workload (cfg1, cfg2, cfg3 or cfg4; for profiling runs), "
                    "'shared': the shared-index study alone, at T = 8 and T = 32, or 'kernel-workload': the paper's "
                    "isolated-kernel workload (32/8 heads of dimension 64, draft lengths 4 and 64, contexts 8K-64K), "
                    "or 'compress': the compressed-cache construction kernel")
    ap.add_argument("--group-size", type=int, default=0, help="verifier queries per workgroup (0 = library default)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="kept for the profiling commands: the plain 1 GiB device-to-device copy (a known-size reference for HBM "
                         "byte counters) now runs in every invocation")
    args = ap.parse_args()
    global COLD_ONLY
    COLD_ONLY = args.cold_only
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
    others = []
    main_res = None
    if args.only in ("", "cfg1"):
        case1 = si.config1(args.rho)
        main_res, _ = measure_workload(torch, oracle, case1, f"cfg1: B=1 L=32768 T=8 chain rho={args.rho} H=64/4 d_k=192 d_v=128 "
                                       "l=32 d=16 l'=64 n=16 w=512", "cfg1", args.steps, args.warmup, n_copies=8)
    for tag, make, label, copies in (
            ("cfg3", lambda: si.config3("bfs"), "cfg3: B=4 L=131072 T=40 tree (4,3,2) BFS order", 1),
            ("cfg4", lambda: si.config4(), "cfg4: B=32 L log-uniform 4K..128K T=16 chain rho=0.7", 1)):
        if args.only == tag:
            casex = make()
            main_res, _ = measure_workload(torch, oracle, casex, label, tag, max(10, args.steps // 10), 3, n_copies=copies,
                                           group_size=args.group_size)
            del casex
    if args.only == "cfg2" or (not args.no_extra and args.only == ""):
        case2 = si.config2()
        r2, _ = measure_workload(torch, oracle, case2, "cfg2: B=16 L=65536 T=4 chain rho=0.7, 5% keys x4", "cfg2",
                                 max(20, args.steps // 4), max(5, args.warmup // 4), n_copies=2)
        del case2
        if main_res is None:
            main_res = r2
        else:
            others.append(r2)
    if args.only == "compress":
        print(json.dumps({"compressed_cache_construction": compress_study(torch, si, max(20, args.steps // 10), 5),
                          "device_copy_GBs": copy_gbs}))
        return
    if args.only == "kernel-workload":
        rows = kernel_workload_study(torch, oracle, si, max(50, args.steps // 3), max(5, args.warmup // 3))
        print(json.dumps({"paper_kernel_workload": rows}))
        return
    shared_rows = None
    if args.only in ("", "shared"):
        shared_rows = shared_index_study(torch, oracle, si, 8, (0.0, 0.5, 0.9), 4, max(50, args.steps // 3), args.warmup)
        if args.only == "shared":
            shared_rows += shared_index_study(torch, oracle, si, 32, (0.0, 0.5, 0.9), 4, max(50, args.steps // 3), args.warmup)
            print(json.dumps({"approx_shared_index_variant": shared_rows}))
            return
    base = None
    if not args.no_cpu_baseline and args.only in ("", "cfg1"):
        base = cpu_baseline(oracle, case1)

    refresh = main_res["modes"]["refresh"]
    tokens_per_s = refresh["tokens_per_s_cold"]
    line = {
        "metric": "verified query-tokens/s, NSA verify attention (refresh path: routing + selected/window/compressed + gates)",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": refresh["us_per_call_cold"] / 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": main_res["workload"], "mode": "refresh", "cache": "cold (rotating input copies)",
                   "plan": main_res["modes"]["refresh"]["plan"]},
        "roofline": main_res["roofline"],
        "cpu_baseline": base,
        "us_per_call": refresh["us_per_call_cold"],
        "hbm_frac_whole_call": refresh["hbm_frac_whole_call_cold"],
        "algorithmic_bytes": main_res["algorithmic_bytes"],
        "parity": main_res.get("parity"),
        "modes": main_res["modes"],
        "other_workloads": others,
        "approx_shared_index_variant": shared_rows,
        "device_copy_GBs": copy_gbs,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
