"""Address- and undefined-behaviour-sanitizer leg (CPU only): the C oracle and the library's host-only planner
pieces are rebuilt with -fsanitize=address,undefined and driven through the brute-force and guard / flattening
cases; any report aborts the run (-fno-sanitize-recover) and results must equal the plain builds'."""
import os
import subprocess

import numpy as np
import pytest

import ssv_inputs as si
from brute_force import brute_force_verify
from oracle import planner as op

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
# (a preloaded library may precede the sanitizer runtime in the link order: that is accepted, not an error)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")


@pytest.fixture(scope="module")
def oracle_exe(tmp_path_factory):
    exe = tmp_path_factory.mktemp("san") / "oracle_harness"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", *SAN, os.path.join(HERE, "sanitize", "oracle_harness.c"),
                           os.path.join(ROOT, "oracle", "nsa_verify_oracle.c"), "-o", str(exe), "-lm"])
    return str(exe)


@pytest.fixture(scope="module")
def planner_exe(tmp_path_factory):
    exe = tmp_path_factory.mktemp("san") / "planner_harness"
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", *SAN, os.path.join(HERE, "sanitize", "planner_harness.cpp"),
                           "-o", str(exe)])
    return str(exe)


def run_sanitized_oracle(exe, case, tmp_path, sel_idx=None):
    nsa = case.nsa
    NS_cap = (int(case.seq_lens.max()) + case.T) // nsa.l_sel + 1
    head = np.array([case.B, case.T, case.H, case.H_kv, case.d_k, case.d_v, nsa.l, nsa.d, nsa.l_sel, nsa.n_sel, nsa.w,
                     nsa.n_init, nsa.n_local, 0 if case.dtype == "f32" else 1, int(sel_idx is not None),
                     int(case.parents is not None), case.k.shape[2], case.k_cmp.shape[2], NS_cap, 0], np.int32)
    sel = np.full((case.B, case.T, case.H_kv, nsa.n_sel), -1, np.int32) if sel_idx is None else sel_idx.astype(np.int32)
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        for a in (head, case.q, case.k, case.v, case.k_cmp, case.v_cmp, case.gates.astype(np.float32),
                  case.seq_lens.astype(np.int32), case.n_cmp.astype(np.int32), case.n_query.astype(np.int32)):
            f.write(np.ascontiguousarray(a).tobytes())
        if case.parents is not None:
            f.write(np.ascontiguousarray(case.parents, np.int32).tobytes())
        f.write(np.ascontiguousarray(sel).tobytes())
    r = subprocess.run([exe, str(src), str(dst)], env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    raw = open(dst, "rb").read()
    n_out = case.B * case.T * case.H * case.d_v
    out = np.frombuffer(raw, np.float64, n_out).reshape(case.B, case.T, case.H, case.d_v)
    sel_o = np.frombuffer(raw, np.int32, sel.size, n_out * 8).reshape(sel.shape)
    return out, sel_o


CASES = [
    dict(seed=1, L=[40, 47], T=3, n_sel=3, w=8, dtype="f32", parents=None, n_query=None),
    dict(seed=3, L=[130, 137], T=4, n_sel=4, w=8, dtype="bf16", parents=None, n_query=None),
    dict(seed=6, L=[3, 10], T=4, n_sel=3, w=8, dtype="f32", parents=None, n_query=None),          # context shorter than a block
    dict(seed=11, L=[129, 70], T=6, n_sel=4, w=8, dtype="f32", parents=si.tree_parents((3, 1), "bfs"), n_query=None),
    dict(seed=21, L=[50, 9], T=6, n_sel=5, w=10, dtype="f32", parents=None, n_query=[6, 2]),     # ragged
]


@pytest.mark.parametrize("c", CASES, ids=[f"seed{c['seed']}" for c in CASES])
def test_oracle_under_sanitizers_matches_brute_force(oracle_exe, oracle, tmp_path, c):
    nsa = si.NsaParams(l=8, d=4, l_sel=16, n_sel=c["n_sel"], w=c["w"])
    case = si.make_case("san", c["dtype"], 2, c["T"], 4, 2, 8, 6, nsa, c["L"], c["seed"], rho=0.3, parents=c["parents"],
                        n_query=c["n_query"], workers=1)
    out, sel = run_sanitized_oracle(oracle_exe, case, tmp_path)
    want_out, want_sel, _, _ = brute_force_verify(case)
    assert np.array_equal(sel, want_sel)
    np.testing.assert_allclose(out, want_out, rtol=0, atol=1e-12)
    plain = oracle.nsa_verify(case)
    assert np.array_equal(plain.sel_idx, sel) and np.array_equal(plain.out, out)
    # reuse mode with messy indices (negative, repeated, out of range) reads nothing out of bounds
    messy = sel.copy()
    messy[..., 0] = -7
    messy[..., -1] = 10 ** 6
    messy[:, :, :, 1] = messy[:, :, :, 2]
    out2, _ = run_sanitized_oracle(oracle_exe, case, tmp_path, sel_idx=messy)
    assert np.array_equal(out2, oracle.nsa_verify(case, sel_idx=messy).out)


def test_planner_under_sanitizers_matches_the_python_statement(planner_exe):
    rng = np.random.default_rng(5)
    lines, want = [], []
    for _ in range(24):
        n = int(rng.integers(1, 17))
        expected = np.sort(rng.uniform(2.0, 5.0, n))[::-1].tolist()
        valid = (rng.random(n) < 0.8).tolist()
        if not any(valid):
            valid[int(rng.integers(0, n))] = True
        cfg = op.GuardConfig(alpha=float(rng.choice([0.4, 0.25, 1.0])), ratio=float(rng.choice([0.85, 0.6])),
                             warmup_steps=int(rng.integers(0, 10)), patience=int(rng.integers(1, 7)),
                             max_transitions=int(rng.integers(0, 4)), early_steps=int(rng.choice([0, 0, 40])))
        obs = [(float(rng.integers(8, 40)) / 8.0, float(rng.integers(1, 9)) / 4.0) for _ in range(100)]
        lines.append(" ".join(["guard", repr(cfg.alpha), repr(cfg.ratio), str(cfg.warmup_steps), str(cfg.patience),
                               str(cfg.max_transitions), str(cfg.early_steps), str(n)] + [repr(e) for e in expected] +
                              [str(int(v)) for v in valid] + [str(len(obs))] + [f"{a!r} {t!r}" for a, t in obs]))
        want.append(" ".join(str(x) for x in op.guard_trace(cfg, expected, valid, obs)))
    lines.append("guard 0.4 0.85 8 5 2 0 17 " + " ".join(["1.0"] * 17) + " " + " ".join(["1"] * 17) + " 0")   # too many candidates
    want.append("EINVAL")
    for n in (0, 1, 2, 7, 64, 128):
        parents = [-1] + [int(rng.integers(-1, i)) for i in range(1, n)] if n else []
        for order, name in ((0, "bfs"), (1, "dfs")):
            lines.append(" ".join(["flatten", str(order), str(n)] + [str(p) for p in parents]))
            perm, newp = op.flatten_tree(parents, name)
            want.append("perm" + "".join(f" {x}" for x in perm) + " | new_parents" + "".join(f" {x}" for x in newp))
    for bad in ([0], [-1, 1], [-1, -2], [-1, 5]):
        lines.append(" ".join(["flatten", "0", str(len(bad))] + [str(p) for p in bad]))
        want.append("EINVAL")
    r = subprocess.run([planner_exe], input="\n".join(lines) + "\n", env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    got = [ln.strip() for ln in r.stdout.strip().split("\n")]
    assert got == want
