"""Mutation check of the oracle's pins (CPU only): each plausible mistake planted in a copy of
oracle/nsa_verify_oracle.c (a dropped factor, a wrong sign or index, an off-by-one boundary, swapped
operands) must make at least one pin of tests/test_oracle_pins.py fail.  The mistakes are planted in the
oracle, on the CPU; nothing here touches the GPU path."""
import ctypes
import inspect
import os
import subprocess

import pytest

import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "nsa_verify_oracle.c")

MUTATIONS = [
    ("softmax scale dropped", "score_tmp[r] = scale * acc;", "score_tmp[r] = acc;"),
    ("softmax exponent sign", "exp(score_tmp[r] - mx)", "exp(mx - score_tmp[r])"),
    ("compressed block visible one token early", "c * p->d + p->l <= E", "c * p->d + p->l <= E + 1"),
    ("importance index sign (earlier blocks)", "(int64_t)a_ratio * j + m - n2", "(int64_t)a_ratio * j - m - n2"),
    ("window one position too wide", "kpos > pos_i - p->w &&", "kpos >= pos_i - p->w &&"),
    ("ties to the larger index", "imp[j] > imp[best])) best = j;", "imp[j] >= imp[best])) best = j;"),
    ("one local block too many", "int64_t j = J - p->n_local + 1; j <= J", "int64_t j = J - p->n_local; j <= J"),
    ("selected and window gates swapped", "(double)gt[1] * oslc[e] + (double)gt[2] * owin[e]",
     "(double)gt[2] * oslc[e] + (double)gt[1] * owin[e]"),
    ("draft key position by slot instead of depth", "s < L ? s : L + depth[s - L];", "s;"),
    ("K and V row strides transposed in the compressed branch",
     "attend(q, q_off, k_cmp, kc_off, d_k, v_cmp, vc_off, d_v, cmp_rows", "attend(q, q_off, k_cmp, kc_off, d_v, v_cmp, vc_off, d_k, cmp_rows"),
    ("heads of the group not summed into the importance", "if (c >= 0 && c < ncv) imp[j] += prob[c];",
     "if (c >= 0 && c < ncv) imp[j] = prob[c];"),
    ("own block taken from the depth instead of the slot", "const int64_t J = (L + i) / p->l_sel;",
     "const int64_t J = (L + depth[i]) / p->l_sel;"),
]


def _pin_calls():
    """Every pin of test_oracle_pins as a zero-argument callable per parameter set."""
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_"):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        sets = [{}]
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            new = []
            for vals in m.args[1]:
                vals = vals if len(names) > 1 else (vals,)
                new += [dict(s, **dict(zip(names, vals))) for s in sets]
            sets = new
        for kw in sets:
            calls.append((name, fn, kw))
    return calls


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_fails_a_pin(oracle, tmp_path, monkeypatch, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not unique: {old!r}"
    mutated = tmp_path / "mutated.c"
    mutated.write_text(text.replace(old, new))
    lib_path = tmp_path / "libmutated.so"
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", str(lib_path), str(mutated), "-lm"])
    oracle._load()                                        # the genuine library's prototypes are the template
    lib = ctypes.CDLL(str(lib_path))
    lib.ssv_oracle_nsa_verify.restype = ctypes.c_int
    lib.ssv_oracle_nsa_verify.argtypes = [ctypes.c_void_p] * 20
    lib.ssv_oracle_threads.restype = ctypes.c_int
    monkeypatch.setattr(oracle, "_lib", lib)
    failed = []
    for name, fn, kw in _pin_calls():
        try:
            fn(oracle, **kw)
        except Exception:                                 # any failing pin counts (assertion, shape, lookup)
            failed.append(name)
    assert failed, f"no pin noticed: {what}"


def test_unmutated_oracle_passes_every_pin_through_this_harness(oracle):
    for name, fn, kw in _pin_calls():
        fn(oracle, **kw)
