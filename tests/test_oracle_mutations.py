"""How sharp are the oracle's pins?  Each case plants ONE plausible mistake in a copy of the C oracle (a dropped
diagonal term, transposed operands, a wrong weight, a missing decay, a wrong head index, ...), builds that copy,
and runs the pins of test_oracle_pins.py against it: at least one pin has to fail.  Everything here runs on
the CPU and touches only copies of the oracle."""
import ctypes
import importlib
import inspect
import itertools
import os
import subprocess

import pytest

import oracle
from oracle import ref

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "la2_oracle.c")

# (name, function the mistake is planted in, text to replace inside that function, replacement, which occurrence)
MUTATIONS = [
    ("fwd_direct drops the diagonal term", "la2_oracle_fwd_direct", "s <= t", "s < t", 0),
    ("fwd_direct swaps the rows of q and k", "la2_oracle_fwd_direct",
     "dot(q + off + t * d, k + off + s * d, d)", "dot(q + off + s * d, k + off + t * d, d)", 0),
    ("fwd_direct weights with v_t instead of v_s", "la2_oracle_fwd_direct", "w * v[off + s * d + j]", "w * v[off + t * d + j]", 0),
    ("bwd_direct: dk takes dv's weight", "la2_oracle_bwd_direct", "dkp[j] += wk * q[", "dkp[j] += wv * q[", 0),
    ("bwd_direct: dk, dv drop the diagonal term", "la2_oracle_bwd_direct", "for (int64_t t = p; t < n; t++)",
     "for (int64_t t = p + 1; t < n; t++)", 0),
    ("bwd_direct: dq contracts do with k instead of v", "la2_oracle_bwd_direct",
     "dot(d_o + off + p * d, v + off + s * d, d)", "dot(d_o + off + p * d, k + off + s * d, d)", 0),
    ("fwd_recurrent: transposed outer product", "la2_oracle_fwd_recurrent", "kt[i] * vt[j]", "kt[j] * vt[i]", 0),
    ("fwd_recurrent: no decay", "la2_oracle_fwd_recurrent", "lam * kv[i * d + j] + kt[i] * vt[j]", "kv[i * d + j] + kt[i] * vt[j]", 0),
    ("fwd_recurrent: output from the transposed state", "la2_oracle_fwd_recurrent", "s += qt[i] * kv[i * d + j]", "s += qt[i] * kv[j * d + i]", 0),
    ("bwd_recurrent: dkv without decay", "la2_oracle_bwd_recurrent(", "lam * dkv[i * d + j] + qt[i] * dot_[j]", "dkv[i * d + j] + qt[i] * dot_[j]", 0),
    ("bwd_recurrent: dk from dkv instead of its transpose", "la2_oracle_bwd_recurrent(", "s += vt[j] * dkv[i * d + j]", "s += vt[j] * dkv[j * d + i]", 0),
    ("bwd_recurrent_state: d_kv_init without the last decay", "la2_oracle_bwd_recurrent_state", "(n > 0) ? lam * g[i]", "(n > 0) ? g[i]", 0),
    ("bwd_recurrent_state: d_kv_final decayed once too often", "la2_oracle_bwd_recurrent_state",
     "(d_kv_final ? d_kv_final[c * d * d + i * d + j] : 0.0)", "(d_kv_final ? lam * d_kv_final[c * d * d + i * d + j] : 0.0)", 0),
    ("decode_step: update without k^T v", "la2_oracle_decode_step",
     "lam * s[i * d + j] + kc[i] * vc[j]", "lam * s[i * d + j]", 0),
    ("decode_step: decay of head 0 for every head", "la2_oracle_decode_step", "lambda[c % H]", "lambda[0]", 0),
    ("power table off by one", "static double *power_table", "pow(lambda, (double)m)", "pow(lambda, (double)(m + 1))", 0),
    ("fwd_direct: decay of the wrong head", "la2_oracle_fwd_direct", "lambda[c % H]", "lambda[c / H % H]", 0),
    ("fwd_rows: drops the diagonal term", "la2_oracle_fwd_rows", "s <= t", "s < t", 0),
    ("bwd_rows: dv contracts q with v instead of k", "la2_oracle_bwd_rows", "dot(q + t * d, k + p * d, d)", "dot(q + t * d, v + p * d, d)", 0),
]


def mutate(source, where, old, new, occurrence):
    start = source.index(where)
    # the function's text runs to the next function definition at column 0 ("\nvoid " / "\nstatic ")
    ends = [e for e in (source.find("\nvoid ", start + 1), source.find("\nstatic ", start + 1)) if e > 0]
    end = min(ends) if ends else len(source)
    body = source[start:end]
    assert body.count(old) > occurrence, "mutation target not found: %r in %s" % (old, where)
    pos = -1
    for _ in range(occurrence + 1):
        pos = body.index(old, pos + 1)
    return source[:start] + body[:pos] + new + body[pos + len(old):] + source[end:]


def pins():
    """Every pin of test_oracle_pins.py as a (name, zero-argument callable), parametrisations expanded."""
    mod = importlib.import_module("test_oracle_pins")
    out = []
    for name, fn in inspect.getmembers(mod, inspect.isfunction):
        if not name.startswith("test_") or "norm" in name:   # the Norm pins test oracle/norm.py, which is numpy
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            out.append((name, fn))
            continue
        names = [m.args[0] for m in marks]
        for combo in itertools.product(*[m.args[1] for m in marks]):
            kwargs = dict(zip(names, combo))
            out.append(("%s%s" % (name, list(combo)), lambda fn=fn, kwargs=kwargs: fn(**kwargs)))
    return out


def test_the_pins_pass_on_the_real_oracle():
    for name, pin in pins():
        pin()


@pytest.mark.parametrize("mutation", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_is_caught(mutation, tmp_path):
    name, where, old, new, occurrence = mutation
    source = open(SRC).read()
    mutant_c = tmp_path / "mutant.c"
    mutant_so = tmp_path / "libmutant.so"
    mutant_c.write_text(mutate(source, where, old, new, occurrence))
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", str(mutant_c), "-o", str(mutant_so), "-lm"])
    ref._load()                      # make sure the real library is built and loaded, then swap it out
    real = ref._lib
    mutant = ctypes.CDLL(str(mutant_so))
    mutant.la2_oracle_num_threads.restype = ctypes.c_int
    caught = []
    try:
        ref._lib = mutant
        for pin_name, pin in pins():
            try:
                pin()
            except AssertionError:
                caught.append(pin_name)
    finally:
        ref._lib = real
    assert caught, "no pin noticed: " + name
    # and the real oracle is back in place
    assert oracle.fwd_direct([[[[1.0]]]], [[[[1.0]]]], [[[[1.0]]]], 0.5)[0, 0, 0, 0] == 1.0


# ---- the same for the numpy oracle of the normalised operator (oracle/norm.py) -----------------------------------
def _norm_mutants():
    import numpy as np

    def fwd_sum_instead_of_mean(q, k, v, lam, eps):
        u = ref.fwd_direct(q, k, v, lam)
        r = 1.0 / np.sqrt(np.sum(u * u, axis=-1) + eps)
        return u * r[..., None], r

    def fwd_eps_outside_the_root(q, k, v, lam, eps):
        u = ref.fwd_direct(q, k, v, lam)
        r = 1.0 / (np.sqrt(np.mean(u * u, axis=-1)) + eps)
        return u * r[..., None], r

    def rows_without_projection(o, rstd, g):
        return np.asarray(rstd)[..., None] * np.asarray(g, dtype=np.float64)

    def rows_projection_not_averaged(o, rstd, g):
        o, g = np.asarray(o, dtype=np.float64), np.asarray(g, dtype=np.float64)
        return np.asarray(rstd)[..., None] * (g - o * np.sum(g * o, axis=-1, keepdims=True))

    def rows_without_rstd(o, rstd, g):
        o, g = np.asarray(o, dtype=np.float64), np.asarray(g, dtype=np.float64)
        return g - o * np.mean(g * o, axis=-1, keepdims=True)

    def state_output_ignores_the_start_state(q, k, v, lam, eps, kv_init=None):
        u = ref.fwd_recurrent(q, k, v, lam)
        _, kvn = ref.fwd_recurrent(q, k, v, lam, kv_init=kv_init, return_state=True)
        r = 1.0 / np.sqrt(np.mean(u * u, axis=-1) + eps)
        return u * r[..., None], r, kvn

    def state_backward_drops_the_final_state_gradient(q, k, v, d_o, lam, eps, kv_init=None, d_kv_final=None):
        from oracle import norm as nm
        o, rstd, _ = nm.fwd_norm_state(q, k, v, lam, eps, kv_init)
        return ref.bwd_recurrent_state(q, k, v, nm.norm_backward_rows(o, rstd, d_o), lam, kv_init=kv_init)

    def state_backward_without_the_row_pass(q, k, v, d_o, lam, eps, kv_init=None, d_kv_final=None):
        return ref.bwd_recurrent_state(q, k, v, d_o, lam, kv_init=kv_init, d_kv_final=d_kv_final)

    return [("segment output ignores the start state", {"fwd_norm_state": state_output_ignores_the_start_state}),
            ("segment backward drops d_kv_final", {"bwd_norm_state": state_backward_drops_the_final_state_gradient}),
            ("segment backward takes d_o for d_u", {"bwd_norm_state": state_backward_without_the_row_pass}),
            ("rstd from the sum of squares", {"fwd_norm": fwd_sum_instead_of_mean}),
            ("eps added outside the root", {"fwd_norm": fwd_eps_outside_the_root}),
            ("backward without the projection term", {"norm_backward_rows": rows_without_projection}),
            ("backward projection not averaged", {"norm_backward_rows": rows_projection_not_averaged}),
            ("backward without rstd", {"norm_backward_rows": rows_without_rstd})]


@pytest.mark.parametrize("mutant", _norm_mutants(), ids=[m[0] for m in _norm_mutants()])
def test_a_planted_mistake_in_the_norm_oracle_is_caught(mutant, monkeypatch):
    from oracle import norm as norm_mod
    name, patches = mutant
    for attr, fn in patches.items():
        monkeypatch.setattr(norm_mod, attr, fn)
        monkeypatch.setattr(oracle, attr, fn)
    if "norm_backward_rows" in patches or "fwd_norm" in patches:   # bwd_norm looks both up in its own module
        monkeypatch.setattr(oracle, "bwd_norm", norm_mod.bwd_norm)
    mod = importlib.import_module("test_oracle_pins")
    caught = []
    for pin_name, fn in inspect.getmembers(mod, inspect.isfunction):
        if not (pin_name.startswith("test_") and "norm" in pin_name):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        combos = itertools.product(*[m.args[1] for m in marks]) if marks else [()]
        for combo in combos:
            try:
                fn(**dict(zip([m.args[0] for m in marks], combo)))
            except AssertionError:
                caught.append(pin_name)
    assert caught, "no pin noticed: " + name
