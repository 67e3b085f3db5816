"""The pins must be able to fail: each planted mistake below is compiled into a copy of the oracle's C source
(on the CPU, in a temporary directory) and the pin functions of test_oracle_pins.py are run against that copy;
at least one of them has to raise.  The mistakes are the plausible ones: a dropped term, a wrong sign or index,
a swapped operand."""
import ctypes
import inspect
import os
import subprocess

import pytest

from oracle import build as oracle_build
from oracle import pq_oracle as O

import test_oracle_pins as pins

HERE = os.path.dirname(os.path.abspath(oracle_build.__file__))

MISTAKES = {
    "scale dropped": ("        s[t] = scale * dot;", "        s[t] = dot;"),
    "maximum not subtracted and overflow": ("        s[t] = exp(s[t] - smax);", "        s[t] = exp(s[t] + 700.0);"),
    "weights not normalised": ("        const double p = s[t] / denom;", "        const double p = s[t];"),
    "wrong sign of the scores": ("            dot += q[k] * keys[t * d + k];", "            dot -= q[k] * keys[t * d + k];"),
    "grouped heads mapped round-robin": ("        const int hkv = hq / G;", "        const int hkv = hq % Hkv;"),
    "value codes read through the key codebook": (
        "v_codes + head * ctx_cap * M, v_codebook + (int64_t)hkv", "v_codes + head * ctx_cap * M, k_codebook + (int64_t)hkv"),
    "key and value codes swapped": (
        "(k_codes + head * ctx_cap * M, k_codebook", "(v_codes + head * ctx_cap * M, k_codebook"),
    "sub-vector gathered back to front": (
        "                out[t * d + i * ds + j] = codebook[((int64_t)i * C + c) * ds + j];",
        "                out[t * d + i * ds + j] = codebook[((int64_t)i * C + c) * ds + (ds - 1 - j)];"),
    "centroid of the neighbouring subspace": (
        "            const int c = codes[t * M + i];", "            const int c = codes[t * M + (i + 1) % M];"),
    "recent rows skipped": ("        if (R > 0) {\n            memcpy(keys", "        if (R > 1000000) {\n            memcpy(keys"),
    "argmin keeps the last of equal distances": ("if (c == 0 || dist < best_dist) {", "if (c == 0 || dist <= best_dist) {"),
    "absolute instead of squared distance": ("dist = fma(diff, diff, dist);", "dist = dist + fabs(diff);"),
    "distance over the first coordinate only": (
        "                for (int j = 0; j < ds; ++j) {\n                    const double diff",
        "                for (int j = 0; j < 1; ++j) {\n                    const double diff"),
    "distance accumulated in single precision": (
        "dist = fma(diff, diff, dist);", "dist = (double)((float)dist + (float)diff * (float)diff);"),
    "differences rounded to single precision": (
        "                    dist = fma(diff, diff, dist);", "                    dist = fma((double)(float)diff, (double)(float)diff, dist);"),
    "farthest centroid": ("if (c == 0 || dist < best_dist) {", "if (c == 0 || dist > best_dist) {"),
}


def pin_functions():
    """Zero-argument callables: every plain pin, and every parameter combination of the parametrized ones."""
    import itertools
    out = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_") or "hypothesis" in name or "random_tiny" in name:
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            if not inspect.signature(fn).parameters:
                out.append(fn)
            continue
        names = [[n.strip() for n in m.args[0].split(",")] for m in marks]
        for combo in itertools.product(*[m.args[1] for m in marks]):
            kw = {}
            for ns, values in zip(names, combo):
                values = values if len(ns) > 1 else (values,)
                kw.update(dict(zip(ns, values)))
            call = lambda fn=fn, kw=kw: fn(**kw)
            call.__name__ = f"{name}[{kw}]"
            out.append(call)
    return out


def load_mutant(tmp_path, old, new):
    src = open(os.path.join(HERE, "pq_oracle.c")).read()
    assert src.count(old) == 1, f"mutation anchor not unique: {old!r}"
    c = tmp_path / "pq_oracle.c"
    c.write_text(src.replace(old, new))
    (tmp_path / "pq_oracle16.c").write_text(open(os.path.join(HERE, "pq_oracle16.c")).read())
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", str(lib),
                           str(c), str(tmp_path / "pq_oracle16.c"), "-lm"])
    return lib


def run_pins_against(lib_path, monkeypatch):
    good = O.lib()                                   # make sure the real library is loaded and typed first
    mutant = ctypes.CDLL(str(lib_path))
    for name in ("oracle_pq_decode", "oracle_pq_encode", "oracle_pq_dequantize", "oracle_dense_attention",
                 "oracle_num_threads", "oracle_set_num_threads"):
        for suffix in ("", "_u16"):
            if hasattr(good, name + suffix):
                fn = getattr(mutant, name + suffix)
                fn.restype = getattr(good, name + suffix).restype
                fn.argtypes = getattr(good, name + suffix).argtypes
    monkeypatch.setattr(O, "_lib", mutant)
    caught = []
    for fn in pin_functions():
        try:
            fn()
        except Exception as e:                       # AssertionError from a pin, or the oracle reporting failure
            caught.append(fn.__name__)
    return caught


def test_unchanged_copy_passes_every_pin(tmp_path, monkeypatch):
    """Control: the same machinery around an unmodified copy reports nothing."""
    old = MISTAKES["scale dropped"][0]
    assert len(pin_functions()) >= 10
    assert run_pins_against(load_mutant(tmp_path, old, old), monkeypatch) == []


@pytest.mark.parametrize("what", sorted(MISTAKES))
def test_planted_mistake_fails_a_pin(what, tmp_path, monkeypatch):
    old, new = MISTAKES[what]
    caught = run_pins_against(load_mutant(tmp_path, old, new), monkeypatch)
    assert caught, f"no pin noticed: {what}"


# ---- the k-means oracle (numpy): the same check, with the mistakes planted in a copy of its source ----
import importlib.util
import sys

import test_kmeans_oracle_pins as kpins
from oracle import pq_kmeans_oracle as KO

KMEANS_MISTAKES = {
    "mean divides by count + 1": ("/ counts[has, None].astype(np.float64)", "/ (counts[has, None].astype(np.float64) + 1.0)"),
    "float64 mean divides by count + 1": ("new[has] = sums[has] / counts[has, None]", "new[has] = sums[has] / (counts[has, None] + 1)"),
    "sum instead of mean": ("mean = sums[has].astype(np.float64) * 2.0 ** -24 / counts[has, None].astype(np.float64)",
                            "mean = sums[has].astype(np.float64) * 2.0 ** -24"),
    "mean rounded through float16 sums": ("fixed = (x.astype(np.float64) * 2.0 ** 24).astype(np.int64)",
                                          "fixed = (x.astype(np.float64) * 2.0 ** 10).astype(np.int64) << 14"),
    "empty cluster moved to the origin": ("    new = np.array(centroids, dtype=np.float16)\n", "    new = np.zeros(centroids.shape, dtype=np.float16)\n"),
    "update uses the labels of the neighbouring subspace": ("labels[h, :, i], cb[h, i], store_dtype)", "labels[h, :, (i + 1) % M], cb[h, i], store_dtype)"),
    "one iteration too few": ("    for _ in range(n_iters):", "    for _ in range(n_iters - 1):"),
    "mean rounded straight from double to float16": ("mean.astype(np.float32).astype(np.float16)", "(mean * (1 + 2.0 ** -12)).astype(np.float16)"),
}


def kmeans_pin_calls():
    calls = []
    for name, fn in inspect.getmembers(kpins, inspect.isfunction):
        if not name.startswith("test_") or "generator" in name:
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if marks:
            for values in marks[0].args[1]:
                calls.append((name, lambda fn=fn, values=values: fn(*values)))
        else:
            calls.append((name, fn))
    return calls


def run_kmeans_pins(src, monkeypatch):
    spec = importlib.util.spec_from_loader("oracle._kmeans_mutant", loader=None)
    mod = importlib.util.module_from_spec(spec)
    mod.__package__ = "oracle"
    exec(compile(src, "pq_kmeans_oracle_mutant.py", "exec"), mod.__dict__)
    for name in ("lloyd_update", "kmeans_lloyd", "inertia"):
        monkeypatch.setattr(KO, name, getattr(mod, name))
    caught = []
    for name, call in kmeans_pin_calls():
        try:
            call()
        except Exception:
            caught.append(name)
    return caught


def test_unchanged_kmeans_copy_passes_every_pin(monkeypatch):
    src = open(KO.__file__).read()
    assert len(kmeans_pin_calls()) >= 6
    assert run_kmeans_pins(src, monkeypatch) == []


@pytest.mark.parametrize("what", sorted(KMEANS_MISTAKES))
def test_planted_kmeans_mistake_fails_a_pin(what, monkeypatch):
    old, new = KMEANS_MISTAKES[what]
    src = open(KO.__file__).read()
    assert src.count(old) == 1, f"mutation anchor not unique: {old!r}"
    caught = run_kmeans_pins(src.replace(old, new), monkeypatch)
    assert caught, f"no pin noticed: {what}"
