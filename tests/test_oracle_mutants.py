"""The pins must bite: plant one mistake at a time in a copy of the oracle's C
source (CPU only), load the mutant in place of the real library, and require
that at least one pin fails."""
import ctypes
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_pins as pins
from tests import test_oracle_prefill_pins as ppins

SRC = os.path.join(os.path.dirname(oracle.__file__), "fs_oracle.c")

# (name, text in the oracle, replacement)
MUTANTS = [
    ("dropped_scale", "s[t] = scale * dot;", "s[t] = dot;"),
    ("wrong_exp_sign", "s[t] = exp(s[t] - smax);", "s[t] = exp(smax - s[t]);"),
    ("no_normalisation", "double w = s[t] / denom;", "double w = s[t];"),
    ("values_read_from_keys", "o[d] += w * load_elem(V,", "o[d] += w * load_elem(K,"),
    ("key_index_transposed", "load_elem(K, dtype, ((size_t)t * H + h) * D + d);",
     "load_elem(K, dtype, ((size_t)t * H + h) + (size_t)d * H);"),
    ("query_head_ignored", "load_elem(q, dtype, (size_t)h * D + d)", "load_elem(q, dtype, (size_t)d)"),
    ("last_token_skipped", "for (long t = 0; t < L; ++t) {\n            double dot", "for (long t = 0; t + 1 < L || t == 0; ++t) {\n            double dot"),
    ("scale_is_inverse_d", "scale = 1.0 / sqrt((double)D);", "scale = 1.0 / (double)D;"),
    ("append_off_by_one", "(char *)K + (size_t)len * row", "(char *)K + (size_t)(len > 0 ? len - 1 : 0) * row"),
    ("append_swaps_k_and_v", "memcpy((char *)V + (size_t)len * row, v_new, row);",
     "memcpy((char *)V + (size_t)len * row, k_new, row);"),
    ("bf16_shift_wrong", "<< 16;", "<< 15;"),
]

# the same for the prompt-phase function (its loop variables differ, so each text is unique)
PREFILL_MUTANTS = [
    ("prefill_no_causal_mask", "for (long t = 0; t <= i; ++t) {\n                double dot", "for (long t = 0; t < s; ++t) {\n                double dot"),
    ("prefill_excludes_itself", "for (long t = 0; t <= i; ++t) {\n                double w", "for (long t = 0; t < i || t == 0; ++t) {\n                double w"),
    ("prefill_query_row_fixed", "load_elem(Q, dtype, ((size_t)i * H + h) * D + d)", "load_elem(Q, dtype, ((size_t)0 * H + h) * D + d)"),
    ("prefill_dropped_scale", "sc[t] = scale * dot;", "sc[t] = dot;"),
    ("prefill_wrong_exp_sign", "sc[t] = exp(sc[t] - smax);", "sc[t] = exp(smax - sc[t]);"),
    ("prefill_no_normalisation", "double w = sc[t] / denom;", "double w = sc[t];"),
    ("prefill_output_row_transposed", "double *o = out + ((size_t)i * H + h) * D;", "double *o = out + ((size_t)h * s + i) * D;"),
]

PIN_FUNCS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_") and
             not hasattr(getattr(pins, n), "pytestmark")]
PARAM_PINS = [
    lambda: pins.test_matches_torch_cpu_sdpa_fp64(130, 5, 128),
    lambda: pins.test_stored_types_widen_exactly("bf16"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_planted_mistake_is_caught(name, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found"
    mutated = text.replace(old, new, 1)
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    real = oracle._load()
    lib = ctypes.CDLL(str(so))
    for fn in ("fso_append", "fso_attention_job", "fso_decode_step", "fso_prefill_attention_job"):
        getattr(lib, fn).argtypes = getattr(real, fn).argtypes
        getattr(lib, fn).restype = getattr(real, fn).restype
    monkeypatch.setattr(oracle, "_lib", lib)
    caught = []
    for f in PIN_FUNCS + PARAM_PINS:
        try:
            f()
        except (AssertionError, RuntimeError):
            caught.append(getattr(f, "__name__", "param"))
    assert caught, f"no pin noticed mutant {name}"


PREFILL_PIN_FUNCS = [getattr(ppins, n) for n in dir(ppins) if n.startswith("test_") and
                     not hasattr(getattr(ppins, n), "pytestmark")]
PREFILL_PARAM_PINS = [
    lambda: ppins.test_matches_torch_cpu_causal_sdpa_fp64(19, 4, 64),
    lambda: ppins.test_stored_types_widen_exactly("bf16"),
]


@pytest.mark.parametrize("name,old,new", PREFILL_MUTANTS, ids=[m[0] for m in PREFILL_MUTANTS])
def test_every_planted_mistake_in_the_prompt_phase_is_caught(name, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found or not unique"
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(text.replace(old, new, 1))
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"])
    real = oracle._load()
    lib = ctypes.CDLL(str(so))
    for fn in ("fso_append", "fso_attention_job", "fso_decode_step", "fso_prefill_attention_job"):
        getattr(lib, fn).argtypes = getattr(real, fn).argtypes
        getattr(lib, fn).restype = getattr(real, fn).restype
    monkeypatch.setattr(oracle, "_lib", lib)
    caught = []
    for f in PREFILL_PIN_FUNCS + PREFILL_PARAM_PINS:
        try:
            f()
        except (AssertionError, RuntimeError):
            caught.append(getattr(f, "__name__", "param"))
    assert caught, f"no pin noticed mutant {name}"
