"""Do the pins bite?  Each case plants one plausible mistake in a copy of the C oracle (a dropped
term, a wrong sign or index, swapped operands), builds it, and runs the pins of test_oracle_pins.py
against the broken copy: at least one pin must fail for every planted mistake.  Everything here
happens on the CPU, in copies under a temporary directory; the oracle itself is never touched.
"""
import inspect
import os
import subprocess

import pytest

from oracle import reference
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(reference.__file__)), "pod_oracle.c")

# (name, text in pod_oracle.c, replacement); every text must occur in the source
MUTATIONS = [
    ("causal limit one key short", "for (int j = 0; j <= pos; ++j)", "for (int j = 0; j < pos + (pos == 0); ++j)"),
    ("causal limit one key long", "const int pos = kv_len - q_len + i;", "const int pos = kv_len - q_len + i + (i + 1 < q_len);"),
    ("position ignores the cached prefix", "const int pos = kv_len - q_len + i;", "const int pos = i;"),
    ("query head mapped round-robin", "const int kvh = h / group;", "const int kvh = h % n_kv_heads;"),
    ("exponent sign flipped", "score[j] = exp(score[j] - smax);", "score[j] = exp(smax - score[j]);"),
    ("normalisation dropped", "for (int c = 0; c < head_dim; ++c) o[c] /= wsum;", "(void)wsum;"),
    ("scale dropped", "score[j] = softmax_scale * dot;", "score[j] = dot;"),
    ("scores read V instead of K", "const uint16_t *kr = k_cache + cache_offset(&cv, cache_row, j, kvh);",
     "const uint16_t *kr = v_cache + cache_offset(&cv, cache_row, j, kvh);"),
    ("block offset uses the block index", "slot = t % c->block_size;", "slot = (t / c->block_size) % c->block_size;"),
    ("block table row ignored", "c->block_table[(int64_t)row * c->max_blocks_per_seq + t / c->block_size]",
     "c->block_table[t / c->block_size]"),
    ("head-major order ignored", "if (c->head_major)", "if (0)"),
    ("head-major strides swapped", "((int64_t)kvh * n_slots + slot) * c->head_dim", "((int64_t)slot * c->n_kv_heads + kvh) * c->head_dim"),
    ("bfloat16 widened from the wrong half", "uint32_t w = (uint32_t)b << 16;", "uint32_t w = (uint32_t)b << 15;"),
    ("binary16 exponent bias off by one", "v = ldexp((double)(mant | 0x400), expo - 25);", "v = ldexp((double)(mant | 0x400), expo - 24);"),
    ("decode rows taken from the prefill queries", ": decode_q + ((int64_t)m[0] * n_q_heads + h) * head_dim;",
     ": decode_q + ((int64_t)0 * n_q_heads + h) * head_dim;"),
    ("maximum not subtracted", "if (score[j] > smax) smax = score[j];", "if (j == 0) smax = score[j] + 800.0;"),
]


def _pin_cases():
    """Every pin with the argument sets its parametrize marks give it."""
    cases = []
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not inspect.isfunction(fn):
            continue
        arg_sets = [{}]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [n.strip() for n in mark.args[0].split(",")]
            values = [v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,) for v in mark.args[1]]
            arg_sets = [dict(a, **dict(zip(names, v))) for a in arg_sets for v in values]
        cases += [(name, fn, kw) for kw in arg_sets]
    return cases


def _failing_pins(lib):
    saved = reference._lib
    reference._lib = lib
    failed = []
    try:
        for name, fn, kw in _pin_cases():
            try:
                fn(**kw)
            except Exception:              # an assertion, or the broken oracle rejecting its input
                failed.append((name, kw))
    finally:
        reference._lib = saved
    return failed


def test_the_unbroken_oracle_passes_every_pin_when_run_this_way():
    assert _failing_pins(reference._load()) == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_at_least_one_pin(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation text not found in the oracle: {old!r}"
    src = tmp_path / "broken_oracle.c"
    src.write_text(text.replace(old, new))
    lib_path = tmp_path / "libbroken_oracle.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-w", str(src), "-o", str(lib_path), "-lm"],
                   check=True)
    failed = _failing_pins(reference.bind(str(lib_path)))
    print(f"{name}: {len(failed)} pins fail, e.g. {failed[:3]}")
    assert failed, f"no pin notices the planted mistake: {name}"
