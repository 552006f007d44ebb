"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of oracle/attn_oracle.c (a
flipped sign, a dropped factor, an off-by-one bound, a swapped operand, a wrong head mapping),
builds the copy and runs the pin functions of tests/test_oracle_pins.py against it: at least one
pin must fail.  The mistakes are planted in the oracle, on the CPU; the unmodified source must
pass the same runner."""
import ctypes
import os
import subprocess

import pytest

from oracle import attn_oracle as orc
import test_oracle_pins as pins

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "attn_oracle.c")

PIN_FUNCS = [
    lambda: [pins.test_brute_force(l, hq, hkv, d) for l, hq, hkv, d in
             (([3, 5], 2, 1, 4), ([8, 1, 2], 4, 2, 2), ([33, 0, 17], 4, 1, 8))],
    pins.test_packed_equals_unpacked_and_no_cross_contamination,
    pins.test_softmax_rows_sum_to_one_and_match_lse,
    pins.test_length_one_and_first_rows,
    pins.test_uniform_attention_closed_forms,
    pins.test_constant_v_gives_zero_dq_dk,
    pins.test_key_shift_invariance,
    pins.test_causality,
    pins.test_gqa_equals_mha_with_replicated_kv,
    pins.test_finite_differences,
    pins.test_linearity_in_v_and_do,
    pins.test_backward_given_stored_forward_results,
    pins.test_sampled_rows_and_cols_agree_with_full,
]

# (name, text to find, replacement, which occurrence of the text: 0-based)
MUTATIONS = [
    ("sign of dS", "ds[j] = p[j] * (ds[j] - D);", "ds[j] = p[j] * (D - ds[j]);", 0),
    ("scale dropped from dK", "dk[(size_t)j * d + c] += scale * ds[j] * q_i[c];", "dk[(size_t)j * d + c] += ds[j] * q_i[c];", 0),
    ("dS instead of P in dV", "dv[(size_t)j * d + c] += p[j] * do_i[c];", "dv[(size_t)j * d + c] += ds[j] * do_i[c];", 0),
    ("softmax sum misses the diagonal", "for (int j = 0; j <= i; ++j) { p[j] = exp(p[j] - m); l += p[j]; }",
     "for (int j = 0; j <= i; ++j) { p[j] = exp(p[j] - m); if (j < i || i == 0) l += p[j]; }", 0),
    ("score of the diagonal key halved", "p[j] = scale * dot(q_i, k + (size_t)j * d, d);",
     "p[j] = scale * dot(q_i, k + (size_t)j * d, d) * (j == i && i > 0 ? 0.5 : 1.0);", 0),
    ("K and Q swapped in dQ", "dq_i[c] += scale * ds[j] * k[(size_t)j * d + c];", "dq_i[c] += scale * ds[j] * q[(size_t)j * d + c];", 0),
    ("natural log replaced by log2 in LSE", "return m + log(l);", "return m + log2(l);", 0),
    ("GQA group mapping", "unpack(k, hkv, d, row0, L, h / G, ks);", "unpack(k, hkv, d, row0, L, h % hkv, ks);", 0),
    ("O accumulates from the wrong row of V", "o_i[c] += p[j] * v[(size_t)j * d + c];", "o_i[c] += p[j] * v[(size_t)(i - j) * d + c];", 0),
    ("given backward ignores the stored LSE", "p[j] = exp(scale * dot(q_i, k + (size_t)j * d, d) - lse_in[i]);",
     "p[j] = exp(scale * dot(q_i, k + (size_t)j * d, d) - lse_in[0]);", 0),
    ("given backward: D from the wrong row of O", "const double D = dot(do_i, o_in + (size_t)i * d, d);",
     "const double D = dot(do_i, o_in + (size_t)(i > 0 ? i - 1 : 0) * d, d);", 0),
    ("sampled rows: dQ without the scale", "dq_i[c] += scale * p[j] * (ds[j] - D) * ks[(size_t)j * d + c];",
     "dq_i[c] += p[j] * (ds[j] - D) * ks[(size_t)j * d + c];", 0),
]


def run_pins_against(lib_path):
    """Number of pin functions that fail with the oracle library at lib_path."""
    saved = orc._lib
    orc._lib = None
    lib = ctypes.CDLL(lib_path)
    for name in ("hyd_oracle_fwd", "hyd_oracle_bwd", "hyd_oracle_bwd_given", "hyd_oracle_rows", "hyd_oracle_cols",
                 "hyd_oracle_probs", "hyd_oracle_threads"):
        getattr(lib, name).restype = ctypes.c_int
    orc._lib = lib
    failed = 0
    try:
        for f in PIN_FUNCS:
            try:
                f()
            except (AssertionError, ValueError, FloatingPointError):
                failed += 1
    finally:
        orc._lib = saved
    return failed


def build(src_text, out_dir, tag):
    c = os.path.join(out_dir, f"oracle_{tag}.c")
    so = os.path.join(out_dir, f"oracle_{tag}.so")
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", so, c, "-lm"])
    return so


def test_unmodified_oracle_passes_the_runner(tmp_path):
    assert run_pins_against(build(open(SRC).read(), str(tmp_path), "clean")) == 0


@pytest.mark.parametrize("name,old,new,occ", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_at_least_one_pin(tmp_path, name, old, new, occ):
    text = open(SRC).read()
    parts = text.split(old)
    assert len(parts) > occ + 1, f"mutation site not found: {name}"
    mutated = old.join(parts[:occ + 1]) + new + old.join(parts[occ + 1:])
    assert mutated != text
    failed = run_pins_against(build(mutated, str(tmp_path), "mut"))
    assert failed >= 1, f"no pin noticed: {name}"
