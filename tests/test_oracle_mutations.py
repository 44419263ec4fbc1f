"""The pins must bite: plant one plausible mistake at a time in a copy of the
oracle's C source (on the CPU, in a temporary directory), and check that at
least one pin test fails for it.  The unmodified source must pass them all."""
import os
import subprocess

import pytest

from oracle import tempo_oracle as oracle_mod
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle_mod.__file__)), "tempo_oracle.c")

PIN_TESTS = [
    pins.test_p1_first_step_returns_v0_bits,
    pins.test_p2_window_clamps_to_causal_and_w1_is_vt,
    pins.test_p2_window_counts_exactly_w_keys,
    pins.test_p3_uniform_weights_give_mean,
    pins.test_p4_padded_masked_formulation,
    lambda: pins.test_p5_static_tiling_equals_plain(3),
    pins.test_p6_two_key_closed_form_and_dominant_logit,
    pins.test_p7_gqa_mapping,
    pins.test_p8_invariances,
    pins.test_p9_brute_force_tiny,
    pins.test_p9_per_sequence_steps,
    pins.test_p10_integer_closed_forms,
    pins.test_p10_printed_inverse_window_example,
    pins.test_p10_static_tiling_fixture,
    pins.test_p11_rope_closed_forms,
    pins.test_p11_rope_is_a_rotation_with_relative_positions,
    pins.test_p11_rope_table_matches_closed_forms_and_rope,
    pins.test_p12_release_follows_the_printed_inverse_window,
    pins.test_p12_release_closed_forms_and_safety,
    pins.test_p12_ring_blocks_is_the_smallest_circular_store_that_holds,
    pins.test_p13_discounted_sum_printed_parameters_and_closed_forms,
    pins.test_p13_discounted_sum_impulse_recurrence_and_second_evaluator,
]

# (name, text to find, replacement) -- each is a mistake someone could make.
MUTATIONS = [
    ("scale dropped", "z *= scale;", "z *= 1.0;"),
    ("scale applied twice", "z *= scale;", "z *= scale * scale;"),
    ("sign of the exponent", "exp(z - zmax)", "exp(zmax - z)"),
    ("no normalisation", "ov[d] /= denom;", "ov[d] /= 1.0;"),
    ("gqa by modulo", "const int g = h / group;", "const int g = h % Hkv;"),
    ("window one key too wide", "hi - window + 1 > 0 ? hi - window + 1 : 0", "hi - window > 0 ? hi - window : 0"),
    ("window one key too narrow", "hi - window + 1 > 0 ? hi - window + 1 : 0", "hi - window + 2 > 0 ? hi - window + 2 : 0"),
    ("query does not see its own key", "for (int j = lo; j <= hi; ++j) {\n        const double* kv = K + (((size_t)b * T + j) * Hkv + g) * D;\n        const double* vv",
     "for (int j = lo; j < hi + (hi == lo); ++j) {\n        const double* kv = K + (((size_t)b * T + j) * Hkv + g) * D;\n        const double* vv"),
    ("K indexed head-major", "const double* kv = K + (((size_t)b * T + j) * Hkv + g) * D;\n        const double* vv",
     "const double* kv = K + (((size_t)b * Hkv + g) * T + j) * D;\n        const double* vv"),
    ("V taken from K", "ov[d] += p * vv[d];", "ov[d] += p * kv[d];"),
    ("dot product drops the last term", "for (int d = 0; d < D; ++d) z += qv[d] * kv[d];\n        z *= scale;\n        const double p",
     "for (int d = 0; d + 1 < D || d == 0; ++d) z += qv[d] * kv[d];\n        z *= scale;\n        const double p"),
    ("per-sequence step ignored", "const int hi = t[b];", "const int hi = t[0];"),
    ("visibility off by one", "return (t - j) < window;", "return (t - j) <= window;"),
    ("tile opens one key late", "if (++slot == Z) { slot = 0; ++tile; }\n  }\n  tile = 0; slot = 0;",
     "if (++slot > Z) { slot = 0; ++tile; }\n  }\n  tile = 0; slot = 0;"),
    ("tile count floor instead of ceil", "for (int j = 0; j <= t; j += Z) ++tiles;", "for (int j = Z; j <= t; j += Z) ++tiles;"),
    ("rope turns clockwise", "yv[i] = xv[i] * c - xv[i + half] * sn;\n        yv[i + half] = xv[i + half] * c + xv[i] * sn;",
     "yv[i] = xv[i] * c + xv[i + half] * sn;\n        yv[i + half] = xv[i + half] * c - xv[i] * sn;"),
    ("rope pairs neighbours", "yv[i] = xv[i] * c - xv[i + half] * sn;\n        yv[i + half] = xv[i + half] * c + xv[i] * sn;",
     "yv[2 * i] = xv[2 * i] * c - xv[2 * i + 1] * sn;\n        yv[2 * i + 1] = xv[2 * i + 1] * c + xv[2 * i] * sn;"),
    ("rope exponent over D/2", "const double angle = (double)t[b] * pow(theta, -2.0 * (double)i / (double)D);",
     "const double angle = (double)t[b] * pow(theta, -2.0 * (double)i / (double)half);"),
    ("rope exponent sign", "const double angle = (double)t[b] * pow(theta, -2.0 * (double)i / (double)D);",
     "const double angle = (double)t[b] * pow(theta, 2.0 * (double)i / (double)D);"),
    ("rope position of sequence 0", "const double angle = (double)t[b] * pow(", "const double angle = (double)t[0] * pow("),
    ("rope second half not rotated", "yv[i + half] = xv[i + half] * c + xv[i] * sn;", "yv[i + half] = xv[i + half];"),
    ("rope table sin and cos swapped", "cos_out[(size_t)t * half + i] = cos(angle);\n      sin_out[(size_t)t * half + i] = sin(angle);",
     "cos_out[(size_t)t * half + i] = sin(angle);\n      sin_out[(size_t)t * half + i] = cos(angle);"),
    ("rope table exponent", "const double angle = (double)t * pow(theta, -2.0 * (double)i / (double)D);",
     "const double angle = (double)t * pow(theta, -(double)i / (double)D);"),
    ("release counts the step just answered as a reader", "for (int later = t + 1; !seen_later && later <= t + window; ++later) {",
     "for (int later = t; !seen_later && later <= t + window; ++later) {"),
    ("release skips the next step", "for (int later = t + 1; !seen_later && later <= t + window; ++later) {",
     "for (int later = t + 2; !seen_later && later <= t + window; ++later) {"),
    ("release counts partial tiles", "for (int first = 0; first + Z <= dead; first += Z) ++tiles;",
     "for (int first = 0; first < dead; first += Z) ++tiles;"),
    ("release under a causal pattern", "if (window == 0) seen_later = 1;", "if (window == 0) seen_later = 0;"),
    ("ring forgets the block of queries", "const int last = first + queries - 1;", "const int last = first;"),
    ("ring measured from the newest key only", "if (visible(j, first, window)) { oldest = j; break; }",
     "if (visible(j, first, window)) { oldest = first; break; }"),
    ("ring counts keys of the first step only", "for (int j = 0; j <= last; ++j) {\n      if (j >= oldest && tile != counted_tile)",
     "for (int j = 0; j <= first; ++j) {\n      if (j >= oldest && tile != counted_tile)"),
    ("discounted sum looks into the past", "for (int j = t; j < stop; ++j) {\n        sum += weight * r[(size_t)b * T + j];",
     "for (int j = t; j < stop; ++j) {\n        sum += weight * r[(size_t)b * T + (2 * t - j < 0 ? 0 : 2 * t - j)];"),
    ("discounted sum window one step too wide", "(n == 0 || t + n > T) ? T : t + n;", "(n == 0 || t + n + 1 > T) ? T : t + n + 1;"),
    ("discounted sum discounts the first reward", "double sum = 0.0, weight = 1.0;", "double sum = 0.0, weight = gamma;"),
    ("discounted sum not clipped at T", "(n == 0 || t + n > T) ? T : t + n;", "(n == 0) ? T : (t + n > T ? T - 1 : t + n);"),
    ("discounted sum forgets to discount", "weight *= gamma;", "weight *= 1.0;"),
    ("discounted sum mixes sequences", "sum += weight * r[(size_t)b * T + j];", "sum += weight * r[j];"),
    ("append slot one late", "for (int j = 0; j < t; ++j) {\n    if (++s == Z)", "for (int j = 0; j <= t; ++j) {\n    if (++s == Z)"),
]


def _build(text, path):
    src = path + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", path, src, "-lm"])
    return oracle_mod._bind(path)


def _failures(lib, monkeypatch):
    monkeypatch.setattr(oracle_mod, "_lib", lib)
    failed = 0
    for test in PIN_TESTS:
        try:
            test()
        except (AssertionError, ValueError):
            failed += 1
    return failed


def test_unmodified_source_passes_every_pin(tmp_path, monkeypatch):
    lib = _build(open(SRC).read(), str(tmp_path / "clean.so"))
    assert _failures(lib, monkeypatch) == 0


@pytest.mark.parametrize("name,find,repl", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, find, repl, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(find) >= 1, f"mutation site for {name!r} not found"
    lib = _build(text.replace(find, repl), str(tmp_path / "mut.so"))
    assert _failures(lib, monkeypatch) >= 1, f"no pin caught: {name}"
