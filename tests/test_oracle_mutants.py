"""Do the pins have teeth?  Each case plants one plausible mistake (a dropped term, a wrong sign, index
or tie rule, a swapped bit order) in a copy of the oracle's C source, builds it, and runs the pin tests
named for it against that copy in a child process: at least one of them has to fail.  CPU only; the
oracle in the tree is never touched."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "co3_oracle.c")
PINS = "tests/test_oracle_pins.py"
BIAS = "tests/test_oracle_bias_rule.py"
LAYERS = "tests/test_oracle_layer_codes.py"

# (name, text in the source (must occur exactly once), replacement, test file, -k expression)
MUTANTS = [
    ("ties_round_up", "return (fmod(lo, 2.0) == 0.0) ? lo : lo + 1.0;", "return lo + 1.0;",
     PINS, "float16 or float8 or ties_to_even"),
    ("no_gradual_underflow", "int e = ex > e_min ? ex : e_min; /* clamped exponent */", "int e = ex;",
     PINS, "float16 or ties_to_even"),
    ("mantissa_carry_dropped", "            e += 1;\n            r = two_M;", "            r = two_M;",
     PINS, "idempotent or monotone or float16"),
    ("saturation_one_binade_late", "if (f > F) { /* above the top binade", "if (f > F + 1) { /* above the top binade",
     PINS, "ties_to_even or monotone or error_feedback_identities"),
    ("level_exponent_off_by_one", "return ldexp(1.0 + frac, e_min + f - 1);", "return ldexp(1.0 + frac, e_min + f);",
     PINS, "float16 or float8 or e1m2"),
    ("negative_zero_emitted", "int s = (signbit(x) && !(f == 0 && m == 0)) ? 1 : 0;", "int s = signbit(x) ? 1 : 0;",
     PINS, "monotone_and_odd or idempotent or empirical_histogram"),
    ("anchor_ceil_instead_of_floor", "            A = ex2 - 1;", "            A = ex2;",
     PINS, "anchor_is_binade"),
    ("memory_subtracted", "volatile float x = g[i] + decayed;       /* one rounding */", "volatile float x = g[i] - decayed;",
     PINS, "telescopes or error_feedback_identities"),
    ("new_memory_sign", "volatile float e_new = x - v;            /* one rounding */", "volatile float e_new = v - x;",
     PINS, "telescopes or error_feedback_identities"),
    ("node_wins_weight_tie", "if (have_leaf && (!have_node || w[q1] <= w[q2]))", "if (have_leaf && (!have_node || w[q1] < w[q2]))",
     PINS, "huffman_hand_worked or huffman_closed_forms"),
    ("leaf_order_tie_reversed", "(weights[leaf_sym[j]] == weights[s] && leaf_sym[j] > s))) {",
     "(weights[leaf_sym[j]] == weights[s] && leaf_sym[j] < s))) {", PINS, "huffman_hand_worked"),
    ("canonical_increment_after_shift", "code[k] = (prev_code + 1) << (l - prev_len);",
     "code[k] = (prev_code << (l - prev_len)) + 1;", PINS, "canonical_codes"),
    ("stream_lsb_first", "if ((c >> b) & 1)\n                words[p / 64] |= (uint64_t)1 << (63 - (p % 64));",
     "if ((c >> b) & 1)\n                words[p / 64] |= (uint64_t)1 << (p % 64);", PINS,
     "bitstream_hand_worked or bitstream_roundtrip"),
    ("chunk_offset_after_symbol", None, None, PINS, "bitstream_hand_worked or bitstream_roundtrip"),
    ("mean_by_reciprocal", "                acc = acc + v;\n            }\n            volatile float mean = acc / (float)U;",
     "                acc = acc + v;\n            }\n            volatile float mean = acc * (1.0f / (float)U);",
     PINS, "average_exact"),
    ("anchor_of_user_zero_for_all",
     "co3o_symbol_value(sym[(int64_t)u * stride + i], anchor[(int64_t)u * nseg + s], E, M);\n                acc = acc + v;",
     "co3o_symbol_value(sym[(int64_t)u * stride + i], anchor[s], E, M);\n                acc = acc + v;", PINS,
     "average_exact"),
    ("histogram_drops_last_element", "    for (int64_t i = 0; i < n; ++i) {\n        if (sym[i] >= K)\n            return CO3O_EINVAL;",
     "    for (int64_t i = 0; i + 1 < n; ++i) {\n        if (sym[i] >= K)\n            return CO3O_EINVAL;", PINS,
     "histogram_is_bincount"),
    ("level_divided_before_rounding", "volatile float ghat = co3o_symbol_value(q, A, E, M) / c;",
     "volatile float ghat = co3o_symbol_value(q, A, E, M) * c;", BIAS, "scaled_conversion or power_of_two_multiplier"),
    ("multiplier_not_applied", "volatile float y = c * x;", "volatile float y = x;", BIAS,
     "scaled_conversion or power_of_two_multiplier or rule_beats"),
    ("layer_code_of_first_tensor", "            int l = len[(int64_t)s * K + sym[i]];\n            uint64_t c = code[(int64_t)s * K + sym[i]];",
     "            int l = len[sym[i]];\n            uint64_t c = code[sym[i]];", LAYERS, "concatenation or single_tensor"),
    ("layer_counts_pooled", "            counts[(int64_t)s * K + sym[i]] += 1;\n        }", "            counts[sym[i]] += 1;\n        }", LAYERS,
     "concatenation or single_tensor"),
    ("second_moment_is_first", "            s2 += xd * xd;", "            s2 += fabs(xd);", BIAS, "moments_against_exact"),
    ("ratio_wrong_gamma", "return exp(2.0 * lgamma(2.0 / beta) - lgamma(1.0 / beta) - lgamma(3.0 / beta));",
     "return exp(2.0 * lgamma(2.0 / beta) - lgamma(1.0 / beta) - lgamma(2.0 / beta));", BIAS, "ratio_closed_forms or fit_inverts"),
    ("polynomial_sign", "0.46 - 2.85 * b + 5.37 * b * b", "0.46 + 2.85 * b + 5.37 * b * b", BIAS, "polynomial_matches or printed_fit"),
    ("scale_multiplies_alpha", "double c = co3o_bias_poly(beta) / alpha;", "double c = co3o_bias_poly(beta) * alpha;",
     BIAS, "scale_limits or rule_beats or printed_fit"),
]


def mutated_source(name, old, new):
    text = open(SRC).read()
    if name == "chunk_offset_after_symbol":
        # the chunk index is recorded after the chunk's first codeword instead of before it
        old = ("        if (i % chunk_syms == 0)\n            chunk_bitoff[i / chunk_syms] = p;\n"
               "        int l = len[sym[i]];\n        uint64_t c = code[sym[i]];\n")
        new = "        int l = len[sym[i]];\n        uint64_t c = code[sym[i]];\n"
        assert text.count(old) == 1, name
        text = text.replace(old, new)
        tail = "            ++p;\n        }\n    }\n    int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;"
        assert text.count(tail) == 1, name
        return text.replace(tail, "            ++p;\n        }\n        if (i % chunk_syms == 0)\n"
                                  "            chunk_bitoff[i / chunk_syms] = p;\n    }\n"
                                  "    int64_t nchunks = (n + chunk_syms - 1) / chunk_syms;")
    assert text.count(old) == 1, f"{name}: the text to replace occurs {text.count(old)} times"
    return text.replace(old, new)


def run_pins(lib, path, expr):
    env = dict(os.environ, CO3_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", path, "-x", "-q", "-k", expr, "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


def build(src_text, out_dir, name):
    c = os.path.join(out_dir, name + ".c")
    so = os.path.join(out_dir, name + ".so")
    open(c, "w").write(src_text)
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-o", so,
                           c, "-lm"])
    return so


def test_unchanged_copy_passes_the_selected_pins(tmp_path):
    """The harness itself: a verbatim copy of the oracle passes what the mutants are run against."""
    so = build(open(SRC).read(), str(tmp_path), "verbatim")
    r = run_pins(so, PINS, "anchor_is_binade or canonical_codes or huffman_hand_worked or average_exact")
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new,path,expr", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, path, expr):
    so = build(mutated_source(name, old, new), str(tmp_path), name)
    r = run_pins(so, path, expr)
    assert r.returncode == 1, f"no pin among '{expr}' failed for the mistake '{name}':\n" + r.stdout[-1500:]
    assert " failed" in r.stdout
