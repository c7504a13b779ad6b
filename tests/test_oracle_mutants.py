"""CPU-only: every deliberately broken copy of the oracle must be caught by at least one pin.

The mistakes are planted in a temporary copy of the oracle's source text (never in the tree, never
on the GPU), compiled with the oracle's own flags and run through tests/pins.py."""
import os
import shutil
import subprocess
import sys

import pytest

import pins as pins_mod

TESTS = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(TESTS)

# (name, file, text to replace, replacement)
MUTANTS = [
    ("dev_uses_old_est", "ewma_body.inc", "est = a_est + a_new;\n        REAL diff = est - L[q];",
     "REAL diff = est - L[q];\n        est = a_est + a_new;"),
    ("non_strict_compare", "ewma_body.inc", "(L[q] < thr)", "(L[q] <= thr)"),
    ("threshold_sign", "ewma_body.inc", "REAL thr = est - t;", "REAL thr = est + t;"),
    ("alpha_beta_swapped_est", "ewma_body.inc", "REAL a_new = alpha * L[q];", "REAL a_new = beta * L[q];"),
    ("alpha_beta_swapped_dev", "ewma_body.inc", "REAL b_new = beta * FABS(diff);", "REAL b_new = alpha * FABS(diff);"),
    ("est_not_initialised_to_L0", "ewma_body.inc", "if (q == 0)\n            est = L[0];", ""),
    ("decay_is_alpha", "ewma_body.inc", "const REAL A = one - alpha;", "const REAL A = alpha;"),
    ("decay_b_is_alpha", "ewma_body.inc", "const REAL B = one - beta;", "const REAL B = one - alpha;"),
    ("dev_no_abs", "ewma_body.inc", "beta * FABS(diff)", "beta * (diff)"),
    ("decision_after_update", "ewma_body.inc",
     "REAL t = la * dev;\n        REAL thr = est - t;\n        prune[q] = (uint8_t)(L[q] < thr);\n        REAL a_est = A * est;",
     "REAL a_est = A * est;"),
    ("score_not_squared", "ewma_body.inc", "REAL w2 = w * w;", "REAL w2 = FABS(w);"),
    ("score_ignores_channel", "ewma_body.inc", "L[q] = w2 * hr[q];", "L[q] = w2 * hr[0];"),
    ("nm_keeps_wrong_count", "ewma_body.inc", "if (rank >= m_group - n_keep)", "if (rank >= n_keep)"),
    ("nm_tie_break_reversed", "ewma_body.inc", "L[g + p] == L[g + i] && p < i", "L[g + p] == L[g + i] && p > i"),
    ("nm_keeps_smallest", "ewma_body.inc", "if (L[g + p] < L[g + i]) ++rank;", "if (L[g + p] > L[g + i]) ++rank;"),
    ("mask_bit_order", "ewma_body.inc", "else keep_mask[r * words + (q >> 5)] |= (uint32_t)1 << (q & 31);",
     "else keep_mask[r * words + (q >> 5)] |= (uint32_t)1 << (31 - (q & 31));"),
    ("stats_not_squared", "swiftprune_oracle.c", "acc[q] += x * x;", "acc[q] += fabs(x);"),
    ("stats_ignores_pitch", "swiftprune_oracle.c", "load_elem(X, t * ldx + q, dt)", "load_elem(X, t * in + q, dt)"),
    ("partials_ignore_pitch", "swiftprune_oracle.c", "acc[q] += (double)P[p * ld + q];", "acc[q] += (double)P[p * in + q];"),
    ("partials_squared_again", "swiftprune_oracle.c", "acc[q] += (double)P[p * ld + q];",
     "acc[q] += (double)P[p * ld + q] * (double)P[p * ld + q];"),
    ("partials_skip_first_piece", "swiftprune_oracle.c", "for (int64_t p = 0; p < parts; ++p) {\n        for (int64_t q = 0; q < in; ++q) {\n            acc[q] += (double)P",
     "for (int64_t p = 1; p < parts; ++p) {\n        for (int64_t q = 0; q < in; ++q) {\n            acc[q] += (double)P"),
    ("partials_overwrite", "swiftprune_oracle.c", "acc[q] += (double)P[p * ld + q];", "acc[q] = (double)P[p * ld + q];"),
    ("factor_plus", "swiftprune_oracle.c", "float den = 1.0f - rho;\n        if (!(den > 0.0f))\n            den = FLT_EPSILON;\n        hr[q] = 0.5f / den;",
     "float den = 1.0f + rho;\n        if (!(den > 0.0f))\n            den = FLT_EPSILON;\n        hr[q] = 0.5f / den;"),
    ("factor_f64_no_half", "swiftprune_oracle.c", "hr[q] = 0.5 / den;", "hr[q] = 1.0 / den;"),
    ("S_is_mean", "swiftprune_oracle.c", "*S = (float)s;", "*S = (float)(s / (double)in);"),
    ("f16_wrong_rebias", "swiftprune_oracle.c", "((e + 112u) << 23)", "((e + 127u) << 23)"),
    ("f16_fraction_shift", "swiftprune_oracle.c", "| (m << 13);\n    }\n    memcpy(&f, &u, sizeof f);", "| (m << 12);\n    }\n    memcpy(&f, &u, sizeof f);"),
    ("f16_subnormal_scale", "swiftprune_oracle.c", "(float)m * 0x1p-24f", "(float)m * 0x1p-25f"),
    ("f16_read_as_bf16", "swiftprune_oracle.c", "return f16_to_f32(((const uint16_t *)base)[idx]);", "return bf16_to_f32(((const uint16_t *)base)[idx]);"),
    ("bf16_low_half", "swiftprune_oracle.c", "uint32_t u = (uint32_t)b << 16;", "uint32_t u = (uint32_t)b;"),
    ("literal_never_updates_S", "swiftprune_oracle.c", "S_r = S_new;", ""),
    ("literal_S_grows", "swiftprune_oracle.c", "float S_new = S_r - w2;", "float S_new = S_r + w2;"),
    ("literal_S_loses_w_not_squared", "swiftprune_oracle.c", "float S_new = S_r - w2;", "float S_new = S_r - fabsf(w);"),
    ("literal_S_loses_half_w2", "swiftprune_oracle.c", "float S_new = S_r - w2;", "float S_new = S_r - half_w2;"),
    ("literal_S_updated_when_kept", "swiftprune_oracle.c",
     "                keep_mask[r * words + (i >> 5)] |= (uint32_t)1 << (i & 31);\n            }\n            float a_est",
     "                keep_mask[r * words + (i >> 5)] |= (uint32_t)1 << (i & 31);\n                S_r = S_r - w2;\n            }\n            float a_est"),
    ("literal_S_not_reset_per_row", "swiftprune_oracle.c",
     "    for (int64_t r = 0; r < out; ++r) {\n        float S_r = S;", "    float S_r = S;\n    for (int64_t r = 0; r < out; ++r) {"),
    ("literal_score_uses_initial_S", "swiftprune_oracle.c", "float rho = xsq[i] / S_r;", "float rho = xsq[i] / S;"),
    ("literal_no_half", "swiftprune_oracle.c", "float half_w2 = 0.5f * w2;", "float half_w2 = w2;"),
    ("topk_nan_by_payload", "swiftprune_oracle.c", "s[q].index = (L[q] != L[q]) ? q + in : q;",
     "s[q].index = (L[q] != L[q]) ? in + in - q : q;"),
    ("topk_nan_below_inf", "swiftprune_oracle.c", "s[q].score = (L[q] != L[q]) ? INFINITY : L[q];\n            s[q].index = (L[q] != L[q]) ? q + in : q;",
     "s[q].score = (L[q] != L[q]) ? INFINITY : L[q];\n            s[q].index = q;"),
    ("topk_descending", "swiftprune_oracle.c", "if (x->score < y->score) return -1;\n    if (x->score > y->score) return 1;",
     "if (x->score < y->score) return 1;\n    if (x->score > y->score) return -1;"),
    ("topk_tie_break_reversed", "swiftprune_oracle.c", "return (x->index > y->index) - (x->index < y->index);",
     "return (x->index < y->index) - (x->index > y->index);"),
    ("topk_off_by_one", "swiftprune_oracle.c", "for (int64_t j = k; j < in; ++j) {", "for (int64_t j = k + 1; j < in; ++j) {"),
    ("compact_wrong_field_width", "swiftprune_oracle.c", "return m_group == 4 ? 2 : 4;", "return m_group == 4 ? 2 : 2;"),
    ("compact_takes_pruned", "swiftprune_oracle.c",
     "if (!((keep_mask[r * words + (q >> 5)] >> (q & 31)) & 1u)) continue;\n                int64_t f",
     "if (((keep_mask[r * words + (q >> 5)] >> (q & 31)) & 1u)) continue;\n                int64_t f"),
    ("expand_wrong_group", "swiftprune_oracle.c", "int64_t q = f / n_keep * m_group + pos;", "int64_t q = f / m_group * m_group + pos;"),
    ("apply_zeroes_kept", "swiftprune_oracle.c", "if (keep) continue;", "if (!keep) continue;"),
]


@pytest.fixture(scope="module")
def src_dir(orc):
    return os.path.dirname(os.path.abspath(orc.__file__))


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(orc, src_dir, tmp_path, mutant):
    name, fname, old, new = mutant
    for f in ("swiftprune_oracle.c", "ewma_body.inc"):
        shutil.copy(os.path.join(src_dir, f), tmp_path / f)
    text = (tmp_path / fname).read_text()
    assert text.count(old) >= 1, f"mutation site for {name} not found"
    (tmp_path / fname).write_text(text.replace(old, new))
    so = str(tmp_path / f"liboracle_{name}.so")
    subprocess.run(["gcc", *[f for f in orc.CFLAGS if f not in ("-Wall", "-Wextra")],
                    str(tmp_path / "swiftprune_oracle.c"), "-o", so, "-lm"], check=True)
    # The pins run in a child process: a planted mistake may write out of bounds (a wider meta field,
    # a wrong group index), and that must not reach the heap of the test runner.  A child that dies on a
    # signal has caught nothing: the pin it died in is skipped and the rest run in a fresh child, and
    # only a failed assertion of some pin counts.
    child = (
        "import sys\n"
        f"sys.path[:0] = [{ROOT!r}, {TESTS!r}]\n"
        "import oracle, pins\n"
        f"L = oracle.lib({so!r})\n"
        "skip = set(sys.argv[1:])\n"
        "for pin in pins.ALL_PINS:\n"
        "    if pin.__name__ in skip:\n"
        "        continue\n"
        "    print('RUN ' + pin.__name__, flush=True)\n"
        "    try:\n"
        "        pin(oracle, L)\n"
        "    except AssertionError:\n"
        "        print('CAUGHT ' + pin.__name__, flush=True)\n"
        "    print('DONE ' + pin.__name__, flush=True)\n")
    caught, done, died_in = [], [], []
    for _ in range(len(pins_mod.ALL_PINS) + 1):
        res = subprocess.run([sys.executable, "-c", child, *done], capture_output=True, text=True, timeout=300)
        lines = res.stdout.splitlines()
        caught += [ln[len("CAUGHT "):] for ln in lines if ln.startswith("CAUGHT ")]
        done += [ln[len("DONE "):] for ln in lines if ln.startswith("DONE ")]
        if res.returncode == 0:
            break
        assert res.returncode < 0 or res.returncode == 134, res.stderr[-2000:]   # anything else is a bug of the test
        running = [ln[len("RUN "):] for ln in lines if ln.startswith("RUN ")][-1]
        died_in.append(running)
        done.append(running)
    if died_in:
        print(f"{name}: the planted mistake also corrupts memory (child died in {', '.join(died_in)}); not counted")
    assert caught, f"no pin fails an assertion on the planted mistake '{name}'"
    print(f"{name}: caught by {', '.join(caught)}")
