"""The pins have teeth: a plausible mistake planted in a copy of the oracle's C source
(a dropped term, a wrong sign or index, a transposed operand) must fail at least one pin.
Everything here runs on the CPU; the real oracle is never modified."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTANTS = {
    "eps_dropped": [("ss / (double)d + eps", "ss / (double)d")],
    "eps_outside_root": [("1.0 / sqrt(ss / (double)d + eps)", "1.0 / (sqrt(ss / (double)d) + eps)")],
    "mean_over_d_minus_1": [("ss / (double)d", "ss / (double)(d - 1)")],
    "W1_transposed": [("(double)W1[i * b + j]", "(double)W1[j * d + i]")],
    "gain_dropped": [("norm[i] = widen(hidden, dtype, off + i) * r * g;", "norm[i] = widen(hidden, dtype, off + i) * r;"),
                     ("out[t * d + i] = widen(hidden, dtype, t * row_stride + i) * r * g;",
                      "out[t * d + i] = widen(hidden, dtype, t * row_stride + i) * r;")],
    "silu_is_identity": [("static double silu(double x) { return x * sigmoid(x); }",
                          "static double silu(double x) { return x; }")],
    "silu_is_sigmoid": [("static double silu(double x) { return x * sigmoid(x); }",
                         "static double silu(double x) { return sigmoid(x); }")],
    "threshold_not_strict": [("return z > log(", "return z >= log(")],
    "b1_dropped": [("act[j] = b1 ? (double)b1[j] : 0.0;", "act[j] = 0.0;")],
    "b2_dropped": [("double z = b2;", "double z = 0.0;")],
    "w2_dropped": [("z += (double)w2[j] * silu(act[j]);", "z += silu(act[j]);")],
    "latest_instead_of_earliest": [("if (f && !found && layer_ids[c] >= min_layer)", "if (f && layer_ids[c] >= min_layer)"),
                                   ("exit_layer[t] = layer_ids[c];\n                break;", "exit_layer[t] = layer_ids[c];")],
    "k_min_ignored": [("if (f && !found && layer_ids[c] >= min_layer)", "if (f && !found)"),
                      ("if (layer_ids[c] < min_layer) continue;", "")],
    "sigmoid_sign": [("if (x >= 0.0) return 1.0 / (1.0 + exp(-x));", "if (x >= 0.0) return 1.0 / (1.0 + exp(x));")],
    "theta_off_fires": [("if (theta >= 1.0) return 0;", "if (theta >= 1.0) return 1;")],
    "bf16_shift": [("(uint32_t)h << 16", "(uint32_t)h << 15")],
    "f16_bias": [("ex - 15)", "ex - 16)")],
    "f16_subnormal": [("ldexp((double)fr, -24)", "ldexp((double)fr, -25)")],
    "compact_strict_comparison": [("if (exit_layer[t] <= layer) exit_idx[ne++] = (int32_t)t;", "if (exit_layer[t] < layer) exit_idx[ne++] = (int32_t)t;")],
    "cosine_not_normalised_by_final": [("double s = dot / (sqrt(nk) * sqrt(nl));", "double s = dot / (sqrt(nk) * sqrt(nk));")],
    "cosine_label_not_strict": [("label[c * T + t] = (uint8_t)(s > tau);", "label[c * T + t] = (uint8_t)(s >= tau);")],
    "cosine_dot_of_squares": [("dot += x * y;", "dot += x * x;")],
    "batch_exit_any_instead_of_all": [("n == T && T > 0", "n > 0 && T > 0")],
    "batch_exit_ignores_k_min": [("if (!decided && layer_ids[c] >= min_layer && n == T && T > 0)", "if (!decided && n == T && T > 0)")],
    "projection_takes_first_checkpoint": [("off = c * ckpt_stride + t * row_stride;\n                break;", "off = t * row_stride;\n                break;")],
    "projection_drops_gain": [("double y = widen(src, dtype, off + i) * r * g;", "double y = widen(src, dtype, off + i) * r;")],
    "projection_truncates": [("double r = ldexp(rint(ldexp(m, bits)), e - bits);", "double r = ldexp(trunc(ldexp(m, bits)), e - bits);")],
    "projection_ignores_final_state": [("if (!src && final_hidden) {", "if (0) {")],
    "bf16_rounds_to_9_bits": [("default:         return round_to_format(v, 8, -125, 128);", "default:         return round_to_format(v, 9, -125, 128);")],
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name, tmp_path):
    parent = tmp_path / "mut"
    shutil.copytree(os.path.join(ROOT, "oracle"), parent / "oracle",
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    src = parent / "oracle" / "tide_oracle.c"
    text = src.read_text()
    for old, new in MUTANTS[name]:
        assert old in text, f"mutation site for {name!r} not found: {old!r}"
        text = text.replace(old, new)
    src.write_text(text)
    env = dict(os.environ, TIDE_ORACLE_PARENT=str(parent), PYTHONDONTWRITEBYTECODE="1")
    run = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 1, f"mutant {name!r} survived the pins:\n{run.stdout[-2000:]}\n{run.stderr[-2000:]}"
    assert "failed" in run.stdout


def test_unmodified_copy_passes_through_the_same_mechanism(tmp_path):
    """Control: the copy-and-redirect machinery itself does not cause the failures."""
    parent = tmp_path / "ctl"
    shutil.copytree(os.path.join(ROOT, "oracle"), parent / "oracle",
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    env = dict(os.environ, TIDE_ORACLE_PARENT=str(parent), PYTHONDONTWRITEBYTECODE="1")
    run = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]
    assert (parent / "oracle" / "libtide_oracle.so").exists()
