"""The pins of ``test_oracle_pins.py`` catch planted mistakes.

Each case below changes one expression of a COPY of ``oracle/dlrt_oracle.c`` (a transposed operand, a wrong
sign, index, stride, rounding mode or bound), rebuilds the copy in a scratch directory and runs the pin tests
against it in a child process: every such copy must fail at least one pin, and the unchanged copy must pass.
Everything here runs on the CPU; the oracle in the tree is never touched.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PACKAGE = "paper_2207_08820_amd"

PACK_PATTERN = """if (enc == 2)
                pattern = v > 0 ? {one}u : {zero}u;
            else
                pattern = (unsigned)v & ((1u << bits) - 1u);
            for (int p = 0; p < bits; ++p) {{
                if ((pattern >> p) & 1u)
                    dst[(r * bits"""

# (name, text in the oracle's source, what replaces it)
MUTANTS = [
    ("unchanged", "", ""),
    ("gemm_w_transposed", "(int32_t)w[n * K + k]", "(int32_t)w[(k * N + n) % (N * K)]"),
    ("gemm_k_reversed_on_one_operand", "(int32_t)a[m * K + k] *", "(int32_t)a[m * K + (K - 1 - k)] *"),
    ("gemm_output_transposed", "c[m * N + n] = s;", "c[(n * M + m) % (M * N)] = s;"),
    ("conv_padding_sign", "oh * stride_h - pad_h + kh", "oh * stride_h + pad_h - kh"),
    ("conv_taps_swapped_in_weights", "(((size_t)co * KH + kh) * KW + kw) * Ci", "(((size_t)co * KH + kw % KH) * KW + kh % KW) * Ci"),
    ("conv_stride_w_taken_from_h", "ow * stride_w - pad_w + kw", "ow * stride_h - pad_w + kw"),
    ("conv_pad_w_taken_from_h", "ow * stride_w - pad_w + kw", "ow * stride_w - pad_h + kw"),
    ("conv_left_border_not_skipped", "if (iw < 0 || iw >= W) continue;", "if (iw >= W) continue; if (iw < 0 && (ow > 0 || n > 0 || oh > 0)) continue;"),
    ("conv_rows_replicated_at_the_border", "const int ih = oh * stride_h - pad_h + kh;\n                        if (ih < 0 || ih >= H) continue;",
     "int ih = oh * stride_h - pad_h + kh;\n                        if (ih < 0) ih = 0;\n                        if (ih >= H) ih = H - 1;"),
    ("epilogue_multiply_then_add", "fmaf((float)acc[r * C + c], scale[c], bias ? bias[c] : 0.0f)",
     "((float)((float)acc[r * C + c] * scale[c]) + (bias ? bias[c] : 0.0f))"),
    ("epilogue_ties_away_from_zero", "fminf(fmaxf(nearbyintf(y), 0.0f), qmax)", "fminf(fmaxf(roundf(y), 0.0f), qmax)"),
    ("epilogue_upper_clamp_off_by_one", "(float)((1 << qbits) - 1)", "(float)(1 << qbits)"),
    ("epilogue_no_lower_clamp", "fminf(fmaxf(nearbyintf(y), 0.0f), qmax)", "fminf(fabsf(nearbyintf(y)), qmax)"),
    ("epilogue_bias_dropped", "bias ? bias[c] : 0.0f", "0.0f"),
    ("epilogue_scale_indexed_by_row", "scale[c], bias", "scale[r % C], bias"),
    ("quantize_truncates", "(int8_t)nearbyintf(v)", "(int8_t)v"),
    ("quantize_multiplies_by_scale", "float v = x[r * K + k] / s", "float v = x[r * K + k] * s"),
    ("quantize_no_upper_clip", "fminf(fmaxf(v, lo), hi)", "fmaxf(v, lo)"),
    ("quantize_scale_of_row_0", "scale[per_row ? r : 0];\n        for (int64_t k = 0; k < K; ++k) {", "scale[0];\n        for (int64_t k = 0; k < K; ++k) {"),
    ("quantize_bipolar_zero_is_minus_one", "/ s >= 0.0f) ? 1 : -1", "/ s > 0.0f) ? 1 : -1"),
    ("quantize_bipolar_sign_flipped", "/ s >= 0.0f) ? 1 : -1", "/ s >= 0.0f) ? -1 : 1"),
    ("quantize_bipolar_rounds_small_values_to_minus_one", "/ s >= 0.0f) ? 1 : -1", "/ s > 0.5f) ? 1 : -1"),
    ("pack_msb_first", "|= 1u << (k % 32);", "|= 1u << (31 - k % 32);"),
    ("pack_bipolar_inverted", PACK_PATTERN.format(one=1, zero=0), PACK_PATTERN.format(one=0, zero=1)),
    ("pack_planes_reversed", "dst[(r * bits + p) * Kw + k / 32]", "dst[(r * bits + (bits - 1 - p)) * Kw + k / 32]"),
    ("pack_weights_taps_not_padded", "((size_t)p * KH * KW + t) * Cw + ci / 32]\n                            |= 1u << (ci % 32);",
     "((size_t)p * KH * KW) * Cw + (t * Ci + ci) / 32]\n                            |= 1u << ((t * Ci + ci) % 32);"),
    ("pack_weights_tap_major", "dst[co * per_co + ((size_t)p * KH * KW + t) * Cw + ci / 32]", "dst[co * per_co + ((size_t)t * bits + p) * Cw + ci / 32]"),
]


def run_pins_on_copy(base, name, old, new):
    """Copy what the pin tests import into base/name, apply the change, run the pins there; returns (rc, tail)."""
    dst = os.path.join(base, name)
    for d in ("oracle", "tests"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(dst, d), ignore=shutil.ignore_patterns("__pycache__", "*.so", "test_oracle_mutants.py"))
    os.makedirs(os.path.join(dst, PACKAGE))
    for f in os.listdir(os.path.join(ROOT, PACKAGE)):
        if f.endswith(".py"):
            shutil.copy(os.path.join(ROOT, PACKAGE, f), os.path.join(dst, PACKAGE, f))
    path = os.path.join(dst, "oracle", "dlrt_oracle.c")
    src = open(path).read()
    if old:
        assert src.count(old) == 1, f"{name}: the text to change occurs {src.count(old)} times in the oracle"
        open(path, "w").write(src.replace(old, new))
    env = dict(os.environ, OMP_NUM_THREADS="1", MKL_NUM_THREADS="1")  # several children run side by side
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=dst, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode, (r.stdout + r.stderr)[-1500:]


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    base = str(tmp_path_factory.mktemp("oracle_mutants"))
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        futures = {name: pool.submit(run_pins_on_copy, base, name, old, new) for name, old, new in MUTANTS}
        return {name: f.result() for name, f in futures.items()}


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_pins_catch_the_planted_mistake(outcomes, name):
    rc, tail = outcomes[name]
    if name == "unchanged":
        assert rc == 0, tail
    else:
        assert rc != 0, f"no pin failed for the oracle with {name}"
        last = tail.splitlines()[-1]  # a pin's assertion failed, not the build of the copy or its collection
        assert "failed" in last and "error" not in last, tail
