"""The pins must notice a mistake planted in the oracle (CPU only).

Each case builds a copy of oracle/forward.c with one plausible slip (a wrong sign, a dropped
scale, an off-by-one, a swapped operand, a wrong index) and runs the forward-pass pins against
it in a subprocess; at least one pin has to fail. The unmodified source must pass.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "forward.c")

MUTATIONS = {
    "rope_sign": ("v[i] = a * c - b * s;", "v[i] = a * c + b * s;"),
    "rope_pairing": ("double a = v[i], b = v[i + half];", "double a = v[i], b = v[(i + 1) % head_dim];"),
    "rope_frequency": ("pow(base, -2.0 * (double)i / (double)head_dim)", "pow(base, -(double)i / (double)head_dim)"),
    "score_scale": ("const double scale = 1.0 / sqrt((double)hd);", "const double scale = 1.0 / (double)hd;"),
    "causal_off_by_one": ("int len = start + r + 1;", "int len = start + r + (r > 0 ? 0 : 1);"),
    "silu": ("u[i] = (a / (1.0 + exp(-a))) * u[i];", "u[i] = (1.0 / (1.0 + exp(-a))) * u[i];"),
    "gate_up_swapped": ("matmul_rows(m->wg[b], c->weight_dtype, F, d, nrm, n, g);\n            matmul_rows(m->wu[b], c->weight_dtype, F, d, nrm, n, u);",
                        "matmul_rows(m->wu[b], c->weight_dtype, F, d, nrm, n, g);\n            matmul_rows(m->wg[b], c->weight_dtype, F, d, nrm, n, u);"),
    "gqa_head_mapping": ("int kvh = hh / group;", "int kvh = hh % Hkv;"),
    "rms_mean": ("double r = 1.0 / sqrt(ss / (double)d + eps);", "double r = 1.0 / sqrt(ss + eps);"),
    "rms_gain_dropped": ("out[i] = x[i] * r * (double)gain[i];", "out[i] = x[i] * r;"),
    "mask_index": ("if (!(mask && mask[2 * b + 1])) {", "if (!(mask && mask[2 * b])) {"),
    "residual_dropped": ("for (size_t i = 0; i < (size_t)n * d; ++i) h[i] += proj[i];\n        }\n        if (!(mask && mask[2 * b + 1])) {",
                         "for (size_t i = 0; i < (size_t)n * d; ++i) h[i] = proj[i];\n        }\n        if (!(mask && mask[2 * b + 1])) {"),
    "kv_rounding_truncates": ("u += 0x7fffu + lsb;", "u += 0u * lsb;"),
    "value_uses_keys": ("const float *vt = vc + (size_t)t * kvd + kvh * hd;", "const float *vt = kc + (size_t)t * kvd + kvh * hd;"),
}


def _run_pins(tmp_path, src_path, tag):
    env = dict(os.environ)
    env["KNNSSD_ORACLE_SRC"] = str(src_path)
    env["KNNSSD_ORACLE_LIB"] = str(tmp_path / f"liborc_{tag}.so")
    env["OMP_NUM_THREADS"] = "2"
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", "test_oracle_forward_pins.py")],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_unmodified_source_passes(tmp_path):
    r = _run_pins(tmp_path, SRC, "clean")
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_planted_mistake(tmp_path, name):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor for {name} not found exactly once"
    mutated = tmp_path / f"forward_{name}.c"
    mutated.write_text(text.replace(old, new))
    r = _run_pins(tmp_path, mutated, name)
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert "failed" in r.stdout
