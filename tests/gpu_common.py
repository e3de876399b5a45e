"""Helpers shared by the GPU parity tests: build both sides from the same seeded inputs."""
import numpy as np
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import binding, synth


def make_pair(shape, seed=1, gains="random", std=0.02, max_anchors=0, lm_scale=None, **gpu_kw):
    w = synth.make_weights(shape, seed=seed, gains=gains, std=std)
    if lm_scale is not None:
        w["lm_head"] = (w["lm_head"].float() * lm_scale).to(w["lm_head"].dtype)
    oracle = O.OracleModel(shape, w)
    gpu = binding.KnnSsd(shape, w, max_anchors=max_anchors, **gpu_kw)
    return w, oracle, gpu


# Largest logit error seen so far per shape name, relative to the row's largest logit (bf16 path) or absolute (fp32
# path). The session summary prints the table (conftest.py), so every GPU run records what the kernels deliver
# next to the bound the tests enforce.
ACHIEVED = {}

# The stated tolerances (outer bounds): fp32 path max abs diff <= 1e-3; bf16 path max diff <= 5e-2 of the row's largest
# logit. What the kernels deliver is far less; the tests enforce ten times the largest error measured on an MI355X per
# shape (below; the bf16 figures come from cache entries that land on neighbouring bf16 values in fp32 and fp64 and grow
# with depth), never more than the stated tolerance.
FP32_ABS_BOUND = 1e-3
BF16_REL_BOUND = 5e-2
MEASURED = {
    # fp32 weights and cache: absolute
    "tiny": 1.6e-6, "fp32_gqa": 1.1e-6,
    # bf16: relative to the row's largest logit
    "mixed": 6.5e-7, "bf16_mha": 3.4e-5, "bf16_gqa": 1.4e-4, "bf16_mfma": 2.9e-4, "llama7b_w3": 4.1e-4,
    "long_ctx": 4.5e-5, "long_k": 3.1e-4, "narrow": 1.8e-5, "tiles356": 6.8e-5, "va_gqa": 5.4e-4, "va_mha": 1.6e-4,
    "llama13b": 4.2e-3, "llama13b_w2": 3.3e-3, "llama7b_w2": 1.1e-3, "qwen14b_w1": 2.4e-4, "qwen_w4": 1.2e-3,
    "llama7b": 5.1e-3, "qwen14b": 5.9e-3,      # full depth (32 and 48 blocks)
}
DEFAULT_MEASURED = {"fp32": 2e-6, "bf16": 5e-4}


def bound_for(shape):
    fp32 = shape.weight_dtype == "fp32" and shape.kv_dtype == "fp32"
    m = MEASURED.get(shape.name, DEFAULT_MEASURED["fp32" if fp32 else "bf16"])
    return min(FP32_ABS_BOUND if fp32 else BF16_REL_BOUND, 10.0 * m)


def logits_close(got, want, shape):
    """Max abs diff (fp32 path) or max diff relative to the row's largest logit magnitude (bf16 path) against
    bound_for(shape). Returns (ok, max abs diff)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want).max()
    if not (shape.weight_dtype == "fp32" and shape.kv_dtype == "fp32"):
        val = err / np.abs(want).max()
    else:
        val = err
    ACHIEVED[shape.name] = max(ACHIEVED.get(shape.name, 0.0), float(val))
    return val <= bound_for(shape), err
