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

# What the kernels deliver, measured: fp32 path 1e-6 absolute; bf16 path at most 5e-3 of the row's largest logit (the
# bf16 cache roundings that fall on different sides in fp32 and fp64, see the design notes). The tests enforce 10x
# the measured figure, with the stated tolerance (1e-3 absolute / 5e-2 relative) as the outer bound.
FP32_ABS_BOUND = 1e-3
BF16_REL_BOUND = 5e-2
FP32_ABS_TIGHT = 1e-5
BF16_REL_TIGHT = 2.5e-2


def logits_close(got, want, shape):
    """fp32 path: max abs diff <= 1e-3 (stated tolerance), and <= 1e-5 (10x what the kernels deliver).
    bf16 path: max diff relative to the row's largest logit magnitude <= 5e-2 (stated), and <= 2.5e-2."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want).max()
    if shape.weight_dtype == "fp32" and shape.kv_dtype == "fp32":
        ACHIEVED[shape.name] = max(ACHIEVED.get(shape.name, 0.0), float(err))
        return err <= min(FP32_ABS_BOUND, FP32_ABS_TIGHT), err
    rel = err / np.abs(want).max()
    ACHIEVED[shape.name] = max(ACHIEVED.get(shape.name, 0.0), float(rel))
    return rel <= min(BF16_REL_BOUND, BF16_REL_TIGHT), err
