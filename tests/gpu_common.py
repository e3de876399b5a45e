"""Helpers shared by the GPU parity tests: build both sides from the same seeded inputs."""
import numpy as np
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import binding, synth


def make_pair(shape, seed=1, gains="random", std=0.02, max_anchors=0, lm_scale=None):
    w = synth.make_weights(shape, seed=seed, gains=gains, std=std)
    if lm_scale is not None:
        w["lm_head"] = (w["lm_head"].float() * lm_scale).to(w["lm_head"].dtype)
    oracle = O.OracleModel(shape, w)
    gpu = binding.KnnSsd(shape, w, max_anchors=max_anchors)
    return w, oracle, gpu


def logits_close(got, want, shape):
    """fp32 path: max abs diff <= 1e-3. bf16 path: max diff <= 5e-2 relative to the row's
    largest logit magnitude."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want).max()
    if shape.weight_dtype == "fp32" and shape.kv_dtype == "fp32":
        return err <= 1e-3, err
    return err <= 5e-2 * np.abs(want).max(), err
