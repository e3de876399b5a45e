"""Seeded synthetic inputs for the KNN-SSD decode path.

This module only draws random numbers and lays them out as tensors: model
weights, prompts, anchor tables, skip masks and query vectors. It contains none
of the method's arithmetic (no forward pass, no similarity search, no accept
rule), so both the CPU oracle and the HIP path can consume what it produces as
plain data without sharing any computation.

Every tensor is materialised once (on the device asked for) and the same bytes
are then handed to both sides. Seeds are derived from one base seed plus a
fixed tensor id, so a (config, seed, device-kind) triple always gives the same
bytes.

The shapes stand in for the paper's LLaMA-2 / Qwen-2.5 checkpoints and its five
task datasets (Sec. 5 "Experimental Setup"): only shapes carry over, the values
are random.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import torch

BASE_SEED = 20250516


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder shape. ``n_blocks`` decoder blocks = 2*n_blocks skippable sublayers
    (the paper's L counts attention and MLP sublayers separately, Sec. 3.1)."""
    name: str
    n_blocks: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    max_seq: int
    weight_dtype: str  # "fp32" | "bf16"
    kv_dtype: str      # "fp32" | "bf16"
    rope_base: float = 10000.0
    rms_eps: float = 1e-5

    @property
    def n_sublayers(self) -> int:
        return 2 * self.n_blocks

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration: model shape plus generation recipe."""
    shape: ModelShape
    prompt_len: int
    max_new: int
    max_draft: int
    conf_threshold: float     # <= 0 disables the confidence stop
    n_anchors: int
    n_domains: int
    skipped_blocks: int       # whole blocks skipped per domain mask
    anchor_sigma: float       # spread of anchors round their domain centre
    n_samples: int = 1


def _shape(name, nb, d, h, hkv, hd, f, v, max_seq, dt) -> ModelShape:
    return ModelShape(name, nb, d, h, hkv, hd, f, v, max_seq, dt, dt)


def workload(name: str) -> Workload:
    """The five configurations of the benchmark contract, by name."""
    if name == "tiny":      # fp32 correctness configuration
        s = _shape("tiny", 4, 256, 4, 4, 64, 688, 1024, 32 + 32 + 8, "fp32")
        return Workload(s, 32, 32, 4, 0.0, 8, 8, 2, 1.0)
    if name == "llama7b":
        s = _shape("llama7b", 32, 4096, 32, 32, 128, 11008, 32000, 512 + 256 + 16, "bf16")
        return Workload(s, 512, 256, 8, 0.6, 1000, 5, 16, 0.1)
    if name == "llama13b":
        s = _shape("llama13b", 40, 5120, 40, 40, 128, 13824, 32000, 1024 + 512 + 16, "bf16")
        return Workload(s, 1024, 512, 8, 0.6, 1000, 5, 20, 0.1)
    if name == "qwen14b":
        s = _shape("qwen14b", 48, 5120, 40, 8, 128, 13824, 152064, 1024 + 512 + 16, "bf16")
        return Workload(s, 1024, 512, 8, 0.0, 1000, 5, 24, 0.1)
    if name == "llama13b_stream":
        s = _shape("llama13b_stream", 40, 5120, 40, 40, 128, 13824, 32000, 4096 + 256 + 16, "bf16")
        return Workload(s, 4096, 256, 8, 0.6, 5000, 5, 20, 0.1, n_samples=50)
    raise KeyError(name)


def small_shape(name: str, **kw) -> ModelShape:
    """Small shapes for parity tests (several tiles, ragged tails)."""
    base = dict(name=name, n_blocks=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64,
                d_ffn=688, vocab=1000, max_seq=96, weight_dtype="bf16", kv_dtype="bf16")
    base.update(kw)
    return ModelShape(**base)


_TORCH_DT = {"fp32": torch.float32, "bf16": torch.bfloat16}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, std, seed, device, dtype) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 on `device`, then rounded (nearest-even) to dtype."""
    g = _gen(seed, device)
    n = 1
    for s in shape:
        n *= s
    # draw in bounded chunks so a 0.8G-element matrix never needs a second fp32 copy
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    chunk = 1 << 26
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        flat[lo:hi] = (torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32) * std).to(dtype)
    return out


def _s64(v: int) -> int:
    """A 64-bit pattern as the signed integer torch's int64 holds."""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """The finaliser of the SplitMix64 generator on int64 tensors (wrapping products; the logical right shifts are
    arithmetic shifts with the sign bits masked off). Integer work only: the same bits on every device."""
    x = (x ^ ((x >> 30) & ((1 << 34) - 1))) * _s64(0xBF58476D1CE4E5B9)
    x = (x ^ ((x >> 27) & ((1 << 37) - 1))) * _s64(0x94D049BB133111EB)
    return x ^ ((x >> 31) & ((1 << 33) - 1))


def _counter_normal(shape, std, seed, device, dtype) -> torch.Tensor:
    """Approximately N(0, std^2), the SAME bytes whichever device draws them (torch's own generators differ between
    host and GPU, so a tensor that both a host-side and a device-side consumer must regenerate independently comes
    from here). Element i is a function of (seed, i) alone: two 64-bit hashes give eight 16-bit uniforms, whose sum
    (Irwin-Hall, n = 8: Gaussian to within a kurtosis of -0.15, support +-4.9 sigma) is centred and scaled with one
    fp32 multiplication, then rounded (nearest-even) to dtype. Every step is integer arithmetic or a single IEEE
    operation, so host and device agree bit for bit."""
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    key = _s64((int(seed) * 0x9E3779B97F4A7C15) ^ 0xD1B54A32D192ED03)
    scale = float(std) / (8.0 * (65536.0 ** 2 - 1.0) / 12.0) ** 0.5
    chunk = 1 << 25
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        i = torch.arange(lo, hi, dtype=torch.int64, device=device)
        total = torch.zeros(hi - lo, dtype=torch.int64, device=device)
        for stream in (0, 1):
            h = _mix64((2 * i + stream) * _s64(0x9E3779B97F4A7C15) + key)
            for f in range(4):
                total += (h >> (16 * f)) & 0xFFFF
        flat[lo:hi] = ((total - 4 * 65535).to(torch.float32) * scale).to(dtype)
    return out


def make_weights(shape: ModelShape, seed: int = BASE_SEED, device="cpu",
                 gains: str = "ones", std: float = 0.02, counter: bool = False) -> Dict:
    """Random-init decoder weights, all matrices row-major [out_features][in_features].

    gains="ones" gives unit RMSNorm gains (the benchmark recipe); gains="random"
    draws them from U(0.5, 1.5) so tests notice a missing or misplaced gain.
    Norm gains are always fp32. counter=True draws the matrices from the counter-based
    generator (_counter_normal): the same bytes on the host and on the GPU.
    """
    dt = _TORCH_DT[shape.weight_dtype]
    d, f = shape.d_model, shape.d_ffn
    if counter:
        assert gains == "ones", "the device-independent recipe uses unit gains"
        _normal = _counter_normal       # noqa: F811 (same signature)
    else:
        _normal = globals()["_normal"]

    def gain(tid):
        if gains == "ones":
            return torch.ones(d, dtype=torch.float32, device=device)
        g = _gen(seed * 1000003 + 500000 + tid, device)
        return (torch.rand(d, generator=g, device=device, dtype=torch.float32) + 0.5)

    w = {
        "embed": _normal((shape.vocab, d), std, seed * 1000003 + 1, device, dt),
        "lm_head": _normal((shape.vocab, d), std, seed * 1000003 + 2, device, dt),
        "final_norm": gain(0),
        "blocks": [],
    }
    for b in range(shape.n_blocks):
        t = seed * 1000003 + 100 + 16 * b
        w["blocks"].append({
            "attn_norm": gain(1 + 2 * b),
            "wq": _normal((shape.q_dim, d), std, t + 0, device, dt),
            "wk": _normal((shape.kv_dim, d), std, t + 1, device, dt),
            "wv": _normal((shape.kv_dim, d), std, t + 2, device, dt),
            "wo": _normal((d, shape.q_dim), std, t + 3, device, dt),
            "mlp_norm": gain(2 + 2 * b),
            "wg": _normal((f, d), std, t + 4, device, dt),
            "wu": _normal((f, d), std, t + 5, device, dt),
            "wd": _normal((d, f), std, t + 6, device, dt),
        })
    return w


def weights_to(w: Dict, device, pin: bool = False) -> Dict:
    """Copy a weight dictionary to another device (same bytes)."""
    def mv(t):
        return t.to(device)
    out = {k: mv(v) for k, v in w.items() if k != "blocks"}
    out["blocks"] = [{k: mv(v) for k, v in blk.items()} for blk in w["blocks"]]
    return out


def make_prompt(vocab: int, length: int, seed: int = BASE_SEED + 1) -> torch.Tensor:
    """Token ids uniform on [0, vocab), int32, on the host."""
    g = _gen(seed, "cpu")
    return torch.randint(0, vocab, (length,), generator=g, dtype=torch.int64).to(torch.int32)


def make_block_masks(n_blocks: int, n_domains: int, skipped_blocks: int,
                     seed: int = BASE_SEED + 2) -> torch.Tensor:
    """One skip mask per domain, uint8 [n_domains][2*n_blocks].

    Entry 2b is the attention sublayer of block b, entry 2b+1 its MLP sublayer;
    1 = skip. Each mask skips `skipped_blocks` whole blocks chosen uniformly.
    """
    g = _gen(seed, "cpu")
    m = torch.zeros((n_domains, 2 * n_blocks), dtype=torch.uint8)
    for i in range(n_domains):
        perm = torch.randperm(n_blocks, generator=g)[:skipped_blocks]
        for b in perm.tolist():
            m[i, 2 * b] = 1
            m[i, 2 * b + 1] = 1
    return m


def make_sublayer_masks(n_blocks: int, n_domains: int, p_skip_attn: float, p_skip_mlp: float,
                        seed: int = BASE_SEED + 2) -> torch.Tensor:
    """Masks that skip attention and MLP sublayers independently (Appendix A's pattern)."""
    g = _gen(seed, "cpu")
    r = torch.rand((n_domains, n_blocks, 2), generator=g)
    m = torch.zeros((n_domains, n_blocks, 2), dtype=torch.uint8)
    m[:, :, 0] = (r[:, :, 0] < p_skip_attn).to(torch.uint8)
    m[:, :, 1] = (r[:, :, 1] < p_skip_mlp).to(torch.uint8)
    return m.reshape(n_domains, 2 * n_blocks).contiguous()


def make_anchors(dim: int, n_anchors: int, n_domains: int, sigma: float,
                 seed: int = BASE_SEED + 3, device="cpu", clustered: bool = True, counter: bool = False):
    """Anchor table (fp32 [N][D]), labels (int32 [N]) and domain centres (fp32 [n_domains][D]).

    clustered=True: centres ~ N(0, I); anchor n belongs to domain n % n_domains and
    is centre + sigma*N(0, I) (stored domain-interleaved so a scan cannot stop early).
    clustered=False: anchors ~ N(0, I) and label n = n % n_domains (the tiny config:
    eight unrelated anchors, eight labels).
    """
    if counter:     # the same bytes on the host and on the GPU (see _counter_normal)
        centres = _counter_normal((n_domains, dim), 1.0, seed * 7 + 1, device, torch.float32)
        noise = _counter_normal((n_anchors, dim), 1.0, seed * 7 + 2, device, torch.float32)
    else:
        g = _gen(seed, device)
        centres = torch.randn((n_domains, dim), generator=g, device=device, dtype=torch.float32)
        noise = torch.randn((n_anchors, dim), generator=g, device=device, dtype=torch.float32)
    labels = (torch.arange(n_anchors, device=device) % n_domains).to(torch.int32)
    if clustered:
        anchors = centres[labels.long()] + sigma * noise
    else:
        anchors = noise
    return anchors.contiguous(), labels.contiguous(), centres


def make_domain_query(centres: torch.Tensor, domain: int, sigma: float, seed: int) -> torch.Tensor:
    """A query near one domain's centre: centre + sigma*N(0, I) (the domain-shift stream)."""
    g = _gen(seed, centres.device)
    return (centres[domain] + sigma * torch.randn(centres.shape[1], generator=g,
                                                  device=centres.device, dtype=torch.float32)).contiguous()


def mix_ratio_stream(n_domains: int, n_samples: int, r: float, seed: int) -> torch.Tensor:
    """Uniform draws that drive a domain stream: float64 [n_samples][2] on [0, 1).

    Only the random numbers live here: row i is the pair (u_switch, u_pick) for sample i.
    How the pair becomes the next domain (Sec. 4.2, Eq. 8) is the method's business and is
    implemented separately by the oracle and by the library.
    """
    g = _gen(seed, "cpu")
    return torch.rand((n_samples, 2), generator=g, dtype=torch.float64)
