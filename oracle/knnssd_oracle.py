"""CPU oracle for the KNN-SSD decode path (TEST INFRASTRUCTURE ONLY).

Slow, plain and meant to be checked against the paper by eye. Only tests,
the smoke check and the benchmark's CPU-baseline leg may import this module;
the product path never does. It shares no code with the HIP sources.

Pieces, each following the passage named:
  * knn_select        Sec. 4.2, Eq. 4-6: cosine-similarity nearest anchor -> domain -> mask.
  * OracleModel       Sec. 3.1: decoder forward with skip mask z (C code in forward.c).
  * greedy_ar         the "Vanilla" autoregressive baseline of Table 1.
  * ssd_generate      Sec. 4.2 (Eq. 7 and the verification paragraph): draft with M(z),
                      verify with M in one forward pass, accept or re-draft.
  * expected_speedup  Sec. 5.1 Eq. 9 / App. C.2 Eq. 10;  cost_coefficient App. C.2 Eq. 11.
  * next_domain       Sec. 4.2 Eq. 8, the mix-ratio stream.

Readings where the paper is silent (all listed in the design notes of the repo):
ties go to the lowest index; K = 1 neighbour; the draft stops after max_draft
tokens or after the first drafted token whose top-1 probability is below the
threshold (that token is kept as a draft); verification takes the last emitted
token plus the k drafts as k+1 rows and emits the matching prefix plus one token
of its own; the verification pass overwrites the cache entries the draft wrote.
"""
from __future__ import annotations

import ctypes
import dataclasses
from typing import List, Optional, Sequence

import numpy as np

from .build import build_oracle

_DT = {"fp32": 0, "bf16": 1}


class _Cfg(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32),
                ("vocab", ctypes.c_int32), ("max_seq", ctypes.c_int32),
                ("rope_base", ctypes.c_double), ("rms_eps", ctypes.c_double),
                ("weight_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        lib.orc_create.restype = ctypes.c_void_p
        lib.orc_create.argtypes = [ctypes.POINTER(_Cfg)] + [ctypes.c_void_p] * 12
        lib.orc_destroy.argtypes = [ctypes.c_void_p]
        lib.orc_forward.restype = ctypes.c_int
        lib.orc_forward.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.orc_read_kv.restype = ctypes.c_int
        lib.orc_read_kv.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def _host_array(t, dtype_name):
    """A torch CPU tensor (fp32 or bf16) or numpy array -> contiguous numpy array of raw storage."""
    if isinstance(t, np.ndarray):
        return np.ascontiguousarray(t)
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


class OracleModel:
    """Layer-masked decoder forward with a KV cache (Sec. 3.1; the C code does the arithmetic).

    `shape` needs the attributes n_blocks, d_model, n_heads, n_kv_heads, head_dim, d_ffn,
    vocab, max_seq, rope_base, rms_eps, weight_dtype, kv_dtype. `weights` is the dictionary
    produced by the input generator: embed, lm_head, final_norm and per block attn_norm,
    wq, wk, wv, wo, mlp_norm, wg, wu, wd (host tensors; bf16 weights as bit patterns).
    """

    def __init__(self, shape, weights):
        lib = _load()
        self.shape = shape
        self._keep = []

        def arr(t):
            a = _host_array(t, shape.weight_dtype)
            self._keep.append(a)
            return a.ctypes.data

        nb = shape.n_blocks
        cfg = _Cfg(nb, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                   shape.vocab, shape.max_seq, float(shape.rope_base), float(shape.rms_eps),
                   _DT[shape.weight_dtype], _DT[shape.kv_dtype])

        def ptr_array(key):
            pa = (ctypes.c_void_p * max(nb, 1))()
            for b in range(nb):
                pa[b] = arr(weights["blocks"][b][key])
            self._keep.append(pa)
            return ctypes.cast(pa, ctypes.c_void_p)

        self._h = lib.orc_create(ctypes.byref(cfg), arr(weights["embed"]), arr(weights["lm_head"]),
                                 arr(weights["final_norm"]), ptr_array("attn_norm"), ptr_array("wq"),
                                 ptr_array("wk"), ptr_array("wv"), ptr_array("wo"), ptr_array("mlp_norm"),
                                 ptr_array("wg"), ptr_array("wu"), ptr_array("wd"))
        self._lib = lib

    def __del__(self):
        try:
            if getattr(self, "_h", None):
                self._lib.orc_destroy(self._h)
                self._h = None
        except Exception:
            pass

    def forward(self, tokens: Sequence[int], start: int, mask=None, logits_from: int = 0,
                want_hidden: bool = False):
        """Rows tokens[r] at positions start+r through M(mask). Returns fp32 logits
        [n - logits_from, vocab] (and the final-normed hidden states [n, d] if asked)."""
        tok = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
        n = int(tok.shape[0])
        m = None
        if mask is not None:
            m = np.ascontiguousarray(np.asarray(mask, dtype=np.uint8))
            assert m.shape == (2 * self.shape.n_blocks,)
        logits = np.empty((max(n - logits_from, 0), self.shape.vocab), dtype=np.float32)
        hidden = np.empty((n, self.shape.d_model), dtype=np.float32) if want_hidden else None
        rc = self._lib.orc_forward(self._h, tok.ctypes.data, n, int(start),
                                   m.ctypes.data if m is not None else None, int(logits_from),
                                   logits.ctypes.data if logits.size else None,
                                   hidden.ctypes.data if hidden is not None else None)
        if rc != 0:
            raise ValueError("oracle forward: argument out of range")
        return (logits, hidden) if want_hidden else logits

    def read_kv(self, block: int, pos: int):
        kvd = self.shape.n_kv_heads * self.shape.head_dim
        k = np.empty(kvd, dtype=np.float32)
        v = np.empty(kvd, dtype=np.float32)
        rc = self._lib.orc_read_kv(self._h, block, pos, k.ctypes.data, v.ctypes.data)
        if rc != 0:
            raise ValueError("oracle read_kv: out of range")
        return k, v


# ----------------------------------------------------------------------------------------------
# token decisions on fp32 logits
# ----------------------------------------------------------------------------------------------

def argmax_lowest(x: np.ndarray) -> int:
    """Index of the maximum; the lowest index wins a tie."""
    return int(np.argmax(x))  # numpy returns the first occurrence of the maximum


def top1_prob(logits_row: np.ndarray) -> float:
    """Softmax probability of the arg-max token at temperature 1: 1 / sum_v exp(l_v - l_max)."""
    l = logits_row.astype(np.float64)
    return float(1.0 / np.exp(l - l.max()).sum())


def top2_margin(logits_row: np.ndarray) -> float:
    """Gap between the largest and second-largest logit (near-tie bookkeeping for parity tests)."""
    part = np.partition(logits_row.astype(np.float64), -2)
    return float(part[-1] - part[-2])


# ----------------------------------------------------------------------------------------------
# Sec. 4.2, Eq. 4-6: nearest anchor by cosine similarity -> domain -> skip mask
# ----------------------------------------------------------------------------------------------

def cosine_scores(query: np.ndarray, anchors: np.ndarray) -> np.ndarray:
    """cos(v, a_n) for every anchor, in double precision."""
    v = np.asarray(query, dtype=np.float64)
    a = np.asarray(anchors, dtype=np.float64)
    vn = np.sqrt((v * v).sum())
    an = np.sqrt((a * a).sum(axis=1))
    if not np.isfinite(vn) or vn == 0.0 or np.any(an == 0.0) or not np.all(np.isfinite(an)):
        raise ValueError("cosine similarity undefined: zero-norm or non-finite vector")
    return (a @ v) / (vn * an)


def knn_select(query, anchors, labels, masks):
    """(anchor index, domain, mask, scores): Eq. 4 arg-max over all anchors (lowest index on a
    tie, decided on fp32-rounded scores), Eq. 5 domain = the anchor's label, Eq. 6 mask = the
    domain's stored skip set."""
    s = cosine_scores(query, anchors)
    n_star = argmax_lowest(s.astype(np.float32))
    dom = int(np.asarray(labels)[n_star])
    return n_star, dom, np.asarray(masks, dtype=np.uint8)[dom].copy(), s


# ----------------------------------------------------------------------------------------------
# decoding loops
# ----------------------------------------------------------------------------------------------

def knn_topk_vote(query, anchors, labels, k: int):
    """The K nearest anchors by cosine similarity (Eq. 4 generalised from the arg-max to the K best; equal
    scores in index order) and the majority domain among them; a tie between domains goes to the tied domain
    whose best anchor ranks first. Exhaustive: every score is computed and the whole table is sorted."""
    scores = cosine_scores(np.asarray(query, dtype=np.float64), np.asarray(anchors, dtype=np.float64))
    s32 = scores.astype(np.float32)              # ties are decided on fp32-rounded scores, as in knn_select
    order = sorted(range(len(scores)), key=lambda n: (-s32[n], n))[:k]
    counts = {}
    for rank, n in enumerate(order):
        lab = int(labels[n])
        c, first = counts.get(lab, (0, rank))
        counts[lab] = (c + 1, first)
    domain = min(counts, key=lambda lab: (-counts[lab][0], counts[lab][1]))
    return order, [float(scores[n]) for n in order], domain


@dataclasses.dataclass
class GenStats:
    rounds: int = 0          # verification passes
    drafted: int = 0         # draft steps
    accepted: int = 0        # drafted tokens that verification kept
    emitted: int = 0         # tokens produced after the prompt (including the prefill's token)

    @property
    def mean_generated_length(self) -> float:
        """M of App. C.2: output tokens per forward pass of the target model."""
        return (self.emitted - 1) / self.rounds if self.rounds else 0.0

    @property
    def acceptance_rate(self) -> float:
        """alpha of App. C.2: accepted tokens / draft steps."""
        return self.accepted / self.drafted if self.drafted else 0.0


@dataclasses.dataclass
class Round:
    start: int                 # cache length when the round began
    drafts: List[int]
    draft_probs: List[float]
    targets: List[int]         # the full model's tokens for the k+1 rows
    n_accepted: int
    margins: List[float]       # top-1/top-2 logit gap of each verify row


def prefill(model: OracleModel, prompt: Sequence[int]):
    """Full model over the prompt: fills the cache, returns (first generated token, last hidden
    vector = final-normed hidden state of the last prompt token, its logits row)."""
    n = len(prompt)
    logits, hidden = model.forward(prompt, 0, None, logits_from=n - 1, want_hidden=True)
    return argmax_lowest(logits[0]), hidden[n - 1].copy(), logits[0]


def greedy_ar(model: OracleModel, prompt: Sequence[int], max_new: int, return_logits: bool = False):
    """Plain greedy autoregressive decoding with the full model: max_new tokens after the prompt."""
    tok, _, row = prefill(model, prompt)
    out, rows = [tok], [row]
    pos = len(prompt)
    while len(out) < max_new:
        row = model.forward([out[-1]], pos, None)[0]
        out.append(argmax_lowest(row))
        rows.append(row)
        pos += 1
    return (out, rows) if return_logits else out


def accept_length(drafts: Sequence[int], targets: Sequence[int]) -> int:
    """Number of leading drafts that equal the full model's own token at the same place."""
    j = 0
    while j < len(drafts) and drafts[j] == targets[j]:
        j += 1
    return j


def ssd_generate(model: OracleModel, prompt: Sequence[int], mask, max_new: int, max_draft: int,
                 conf_threshold: float = 0.0, first_token: Optional[int] = None):
    """Self-speculative decoding with skip mask `mask` (Sec. 4.2). Returns (tokens, stats, rounds).

    The first token comes from the prefill. Then, per round: draft up to max_draft tokens with
    M(mask) one at a time on the shared cache; verify x_last and the k drafts as k+1 rows of the
    full model in one pass; keep the longest prefix of drafts that matches, plus the full model's
    own next token; move the cache length to just behind the last kept token.
    `first_token`, when given, says the cache already holds the prompt's prefill.
    """
    tok = prefill(model, prompt)[0] if first_token is None else int(first_token)
    out = [tok]
    stats = GenStats(emitted=1)
    rounds: List[Round] = []
    cache_len = len(prompt)
    x_last = tok
    while len(out) < max_new:
        remaining = max_new - len(out)
        k_max = min(max_draft, remaining - 1)
        drafts, probs = [], []
        prev = x_last
        for i in range(k_max):
            row = model.forward([prev], cache_len + i, mask)[0]
            d = argmax_lowest(row)
            p = top1_prob(row)
            drafts.append(d)
            probs.append(p)
            prev = d
            if conf_threshold > 0.0 and p < conf_threshold:
                break
        k = len(drafts)
        rows = model.forward([x_last] + drafts, cache_len, None)
        targets = [argmax_lowest(rows[i]) for i in range(k + 1)]
        j = accept_length(drafts, targets)
        out.extend(drafts[:j])
        out.append(targets[j])
        rounds.append(Round(cache_len, drafts, probs, targets, j, [top2_margin(rows[i]) for i in range(k + 1)]))
        cache_len += j + 1
        x_last = targets[j]
        stats.rounds += 1
        stats.drafted += k
        stats.accepted += j
        stats.emitted = len(out)
    return out, stats, rounds


def knnssd_generate(model: OracleModel, prompt, anchors, labels, masks, max_new, max_draft,
                    conf_threshold=0.0, query=None):
    """The whole per-sample path (Sec. 4.2): last hidden vector -> KNN -> mask -> Self-SD.
    `query`, when given, replaces the prompt's own last hidden vector."""
    first, hidden, _ = prefill(model, prompt)
    if query is None:
        query = hidden
    n_star, dom, mask, _ = knn_select(query, anchors, labels, masks)
    toks, stats, rounds = ssd_generate(model, prompt, mask, max_new, max_draft, conf_threshold,
                                       first_token=first)
    return dict(anchor=n_star, domain=dom, mask=mask, tokens=toks, stats=stats, rounds=rounds)


# ----------------------------------------------------------------------------------------------
# report-side closed forms
# ----------------------------------------------------------------------------------------------

def expected_speedup(mean_len: float, alpha: float, c: float) -> float:
    """Eq. 9 / Eq. 10: E = M*alpha / ((M-1)*c + alpha)."""
    return mean_len * alpha / ((mean_len - 1.0) * c + alpha)


def cost_coefficient(s_mlp: float, s_attn: float, beta: float) -> float:
    """Eq. 11: c = ((1-s_mlp) + (1-s_attn)*beta) / (1+beta)."""
    return ((1.0 - s_mlp) + (1.0 - s_attn) * beta) / (1.0 + beta)


def next_domain(current: int, n_domains: int, r: float, u_switch: float, u_pick: float) -> int:
    """Eq. 8: stay with probability 1-r, otherwise move to one of the other N-1 domains
    uniformly. u_switch, u_pick are uniforms on [0,1) supplied by the caller."""
    if n_domains < 2 or u_switch >= r:
        return current
    others = [j for j in range(n_domains) if j != current]
    return others[min(int(u_pick * (n_domains - 1)), n_domains - 2)]
