"""Domain-shift stream driver (Sec. 4.2, Eq. 8; the task streams of Sec. 5.2).

A stream is a sequence of samples, each from one of N domains. The next sample changes domain with
probability r (the mix ratio) and then lands on each of the other N-1 domains with equal probability;
r = 0 is a task-by-task stream, r = 1 switches domain at every sample. For every sample the library runs
the whole per-sample path (`knnssd_generate`: prefill, 1-NN routing of the sample's query vector, Self-SD
rounds with the routed mask). With `reselect=False` the mask routed for the FIRST sample is kept for the
whole stream, which is the fixed-configuration Self-SD baseline of Sec. 5.1.

Host code only, and bookkeeping only: every step of the path runs in the library's kernels and the chain's
transition rule is the library's `knnssd_stream_next_domain`. The uniform draws that drive the chain and the
synthetic prompts / queries come from the seeded generators in `synth`.
"""
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import torch

from . import binding, synth


def domain_after(current: int, n_domains: int, r: float, u_switch: float, u_pick: float) -> int:
    """One transition of the Eq. 8 chain from two uniforms on [0, 1): the library's knnssd_stream_next_domain."""
    return binding.knnssd_stream_next_domain(current, n_domains, r, u_switch, u_pick)


def domain_sequence(n_domains: int, n_samples: int, r: float, seed: int, first: int = 0) -> List[int]:
    """Domains of a stream of n_samples samples; sample 0 is in `first`."""
    draws = synth.mix_ratio_stream(n_domains, n_samples, r, seed)
    out, cur = [], first
    for i in range(n_samples):
        if i > 0:
            cur = domain_after(cur, n_domains, r, float(draws[i, 0]), float(draws[i, 1]))
        out.append(cur)
    return out


@dataclass
class DomainTotals:
    samples: int = 0
    routed_right: int = 0
    rounds: int = 0
    drafted: int = 0
    accepted: int = 0
    emitted: int = 0
    decode_ns: int = 0        # KNN routing + draft + verify GPU time
    prefill_ns: int = 0

    @property
    def mean_generated_length(self) -> float:      # M of App. C.2: tokens per verification pass
        return (self.emitted - self.samples) / self.rounds if self.rounds else 0.0

    @property
    def acceptance_rate(self) -> float:            # alpha of App. C.2: accepted / drafted
        return self.accepted / self.drafted if self.drafted else 0.0

    @property
    def tokens_per_s(self) -> float:
        return (self.emitted - self.samples) / (self.decode_ns * 1e-9) if self.decode_ns else 0.0


@dataclass
class StreamResult:
    domains: List[int]                     # true domain of each sample
    routed: List[int]                      # domain the 1-NN routing chose (mask in force for the sample)
    tokens: List[List[int]]
    per_domain: Dict[int, DomainTotals] = field(default_factory=dict)
    total: DomainTotals = field(default_factory=DomainTotals)


def run_stream(gpu, n_domains: int, domains: Sequence[int], prompt_of: Callable[[int], Sequence[int]],
               query_of: Callable[[int, int], Optional[torch.Tensor]], max_new: int, max_draft: int,
               conf_threshold: float = 0.0, reselect: bool = True) -> StreamResult:
    """Runs the samples of a stream one after the other on one `KnnSsd` handle whose anchors are installed.

    prompt_of(i) gives sample i's token ids; query_of(i, domain) its routing query (None: the prompt's own
    last hidden vector, the paper's method). reselect=False routes only sample 0 and keeps that mask.
    """
    res = StreamResult(domains=list(domains), routed=[], tokens=[])
    kept_domain = None
    for i, dom in enumerate(domains):
        prompt = prompt_of(i)
        query = query_of(i, dom)
        if reselect or i == 0:
            toks, st = gpu.knnssd_generate(prompt, max_new, max_draft, conf_threshold, query=query)
            routed = gpu.last_domain()
            kept_domain = routed
        else:
            # the mask installed by sample 0 stays in force: generate without routing
            toks, st = gpu.knnssd_generate(prompt, max_new, max_draft, conf_threshold, query=None, route=False)
            routed = kept_domain
        res.routed.append(routed)
        res.tokens.append(toks)
        for tot in (res.per_domain.setdefault(dom, DomainTotals()), res.total):
            tot.samples += 1
            tot.routed_right += int(routed == dom)
            tot.rounds += st["rounds"]
            tot.drafted += st["drafted"]
            tot.accepted += st["accepted"]
            tot.emitted += st["emitted"]
            tot.decode_ns += st["ns_knn"] + st["ns_draft"] + st["ns_verify"]
            tot.prefill_ns += st["ns_prefill"]
    return res
