"""Writes tests/golden/config3_prompt1024_first16.json: the CPU oracle's run of the 13B-shaped benchmark
configuration as specified (40 blocks, prompt of 1024 random ids, the first 16 generated tokens, draft rule
max 8 / confidence 0.6, 1-NN routing over 1000 anchors in 5 clusters with 20-block skip masks).

Imports only the oracle and the seeded input generators. The weights and anchors come from the counter-based
generator (synth.make_weights(counter=True)), which gives the same bytes on the host and on the GPU, so the GPU
test regenerates them on the device instead of shipping 26 GB. Nothing here comes from the HIP path.

Run from the repository root (about half an hour on 8 cores, 30 GB of memory):
    python tests/golden/make_config3_golden.py
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import knnssd_oracle as O                    # noqa: E402
from paper_2505_16162_amd import synth                   # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config3_prompt1024_first16.json")
N_TOKENS = 16
KV_BLOCKS = (0, 19, 39)
KV_POSITIONS = (0, 15, 16, 511, 1007, 1008, 1023)


def main():
    wl = synth.workload("llama13b")
    shape = wl.shape
    t0 = time.time()
    w = synth.make_weights(shape, device="cpu", counter=True)
    print("weights: %.0f s" % (time.time() - t0), flush=True)
    anchors, labels, _ = synth.make_anchors(shape.d_model, wl.n_anchors, wl.n_domains, wl.anchor_sigma, counter=True)
    masks = synth.make_block_masks(shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    prompt = synth.make_prompt(shape.vocab, wl.prompt_len).tolist()
    orc = O.OracleModel(shape, w)

    t0 = time.time()
    first, hidden, row = O.prefill(orc, prompt)
    print("prefill: %.0f s, first token %d" % (time.time() - t0, first), flush=True)
    kv = {}
    for b in KV_BLOCKS:
        for pos in KV_POSITIONS:
            k, v = orc.read_kv(b, pos)
            # the first eight dimensions of the first head and the last eight of the last head
            kv["%d:%d" % (b, pos)] = {"k": [float(x) for x in np.concatenate([k[:8], k[-8:]])],
                                      "v": [float(x) for x in np.concatenate([v[:8], v[-8:]])]}
    top = np.argsort(-row.astype(np.float64), kind="stable")[:5]
    n_star, dom, mask, scores = O.knn_select(hidden, anchors.numpy(), labels.numpy(), masks.numpy())
    order = np.argsort(-scores, kind="stable")
    t0 = time.time()
    toks, stats, rounds = O.ssd_generate(orc, prompt, mask, N_TOKENS, wl.max_draft, wl.conf_threshold, first_token=first)
    print("decode: %.0f s" % (time.time() - t0), flush=True)
    out = {
        "what": "CPU oracle, 13B-shaped configuration, counter-based weights (synth.make_weights(counter=True))",
        "prompt_len": len(prompt), "n_tokens": N_TOKENS, "max_draft": wl.max_draft, "conf_threshold": wl.conf_threshold,
        "first_token": int(first),
        "first_logits_top5": [[int(i), float(row[i])] for i in top],
        "first_logits_absmax": float(np.abs(row).max()),
        "hidden_head16": [float(x) for x in hidden[:16]],
        "hidden_norm": float(np.sqrt((hidden.astype(np.float64) ** 2).sum())),
        "anchor": int(n_star), "domain": int(dom), "mask": [int(x) for x in mask],
        "cosine_best": float(scores[order[0]]), "cosine_second": float(scores[order[1]]),
        "tokens": [int(t) for t in toks],
        "rounds": stats.rounds, "drafted": stats.drafted, "accepted": stats.accepted,
        "round_drafts": [[int(d) for d in r.drafts] for r in rounds],
        "round_draft_probs": [[float(p) for p in r.draft_probs] for r in rounds],
        "round_targets": [[int(t) for t in r.targets] for r in rounds],
        "round_margins": [[float(m) for m in r.margins] for r in rounds],
        "kv_samples": kv,
    }
    with open(OUT, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", OUT, flush=True)


if __name__ == "__main__":
    main()
