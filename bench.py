#!/usr/bin/env python3
"""Benchmark of the KNN-SSD decode path on one MI355X.

One "step" is one pass of the whole per-sample path over one synthetic sample: prefill of the
prompt, KNN routing of its last hidden vector, then draft/verify rounds until max_new tokens
are out. The default workload is the 13B-shaped configuration; weights are seeded random-init
values of that shape (there are no checkpoints here), generated directly in HBM.

Prints ONE JSON line. `value` is decoded tokens per second of KNN-SSD (tokens emitted after the
prefill's own token, divided by the GPU time of KNN routing plus all draft and verify passes;
inputs resident in HBM). The plain autoregressive baseline, the prefill time, the acceptance
counters and the end-to-end rate are reported beside it, as are the roofline figures of the
verify pass and the draft pass and the CPU oracle's rate on a bounded sample.

On seeded random-init weights the top-1 probability is far below the 0.6 confidence threshold,
so every round drafts one token, and acceptance is whatever random weights give: the SSD/AR
ratio here says nothing about the paper's 1.3-1.6x, which needs trained weights.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COPY_BYTES = 1 << 30          # size of the calibration copy of --traffic-probe
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "knnssd_kernels_llama13b_hbm_traffic.md")


FAMILIES = (("gemm_mfma_kernel<false", "verification GEMM"), ("gemv_kernel", "draft GEMV"),
            ("attn_partial_mfma_kernel", "attention, matrix cores (verification)"),
            ("attn_partial_kernel", "attention, vector ALUs (draft)"), ("attn_combine_kernel", "attention merge launch"))


def traffic_parse(fetch_csv, write_csv):
    """Per-launch HBM traffic of the path's kernels from two `rocprofv3 --pmc` runs of `bench.py --traffic-probe`
    (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch). Each counter is scaled by what it reads for the plain copy of
    COPY_BYTES in the same run."""
    import csv

    def per_kernel(path, counter):
        rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]
        rows.sort(key=lambda r: int(r["Dispatch_Id"]))
        copy, fam, seen_ours = None, {}, False
        for r in rows:
            name = r["Kernel_Name"]
            hit = next((f for f, _ in FAMILIES if f in name), None)
            if hit:
                fam.setdefault(hit, []).append(float(r["Counter_Value"]))
                seen_ours = seen_ours or hit.startswith(("gemm", "gemv"))
            elif "MulFunctor" in name and not seen_ours:
                copy = float(r["Counter_Value"])           # the last multiply before the passes is the calibration copy
        return copy, fam

    out = {}
    for tag, path, counter in (("read", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        copy, fam = per_kernel(path, counter)
        scale = COPY_BYTES / (copy * 1024.0)             # true bytes per counted byte
        print(f"{tag}: copy of {COPY_BYTES} B counted as {copy:.0f} KiB -> scale {scale:.4f}")
        out[tag] = {f: (len(v), scale * 1024.0 * sum(v) / len(v)) for f, v in fam.items()}
    print("| kernel | launches | fetched B per launch | written B per launch | total B per launch |")
    print("|---|---|---|---|---|")
    for f, label in FAMILIES:
        if f in out["read"]:
            n, rd = out["read"][f]
            wr = out["write"].get(f, (0, 0.0))[1]
            print(f"| `{f}` ({label}) | {n} | {rd:.0f} | {wr:.0f} | {rd + wr:.0f} |")
    g = "gemm_mfma_kernel<false"
    print(f"traffic_bytes_per_launch: {out['read'][g][1] + out['write'][g][1]:.0f}")
    print(f"kernel_source_sha16: {kernel_source_sha16()}")


def kernel_source_sha16():
    """Hash of the library's sources: a counter measurement belongs to the kernels it was taken on."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2505_16162_amd", "csrc")
    for name in sorted(os.listdir(src)):
        h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic():
    """HBM bytes per launch of the verification GEMM as measured with the counters (profiles/), or None when
    there is no measurement or it was taken on other kernel sources than the ones this run uses."""
    val, sha = None, None
    try:
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":")[1])
            if line.startswith("kernel_source_sha16:"):
                sha = line.split(":")[1].strip()
    except OSError:
        return None
    return val if sha == kernel_source_sha16() else None


def pass_bytes(shape, mask, ctx, rows):
    """Algorithmic HBM bytes of one forward pass: weights of the retained sublayers and the LM
    head, the cached keys/values the retained attention sublayers read at context length ctx,
    the keys/values they write and one embedding row per input row."""
    wb = 2 if shape.weight_dtype == "bf16" else 4
    kb = 2 if shape.kv_dtype == "bf16" else 4
    d, f = shape.d_model, shape.d_ffn
    qd, kvd = shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    attn_w = ((qd + 2 * kvd) * d + d * qd) * wb
    mlp_w = (3 * f * d) * wb
    total = shape.vocab * d * wb + rows * d * wb
    for b in range(shape.n_blocks):
        if not mask[2 * b]:
            total += attn_w + 2 * kvd * kb * (ctx + rows)
        if not mask[2 * b + 1]:
            total += mlp_w
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama13b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the planted-acceptance and routing-scan sub-records of the benchmark line")
    ap.add_argument("--cpu-tokens", type=int, default=6, help="tokens the CPU oracle decodes for its baseline")
    ap.add_argument("--max-new", type=int, default=0, help="override the workload's generation length")
    ap.add_argument("--prompt-len", type=int, default=0, help="override the workload's prompt length")
    ap.add_argument("--stream", type=int, default=0, metavar="N",
                    help="run N samples of the workload's domain-shift stream (Eq. 8) through the stream driver and "
                         "print per-domain figures instead of the benchmark line (use with --workload llama13b_stream)")
    ap.add_argument("--mix-ratio", type=float, default=0.7, help="r of Eq. 8 for --stream")
    ap.add_argument("--no-reselect", action="store_true", help="--stream: keep the first sample's mask (fixed Self-SD)")
    ap.add_argument("--beta-probe", action="store_true",
                    help="measure the attention:MLP sublayer latency ratio (beta of Eq. 11) of the draft step and the "
                         "cost coefficient of a sublayer-granular mask with skip ratios --s-attn / --s-mlp")
    ap.add_argument("--s-attn", type=float, default=0.48)
    ap.add_argument("--s-mlp", type=float, default=0.42)
    ap.add_argument("--knn-probe", type=int, default=0, metavar="N",
                    help="time the K-nearest-anchor scan (knnssd_knn_topk, K = 8) over N anchors of dimension 5120, for 1 and 4 "
                         "queries per pass, and print its HBM rate instead of the benchmark line")
    ap.add_argument("--full-acceptance", action="store_true",
                    help="probe, not the benchmark line: the skipped blocks' output projections are zeroed in the synthetic "
                         "weights, so the draft model equals the full model and every draft is accepted; no confidence "
                         "stop. Prints tokens/s of KNN-SSD rounds of max_draft drafts against AR on the same weights")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="run under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE): one plain 1 GiB copy for calibration, "
                         "then verification passes with only the weight-streaming launches; prints nothing else")
    ap.add_argument("--traffic-parse", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="summarise the two counter_collection.csv files written by the --traffic-probe runs")
    args = ap.parse_args()
    if args.traffic_parse:
        traffic_parse(*args.traffic_parse)
        return
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU path; run with --gpus 1 "
              "(independent samples would shard round-robin over GPUs with no communication)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_16162_amd import binding, synth

    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_16162_amd.build import build_library
        build_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.knn_probe:
        print(json.dumps(knn_probe(args.knn_probe, dev)))
        return
    wl = synth.workload(args.workload)
    shape = wl.shape
    max_new = args.max_new or wl.max_new
    prompt_len = args.prompt_len or wl.prompt_len

    t0 = time.time()
    w = synth.make_weights(shape, device=dev)
    if args.full_acceptance:
        print(json.dumps(full_acceptance_probe(args, wl, shape, w, prompt_len, max_new)))
        return
    gpu = binding.KnnSsd(shape, w, max_anchors=wl.n_anchors)
    anchors, labels, centres = synth.make_anchors(shape.d_model, wl.n_anchors, wl.n_domains, wl.anchor_sigma,
                                                  device=dev, clustered=wl.n_domains < wl.n_anchors)
    masks = synth.make_block_masks(shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    prompt = synth.make_prompt(shape.vocab, prompt_len).tolist()
    torch.cuda.synchronize()
    t_setup = time.time() - t0

    if args.stream:
        print(json.dumps(stream_mode(args, gpu, wl, shape, centres, prompt_len, max_new, dev)))
        gpu.close()
        return
    if args.beta_probe:
        print(json.dumps(beta_probe(args, gpu, shape, prompt, prompt_len)))
        gpu.close()
        return
    if args.traffic_probe:
        src = torch.empty(COPY_BYTES // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)         # the calibration kernel: a plain elementwise copy, reads and writes COPY_BYTES
        torch.cuda.synchronize()
        # a few whole rounds of the benchmark's own generation: draft steps (GEMV, vector-ALU attention) and two-row
        # verification passes (GEMM, matrix-core attention) at context 1024..., every kernel of the path included
        gpu.knnssd_generate(prompt, 6, wl.max_draft, wl.conf_threshold)
        torch.cuda.synchronize()
        gpu.close()
        return

    def one_step():
        return gpu.knnssd_generate(prompt, max_new, wl.max_draft, wl.conf_threshold)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t1 = time.time()
    agg = None
    toks = None
    for _ in range(args.steps):
        toks, st = one_step()
        agg = st if agg is None else {k: agg[k] + v for k, v in st.items()}
    torch.cuda.synchronize()
    wall = time.time() - t1
    ms_per_step = wall * 1e3 / args.steps

    decode_ns = agg["ns_knn"] + agg["ns_draft"] + agg["ns_verify"]
    new_tokens = agg["emitted"] - args.steps           # the first token of each step is the prefill's
    ssd_tps = new_tokens / (decode_ns * 1e-9)
    e2e_tps = agg["emitted"] / wall

    # plain autoregressive baseline through the same entry point (max_draft = 0), same prompt
    ar_toks, ar_st = gpu.knnssd_generate(prompt, max_new, 0)
    ar_tps = (ar_st["emitted"] - 1) / (ar_st["ns_verify"] * 1e-9)
    lossless = ar_toks == toks

    # roofline of the two passes at the mean context of the run
    idx, dom, mask = gpu.knnssd_select_skipset(gpu.knnssd_prefill(prompt)[1])
    ctx_mean = prompt_len + max_new // 2
    full = [0] * (2 * shape.n_blocks)
    verify_rows = (agg["drafted"] / max(agg["rounds"], 1)) + 1
    vb = pass_bytes(shape, full, ctx_mean, verify_rows)
    db = pass_bytes(shape, mask, ctx_mean, 1)
    verify_ms = agg["ns_verify"] * 1e-6 / max(agg["verify_passes"], 1)
    draft_ms = agg["ns_draft"] * 1e-6 / max(agg["draft_passes"], 1)
    verify_gbs = vb / (verify_ms * 1e-3) / 1e9
    draft_gbs = db / (draft_ms * 1e-3) / 1e9 if agg["draft_passes"] else 0.0

    # dominant kernel (the verification GEMM, gemm_mfma_kernel): every launch of it in a verification pass
    # bracketed by HIP events on the library's stream; bytes = the weight bytes those launches stream
    roof = {"bound": "hbm", "kernel": "verify pass (all kernels)", "achieved": round(verify_gbs, 1),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(verify_gbs / HBM_PEAK_GBS, 4), "traffic": None}
    try:
        n_ver = max(1, int(round(verify_rows)))
        rows = [ar_toks[0]] + ar_toks[1:n_ver]
        acc = {"n_launches": 0, "gemm_ns": 0, "gemm_bytes": 0, "pass_ns": 0}
        reps = 5
        gpu.knnssd_profile_pass(1, rows, prompt_len)                     # warm
        for _ in range(reps):
            r = gpu.knnssd_profile_pass(1, rows, prompt_len)
            acc = {k: acc[k] + r[k] for k in acc}
        gemm_gbs = acc["gemm_bytes"] / (acc["gemm_ns"] * 1e-9) / 1e9
        # the library runs the <false, true> instance instead when a launch stages its activations in four chunks or
        # more (many rows); the headline workload's two-row passes never do
        inst = "gemm_mfma_kernel<false, false>" if args.workload == "llama13b" else "gemm_mfma_kernel<false, *>"
        roof = {"bound": "hbm", "kernel": f"{inst} (verification GEMM: the {acc['n_launches'] // reps} launches of one "
                                          "pass, back to back between two HIP events)",
                "achieved": round(gemm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gemm_gbs / HBM_PEAK_GBS, 4),
                "traffic": recorded_traffic() if args.workload == "llama13b" else None,
                "launches_per_pass": acc["n_launches"] // reps,
                "avg_launch_us": round(acc["gemm_ns"] * 1e-3 / acc["n_launches"], 2),
                "avg_bytes_per_launch": acc["gemm_bytes"] // acc["n_launches"],
                "rows": n_ver, "context": prompt_len}
        d = gpu.knnssd_profile_pass(0, rows[:1], prompt_len)
        roof["draft_gemv_kernel_GBps"] = round(d["gemm_bytes"] / (d["gemm_ns"] * 1e-9) / 1e9, 1)
        if roof["traffic"] is None:
            roof["traffic_note"] = "no counter measurement for these kernel sources under profiles/"
    except binding.KnnSsdError as e:       # shape runs on the generic kernels
        roof["note"] = f"per-kernel events unavailable: {e}"

    out = {
        "metric": "decoded tokens/s at batch 1 (KNN-SSD)", "value": round(ssd_tps, 3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights/KV, f32 activations" if shape.weight_dtype == "bf16" else "f32",
        "data": "synthetic (seeded random-init weights, uniform random prompt, Gaussian anchor clusters)",
        "config": {"workload": f"{shape.name}: {shape.n_blocks} blocks d={shape.d_model} H={shape.n_heads}/"
                               f"{shape.n_kv_heads} ffn={shape.d_ffn} V={shape.vocab}; batch 1, prompt {prompt_len}, "
                               f"generate {max_new}, max_draft {wl.max_draft}, conf_thr {wl.conf_threshold}, "
                               f"{wl.skipped_blocks}-block skip masks from 1-NN over {wl.n_anchors} anchors"},
        "ar_tokens_per_s": round(ar_tps, 3),
        "ssd_over_ar": round(ssd_tps / ar_tps, 4),
        "ssd_equals_ar_tokens": bool(lossless),
        "e2e_tokens_per_s_incl_prefill": round(e2e_tps, 3),
        "prefill_ms": round(agg["ns_prefill"] * 1e-6 / args.steps, 3),
        "knn_us": round(agg["ns_knn"] * 1e-3 / args.steps, 2),
        "mean_generated_length_M": round((agg["emitted"] - args.steps) / max(agg["rounds"], 1), 4),
        "acceptance_rate_alpha": round(agg["accepted"] / max(agg["drafted"], 1), 4),
        "drafts_per_round": round(agg["drafted"] / max(agg["rounds"], 1), 3),
        # App. C.2 accounting with the measured pass times: a round costs k draft steps + one verification and
        # emits M tokens, plain decoding costs one verification-sized pass per token
        "ssd_over_ar_from_pass_times": round(
            ((agg["emitted"] - args.steps) / max(agg["rounds"], 1)) * (1e3 / ar_tps)
            / ((agg["drafted"] / max(agg["rounds"], 1)) * draft_ms + verify_ms), 4),
        "cost_ratio_draft_over_verify": round(draft_ms / verify_ms, 4) if verify_ms else None,
        "verify_pass": {"ms": round(verify_ms, 4), "GB": round(vb / 1e9, 3), "GBps": round(verify_gbs, 1),
                        "frac_of_peak": round(verify_gbs / HBM_PEAK_GBS, 4)},
        "draft_pass": {"ms": round(draft_ms, 4), "GB": round(db / 1e9, 3), "GBps": round(draft_gbs, 1),
                       "frac_of_peak": round(draft_gbs / HBM_PEAK_GBS, 4)},
        "roofline": roof,
        # the target the path is built against: each pass as a whole (every kernel and gap) against the HBM peak
        "pass_roofline": {"target_frac": 0.70, "verify_frac": round(verify_gbs / HBM_PEAK_GBS, 4),
                          "draft_frac": round(draft_gbs / HBM_PEAK_GBS, 4),
                          "met": bool(verify_gbs / HBM_PEAK_GBS >= 0.70 and draft_gbs / HBM_PEAK_GBS >= 0.70)},
        "setup_s": round(t_setup, 1),
    }
    gpu.close()
    gpu = None
    if not args.no_extras and args.workload == "llama13b":
        # what the rounds are worth when drafts are accepted (random weights accept none), and the routing scan where
        # it is bound by HBM: sub-records of the same line
        out["planted_acceptance"] = planted_acceptance_record(wl, shape, w, prompt, max_new)
        out["knn_scan"] = {k: v for k, v in knn_probe(200000, dev).items() if k not in ("mode",)}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, w, wl, mask, args.cpu_tokens)
        out["cpu_baseline_tiny_config"] = cpu_baseline_tiny()
    print(json.dumps(out))


def stream_mode(args, gpu, wl, shape, centres, prompt_len, max_new, dev):
    """N samples of the domain-shift stream: fresh prompt and a query near the sample's domain centre per
    sample, mask re-selected per sample by the 1-NN routing (or kept from the first sample)."""
    from paper_2505_16162_amd import stream, synth
    domains = stream.domain_sequence(wl.n_domains, args.stream, args.mix_ratio, seed=synth.BASE_SEED + 7)
    res = stream.run_stream(
        gpu, wl.n_domains, domains,
        prompt_of=lambda i: synth.make_prompt(shape.vocab, prompt_len, seed=synth.BASE_SEED + 100 + i).tolist(),
        query_of=lambda i, d: synth.make_domain_query(centres, d, wl.anchor_sigma, seed=synth.BASE_SEED + 1000 + i),
        max_new=max_new, max_draft=wl.max_draft, conf_threshold=wl.conf_threshold, reselect=not args.no_reselect)

    def fig(t):
        return {"samples": t.samples, "routed_right": t.routed_right, "M": round(t.mean_generated_length, 4),
                "alpha": round(t.acceptance_rate, 4), "tokens_per_s": round(t.tokens_per_s, 2),
                "prefill_ms_per_sample": round(t.prefill_ns * 1e-6 / max(t.samples, 1), 2)}
    return {"mode": "stream", "workload": shape.name, "samples": args.stream, "mix_ratio": args.mix_ratio,
            "reselect": not args.no_reselect, "prompt_len": prompt_len, "max_new": max_new,
            "domains": domains, "routed": res.routed, "total": fig(res.total),
            "per_domain": {str(d): fig(t) for d, t in sorted(res.per_domain.items())}}


def knn_probe(n_anchors, dev):
    """The anchor scan at a size where it is bound by HBM bandwidth rather than by launch latency."""
    import torch
    from paper_2505_16162_amd import binding, synth
    d, n_dom, k = 5120, 5, 8
    shape = synth.small_shape("knn_probe", n_blocks=1, d_model=d, n_heads=40, n_kv_heads=40, head_dim=128, d_ffn=64, vocab=64,
                              max_seq=32)
    gpu = binding.KnnSsd(shape, synth.make_weights(shape, device=dev), max_anchors=n_anchors)
    anchors, labels, centres = synth.make_anchors(d, n_anchors, n_dom, 0.1, device=dev)
    gpu.knnssd_set_anchors(anchors, labels, synth.make_block_masks(1, n_dom, 1))
    out = {"mode": "knn-probe", "anchors": n_anchors, "dim": d, "k": k, "table_GB_fp32": round(n_anchors * d * 4 / 1e9, 3)}
    for tag, table, eb in (("fp32", anchors, 4), ("bf16", anchors.to(torch.bfloat16), 2)):
        gpu.knnssd_set_anchors(table, labels, synth.make_block_masks(1, n_dom, 1))
        for nq in (1, 4):
            queries = torch.stack([synth.make_domain_query(centres, i % n_dom, 0.1, seed=i) for i in range(nq)])
            idx, _, dom = gpu.knnssd_knn_topk(queries, k)
            assert dom == [i % n_dom for i in range(nq)]
            torch.cuda.synchronize()
            reps = 5
            t0 = time.time()
            for _ in range(reps):
                gpu.knnssd_knn_topk(queries, k)
            dt = (time.time() - t0) / reps
            out[f"{tag}_q{nq}"] = {"ms": round(dt * 1e3, 3), "scan_GBps": round(n_anchors * d * eb / dt / 1e9, 1),
                                   "frac_of_peak": round(n_anchors * d * eb / dt / 1e9 / HBM_PEAK_GBS, 4)}
    out["note"] = "K = 8 nearest anchors per query, whole call (scan, two-stage selection, read-back), host-timed"
    gpu.close()
    return out


def planted_acceptance_record(wl, shape, w, prompt, max_new):
    """Sub-record of the benchmark line: acceptance 1 planted as in full_acceptance_probe (the skipped blocks'
    output projections zeroed, which makes them identities), rounds of max_draft drafts and max_draft + 1 verified
    rows, no confidence stop. Reports tokens/s against AR on the same weights and the many-row verification pass."""
    import torch
    from paper_2505_16162_amd import binding, synth
    mask = synth.make_block_masks(shape.n_blocks, 1, wl.skipped_blocks)[0].tolist()
    saved = {}
    for b, blk in enumerate(w["blocks"]):
        for key, bit in (("wo", 2 * b), ("wd", 2 * b + 1)):
            if mask[bit]:
                saved[(b, key)] = blk[key].clone()
                blk[key].zero_()
    gpu = binding.KnnSsd(shape, w)
    for (b, key), t in saved.items():
        w["blocks"][b][key].copy_(t)           # the caller's weights are left as they were
    gpu.knnssd_set_skipset(mask)
    gpu.knnssd_generate(prompt, max_new, 0)
    ar_toks, ar_st = gpu.knnssd_generate(prompt, max_new, 0)
    ar_tps = (ar_st["emitted"] - 1) / (ar_st["ns_verify"] * 1e-9)
    k = wl.max_draft
    gpu.knnssd_generate(prompt, max_new, k, 0.0, route=False)
    toks, st = gpu.knnssd_generate(prompt, max_new, k, 0.0, route=False)
    dec = st["ns_draft"] + st["ns_verify"]
    tps = (st["emitted"] - 1) / (dec * 1e-9)
    rows = st["drafted"] / max(st["rounds"], 1) + 1
    v_ms = st["ns_verify"] * 1e-6 / max(st["verify_passes"], 1)
    d_ms = st["ns_draft"] * 1e-6 / max(st["draft_passes"], 1)
    ctx_mean = len(prompt) + max_new // 2
    vb = pass_bytes(shape, [0] * (2 * shape.n_blocks), ctx_mean, rows)
    gpu.close()
    return {"what": "acceptance 1 planted (skipped blocks made identities), no confidence stop", "max_draft": k,
            "tokens_per_s": round(tps, 2), "ar_tokens_per_s_same_weights": round(ar_tps, 2),
            "speedup_over_ar": round(tps / ar_tps, 3), "equals_ar_tokens": toks == ar_toks,
            "mean_generated_length_M": round((st["emitted"] - 1) / max(st["rounds"], 1), 3),
            "acceptance_rate_alpha": round(st["accepted"] / max(st["drafted"], 1), 4),
            "verify_pass": {"rows": round(rows, 2), "ms": round(v_ms, 4), "GBps": round(vb / (v_ms * 1e-3) / 1e9, 1),
                            "frac_of_peak": round(vb / (v_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
            "draft_pass_ms": round(d_ms, 4), "ms_per_round": round(dec * 1e-6 / max(st["rounds"], 1), 3)}


def cpu_baseline_tiny():
    """The oracle on the tiny configuration in full (prompt 32, 32 greedy tokens, 4 drafts per round, routing over
    8 anchors), plain autoregressive and KNN-SSD, with one thread and with every core of this box."""
    import ctypes
    import numpy as np
    from oracle import knnssd_oracle as O
    from paper_2505_16162_amd import synth
    wl = synth.workload("tiny")
    w = synth.make_weights(wl.shape)
    prompt = synth.make_prompt(wl.shape.vocab, wl.prompt_len).tolist()
    anchors, labels, _ = synth.make_anchors(wl.shape.d_model, wl.n_anchors, wl.n_domains, 1.0, clustered=False)
    masks = synth.make_block_masks(wl.shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    model = O.OracleModel(wl.shape, w)
    all_cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    try:
        omp = ctypes.CDLL("libgomp.so.1")
    except OSError:
        omp = None
    out = {"config": "tiny: 4 blocks d=256 fp32, prompt 32, 32 tokens, 4 drafts per round, 8 anchors"}
    for threads in ((1, all_cores) if omp is not None else (all_cores,)):
        if omp is not None:
            omp.omp_set_num_threads(int(threads))
        t0 = time.time()
        O.greedy_ar(model, prompt, wl.max_new)
        t_ar = time.time() - t0
        t0 = time.time()
        O.knnssd_generate(model, prompt, anchors.numpy(), labels.numpy(), masks.numpy(), wl.max_new, wl.max_draft,
                          wl.conf_threshold)
        t_ssd = time.time() - t0
        out["threads_%d" % threads] = {"ar_tokens_per_s": round(wl.max_new / t_ar, 2),
                                       "knnssd_tokens_per_s": round(wl.max_new / t_ssd, 2)}
    if omp is not None:
        omp.omp_set_num_threads(int(all_cores))
    return out


def full_acceptance_probe(args, wl, shape, w, prompt_len, max_new):
    """What the rounds cost when every draft is accepted (alpha = 1, the upper end of the regime the paper
    works in: App. C.2 reports alpha 0.8-0.95). Random-init weights accept nothing, so this probe plants the
    acceptance: the output projections (attention O, MLP down) of the blocks the mask skips are zeroed, which
    makes those blocks identities, so the draft model IS the full model. Rounds then draft max_draft tokens
    (no confidence stop), verify max_draft + 1 rows and emit max_draft + 1 tokens."""
    import torch
    from paper_2505_16162_amd import binding, synth
    mask = synth.make_block_masks(shape.n_blocks, 1, wl.skipped_blocks)[0].tolist()
    for b, blk in enumerate(w["blocks"]):
        if mask[2 * b]:
            blk["wo"].zero_()
        if mask[2 * b + 1]:
            blk["wd"].zero_()
    gpu = binding.KnnSsd(shape, w)
    prompt = synth.make_prompt(shape.vocab, prompt_len).tolist()
    gpu.knnssd_set_skipset(mask)
    out = {"probe": "full acceptance (planted: skipped blocks are identities)", "workload": shape.name,
           "skipped_blocks": wl.skipped_blocks, "prompt": prompt_len, "generate": max_new}
    ar_toks, ar_st = gpu.knnssd_generate(prompt, max_new, 0)
    ar_toks, ar_st = gpu.knnssd_generate(prompt, max_new, 0)
    ar_tps = (ar_st["emitted"] - 1) / (ar_st["ns_verify"] * 1e-9)
    out["ar_tokens_per_s"] = round(ar_tps, 2)
    rows = []
    for k in (1, 2, 4, 8, 15):
        gpu.knnssd_generate(prompt, max_new, k, 0.0)
        toks, st = gpu.knnssd_generate(prompt, max_new, k, 0.0)
        dec = st["ns_draft"] + st["ns_verify"]
        tps = (st["emitted"] - 1) / (dec * 1e-9)
        rows.append({"max_draft": k, "tokens_per_s": round(tps, 2), "speedup_over_ar": round(tps / ar_tps, 3),
                     "mean_generated_length_M": round((st["emitted"] - 1) / max(st["rounds"], 1), 3),
                     "acceptance_rate_alpha": round(st["accepted"] / max(st["drafted"], 1), 4),
                     "ms_per_round": round(dec * 1e-6 / max(st["rounds"], 1), 3),
                     "equals_ar_tokens": toks == ar_toks})
    out["rounds_by_max_draft"] = rows
    gpu.close()
    return out


def beta_probe(args, gpu, shape, prompt, prompt_len):
    """Latency of the draft step with nothing / only attention / only MLP / everything retained gives the
    per-sublayer costs and beta = attention : MLP latency (App. C.2); the cost coefficient of a
    sublayer-granular mask is then compared with Eq. 11 evaluated at that beta."""
    import torch
    from paper_2505_16162_amd import synth
    nb = shape.n_blocks
    gpu.knnssd_prefill(prompt)
    tok = prompt[0]

    def draft_ms(mask, reps=12):
        gpu.knnssd_set_skipset(mask)
        gpu.knnssd_draft_step(tok, prompt_len)
        torch.cuda.synchronize()
        t0 = time.time()
        for _ in range(reps):
            gpu.knnssd_draft_step(tok, prompt_len)
        torch.cuda.synchronize()
        return (time.time() - t0) * 1e3 / reps

    t_none = draft_ms([1] * (2 * nb))                       # embedding + LM head only
    t_attn = draft_ms([0, 1] * nb)                          # every attention sublayer, no MLP
    t_mlp = draft_ms([1, 0] * nb)                           # every MLP sublayer, no attention
    t_full = draft_ms([0] * (2 * nb))
    per_attn = (t_attn - t_none) / nb
    per_mlp = (t_mlp - t_none) / nb
    beta = per_attn / per_mlp
    m = synth.make_sublayer_masks(nb, 1, args.s_attn, args.s_mlp, seed=synth.BASE_SEED + 9).numpy()[0]
    s_attn = float(m[0::2].mean())
    s_mlp = float(m[1::2].mean())
    t_mask = draft_ms(m.tolist())
    c_eq11 = ((1 - s_mlp) + (1 - s_attn) * beta) / (1 + beta)          # Eq. 11
    c_uniform = 1 - (s_attn + s_mlp) / 2                               # c = 1 - s (Eq. 9's cost model)
    return {"mode": "beta-probe", "workload": shape.name, "context": prompt_len,
            "draft_ms": {"head_only": round(t_none, 4), "attention_only": round(t_attn, 4), "mlp_only": round(t_mlp, 4),
                         "full": round(t_full, 4), "masked": round(t_mask, 4)},
            "attention_sublayer_us": round(per_attn * 1e3, 2), "mlp_sublayer_us": round(per_mlp * 1e3, 2),
            "beta": round(beta, 4), "mask_skip_ratio_attn": round(s_attn, 4), "mask_skip_ratio_mlp": round(s_mlp, 4),
            "c_measured_sublayers_only": round((t_mask - t_none) / (t_full - t_none), 4),
            "c_measured_whole_step": round(t_mask / t_full, 4),
            "c_eq11_at_measured_beta": round(c_eq11, 4), "c_one_minus_s": round(c_uniform, 4),
            "note": "times include one host round trip per draft step (the call returns the token)"}


def cpu_baseline(shape, w_dev, wl, mask, n_tokens):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample: same model
    and weights, a 16-token prompt, n_tokens decoded by Self-SD rounds with the routed mask."""
    import numpy as np
    from oracle import knnssd_oracle as O
    from paper_2505_16162_amd import synth
    w_host = synth.weights_to(w_dev, "cpu")
    prompt = synth.make_prompt(shape.vocab, 16, seed=77).tolist()
    model = O.OracleModel(shape, w_host)
    t0 = time.time()
    first = O.prefill(model, prompt)[0]
    t_prefill = time.time() - t0
    t0 = time.time()
    toks, st, _ = O.ssd_generate(model, prompt, np.asarray(mask, np.uint8), n_tokens + 1, wl.max_draft,
                                 wl.conf_threshold, first_token=first)
    dt = time.time() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    return {"value": round(n_tokens / dt, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"same {shape.name} weights, 16-token prompt (prefill {t_prefill:.1f}s not counted), "
                      f"{n_tokens} tokens by Self-SD rounds ({st.rounds} verify + {st.drafted} draft passes) in {dt:.1f}s"}


if __name__ == "__main__":
    main()
