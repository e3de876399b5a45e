"""GPU parity at the benchmark's real shapes, in the launch configuration bench.py times.

The oracle cannot decode hundreds of 13B-shaped tokens in a test, so the full-size check has
two parts: (i) the oracle runs the same 13B-shaped model on a short prompt and a few tokens and
everything is compared (KNN index, mask, tokens, acceptance counts, logits); (ii) at the
benchmark's own prompt length the properties that hold at any size are asserted on the GPU
path itself: the speculative output equals plain autoregressive decoding, an empty skip set is
accepted in full, and a row's result does not depend on how many rows share the pass.
"""
import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import binding, synth
from gpu_common import logits_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def llama13b():
    wl = synth.workload("llama13b")
    print("building 13B-shaped model on the GPU", flush=True)
    w = synth.make_weights(wl.shape, device="cuda:0")
    gpu = binding.KnnSsd(wl.shape, w, max_anchors=wl.n_anchors)
    anchors, labels, centres = synth.make_anchors(wl.shape.d_model, wl.n_anchors, wl.n_domains, wl.anchor_sigma,
                                                  device="cuda:0")
    masks = synth.make_block_masks(wl.shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    yield wl, w, gpu, anchors, labels, masks
    gpu.close()


@pytest.mark.timeout(900)
def test_13b_short_run_matches_oracle(llama13b):
    wl, w, gpu, anchors, labels, masks = llama13b
    shape = wl.shape
    print("copying 26 GB of weights to the host for the oracle", flush=True)
    orc = O.OracleModel(shape, synth.weights_to(w, "cpu"))
    prompt = synth.make_prompt(shape.vocab, 24, seed=123).tolist()      # one full 16-row chunk + a ragged one
    print("oracle prefill", flush=True)
    first_o, hidden_o, row_o = O.prefill(orc, prompt)
    first_g, hidden_g = gpu.knnssd_prefill(prompt)
    ok, err = logits_close(gpu.knnssd_get_logits(7).numpy(), row_o, shape)
    assert ok, err
    assert first_g == first_o
    assert np.abs(hidden_g.cpu().numpy() - hidden_o).max() <= 2e-2 * np.abs(hidden_o).max()
    # KNN routing of the prompt's own last hidden vector over the 1000-anchor table
    idx_g, dom_g, mask_g = gpu.knnssd_select_skipset(hidden_g)
    idx_o, dom_o, mask_o, scores = O.knn_select(hidden_o, anchors.cpu().numpy(), labels.cpu().numpy(), masks.numpy())
    assert (idx_g, dom_g, mask_g) == (idx_o, dom_o, mask_o.tolist())
    # one draft step and one 3-row verification, logits compared
    print("oracle draft + verify", flush=True)
    row = orc.forward([first_o], len(prompt), mask_o)[0]
    tok_g, p_g = gpu.knnssd_draft_step(first_o, len(prompt))
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    print("draft logits max abs err", err, "top-1 prob", p_g, O.top1_prob(row), flush=True)
    # p = 1 / sum exp(l - l_max): an absolute logit error e moves it by about e relative (bf16 KV rounding
    # differences of one ulp in a few cache entries give e ~ 1e-3 here)
    assert tok_g == O.argmax_lowest(row) and abs(p_g - O.top1_prob(row)) <= 1e-2 * O.top1_prob(row)
    rows_in = [first_o, tok_g, 17]
    rows_o = orc.forward(rows_in, len(prompt), None)
    j, nxt, new_len = gpu.knnssd_verify(rows_in, len(prompt))
    for r in range(3):
        ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
        assert ok, (r, err)
    targets = [O.argmax_lowest(rows_o[r]) for r in range(3)]
    assert j == O.accept_length(rows_in[1:], targets) and nxt == targets[j] and new_len == len(prompt) + j + 1
    # the whole path for a few tokens, with the benchmark's draft rule (threshold 0.6 => one draft per round)
    print("oracle generate", flush=True)
    res = O.knnssd_generate(orc, prompt, anchors.cpu().numpy(), labels.cpu().numpy(), masks.numpy(), 5, wl.max_draft,
                            wl.conf_threshold)
    toks, st = gpu.knnssd_generate(prompt, 5, wl.max_draft, wl.conf_threshold)
    margins = [min(r.margins) for r in res["rounds"]]
    assert toks == res["tokens"], f"oracle top-2 margins {margins}"
    assert (st["rounds"], st["drafted"], st["accepted"]) == (res["stats"].rounds, res["stats"].drafted, res["stats"].accepted)
    del orc


@pytest.mark.timeout(600)
def test_13b_properties_at_benchmark_size(llama13b):
    wl, w, gpu, anchors, labels, masks = llama13b
    shape = wl.shape
    prompt = synth.make_prompt(shape.vocab, wl.prompt_len).tolist()
    max_new = 48
    print("AR", flush=True)
    ar, st_ar = gpu.knnssd_generate(prompt, max_new, 0)
    assert len(ar) == max_new and st_ar["rounds"] == max_new - 1
    # losslessness: KNN-routed mask, benchmark draft rule, and an unconditional 8-token draft
    print("SSD", flush=True)
    for max_draft, thr in ((wl.max_draft, wl.conf_threshold), (wl.max_draft, 0.0)):
        toks, st = gpu.knnssd_generate(prompt, max_new, max_draft, thr)
        assert toks == ar
        assert st["emitted"] == max_new and st["accepted"] <= st["drafted"]
        if thr > 0:
            assert st["drafted"] <= st["rounds"]          # random-init top-1 probability << 0.6: one draft per round
    # empty skip set: the draft model is the full model, so drafts are accepted (the draft step sums on the
    # vector ALUs and verification on the matrix cores, so a near-tie may flip a token: allow a few)
    print("empty mask", flush=True)
    gpu.knnssd_set_skipset(None)      # generate() would re-route through the anchors, so use the step calls
    first, _ = gpu.knnssd_prefill(prompt)
    assert first == ar[0]
    pos, x_last, out, drafted, accepted = len(prompt), first, [first], 0, 0
    while len(out) < 24:
        drafts, prev = [], x_last
        for i in range(4):
            d, p = gpu.knnssd_draft_step(prev, pos + i)
            drafts.append(d)
            prev = d
        j, nxt, new_len = gpu.knnssd_verify([x_last] + drafts, pos)
        out += drafts[:j] + [nxt]
        drafted += 4
        accepted += j
        pos, x_last = new_len, nxt
    assert out[:24] == ar[:24]
    assert accepted >= drafted - 2
    # a row's logits do not depend on how many rows share the verification pass
    print("row independence", flush=True)
    gpu.knnssd_prefill(prompt)
    rows_in = [ar[0]] + ar[1:9]
    gpu.knnssd_verify(rows_in, len(prompt))
    many = [gpu.knnssd_get_logits(r).clone() for r in range(9)]
    gpu.knnssd_prefill(prompt)
    for r in range(3):
        gpu.knnssd_verify(rows_in[r:r + 1], len(prompt) + r)
        assert torch.equal(gpu.knnssd_get_logits(0), many[r]), r


@pytest.mark.timeout(600)
def test_13b_stream_configuration_properties(llama13b):
    """The domain-shift stream's configuration on the full 13B-shaped model: a 4096-token prompt (17 split-KV chunks
    of 40 heads x 128: more attention work items than workgroups on both kernels) and routing over 5000 anchors.
    The oracle cannot prefill that, so: the routing of the GPU's own hidden vector is compared with the exhaustive
    oracle (index, domain, mask), and the properties that hold at any size are asserted at that context."""
    _, w, _, _, _, _ = llama13b
    wl = synth.workload("llama13b_stream")
    shape = wl.shape
    gpu = binding.KnnSsd(shape, w, max_anchors=wl.n_anchors)
    anchors, labels, centres = synth.make_anchors(shape.d_model, wl.n_anchors, wl.n_domains, wl.anchor_sigma, device="cuda:0")
    masks = synth.make_block_masks(shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    prompt = synth.make_prompt(shape.vocab, wl.prompt_len, seed=31).tolist()
    print("prefill of", len(prompt), "rows", flush=True)
    first, hidden = gpu.knnssd_prefill(prompt)
    a_np, l_np = anchors.cpu().numpy(), labels.cpu().numpy()
    for dom in range(wl.n_domains):
        # the model's own hidden vector, then a query near each domain's centre (what the stream hands over)
        q = hidden if dom == 0 else synth.make_domain_query(centres.cpu(), dom, wl.anchor_sigma, seed=60 + dom).to("cuda:0")
        n_star, d_star, mask, _ = O.knn_select(q.cpu().numpy(), a_np, l_np, masks.numpy())
        assert gpu.knnssd_select_skipset(q) == (n_star, d_star, mask.tolist()), dom
        if dom > 0:
            assert d_star == dom
    max_new = 24
    print("AR", flush=True)
    ar, st_ar = gpu.knnssd_generate(prompt, max_new, 0)
    assert len(ar) == max_new and ar[0] == first
    print("SSD", flush=True)
    for thr in (wl.conf_threshold, 0.0):
        toks, st = gpu.knnssd_generate(prompt, max_new, wl.max_draft, thr)
        assert toks == ar, thr
        assert st["emitted"] == max_new and st["accepted"] <= st["drafted"]
    print("row independence", flush=True)
    gpu.knnssd_prefill(prompt)
    rows_in = [ar[0]] + ar[1:9]
    gpu.knnssd_verify(rows_in, len(prompt))
    many = [gpu.knnssd_get_logits(r).clone() for r in range(9)]
    gpu.knnssd_prefill(prompt)
    for r in range(3):
        gpu.knnssd_verify(rows_in[r:r + 1], len(prompt) + r)
        assert torch.equal(gpu.knnssd_get_logits(0), many[r]), r
    gpu.close()


@pytest.mark.timeout(600)
def test_13b_many_row_prefill_equals_16_row_passes(llama13b):
    """The prompt prefill the benchmark runs (many-row kernels over 1008 of the 1024 rows) against the same prompt
    sent through 16-row verification passes (cfg.prefill_mode = KNNSSD_PREFILL_CHUNKED), on the full 40-block model:
    the two paths sum in different orders, so cached values may sit on neighbouring bf16 values and the divergence
    grows with depth; keys, values, the last hidden vector and the first token's logits must stay within the
    tolerances of the bf16 path. (The 16-row passes are the kernels every oracle comparison covers.)"""
    wl, w, gpu, anchors, labels, masks = llama13b
    shape = wl.shape
    prompt = synth.make_prompt(shape.vocab, wl.prompt_len).tolist()
    first_t, hidden_t = gpu.knnssd_prefill(prompt)
    where = [(b, pos) for b in (0, 1, 20, 39) for pos in (0, 15, 16, 511, 1007, 1008, 1023)]
    kv_t = {bp: gpu.knnssd_read_kv(*bp) for bp in where}
    logits_t = gpu.knnssd_get_logits(15).clone()
    print("second context: 16-row passes", flush=True)
    gpu2 = binding.KnnSsd(shape, w, chunked_prefill=True)
    first_c, hidden_c = gpu2.knnssd_prefill(prompt)
    worst = 0.0
    for bp in where:
        for got, want in zip(kv_t[bp], gpu2.knnssd_read_kv(*bp)):
            g, r = got.numpy().astype(np.float64), want.numpy().astype(np.float64)
            # neighbouring bf16 values (2^-7 of the value), plus what the divergence of the inputs adds at depth
            tol = np.abs(r) * 2.0 ** -7 + (2e-3 if bp[0] == 0 else 2e-2) * np.abs(r).max()
            worst = max(worst, float((np.abs(g - r) / tol).max()))
    print("largest cache difference / tolerance: %.3f" % worst, flush=True)
    assert worst <= 1.0
    ht, hc = hidden_t.cpu().numpy(), hidden_c.cpu().numpy()
    assert np.abs(ht - hc).max() <= 2e-2 * np.abs(hc).max()
    ok, err = logits_close(logits_t.numpy(), gpu2.knnssd_get_logits(15).numpy(), shape)
    assert ok, err
    assert first_t == first_c
    gpu2.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["llama7b", "qwen14b"])
def test_full_depth_short_run_matches_oracle(name):
    """The 7B-shaped and the Qwen-14B-shaped configurations at their full depth (32 and 48 blocks, the benchmark's
    anchor tables and draft rules) on a prompt short enough for the oracle: first token and its logits, routing of the
    prompt's own hidden vector, a draft step, a verification pass, and a few generated tokens with their counters; then, at
    the benchmark's prompt length, the properties that need no oracle."""
    wl = synth.workload(name)
    shape = wl.shape
    print("building", name, flush=True)
    w = synth.make_weights(shape, device="cuda:0", seed=17)
    gpu = binding.KnnSsd(shape, w, max_anchors=wl.n_anchors)
    anchors, labels, _ = synth.make_anchors(shape.d_model, wl.n_anchors, wl.n_domains, wl.anchor_sigma, seed=5)
    masks = synth.make_block_masks(shape.n_blocks, wl.n_domains, wl.skipped_blocks, seed=4)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    print("copying the weights to the host for the oracle", flush=True)
    orc = O.OracleModel(shape, synth.weights_to(w, "cpu"))
    prompt = synth.make_prompt(shape.vocab, 24, seed=77).tolist()
    first_o, hidden_o, row_o = O.prefill(orc, prompt)
    first_g, hidden_g = gpu.knnssd_prefill(prompt)
    ok, err = logits_close(gpu.knnssd_get_logits(7).numpy(), row_o, shape)
    assert ok, err
    assert first_g == first_o, O.top2_margin(row_o)
    idx_o, dom_o, mask_o, _ = O.knn_select(hidden_o, anchors.numpy(), labels.numpy(), masks.numpy())
    assert gpu.knnssd_select_skipset(hidden_g) == (idx_o, dom_o, mask_o.tolist())
    row = orc.forward([first_o], len(prompt), mask_o)[0]
    tok_g, p_g = gpu.knnssd_draft_step(first_o, len(prompt))
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    assert tok_g == O.argmax_lowest(row) and abs(p_g - O.top1_prob(row)) <= 1e-2 * O.top1_prob(row)
    rows_in = [first_o, tok_g, 17, 5]
    rows_o = orc.forward(rows_in, len(prompt), None)
    j, nxt, new_len = gpu.knnssd_verify(rows_in, len(prompt))
    for r in range(4):
        ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
        assert ok, (r, err)
    targets = [O.argmax_lowest(rows_o[r]) for r in range(4)]
    assert j == O.accept_length(rows_in[1:], targets) and nxt == targets[j] and new_len == len(prompt) + j + 1
    print("oracle generate", flush=True)
    res = O.knnssd_generate(orc, prompt, anchors.numpy(), labels.numpy(), masks.numpy(), 5, wl.max_draft, wl.conf_threshold)
    toks, st = gpu.knnssd_generate(prompt, 5, wl.max_draft, wl.conf_threshold)
    margins = [min(r.margins) for r in res["rounds"]]
    assert toks == res["tokens"], f"oracle top-2 margins {margins}"
    assert (st["rounds"], st["drafted"], st["accepted"]) == (res["stats"].rounds, res["stats"].drafted, res["stats"].accepted)
    del orc
    # at the benchmark's own prompt length, what holds at any size: SSD output = AR output, rows independent of the pass
    print("benchmark prompt length", flush=True)
    prompt_b = synth.make_prompt(shape.vocab, wl.prompt_len).tolist()
    ar, st_ar = gpu.knnssd_generate(prompt_b, 24, 0)
    assert len(ar) == 24 and st_ar["rounds"] == 23
    for thr in (wl.conf_threshold, 0.0) if wl.conf_threshold > 0 else (0.0,):
        toks, st = gpu.knnssd_generate(prompt_b, 24, wl.max_draft, thr)
        assert toks == ar, thr
        assert st["emitted"] == 24 and st["accepted"] <= st["drafted"]
    gpu.knnssd_prefill(prompt_b)
    rows_b = [ar[0]] + ar[1:9]
    gpu.knnssd_verify(rows_b, len(prompt_b))
    many = [gpu.knnssd_get_logits(r).clone() for r in range(9)]
    gpu.knnssd_prefill(prompt_b)
    for r in range(3):
        gpu.knnssd_verify(rows_b[r:r + 1], len(prompt_b) + r)
        assert torch.equal(gpu.knnssd_get_logits(0), many[r]), r
    gpu.close()


@pytest.mark.timeout(600)
def test_qwen_widths_gqa_big_vocab_matches_oracle():
    """Qwen-2.5-14B-shaped widths (GQA 40/8, vocab 152064, FFN 13824) at reduced depth so that the oracle
    finishes in seconds; exercises the tile shapes of the 14B-shaped configuration, 9-row verification
    and the 1.56 GB LM head."""
    full = synth.workload("qwen14b")
    s = full.shape
    shape = synth.ModelShape("qwen_w4", 4, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 320,
                             "bf16", "bf16")
    w = synth.make_weights(shape, device="cuda:0", seed=5)
    gpu = binding.KnnSsd(shape, w)
    orc = O.OracleModel(shape, synth.weights_to(w, "cpu"))
    prompt = synth.make_prompt(shape.vocab, 40, seed=9).tolist()
    mask = synth.make_block_masks(shape.n_blocks, 1, 2, seed=1).numpy()[0]
    print("oracle", flush=True)
    toks_o, st_o, rounds = O.ssd_generate(orc, prompt, mask, 20, 8, 0.0)
    gpu.knnssd_set_skipset(mask.tolist())
    toks_g, st_g = gpu.knnssd_generate(prompt, 20, 8, 0.0)
    assert toks_g == toks_o, [min(r.margins) for r in rounds]
    assert (st_g["rounds"], st_g["drafted"], st_g["accepted"]) == (st_o.rounds, st_o.drafted, st_o.accepted)
    # logits of a 9-row verification
    first = toks_o[0]
    gpu.knnssd_prefill(prompt)
    rows_in = [first] + toks_o[1:9]
    orc2 = O.OracleModel(shape, synth.weights_to(w, "cpu"))
    orc2.forward(prompt, 0, None, logits_from=len(prompt))
    rows_o = orc2.forward(rows_in, len(prompt), None)
    j, nxt, _ = gpu.knnssd_verify(rows_in, len(prompt))
    for r in range(9):
        ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
        assert ok, (r, err)
    assert j == 8 and nxt == toks_o[9]
    gpu.close()
