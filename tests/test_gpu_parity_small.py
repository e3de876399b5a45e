"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element,
on seeded inputs small enough for the oracle to finish in seconds."""
import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import binding, synth
from gpu_common import logits_close, make_pair

pytestmark = pytest.mark.gpu

SHAPES = {
    "tiny_fp32": synth.workload("tiny").shape,
    "bf16_mha": synth.small_shape("bf16_mha", max_seq=160),
    # d_ffn a multiple of 32: verification runs on the matrix-core kernels (688 above falls back to the generic ones)
    "bf16_gqa_hd128": synth.small_shape("bf16_gqa", n_blocks=3, d_model=384, n_heads=6, n_kv_heads=2, head_dim=128,
                                        d_ffn=992, vocab=1531, max_seq=160),
    "bf16_mfma_hd64": synth.small_shape("bf16_mfma", d_ffn=704, vocab=2000, max_seq=160),
    "fp32_gqa": synth.small_shape("fp32_gqa", n_heads=4, n_kv_heads=1, weight_dtype="fp32", kv_dtype="fp32",
                                  d_ffn=344, vocab=777, max_seq=160),
    "bf16_w_fp32_kv": synth.small_shape("mixed", kv_dtype="fp32", max_seq=160),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_prefill_draft_verify_logits(name):
    shape = SHAPES[name]
    print("case", name, flush=True)
    w, orc, gpu = make_pair(shape, seed=11, std=0.05)
    prompt = synth.make_prompt(shape.vocab, 37, seed=5).tolist()   # 37: two full 16-row chunks + ragged tail
    first_o, hidden_o, row_o = O.prefill(orc, prompt)
    first_g, hidden_g = gpu.knnssd_prefill(prompt)
    ok, err = logits_close(gpu.knnssd_get_logits(4).numpy(), row_o, shape)   # row 4 of the last chunk (rows 32..36)
    assert ok, err
    assert first_g == first_o
    assert np.abs(hidden_g.cpu().numpy() - hidden_o).max() <= (1e-4 if shape.weight_dtype == "fp32" else 2e-2)
    # cached keys/values of the prompt
    for blk in range(shape.n_blocks):
        for pos in (0, 15, 16, 36):
            kg, vg = gpu.knnssd_read_kv(blk, pos)
            ko, vo = orc.read_kv(blk, pos)
            tol = 1e-4 if shape.kv_dtype == "fp32" else 2e-2
            assert np.abs(kg.numpy() - ko).max() <= tol * max(1.0, np.abs(ko).max())
            assert np.abs(vg.numpy() - vo).max() <= tol * max(1.0, np.abs(vo).max())
    # one draft step with a mixed sublayer mask
    mask = synth.make_sublayer_masks(shape.n_blocks, 1, 0.5, 0.5, seed=3).numpy()[0]
    gpu.knnssd_set_skipset(mask.tolist())
    tok_g, p_g = gpu.knnssd_draft_step(first_o, len(prompt))
    row = orc.forward([first_o], len(prompt), mask)[0]
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    assert tok_g == O.argmax_lowest(row)
    assert abs(p_g - O.top1_prob(row)) <= 1e-3 * max(1e-3, O.top1_prob(row)) + 1e-6
    # verification of 5 rows: x_last + 4 "drafts" of which the first two are the model's own tokens
    ar = O.greedy_ar(O.OracleModel(shape, w), prompt, 4)
    rows_in = [ar[0], ar[1], ar[2], (ar[3] + 1) % shape.vocab, 7]
    rows_o = orc.forward(rows_in, len(prompt), None)
    j, nxt, new_len = gpu.knnssd_verify(rows_in, len(prompt))
    for r in range(5):
        ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
        assert ok, (r, err)
    targets = [O.argmax_lowest(rows_o[r]) for r in range(5)]
    assert j == O.accept_length(rows_in[1:], targets) == 2
    assert nxt == targets[2] and new_len == len(prompt) + 3
    gpu.close()


@pytest.mark.parametrize("name,max_draft,thr", [("tiny_fp32", 4, 0.0), ("tiny_fp32", 1, 0.0), ("bf16_mha", 4, 0.0),
                                                ("bf16_gqa_hd128", 8, 0.0), ("bf16_mfma_hd64", 15, 0.0),
                                                ("bf16_mfma_hd64", 3, 0.6), ("fp32_gqa", 3, 0.6)])
def test_generate_tokens_and_counts_match_oracle(name, max_draft, thr):
    shape = SHAPES[name]
    print("case", name, max_draft, thr, flush=True)
    w, orc, gpu = make_pair(shape, seed=21, std=0.05, lm_scale=(30.0 if thr > 0 else None))
    prompt = synth.make_prompt(shape.vocab, 32, seed=9).tolist()
    max_new = 32
    ar = O.greedy_ar(orc, prompt, max_new)
    for mask in [np.zeros(2 * shape.n_blocks, np.uint8)] + list(
            synth.make_block_masks(shape.n_blocks, 2, max(1, shape.n_blocks // 2), seed=4).numpy()):
        toks_o, st_o, rounds_o = O.ssd_generate(orc, prompt, mask, max_new, max_draft, thr)
        assert toks_o == ar
        gpu.knnssd_set_skipset(mask.tolist())
        toks_g, st_g = gpu.knnssd_generate(prompt, max_new, max_draft, thr)
        min_margin = min(min(r.margins) for r in rounds_o)
        assert toks_g == toks_o, f"tokens differ (oracle min top-2 margin {min_margin:.2e})"
        assert (st_g["rounds"], st_g["drafted"], st_g["accepted"], st_g["emitted"]) == \
            (st_o.rounds, st_o.drafted, st_o.accepted, st_o.emitted), f"min margin {min_margin:.2e}"
    # plain autoregressive decoding through the same entry point
    toks_ar, st_ar = gpu.knnssd_generate(prompt, max_new, 0)
    assert toks_ar == ar and st_ar["drafted"] == 0 and st_ar["rounds"] == max_new - 1
    gpu.close()


def test_knn_select_tiny_and_clustered():
    wl = synth.workload("tiny")
    w, orc, gpu = make_pair(wl.shape, seed=31, gains="ones", max_anchors=1200)
    # the tiny configuration: 8 unrelated anchors, query = the prompt's own last hidden vector
    anchors, labels, _ = synth.make_anchors(wl.shape.d_model, wl.n_anchors, wl.n_domains, 1.0, clustered=False)
    masks = synth.make_block_masks(wl.shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    prompt = synth.make_prompt(wl.shape.vocab, wl.prompt_len).tolist()
    _, hidden = gpu.knnssd_prefill(prompt)
    idx, dom, mask = gpu.knnssd_select_skipset(hidden)
    _, hidden_o, _ = O.prefill(orc, prompt)
    idx_o, dom_o, mask_o, _ = O.knn_select(hidden_o, anchors.numpy(), labels.numpy(), masks.numpy())
    assert (idx, dom, mask) == (idx_o, dom_o, mask_o.tolist())
    # random queries, ragged anchor counts (not a multiple of the wavefronts in flight)
    for n_anchors in (1, 7, 1000, 1037):
        a, l, c = synth.make_anchors(wl.shape.d_model, n_anchors, 5, 0.1, seed=50 + n_anchors)
        m = synth.make_block_masks(wl.shape.n_blocks, 5, 2, seed=8)
        gpu.knnssd_set_anchors(a, l, m)
        for s in range(6):
            q = synth.make_domain_query(c, s % 5, 0.1, seed=900 + s) if s < 5 else torch.randn(wl.shape.d_model)
            got = gpu.knnssd_select_skipset(q)
            io, do, mo, _ = O.knn_select(q.numpy(), a.numpy(), l.numpy(), m.numpy())
            assert got == (io, do, mo.tolist())
    # the whole path: prefill -> KNN on the prompt's own hidden vector -> draft/verify rounds
    gpu.knnssd_set_anchors(anchors, labels, masks)
    toks, st = gpu.knnssd_generate(prompt, wl.max_new, wl.max_draft, wl.conf_threshold)
    res = O.knnssd_generate(orc, prompt, anchors.numpy(), labels.numpy(), masks.numpy(), wl.max_new, wl.max_draft)
    assert toks == res["tokens"]
    assert (st["rounds"], st["drafted"], st["accepted"]) == (res["stats"].rounds, res["stats"].drafted, res["stats"].accepted)
    gpu.close()


def test_error_paths_on_device():
    wl = synth.workload("tiny")
    w, orc, gpu = make_pair(wl.shape, seed=41, max_anchors=16)
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_draft_step(1, 0)                      # before any prefill
    assert e.value.code == -5
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_select_skipset(torch.ones(wl.shape.d_model))   # no anchors yet
    assert e.value.code == -5
    prompt = synth.make_prompt(wl.shape.vocab, 8).tolist()
    gpu.knnssd_prefill(prompt)
    for bad in (lambda: gpu.knnssd_draft_step(wl.shape.vocab, 8), lambda: gpu.knnssd_draft_step(1, wl.shape.max_seq),
                lambda: gpu.knnssd_verify([1] * 17, 8), lambda: gpu.knnssd_verify([1, 2], wl.shape.max_seq - 1),
                lambda: gpu.knnssd_prefill([0] * (wl.shape.max_seq + 1)), lambda: gpu.knnssd_prefill([-1]),
                lambda: gpu.knnssd_generate(prompt, wl.shape.max_seq, 4),
                # positions nobody wrote: a draft step two past the prompt, a verification that starts past the cache
                lambda: gpu.knnssd_draft_step(1, 10), lambda: gpu.knnssd_verify([1, 2], 9)):
        with pytest.raises(binding.KnnSsdError) as e:
            bad()
        assert e.value.code == -3
    # ... while consecutive draft steps extend what the next one may attend to, and a verification resets it
    gpu.knnssd_draft_step(1, 8)
    gpu.knnssd_draft_step(2, 9)
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_verify([1, 2], 9)                       # the full model's cache still ends at 8
    assert e.value.code == -3
    j, nxt, new_len = gpu.knnssd_verify([1, 2, 3], 8)
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_draft_step(1, new_len + 1)
    assert e.value.code == -3
    gpu.knnssd_draft_step(1, new_len)
    anchors, labels, _ = synth.make_anchors(wl.shape.d_model, 8, 4, 1.0)
    masks = synth.make_block_masks(wl.shape.n_blocks, 4, 2)
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_set_anchors(torch.cat([anchors] * 3), torch.cat([labels] * 3), masks)   # 24 > max_anchors
    assert e.value.code == -3
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_set_anchors(anchors, labels, masks[:, :-2])     # a mask table of the wrong row length
    assert e.value.code == -2
    zero = anchors.clone()
    zero[3] = 0
    gpu.knnssd_set_anchors(zero, labels, masks)
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_select_skipset(torch.ones(wl.shape.d_model))
    assert e.value.code == -4
    gpu.knnssd_set_anchors(anchors, labels, masks)
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_select_skipset(torch.zeros(wl.shape.d_model))
    assert e.value.code == -4
    nanq = torch.ones(wl.shape.d_model)
    nanq[5] = float("nan")
    with pytest.raises(binding.KnnSsdError) as e:
        gpu.knnssd_select_skipset(nanq)
    assert e.value.code == -4
    gpu.close()
