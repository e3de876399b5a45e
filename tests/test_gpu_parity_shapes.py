"""GPU parity on further shapes and on the edges of the path: 7B-shaped widths, a context of several
thousand positions (many split-KV chunks, the domain-shift stream's prompt length), and the degenerate
cases of the round loop (one-token prompt, one or two tokens to generate, 16-row verification)."""
import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import binding, synth
from gpu_common import logits_close, make_pair

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(600)
def test_llama7b_widths_match_oracle():
    """7B-shaped widths (d 4096, 32 heads, FFN 11008: 43 FFN rows per workgroup, K = 11008 = 21.5 column blocks)
    at reduced depth; draft with a block mask, verification of 5 rows, a short generation."""
    s = synth.workload("llama7b").shape
    shape = synth.ModelShape("llama7b_w3", 3, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 200,
                             "bf16", "bf16")
    w = synth.make_weights(shape, device="cuda:0", seed=3)
    gpu = binding.KnnSsd(shape, w)
    orc = O.OracleModel(shape, synth.weights_to(w, "cpu"))
    prompt = synth.make_prompt(shape.vocab, 45, seed=2).tolist()
    mask = synth.make_block_masks(shape.n_blocks, 1, 1, seed=4).numpy()[0]
    print("oracle generate", flush=True)
    toks_o, st_o, rounds = O.ssd_generate(orc, prompt, mask, 12, 4, 0.0)
    gpu.knnssd_set_skipset(mask.tolist())
    print("gpu generate", flush=True)
    toks_g, st_g = gpu.knnssd_generate(prompt, 12, 4, 0.0)
    assert toks_g == toks_o, [min(r.margins) for r in rounds]
    assert (st_g["rounds"], st_g["drafted"], st_g["accepted"]) == (st_o.rounds, st_o.drafted, st_o.accepted)
    # logits: one draft step and a 5-row verification behind a fresh prefill
    orc2 = O.OracleModel(shape, synth.weights_to(w, "cpu"))
    first_o, _, _ = O.prefill(orc2, prompt)
    first_g, _ = gpu.knnssd_prefill(prompt)
    assert first_g == first_o
    gpu.knnssd_draft_step(first_o, len(prompt))
    row = orc2.forward([first_o], len(prompt), mask)[0]
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    rows_in = [first_o] + toks_o[1:5]
    rows_o = orc2.forward(rows_in, len(prompt), None)
    gpu.knnssd_verify(rows_in, len(prompt))
    for r in range(5):
        ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
        assert ok, (r, err)
    gpu.close()


@pytest.mark.timeout(900)
def test_long_context_many_kv_chunks():
    """Context of 4100+ positions (17 split-KV chunks of 256, the stream configuration's prompt length) on a
    narrow model, so that the oracle's prefill stays in seconds: draft and verification logits, cached keys
    at both ends, tokens of a short generation."""
    shape = synth.small_shape("long_ctx", n_blocks=2, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=704,
                              vocab=1200, max_seq=4200)
    w, orc, gpu = make_pair(shape, seed=8, std=0.05)
    P = 4101                                             # 256 full 16-row chunks + 5 rows; 17th KV chunk holds 5 positions
    prompt = synth.make_prompt(shape.vocab, P, seed=6).tolist()
    print("oracle prefill", flush=True)
    first_o, hidden_o, row_o = O.prefill(orc, prompt)
    print("gpu prefill", flush=True)
    first_g, hidden_g = gpu.knnssd_prefill(prompt)
    assert first_g == first_o
    ok, err = logits_close(gpu.knnssd_get_logits((P - 1) % 16).numpy(), row_o, shape)
    assert ok, err
    for pos in (0, 255, 256, 4095, 4096, 4100):
        kg, vg = gpu.knnssd_read_kv(1, pos)
        ko, vo = orc.read_kv(1, pos)
        assert np.abs(kg.numpy() - ko).max() <= 2e-2 * max(1.0, np.abs(ko).max())
        assert np.abs(vg.numpy() - vo).max() <= 2e-2 * max(1.0, np.abs(vo).max())
    mask = [0, 1, 0, 0]                                  # skip the MLP of block 0
    gpu.knnssd_set_skipset(mask)
    tok_g, _ = gpu.knnssd_draft_step(first_o, P)
    row = orc.forward([first_o], P, np.array(mask, dtype=np.uint8))[0]
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    assert tok_g == O.argmax_lowest(row)
    rows_in = [first_o, 5, 17, 1199, 0, 3, 3]
    rows_o = orc.forward(rows_in, P, None)
    gpu.knnssd_verify(rows_in, P)
    for r in range(len(rows_in)):
        ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
        assert ok, (r, err)
    gpu.close()


def test_round_loop_edges():
    """One-token prompt; max_new of 1 (nothing after the prefill's token), 2 (one verification of one row) and 3;
    16-row verification (15 drafts); a generation that ends exactly at max_seq."""
    shape = synth.small_shape("edges", d_ffn=704, vocab=900, max_seq=64)
    w, orc, gpu = make_pair(shape, seed=13, std=0.05)
    mask = synth.make_block_masks(shape.n_blocks, 1, 1, seed=2).numpy()[0]
    gpu.knnssd_set_skipset(mask.tolist())
    for prompt_len, max_new, max_draft in ((1, 1, 4), (1, 2, 4), (1, 3, 4), (5, 20, 15), (7, 17, 1), (16, 33, 15)):
        prompt = synth.make_prompt(shape.vocab, prompt_len, seed=prompt_len).tolist()
        print("case", prompt_len, max_new, max_draft, flush=True)
        o = O.OracleModel(shape, w)
        toks_o, st_o, rounds = O.ssd_generate(o, prompt, mask, max_new, max_draft, 0.0)
        toks_g, st_g = gpu.knnssd_generate(prompt, max_new, max_draft, 0.0)
        assert toks_g == toks_o, (prompt_len, max_new, max_draft, [min(r.margins) for r in rounds if r.margins])
        assert len(toks_g) == max_new
        assert (st_g["rounds"], st_g["drafted"], st_g["accepted"]) == (st_o.rounds, st_o.drafted, st_o.accepted)
    # the generation may use the cache up to its last position but not beyond: prompt + max_new + max_draft <= max_seq
    prompt = synth.make_prompt(shape.vocab, 40, seed=1).tolist()
    toks_g, _ = gpu.knnssd_generate(prompt, 20, 4, 0.0)          # 40 + 20 + 4 = 64 = max_seq
    toks_o, _, _ = O.ssd_generate(O.OracleModel(shape, w), prompt, mask, 20, 4, 0.0)
    assert toks_g == toks_o
    with pytest.raises(binding.KnnSsdError):
        gpu.knnssd_generate(prompt, 21, 4, 0.0)
    gpu.close()


@pytest.mark.timeout(600)
def test_many_rows_long_k_many_activation_chunks():
    """Verification of 16, 11 and 6 rows on a shape whose reduction lengths (2048 and 3072 columns) make the
    matrix-core GEMM stage its token rows in four to six chunks: the launches take the variant whose weight
    stream runs on across chunk boundaries. Its logits must equal, bit for bit, those of the same rows verified
    alone (one chunk, the other variant), and match the oracle."""
    shape = synth.small_shape("long_k", n_blocks=2, d_model=2048, n_heads=16, n_kv_heads=16, head_dim=128,
                              d_ffn=3072, vocab=2500, max_seq=80)
    w, orc, gpu = make_pair(shape, seed=17, std=0.02)
    prompt = synth.make_prompt(shape.vocab, 21, seed=3).tolist()
    first_o, _, _ = O.prefill(orc, prompt)
    first_g, _ = gpu.knnssd_prefill(prompt)
    assert first_g == first_o
    rows_in = [first_o] + synth.make_prompt(shape.vocab, 15, seed=8).tolist()
    rows_o = orc.forward(rows_in, len(prompt), None)
    kept = {}
    for n in (16, 11, 6):
        print("rows", n, flush=True)
        gpu.knnssd_prefill(prompt)
        gpu.knnssd_verify(rows_in[:n], len(prompt))
        for r in range(n):
            got = gpu.knnssd_get_logits(r).clone()
            ok, err = logits_close(got.numpy(), rows_o[r], shape)
            assert ok, (n, r, err)
            if r in kept:
                assert torch.equal(got, kept[r]), (n, r)     # independent of how many rows share the pass
            kept[r] = got
    # the same rows one at a time: a single chunk per launch, i.e. the other kernel variant
    gpu.knnssd_prefill(prompt)
    for r in range(3):
        gpu.knnssd_verify(rows_in[r:r + 1], len(prompt) + r)
        assert torch.equal(gpu.knnssd_get_logits(0), kept[r]), r
    gpu.close()


def test_fewer_rows_than_workgroups():
    """d_model = 128: the output projections have 128 rows for 256 workgroups, so every other workgroup owns no row
    of them (it still stages its share of the activations and meets the others); QKV and gate/up shares of 0-2 rows.
    Draft steps, 1-, 5- and 16-row verification, a generation."""
    shape = synth.small_shape("narrow", n_blocks=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, d_ffn=352,
                              vocab=700, max_seq=96)
    w, orc, gpu = make_pair(shape, seed=29, std=0.06)
    assert gpu.packed                                   # the tuned kernels, not the any-shape fallback
    prompt = synth.make_prompt(shape.vocab, 19, seed=12).tolist()
    mask = np.array([0, 1, 0, 0], dtype=np.uint8)
    toks_o, st_o, rounds = O.ssd_generate(orc, prompt, mask, 24, 6, 0.0)
    gpu.knnssd_set_skipset(mask.tolist())
    toks_g, st_g = gpu.knnssd_generate(prompt, 24, 6, 0.0)
    assert toks_g == toks_o, [min(r.margins) for r in rounds if r.margins]
    assert (st_g["rounds"], st_g["drafted"], st_g["accepted"]) == (st_o.rounds, st_o.drafted, st_o.accepted)
    orc2 = O.OracleModel(shape, w)
    first_o, _, _ = O.prefill(orc2, prompt)
    first_g, _ = gpu.knnssd_prefill(prompt)
    assert first_g == first_o
    gpu.knnssd_draft_step(first_o, len(prompt))
    row = orc2.forward([first_o], len(prompt), mask)[0]
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    rows_in = [first_o] + synth.make_prompt(shape.vocab, 15, seed=5).tolist()
    rows_o = orc2.forward(rows_in, len(prompt), None)
    for n in (1, 5, 16):
        gpu.knnssd_verify(rows_in[:n], len(prompt))
        for r in range(n):
            ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
            assert ok, (n, r, err)
    gpu.close()


@pytest.mark.parametrize("plen", [283, 250])
@pytest.mark.parametrize("kernel", ["mfma", "valu"])
@pytest.mark.parametrize("gqa", [False, True])
def test_verification_attention_kernels(kernel, gqa, plen):
    """Both split-KV attention kernels of the verification pass (matrix cores / vector ALUs; the library uses the first
    unless cfg.verify_attn names the other) on a multi-head and a grouped-query shape: 1, 3, 9 and 16 rows behind
    a prompt that spans two 256-position chunks (283 positions), or that ends just before the chunk boundary (250: the
    first rows of the pass see one chunk, the later ones two), logits against the oracle, and rows independent of the
    row count."""
    shape = synth.small_shape("va_gqa" if gqa else "va_mha", n_blocks=2, d_model=512, n_heads=8, n_kv_heads=2 if gqa else 8,
                              head_dim=64, d_ffn=1408, vocab=900, max_seq=320)
    w, orc, gpu = make_pair(shape, seed=31, std=0.04, verify_attn=kernel)
    prompt = synth.make_prompt(shape.vocab, plen, seed=2).tolist()
    first_o, _, _ = O.prefill(orc, prompt)
    first_g, _ = gpu.knnssd_prefill(prompt)
    assert first_g == first_o
    rows_in = [first_o] + synth.make_prompt(shape.vocab, 15, seed=4).tolist()
    rows_o = orc.forward(rows_in, len(prompt), None)
    kept = {}
    for n in (16, 9, 3, 1):
        gpu.knnssd_prefill(prompt)
        gpu.knnssd_verify(rows_in[:n], len(prompt))
        for r in range(n):
            got = gpu.knnssd_get_logits(r).clone()
            ok, err = logits_close(got.numpy(), rows_o[r], shape)
            assert ok, (kernel, gqa, n, r, err)
            if r in kept:
                assert torch.equal(got, kept[r]), (kernel, gqa, n, r)
            kept[r] = got
    gpu.close()


def test_tile_counts_of_three_five_and_six_per_workgroup():
    """Shares of 33-48, 65-80 and 81-96 matrix rows per workgroup (3, 5 and 6 tiles of 16): three tiles run on three
    of four tile lanes in one round; five or six take two rounds whose second keeps at most half of the lanes busy,
    so the verification GEMM sums both rounds after its loop without a meeting in between. QKV has 48 rows per
    workgroup here, gate/up 88, the LM head 79. Draft step, verification rows (also bit-identical across row counts)
    and a generation against the oracle."""
    shape = synth.small_shape("tiles356", n_blocks=2, d_model=256, n_heads=64, n_kv_heads=64, head_dim=64,
                              d_ffn=11264, vocab=20000, max_seq=64)
    w, orc, gpu = make_pair(shape, seed=41, std=0.03)
    assert gpu.packed
    prompt = synth.make_prompt(shape.vocab, 21, seed=3).tolist()
    first_o, _, _ = O.prefill(orc, prompt)
    first_g, _ = gpu.knnssd_prefill(prompt)
    assert first_g == first_o
    mask = np.array([0, 0, 1, 0], dtype=np.uint8)
    gpu.knnssd_set_skipset(mask.tolist())
    gpu.knnssd_draft_step(first_o, len(prompt))
    row = orc.forward([first_o], len(prompt), mask)[0]
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    rows_in = [first_o] + synth.make_prompt(shape.vocab, 15, seed=9).tolist()
    rows_o = orc.forward(rows_in, len(prompt), None)
    kept = {}
    for n in (16, 2, 1):
        gpu.knnssd_prefill(prompt)
        gpu.knnssd_verify(rows_in[:n], len(prompt))
        for r in range(n):
            got = gpu.knnssd_get_logits(r).clone()
            ok, err = logits_close(got.numpy(), rows_o[r], shape)
            assert ok, (n, r, err)
            if r in kept:
                assert torch.equal(got, kept[r]), (n, r)
            kept[r] = got
    orc2 = O.OracleModel(shape, w)
    toks_o, st_o, rounds = O.ssd_generate(orc2, prompt, mask, 12, 4, 0.0)
    gpu.knnssd_set_skipset(mask.tolist())
    toks_g, st_g = gpu.knnssd_generate(prompt, 12, 4, 0.0)
    assert toks_g == toks_o, [min(r.margins) for r in rounds if r.margins]
    gpu.close()


@pytest.mark.parametrize("gqa", [False, True])
def test_merge_inside_the_attention_launch(gqa):
    """With few (row, head) pairs per kv head the attention launch merges its own chunks (cfg.attn_merge =
    KNNSSD_MERGE_FUSED, the default: the workgroup that finishes a group's last chunk does it); the same steps with the
    merge as a launch of its own (KNNSSD_MERGE_SEPARATE) must give the same bits, at one, two, six, seven and nine chunks,
    for draft steps (vector-ALU kernel, or the matrix-core one with grouped-query heads) and for verification passes of
    1 to 16 rows (at the last context, 2100 positions = nine chunks, more than four pairs per kv head keep the launch;
    the rows are compared between the two contexts only), and the draft steps are checked against the oracle."""
    shape = synth.small_shape("fuse_gqa" if gqa else "fuse_mha", n_blocks=2, d_model=512, n_heads=8, n_kv_heads=2 if gqa else 8,
                              head_dim=64, d_ffn=1408, vocab=900, max_seq=2200)
    w, orc, gpu = make_pair(shape, seed=37, std=0.04)
    gpu2 = binding.KnnSsd(shape, w, separate_merge=True)
    mask = [0, 1, 0, 0]
    for plen in (37, 283, 1300, 1600, 2100):         # 2100: past the context up to which the launch merges itself
        print("case", gqa, plen, flush=True)
        prompt = synth.make_prompt(shape.vocab, plen, seed=2).tolist()
        first_o, _, _ = O.prefill(orc, prompt)
        for g in (gpu, gpu2):
            assert g.knnssd_prefill(prompt)[0] == first_o
            g.knnssd_set_skipset(mask)
        tok, rows = first_o, []
        for i in range(3):                                   # consecutive steps: each reads what the one before wrote
            t1, p1 = gpu.knnssd_draft_step(tok, plen + i)
            t2, p2 = gpu2.knnssd_draft_step(tok, plen + i)
            l1, l2 = gpu.knnssd_get_logits(0).clone(), gpu2.knnssd_get_logits(0).clone()
            assert torch.equal(l1, l2), (plen, i)
            assert (t1, p1) == (t2, p2)
            row = orc.forward([tok], plen + i, np.asarray(mask, np.uint8))[0]
            ok, err = logits_close(l1.numpy(), row, shape)
            assert ok, (plen, i, err)
            assert t1 == O.argmax_lowest(row)
            tok = t1
    # verification rows on the three contexts (the matrix-core kernel merges one- and three-row passes itself unless
    # the merge is a launch of its own)
    rows_in = [first_o] + synth.make_prompt(shape.vocab, 15, seed=8).tolist()
    for vlen in (283, 1300, 2100):        # two, six and nine chunks
        vprompt = synth.make_prompt(shape.vocab, vlen, seed=2).tolist()
        for n in (1, 3, 5, 9, 16):        # 9 and 16 rows: whole tiles of pairs, merged four items per thread
            print("verify case", gqa, vlen, n, flush=True)
            got = []
            for g in (gpu, gpu2):
                g.knnssd_prefill(vprompt)
                g.knnssd_verify(rows_in[:n], vlen)
                got.append([g.knnssd_get_logits(r).clone() for r in range(n)])
            for r in range(n):
                assert torch.equal(got[0][r], got[1][r]), (vlen, n, r)
    gpu.close()
    gpu2.close()


@pytest.mark.parametrize("hd", [64, 128])
def test_merge_inside_the_attention_launch_up_to_24_chunks(hd):
    """The matrix-core kernel's build for long contexts merges its own chunks up to 24 of them (6144 positions) in one
    batch of loads; one position further the merge is a launch of its own. Draft steps and 1- to 4-row verification
    passes around that edge and at 9 and 17 chunks, fused against separate merge, bit for bit (the separate merge is
    the one the oracle comparisons at long contexts run)."""
    shape = synth.small_shape("edge24_%d" % hd, n_blocks=2, d_model=256, n_heads=4, n_kv_heads=2, head_dim=hd, d_ffn=704,
                              vocab=900, max_seq=6200)
    w = synth.make_weights(shape, seed=41, gains="random", std=0.05)
    gpu = binding.KnnSsd(shape, w)
    gpu2 = binding.KnnSsd(shape, w, separate_merge=True)
    mask = [0, 1, 0, 0]
    rows_in = synth.make_prompt(shape.vocab, 4, seed=3).tolist()
    for plen in (2300, 4200, 6139, 6141, 6144):      # 9 and 17 chunks; 24 chunks exactly, then across the edge
        print("case", hd, plen, flush=True)
        prompt = synth.make_prompt(shape.vocab, plen, seed=2).tolist()
        firsts = []
        for g in (gpu, gpu2):
            firsts.append(g.knnssd_prefill(prompt)[0])
            g.knnssd_set_skipset(mask)
        assert firsts[0] == firsts[1]
        tok = firsts[0]
        for i in range(4):                                   # the steps walk over the edge
            r1, r2 = gpu.knnssd_draft_step(tok, plen + i), gpu2.knnssd_draft_step(tok, plen + i)
            assert r1 == r2, (plen, i)
            assert torch.equal(gpu.knnssd_get_logits(0), gpu2.knnssd_get_logits(0)), (plen, i)
            tok = r1[0]
        for n in (1, 2, 4):
            got = []
            for g in (gpu, gpu2):
                g.knnssd_prefill(prompt)
                res = g.knnssd_verify([firsts[0]] + rows_in[:n - 1], plen)
                got.append((res, [g.knnssd_get_logits(r).clone() for r in range(n)]))
            assert got[0][0] == got[1][0], (plen, n)
            for r in range(n):
                assert torch.equal(got[0][1][r], got[1][1][r]), (plen, n, r)
    gpu.close()
    gpu2.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("hd,heads,kv_heads,plen,row_counts", [(64, 32, 32, 4101, (2, 9)), (128, 32, 8, 6200, (9, 2))])
def test_attention_with_more_work_items_than_workgroups(hd, heads, kv_heads, plen, row_counts):
    """Many heads on a long context: a verification pass brings more (pair tile, kv head, 256-position chunk) items
    than the matrix-core attention launch has workgroups (32 kv heads x 17 chunks; 3 pair tiles x 8 kv heads x 25
    chunks), so workgroups run several items one after the other, with the padding slots of the item order in
    between; the 2-row pass of the grouped-query shape has fewer items than workgroups. Logits against the oracle."""
    shape = synth.small_shape("items%d" % hd, n_blocks=1, d_model=256, n_heads=heads, n_kv_heads=kv_heads, head_dim=hd,
                              d_ffn=704, vocab=1200, max_seq=plen + 40)
    w, orc, gpu = make_pair(shape, seed=8, std=0.05)
    prompt = synth.make_prompt(shape.vocab, plen, seed=6).tolist()
    print("oracle prefill of", plen, "rows,", heads, "heads", flush=True)
    first_o, _, _ = O.prefill(orc, prompt)
    assert gpu.knnssd_prefill(prompt)[0] == first_o
    rows_in = [first_o] + synth.make_prompt(shape.vocab, 8, seed=12).tolist()
    for n in row_counts:
        print("case", hd, plen, n, flush=True)
        j, nxt, new_len = gpu.knnssd_verify(rows_in[:n], plen)
        rows_o = orc.forward(rows_in[:n], plen, None)
        for r in range(n):
            ok, err = logits_close(gpu.knnssd_get_logits(r).numpy(), rows_o[r], shape)
            assert ok, (n, r, err)
        targets = [O.argmax_lowest(rows_o[r]) for r in range(n)]
        assert j == O.accept_length(rows_in[1:n], targets) and nxt == targets[j] and new_len == plen + j + 1
    # a draft step at that context: with one pair per kv head and that many items it runs on the matrix-core kernel too
    mask = [0, 1]
    gpu.knnssd_prefill(prompt)
    gpu.knnssd_set_skipset(mask)
    tok, p = gpu.knnssd_draft_step(first_o, plen)
    row = orc.forward([first_o], plen, np.asarray(mask, np.uint8))[0]
    ok, err = logits_close(gpu.knnssd_get_logits(0).numpy(), row, shape)
    assert ok, err
    assert tok == O.argmax_lowest(row) and abs(p - O.top1_prob(row)) <= 1e-2 * O.top1_prob(row)
    gpu.close()


def test_two_identical_runs_give_identical_bits():
    """Run-to-run determinism of the tuned kernels (no atomics, fixed reduction orders): the same prefill, draft
    steps, verification passes and generation twice on one context, and once more on a second context built from
    the same weights; logits, cached keys/values, tokens and counters must be identical bit for bit."""
    shape = synth.small_shape("det", n_blocks=3, d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1408, vocab=1531,
                              max_seq=400)
    w = synth.make_weights(shape, seed=51, gains="random", std=0.05)
    prompt = synth.make_prompt(shape.vocab, 283, seed=6).tolist()
    mask = synth.make_block_masks(shape.n_blocks, 1, 1, seed=9).numpy()[0].tolist()

    def run(gpu):
        out = {}
        first, hidden = gpu.knnssd_prefill(prompt)
        out["first"], out["hidden"] = first, hidden.cpu().clone()
        out["kv"] = [torch.cat(gpu.knnssd_read_kv(b, p)) for b in range(shape.n_blocks) for p in (0, 100, 271, 272, 282)]
        gpu.knnssd_set_skipset(mask)
        tok, drafts = first, []
        for i in range(4):
            tok, p = gpu.knnssd_draft_step(tok, len(prompt) + i)
            drafts.append((tok, p, gpu.knnssd_get_logits(0).clone()))
        out["drafts"] = drafts
        out["verify"] = gpu.knnssd_verify([first] + [d[0] for d in drafts], len(prompt))
        out["vlogits"] = [gpu.knnssd_get_logits(r).clone() for r in range(5)]
        toks, st = gpu.knnssd_generate(prompt, 40, 6, 0.0, route=False)
        out["gen"] = (toks, st["rounds"], st["drafted"], st["accepted"])
        return out

    def same(a, b):
        assert a["first"] == b["first"] and torch.equal(a["hidden"], b["hidden"])
        assert all(torch.equal(x, y) for x, y in zip(a["kv"], b["kv"]))
        for (t1, p1, l1), (t2, p2, l2) in zip(a["drafts"], b["drafts"]):
            assert t1 == t2 and p1 == p2 and torch.equal(l1, l2)
        assert a["verify"] == b["verify"]
        assert all(torch.equal(x, y) for x, y in zip(a["vlogits"], b["vlogits"]))
        assert a["gen"] == b["gen"]

    gpu = binding.KnnSsd(shape, w)
    assert gpu.packed
    r1 = run(gpu)
    r2 = run(gpu)
    same(r1, r2)
    gpu2 = binding.KnnSsd(shape, w)
    same(r1, run(gpu2))
    gpu.close()
    gpu2.close()
