"""K > 1 nearest anchors with a majority vote, batched queries: oracle pins (CPU) and GPU parity."""
import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import synth


def _table(n, d, n_dom, seed, sigma=0.3):
    anchors, labels, centres = synth.make_anchors(d, n, n_dom, sigma, seed=seed)
    return anchors, labels, centres


def test_k1_is_the_routing_argmax():
    anchors, labels, centres = _table(200, 64, 5, seed=1)
    masks = np.zeros((5, 8), dtype=np.uint8)
    for i in range(20):
        q = synth.make_domain_query(centres, i % 5, 0.3, seed=50 + i).numpy()
        n_star, dom, _, _ = O.knn_select(q, anchors.numpy(), labels.numpy(), masks)
        order, cos, d1 = O.knn_topk_vote(q, anchors.numpy(), labels.numpy(), 1)
        assert order == [n_star] and d1 == dom


def test_topk_against_brute_force_and_planted_neighbours():
    rng = np.random.default_rng(3)
    anchors = rng.standard_normal((40, 16))
    labels = np.arange(40) % 4
    q = rng.standard_normal(16)
    # brute force written out: cosine of every pair, full sort
    cos = [float(np.dot(q, a) / (np.linalg.norm(q) * np.linalg.norm(a))) for a in anchors]
    want = sorted(range(40), key=lambda n: (-np.float32(cos[n]), n))[:7]
    order, scores, _ = O.knn_topk_vote(q, anchors, labels, 7)
    assert order == want
    assert np.allclose(scores, [cos[n] for n in want], atol=1e-12)
    assert all(scores[i] >= scores[i + 1] for i in range(6))
    # planted: three anchors are positive multiples of the query -> cosine 1, index order among them
    anchors[[31, 5, 17]] = np.outer([2.0, 0.5, 7.0], q)
    order, scores, _ = O.knn_topk_vote(q, anchors, labels, 3)
    assert order == [5, 17, 31] and np.allclose(scores, 1.0)


def test_vote_rule():
    q = np.array([1.0, 0.0])
    # ranked by cosine: anchors 0,1,2,3,4 with labels B A A B C
    ang = [0.01, 0.02, 0.03, 0.04, 0.05]
    anchors = np.array([[np.cos(t), np.sin(t)] for t in ang])
    labels = np.array([1, 0, 0, 1, 2])
    assert O.knn_topk_vote(q, anchors, labels, 1)[2] == 1
    assert O.knn_topk_vote(q, anchors, labels, 3)[2] == 0          # A has two of three
    assert O.knn_topk_vote(q, anchors, labels, 2)[2] == 1          # one each: the better-ranked label
    assert O.knn_topk_vote(q, anchors, labels, 4)[2] == 1          # two each: B's best anchor ranks first
    assert O.knn_topk_vote(q, anchors, labels, 5)[2] == 1


@pytest.mark.gpu
@pytest.mark.parametrize("n,k,nq", [(40, 1, 1), (777, 3, 5), (777, 16, 4), (5000, 8, 9)])
def test_gpu_topk_matches_oracle(n, k, nq):
    from paper_2505_16162_amd import binding
    from gpu_common import make_pair
    shape = synth.small_shape("knnk", d_ffn=704, max_seq=64)
    n_dom = 5
    w, orc, gpu = make_pair(shape, seed=2, max_anchors=n)
    anchors, labels, centres = _table(n, shape.d_model, n_dom, seed=9)
    masks = synth.make_block_masks(shape.n_blocks, n_dom, 1, seed=6)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    queries = torch.stack([synth.make_domain_query(centres, i % n_dom, 0.3, seed=300 + i) for i in range(nq)])
    idx, cos, dom = gpu.knnssd_knn_topk(queries, k)
    for i in range(nq):
        order, scores, d = O.knn_topk_vote(queries[i].numpy(), anchors.numpy(), labels.numpy(), k)
        # fp32 sums on the GPU against fp64 in the oracle: the ranking is unique wherever neighbouring scores differ
        # by more than the rounding error, which seeded Gaussian data satisfies with a wide margin
        assert idx[i] == order, (i, idx[i], order)
        assert np.allclose(cos[i], scores, atol=2e-6)
        assert dom[i] == d
    # the K = 1 result is the routing call's
    a1, d1, _ = gpu.knnssd_select_skipset(queries[0])
    assert [a1] == gpu.knnssd_knn_topk(queries[:1], 1)[0][0] and d1 == gpu.knnssd_knn_topk(queries[:1], 1)[2][0]
    with pytest.raises(binding.KnnSsdError):
        gpu.knnssd_knn_topk(queries, 17)
    with pytest.raises(binding.KnnSsdError):
        gpu.knnssd_knn_topk(torch.zeros_like(queries), k)      # zero-norm query
    gpu.close()


@pytest.mark.gpu
@pytest.mark.parametrize("n,k", [(16, 16), (20, 16), (70, 5), (3000, 16), (9000, 7)])
def test_gpu_topk_ties_short_tables_and_bad_anchors(n, k):
    """The selection's own edges: exact ties (every anchor stored several times, so equal scores must come out lowest
    index first, across the lanes, wavefronts and slices that rank parts of the table), tables shorter than a
    wavefront's share or than K allows to be dropped, and a non-finite anchor anywhere in the table."""
    from paper_2505_16162_amd import binding
    from gpu_common import make_pair
    shape = synth.small_shape("knnties", d_ffn=704, max_seq=64)
    n_dom = 4
    w, orc, gpu = make_pair(shape, seed=2, max_anchors=n)
    base, _, centres = _table((n + 3) // 4, shape.d_model, n_dom, seed=11)
    # copies of one anchor sit a quarter of the table apart (different lanes, wavefronts, slices); scaled copies have
    # the same cosine up to rounding only, so the copies are exact
    anchors = torch.cat([base, base, base, base])[:n].contiguous()
    labels = (torch.arange(n) % n_dom).to(torch.int32)
    masks = synth.make_block_masks(shape.n_blocks, n_dom, 1, seed=6)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    queries = torch.stack([synth.make_domain_query(centres, i % n_dom, 0.3, seed=40 + i) for i in range(4)])
    idx, cos, dom = gpu.knnssd_knn_topk(queries, k)
    for i in range(4):
        order, scores, d = O.knn_topk_vote(queries[i].numpy(), anchors.numpy(), labels.numpy(), k)
        assert idx[i] == order, (i, idx[i], order)
        assert np.allclose(cos[i], scores, atol=2e-6)
        assert dom[i] == d
    a1, d1, _ = gpu.knnssd_select_skipset(queries[1])
    assert a1 == idx[1][0]
    bad = anchors.clone()
    bad[n - 1, 3] = float("nan")
    gpu.knnssd_set_anchors(bad, labels, masks)
    with pytest.raises(binding.KnnSsdError):
        gpu.knnssd_knn_topk(queries, min(k, 2))
    with pytest.raises(binding.KnnSsdError):
        gpu.knnssd_select_skipset(queries[0])
    gpu.close()


@pytest.mark.gpu
@pytest.mark.timeout(600)
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gpu_scan_of_a_large_table_matches_oracle(dtype):
    """The regime in which the scan is bound by HBM: 100 000 anchors of dimension 5120 (2 GB in fp32, 1 GB in bf16),
    the routing arg-max and the 8 nearest with their vote against the exhaustive oracle. A bf16 table is rounded
    once by the caller; both sides then search the same rounded values."""
    from paper_2505_16162_amd import binding
    n, d, n_dom, k = 100_000, 5120, 5, 8
    shape = synth.small_shape("knn_big", n_blocks=1, d_model=d, n_heads=40, n_kv_heads=40, head_dim=128, d_ffn=1024,
                              vocab=1024, max_seq=64)
    w = synth.make_weights(shape, device="cuda:0", seed=3)
    gpu = binding.KnnSsd(shape, w, max_anchors=n)
    print("anchors", flush=True)
    # sigma 1: neighbouring scores are well apart (a table of near-duplicates would make the ranking a coin toss)
    anchors, labels, centres = synth.make_anchors(d, n, n_dom, 1.0, seed=21, device="cuda:0")
    if dtype == "bf16":
        anchors = anchors.to(torch.bfloat16)
    masks = synth.make_block_masks(shape.n_blocks, n_dom, 1, seed=6)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    a64 = anchors.float().cpu().numpy()          # the stored values, exactly
    lab = labels.cpu().numpy()
    queries = torch.stack([synth.make_domain_query(centres.cpu(), i % n_dom, 1.0, seed=700 + i) for i in range(3)])
    print("gpu", flush=True)
    idx, cos, dom = gpu.knnssd_knn_topk(queries, k)
    for i in range(3):
        print("oracle query", i, flush=True)
        order, scores, dvote = O.knn_topk_vote(queries[i].numpy(), a64, lab, k)
        gaps = [scores[r] - scores[r + 1] for r in range(k - 1)]
        assert idx[i] == order, (i, idx[i], order, min(gaps))
        assert np.allclose(cos[i], scores, atol=3e-6)
        assert dom[i] == dvote
        n_star, d_star, mask, _ = O.knn_select(queries[i].numpy(), a64, lab, masks.numpy())
        a1, d1, m1 = gpu.knnssd_select_skipset(queries[i])
        assert (a1, d1, m1) == (n_star, d_star, mask.tolist())
    gpu.close()
