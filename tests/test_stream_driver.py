"""Domain-shift stream (Sec. 4.2, Eq. 8): the library-side chain against the oracle's and against the
closed-form transition probabilities (CPU), and the stream driver against the oracle sample by sample (GPU)."""
import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import stream, synth


def test_chain_matches_oracle_transition_everywhere():
    for n in (1, 2, 3, 5, 8):
        for r in (0.0, 0.3, 0.7, 1.0):
            for cur in range(n):
                for us in np.linspace(0.0, 0.999, 23):
                    for up in np.linspace(0.0, 0.999999, 31):
                        assert stream.domain_after(cur, n, r, us, up) == O.next_domain(cur, n, r, us, up), (n, r, cur, us, up)


@pytest.mark.parametrize("r", [0.0, 0.3, 0.7, 1.0])
def test_chain_frequencies_follow_eq8(r):
    n, samples = 5, 40000
    seq = stream.domain_sequence(n, samples, r, seed=77, first=2)
    assert seq[0] == 2 and len(seq) == samples
    seq = np.asarray(seq)
    switches = seq[1:] != seq[:-1]
    # P(stay) = 1 - r; on a switch every other domain has probability r / (N - 1)  (Eq. 8)
    assert abs(switches.mean() - r) < 4 * np.sqrt(max(r * (1 - r), 1e-6) / samples) + 1e-9
    if r > 0:
        prev, nxt = seq[:-1][switches], seq[1:][switches]
        for k in range(n):
            sel = nxt[prev == k]
            assert not np.any(sel == k)
            counts = np.bincount(sel, minlength=n)[[j for j in range(n) if j != k]]
            expect = len(sel) / (n - 1)
            assert np.all(np.abs(counts - expect) < 5 * np.sqrt(expect) + 1)
    if r == 0.0:
        assert np.all(seq == 2)          # task-by-task stream
    if r == 1.0:
        assert switches.all()            # every two consecutive samples differ


@pytest.mark.gpu
@pytest.mark.parametrize("reselect", [True, False])
def test_stream_driver_matches_oracle_sample_by_sample(reselect):
    from paper_2505_16162_amd import binding
    from gpu_common import make_pair
    shape = synth.small_shape("stream", n_blocks=4, d_ffn=704, vocab=1100, max_seq=96)
    n_dom, n_anchor, sigma = 5, 40, 0.1
    w, orc, gpu = make_pair(shape, seed=31, std=0.05, max_anchors=n_anchor)
    anchors, labels, centres = synth.make_anchors(shape.d_model, n_anchor, n_dom, sigma, seed=5)
    masks = synth.make_block_masks(shape.n_blocks, n_dom, 2, seed=6)
    gpu.knnssd_set_anchors(anchors, labels, masks)
    domains = stream.domain_sequence(n_dom, 7, 0.7, seed=3, first=1)
    assert len(set(domains)) > 1
    prompts = [synth.make_prompt(shape.vocab, 20 + i, seed=100 + i).tolist() for i in range(len(domains))]
    queries = [synth.make_domain_query(centres, d, sigma, seed=200 + i) for i, d in enumerate(domains)]
    res = stream.run_stream(gpu, n_dom, domains, lambda i: prompts[i], lambda i, d: queries[i], max_new=12, max_draft=4,
                            conf_threshold=0.0, reselect=reselect)
    kept_mask = None
    for i, dom in enumerate(domains):
        if reselect or i == 0:
            o = O.knnssd_generate(orc, prompts[i], anchors.numpy(), labels.numpy(), masks.numpy(), 12, 4, 0.0,
                                  query=queries[i].numpy())
            kept_mask, routed, toks, st = o["mask"], o["domain"], o["tokens"], o["stats"]
            kept_domain = routed
        else:
            toks, st, _ = O.ssd_generate(orc, prompts[i], kept_mask, 12, 4, 0.0)
            routed = kept_domain
        assert res.routed[i] == routed, i
        assert res.tokens[i] == toks, i
        if reselect:
            assert routed == dom          # sigma = 0.1 clusters: the 1-NN routing finds the true domain (Sec. 5.3)
    tot = res.total
    assert tot.samples == len(domains) and tot.emitted == 12 * len(domains)
    assert sum(t.samples for t in res.per_domain.values()) == len(domains)
    assert 1.0 <= tot.mean_generated_length <= 5.0 and 0.0 <= tot.acceptance_rate <= 1.0
    gpu.close()
