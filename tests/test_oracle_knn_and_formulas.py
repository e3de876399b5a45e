"""Pins for the oracle's KNN routing, accept rule and report-side closed forms (CPU only).

Each test ties the oracle to something outside itself: a brute-force search, an
invariance the cosine measure must have, a value the paper prints, or a limit
the formula must reach.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import knnssd_oracle as O
from paper_2505_16162_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Eq. 4-6: KNN routing

def _brute_force_nearest(query, anchors):
    """Exhaustive search written with python floats and an explicit full sort."""
    q = [float(x) for x in query]
    qn = math.sqrt(math.fsum(x * x for x in q))
    scored = []
    for n, a in enumerate(anchors):
        a = [float(x) for x in a]
        an = math.sqrt(math.fsum(x * x for x in a))
        cos = math.fsum(x * y for x, y in zip(q, a)) / (qn * an)
        scored.append((-cos, n))
    scored.sort()           # largest cosine first, lowest index first among equals
    return scored[0][1], -scored[0][0]


def test_knn_equals_exhaustive_sort_on_tiny_inputs():
    rng = np.random.default_rng(7)
    for trial in range(20):
        n, d = int(rng.integers(1, 9)), int(rng.integers(2, 40))
        anchors = rng.standard_normal((n, d)).astype(np.float32)
        query = rng.standard_normal(d).astype(np.float32)
        labels = np.arange(n, dtype=np.int32)
        masks = rng.integers(0, 2, size=(n, 6)).astype(np.uint8)
        idx, dom, mask, scores = O.knn_select(query, anchors, labels, masks)
        want, want_cos = _brute_force_nearest(query, anchors)
        assert idx == want and dom == want
        assert abs(scores[idx] - want_cos) < 1e-12
        assert (mask == masks[want]).all()


def test_knn_tiny_config_matches_brute_force():
    wl = synth.workload("tiny")
    anchors, labels, _ = synth.make_anchors(wl.shape.d_model, wl.n_anchors, wl.n_domains, 1.0, clustered=False)
    masks = synth.make_block_masks(wl.shape.n_blocks, wl.n_domains, wl.skipped_blocks)
    rng = np.random.default_rng(3)
    for _ in range(10):
        q = rng.standard_normal(wl.shape.d_model).astype(np.float32)
        idx, dom, mask, _ = O.knn_select(q, anchors.numpy(), labels.numpy(), masks.numpy())
        assert idx == _brute_force_nearest(q, anchors.numpy())[0]
        assert dom == int(labels[idx]) and (mask == masks[dom].numpy()).all()
        assert mask.sum() == 2 * wl.skipped_blocks


def test_knn_planted_query_has_cosine_one():
    rng = np.random.default_rng(11)
    anchors = rng.standard_normal((50, 64)).astype(np.float32)
    labels = (np.arange(50) % 5).astype(np.int32)
    masks = np.eye(5, 8, dtype=np.uint8)
    for n in (0, 17, 49):
        idx, dom, _, scores = O.knn_select(3.7 * anchors[n], anchors, labels, masks)
        assert idx == n and dom == n % 5
        assert abs(scores[n] - 1.0) < 1e-12
        assert scores.max() <= 1.0 + 1e-12


def test_knn_invariances_scale_and_permutation():
    rng = np.random.default_rng(5)
    anchors = rng.standard_normal((40, 32)).astype(np.float32)
    labels = (np.arange(40) % 4).astype(np.int32)
    masks = np.zeros((4, 4), np.uint8)
    q = rng.standard_normal(32).astype(np.float32)
    idx, _, _, _ = O.knn_select(q, anchors, labels, masks)
    # cosine ignores positive rescaling of the query and of any single anchor
    assert O.knn_select(4.0 * q, anchors, labels, masks)[0] == idx
    scaled = anchors.copy()
    scaled[::3] *= 8.0
    scaled[1::3] *= 0.125
    assert O.knn_select(q, scaled, labels, masks)[0] == idx
    # cosine, not Euclidean distance: the far anchor that points the query's way must win
    two = np.array([[10.0, 0.0], [1.0, 0.5]], np.float32)
    qq = np.array([1.0, 0.1], np.float32)
    assert int(np.argmin(((two - qq) ** 2).sum(1))) == 1
    assert O.knn_select(qq, two, np.array([0, 1], np.int32), np.zeros((2, 2), np.uint8))[0] == 0
    # permuting the anchors permutes the answer
    perm = rng.permutation(40)
    pidx = O.knn_select(q, anchors[perm], labels[perm], masks)[0]
    assert perm[pidx] == idx
    # negating the query sends the arg-max to the arg-min
    s = O.cosine_scores(q, anchors)
    assert O.knn_select(-q, anchors, labels, masks)[0] == int(np.argmin(s))


def test_knn_tie_goes_to_lowest_index():
    a = np.array([[1, 0], [0, 1], [2, 0], [1, 0]], np.float32)
    idx, dom, _, _ = O.knn_select(np.array([5, 0], np.float32), a, np.array([3, 2, 1, 0], np.int32),
                                  np.zeros((4, 2), np.uint8))
    assert idx == 0 and dom == 3


def test_knn_degenerate_vectors_are_errors():
    a = np.array([[1, 0], [0, 0]], np.float32)
    with pytest.raises(ValueError):
        O.cosine_scores(np.array([1, 1], np.float32), a)
    with pytest.raises(ValueError):
        O.cosine_scores(np.zeros(2, np.float32), np.ones((2, 2), np.float32))


@pytest.mark.parametrize("dim,n_anchors", [(256, 100), (4096, 1000)])
def test_well_separated_clusters_classify_perfectly(dim, n_anchors):
    """Sec. 5.3 reports 100 % routing accuracy for separated domains; synthetic clusters with
    sigma = 0.1 round N(0, I) centres are far better separated, so every query must come back
    with its own domain's label."""
    anchors, labels, centres = synth.make_anchors(dim, n_anchors, 5, 0.1, seed=99)
    masks = synth.make_block_masks(8, 5, 4)
    for s in range(25):
        dom = s % 5
        q = synth.make_domain_query(centres, dom, 0.1, seed=1000 + s)
        idx, got, mask, _ = O.knn_select(q.numpy(), anchors.numpy(), labels.numpy(), masks.numpy())
        assert got == dom and int(labels[idx]) == dom
        assert (mask == masks[dom].numpy()).all()


# ------------------------------------------------------------------ accept rule (verification paragraph of Sec. 4.2)

def test_accept_length_brute_force():
    for k in range(0, 5):
        for drafts in itertools.product(range(3), repeat=k):
            for targets in itertools.product(range(3), repeat=k + 1):
                j = O.accept_length(list(drafts), list(targets))
                # definition: largest j such that every one of the first j drafts matches
                want = max(i for i in range(k + 1) if all(drafts[m] == targets[m] for m in range(i)))
                assert j == want


# ------------------------------------------------------------------ Eq. 9-11

def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(x) for x in line.split()])
    return rows


def test_eq11_worked_example_from_paper():
    refined, plain = _read_golden("eq11_worked_example.txt")
    s_mlp, s_attn, beta, c_printed = refined
    assert round(O.cost_coefficient(s_mlp, s_attn, beta), 3) == c_printed
    s, c_plain = plain
    # beta = 1 with equal ratios reduces to 1 - s, the value printed for the unrefined formula
    assert abs(O.cost_coefficient(s, s, 1.0) - c_plain) < 1e-12
    # with beta = 1 the refined cost is 1 - (average of the two ratios)
    assert abs(O.cost_coefficient(s_mlp, s_attn, 1.0) - (1 - (s_mlp + s_attn) / 2)) < 1e-12


def test_eq9_limits_and_monotonicity():
    assert O.expected_speedup(1.0, 0.7, 0.5) == pytest.approx(1.0)      # one token per pass: no gain
    assert O.expected_speedup(4.0, 1.0, 0.0) == pytest.approx(4.0)      # free, perfect drafts: M-fold
    assert O.expected_speedup(3.0, 1.0, 1.0) == pytest.approx(1.0)      # drafts as dear as the target
    for c_lo, c_hi in [(0.2, 0.4), (0.5, 0.9)]:
        assert O.expected_speedup(3.0, 0.8, c_lo) > O.expected_speedup(3.0, 0.8, c_hi)
    # a row of the paper's Table 3 with c = 1 - s at the skip ratio the paper's example uses:
    # M = 3.12, alpha = 0.88, c = 0.55  ->  3.12*0.88 / (2.12*0.55 + 0.88)
    assert O.expected_speedup(3.12, 0.88, 0.55) == pytest.approx(2.7456 / 2.046, rel=1e-12)


# ------------------------------------------------------------------ Eq. 8: mix-ratio stream

def test_eq8_stream_extremes_and_frequencies():
    n = 5
    u = synth.mix_ratio_stream(n, 20000, 0.3, seed=4).numpy()
    # r = 0 never switches; r = 1 always switches
    cur = 2
    for us, up in u[:200]:
        assert O.next_domain(cur, n, 0.0, us, up) == cur
        nxt = O.next_domain(cur, n, 1.0, us, up)
        assert nxt != cur and 0 <= nxt < n
    # r = 0.3: stay with frequency 0.7, each other domain with 0.3/4
    counts = np.zeros(n)
    for us, up in u:
        counts[O.next_domain(cur, n, 0.3, us, up)] += 1
    freq = counts / counts.sum()
    assert abs(freq[cur] - 0.7) < 0.02
    for j in range(n):
        if j != cur:
            assert abs(freq[j] - 0.3 / 4) < 0.01
