"""Pins for the oracle's pair selector (Alg. 1, second loop; Sec. 4.2) -- CPU only.

The reference here states the greedy rule without any sorting: again and again take the
best pair that is still free (both layers unused and eligible; equal scores: the lower
layer), until the budget of shared layers is met or no pair is left.  A sorted list walked
once picks exactly these pairs, in this order.  It is run over every ordering of the scores
for small layer counts, beside the properties the rule implies.
"""
import itertools
import math
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def best_free_pair_repeatedly(scores, eligible, n_layers, r_l):
    """Pairs (lower layer index) in the order taken; the budget is n_layers * r_l shared layers."""
    free = [bool(e) for e in eligible]
    taken = []
    while 2 * len(taken) < n_layers * r_l:
        open_pairs = [l for l in range(n_layers - 1)
                      if free[l] and free[l + 1] and not math.isnan(scores[l])]
        if not open_pairs:
            break
        top = max(scores[l] for l in open_pairs)
        l = min(l for l in open_pairs if scores[l] == top)
        free[l] = free[l + 1] = False
        taken.append(l)
    return taken


def test_exhaustive_orderings_small(oracle):
    for L in (2, 3, 4, 5, 6):
        NP = L - 1
        for perm in itertools.permutations(range(NP)):
            scores = np.array([0.1 + 0.1 * p for p in perm])
            for r_l in (0.25, 0.5, 1.0):
                n_select = math.ceil(L * r_l / 2)
                pairs, count = oracle.select_pairs(scores, n_select)
                want = best_free_pair_repeatedly(scores, [1] * L, L, r_l)
                assert list(pairs[0, :count[0]]) == want, (L, perm, r_l)
                assert all(p == -1 for p in pairs[0, count[0]:])


def test_exhaustive_masks_and_ties(oracle):
    L = 6
    rng = np.random.default_rng(0)
    for mask in itertools.product((0, 1), repeat=L):
        for _ in range(3):
            scores = rng.integers(0, 3, size=L - 1) / 4.0        # many exact ties
            for n_select in (1, 2, 3):
                pairs, count = oracle.select_pairs(scores, n_select, eligible=np.array(mask))
                want = best_free_pair_repeatedly(scores, mask, L, 2 * n_select / L)
                assert list(pairs[0, :count[0]]) == want, (mask, scores, n_select)


def test_properties_random(oracle):
    rng = np.random.default_rng(1)
    for _ in range(200):
        L = int(rng.integers(2, 81))
        B = int(rng.integers(1, 4))
        scores = rng.random((B, L - 1))
        el = (rng.random((B, L)) > 0.2).astype(np.uint8)
        n_select = int(rng.integers(0, L // 2 + 1))
        pairs, count = oracle.select_pairs(scores, n_select, eligible=el)
        bigger, _ = oracle.select_pairs(scores, min(n_select + 1, L // 2), eligible=el)
        for b in range(B):
            chosen = list(pairs[b, :count[b]])
            used = [l for p in chosen for l in (p, p + 1)]
            assert len(set(used)) == len(used)                       # disjoint
            assert all(el[b, l] for l in used)                       # never an excluded layer
            assert count[b] <= n_select
            cand = [l for l in range(L - 1) if el[b, l] and el[b, l + 1]]
            if n_select > 0 and cand:
                best = max(cand, key=lambda l: (scores[b, l], -l))
                assert chosen[0] == best                             # first pick = best candidate
            assert list(bigger[b, :count[b]]) == chosen              # monotone prefix
            sc = [scores[b, p] for p in chosen]
            assert sc == sorted(sc, reverse=True)                    # taken in descending score
            if count[b] < n_select:                                  # stopped early => nothing left
                free = [l for l in cand if l not in used and l + 1 not in used]
                assert not free


def test_taking_a_pair_blocks_both_neighbours(oracle):
    # scores: pair 1 best; taking it blocks pairs 0 and 2 even though they are next best.
    pairs, count = oracle.select_pairs([0.8, 0.9, 0.7, 0.1, 0.2], 2)
    assert list(pairs[0]) == [1, 4] and count[0] == 2
    # greedy is not a maximum matching: with 4 layers and scores (.5,.9,.5) only one pair fits
    pairs, count = oracle.select_pairs([0.5, 0.9, 0.5], 2)
    assert list(pairs[0]) == [1, -1] and count[0] == 1


def test_ties_prefer_lower_layer(oracle):
    pairs, count = oracle.select_pairs([1.0, 1.0, 1.0, 1.0, 1.0], 3)
    assert list(pairs[0]) == [0, 2, 4]


def test_six_layer_golden(oracle):
    vals = {}
    with open(os.path.join(GOLDEN, "six_layer_full_share.txt")) as f:
        for line in f:
            if line.startswith("#") or "=" not in line:
                continue
            name, v = line.split("=")
            vals[name.strip()] = v.split()
    scores = [float(x) for x in vals["scores"]]
    pairs, count = oracle.select_pairs(scores, int(vals["n_select"][0]))
    assert list(pairs[0]) == [int(x) for x in vals["pairs"]]
    assert sorted(l for p in pairs[0] for l in (p, p + 1)) == list(range(6))


def test_nan_scores_are_no_candidates(oracle):
    # the paper is silent on non-finite scores: a pair whose score is NaN is never taken and blocks nothing
    nan = float("nan")
    pairs, count = oracle.select_pairs([0.8, nan, 0.7, nan, 0.2], 3)
    assert list(pairs[0]) == [0, 2, 4] and count[0] == 3
    pairs, count = oracle.select_pairs([nan, nan, nan], 2)
    assert list(pairs[0]) == [-1, -1] and count[0] == 0
    rng = np.random.default_rng(7)
    for _ in range(200):
        L = int(rng.integers(2, 12))
        scores = rng.integers(0, 4, size=L - 1) / 4.0
        scores[rng.random(L - 1) < 0.3] = nan
        el = (rng.random(L) > 0.2).astype(np.uint8)
        n_select = int(rng.integers(0, L // 2 + 1))
        pairs, count = oracle.select_pairs(scores, n_select, eligible=el)
        want = best_free_pair_repeatedly(scores, el, L, 2 * n_select / L)
        assert list(pairs[0, :count[0]]) == want
        assert all(p == -1 for p in pairs[0, count[0]:])
