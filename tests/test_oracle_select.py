"""Pins for the oracle's pair selector (Alg. 1, second loop; Sec. 4.2) -- CPU only.

The reference here is a literal Python transcription of the algorithm's steps with
sets and the built-in sort, run over every ordering of the scores for small layer
counts, plus the properties the greedy rule implies.
"""
import itertools
import math
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def alg1_literal(scores, eligible, n_layers, r_l):
    """Alg. 1 as stated: distances ascending, take (i,j) iff i,j not in S, stop when
    |S| >= N * r_l.  Distance = -score; candidates are the adjacent pairs of
    eligible layers."""
    D = []
    for j in range(n_layers - 1):
        i = j + 1
        if eligible[i] and eligible[j]:
            D.append((-scores[j], j, i))
    D = sorted(D, key=lambda e: e[0])          # stable: ties keep ascending j
    S, M = set(), []
    if n_layers * r_l <= 0:
        return M
    for _, j, i in D:
        if i not in S and j not in S:
            S |= {i, j}
            M.append(j)
        else:
            continue
        if len(S) >= n_layers * r_l:
            break
    return M


def test_exhaustive_orderings_small(oracle):
    for L in (2, 3, 4, 5, 6):
        NP = L - 1
        for perm in itertools.permutations(range(NP)):
            scores = np.array([0.1 + 0.1 * p for p in perm])
            for r_l in (0.25, 0.5, 1.0):
                n_select = math.ceil(L * r_l / 2)
                pairs, count = oracle.select_pairs(scores, n_select)
                want = alg1_literal(scores, [1] * L, L, r_l)
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
                want = alg1_literal(scores, mask, L, 2 * n_select / L)
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
