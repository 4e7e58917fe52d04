"""Pins for the oracle's all-pairs reading of Alg. 1 (every two layers i > j are scored and the
greedy choice runs over all of them; Sec. 4.2) -- CPU only.  None re-uses the oracle's loops:
scipy's softmax and cdist on small inputs, closed forms, relabelling invariance, a literal
set-and-sort transcription of the selection run over exhaustive small cases, and a hand-worked
fixture."""
import itertools
import math
import os

import numpy as np
from scipy.spatial.distance import cdist
from scipy.special import softmax

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qk(rng, B, L, Hq, Hkv, d, S, Tq):
    q = rng.standard_normal((B, L, Hq, Tq, d)).astype(np.float32)
    k = rng.standard_normal((B, L, Hkv, S, d)).astype(np.float32)
    return q, k


def library_all_pairs(q, k, causal=False):
    """[B,Hq,L,L] token means of cosine and distance: scipy softmax, then cdist between the L rows
    that the layers give one token."""
    B, L, Hq, Tq, d = q.shape
    Hkv, S = k.shape[2], k.shape[3]
    g = Hq // Hkv
    cos = np.zeros((B, Hq, L, L))
    dist = np.zeros((B, Hq, L, L))
    for b in range(B):
        for h in range(Hq):
            P = np.empty((L, Tq, S))
            for l in range(L):
                s = q[b, l, h].astype(np.float64) @ k[b, l, h // g].astype(np.float64).T / np.sqrt(d)
                if causal:
                    t = np.arange(Tq)[:, None]
                    j = np.arange(S)[None, :]
                    s = np.where(j <= S - Tq + t, s, -np.inf)
                P[l] = softmax(s, axis=1)
            for t in range(Tq):
                rows = P[:, t, :]
                cos[b, h] += 1.0 - cdist(rows, rows, "cosine")
                dist[b, h] += cdist(rows, rows, "euclidean")
    return cos / Tq, dist / Tq


def test_matches_scipy_softmax_and_cdist(oracle):
    rng = np.random.default_rng(31)
    for (B, L, Hq, Hkv, d, S, Tq, causal) in [(2, 4, 4, 2, 16, 9, 3, False), (1, 5, 2, 2, 8, 17, 1, False),
                                               (1, 3, 4, 1, 16, 12, 5, True), (1, 7, 2, 1, 8, 6, 2, False)]:
        q, k = rand_qk(rng, B, L, Hq, Hkv, d, S, Tq)
        got = oracle.all_pairs(q, k, causal=causal)
        cos, dist = library_all_pairs(q, k, causal)
        np.testing.assert_allclose(got["head_score"], cos, rtol=0, atol=1e-12)
        np.testing.assert_allclose(got["head_dist"], dist, rtol=0, atol=1e-9)   # cdist's sqrt of tiny self-distances
        np.testing.assert_allclose(got["pair_score"], cos.mean(1), rtol=0, atol=1e-12)
        np.testing.assert_allclose(got["pair_dist"], dist.mean(1), rtol=0, atol=1e-9)


def test_chosen_heads_are_the_same_numbers(oracle):
    rng = np.random.default_rng(38)
    q, k = rand_qk(rng, 2, 4, 4, 2, 8, 11, 3)
    full = oracle.all_pairs(q, k)
    hc, hd = oracle.all_pairs_heads(q, k, [(1, 3), (0, 0), (1, 0)])
    for u, (b, h) in enumerate([(1, 3), (0, 0), (1, 0)]):
        np.testing.assert_array_equal(hc[u], full["head_score"][b, h])
        np.testing.assert_array_equal(hd[u], full["head_dist"][b, h])


def test_symmetric_unit_diagonal_and_bounds(oracle):
    rng = np.random.default_rng(32)
    q, k = rand_qk(rng, 2, 6, 4, 2, 16, 40, 4)
    got = oracle.all_pairs(q, k)
    for n in ("pair_score", "pair_dist", "head_score", "head_dist"):
        np.testing.assert_array_equal(got[n], np.swapaxes(got[n], -1, -2))
    i = np.arange(6)
    assert np.all(got["pair_score"][:, i, i] == 1.0) and np.all(got["pair_dist"][:, i, i] == 0.0)
    assert np.all(got["head_score"] > 0) and np.all(got["head_score"] <= 1 + 1e-15)   # rows are positive vectors
    assert np.all(got["head_dist"] <= math.sqrt(2) + 1e-12)                           # two probability vectors


def test_relabelling_the_layers_permutes_the_matrix(oracle):
    # a wrong layer index anywhere breaks this
    rng = np.random.default_rng(33)
    q, k = rand_qk(rng, 1, 6, 2, 2, 8, 25, 3)
    perm = np.array([4, 0, 5, 2, 1, 3])
    a = oracle.all_pairs(q, k)
    b = oracle.all_pairs(q[:, perm], k[:, perm])
    for n in ("pair_score", "pair_dist"):
        np.testing.assert_allclose(b[n], a[n][:, perm][:, :, perm], rtol=0, atol=1e-14)
    for n in ("head_score", "head_dist"):
        np.testing.assert_allclose(b[n], a[n][:, :, perm][:, :, :, perm], rtol=0, atol=1e-14)


def test_neighbours_agree_with_the_adjacent_reading_and_closed_forms(oracle):
    rng = np.random.default_rng(34)
    q, k = rand_qk(rng, 2, 5, 4, 2, 16, 30, 2)
    allp = oracle.all_pairs(q, k)
    adj = oracle.pair_similarity(q, k)
    l = np.arange(4)
    np.testing.assert_allclose(allp["pair_score"][:, l + 1, l], adj["pair_score"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(allp["pair_dist"][:, l + 1, l], adj["pair_dist"], rtol=0, atol=1e-14)
    # copies of one layer: every two layers are alike
    q1 = np.repeat(q[:, :1], 4, axis=1)
    k1 = np.repeat(k[:, :1], 4, axis=1)
    same = oracle.all_pairs(q1, k1)
    np.testing.assert_allclose(same["pair_score"], 1.0, atol=1e-15)
    np.testing.assert_allclose(same["pair_dist"], 0.0, atol=1e-15)
    # one-hot against uniform: layer 0 has zero keys (uniform row 1/S), layer 2 one huge key (one-hot),
    # layer 1 zero keys again: cos(uniform, one-hot) = 1/sqrt(S), distance sqrt(1 - 1/S); layers 0,1 equal
    S, d = 16, 8
    qq = np.ones((1, 3, 1, 1, d), dtype=np.float32)
    kk = np.zeros((1, 3, 1, S, d), dtype=np.float32)
    kk[0, 2, 0, 5, :] = 200.0
    got = oracle.all_pairs(qq, kk)
    np.testing.assert_allclose(got["pair_score"][0, 2, 0], 1 / math.sqrt(S), atol=1e-12)
    np.testing.assert_allclose(got["pair_score"][0, 2, 1], 1 / math.sqrt(S), atol=1e-12)
    np.testing.assert_allclose(got["pair_dist"][0, 2, 0], math.sqrt(1 - 1 / S), atol=1e-12)
    np.testing.assert_allclose(got["pair_score"][0, 1, 0], 1.0, atol=1e-15)


# ---------------------------------------------------------------- selection over every two layers

def best_free_two_layers_repeatedly(D, eligible, n_layers, r_l):
    """The greedy rule with no sorting: again and again take the closest two layers that are both still free and
    eligible (D[i][j], i > j; equal values: the lower j, then the lower i), until n_layers * r_l layers are
    shared or none is left.  Pairs as (j, i) in the order taken."""
    free = [bool(e) for e in eligible]
    taken = []
    while 2 * len(taken) < n_layers * r_l:
        open_pairs = [(j, i) for j in range(n_layers) for i in range(j + 1, n_layers)
                      if free[i] and free[j] and not math.isnan(D[i][j])]
        if not open_pairs:
            break
        closest = min(D[i][j] for j, i in open_pairs)
        j, i = min((j, i) for j, i in open_pairs if D[i][j] == closest)
        free[i] = free[j] = False
        taken.append((j, i))
    return taken


def test_selection_exhaustive_orderings_small(oracle):
    for L in (2, 3, 4):
        nc = L * (L - 1) // 2
        tri = [(i, j) for j in range(L) for i in range(j + 1, L)]
        for perm in itertools.permutations(range(nc)):
            D = np.zeros((L, L))
            for (i, j), p in zip(tri, perm):
                D[i, j] = 0.1 + 0.1 * p
                D[j, i] = -7.0           # the upper triangle must not be read
            for n_select in range(0, L // 2 + 1):
                pairs, count = oracle.select_pairs_all(D, n_select, closer_is_smaller=True)
                want = best_free_two_layers_repeatedly(D, [1] * L, L, 2 * n_select / L)
                assert [tuple(p) for p in pairs[0, :count[0]]] == want, (L, perm, n_select)
                assert np.all(pairs[0, count[0]:] == -1)
                # a similarity is the same choice on the negated matrix
                pairs2, count2 = oracle.select_pairs_all(-D, n_select, closer_is_smaller=False)
                assert count2[0] == count[0] and np.array_equal(pairs2, pairs)


def test_selection_random_masks_and_ties(oracle):
    rng = np.random.default_rng(35)
    for _ in range(300):
        L = int(rng.integers(2, 9))
        D = rng.integers(0, 4, size=(L, L)) / 4.0              # many exact ties
        el = (rng.random(L) > 0.25).astype(np.uint8)
        n_select = int(rng.integers(0, L // 2 + 1))
        pairs, count = oracle.select_pairs_all(D, n_select, closer_is_smaller=True, eligible=el)
        want = best_free_two_layers_repeatedly(D, el, L, 2 * n_select / L)
        assert [tuple(p) for p in pairs[0, :count[0]]] == want, (D, el, n_select)


def test_selection_nan_is_no_candidate(oracle):
    rng = np.random.default_rng(37)
    for _ in range(200):
        L = int(rng.integers(2, 9))
        D = rng.integers(0, 4, size=(L, L)) / 4.0
        D[rng.random((L, L)) < 0.3] = float("nan")
        el = (rng.random(L) > 0.2).astype(np.uint8)
        n_select = int(rng.integers(0, L // 2 + 1))
        for smaller in (True, False):
            pairs, count = oracle.select_pairs_all(D, n_select, closer_is_smaller=smaller, eligible=el)
            want = best_free_two_layers_repeatedly(D if smaller else -D, el, L, 2 * n_select / L)
            assert [tuple(p) for p in pairs[0, :count[0]]] == want, (D, el, n_select)


def test_selection_properties_large(oracle):
    rng = np.random.default_rng(36)
    for _ in range(40):
        L = int(rng.integers(2, 81))
        B = int(rng.integers(1, 4))
        sim = rng.random((B, L, L))
        el = (rng.random((B, L)) > 0.2).astype(np.uint8)
        n_select = int(rng.integers(0, L // 2 + 1))
        pairs, count = oracle.select_pairs_all(sim, n_select, closer_is_smaller=False, eligible=el)
        for b in range(B):
            chosen = [tuple(p) for p in pairs[b, :count[b]]]
            used = [l for p in chosen for l in p]
            assert len(set(used)) == len(used) and all(el[b, l] for l in used)
            assert all(j < i for j, i in chosen)
            vals = [sim[b, i, j] for j, i in chosen]
            assert vals == sorted(vals, reverse=True)          # taken in order of similarity
            if count[b] == n_select:
                continue
            free = [l for l in range(L) if el[b, l] and l not in used]
            assert len(free) < 2                               # budget not met: no candidate was left


def test_selection_worked_example(oracle):
    """tests/golden/all_pairs_selection.txt: a 5-layer distance matrix worked by hand."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "all_pairs_selection.txt")) if ln.strip() and ln[0] != "#"]
    L = int(rows[0][0])
    D = np.array([[float(x) for x in r] for r in rows[1:1 + L]])
    want = [(int(r[0]), int(r[1])) for r in rows[1 + L:]]
    pairs, count = oracle.select_pairs_all(D, 2, closer_is_smaller=True)
    assert [tuple(p) for p in pairs[0, :count[0]]] == want
