"""Pins for the oracle's causal reading (decode and chunked prefill, Sec. 5: a token attends to
the tokens before it and to itself): the Tq query rows are the last Tq tokens of the S-token
sequence, row t sees keys j <= S - Tq + t.  None of these re-uses the oracle's own loops:
library softmax on a hand-masked matrix, reduction to the unmasked case on truncated keys,
closed forms."""
import numpy as np
from scipy.special import softmax

import workloads


def rand_qk(rng, B, L, Hq, Hkv, d, S, Tq):
    q = rng.standard_normal((B, L, Hq, Tq, d)).astype(np.float32)
    k = rng.standard_normal((B, L, Hkv, S, d)).astype(np.float32)
    return q, k


def library_scores(q, k, causal):
    """cosine / distance means per (b, pair, head) with scipy's softmax on a masked logit matrix"""
    B, L, Hq, Tq, d = q.shape
    Hkv, S = k.shape[2], k.shape[3]
    g = Hq // Hkv
    P = np.empty((B, L, Hq, Tq, S))
    for b in range(B):
        for l in range(L):
            for h in range(Hq):
                s = q[b, l, h].astype(np.float64) @ k[b, l, h // g].astype(np.float64).T / np.sqrt(d)
                if causal:
                    t = np.arange(Tq)[:, None]
                    j = np.arange(S)[None, :]
                    s = np.where(j <= S - Tq + t, s, -np.inf)
                P[b, l, h] = softmax(s, axis=1)
    a, c = P[:, :-1], P[:, 1:]
    cos = (a * c).sum(-1) / np.sqrt((a * a).sum(-1) * (c * c).sum(-1))
    dist = np.sqrt(((a - c) ** 2).sum(-1))
    return cos.mean(-1), dist.mean(-1)


def test_causal_matches_library_softmax_on_masked_logits(oracle):
    rng = np.random.default_rng(11)
    for (S, Tq) in [(9, 4), (7, 7), (12, 1), (33, 5)]:
        q, k = rand_qk(rng, 2, 3, 4, 2, 16, S, Tq)
        got = oracle.pair_similarity(q, k, causal=True)
        cos, dist = library_scores(q, k, True)
        np.testing.assert_allclose(got["head_score"], cos, rtol=0, atol=1e-12)
        np.testing.assert_allclose(got["head_dist"], dist, rtol=0, atol=1e-12)
        np.testing.assert_allclose(got["pair_score"], cos.mean(-1), atol=1e-12)
        # and the mask matters: the unmasked scores differ (unless there is nothing to mask)
        plain = oracle.pair_similarity(q, k)
        if Tq > 1:
            assert np.max(np.abs(plain["head_score"] - got["head_score"])) > 1e-3


def test_single_query_row_is_the_unmasked_case(oracle):
    # Tq = 1: the one row is the last token and sees everything
    rng = np.random.default_rng(12)
    q, k = rand_qk(rng, 1, 4, 4, 4, 8, 21, 1)
    a = oracle.pair_similarity(q, k, causal=True)
    b = oracle.pair_similarity(q, k, causal=False)
    for n in ("pair_score", "head_score", "pair_dist", "head_dist"):
        np.testing.assert_array_equal(a[n], b[n])


def test_each_row_equals_the_unmasked_case_on_truncated_keys(oracle):
    # row t with keys j <= S - Tq + t  ==  a one-row unmasked problem on the first S - Tq + t + 1 keys
    rng = np.random.default_rng(13)
    B, L, Hq, Hkv, d, S, Tq = 1, 3, 2, 1, 8, 10, 4
    q, k = rand_qk(rng, B, L, Hq, Hkv, d, S, Tq)
    got = oracle.pair_similarity(q, k, causal=True)
    acc_c = np.zeros((B, L - 1, Hq))
    acc_d = np.zeros((B, L - 1, Hq))
    for t in range(Tq):
        vis = S - Tq + t + 1
        one = oracle.pair_similarity(q[:, :, :, t:t + 1], k[:, :, :, :vis])
        acc_c += one["head_score"]
        acc_d += one["head_dist"]
    np.testing.assert_allclose(got["head_score"], acc_c / Tq, atol=1e-13)
    np.testing.assert_allclose(got["head_dist"], acc_d / Tq, atol=1e-13)


def test_first_token_sees_only_itself(oracle):
    # S = Tq (a whole sequence as one chunk): row 0 has weight 1 on key 0 in every layer, so its
    # rows agree exactly; with Tq = S = 1 every score is cos 1, dist 0
    rng = np.random.default_rng(14)
    q, k = rand_qk(rng, 1, 3, 2, 2, 8, 1, 1)
    got = oracle.pair_similarity(q, k, causal=True)
    np.testing.assert_allclose(got["head_score"], 1.0, atol=1e-15)
    np.testing.assert_allclose(got["head_dist"], 0.0, atol=1e-15)
    # two tokens: row 0 -> (1, 0); row 1 -> softmax of two logits; closed form for the pair
    q, k = rand_qk(rng, 1, 2, 1, 1, 4, 2, 2)
    got = oracle.pair_similarity(q, k, causal=True)
    rows = []
    for l in range(2):
        z = (q[0, l, 0, 1].astype(np.float64) @ k[0, l, 0].astype(np.float64).T) / 2.0   # sqrt(4)
        p1 = 1.0 / (1.0 + np.exp(z[0] - z[1]))       # weight of key 1
        rows.append(np.array([1.0 - p1, p1]))
    a, c = rows
    cos1 = (a @ c) / np.sqrt((a @ a) * (c @ c))
    np.testing.assert_allclose(got["head_score"][0, 0, 0], (1.0 + cos1) / 2, atol=1e-14)
    np.testing.assert_allclose(got["head_dist"][0, 0, 0], (0.0 + np.linalg.norm(a - c)) / 2, atol=1e-14)


def test_causal_needs_at_least_as_many_keys_as_rows(oracle):
    import pytest
    rng = np.random.default_rng(15)
    q, k = rand_qk(rng, 1, 2, 1, 1, 4, 3, 5)
    with pytest.raises(ValueError):
        oracle.pair_similarity(q, k, causal=True)


def test_bf16_inputs_take_the_same_mask(oracle):
    w = workloads.make("causal-bf16", B=1, L=3, Hq=4, Hkv=2, d=64, S=40, Tq=9, dtype="bf16", seed=3)
    got = oracle.pair_similarity(w.q, w.k, causal=True)
    cos, dist = library_scores(workloads.bf16_bits_to_f32(w.q), workloads.bf16_bits_to_f32(w.k), True)
    np.testing.assert_allclose(got["head_score"], cos, atol=1e-12)
    np.testing.assert_allclose(got["head_dist"], dist, atol=1e-12)
