"""Pins for the fp64 oracle's similarity functions (CPU only).

Each test checks the oracle against something it did not compute itself: a closed
form, an invariant of softmax / cosine, a library routine (scipy) on a small
input, a hand-derived value, or a naive brute force.  Together they are chosen so
that a dropped term, a wrong index, a transposed operand or a forgotten
normalisation fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist
from scipy.special import softmax

import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qk(rng, B=1, L=3, Hq=2, Hkv=2, Tq=3, S=7, d=4):
    q = rng.standard_normal((B, L, Hq, Tq, d)).astype(np.float32)
    k = rng.standard_normal((B, L, Hkv, S, d)).astype(np.float32)
    return q, k


def library_scores(q, k, scale=None):
    """Same quantities through scipy's softmax and cdist (library routines)."""
    B, L, Hq, Tq, d = q.shape
    Hkv, S = k.shape[2], k.shape[3]
    g = Hq // Hkv
    sc = scale if scale else 1.0 / math.sqrt(d)
    P = np.empty((B, L, Hq, Tq, S))
    for b, l, h in itertools.product(range(B), range(L), range(Hq)):
        logits = q[b, l, h].astype(np.float64) @ k[b, l, h // g].astype(np.float64).T * sc
        P[b, l, h] = softmax(logits, axis=-1)
    hs = np.empty((B, L - 1, Hq))
    hd = np.empty((B, L - 1, Hq))
    for b, l, h in itertools.product(range(B), range(L - 1), range(Hq)):
        hs[b, l, h] = np.mean(1.0 - np.diag(cdist(P[b, l, h], P[b, l + 1, h], "cosine")))
        hd[b, l, h] = np.mean(np.diag(cdist(P[b, l, h], P[b, l + 1, h], "euclidean")))
    return hs, hd, P


def test_matches_scipy_softmax_and_cdist(oracle):
    rng = np.random.default_rng(1)
    for (B, L, Hq, Hkv, Tq, S, d) in [(1, 3, 2, 2, 3, 7, 4), (2, 4, 4, 2, 5, 33, 8), (1, 2, 6, 2, 1, 1, 16),
                                      (3, 5, 3, 1, 2, 19, 5)]:
        q, k = rand_qk(rng, B, L, Hq, Hkv, Tq, S, d)
        q *= 2.0
        o = oracle.pair_similarity(q, k)
        hs, hd, _ = library_scores(q, k)
        np.testing.assert_allclose(o["head_score"], hs, rtol=0, atol=1e-12)
        np.testing.assert_allclose(o["head_dist"], hd, rtol=0, atol=1e-12)
        np.testing.assert_allclose(o["pair_score"], hs.mean(axis=2), rtol=0, atol=1e-12)
        np.testing.assert_allclose(o["pair_dist"], hd.mean(axis=2), rtol=0, atol=1e-12)


def test_explicit_scale_argument(oracle):
    rng = np.random.default_rng(2)
    q, k = rand_qk(rng, 1, 3, 2, 1, 4, 11, 8)
    o = oracle.pair_similarity(q, k, scale=0.7)
    hs, hd, _ = library_scores(q, k, scale=0.7)
    np.testing.assert_allclose(o["head_score"], hs, atol=1e-12)
    np.testing.assert_allclose(o["head_dist"], hd, atol=1e-12)
    # default scale is 1/sqrt(head_dim)  (Sec. 2.1)
    o0 = oracle.pair_similarity(q, k)
    o1 = oracle.pair_similarity(q, k, scale=1.0 / math.sqrt(8))
    np.testing.assert_allclose(o0["head_score"], o1["head_score"], atol=1e-15)


def test_bf16_bits_are_widened_exactly(oracle):
    rng = np.random.default_rng(3)
    q, k = rand_qk(rng, 1, 3, 4, 2, 3, 9, 8)
    qb, kb = workloads.f32_to_bf16_bits(q), workloads.f32_to_bf16_bits(k)
    o_bits = oracle.pair_similarity(qb, kb)
    o_f32 = oracle.pair_similarity(workloads.bf16_bits_to_f32(qb), workloads.bf16_bits_to_f32(kb))
    for key in o_bits:
        np.testing.assert_array_equal(o_bits[key], o_f32[key])
    # rounding really happened (bf16 keeps 8 significant bits)
    assert np.max(np.abs(workloads.bf16_bits_to_f32(qb) - q)) > 1e-4
    assert np.max(np.abs(workloads.bf16_bits_to_f32(qb) / q - 1)) < 2.0 ** -8


def test_f16_bits_are_widened_exactly(oracle):
    """IEEE binary16 inputs: the same numbers as their float32 images (numpy's conversion), over
    normal, subnormal, tiny and large finite values."""
    rng = np.random.default_rng(4)
    q, k = rand_qk(rng, 1, 3, 4, 2, 3, 9, 8)
    qh, kh = q.astype(np.float16), k.astype(np.float16)
    # plant special patterns: subnormals, the smallest and largest normals, signed zeros
    special = np.array([0x0001, 0x03FF, 0x0400, 0x7BFF, 0x8001, 0x8000, 0x0000, 0x3555, 0xFBFF, 0x0200],
                       dtype=np.uint16).view(np.float16) * np.float16(1.0)
    kh.reshape(-1)[:special.size] = special * np.float16(1e-3)     # keep the logits finite ...
    kh.reshape(-1)[special.size:2 * special.size] = special.view(np.uint16).view(np.float16)
    kh = np.where(np.abs(kh.astype(np.float32)) > 100, np.float16(0.5), kh)   # ... and drop the huge ones
    kh.reshape(-1)[40] = np.uint16(0x0001).view(np.float16)          # a subnormal stays
    o_h = oracle.pair_similarity(qh, kh)
    o_f = oracle.pair_similarity(qh.astype(np.float32), kh.astype(np.float32))
    for key in o_h:
        np.testing.assert_array_equal(o_h[key], o_f[key])
    assert np.max(np.abs(qh.astype(np.float32) - q)) > 1e-5          # rounding really happened
    # every bit pattern, through a one-key problem whose single logit is q * k with q = 1:
    # distance of the two layers' rows is 0 (one key), so use the scale to read values back instead:
    # softmax over two keys (k, 0) with q = 1, d = 1: p0 = 1 / (1 + exp(-k * scale))
    pats = np.arange(0, 0x7C00, 37, dtype=np.uint16)                 # finite non-negative patterns
    vals = pats.view(np.float16)
    kk = np.zeros((1, 2, 1, 2, 1), dtype=np.float16)
    qq = np.ones((1, 2, 1, 1, 1), dtype=np.float16)
    for v in vals[::16]:
        kk[0, 0, 0, 0, 0] = v
        kk[0, 1, 0, 0, 0] = v
        a = oracle.pair_similarity(qq, kk, scale=1e-3)
        b = oracle.pair_similarity(qq.astype(np.float32), kk.astype(np.float32), scale=1e-3)
        assert a["head_dist"][0, 0, 0] == b["head_dist"][0, 0, 0] == 0.0
        # and against a second layer with k = 0 the distance is a strictly monotone function of the value
        kk[0, 1, 0, 0, 0] = 0
        a = oracle.pair_similarity(qq, kk, scale=1e-3)
        b = oracle.pair_similarity(qq.astype(np.float32), kk.astype(np.float32), scale=1e-3)
        assert a["head_dist"][0, 0, 0] == b["head_dist"][0, 0, 0]
        p0 = 1.0 / (1.0 + np.exp(-float(v) * 1e-3))
        np.testing.assert_allclose(a["head_dist"][0, 0, 0], np.sqrt(2) * abs(p0 - 0.5), rtol=1e-9, atol=1e-15)


def test_identical_layers_score_one(oracle):
    rng = np.random.default_rng(4)
    q, k = rand_qk(rng, 2, 2, 4, 2, 5, 40, 8)
    q[:, 1], k[:, 1] = q[:, 0], k[:, 0]
    o = oracle.pair_similarity(q, k)
    np.testing.assert_allclose(o["head_score"], 1.0, atol=1e-14)
    np.testing.assert_allclose(o["head_dist"], 0.0, atol=1e-14)


def test_uniform_keys_closed_form(oracle):
    # All S keys of a layer equal => every attention row is exactly 1/S.
    rng = np.random.default_rng(5)
    S, d, Tq = 23, 8, 4
    q, k = rand_qk(rng, 1, 3, 2, 2, Tq, S, d)
    k[0, 0] = k[0, 0, :, :1, :]          # layer 0 uniform
    k[0, 1] = k[0, 1, :, :1, :]          # layer 1 uniform
    o = oracle.pair_similarity(q, k)
    # two uniform layers: cosine 1, distance 0
    np.testing.assert_allclose(o["head_score"][0, 0], 1.0, atol=1e-14)
    np.testing.assert_allclose(o["head_dist"][0, 0], 0.0, atol=1e-14)
    # uniform row u vs arbitrary row p: cos = 1/(sqrt(S) |p|), dist^2 = |p|^2 - 1/S
    for h in range(2):
        logits = q[0, 2, h].astype(np.float64) @ k[0, 2, h].astype(np.float64).T / math.sqrt(d)
        p = softmax(logits, axis=-1)
        pn = np.sqrt((p * p).sum(axis=1))
        assert o["head_score"][0, 1, h] == pytest.approx(np.mean(1.0 / (math.sqrt(S) * pn)), abs=1e-13)
        assert o["head_dist"][0, 1, h] == pytest.approx(np.mean(np.sqrt(pn ** 2 - 1.0 / S)), abs=1e-13)


def test_single_key_scores_one(oracle):
    rng = np.random.default_rng(6)
    q, k = rand_qk(rng, 1, 4, 2, 1, 3, 1, 8)
    o = oracle.pair_similarity(q, k)
    np.testing.assert_allclose(o["head_score"], 1.0, atol=1e-15)
    np.testing.assert_allclose(o["head_dist"], 0.0, atol=1e-15)


def test_two_keys_hand_derived(oracle):
    # golden/two_key_rows.txt: with d = 1, scale = 1 and q = 1 the logits are the keys.
    # Layer 0 keys (ln 2, 0) give the row (2/3, 1/3); layer 1 keys (0, ln 2) give
    # (1/3, 2/3); layer 2 keys (0, 0) give (1/2, 1/2).
    rows = {}
    with open(os.path.join(GOLDEN, "two_key_rows.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val = line.split("=")
            rows[name.strip()] = float(val)
    q = np.ones((1, 3, 1, 1, 1), dtype=np.float32)
    k = np.zeros((1, 3, 1, 2, 1), dtype=np.float64)
    k[0, 0, 0, 0, 0] = math.log(2.0)
    k[0, 1, 0, 1, 0] = math.log(2.0)
    k32 = k.astype(np.float32)
    o = oracle.pair_similarity(q, k32, scale=1.0)
    # float32 rounding of ln 2 moves the rows by ~1e-8
    assert o["pair_score"][0, 0] == pytest.approx(rows["cos_01"], abs=1e-7)
    assert o["pair_dist"][0, 0] == pytest.approx(rows["dist_01"], abs=1e-7)
    assert o["pair_score"][0, 1] == pytest.approx(rows["cos_12"], abs=1e-7)
    assert o["pair_dist"][0, 1] == pytest.approx(rows["dist_12"], abs=1e-7)


def test_sigmoid_closed_form_two_keys(oracle):
    # S = 2: p = (sigma(D), 1 - sigma(D)) with D the logit difference.
    rng = np.random.default_rng(7)
    q, k = rand_qk(rng, 1, 2, 1, 1, 6, 2, 4)
    o = oracle.pair_similarity(q, k)
    cs, ds = [], []
    for t in range(6):
        rows = []
        for l in range(2):
            D = float(q[0, l, 0, t].astype(np.float64) @ (k[0, l, 0, 0].astype(np.float64) - k[0, l, 0, 1].astype(np.float64))) / 2.0
            s = 1.0 / (1.0 + math.exp(-D))
            rows.append((s, 1.0 - s))
        (a0, a1), (b0, b1) = rows
        cs.append((a0 * b0 + a1 * b1) / math.sqrt((a0 * a0 + a1 * a1) * (b0 * b0 + b1 * b1)))
        ds.append(math.hypot(a0 - b0, a1 - b1))
    assert o["head_score"][0, 0, 0] == pytest.approx(np.mean(cs), abs=1e-13)
    assert o["head_dist"][0, 0, 0] == pytest.approx(np.mean(ds), abs=1e-13)


def test_one_hot_limit(oracle):
    # A huge scale turns each row into the indicator of its arg-max key: cosine is
    # 1 if the two layers agree on the arg-max and 0 otherwise; distance 0 or sqrt 2.
    rng = np.random.default_rng(8)
    q, k = rand_qk(rng, 1, 2, 2, 2, 16, 5, 8)
    o = oracle.pair_similarity(q, k, scale=1.0e4)
    for h in range(2):
        am0 = np.argmax(q[0, 0, h].astype(np.float64) @ k[0, 0, h].astype(np.float64).T, axis=1)
        am1 = np.argmax(q[0, 1, h].astype(np.float64) @ k[0, 1, h].astype(np.float64).T, axis=1)
        agree = np.mean(am0 == am1)
        assert o["head_score"][0, 0, h] == pytest.approx(agree, abs=1e-9)
        assert o["head_dist"][0, 0, h] == pytest.approx((1.0 - agree) * math.sqrt(2.0), abs=1e-9)
    assert np.all(np.isfinite(o["head_score"]))


def test_pair_symmetry_and_layer_reversal(oracle):
    rng = np.random.default_rng(9)
    q, k = rand_qk(rng, 1, 5, 2, 1, 3, 17, 8)
    o = oracle.pair_similarity(q, k)
    r = oracle.pair_similarity(q[:, ::-1], k[:, ::-1])
    np.testing.assert_allclose(r["pair_score"], o["pair_score"][:, ::-1], atol=1e-14)
    np.testing.assert_allclose(r["head_dist"], o["head_dist"][:, ::-1], atol=1e-14)
    # distinct pairs do have distinct scores here, so the reversal is observable
    assert np.ptp(o["pair_score"]) > 1e-3


def test_softmax_shift_invariance(oracle):
    # Adding one vector c to every key of a layer shifts each row's logits by q.c
    # (a per-row constant): attention rows, hence all scores, do not change.
    rng = np.random.default_rng(10)
    q, k = rand_qk(rng, 1, 3, 2, 2, 4, 29, 8)
    o = oracle.pair_similarity(q, k)
    k2 = k.astype(np.float64)
    c = rng.standard_normal(8) * 60.0
    k2[0, 1] += c
    # keep the shifted keys exactly representable: work in float64 -> float32 may
    # round, so compare against the oracle run on the rounded values' own shift
    k2f = k2.astype(np.float32)
    c_eff = (k2f[0, 1].astype(np.float64) - k[0, 1].astype(np.float64))
    assert np.max(np.abs(c_eff - c)) < 1e-4          # rounding is small next to c
    o2 = oracle.pair_similarity(q, k2f)
    shift = np.abs(q[0, 1].astype(np.float64) @ c / math.sqrt(8))
    assert shift.max() > 50.0                        # logits really moved by tens
    np.testing.assert_allclose(o2["head_score"], o["head_score"], atol=2e-4)
    np.testing.assert_allclose(o2["head_dist"], o["head_dist"], atol=2e-4)


def test_key_permutation_invariance(oracle):
    rng = np.random.default_rng(11)
    q, k = rand_qk(rng, 1, 4, 4, 2, 3, 31, 8)
    perm = rng.permutation(31)
    o = oracle.pair_similarity(q, k)
    p = oracle.pair_similarity(q, k[:, :, :, perm])
    np.testing.assert_allclose(p["head_score"], o["head_score"], atol=1e-13)
    np.testing.assert_allclose(p["head_dist"], o["head_dist"], atol=1e-13)
    # permuting only ONE layer of a pair must change the score (keys are matched by position)
    k3 = k.copy()
    k3[:, 1] = k[:, 1][:, :, perm]
    assert np.max(np.abs(oracle.pair_similarity(q, k3)["head_score"] - o["head_score"])) > 1e-3


def test_cauchy_schwarz_range_and_distance_identity(oracle):
    rng = np.random.default_rng(12)
    q, k = rand_qk(rng, 2, 4, 4, 2, 6, 50, 16)
    q *= 3.0
    o = oracle.pair_similarity(q, k)
    assert np.all(o["head_score"] > 0.0) and np.all(o["head_score"] <= 1.0 + 1e-15)
    assert np.all(o["head_dist"] >= 0.0) and np.all(o["head_dist"] <= math.sqrt(2.0))
    # Sec. 7: |a-b|^2 = a^2 + b^2 - 2ab, evaluated from library softmax rows
    _, _, P = library_scores(q, k)
    a, b = P[:, :-1], P[:, 1:]
    d2 = (a * a).sum(-1) + (b * b).sum(-1) - 2.0 * (a * b).sum(-1)
    np.testing.assert_allclose(np.sqrt(np.maximum(d2, 0)).mean(-1), o["head_dist"], atol=1e-9)


def test_gqa_equals_repeated_mha(oracle):
    rng = np.random.default_rng(13)
    q, k = rand_qk(rng, 1, 3, 6, 2, 3, 21, 8)
    o = oracle.pair_similarity(q, k)
    k_rep = np.repeat(k, 3, axis=2)                  # query head h reads kv head h // 3
    m = oracle.pair_similarity(q, k_rep)
    np.testing.assert_array_equal(m["head_score"], o["head_score"])
    # and the mapping is not h % Hkv: that variant gives different numbers
    k_mod = np.tile(k, (1, 1, 3, 1, 1))
    assert np.max(np.abs(oracle.pair_similarity(q, k_mod)["head_score"] - o["head_score"])) > 1e-3


def test_batch_and_token_partition(oracle):
    rng = np.random.default_rng(14)
    q, k = rand_qk(rng, 3, 3, 2, 1, 6, 13, 8)
    o = oracle.pair_similarity(q, k)
    for b in range(3):
        ob = oracle.pair_similarity(q[b:b + 1], k[b:b + 1])
        np.testing.assert_array_equal(ob["head_score"][0], o["head_score"][b])
    # rows 0..1 and rows 2..5 scored apart, combined with weights 2/6 and 4/6
    a = oracle.pair_similarity(q[:, :, :, :2], k)
    c = oracle.pair_similarity(q[:, :, :, 2:], k)
    np.testing.assert_allclose((2 * a["head_score"] + 4 * c["head_score"]) / 6, o["head_score"], atol=1e-14)
    np.testing.assert_allclose((2 * a["pair_dist"] + 4 * c["pair_dist"]) / 6, o["pair_dist"], atol=1e-14)


def test_unit_subset_matches_full(oracle):
    rng = np.random.default_rng(15)
    q, k = rand_qk(rng, 2, 4, 4, 2, 3, 12, 8)
    o = oracle.pair_similarity(q, k)
    units = [(1, 2, 3), (0, 0, 0), (1, 0, 2)]
    hc, hd = oracle.unit_scores(q, k, units)
    for i, (b, l, h) in enumerate(units):
        assert hc[i] == o["head_score"][b, l, h]
        assert hd[i] == o["head_dist"][b, l, h]


def test_brute_force_tiny(oracle):
    # A second, deliberately naive evaluation with Python floats and math.fsum.
    rng = np.random.default_rng(16)
    B, L, Hq, Hkv, Tq, S, d = 1, 4, 2, 1, 2, 8, 4
    q, k = rand_qk(rng, B, L, Hq, Hkv, Tq, S, d)
    o = oracle.pair_similarity(q, k)

    def row(l, h, t):
        lg = [math.fsum(float(q[0, l, h, t, i]) * float(k[0, l, 0, j, i]) for i in range(d)) / math.sqrt(d)
              for j in range(S)]
        ex = [math.exp(x) for x in lg]
        z = math.fsum(ex)
        return [e / z for e in ex]

    for l in range(L - 1):
        tot = []
        for h in range(Hq):
            per_t = []
            for t in range(Tq):
                a, b = row(l, h, t), row(l + 1, h, t)
                per_t.append(math.fsum(x * y for x, y in zip(a, b)) /
                             math.sqrt(math.fsum(x * x for x in a) * math.fsum(y * y for y in b)))
            assert o["head_score"][0, l, h] == pytest.approx(math.fsum(per_t) / Tq, abs=1e-13)
            tot.append(math.fsum(per_t) / Tq)
        assert o["pair_score"][0, l] == pytest.approx(math.fsum(tot) / Hq, abs=1e-13)


def test_gaussian_large_s_limit(oracle):
    # If the paired logits are jointly Gaussian with variance s2 and correlation r,
    # then for many keys cos -> E[e^{x+y}] / sqrt(E[e^{2x}] E[e^{2y}]) = exp(s2 (r - 1)).
    # Build it exactly: the same unit-norm-scaled query in both layers (|q|^2 = d, so
    # s2 = scale^2 * d), keys K1 = r K0 + sqrt(1-r^2) noise.
    rng = np.random.default_rng(17)
    d, S, Tq = 32, 16384, 8
    s2 = 0.5
    for r in (0.0, 0.6, 0.9):
        q0 = rng.standard_normal((Tq, d))
        q0 *= math.sqrt(d) / np.linalg.norm(q0, axis=1, keepdims=True)
        k0 = rng.standard_normal((S, d))
        k1 = r * k0 + math.sqrt(1 - r * r) * rng.standard_normal((S, d))
        q = np.stack([q0, q0])[None, :, None].astype(np.float32)
        k = np.stack([k0, k1])[None, :, None].astype(np.float32)
        o = oracle.pair_similarity(q, k, scale=math.sqrt(s2 / d))
        assert o["pair_score"][0, 0] == pytest.approx(math.exp(s2 * (r - 1.0)), rel=0.02)


def test_generator_recipe_matches_limit(oracle):
    # The benchmark recipe (rho_q = 0.95, unit marginals) puts pair scores near
    # exp(rho_q * rho_k - 1) and orders them by rho_k.
    w = workloads.make(B=1, L=4, Hq=2, Hkv=1, d=64, S=8192, Tq=8, dtype="bf16",
                       rho_k=np.array([0.9, 0.5, 0.7]).reshape(1, 3, 1), seed=99)
    o = oracle.pair_similarity(w.q, w.k)
    ps = o["pair_score"][0]
    assert ps[0] > ps[2] > ps[1]
    for l, rk in enumerate((0.9, 0.5, 0.7)):
        assert ps[l] == pytest.approx(math.exp(0.95 * rk - 1.0), rel=0.12)


def test_float32_evaluation_has_room_under_tolerance(oracle):
    # The same definition evaluated in float32 (numpy) stays far inside the 2e-3
    # bar the GPU path is held to, so that bar is not met by luck.
    w = workloads.make(B=1, L=3, Hq=4, Hkv=2, d=64, S=512, Tq=8, dtype="bf16", rho_k=0.8, seed=5)
    o = oracle.pair_similarity(w.q, w.k)
    qf, kf = workloads.bf16_bits_to_f32(w.q), workloads.bf16_bits_to_f32(w.k)
    hs = np.empty((2, 4), dtype=np.float32)
    for l in range(2):
        for h in range(4):
            rows = []
            for ll in (l, l + 1):
                lg = (qf[0, ll, h] @ kf[0, ll, h // 2].T) * np.float32(1 / 8.0)
                e = np.exp(lg - lg.max(axis=1, keepdims=True), dtype=np.float32)
                rows.append(e / e.sum(axis=1, keepdims=True, dtype=np.float32))
            a, b = rows
            hs[l, h] = np.mean((a * b).sum(1) / np.sqrt((a * a).sum(1) * (b * b).sum(1)))
    assert np.max(np.abs(hs - o["head_score"][0])) < 2e-5


# ---------------------------------------------------------------- I-R layer test

def test_ir_mass_uniform_closed_form(oracle):
    rng = np.random.default_rng(20)
    for S in (10, 25, 37, 100):
        q, k = rand_qk(rng, 1, 2, 2, 1, 3, S, 4)
        k[0, :] = k[0, :, :, :1, :]
        mass, _ = oracle.ir_mass(q, k, 0.5)
        n_init, recent0 = int(math.floor(0.1 * S)), int(math.floor(0.9 * S))
        np.testing.assert_allclose(mass, (n_init + S - recent0) / S, atol=1e-14)


def test_ir_mass_matches_scipy_and_threshold(oracle):
    rng = np.random.default_rng(21)
    q, k = rand_qk(rng, 2, 3, 4, 2, 5, 40, 8)
    k[:, 1, :, :4] *= 6.0                      # layer 1 leans on the first keys
    mass, el = oracle.ir_mass(q, k, 0.5)
    _, _, P = library_scores(q, k)
    ref = (P[..., :4].sum(-1) + P[..., 36:].sum(-1)).mean(axis=(2, 3))
    np.testing.assert_allclose(mass, ref, atol=1e-13)
    np.testing.assert_array_equal(el, (ref >= 0.5).astype(np.uint8))
    assert mass[:, 1].min() > mass[:, 0].max()   # the boosted layer stands out
    assert 0 < el.sum() < el.size                # the threshold splits the layers


def test_ir_mass_one_hot(oracle):
    # With a huge scale each row's whole mass sits on its arg-max key.
    rng = np.random.default_rng(22)
    q, k = rand_qk(rng, 1, 2, 1, 1, 32, 20, 8)
    mass, _ = oracle.ir_mass(q, k, 0.5, scale=1e4)
    for l in range(2):
        am = np.argmax(q[0, l, 0].astype(np.float64) @ k[0, l, 0].astype(np.float64).T, axis=1)
        assert mass[0, l] == pytest.approx(np.mean((am < 2) | (am >= 18)), abs=1e-9)
