"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs, element by element.  Similarities must agree within 2e-3
absolute; selections must be bit-exact (see gpu_util.check_selection)."""
import math
import zlib

import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu



@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def run_case(G, oracle, w, flags=0, tol=None):
    import paper_2507_08045_amd as kr  # noqa: F401
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k, flags=flags)
    want = oracle.pair_similarity(w.q, w.k)
    tol = tol or G.TOL
    e1 = G.assert_close(got["head_score"], want["head_score"], tol, f"{w.name} head_score")
    e2 = G.assert_close(got["pair_score"], want["pair_score"], tol, f"{w.name} pair_score")
    e3 = G.assert_close(got["pair_dist"], want["pair_dist"], tol, f"{w.name} pair_dist")
    G.check_selection(oracle, got["pair_score"], want["pair_score"], w.n_select)
    print(f"[{w.name} flags={flags}] max err head={e1:.2e} pair={e2:.2e} dist={e3:.2e}", flush=True)
    return got, want


def test_c1_fp32_full(G, oracle):
    w = workloads.config("C1")
    run_case(G, oracle, w)
    # variant with a forced winner: pair 0 must be selected
    w2 = workloads.make("C1-forced", B=1, L=4, Hq=2, Hkv=2, d=64, S=256, Tq=16, dtype="f32", n_select=1,
                        rho_k=np.array([0.9, 0.5, 0.7]).reshape(1, 3, 1), seed=7)
    got, want = run_case(G, oracle, w2)
    import paper_2507_08045_amd as kr
    pairs, count = kr.select_pairs(torch.from_numpy(got["pair_score"]).cuda(), 1)
    assert pairs.cpu().tolist() == [[0]] and count.cpu().tolist() == [1]


# (name, B, L, Hq, Hkv, d, S, Tq): each spans several tiles and leaves ragged tails
MFMA_CASES = [
    ("wide-ragged", 1, 5, 8, 2, 128, 700, 40),      # Rk=160: 2 row tiles (2nd ragged), S: 3 key tiles
    ("wide-d64", 2, 3, 4, 1, 64, 515, 33),          # Rk=132, head_dim 64, batch 2
    ("mid", 1, 4, 8, 2, 128, 1300, 16),             # Rk=64
    ("mid-ragged-rows", 1, 3, 6, 2, 64, 1030, 17),  # Rk=51
    ("slim", 2, 3, 4, 1, 128, 2500, 3),             # Rk=12
    ("slim-decode", 1, 6, 8, 2, 64, 1111, 1),       # Rk=4: one new token (decode step)
    ("tiny-keys", 1, 3, 4, 2, 128, 5, 40),          # S smaller than one 32-key block
    ("one-key", 1, 2, 2, 2, 64, 1, 2),
]


@pytest.mark.parametrize("case", MFMA_CASES, ids=[c[0] for c in MFMA_CASES])
def test_bf16_mfma_small(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", rho_k=rho, seed=11)
    got, _ = run_case(G, oracle, w)
    # same inputs through the multi-tile path (no key split) and through the portable kernel
    got1, _ = run_case(G, oracle, w, flags=kr.KRUL_FLAG_SINGLE_SPLIT)
    got2, _ = run_case(G, oracle, w, flags=kr.KRUL_FLAG_GENERIC_KERNEL)
    assert np.max(np.abs(got1["head_score"] - got["head_score"])) < 1e-4
    assert np.max(np.abs(got2["head_score"] - got["head_score"])) < 1e-4
    # cosine only (no distance asked for: the kernel then skips the sum it alone needs)
    for fl in (0, kr.KRUL_FLAG_SINGLE_SPLIT):
        q, k = G.to_device(w)
        got3 = G.gpu_scores(q, k, flags=fl, want_pair_dist=False)
        assert got3["pair_dist"] is None
        ref = got if fl == 0 else got1
        assert np.max(np.abs(got3["head_score"] - ref["head_score"])) < 1e-6
        assert np.max(np.abs(got3["pair_score"] - ref["pair_score"])) < 1e-6


def test_identical_layers_give_one(G, oracle):
    w = workloads.make("ident", B=1, L=3, Hq=8, Hkv=2, d=128, S=777, Tq=20, dtype="bf16", rho_k=0.7, seed=3)
    w.q[:, 1], w.k[:, 1] = w.q[:, 0], w.k[:, 0]
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k)
    assert np.max(np.abs(got["head_score"][:, 0] - 1.0)) < 5e-6
    assert np.max(np.abs(got["pair_dist"][:, 0])) < G.TOL
    assert np.all(got["head_score"] <= 1.0 + 5e-6) and np.all(got["head_score"] > 0)


def test_uniform_keys_closed_form(G, oracle):
    # all keys of layer 0 equal => uniform rows; cos with row p of layer 1 is 1/(sqrt(S)|p|)
    w = workloads.make("uniform", B=1, L=2, Hq=4, Hkv=2, d=64, S=600, Tq=9, dtype="bf16", rho_k=0.5, seed=4)
    w.k[0, 0] = w.k[0, 0, :, :1, :]
    run_case(G, oracle, w)


def test_shift_invariance_large_shift(G, oracle):
    # add one vector to every key of a layer: logits of a row move by a constant (tens of
    # units), scores must not move.  Exercises the reference-exponent updates.
    w = workloads.make("shift", B=1, L=3, Hq=8, Hkv=2, d=128, S=900, Tq=12, dtype="bf16", rho_k=0.8, seed=5)
    q, k = G.to_device(w)
    kf = workloads.bf16_bits_to_f32(w.k)
    c = np.random.default_rng(0).standard_normal(128).astype(np.float32) * 24.0
    kf[0, 1] += c
    w2 = workloads.Workload(**{**w.__dict__, "k": workloads.f32_to_bf16_bits(kf), "name": "shifted"})
    shift = np.abs(workloads.bf16_bits_to_f32(w.q)[0, 1].reshape(-1, 128) @ c / math.sqrt(128))
    assert shift.max() > 30.0
    # rounding the shifted keys to bf16 perturbs them, so the check is against the oracle on
    # the same bits (in run_case), not against the unshifted run
    run_case(G, oracle, w2)
    import paper_2507_08045_amd as kr
    run_case(G, oracle, w2, flags=kr.KRUL_FLAG_SINGLE_SPLIT)


def test_sinks_and_late_maximum(G, oracle):
    # heavy-tailed keys: 2% of positions scaled x4; and the largest logit placed in the last tile
    w = workloads.make("sinks", B=1, L=4, Hq=8, Hkv=2, d=128, S=2100, Tq=16, dtype="bf16",
                       rho_k=0.8, seed=6, sink_frac=0.02)
    kf = workloads.bf16_bits_to_f32(w.k)
    kf[0, :, :, -3] *= 6.0
    w.k[:] = workloads.f32_to_bf16_bits(kf)
    run_case(G, oracle, w)
    import paper_2507_08045_amd as kr
    run_case(G, oracle, w, flags=kr.KRUL_FLAG_SINGLE_SPLIT)


def test_one_hot_limit(G, oracle):
    w = workloads.make("onehot", B=1, L=2, Hq=4, Hkv=2, d=64, S=300, Tq=8, dtype="bf16", rho_k=0.9, seed=8)
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k, scale=50.0)
    want = oracle.pair_similarity(w.q, w.k, scale=50.0)
    assert np.all(np.isfinite(got["head_score"]))
    G.assert_close(got["head_score"], want["head_score"], G.TOL, "one-hot head_score")
    # in this limit a row is (nearly) one key: the score of a head is the share of rows whose two layers
    # pick the same key, so the values sit on a grid of 1/Tq
    assert np.max(np.abs(want["head_score"] * 8 - np.round(want["head_score"] * 8))) < 0.05


def test_gqa_equals_repeated_mha(G, oracle):
    w = workloads.make("gqa", B=1, L=3, Hq=8, Hkv=2, d=128, S=500, Tq=10, dtype="bf16", rho_k=0.8, seed=9)
    q, k = G.to_device(w)
    a = G.gpu_scores(q, k)
    k_rep = torch.repeat_interleave(k, 4, dim=2).contiguous()
    b = G.gpu_scores(q, k_rep)
    np.testing.assert_allclose(a["head_score"], b["head_score"], atol=1e-5)


def test_batch_equals_separate_calls(G, oracle):
    w = workloads.make("batch", B=3, L=3, Hq=4, Hkv=2, d=128, S=400, Tq=6, dtype="bf16",
                       rho_k=np.random.default_rng(1).uniform(0.5, 0.95, (3, 2, 1)), seed=10)
    q, k = G.to_device(w)
    full = G.gpu_scores(q, k)
    for b in range(3):
        one = G.gpu_scores(q[b:b + 1].contiguous(), k[b:b + 1].contiguous())
        np.testing.assert_allclose(one["head_score"][0], full["head_score"][b], atol=1e-6)


def test_deterministic(G, oracle):
    w = workloads.make("det", B=1, L=4, Hq=8, Hkv=2, d=128, S=1500, Tq=24, dtype="bf16", rho_k=0.8, seed=12)
    q, k = G.to_device(w)
    a = G.gpu_scores(q, k)
    b = G.gpu_scores(q, k)
    np.testing.assert_array_equal(a["head_score"], b["head_score"])
    np.testing.assert_array_equal(a["pair_dist"], b["pair_dist"])


def test_select_bit_exact_random(G, oracle):
    import paper_2507_08045_amd as kr
    rng = np.random.default_rng(42)
    for trial in range(60):
        L = int(rng.integers(2, 81)) if trial < 50 else int(rng.integers(1000, 4097))
        B = int(rng.integers(1, 9))
        scores = rng.random((B, L - 1)).astype(np.float32)
        if trial % 3 == 0:
            scores = np.round(scores * 4) / 4            # many exact ties
        if trial % 5 == 0:
            scores[:, ::2] = -scores[:, ::2]             # negatives and -0.0/+0.0
        if trial % 7 == 3:
            scores[rng.random(scores.shape) < 0.2] = np.nan   # NaN: no candidate, on both sides
        el = (rng.random((B, L)) > 0.15).astype(np.uint8) if trial % 2 else None
        n_select = int(rng.integers(0, L // 2 + 1))
        ps = torch.from_numpy(scores).cuda()
        eld = torch.from_numpy(el).cuda() if el is not None else None
        pairs, count = kr.select_pairs(ps, n_select, eld)
        torch.cuda.synchronize()
        wp, wc = oracle.select_pairs(scores.astype(np.float64), n_select, el)
        np.testing.assert_array_equal(pairs.cpu().numpy(), wp, err_msg=f"trial {trial} L={L}")
        np.testing.assert_array_equal(count.cpu().numpy(), wc)


def test_six_layer_example_format(G, oracle):
    import paper_2507_08045_amd as kr
    ps = torch.tensor([[0.70, 0.10, 0.90, 0.20, 0.80]], dtype=torch.float32).cuda()
    pairs, count = kr.select_pairs(ps, kr.n_select_from_ratio(6, 1.0))
    assert pairs.cpu().tolist() == [[2, 4, 0]] and count.cpu().tolist() == [3]
