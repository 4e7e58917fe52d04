"""GPU parity at the documented limits of the entry points: the largest layer counts (2048 for the
adjacent reading, 128 for the all-pairs reading), selection over many layers, and a long history with a
single query row."""
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


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f32", 40)], ids=["mfma", "portable"])
def test_adjacent_2048_layers(G, oracle, dtype, d):
    w = workloads.make("limit-L2048", B=1, L=2048, Hq=2, Hkv=1, d=d, S=70, Tq=3, dtype=dtype, seed=71)
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k)
    want = oracle.pair_similarity(w.q, w.k)
    G.assert_close(got["head_score"], want["head_score"], G.TOL, "2048 layers head_score")
    G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, "2048 layers pair_dist")
    # the selector's largest budget; greedy leaves single layers between taken pairs, so it ends short of it
    pairs, count, _ = G.check_selection(oracle, got["pair_score"], want["pair_score"], 1024)
    assert 512 < count[0] <= 1024


def test_all_pairs_128_layers(G, oracle):
    import paper_2507_08045_amd as kr
    w = workloads.make("limit-L128", B=1, L=128, Hq=2, Hkv=1, d=64, S=100, Tq=2, dtype="bf16", seed=73)
    q, k = G.to_device(w)
    out = kr.all_pairs_similarity(q, k, want_head_score=True)
    torch.cuda.synchronize()
    want = oracle.all_pairs(w.q, w.k)
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "128 layers all-pairs head_score")
    G.assert_close(out["pair_dist"].cpu().numpy(), want["pair_dist"], G.TOL, "128 layers all-pairs pair_dist")
    # the whole budget over 8128 candidate pairs
    pairs, count = kr.select_pairs_all(out["pair_dist"], 64, True)
    wp, wc = oracle.select_pairs_all(out["pair_dist"].cpu().numpy().astype(np.float64), 64, True)
    np.testing.assert_array_equal(pairs.cpu().numpy(), wp)
    assert count.cpu().numpy()[0] == 64 == wc[0]


def test_select_all_many_layers(G, oracle):
    import paper_2507_08045_amd as kr
    rng = np.random.default_rng(79)
    L = 200                      # 19900 candidates; beyond the selector's LDS-resident size
    sc = rng.random((2, L, L)).astype(np.float32)
    el = (rng.random((2, L)) > 0.1).astype(np.uint8)
    pairs, count = kr.select_pairs_all(torch.from_numpy(sc).cuda(), 100, False, torch.from_numpy(el).cuda())
    wp, wc = oracle.select_pairs_all(sc.astype(np.float64), 100, False, el)
    np.testing.assert_array_equal(pairs.cpu().numpy(), wp)
    np.testing.assert_array_equal(count.cpu().numpy(), wc)


def test_long_history_single_row(G, oracle):
    """A decode step over 262144 history tokens: one query row per head, 8192 32-key blocks."""
    import paper_2507_08045_amd as kr
    w = workloads.make("limit-long", B=1, L=3, Hq=4, Hkv=1, d=128, S=262144, Tq=1, dtype="bf16", seed=83,
                       sink_frac=0.001, sink_gain=3.0)
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k, flags=kr.KRUL_FLAG_CAUSAL)
    want = oracle.pair_similarity(w.q, w.k, causal=True)
    G.assert_close(got["head_score"], want["head_score"], G.TOL, "long history head_score")
    G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, "long history pair_dist")
    ap = kr.all_pairs_similarity(q, k)
    torch.cuda.synchronize()
    want_ap = oracle.all_pairs(w.q, w.k)
    G.assert_close(ap["pair_score"].cpu().numpy(), want_ap["pair_score"], G.TOL, "long history all-pairs")
