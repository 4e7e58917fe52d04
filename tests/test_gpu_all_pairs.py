"""GPU parity of the all-pairs reading of Alg. 1 (every two layers i > j scored; greedy choice over all
of them; Sec. 4.2) against the fp64 oracle, through the C ABI."""
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


def gpu_all_pairs(q, k, **kw):
    import paper_2507_08045_amd as kr
    out = kr.all_pairs_similarity(q, k, want_head_score=True, **kw)
    torch.cuda.synchronize()
    return {n: out[n].cpu().numpy() for n in ("pair_score", "pair_dist", "head_score")}


# (name, B, L, Hq, Hkv, d, S, Tq, dtype)
CASES = [
    ("ap-wide", 1, 6, 8, 2, 128, 700, 40, "bf16"),        # 160 rows per kv head: two row groups, the second a quarter full
    ("ap-two-blocks-d64", 2, 40, 4, 2, 64, 300, 5, "bf16"),   # 40 layers: 2 x 2 accumulator blocks
    ("ap-three-blocks", 1, 70, 2, 1, 128, 130, 3, "bf16"),
    ("ap-four-blocks", 1, 100, 2, 2, 64, 70, 2, "bf16"),
    ("ap-tiny", 1, 2, 2, 1, 64, 3, 1, "bf16"),
    ("ap-odd-key-blocks", 1, 5, 4, 1, 128, 2080, 2, "bf16"),  # 65 key blocks: the last chunk holds one block
    ("ap-f32", 2, 4, 2, 2, 64, 256, 16, "f32"),             # portable weights kernel
    ("ap-d96", 1, 5, 4, 2, 96, 200, 3, "bf16"),             # portable weights kernel
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_all_pairs_matches_oracle(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq, dtype = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, rho_k=rho, seed=37)
    q, k = G.to_device(w)
    want = oracle.all_pairs(w.q, w.k)
    flag_sets = (0, kr.KRUL_FLAG_GENERIC_KERNEL) if dtype == "bf16" and d in (64, 128) else (0,)
    for fl in flag_sets:
        got = gpu_all_pairs(q, k, flags=fl)
        e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score flags={fl}")
        G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"{name} pair_score flags={fl}")
        e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist flags={fl}")
        for n in ("pair_score", "pair_dist", "head_score"):
            np.testing.assert_array_equal(got[n], np.swapaxes(got[n], -1, -2))
        i = np.arange(L)
        assert np.all(got["pair_score"][:, i, i] == 1.0) and np.all(got["pair_dist"][:, i, i] == 0.0)
        print(f"[{name} flags={fl}] all-pairs max err head={e1:.2e} dist={e3:.2e}", flush=True)
    # neighbours agree with the adjacent entry point
    adj = G.gpu_scores(q, k)
    l = np.arange(L - 1)
    G.assert_close(got["pair_score"][:, l + 1, l], adj["pair_score"].astype(np.float64), G.TOL, f"{name} vs adjacent")


def test_all_pairs_causal(G, oracle):
    import paper_2507_08045_amd as kr
    for name, (B, L, Hq, Hkv, d, S, Tq, dtype) in {"ap-causal": (1, 5, 4, 2, 128, 300, 150, "bf16"),
                                                     "ap-causal-f32": (1, 3, 2, 2, 64, 70, 70, "f32")}.items():
        w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, seed=41)
        q, k = G.to_device(w)
        want = oracle.all_pairs(w.q, w.k, causal=True)
        got = gpu_all_pairs(q, k, flags=kr.KRUL_FLAG_CAUSAL)
        G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score")
        G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist")
        plain = oracle.all_pairs(w.q, w.k)
        assert np.max(np.abs(plain["pair_score"] - want["pair_score"])) > 1e-4   # the mask matters


def test_batches_of_any_size_give_the_same_bits(G):
    """The workspace sets how many rows one batch holds; the result does not depend on it."""
    import paper_2507_08045_amd as kr
    w = workloads.make("ap-batches", B=2, L=7, Hq=8, Hkv=2, d=128, S=400, Tq=50, dtype="bf16", seed=43)   # 200 rows per kv head
    q, k = G.to_device(w)
    shp = kr.make_shape(q, k)
    full = kr.all_pairs_workspace_bytes(shp)
    one = kr.all_pairs_workspace_bytes(shp, 1)            # the smallest batch: one row group
    three = kr.all_pairs_workspace_bytes(shp, one * 3)    # batches that straddle kv heads
    assert one < three < full
    ref = gpu_all_pairs(q, k)
    for budget in (1, one * 3):
        got = gpu_all_pairs(q, k, max_workspace_bytes=budget)
        for n in ref:
            np.testing.assert_array_equal(got[n], ref[n])
    # a workspace smaller than the smallest batch's is refused
    ws = torch.empty(one - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(kr.KrulError) as ei:
        kr.all_pairs_similarity(q, k, workspace=ws)
    assert ei.value.status == kr.KRUL_EWORKSPACE


def test_select_all_is_bit_exact(G, oracle):
    import paper_2507_08045_amd as kr
    rng = np.random.default_rng(47)
    for trial in range(60):
        L = int(rng.integers(2, 81))
        B = int(rng.integers(1, 4))
        if trial % 3 == 0:
            sc = (rng.integers(0, 5, size=(B, L, L)) / 4.0).astype(np.float32)    # many exact ties
        else:
            sc = rng.random((B, L, L)).astype(np.float32)
        if trial % 5 == 1:
            sc[rng.random((B, L, L)) < 0.2] = np.nan                              # NaN: no candidate, on both sides
        el = (rng.random((B, L)) > 0.2).astype(np.uint8)
        n_select = int(rng.integers(0, L // 2 + 1))
        for smaller in (True, False):
            for use_el in (False, True):
                pairs, count = kr.select_pairs_all(torch.from_numpy(sc).cuda(), n_select, smaller,
                                                   torch.from_numpy(el).cuda() if use_el else None)
                torch.cuda.synchronize()
                wp, wc = oracle.select_pairs_all(sc.astype(np.float64), n_select, smaller, el if use_el else None)
                np.testing.assert_array_equal(count.cpu().numpy(), wc)
                np.testing.assert_array_equal(pairs.cpu().numpy(), wp)


def test_all_pairs_then_selection_end_to_end(G, oracle):
    """Alg. 1 as printed: distances of every two layers, ascending, disjoint pairs up to the budget."""
    import paper_2507_08045_amd as kr
    B, L = 2, 12
    rng = np.random.default_rng(53)
    rho = rng.uniform(0.3, 0.95, size=(B, L - 1, 2))
    w = workloads.make("ap-e2e", B=B, L=L, Hq=4, Hkv=2, d=128, S=500, Tq=8, dtype="bf16", rho_k=rho, seed=53)
    q, k = G.to_device(w)
    out = kr.all_pairs_similarity(q, k)
    n_select = kr.n_select_from_ratio(L, 0.5)
    pairs, count = kr.select_pairs_all(out["pair_dist"], n_select, True)
    torch.cuda.synchronize()
    dist = out["pair_dist"].cpu().numpy()
    wp, wc = oracle.select_pairs_all(dist.astype(np.float64), n_select, True)
    np.testing.assert_array_equal(pairs.cpu().numpy(), wp)
    np.testing.assert_array_equal(count.cpu().numpy(), wc)
    # and the oracle's own end-to-end choice wherever its distances are further apart than the tolerance
    want = oracle.all_pairs(w.q, w.k)
    ep, ec = oracle.select_pairs_all(want["pair_dist"], n_select, True)
    for b in range(B):
        tri = want["pair_dist"][b][np.tril_indices(L, -1)]
        if np.min(np.diff(np.sort(tri))) > 2 * G.TOL:
            np.testing.assert_array_equal(pairs.cpu().numpy()[b], ep[b])


def full_size_sample(G, oracle, w, heads, name, **kw):
    """All-pairs at a benchmark configuration's size: the matrices of a few sampled heads are computed
    by the oracle (all query rows, all keys, all layer pairs) and compared entry by entry; properties
    are checked on the whole output."""
    import paper_2507_08045_amd as kr
    q, k = G.to_device(w)
    got = gpu_all_pairs(q, k, **kw)
    hs, ps, pd = got["head_score"], got["pair_score"], got["pair_dist"]
    assert np.all(np.isfinite(hs)) and np.all(hs > 0) and np.all(hs <= 1 + 1e-5)
    assert np.all(pd >= 0) and np.all(pd <= np.sqrt(2) + 1e-5)
    np.testing.assert_allclose(ps, hs.mean(axis=1), atol=1e-6)          # head average
    np.testing.assert_array_equal(ps, np.swapaxes(ps, 1, 2))
    hc, _ = oracle.all_pairs_heads(w.q, w.k, heads)
    err = max(np.max(np.abs(hs[b, h] - hc[u])) for u, (b, h) in enumerate(heads))
    print(f"[{name}] {len(heads)} sampled heads x {w.L * (w.L - 1) // 2} pairs: max |gpu - oracle| = {err:.2e}", flush=True)
    assert err <= G.TOL
    # selection over all pairs on the GPU's own distances: device == oracle selector, bit for bit
    pairs, count = kr.select_pairs_all(torch.from_numpy(pd).cuda(), w.n_select, True)
    wp, wc = oracle.select_pairs_all(pd.astype(np.float64), w.n_select, True)
    np.testing.assert_array_equal(pairs.cpu().numpy(), wp)
    np.testing.assert_array_equal(count.cpu().numpy(), wc)
    return got


def test_all_pairs_c2_full_size(G, oracle):
    full_size_sample(G, oracle, workloads.config("C2"), [(0, 5), (0, 18), (0, 31)], "C2 all pairs")


def test_all_pairs_c3_full_size(G, oracle):
    full_size_sample(G, oracle, workloads.config("C3"), [(0, 9), (0, 30)], "C3 all pairs")


def test_all_pairs_c4_shape_in_batches(G, oracle):
    """C4's layer / head / history shape with 128 query tokens (the oracle keeps a head's weights of all
    layers: 8192 x 2048 rows would be 4 GiB and minutes), in batches of a quarter of the rows."""
    import paper_2507_08045_amd as kr
    w = workloads.scaled("C4", Tq=128)
    q, k = G.to_device(w)
    shp = kr.make_shape(q, k)
    budget = kr.all_pairs_workspace_bytes(shp) // 4
    assert kr.all_pairs_workspace_bytes(shp, budget) <= budget
    full_size_sample(G, oracle, w, [(0, 13)], "C4 shape, Tq=128, four batches", max_workspace_bytes=budget)
