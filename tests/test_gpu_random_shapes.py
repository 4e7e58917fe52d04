"""GPU parity over seeded random shapes, storage types, key sources and entry points, against the fp64
oracle: the cases that nobody thought of (odd head counts, one key, more rows than keys, ...)."""
import numpy as np
import pytest
import torch

import workloads
from test_gpu_paged_k import scatter_pages

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gpu_util


def draw(rng):
    """One case: shape, storage type, flags and which call takes it."""
    while True:
        c = dict(dtype=str(rng.choice(["bf16", "bf16", "f16", "f32"])), d=int(rng.choice([8, 24, 40, 56, 64, 72, 96, 112, 128, 128, 136])),
                 Hkv=int(rng.choice([1, 2, 4, 8])), g=int(rng.choice([1, 2, 4, 8])),
                 Tq=int(rng.choice([1, 1, 2, 3, 5, 8, 9, 16, 17, 33, 64, 70, 130])),
                 S=int(rng.choice([1, 7, 31, 33, 64, 100, 129, 255, 257, 500, 700, 1025, 1500, 2100])),
                 L=int(rng.integers(2, 7)), B=int(rng.choice([1, 1, 2, 3, 5])))
        c["mode"] = str(rng.choice(["dense", "strided", "paged", "select", "ir", "accumulate", "all-pairs", "all-pairs-paged"]))
        c["causal"] = bool(rng.random() < 0.3) and c["S"] >= c["Tq"] and c["mode"] != "ir"
        c["single_split"] = bool(rng.random() < 0.15)
        if c["B"] * c["L"] * c["Hkv"] * c["g"] * c["Tq"] * c["S"] * c["d"] <= 4e8:   # what the oracle does in a moment
            return c


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes(G, oracle, seed):
    import paper_2507_08045_amd as kr
    rng = np.random.default_rng(seed)
    worst = 0.0
    for it in range(40):
        c = draw(rng)
        B, L, Hkv, d, S, Tq = c["B"], c["L"], c["Hkv"], c["d"], c["S"], c["Tq"]
        Hq, mode, causal = Hkv * c["g"], c["mode"], c["causal"]
        flags = (kr.KRUL_FLAG_CAUSAL if causal else 0) | (kr.KRUL_FLAG_SINGLE_SPLIT if c["single_split"] else 0)
        what = f"seed {seed} case {it}: {c}"
        print(what, flush=True)
        w = workloads.make(f"random-{seed}-{it}", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=c["dtype"],
                           seed=7000 + 100 * seed + it, rho_k=rng.uniform(0.3, 0.95, size=(B, L - 1, Hkv)))
        q, k = G.to_device(w)
        keep = None
        if mode.startswith("all-pairs"):
            want = oracle.all_pairs(w.q, w.k, causal=causal)
            if mode == "all-pairs":
                out = kr.all_pairs_similarity(q, k, flags=flags, want_head_score=True)
            else:
                pools, table, keep = scatter_pages(k, int(rng.choice([8, 16, 64])), str(rng.choice(["pbhd", "phbd"])), 2,
                                                   rng, float("nan"))
                out = kr.all_pairs_similarity_in_place(q, kr.PagedKeys(pools, table, S), flags=flags, want_head_score=True)
            names = ("head_score", "pair_dist")
        else:
            want = oracle.pair_similarity(w.q, w.k, causal=causal)
            names = ("head_score", "pair_score", "pair_dist")
            if mode == "dense":
                out = kr.pair_similarity(q, k, flags=flags)
            elif mode == "strided":
                keep = [k[:, l].permute(0, 2, 1, 3).contiguous() for l in range(L)]
                out = kr.pair_similarity_strided(q, [t.permute(0, 2, 1, 3) for t in keep], flags=flags)
            elif mode == "paged":
                pools, table, keep = scatter_pages(k, int(rng.choice([8, 16, 32, 128])), str(rng.choice(["pbhd", "phbd"])),
                                                   3, rng, float("nan"))
                out = kr.pair_similarity_paged(q, pools, table, S, flags=flags)
            elif mode == "select":
                n_sel = int(rng.integers(0, L // 2 + 1))
                el = (rng.random((B, L)) > 0.2).astype(np.uint8)
                out = kr.pair_similarity_select(q, k, n_sel, torch.from_numpy(el).cuda(), flags=flags)
                torch.cuda.synchronize()
                wp, wc = oracle.select_pairs(out["pair_score"].cpu().numpy().astype(np.float64), n_sel, el)
                np.testing.assert_array_equal(out["pairs"].cpu().numpy(), wp, err_msg=what)
                np.testing.assert_array_equal(out["count"].cpu().numpy(), wc, err_msg=what)
            elif mode == "ir":
                out = kr.pair_similarity_ir(q, k, 0.2, flags=flags)
                torch.cuda.synchronize()
                want_mass, _ = oracle.ir_mass(w.q, w.k, 0.2)
                G.assert_close(out["ir_mass"].cpu().numpy(), want_mass, G.TOL, what + " ir_mass")
            else:
                hs = torch.zeros((B, L - 1, Hq), dtype=torch.float32, device="cuda")
                hd = torch.zeros_like(hs)
                kr.pair_similarity_accumulate(q, k, hs, hd, flags=flags)
                out = kr.pair_scores_from_sums(hs, Tq, hd)
        torch.cuda.synchronize()
        for n in names:
            worst = max(worst, G.assert_close(out[n].cpu().numpy(), want[n], G.TOL, f"{what} {n}"))
        del keep
    print(f"seed {seed}: worst |gpu - oracle| = {worst:.2e}", flush=True)
