"""GPU parity of krul_pair_similarity_paged: keys read in place from per-layer pools of fixed-size pages
through a block table (the KV caches of Sec. 2.1 as paged-attention engines keep them), against the fp64
oracle on the same keys gathered into the dense layout."""
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


def scatter_pages(k: torch.Tensor, block: int, layout: str, spare: int, rng, fill: float):
    """Per-layer pools holding the keys of dense k [B,L,Hkv,S,d] in pages of `block` keys placed at random
    in a pool with `spare` unused pages (filled with `fill`, never to be read), and the block table.
    Pools are indexed [page, key in page, kv head, d]; layout says how they lie in memory."""
    B, L, Hkv, S, d = k.shape
    nb = (S + block - 1) // block
    n_pages = B * nb + spare
    perm = rng.permutation(n_pages)[:B * nb].reshape(B, nb)
    table = torch.full((B, nb + 3), -7, dtype=torch.int32)          # entries past the last page: never read
    table[:, :nb] = torch.from_numpy(perm.astype(np.int32))
    pools, keep = [], []
    for l in range(L):
        if layout == "pbhd":      # [pages][block][Hkv][d], the usual layout
            buf = torch.full((n_pages, block, Hkv, d), fill, dtype=k.dtype, device=k.device)
            pool = buf
        elif layout == "phbd":    # [pages][Hkv][block][d]
            buf = torch.full((n_pages, Hkv, block, d), fill, dtype=k.dtype, device=k.device)
            pool = buf.permute(0, 2, 1, 3)
        else:
            raise ValueError(layout)
        for b in range(B):
            for i in range(nb):
                n = min(block, S - i * block)
                pool[perm[b, i], :n] = k[b, l, :, i * block:i * block + n].permute(1, 0, 2)
        pools.append(pool)
        keep.append(buf)
    return pools, table.cuda(), keep


# (name, B, L, Hq, Hkv, d, S, Tq, dtype, block, layout)
CASES = [
    ("paged-wide-16", 2, 4, 8, 2, 128, 900, 40, "bf16", 16, "pbhd"),
    ("paged-slim-16", 1, 5, 4, 2, 128, 2300, 2, "bf16", 16, "pbhd"),
    ("paged-mid-d64-8", 2, 3, 8, 2, 64, 1100, 12, "bf16", 8, "phbd"),
    ("paged-f16-64", 1, 3, 4, 2, 128, 700, 5, "f16", 64, "pbhd"),
    ("paged-big-pages", 1, 3, 4, 1, 64, 1000, 33, "bf16", 512, "phbd"),
    ("paged-tiny", 1, 2, 2, 1, 64, 3, 1, "bf16", 16, "pbhd"),
    ("paged-f32", 2, 3, 4, 2, 64, 300, 4, "f32", 16, "pbhd"),
    ("paged-d96-portable", 1, 3, 4, 2, 96, 200, 3, "bf16", 32, "phbd"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_paged_matches_oracle(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq, dtype, block, layout = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, rho_k=rho, seed=97)
    q, k = G.to_device(w)
    pools, table, keep = scatter_pages(k, block, layout, spare=5, rng=rng, fill=float("nan"))   # a wrong page, or an unmasked key past the last, wrecks the result
    want = oracle.pair_similarity(w.q, w.k)
    dense = G.gpu_scores(q, k)
    for fl in (0, kr.KRUL_FLAG_SINGLE_SPLIT, kr.KRUL_FLAG_GENERIC_KERNEL):
        out = kr.pair_similarity_paged(q, pools, table, S, flags=fl)
        torch.cuda.synchronize()
        got = {n: out[n].cpu().numpy() for n in ("pair_score", "head_score", "pair_dist")}
        e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score flags={fl}")
        G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"{name} pair_score flags={fl}")
        e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist flags={fl}")
        if fl == 0:   # same kernel, same order of operations: the addressing alone differs
            np.testing.assert_array_equal(got["head_score"], dense["head_score"])
            np.testing.assert_array_equal(got["pair_dist"], dense["pair_dist"])
        print(f"[{name} flags={fl}] paged max err head={e1:.2e} dist={e3:.2e}", flush=True)
    del keep


def test_paged_causal(G, oracle):
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, S, Tq = 1, 4, 8, 2, 128, 600, 33
    w = workloads.make("paged-causal", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", seed=99)
    q, k = G.to_device(w)
    pools, table, keep = scatter_pages(k, 16, "pbhd", 3, np.random.default_rng(1), float("nan"))
    want = oracle.pair_similarity(w.q, w.k, causal=True)
    out = kr.pair_similarity_paged(q, pools, table, S, flags=kr.KRUL_FLAG_CAUSAL)
    torch.cuda.synchronize()
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "paged causal head_score")
    G.assert_close(out["pair_dist"].cpu().numpy(), want["pair_dist"], G.TOL, "paged causal pair_dist")
    del keep


def test_paged_rejects_what_the_kernels_cannot_address(G):
    import paper_2507_08045_amd as kr
    q = torch.zeros((1, 2, 2, 1, 128), dtype=torch.bfloat16, device="cuda")
    table = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    pools = [torch.zeros((4, 16, 1, 128), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    kr.pair_similarity_paged(q, pools, table, 60)                       # fine
    with pytest.raises(kr.KrulError) as ei:                             # the table row is too short for 80 keys
        kr.pair_similarity_paged(q, pools, table, 80)
    assert ei.value.status == kr.KRUL_EINVAL
    bad = [torch.zeros((4, 12, 1, 128), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    with pytest.raises(kr.KrulError) as ei:                             # pages of 12 keys: not a power of two
        kr.pair_similarity_paged(q, bad, table, 40)
    assert ei.value.status == kr.KRUL_EINVAL
    torch.cuda.synchronize()
