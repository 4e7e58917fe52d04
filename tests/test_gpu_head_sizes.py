"""GPU parity for head sizes other than 64 and 128 on the matrix-core path (16-bit inputs, any multiple of 8
up to 128: the rows ride zero-padded in LDS), against the fp64 oracle: dense keys, per-layer caches with
strides, page pools; the causal reading, the Initial-Recent test and the selection ride along."""
import zlib

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


# (head_dim, dtype, B, L, Hq, Hkv, S, Tq): rows per kv head from 2 to 160, so every tile shape's short form
# and some ordinary ones are met
CASES = [
    (96, "bf16", 1, 4, 8, 2, 900, 40),
    (96, "f16", 2, 3, 8, 4, 1300, 1),
    (80, "bf16", 2, 4, 8, 2, 700, 12),
    (112, "bf16", 1, 3, 4, 4, 2100, 3),
    (120, "f16", 1, 3, 4, 2, 333, 20),
    (72, "bf16", 12, 3, 16, 8, 1300, 1),      # 288 workgroups of 512 keys: the ordinary 32-row shape
    (56, "bf16", 1, 4, 8, 2, 500, 40),        # below 64: the head_dim-64 kernels
    (40, "f16", 2, 3, 4, 4, 260, 9),
    (8, "bf16", 1, 3, 2, 1, 100, 5),
    (16, "bf16", 3, 2, 4, 2, 65, 33),
]


@pytest.mark.parametrize("case", CASES, ids=[f"d{c[0]}-{c[1]}-rows{(c[4] // c[5]) * c[7]}" for c in CASES])
def test_head_sizes_match_oracle(G, oracle, case):
    import paper_2507_08045_amd as kr
    d, dtype, B, L, Hq, Hkv, S, Tq = case
    name = f"head-size-{d}-{dtype}"
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, seed=500 + d,
                       rho_k=rng.uniform(0.4, 0.95, size=(B, L - 1, Hkv)))
    q, k = G.to_device(w)
    want = oracle.pair_similarity(w.q, w.k)
    keep_s = [k[:, l].permute(0, 2, 1, 3).contiguous() for l in range(L)]            # [B][S][Hkv][d] caches
    pools, table, keep_p = scatter_pages(k, 16, "pbhd", 3, rng, float("nan"))
    outs = {"dense": kr.pair_similarity(q, k),
            "strided": kr.pair_similarity_strided(q, [t.permute(0, 2, 1, 3) for t in keep_s]),
            "paged": kr.pair_similarity_paged(q, pools, table, S),
            "portable": kr.pair_similarity(q, k, flags=kr.KRUL_FLAG_GENERIC_KERNEL)}
    torch.cuda.synchronize()
    for src, out in outs.items():
        e = max(G.assert_close(out[n].cpu().numpy(), want[n], G.TOL, f"{name} {src} {n}")
                for n in ("head_score", "pair_score", "pair_dist"))
        print(f"[{name} {src}] max err {e:.2e}", flush=True)
    for n in ("head_score", "pair_dist"):      # same kernel, same order of operations, whatever the source
        np.testing.assert_array_equal(outs["strided"][n].cpu().numpy(), outs["dense"][n].cpu().numpy())
        np.testing.assert_array_equal(outs["paged"][n].cpu().numpy(), outs["dense"][n].cpu().numpy())
    # the by-products and the other readings
    ir = kr.pair_similarity_ir(q, k, 0.2)
    n_sel = L // 2
    sel = kr.pair_similarity_select(q, k, n_sel)
    torch.cuda.synchronize()
    want_mass, _ = oracle.ir_mass(w.q, w.k, 0.2)
    G.assert_close(ir["ir_mass"].cpu().numpy(), want_mass, G.TOL, f"{name} ir_mass")
    wp, wc = oracle.select_pairs(sel["pair_score"].cpu().numpy().astype(np.float64), n_sel)
    np.testing.assert_array_equal(sel["pairs"].cpu().numpy(), wp)
    if S >= Tq:
        wantc = oracle.pair_similarity(w.q, w.k, causal=True)
        gc = kr.pair_similarity(q, k, flags=kr.KRUL_FLAG_CAUSAL)
        torch.cuda.synchronize()
        G.assert_close(gc["head_score"].cpu().numpy(), wantc["head_score"], G.TOL, f"{name} causal")
    # every two layers, from dense keys and out of the pages
    want_ap = oracle.all_pairs(w.q, w.k)
    ap = kr.all_pairs_similarity(q, k, want_head_score=True)
    ap_paged = kr.all_pairs_similarity_in_place(q, kr.PagedKeys(pools, table, S), want_head_score=True)
    torch.cuda.synchronize()
    G.assert_close(ap["head_score"].cpu().numpy(), want_ap["head_score"], G.TOL, f"{name} all-pairs head_score")
    G.assert_close(ap["pair_dist"].cpu().numpy(), want_ap["pair_dist"], G.TOL, f"{name} all-pairs pair_dist")
    np.testing.assert_array_equal(ap_paged["head_score"].cpu().numpy(), ap["head_score"].cpu().numpy())
    del keep_s, keep_p


def test_strides_need_not_be_multiples_of_the_head_size(G, oracle):
    """Keys 136 elements apart (a cache row with 8 elements of something else after each key)."""
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, S, Tq = 1, 3, 4, 2, 128, 300, 7
    w = workloads.make("odd-stride", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", seed=601)
    q, k = G.to_device(w)
    bufs = [torch.full((B, Hkv, S, 136), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    for l in range(L):
        bufs[l][..., :128] = k[:, l]
    out = kr.pair_similarity_strided(q, [t[..., :128] for t in bufs])
    torch.cuda.synchronize()
    want = oracle.pair_similarity(w.q, w.k)
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "odd stride head_score")
    np.testing.assert_array_equal(out["head_score"].cpu().numpy(), kr.pair_similarity(q, k)["head_score"].cpu().numpy())
