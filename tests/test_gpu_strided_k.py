"""GPU parity of krul_pair_similarity_strided: keys read in place from per-layer allocations with
strides (the KV caches of Sec. 2.1 as an inference engine keeps them), against the fp64 oracle on the
same keys gathered into the dense layout."""
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


def scatter_layers(k: torch.Tensor, layout: str, pad_tokens: int, pad_heads: int, fill: float):
    """Per-layer cache tensors holding the keys of dense k [B,L,Hkv,S,d], each a [B,Hkv,S,d] VIEW of
    a larger allocation whose other elements hold `fill` (never to be read)."""
    B, L, Hkv, S, d = k.shape
    views, keep = [], []
    for l in range(L):
        if layout == "bshd":       # [B][S+pad][Hkv+pad][d], the usual serving layout
            buf = torch.full((B, S + pad_tokens, Hkv + pad_heads, d), fill, dtype=k.dtype, device=k.device)
            v = buf[:, :S, :Hkv, :].permute(0, 2, 1, 3)
        elif layout == "bhsd":     # [B][Hkv+pad][S+pad][d]: room to grow
            buf = torch.full((B, Hkv + pad_heads, S + pad_tokens, d), fill, dtype=k.dtype, device=k.device)
            v = buf[:, :Hkv, :S, :]
        elif layout == "hbsd":     # heads outermost: the stride between conversations is the smaller one
            buf = torch.full((Hkv + pad_heads, B, S + pad_tokens, d), fill, dtype=k.dtype, device=k.device)
            v = buf[:Hkv, :, :S, :].permute(1, 0, 2, 3)
        else:
            raise ValueError(layout)
        v.copy_(k[:, l])
        views.append(v)
        keep.append(buf)
    return views, keep


# (name, B, L, Hq, Hkv, d, S, Tq, dtype, layout, pad_tokens, pad_heads)
CASES = [
    ("strided-wide-bshd", 2, 4, 8, 2, 128, 900, 40, "bf16", "bshd", 7, 1),
    ("strided-slim-bshd", 1, 5, 4, 2, 128, 2300, 2, "bf16", "bshd", 0, 0),
    ("strided-mid-d64-bhsd", 2, 3, 8, 2, 64, 1100, 12, "bf16", "bhsd", 100, 1),
    ("strided-hbsd", 3, 3, 4, 2, 128, 700, 5, "bf16", "hbsd", 1, 0),
    ("strided-tiny", 1, 2, 2, 1, 64, 3, 1, "bf16", "bshd", 0, 3),
    ("strided-f32", 2, 3, 4, 2, 64, 300, 4, "f32", "bshd", 3, 1),
    ("strided-d96-portable", 1, 3, 4, 2, 96, 200, 3, "bf16", "bshd", 2, 1),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_strided_matches_oracle(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq, dtype, layout, pt, ph = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, rho_k=rho, seed=23)
    q, k = G.to_device(w)
    views, keep = scatter_layers(k, layout, pt, ph, fill=1.0e4)   # a read of padding would wreck the softmax
    want = oracle.pair_similarity(w.q, w.k)
    dense = G.gpu_scores(q, k)
    for fl in (0, kr.KRUL_FLAG_SINGLE_SPLIT, kr.KRUL_FLAG_GENERIC_KERNEL):
        out = kr.pair_similarity_strided(q, views, flags=fl)
        torch.cuda.synchronize()
        got = {n: out[n].cpu().numpy() for n in ("pair_score", "head_score", "pair_dist")}
        e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score flags={fl}")
        G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"{name} pair_score flags={fl}")
        e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist flags={fl}")
        if fl == 0:   # same kernel, same order of operations: the addressing alone differs
            np.testing.assert_array_equal(got["head_score"], dense["head_score"])
            np.testing.assert_array_equal(got["pair_dist"], dense["pair_dist"])
        print(f"[{name} flags={fl}] strided max err head={e1:.2e} dist={e3:.2e}", flush=True)
    del keep


def test_strided_causal_and_table_reuse(G, oracle):
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, S, Tq = 1, 4, 8, 2, 128, 600, 33
    w = workloads.make("strided-causal", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", seed=29)
    q, k = G.to_device(w)
    views, keep = scatter_layers(k, "bshd", 9, 0, fill=1.0e4)
    want = oracle.pair_similarity(w.q, w.k, causal=True)
    out = kr.pair_similarity_strided(q, views, flags=kr.KRUL_FLAG_CAUSAL)
    out2 = kr.pair_similarity_strided(q, views, flags=kr.KRUL_FLAG_CAUSAL, k_table=out["k_table"],
                                      workspace=out["workspace"])
    torch.cuda.synchronize()
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "strided causal head_score")
    G.assert_close(out["pair_dist"].cpu().numpy(), want["pair_dist"], G.TOL, "strided causal pair_dist")
    assert torch.equal(out["head_score"], out2["head_score"])
    del keep


def test_strided_rejects_layouts_the_kernels_cannot_address(G):
    import paper_2507_08045_amd as kr
    q = torch.zeros((1, 2, 2, 1, 128), dtype=torch.bfloat16, device="cuda")
    # keys 136 elements apart: any multiple of 8 elements will do, on both kernels
    buf = torch.zeros((1, 1, 64, 136), dtype=torch.bfloat16, device="cuda")
    views = [buf[..., :128], buf[..., :128]]
    for fl in (0, kr.KRUL_FLAG_GENERIC_KERNEL):
        out = kr.pair_similarity_strided(q, views, flags=fl)
        torch.cuda.synchronize()
        assert torch.isfinite(out["pair_score"]).all()
    # a stride that is not a multiple of 8 elements
    buf2 = torch.zeros((1, 1, 64, 132), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(kr.KrulError) as ei:
        kr.pair_similarity_strided(q, [buf2[..., :128], buf2[..., :128]], flags=kr.KRUL_FLAG_GENERIC_KERNEL)
    assert ei.value.status == kr.KRUL_EINVAL
