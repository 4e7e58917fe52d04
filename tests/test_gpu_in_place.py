"""GPU parity of the accumulating call and the Initial-Recent call on keys read in place (per-layer caches
with strides, or page pools behind a block table): the token-wise scoring of Sec. 5 as it runs beside decoding,
against the fp64 oracle on the same keys in the dense layout."""
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


def bshd_layers(k):
    """Per-layer [B][S][Hkv][d] caches holding dense k [B,L,Hkv,S,d], as [B,Hkv,S,d] views."""
    keep = [k[:, l].permute(0, 2, 1, 3).contiguous() for l in range(k.shape[1])]
    return [t.permute(0, 2, 1, 3) for t in keep]


def test_prefill_chunks_and_decode_steps_on_a_paged_cache(G, oracle):
    """A conversation scored as it is served: two prefill chunks, then decode steps one token at a time,
    every call on the page pools as they stand (the cache grows, the pools do not move); the sums equal
    the oracle's token-wise mean over all tokens."""
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, block = 2, 4, 8, 2, 128, 16
    S_all = 180
    w = workloads.make("in-place-serving", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S_all, Tq=S_all, dtype="bf16", seed=401)
    q_all, k_all = G.to_device(w)                                   # row t is the token at position t
    pools, table, keep = scatter_pages(k_all, block, "pbhd", 4, np.random.default_rng(5), float("nan"))
    head_sum = torch.zeros((B, L - 1, Hq), dtype=torch.float32, device="cuda")
    dist_sum = torch.zeros_like(head_sum)
    pos = 0
    for n in (100, 77, 1, 1, 1):                                   # chunk lengths; the last three are decode steps
        q = q_all[:, :, :, pos:pos + n].contiguous()
        keys = kr.PagedKeys(pools, table, pos + n)                  # the conversation so far
        kr.pair_similarity_accumulate_in_place(q, keys, head_sum, dist_sum, flags=kr.KRUL_FLAG_CAUSAL)
        pos += n
    assert pos == S_all
    got = kr.pair_scores_from_sums(head_sum, pos, dist_sum)
    torch.cuda.synchronize()
    want = oracle.pair_similarity(w.q, w.k, causal=True)            # all rows, each seeing its own past
    G.assert_close(got["head_score"].cpu().numpy(), want["head_score"], G.TOL, "paged token-wise head_score")
    G.assert_close(got["pair_score"].cpu().numpy(), want["pair_score"], G.TOL, "paged token-wise pair_score")
    G.assert_close(got["pair_dist"].cpu().numpy(), want["pair_dist"], G.TOL, "paged token-wise pair_dist")
    del keep


@pytest.mark.parametrize("dtype,d,flag", [("bf16", 128, 0), ("f16", 64, 0), ("bf16", 128, "generic"), ("f32", 64, 0)])
def test_accumulate_and_ir_equal_the_dense_calls(G, oracle, dtype, d, flag):
    import paper_2507_08045_amd as kr
    flags = kr.KRUL_FLAG_GENERIC_KERNEL if flag == "generic" else 0
    B, L, Hq, Hkv, S, Tq = 2, 5, 8, 4, 700, 6
    w = workloads.make(f"in-place-{dtype}-{d}-{flag}", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, seed=402)
    q, k = G.to_device(w)
    pools, table, keep = scatter_pages(k, 32, "phbd", 2, np.random.default_rng(6), float("nan"))
    sources = {"dense": k, "strided": kr.StridedKeys(bshd_layers(k)), "paged": kr.PagedKeys(pools, table, S)}
    ref_ir = kr.pair_similarity_ir(q, k, 0.25, flags=flags)
    ref_sum = torch.zeros((B, L - 1, Hq), dtype=torch.float32, device="cuda")
    ref_dist = torch.zeros_like(ref_sum)
    kr.pair_similarity_accumulate(q, k, ref_sum, ref_dist, flags=flags)
    torch.cuda.synchronize()
    want_mass, want_el = oracle.ir_mass(w.q, w.k, 0.25)
    G.assert_close(ref_ir["ir_mass"].cpu().numpy(), want_mass, G.TOL, "dense ir_mass")
    for name, keys in sources.items():
        out = kr.pair_similarity_ir_in_place(q, keys, 0.25, flags=flags)
        hs = torch.zeros_like(ref_sum)
        hd = torch.zeros_like(ref_sum)
        kr.pair_similarity_accumulate_in_place(q, keys, hs, hd, flags=flags)
        torch.cuda.synchronize()
        for n in ("pair_score", "head_score", "pair_dist", "ir_mass", "eligible"):     # same kernels, same order
            np.testing.assert_array_equal(out[n].cpu().numpy(), ref_ir[n].cpu().numpy(), err_msg=f"{name} {n}")
        np.testing.assert_array_equal(hs.cpu().numpy(), ref_sum.cpu().numpy(), err_msg=f"{name} head_sum")
        np.testing.assert_array_equal(hd.cpu().numpy(), ref_dist.cpu().numpy(), err_msg=f"{name} head_dist_sum")
    del keep


@pytest.mark.parametrize("dtype,d,S,Tq,flag", [("bf16", 128, 700, 40, 0), ("f16", 64, 300, 5, 0), ("bf16", 128, 2080, 2, "causal"),
                                              ("f32", 64, 256, 16, 0), ("bf16", 96, 200, 3, 0)])
def test_all_pairs_in_place(G, oracle, dtype, d, S, Tq, flag):
    """Every two layers scored on keys read in place: the same bits as the dense call, and the oracle's values."""
    import paper_2507_08045_amd as kr
    flags = kr.KRUL_FLAG_CAUSAL if flag == "causal" else 0
    B, L, Hq, Hkv = 2, 6, 8, 2
    w = workloads.make(f"ap-in-place-{dtype}-{d}", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, seed=403)
    q, k = G.to_device(w)
    pools, table, keep = scatter_pages(k, 16, "pbhd", 3, np.random.default_rng(7), float("nan"))
    ref = kr.all_pairs_similarity(q, k, flags=flags, want_head_score=True)
    torch.cuda.synchronize()
    want = oracle.all_pairs(w.q, w.k, causal=bool(flags))
    G.assert_close(ref["head_score"].cpu().numpy(), want["head_score"], G.TOL, "dense all-pairs head_score")
    for name, keys in {"dense": k, "strided": kr.StridedKeys(bshd_layers(k)), "paged": kr.PagedKeys(pools, table, S)}.items():
        out = kr.all_pairs_similarity_in_place(q, keys, flags=flags, want_head_score=True)
        torch.cuda.synchronize()
        for n in ("pair_score", "pair_dist", "head_score"):
            np.testing.assert_array_equal(out[n].cpu().numpy(), ref[n].cpu().numpy(), err_msg=f"{name} {n}")
    del keep


def test_in_place_calls_want_exactly_one_source(G):
    import ctypes
    import paper_2507_08045_amd as kr
    q = torch.zeros((1, 2, 2, 1, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((1, 2, 1, 40, 128), dtype=torch.bfloat16, device="cuda")
    shp = kr.make_shape(q, k)
    ws = torch.empty(kr.workspace_bytes(shp), dtype=torch.uint8, device="cuda")
    hs = torch.zeros((1, 1, 2), dtype=torch.float32, device="cuda")
    lay = kr.KrulKLayout(0x1000, 0, 5120, 128)
    vp = ctypes.c_void_p
    for ks in (kr.KrulKeys(None, None, None), kr.KrulKeys(k.data_ptr(), ctypes.pointer(lay), None)):
        rc = kr.lib().krul_pair_similarity_accumulate_in_place(ctypes.byref(shp), vp(q.data_ptr()), ctypes.byref(ks),
                                                               vp(hs.data_ptr()), None, vp(ws.data_ptr()), ws.numel(), None)
        assert rc == kr.KRUL_EINVAL
    torch.cuda.synchronize()
