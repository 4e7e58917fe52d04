"""krul_pair_similarity_static -- the entry point for callers that cannot allocate -- through the C ABI,
against krul_pair_similarity on the same inputs: the same bits, on two calls in a row, the second on a
smaller input (the scratch area keeps the first call's contents), then once more in a shape that needs
another kernel.  A shape beyond the area's size is refused."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def _outs(B, L, Hq):
    return {"pair_score": torch.full((B, L - 1), -7.0, dtype=torch.float32, device="cuda"),
            "head_score": torch.full((B, L - 1, Hq), -7.0, dtype=torch.float32, device="cuda"),
            "pair_dist": torch.full((B, L - 1), -7.0, dtype=torch.float32, device="cuda")}


def test_static_scratch_matches_workspace_call(oracle):
    import gpu_util as G
    import paper_2507_08045_amd as kr
    cases = [
        workloads.make("na-1", B=2, L=6, Hq=8, Hkv=2, d=128, S=3000, Tq=40, dtype="bf16", rho_k=0.8, seed=71),
        workloads.make("na-2", B=1, L=4, Hq=8, Hkv=2, d=128, S=700, Tq=5, dtype="bf16", rho_k=0.6, seed=72),   # smaller
        workloads.make("na-3", B=1, L=3, Hq=2, Hkv=2, d=64, S=300, Tq=9, dtype="f32", rho_k=0.7, seed=73),     # portable kernel
    ]
    dev = [G.to_device(w) for w in cases]
    want = [kr.pair_similarity(q, k) for q, k in dev]
    outs = [_outs(w.B, w.L, w.Hq) for w in cases]
    torch.cuda.synchronize()
    # back to back on one stream, nothing between the calls
    for (q, k), o in zip(dev, outs):
        kr.pair_similarity_static(q, k, o)
    torch.cuda.synchronize()
    for w, o, ref in zip(cases, outs, want):
        for name in ("pair_score", "head_score", "pair_dist"):
            assert torch.equal(o[name], ref[name]), f"{w.name}: {name} differs from the workspace call"
        # and both against the oracle
        ow = oracle.pair_similarity(w.q, w.k)
        G.assert_close(o["head_score"].cpu().numpy(), ow["head_score"], G.TOL, f"{w.name} head_score")
        G.assert_close(o["pair_dist"].cpu().numpy(), ow["pair_dist"], G.TOL, f"{w.name} pair_dist")
    # cosine only (no head scores, no distance asked for)
    o = {"pair_score": torch.empty((2, 5), dtype=torch.float32, device="cuda")}
    kr.pair_similarity_static(*dev[0], o)
    torch.cuda.synchronize()
    np.testing.assert_allclose(o["pair_score"].cpu().numpy(), want[0]["pair_score"].cpu().numpy(), atol=1e-6)


def test_static_scratch_refuses_large_shapes():
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, S, Tq = 1, 32, 32, 8, 128, 8192, 2048     # needs 160 MiB
    shp = kr.KrulShape(B, L, Hq, Hkv, d, S, Tq, kr.KRUL_BF16, 0.0, 0)
    assert kr.workspace_bytes(shp) > kr.KRUL_STATIC_SCRATCH_BYTES
    q = torch.empty((B, L, Hq, Tq, d), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((B, L, Hkv, S, d), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(kr.KrulError) as ei:
        kr.pair_similarity_static(q, k, _outs(B, L, Hq))
    assert ei.value.status == kr.KRUL_ESCRATCH
