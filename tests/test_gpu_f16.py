"""GPU parity with IEEE binary16 (float16) inputs -- the other 16-bit type models run in -- through every
entry point, against the fp64 oracle on the same bits."""
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


# (name, B, L, Hq, Hkv, d, S, Tq)
CASES = [
    ("f16-wide", 1, 4, 8, 2, 128, 700, 40),
    ("f16-mid-d64", 2, 3, 8, 2, 64, 1100, 12),
    ("f16-slim", 1, 5, 4, 2, 128, 2300, 2),
    ("f16-d96-portable", 1, 3, 4, 2, 96, 200, 3),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_adjacent_f16(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="f16", rho_k=rho, seed=91)
    assert w.q.dtype == np.float16
    q, k = G.to_device(w)
    want = oracle.pair_similarity(w.q, w.k)
    for fl in (0, kr.KRUL_FLAG_SINGLE_SPLIT, kr.KRUL_FLAG_GENERIC_KERNEL):
        got = G.gpu_scores(q, k, flags=fl)
        e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score flags={fl}")
        e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist flags={fl}")
        print(f"[{name} flags={fl}] max err head={e1:.2e} dist={e3:.2e}", flush=True)
    G.check_selection(oracle, got["pair_score"], want["pair_score"], max(1, L // 4))
    # the bits matter: the same values rounded to bfloat16 instead give other scores
    wb = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", rho_k=rho, seed=91)
    qb, kb = G.to_device(wb)
    other = G.gpu_scores(qb, kb)
    assert np.max(np.abs(other["head_score"] - got["head_score"])) > 1e-6


def test_other_entry_points_f16(G, oracle):
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, S, Tq = 1, 5, 8, 2, 128, 600, 33
    w = workloads.make("f16-all-entries", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="f16", seed=93,
                       sink_frac=0.02, sink_gain=3.0)
    q, k = G.to_device(w)
    # Initial-Recent layer test
    out = kr.pair_similarity_ir(q, k, 0.25)
    torch.cuda.synchronize()
    mass, el = oracle.ir_mass(w.q, w.k, 0.25)
    G.assert_close(out["ir_mass"].cpu().numpy(), mass, G.TOL, "f16 ir_mass")
    # causal reading
    got = G.gpu_scores(q, k, flags=kr.KRUL_FLAG_CAUSAL)
    want = oracle.pair_similarity(w.q, w.k, causal=True)
    G.assert_close(got["head_score"], want["head_score"], G.TOL, "f16 causal head_score")
    # keys left in per-layer caches
    layers = [k[:, l].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for l in range(L)]
    st = kr.pair_similarity_strided(q, layers)
    dense = kr.pair_similarity(q, k)
    torch.cuda.synchronize()
    assert torch.equal(st["head_score"], dense["head_score"])
    # every two layers
    ap = kr.all_pairs_similarity(q, k, want_head_score=True)
    torch.cuda.synchronize()
    want_ap = oracle.all_pairs(w.q, w.k)
    G.assert_close(ap["head_score"].cpu().numpy(), want_ap["head_score"], G.TOL, "f16 all-pairs head_score")
    G.assert_close(ap["pair_dist"].cpu().numpy(), want_ap["pair_dist"], G.TOL, "f16 all-pairs pair_dist")
    apg = kr.all_pairs_similarity(q, k, flags=kr.KRUL_FLAG_GENERIC_KERNEL)
    torch.cuda.synchronize()
    G.assert_close(apg["pair_score"].cpu().numpy(), want_ap["pair_score"], G.TOL, "f16 all-pairs (portable weights kernel)")
