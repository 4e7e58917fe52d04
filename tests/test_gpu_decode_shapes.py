"""GPU parity of the three workgroup shapes that serve up to 32 query rows per kv head (decode steps and
short chunks; the token-wise scoring of Sec. 5): which one runs depends on how many 512-key workgroups the
problem has (fewer than 256, 256..511, 512 or more), so each case below is sized to land in one of them."""
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


# (name, B, L, Hq, Hkv, d, S, Tq, dtype, 512-key workgroups = B * Hkv * ceil(S / 512))
CASES = [
    ("few-workgroups", 2, 4, 16, 8, 128, 1300, 1, "bf16", 48),          # 256-key tiles, four waves
    ("few-workgroups-d64-rows", 1, 3, 32, 8, 64, 2100, 4, "bf16", 40),   # ... 16 rows per kv head
    ("one-round", 12, 3, 16, 8, 128, 1300, 1, "bf16", 288),              # 512-key tiles, eight waves
    ("one-round-f16", 16, 3, 8, 8, 64, 1100, 2, "f16", 384),
    ("many-rounds", 24, 3, 16, 8, 128, 1300, 1, "bf16", 576),            # 512-key tiles, four waves, deep ring
    ("many-rounds-d64", 40, 3, 8, 8, 64, 700, 3, "bf16", 640),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_decode_shapes_match_oracle(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq, dtype, wgs = case
    assert B * Hkv * ((S + 511) // 512) == wgs and (Hq // Hkv) * Tq <= 32
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, rho_k=rho, seed=211)
    q, k = G.to_device(w)
    want = oracle.pair_similarity(w.q, w.k)
    got = G.gpu_scores(q, k)
    e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score")
    G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"{name} pair_score")
    e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist")
    print(f"[{name}] max err head={e1:.2e} dist={e3:.2e}", flush=True)
    # the Initial-Recent test and the causal reading ride in the same kernels
    ir = kr.pair_similarity_ir(q, k, 0.2)
    torch.cuda.synchronize()
    want_mass, _ = oracle.ir_mass(w.q, w.k, 0.2)
    G.assert_close(ir["ir_mass"].cpu().numpy(), want_mass, G.TOL, f"{name} ir_mass")
    if Tq > 1:
        wc = oracle.pair_similarity(w.q, w.k, causal=True)
        gc = G.gpu_scores(q, k, flags=kr.KRUL_FLAG_CAUSAL)
        G.assert_close(gc["head_score"], wc["head_score"], G.TOL, f"{name} causal head_score")
    # one workgroup walking all key tiles (running records parked in memory between tiles)
    one = G.gpu_scores(q, k, flags=kr.KRUL_FLAG_SINGLE_SPLIT)
    G.assert_close(one["head_score"], want["head_score"], G.TOL, f"{name} single split")
