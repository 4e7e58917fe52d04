"""GPU parity of every workgroup tile shape of the matrix-core kernel.  Which shape runs depends on the
rows per kv head (up to 32, up to 64, more) and on how many workgroups w of the ordinary shape the problem
has (few: a short form with fewer keys per tile; for up to 32 rows also a deep-ring form from 512 on), so
each case below is sized to land in one shape -- the small cases of the other parity tests all land in
the short forms."""
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


def w_of(B, Hq, Hkv, S, Tq):
    rk = (Hq // Hkv) * Tq
    if rk <= 64:
        return B * Hkv * ((S + 511) // 512)
    return B * Hkv * ((rk + 127) // 128) * ((S + 255) // 256)


# (name, B, L, Hq, Hkv, d, S, Tq, dtype, w, shape)
CASES = [
    ("slim-short", 2, 4, 16, 8, 128, 1300, 1, "bf16", 48, "32 x 256, four waves"),
    ("slim-short-d64-rows", 1, 3, 32, 8, 64, 2100, 4, "bf16", 40, "32 x 256, four waves"),
    ("slim", 12, 3, 16, 8, 128, 1300, 1, "bf16", 288, "32 x 512, eight waves"),
    ("slim-f16", 16, 3, 8, 8, 64, 1100, 2, "f16", 384, "32 x 512, eight waves"),
    ("slim-deep", 24, 3, 16, 8, 128, 1300, 1, "bf16", 576, "32 x 512, four waves, deep ring"),
    ("slim-deep-d64", 40, 3, 8, 8, 64, 700, 3, "bf16", 640, "32 x 512, four waves, deep ring"),
    ("mid-short", 2, 3, 16, 4, 128, 900, 12, "bf16", 16, "64 x 128, four waves"),
    ("mid-short-d64", 1, 4, 8, 8, 64, 1500, 40, "f16", 24, "64 x 128, four waves"),
    ("mid", 12, 3, 16, 8, 64, 700, 20, "bf16", 192, "64 x 512, eight waves"),
    ("mid-d128", 9, 3, 8, 8, 128, 1100, 50, "bf16", 216, "64 x 512, eight waves"),
    ("wide-short", 1, 3, 8, 2, 128, 700, 70, "bf16", 18, "128 x 128, eight waves"),
    ("wide-short-d64", 2, 3, 8, 4, 64, 400, 100, "bf16", 32, "128 x 128, eight waves"),
    ("wide", 6, 3, 8, 8, 64, 600, 90, "bf16", 144, "128 x 256, eight waves"),
    ("wide-d128", 9, 3, 4, 4, 128, 500, 130, "f16", 144, "128 x 256, eight waves"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_tile_shapes_match_oracle(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq, dtype, w, shape = case
    assert w_of(B, Hq, Hkv, S, Tq) == w   # (the thresholds: short forms up to 192 / 128 / 128, deep ring from 512)
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, rho_k=rho, seed=211)
    q, k = G.to_device(w)
    want = oracle.pair_similarity(w.q, w.k)
    got = G.gpu_scores(q, k)
    e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score")
    G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"{name} pair_score")
    e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist")
    print(f"[{name}: {shape}] max err head={e1:.2e} dist={e3:.2e}", flush=True)
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
