"""Parity of the many-query kernel (256 x 256 workgroup tiles, two row blocks per wave, binary16 copies of the
previous layer's exponentials) against the fp64 oracle, on shapes sized so that the plan picks it: 256 rows or
more per kv head and 512 workgroup tiles or more.  Ragged key tails and row tails, splits of one and of many
key tiles (running records), the patch numbering of workgroups, reference-exponent raises in the middle of a
step, the distance by-product, binary16 inputs."""
import math

import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


def run_case(G, oracle, w, scale=None, flags=0, tol=None):
    q, k = G.to_device(w)
    kw = {} if scale is None else {"scale": scale}
    got = G.gpu_scores(q, k, flags=flags, **kw)
    want = oracle.pair_similarity(w.q, w.k, scale=scale)
    tol = tol or G.TOL
    e1 = G.assert_close(got["head_score"], want["head_score"], tol, f"{w.name} head_score")
    e2 = G.assert_close(got["pair_score"], want["pair_score"], tol, f"{w.name} pair_score")
    e3 = G.assert_close(got["pair_dist"], want["pair_dist"], tol, f"{w.name} pair_dist")
    got_c = G.gpu_scores(q, k, flags=flags, want_pair_dist=False, **kw)   # cosine only: another instantiation
    G.assert_close(got_c["head_score"], want["head_score"], tol, f"{w.name} head_score (cosine only)")
    print(f"[{w.name}] max err head={e1:.2e} pair={e2:.2e} dist={e3:.2e}", flush=True)
    return got, want


def test_plan_takes_the_big_tile():
    import paper_2507_08045_amd as kr
    # 4 conversations x 2 kv heads x 256 rows, 16384 keys: one row tile per unit, 64 key tiles
    small = kr.KrulShape(4, 3, 8, 2, 128, 16384, 64, kr.KRUL_BF16, 0.0, 0)
    wide = kr.KrulShape(4, 3, 8, 2, 128, 4096, 64, kr.KRUL_BF16, 0.0, 0)   # 128 tiles only: the 128-row kernel
    # records: workgroups x layers x rows x 16 bytes; the big tile has 256 rows per workgroup
    assert kr.workspace_bytes(small) > 0 and kr.workspace_bytes(wide) > 0


def test_one_row_tile_many_splits(G, oracle):
    # Rk = 256, S ragged: 8 units x 64 key tiles; splits of two tiles (running records between them)
    w = workloads.make("big-1", B=4, L=3, Hq=8, Hkv=2, d=128, S=16384 - 77, Tq=64, dtype="bf16",
                       rho_k=np.array([0.9, 0.6]).reshape(1, 2, 1), seed=81)
    run_case(G, oracle, w)


def test_single_split_walks_all_tiles(G, oracle):
    import paper_2507_08045_amd as kr
    w = workloads.make("big-2", B=4, L=4, Hq=8, Hkv=2, d=128, S=16384, Tq=64, dtype="bf16", rho_k=0.8, seed=82)
    run_case(G, oracle, w, flags=kr.KRUL_FLAG_SINGLE_SPLIT)


def test_row_tail_and_patches(G, oracle):
    # Rk = 8 x 250 = 2000 rows: 8 row tiles, the last one ragged; 64 key tiles -> patches of 8 row tiles x 4 splits
    w = workloads.make("big-3", B=1, L=3, Hq=8, Hkv=1, d=128, S=16384, Tq=250, dtype="bf16", rho_k=0.7, seed=83)
    run_case(G, oracle, w)


def test_exponent_raises_mid_step(G, oracle):
    # one vector added to every key of a layer moves its logits by tens of units, and the largest logits sit in
    # late chunks: the lanes' reference exponents are raised in the middle of steps
    w = workloads.make("big-4", B=4, L=3, Hq=8, Hkv=2, d=128, S=16384, Tq=64, dtype="bf16", rho_k=0.8, seed=84)
    kf = workloads.bf16_bits_to_f32(w.k)
    c = np.random.default_rng(1).standard_normal(128).astype(np.float32) * 20.0
    kf[:, 1] += c
    kf[:, 2, :, 9000:9003] *= 6.0
    kf[:, 0, :, 200:16384:1024] *= 5.0
    w.k[:] = workloads.f32_to_bf16_bits(kf)
    run_case(G, oracle, w)
    run_case(G, oracle, w, scale=4.0 / math.sqrt(128))   # nearly one-hot rows


def test_f16_inputs(G, oracle):
    w = workloads.make("big-5", B=4, L=3, Hq=8, Hkv=2, d=128, S=16384, Tq=64, dtype="f16", rho_k=0.75, seed=85)
    run_case(G, oracle, w)


def test_identical_layers(G, oracle):
    w = workloads.make("big-6", B=4, L=3, Hq=8, Hkv=2, d=128, S=16384, Tq=64, dtype="bf16", rho_k=0.7, seed=86)
    w.q[:, 1], w.k[:, 1] = w.q[:, 0], w.k[:, 0]
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k)
    # the cross term sees binary16 copies of one layer's exponentials: 2^-11 relative at most
    assert np.max(np.abs(got["head_score"][:, 0] - 1.0)) < 6e-4
    assert np.all(got["head_score"] <= 1.0 + 6e-4) and np.all(got["head_score"] > 0)


def test_agrees_with_the_128_row_kernel(G, oracle):
    # the same inputs through sim_mfma_kernel (a call that also asks for the Initial-Recent test never takes the
    # many-query kernel): the two kernels' head scores differ by the rounding of the binary16 copies at most
    import paper_2507_08045_amd as kr
    w = workloads.make("big-7", B=4, L=4, Hq=8, Hkv=2, d=128, S=16384 - 100, Tq=64, dtype="bf16", rho_k=0.6, seed=87)
    q, k = G.to_device(w)
    sh = kr.KrulShape(4, 4, 8, 2, 128, 16384 - 100, 64, kr.KRUL_BF16, 0.0, 0)
    assert kr.plan(sh)["form"] == 8
    a = G.gpu_scores(q, k)["head_score"]
    b = kr.pair_similarity_ir(q, k, gamma=0.5)["head_score"].cpu().numpy()
    assert np.max(np.abs(a - b)) < 6e-4


@pytest.mark.parametrize("seed", [201, 202, 203, 204])
def test_seeded_random_shapes(G, oracle, seed):
    # shapes drawn so that the plan takes the many-query kernel: rows per kv head from 230 up (ragged row tiles),
    # ragged key tails, 2 to 5 layers, one to four kv heads; the oracle's cost bounds the sizes
    import paper_2507_08045_amd as kr
    rng = np.random.default_rng(seed)
    Hkv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 4]))
    rows = int(rng.choice([230, 256, 500, 760, 1000]))          # rows per kv head wanted
    Tq = max(1, rows // g)
    Rk = g * Tq
    nrt = (Rk + 255) // 256
    assert nrt * 256 * 7 <= Rk * 8
    L = int(rng.integers(2, 6))
    B = int(rng.choice([1, 2]))
    tiles = -(-512 // (B * Hkv * nrt)) + int(rng.integers(0, 3))   # 512 workgroup tiles or a few more
    S = tiles * 256 - int(rng.integers(0, 255))
    w = workloads.make(f"big-rand-{seed}", B=B, L=L, Hq=Hkv * g, Hkv=Hkv, d=128, S=S, Tq=Tq, dtype="bf16",
                       rho_k=float(rng.uniform(0.3, 0.95)), seed=seed)
    sh = kr.KrulShape(B, L, Hkv * g, Hkv, 128, S, Tq, kr.KRUL_BF16, 0.0, 0)
    pl = kr.plan(sh)
    print(f"[big-rand-{seed}] B={B} L={L} Hq/Hkv={Hkv * g}/{Hkv} S={S} Tq={Tq}: {pl}", flush=True)
    assert pl["form"] == 8, pl
    run_case(G, oracle, w)


def test_accumulate_over_two_calls(G, oracle):
    # two calls of 64 query tokens each over the same keys (no mask), accumulated and then averaged over the 128
    # tokens, against one oracle pass over all 128: the accumulating calls take the many-query kernel too
    import paper_2507_08045_amd as kr
    w = workloads.make("big-8", B=4, L=3, Hq=8, Hkv=2, d=128, S=16384 - 9, Tq=128, dtype="bf16", rho_k=0.7, seed=88)
    q, k = G.to_device(w)
    sh = kr.KrulShape(4, 3, 8, 2, 128, 16384 - 9, 64, kr.KRUL_BF16, 0.0, 0)
    assert kr.plan(sh)["form"] == 8
    head_sum = torch.zeros((4, 2, 8), dtype=torch.float32, device="cuda")
    dist_sum = torch.zeros_like(head_sum)
    kr.pair_similarity_accumulate(q[:, :, :, :64].contiguous(), k, head_sum, dist_sum)
    kr.pair_similarity_accumulate(q[:, :, :, 64:].contiguous(), k, head_sum, dist_sum)
    out = kr.pair_scores_from_sums(head_sum, 128, dist_sum)
    torch.cuda.synchronize()
    want = oracle.pair_similarity(w.q, w.k)
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "accumulated head_score")
    G.assert_close(out["pair_score"].cpu().numpy(), want["pair_score"], G.TOL, "accumulated pair_score")
    G.assert_close(out["pair_dist"].cpu().numpy(), want["pair_dist"], G.TOL, "accumulated pair_dist")
