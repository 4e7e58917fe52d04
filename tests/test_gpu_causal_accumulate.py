"""GPU parity of the causal reading (row t of the last Tq tokens sees keys j <= S - Tq + t) and of
token-wise accumulation over calls (Sec. 5, Sec. 7: prefill chunks and decode steps are scored as they
come and their similarities added up), against the fp64 oracle."""
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
CAUSAL_CASES = [
    ("causal-wide", 1, 4, 8, 2, 128, 700, 40),        # Rk = 160: rows of four heads in one wave tile
    ("causal-prefill", 1, 3, 4, 1, 128, 300, 300),    # S = Tq: a whole prompt as one chunk; row 0 sees one key
    ("causal-mid-d64", 2, 3, 4, 2, 64, 1030, 17),
    ("causal-slim", 1, 5, 4, 1, 128, 2500, 3),
    ("causal-decode", 1, 6, 8, 2, 64, 1111, 1),       # Tq = 1: the mask is empty
    ("causal-tiny", 1, 3, 4, 2, 128, 5, 5),
    ("causal-long-prefill", 1, 3, 4, 2, 128, 1500, 1500),   # row tiles left of the diagonal skip the keys right of it
]


@pytest.mark.parametrize("case", CAUSAL_CASES, ids=[c[0] for c in CAUSAL_CASES])
def test_causal_bf16(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", rho_k=rho, seed=17)
    q, k = G.to_device(w)
    want = oracle.pair_similarity(w.q, w.k, causal=True)
    for fl in (0, kr.KRUL_FLAG_SINGLE_SPLIT, kr.KRUL_FLAG_GENERIC_KERNEL):
        got = G.gpu_scores(q, k, flags=fl | kr.KRUL_FLAG_CAUSAL)
        e1 = G.assert_close(got["head_score"], want["head_score"], G.TOL, f"{name} head_score flags={fl}")
        G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"{name} pair_score flags={fl}")
        e3 = G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, f"{name} pair_dist flags={fl}")
        print(f"[{name} flags={fl}] causal max err head={e1:.2e} dist={e3:.2e}", flush=True)
    if Tq > 1:   # the mask matters
        plain = oracle.pair_similarity(w.q, w.k)
        assert np.max(np.abs(plain["head_score"] - want["head_score"])) > 1e-4


def test_causal_fp32_portable_kernel(G, oracle):
    import paper_2507_08045_amd as kr
    w = workloads.make("causal-f32", B=1, L=4, Hq=2, Hkv=2, d=64, S=256, Tq=16, dtype="f32", seed=19)
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k, flags=kr.KRUL_FLAG_CAUSAL)
    want = oracle.pair_similarity(w.q, w.k, causal=True)
    G.assert_close(got["head_score"], want["head_score"], G.TOL, "causal f32 head_score")
    G.assert_close(got["pair_dist"], want["pair_dist"], G.TOL, "causal f32 pair_dist")


def test_prefill_chunks_and_decode_steps_add_up(G, oracle):
    """A 200-token prompt scored in chunks of 128 + 72 tokens, then 3 decode steps, accumulated on the
    device, equals the oracle's token-wise mean over all 203 tokens (each token against the keys up to
    its own position)."""
    import paper_2507_08045_amd as kr
    B, L, Hq, Hkv, d, T = 1, 4, 8, 2, 128, 203
    w = workloads.make("stream", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=T, Tq=T, dtype="bf16", seed=23,
                       rho_k=np.array([0.9, 0.6, 0.8]).reshape(1, 3, 1))
    qd, kd = G.to_device(w)            # q [B,L,Hq,T,d], k [B,L,Hkv,T,d]: one token's query and key per position
    head_sum = torch.zeros((B, L - 1, Hq), dtype=torch.float32, device="cuda")
    dist_sum = torch.zeros_like(head_sum)
    pos = 0
    for n in (128, 72, 1, 1, 1):
        qc = qd[:, :, :, pos:pos + n].contiguous()
        kc = kd[:, :, :, :pos + n].contiguous()
        kr.pair_similarity_accumulate(qc, kc, head_sum, dist_sum, flags=kr.KRUL_FLAG_CAUSAL)
        pos += n
    assert pos == T
    out = kr.pair_scores_from_sums(head_sum, T, dist_sum)
    torch.cuda.synchronize()
    want = oracle.pair_similarity(w.q, w.k, causal=True)     # S = Tq = T: row t sees keys <= t
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "stream head_score")
    G.assert_close(out["pair_score"].cpu().numpy(), want["pair_score"], G.TOL, "stream pair_score")
    G.assert_close(out["pair_dist"].cpu().numpy(), want["pair_dist"], G.TOL, "stream pair_dist")
    # one call over the whole prompt gives the same scores
    one = G.gpu_scores(qd, kd, flags=kr.KRUL_FLAG_CAUSAL)
    assert np.max(np.abs(one["head_score"] - out["head_score"].cpu().numpy())) < 1e-5
    G.check_selection(oracle, out["pair_score"].cpu().numpy(), want["pair_score"], 1)


def test_accumulate_without_distance_and_without_mask(G, oracle):
    # two disjoint sets of query rows against the same keys, cosine sums only
    import paper_2507_08045_amd as kr
    w = workloads.make("acc-plain", B=2, L=3, Hq=4, Hkv=2, d=64, S=515, Tq=33, dtype="bf16", seed=29)
    qd, kd = G.to_device(w)
    head_sum = torch.zeros((2, 2, 4), dtype=torch.float32, device="cuda")
    kr.pair_similarity_accumulate(qd[:, :, :, :20].contiguous(), kd, head_sum)
    kr.pair_similarity_accumulate(qd[:, :, :, 20:].contiguous(), kd, head_sum)
    out = kr.pair_scores_from_sums(head_sum, 33)
    torch.cuda.synchronize()
    assert out["pair_dist"] is None
    want = oracle.pair_similarity(w.q, w.k)
    G.assert_close(out["head_score"].cpu().numpy(), want["head_score"], G.TOL, "acc head_score")
    G.assert_close(out["pair_score"].cpu().numpy(), want["pair_score"], G.TOL, "acc pair_score")


def test_causal_c2_shape_sampled(G, oracle):
    # the C2 shape read as a 64-token chunk at the end of a 4096-token sequence
    import paper_2507_08045_amd as kr
    w = workloads.config("C2")
    q, k = G.to_device(w)
    got = G.gpu_scores(q, k, flags=kr.KRUL_FLAG_CAUSAL, want_pair_dist=False)
    rng = np.random.default_rng(6)
    units = np.stack([np.zeros(24, dtype=np.int64), rng.integers(0, w.L - 1, 24), rng.integers(0, w.Hq, 24)], axis=1)
    hc, _ = oracle.unit_scores(w.q, w.k, units, causal=True)
    gpu_vals = np.array([got["head_score"][b, l, h] for b, l, h in units])
    err = np.max(np.abs(gpu_vals - hc))
    print(f"[C2 causal] 24 sampled units: max |gpu - oracle| = {err:.2e}", flush=True)
    assert err <= G.TOL
