"""GPU parity of the Initial-Recent layer test (Sec. 4.2, Alg. 1 first loop), computed in the
same pass as the similarity scores, against the fp64 oracle (which materialises the attention
rows and adds up the mass on the first and last tenth of the keys)."""
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


def run_ir(G, oracle, w, gamma, flags=0):
    import paper_2507_08045_amd as kr
    q, k = G.to_device(w)
    out = kr.pair_similarity_ir(q, k, gamma, flags=flags)
    torch.cuda.synchronize()
    mass = out["ir_mass"].cpu().numpy()
    el = out["eligible"].cpu().numpy()
    want_mass, want_el = oracle.ir_mass(w.q, w.k, gamma)
    err = G.assert_close(mass, want_mass, G.TOL, f"{w.name} ir_mass")
    # the decision must agree wherever the mass is further from gamma than the tolerance;
    # and it is exactly the device's own mass compared with gamma
    np.testing.assert_array_equal(el, (mass >= np.float32(gamma)).astype(np.uint8))
    clear = np.abs(want_mass - gamma) > G.TOL
    np.testing.assert_array_equal(el[clear], want_el[clear])
    # the similarity outputs are those of the plain call
    ref = G.gpu_scores(q, k, flags=flags)
    for name in ("pair_score", "head_score", "pair_dist"):
        assert np.max(np.abs(out[name].cpu().numpy() - ref[name])) < 1e-6, name
    print(f"[{w.name} flags={flags}] ir_mass max err {err:.2e}; mass range [{want_mass.min():.3f}, {want_mass.max():.3f}]",
          flush=True)
    return out, want_mass, want_el


def test_c1_fp32(G, oracle):
    w = workloads.config("C1")
    run_ir(G, oracle, w, 0.2)


# (name, B, L, Hq, Hkv, d, S, Tq): region boundaries fall inside 32-key blocks and inside tiles
IR_CASES = [
    ("ir-wide", 1, 4, 8, 2, 128, 700, 40),       # boundaries at keys 70 and 630
    ("ir-mid-d64", 2, 3, 4, 1, 64, 1030, 33),    # 103 and 927
    ("ir-slim", 1, 5, 4, 1, 128, 2500, 3),       # 250 and 2250: several tiles
    ("ir-short", 1, 3, 4, 2, 128, 9, 40),        # floor(0.9) = 0 initial keys, recent = key 8 only
    ("ir-one-key", 1, 2, 2, 2, 64, 1, 2),        # S = 1: the one key is recent, mass 1
]


@pytest.mark.parametrize("case", IR_CASES, ids=[c[0] for c in IR_CASES])
def test_bf16_cases(G, oracle, case):
    import paper_2507_08045_amd as kr
    name, B, L, Hq, Hkv, d, S, Tq = case
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rho = rng.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    w = workloads.make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype="bf16", rho_k=rho, seed=13)
    _, want_mass, _ = run_ir(G, oracle, w, 0.2)
    run_ir(G, oracle, w, float(np.median(want_mass)), flags=kr.KRUL_FLAG_SINGLE_SPLIT)   # multi-tile path
    run_ir(G, oracle, w, 0.2, flags=kr.KRUL_FLAG_GENERIC_KERNEL)


def test_uniform_keys_give_the_region_fraction(G, oracle):
    # identical keys => uniform attention => mass = (floor(0.1 S) + S - floor(0.9 S)) / S exactly
    import paper_2507_08045_amd as kr
    w = workloads.make("ir-uniform", B=1, L=3, Hq=4, Hkv=2, d=128, S=1000, Tq=40, dtype="bf16", seed=5)
    k = w.k.copy()
    k[...] = k[:, :, :, :1, :]
    q, kd = G.arrays_to_device(w.q, k)
    out = kr.pair_similarity_ir(q, kd, 0.5)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out["ir_mass"].cpu().numpy(), (100 + 1000 - 900) / 1000, atol=1e-5)
    assert not out["eligible"].cpu().numpy().any()


def test_sinks_raise_the_mass_and_feed_the_selector(G, oracle):
    # layers whose first keys are scaled up put their mass on T_initial: they pass the test,
    # the others do not; the selector then only pairs layers that passed
    import paper_2507_08045_amd as kr
    w = workloads.make("ir-sinks", B=1, L=6, Hq=4, Hkv=2, d=128, S=1200, Tq=40, dtype="bf16", seed=21,
                       rho_k=np.full((1, 5, 1), 0.9))
    kf = workloads.bf16_bits_to_f32(w.k).copy()
    for l in (0, 1, 4, 5):
        kf[:, l, :, :4, :] *= 6.0
    k = workloads.f32_to_bf16_bits(kf)
    q, kd = G.arrays_to_device(w.q, k)
    out = kr.pair_similarity_ir(q, kd, 0.5)
    torch.cuda.synchronize()
    want_mass, want_el = oracle.ir_mass(w.q, k, 0.5)
    G.assert_close(out["ir_mass"].cpu().numpy(), want_mass, G.TOL, "sinks ir_mass")
    el = out["eligible"].cpu().numpy()
    np.testing.assert_array_equal(el, want_el)
    assert el[0].tolist() == [1, 1, 0, 0, 1, 1]
    pairs, count = kr.select_pairs(out["pair_score"], 3, eligible=out["eligible"])
    torch.cuda.synchronize()
    wp, wc = oracle.select_pairs(out["pair_score"].cpu().numpy().astype(np.float64), 3, eligible=want_el)
    np.testing.assert_array_equal(pairs.cpu().numpy(), wp)
    np.testing.assert_array_equal(count.cpu().numpy(), wc)
    assert sorted(p for p in pairs.cpu().numpy()[0].tolist() if p >= 0) == [0, 4]


def test_c2_full_size(G, oracle):
    w = workloads.config("C2")
    run_ir(G, oracle, w, 0.21)
