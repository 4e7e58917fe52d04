"""The arithmetic behind the parity tolerance of the kernels that keep exponentials in IEEE binary16 (CPU only).

Two kernels round exponentials to binary16 before a product: the many-query similarity kernel keeps the previous
layer's exponentials e = 2^(a - m) that way (reference exponent m between the row's maximum and 15 below it, so
1 <= max e <= 2^15) and uses them in the cross term only; the all-pairs path writes normalised exponentials e <= 1 as
binary16 and forms every sum from the rounded values.  Here the same roundings are applied to fp64 softmax rows in
numpy, on rows of the shapes the workloads have (flat, peaked, nearly one-hot, long with a tail far below the
binary16 normal range), and the change of the cosine is held against the bounds the tolerance is derived from:
2^-11 of the cosine for the cross-term-only scheme, twice that for the all-pairs scheme -- both inside the 2e-3 the
parity tests allow."""
import numpy as np
import pytest

EPS = 2.0 ** -11


def rows(rng, S, kind):
    """Two layers' logits (base-2 exponents) of one query row over S keys, correlated as adjacent layers are."""
    a = rng.standard_normal(S)
    b = 0.8 * a + 0.6 * rng.standard_normal(S)
    if kind == "flat":
        a, b = 0.2 * a, 0.2 * b
    elif kind == "peaked":
        a, b = 4.0 * a, 4.0 * b
    elif kind == "one-hot":
        a, b = 1.5 * a, 1.5 * b
        a[S // 3] += 40.0
        b[S // 3] += 38.0
        b[S // 2] += 37.5
    elif kind == "deep-tail":
        a, b = 3.0 * a - 30.0 * (np.arange(S) % 7 == 0), 3.0 * b - 28.0 * (np.arange(S) % 5 == 0)
    return a, b


def cosine(x, y):
    return float(np.dot(x, y) / np.sqrt(np.dot(x, x) * np.dot(y, y)))


@pytest.mark.parametrize("kind", ["flat", "peaked", "one-hot", "deep-tail"])
@pytest.mark.parametrize("S", [64, 4096, 16384])
@pytest.mark.parametrize("lift", [0.0, 15.0])   # how far the reference exponent sits below the row's maximum
def test_cross_term_with_binary16_copy_of_one_layer(kind, S, lift):
    rng = np.random.default_rng(S + len(kind))
    worst = 0.0
    for _ in range(8):
        a, b = rows(rng, S, kind)
        ea = np.exp2(a - a.max() + lift)     # previous layer: kept as binary16 for the cross term
        eb = np.exp2(b - b.max())            # this layer: fp32 in the kernel, exact here
        exact = cosine(ea, eb)
        ea16 = ea.astype(np.float16).astype(np.float64)
        assert np.all(np.isfinite(ea16))     # 2^15 is inside the binary16 range
        got = float(np.dot(ea16, eb) / np.sqrt(np.dot(ea, ea) * np.dot(eb, eb)))   # sums of squares unrounded
        worst = max(worst, abs(got - exact))
        assert abs(got - exact) <= EPS * exact + 1e-7, (kind, S, lift, got, exact)
    assert worst < 2e-3


@pytest.mark.parametrize("kind", ["flat", "peaked", "one-hot", "deep-tail"])
@pytest.mark.parametrize("S", [64, 4096, 16384])
def test_all_sums_from_binary16_weights(kind, S):
    rng = np.random.default_rng(7 * S + len(kind))
    for _ in range(8):
        a, b = rows(rng, S, kind)
        pa = np.exp2(a - a.max())
        pb = np.exp2(b - b.max())
        pa, pb = pa / pa.sum(), pb / pb.sum()          # attention weights (Sec. 2.1), at most 1
        exact = cosine(pa, pb)
        # the path rounds e = 2^(a - split maximum) <= 1; the normalisation is applied in fp32 afterwards
        ra = np.exp2(a - a.max()).astype(np.float16).astype(np.float64)
        rb = np.exp2(b - b.max()).astype(np.float16).astype(np.float64)
        got = cosine(ra, rb)
        assert abs(got - exact) <= 2 * EPS * max(exact, 0.05) + 1e-7, (kind, S, got, exact)
        assert abs(got - exact) < 2e-3
        # the distance of Alg. 1, formed from the same rounded values
        d_exact = float(np.sqrt(np.sum((pa - pb) ** 2)))
        na, nb = ra / ra.sum(), rb / rb.sum()
        d_got = float(np.sqrt(max(np.dot(na, na) + np.dot(nb, nb) - 2 * np.dot(na, nb), 0.0)))
        assert abs(d_got - d_exact) < 2e-3
