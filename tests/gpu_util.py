"""Helpers for the GPU parity tests: run a workload through the C ABI (via the thin
binding) and through the fp64 oracle, and compare."""
import numpy as np
import torch

import paper_2507_08045_amd as kr
import workloads

TOL = 2e-3   # absolute tolerance on similarities (cosine and distance), from the benchmark spec


def to_device(w: workloads.Workload):
    if w.dtype in ("f32", "f16"):
        q = torch.from_numpy(w.q).cuda()
        k = torch.from_numpy(w.k).cuda()
    else:
        q = torch.from_numpy(w.q.view(np.int16)).cuda().view(torch.bfloat16)
        k = torch.from_numpy(w.k.view(np.int16)).cuda().view(torch.bfloat16)
    return q, k


def arrays_to_device(q: np.ndarray, k: np.ndarray):
    if q.dtype in (np.float32, np.float16):
        return torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda()
    return (torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16),
            torch.from_numpy(k.view(np.int16)).cuda().view(torch.bfloat16))


def gpu_scores(q, k, **kw):
    out = kr.pair_similarity(q, k, **kw)
    torch.cuda.synchronize()
    return {n: (None if out[n] is None else out[n].cpu().numpy()) for n in ("pair_score", "head_score", "pair_dist")}


def assert_close(got, want, tol=TOL, what=""):
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.max(np.abs(got - want))
    assert err <= tol, f"{what}: max |gpu - oracle| = {err:.3e} > {tol}"
    return err


def check_selection(oracle, gpu_pair_score, oracle_pair_score, n_select):
    """The selector run on the GPU scores must equal the oracle selector on the same
    fp32 scores bit for bit.  It must also equal the oracle's own end-to-end choice
    whenever the two score vectors are certain to sort alike: every two oracle scores of a
    conversation further apart than twice the error observed between GPU and oracle scores
    (then no two candidates can have changed places, so the scan sees the same list)."""
    ps = torch.from_numpy(np.ascontiguousarray(gpu_pair_score, dtype=np.float32)).cuda()
    pairs, count = kr.select_pairs(ps, n_select)
    torch.cuda.synchronize()
    pairs, count = pairs.cpu().numpy(), count.cpu().numpy()
    want_pairs, want_count = oracle.select_pairs(np.asarray(gpu_pair_score, dtype=np.float64), n_select)
    np.testing.assert_array_equal(pairs, want_pairs)
    np.testing.assert_array_equal(count, want_count)
    e2e_pairs, e2e_count = oracle.select_pairs(oracle_pair_score, n_select)
    margins, asserted = [], 0
    for b in range(oracle_pair_score.shape[0]):
        s = np.sort(oracle_pair_score[b])
        margins.append(np.min(np.diff(s)) if s.size > 1 else np.inf)
        err = float(np.max(np.abs(np.asarray(gpu_pair_score[b], dtype=np.float64) - oracle_pair_score[b])))
        assert err <= TOL
        if margins[-1] > 2 * err:
            np.testing.assert_array_equal(pairs[b], e2e_pairs[b])
            assert count[b] == e2e_count[b]
            asserted += 1
    check_selection.last_asserted = asserted   # conversations whose end-to-end choice was compared
    return pairs, count, min(margins)
