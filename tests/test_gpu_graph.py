"""The whole step (similarity, head and pair scores, selection) enqueues kernels only -- no allocation, no
memset, no host synchronisation -- so a caller can record it into a HIP graph and replay it: every replay,
on new inputs in the same buffers and with the program's own eager work in between, must give what the
eager call gives."""
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


@pytest.mark.parametrize("shape", [dict(B=2, L=6, Hq=8, Hkv=2, d=128, S=900, Tq=40),      # wide tile, several splits
                                   dict(B=3, L=5, Hq=8, Hkv=4, d=64, S=2300, Tq=2),       # narrow tile
                                   dict(B=4, L=4, Hq=8, Hkv=2, d=128, S=16384 - 50, Tq=64)],  # 256-row tiles (sim_big_kernel)
                         ids=["prefill-chunk", "decode-step", "many-query"])
def test_step_replays_from_a_graph(G, oracle, shape):
    import paper_2507_08045_amd as kr
    n_select = 2
    ws_list = [workloads.make(f"graph-{i}", dtype="bf16", seed=300 + i, **shape) for i in range(3)]
    q, k = G.to_device(ws_list[0])
    workspace = torch.empty(kr.workspace_bytes(kr.make_shape(q, k)), dtype=torch.uint8, device="cuda")
    B, L, Hq = shape["B"], shape["L"], shape["Hq"]
    out = {"pair_score": torch.empty((B, L - 1), dtype=torch.float32, device="cuda"),
           "head_score": torch.empty((B, L - 1, Hq), dtype=torch.float32, device="cuda"),
           "pair_dist": torch.empty((B, L - 1), dtype=torch.float32, device="cuda"),
           "pairs": torch.empty((B, n_select), dtype=torch.int32, device="cuda"),
           "count": torch.empty((B,), dtype=torch.int32, device="cuda")}
    kr.pair_similarity_select(q, k, n_select, workspace=workspace, out=out)     # library loaded, kernels resident
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        kr.pair_similarity_select(q, k, n_select, workspace=workspace, out=out)

    for i, w in enumerate(ws_list + ws_list[:1]):
        qn, kn = G.to_device(w)
        q.copy_(qn)
        k.copy_(kn)
        for t in out.values():
            t.fill_(-7)                        # eager work between the replays; stale results would show
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = {n: t.cpu().numpy().copy() for n, t in out.items()}
        ref = kr.pair_similarity_select(qn, kn, n_select)       # eager, own buffers
        torch.cuda.synchronize()
        for n in out:
            np.testing.assert_array_equal(got[n], ref[n].cpu().numpy(), err_msg=f"replay {i}: {n}")
        want = oracle.pair_similarity(w.q, w.k)
        G.assert_close(got["pair_score"], want["pair_score"], G.TOL, f"replay {i} pair_score")
        wp, wc = oracle.select_pairs(got["pair_score"].astype(np.float64), n_select)
        np.testing.assert_array_equal(got["pairs"], wp)
        np.testing.assert_array_equal(got["count"], wc)
