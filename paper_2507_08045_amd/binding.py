"""ctypes binding of libkrul.so: argument marshalling only.

Every step of the path (logits, online softmax statistics, cross term, row
similarity, token-wise aggregation, pair selection) runs in the library's HIP
kernels; this module only checks tensor types, allocates outputs and workspace with
torch, and passes raw device pointers and the current HIP stream across the C ABI
declared in include/krul.h.  There is no CPU fallback: if the library is missing
or the tensors are not on a GPU, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkrul.so")

KRUL_OK, KRUL_EINVAL, KRUL_EDTYPE, KRUL_EWORKSPACE, KRUL_ELAUNCH, KRUL_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
KRUL_ESCRATCH = -6
KRUL_STATIC_SCRATCH_BYTES = 40 << 20
KRUL_F32, KRUL_BF16, KRUL_F16 = 0, 1, 2
_DTYPES = {torch.float32: KRUL_F32, torch.bfloat16: KRUL_BF16, torch.float16: KRUL_F16}
KRUL_FLAG_CAUSAL = 1 << 0
KRUL_FLAG_GENERIC_KERNEL = 1 << 8
KRUL_FLAG_SINGLE_SPLIT = 1 << 9


class KrulShape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("n_hist", ctypes.c_int32),
        ("n_query", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
        ("flags", ctypes.c_int32),
    ]


class KrulKLayout(ctypes.Structure):
    _fields_ = [("k_layers", ctypes.c_void_p), ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64),
                ("k_stride_s", ctypes.c_int64)]


class KrulKPages(ctypes.Structure):
    _fields_ = [("k_layers", ctypes.c_void_p), ("block_table", ctypes.c_void_p), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("k_stride_block", ctypes.c_int64), ("k_stride_h", ctypes.c_int64),
                ("k_stride_s", ctypes.c_int64)]


class KrulKeys(ctypes.Structure):
    _fields_ = [("dense", ctypes.c_void_p), ("strided", ctypes.POINTER(KrulKLayout)), ("paged", ctypes.POINTER(KrulKPages))]


class KrulError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libkrul: {strerror(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libkrul.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2507_08045_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.krul_pair_similarity_workspace.restype = sz
        L.krul_pair_similarity_workspace.argtypes = [ctypes.POINTER(KrulShape)]
        L.krul_pair_similarity.restype = ctypes.c_int
        L.krul_pair_similarity.argtypes = [ctypes.POINTER(KrulShape), vp, vp, vp, vp, vp, vp, sz, vp]
        L.krul_pair_similarity_static.restype = ctypes.c_int
        L.krul_pair_similarity_static.argtypes = [ctypes.POINTER(KrulShape), vp, vp, vp, vp, vp, vp]
        L.krul_pair_similarity_timed.restype = ctypes.c_int
        L.krul_pair_similarity_timed.argtypes = [ctypes.POINTER(KrulShape), vp, vp, vp, vp, vp, vp, sz, vp, vp, vp]
        L.krul_pair_similarity_ir_workspace.restype = sz
        L.krul_pair_similarity_ir_workspace.argtypes = [ctypes.POINTER(KrulShape)]
        L.krul_pair_similarity_ir.restype = ctypes.c_int
        L.krul_pair_similarity_ir.argtypes = [ctypes.POINTER(KrulShape), vp, vp, ctypes.c_float, vp, vp, vp, vp, vp,
                                              vp, sz, vp]
        L.krul_pair_similarity_strided.restype = ctypes.c_int
        L.krul_pair_similarity_strided.argtypes = [ctypes.POINTER(KrulShape), vp, ctypes.POINTER(KrulKLayout), vp, vp,
                                                   vp, vp, sz, vp]
        L.krul_pair_similarity_paged.restype = ctypes.c_int
        L.krul_pair_similarity_paged.argtypes = [ctypes.POINTER(KrulShape), vp, ctypes.POINTER(KrulKPages), vp, vp,
                                                 vp, vp, sz, vp]
        L.krul_pair_similarity_select.restype = ctypes.c_int
        L.krul_pair_similarity_select.argtypes = [ctypes.POINTER(KrulShape), vp, vp, vp, ctypes.c_int32, vp, vp, vp,
                                                  vp, vp, vp, sz, vp, vp, vp]
        L.krul_pair_similarity_accumulate_in_place.restype = ctypes.c_int
        L.krul_pair_similarity_accumulate_in_place.argtypes = [ctypes.POINTER(KrulShape), vp, ctypes.POINTER(KrulKeys),
                                                               vp, vp, vp, sz, vp]
        L.krul_all_pairs_similarity_in_place.restype = ctypes.c_int
        L.krul_all_pairs_similarity_in_place.argtypes = [ctypes.POINTER(KrulShape), vp, ctypes.POINTER(KrulKeys),
                                                         vp, vp, vp, vp, sz, vp]
        L.krul_pair_similarity_ir_in_place.restype = ctypes.c_int
        L.krul_pair_similarity_ir_in_place.argtypes = [ctypes.POINTER(KrulShape), vp, ctypes.POINTER(KrulKeys),
                                                       ctypes.c_float, vp, vp, vp, vp, vp, vp, sz, vp]
        L.krul_pair_similarity_accumulate.restype = ctypes.c_int
        L.krul_pair_similarity_accumulate.argtypes = [ctypes.POINTER(KrulShape), vp, vp, vp, vp, vp, sz, vp]
        L.krul_pair_scores_from_sums.restype = ctypes.c_int
        L.krul_pair_scores_from_sums.argtypes = [vp, vp, i32, i32, i32, ctypes.c_float, vp, vp, vp, vp]
        L.krul_all_pairs_workspace.restype = sz
        L.krul_all_pairs_workspace.argtypes = [ctypes.POINTER(KrulShape), sz]
        L.krul_all_pairs_similarity.restype = ctypes.c_int
        L.krul_all_pairs_similarity.argtypes = [ctypes.POINTER(KrulShape), vp, vp, vp, vp, vp, vp, sz, vp]
        L.krul_select_pairs_all.restype = ctypes.c_int
        L.krul_select_pairs_all.argtypes = [vp, i32, vp, i32, i32, i32, vp, vp, vp]
        L.krul_select_pairs.restype = ctypes.c_int
        L.krul_select_pairs.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
        L.krul_calibration_copy.restype = ctypes.c_int
        L.krul_calibration_copy.argtypes = [vp, vp, sz, vp]
        L.krul_calibration_block.restype = ctypes.c_int
        L.krul_calibration_block.argtypes = [i32, i32, i32, vp, vp]
        L.krul_pair_similarity_plan.restype = ctypes.c_int
        L.krul_pair_similarity_plan.argtypes = [ctypes.POINTER(KrulShape), ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.krul_n_select_from_ratio.restype = i32
        L.krul_n_select_from_ratio.argtypes = [i32, ctypes.c_float]
        L.krul_strerror.restype = ctypes.c_char_p
        L.krul_strerror.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().krul_strerror(int(status)).decode()


def n_select_from_ratio(n_layers: int, r_l: float) -> int:
    return int(lib().krul_n_select_from_ratio(int(n_layers), float(r_l)))


def make_shape(q: torch.Tensor, k: torch.Tensor, scale: float = 0.0, flags: int = 0) -> KrulShape:
    if q.dim() != 5 or k.dim() != 5:
        raise ValueError("q must be [B,L,Hq,Tq,d] and k [B,L,Hkv,S,d]")
    if q.dtype != k.dtype or q.dtype not in _DTYPES:
        raise ValueError("q and k must both be float32, both bfloat16 or both float16")
    B, L, Hq, Tq, d = q.shape
    B2, L2, Hkv, S, d2 = k.shape
    if (B, L, d) != (B2, L2, d2):
        raise ValueError("q and k disagree on batch, layers or head_dim")
    dt = _DTYPES[q.dtype]
    return KrulShape(B, L, Hq, Hkv, d, S, Tq, dt, float(scale), int(flags))


def workspace_bytes(shape: KrulShape) -> int:
    return int(lib().krul_pair_similarity_workspace(ctypes.byref(shape)))


def workspace_bytes_ir(shape: KrulShape) -> int:
    return int(lib().krul_pair_similarity_ir_workspace(ctypes.byref(shape)))


KERNEL_FORMS = {0: "sim_generic_kernel", 1: "sim_mfma_kernel (wide, 128 x 256)", 2: "sim_mfma_kernel (mid, 64 x 512)",
                3: "sim_mfma_kernel (slim, 32 x 512)", 4: "sim_mfma_kernel (slim, deep ring)",
                5: "sim_mfma_kernel (slim short, 32 x 256)", 6: "sim_mfma_kernel (mid short, 64 x 128)",
                7: "sim_mfma_kernel (wide short, 128 x 128)", 8: "sim_big_kernel (256 x 256)"}


def plan(shape: KrulShape) -> dict:
    """Which kernel form krul_pair_similarity takes for this shape on dense keys, and its grid."""
    nwg, nsp = ctypes.c_int32(0), ctypes.c_int32(0)
    v = int(lib().krul_pair_similarity_plan(ctypes.byref(shape), ctypes.byref(nwg), ctypes.byref(nsp)))
    if v < 0:
        raise KrulError(v)
    return {"form": v, "kernel": KERNEL_FORMS.get(v, str(v)), "n_workgroups": nwg.value, "n_key_splits": nsp.value}


def calibration_block(row_blocks: int, parts: int, iters: int, out: torch.Tensor) -> None:
    """krul_calibration_block on the current stream (out: float32 GPU tensor of 256 * 512 elements)."""
    if not out.is_cuda or out.dtype != torch.float32 or out.numel() < 256 * 512:
        raise ValueError("out must be a float32 GPU tensor of at least 131072 elements")
    rc = lib().krul_calibration_block(int(row_blocks), int(parts), int(iters), _dev_ptr(out), ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)


def _stream_ptr() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _dev_ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def pair_similarity(q: torch.Tensor, k: torch.Tensor, *, scale: float = 0.0, flags: int = 0,
                    want_head_score: bool = True, want_pair_dist: bool = True,
                    workspace: torch.Tensor | None = None, out: dict | None = None,
                    events: tuple | None = None) -> dict:
    """krul_pair_similarity on the current stream.  Returns device tensors
    pair_score [B,L-1], head_score [B,L-1,Hq] (or None), pair_dist [B,L-1] (or None)."""
    if not (q.is_cuda and k.is_cuda):
        raise ValueError("q and k must be GPU tensors (this library has no CPU path)")
    if not (q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous")
    shp = make_shape(q, k, scale, flags)
    need = workspace_bytes(shp)
    if need == 0:
        # let the library name the reason
        rc = lib().krul_pair_similarity(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), None, None, None,
                                        None, 0, None)
        raise KrulError(rc if rc != 0 else KRUL_EINVAL)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    out = out or {}
    ps = out.get("pair_score")
    if ps is None:
        ps = torch.empty((B, L - 1), dtype=torch.float32, device=q.device)
    hs = out.get("head_score")
    if hs is None and want_head_score:
        hs = torch.empty((B, L - 1, Hq), dtype=torch.float32, device=q.device)
    pd = out.get("pair_dist")
    if pd is None and want_pair_dist:
        pd = torch.empty((B, L - 1), dtype=torch.float32, device=q.device)
    if events is not None:   # (hipEvent_t, hipEvent_t) raw handles around the similarity kernel
        rc = lib().krul_pair_similarity_timed(
            ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), _dev_ptr(ps), _dev_ptr(hs), _dev_ptr(pd),
            _dev_ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr()),
            ctypes.c_void_p(events[0]), ctypes.c_void_p(events[1]))
    else:
        rc = lib().krul_pair_similarity(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), _dev_ptr(ps), _dev_ptr(hs),
                                        _dev_ptr(pd), _dev_ptr(workspace), workspace.numel(),
                                        ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd, "workspace": workspace}


def pair_similarity_static(q: torch.Tensor, k: torch.Tensor, out: dict, *, scale: float = 0.0, flags: int = 0) -> dict:
    """krul_pair_similarity_static on the current stream: the scores of pair_similarity with no workspace
    and no allocation anywhere -- the caller passes every output in `out` ("pair_score" required,
    "head_score" and "pair_dist" optional) and gets `out` back."""
    if not (q.is_cuda and k.is_cuda):
        raise ValueError("q and k must be GPU tensors (this library has no CPU path)")
    if not (q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous")
    shp = make_shape(q, k, scale, flags)
    rc = lib().krul_pair_similarity_static(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), _dev_ptr(out["pair_score"]),
                                           _dev_ptr(out.get("head_score")), _dev_ptr(out.get("pair_dist")),
                                           ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return out


class StridedKeys:
    """Keys in one GPU tensor per layer, each indexed [B, Hkv, S, d] (see pair_similarity_strided)."""

    def __init__(self, k_layers):
        self.k_layers = list(k_layers)
        self.table = None


class PagedKeys:
    """Keys in one pool of pages per layer and a block table (see pair_similarity_paged); n_hist keys per
    conversation."""

    def __init__(self, pools, block_table: torch.Tensor, n_hist: int):
        self.pools, self.block_table, self.n_hist = list(pools), block_table, int(n_hist)
        self.table = None


def _keys(q: torch.Tensor, keys, scale: float, flags: int):
    """(shape, KrulKeys, objects to keep alive) for dense keys (a tensor), StridedKeys or PagedKeys."""
    if not q.is_cuda or q.dim() != 5 or not q.is_contiguous() or q.dtype not in _DTYPES:
        raise ValueError("q must be a contiguous GPU tensor [B,L,Hq,Tq,d] of dtype float32, bfloat16 or float16")
    B, L, Hq, Tq, d = q.shape
    if isinstance(keys, torch.Tensor):
        if not keys.is_cuda or not keys.is_contiguous():
            raise ValueError("k must be a contiguous GPU tensor")
        return make_shape(q, keys, scale, flags), KrulKeys(keys.data_ptr(), None, None), (keys,)
    layers = keys.k_layers if isinstance(keys, StridedKeys) else keys.pools
    t0 = layers[0]
    if len(layers) != L or any(not t.is_cuda or t.dim() != 4 or t.shape != t0.shape or t.stride() != t0.stride()
                               or t.dtype != q.dtype for t in layers) or t0.stride(3) != 1 or t0.shape[3] != d:
        raise ValueError("one 4-d GPU tensor per layer, all of one shape, one set of strides, q's dtype and head_dim")
    if keys.table is None:
        keys.table = torch.tensor([t.data_ptr() for t in layers], dtype=torch.int64).to(q.device)
    if isinstance(keys, StridedKeys):
        if t0.shape[0] != B:
            raise ValueError("q and k disagree on the batch")
        shp = KrulShape(B, L, Hq, t0.shape[1], d, t0.shape[2], Tq, _DTYPES[q.dtype], float(scale), int(flags))
        lay = KrulKLayout(keys.table.data_ptr(), t0.stride(0) if B > 1 else 0, t0.stride(1), t0.stride(2))
        return shp, KrulKeys(None, ctypes.pointer(lay), None), (lay, keys)
    bt = keys.block_table
    if not bt.is_cuda or bt.dtype != torch.int32 or bt.dim() != 2 or not bt.is_contiguous() or bt.shape[0] != B:
        raise ValueError("block_table must be a contiguous int32 GPU tensor [B, max_blocks]")
    shp = KrulShape(B, L, Hq, t0.shape[2], d, keys.n_hist, Tq, _DTYPES[q.dtype], float(scale), int(flags))
    pages = KrulKPages(keys.table.data_ptr(), bt.data_ptr(), t0.shape[1], bt.shape[1], t0.stride(0), t0.stride(2),
                       t0.stride(1))
    return shp, KrulKeys(None, None, ctypes.pointer(pages)), (pages, keys)


def _pair_outputs(shp, q, want_head_score, want_pair_dist):
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    ps = torch.empty((B, L - 1), dtype=torch.float32, device=q.device)
    hs = torch.empty((B, L - 1, Hq), dtype=torch.float32, device=q.device) if want_head_score else None
    pd = torch.empty((B, L - 1), dtype=torch.float32, device=q.device) if want_pair_dist else None
    return ps, hs, pd


def pair_similarity_strided(q: torch.Tensor, k_layers, *, scale: float = 0.0, flags: int = 0,
                            want_head_score: bool = True, want_pair_dist: bool = True,
                            workspace: torch.Tensor | None = None, k_table: torch.Tensor | None = None) -> dict:
    """krul_pair_similarity_strided on the current stream.  k_layers: one GPU tensor per layer, each
    indexed [B, Hkv, S, d] with any strides over the first three axes (the same for every layer) and
    contiguous head_dim, e.g. cache[l].permute(0, 2, 1, 3) of a [B, S, Hkv, d] cache.  k_table: the
    device array of the layers' addresses from an earlier call with the same tensors (returned as
    "k_table"), to skip its upload."""
    keys = StridedKeys(k_layers)
    keys.table = k_table
    shp, ks, keep = _keys(q, keys, scale, flags)
    need = workspace_bytes(shp)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ps, hs, pd = _pair_outputs(shp, q, want_head_score, want_pair_dist)
    rc = lib().krul_pair_similarity_strided(ctypes.byref(shp), _dev_ptr(q), ks.strided, _dev_ptr(ps),
                                            _dev_ptr(hs), _dev_ptr(pd), _dev_ptr(workspace),
                                            workspace.numel() if workspace is not None else 0,
                                            ctypes.c_void_p(_stream_ptr()))
    del keep
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd, "workspace": workspace, "k_table": keys.table}


def pair_similarity_paged(q: torch.Tensor, pools, block_table: torch.Tensor, n_hist: int, *, scale: float = 0.0,
                          flags: int = 0, want_head_score: bool = True, want_pair_dist: bool = True,
                          workspace: torch.Tensor | None = None, k_table: torch.Tensor | None = None) -> dict:
    """krul_pair_similarity_paged on the current stream.  pools: one GPU tensor per layer indexed
    [page, key in page, kv head, d] with any strides over the first three axes (the same for every layer) and
    contiguous head_dim; block_table: int32 GPU tensor [B, max_blocks]; n_hist: keys per conversation."""
    keys = PagedKeys(pools, block_table, n_hist)
    keys.table = k_table
    shp, ks, keep = _keys(q, keys, scale, flags)
    need = workspace_bytes(shp)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ps, hs, pd = _pair_outputs(shp, q, want_head_score, want_pair_dist)
    rc = lib().krul_pair_similarity_paged(ctypes.byref(shp), _dev_ptr(q), ks.paged, _dev_ptr(ps),
                                          _dev_ptr(hs), _dev_ptr(pd), _dev_ptr(workspace),
                                          workspace.numel() if workspace is not None else 0,
                                          ctypes.c_void_p(_stream_ptr()))
    del keep
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd, "workspace": workspace, "k_table": keys.table}


def pair_similarity_ir(q: torch.Tensor, k: torch.Tensor, gamma: float, *, scale: float = 0.0, flags: int = 0,
                       want_head_score: bool = True, want_pair_dist: bool = True,
                       workspace: torch.Tensor | None = None) -> dict:
    """krul_pair_similarity_ir on the current stream: the outputs of pair_similarity plus
    ir_mass [B,L] float32 and eligible [B,L] uint8 (the Initial-Recent layer test)."""
    if not (q.is_cuda and k.is_cuda):
        raise ValueError("q and k must be GPU tensors (this library has no CPU path)")
    if not (q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous")
    shp = make_shape(q, k, scale, flags)
    need = workspace_bytes_ir(shp)
    if need == 0:
        rc = lib().krul_pair_similarity_ir(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), float(gamma), None, None,
                                           None, None, None, None, 0, None)
        raise KrulError(rc if rc != 0 else KRUL_EINVAL)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    ps = torch.empty((B, L - 1), dtype=torch.float32, device=q.device)
    hs = torch.empty((B, L - 1, Hq), dtype=torch.float32, device=q.device) if want_head_score else None
    pd = torch.empty((B, L - 1), dtype=torch.float32, device=q.device) if want_pair_dist else None
    mass = torch.empty((B, L), dtype=torch.float32, device=q.device)
    el = torch.empty((B, L), dtype=torch.uint8, device=q.device)
    rc = lib().krul_pair_similarity_ir(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), float(gamma), _dev_ptr(ps),
                                       _dev_ptr(hs), _dev_ptr(pd), _dev_ptr(mass), _dev_ptr(el),
                                       _dev_ptr(workspace), workspace.numel(), ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd, "ir_mass": mass, "eligible": el,
            "workspace": workspace}


def pair_similarity_accumulate(q: torch.Tensor, k: torch.Tensor, head_sum: torch.Tensor,
                               head_dist_sum: torch.Tensor | None = None, *, scale: float = 0.0, flags: int = 0,
                               workspace: torch.Tensor | None = None) -> torch.Tensor:
    """krul_pair_similarity_accumulate on the current stream: adds this call's per-row cosines (and
    distances) to the running sums head_sum (head_dist_sum), both [B,L-1,Hq] float32.  Returns the workspace."""
    if not (q.is_cuda and k.is_cuda and q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous GPU tensors (this library has no CPU path)")
    shp = make_shape(q, k, scale, flags)
    want = (shp.batch, shp.n_layers - 1, shp.n_q_heads)
    for t in (head_sum, head_dist_sum):
        if t is not None and (not t.is_cuda or t.dtype != torch.float32 or tuple(t.shape) != want
                              or not t.is_contiguous()):
            raise ValueError("the running sums must be contiguous float32 GPU tensors [B, L-1, Hq]")
    need = workspace_bytes(shp)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = lib().krul_pair_similarity_accumulate(
        ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), _dev_ptr(head_sum), _dev_ptr(head_dist_sum),
        _dev_ptr(workspace), workspace.numel() if workspace is not None else 0, ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return workspace


def pair_similarity_accumulate_in_place(q: torch.Tensor, keys, head_sum: torch.Tensor,
                                        head_dist_sum: torch.Tensor | None = None, *, scale: float = 0.0,
                                        flags: int = 0, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """krul_pair_similarity_accumulate_in_place on the current stream; keys: a dense tensor, StridedKeys or
    PagedKeys.  Returns the workspace."""
    shp, ks, keep = _keys(q, keys, scale, flags)
    want = (shp.batch, shp.n_layers - 1, shp.n_q_heads)
    for t in (head_sum, head_dist_sum):
        if t is not None and (not t.is_cuda or t.dtype != torch.float32 or tuple(t.shape) != want
                              or not t.is_contiguous()):
            raise ValueError("the running sums must be contiguous float32 GPU tensors [B, L-1, Hq]")
    need = workspace_bytes(shp)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = lib().krul_pair_similarity_accumulate_in_place(
        ctypes.byref(shp), _dev_ptr(q), ctypes.byref(ks), _dev_ptr(head_sum), _dev_ptr(head_dist_sum),
        _dev_ptr(workspace), workspace.numel() if workspace is not None else 0, ctypes.c_void_p(_stream_ptr()))
    del keep
    if rc != KRUL_OK:
        raise KrulError(rc)
    return workspace


def pair_similarity_ir_in_place(q: torch.Tensor, keys, gamma: float, *, scale: float = 0.0, flags: int = 0,
                                want_head_score: bool = True, want_pair_dist: bool = True,
                                workspace: torch.Tensor | None = None) -> dict:
    """krul_pair_similarity_ir_in_place on the current stream; keys: a dense tensor, StridedKeys or PagedKeys."""
    shp, ks, keep = _keys(q, keys, scale, flags)
    need = workspace_bytes_ir(shp)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    ps = torch.empty((B, L - 1), dtype=torch.float32, device=q.device)
    hs = torch.empty((B, L - 1, Hq), dtype=torch.float32, device=q.device) if want_head_score else None
    pd = torch.empty((B, L - 1), dtype=torch.float32, device=q.device) if want_pair_dist else None
    mass = torch.empty((B, L), dtype=torch.float32, device=q.device)
    el = torch.empty((B, L), dtype=torch.uint8, device=q.device)
    rc = lib().krul_pair_similarity_ir_in_place(
        ctypes.byref(shp), _dev_ptr(q), ctypes.byref(ks), float(gamma), _dev_ptr(ps), _dev_ptr(hs), _dev_ptr(pd),
        _dev_ptr(mass), _dev_ptr(el), _dev_ptr(workspace), workspace.numel() if workspace is not None else 0,
        ctypes.c_void_p(_stream_ptr()))
    del keep
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd, "ir_mass": mass, "eligible": el,
            "workspace": workspace}


def pair_scores_from_sums(head_sum: torch.Tensor, n_tokens: float, head_dist_sum: torch.Tensor | None = None) -> dict:
    """krul_pair_scores_from_sums: running sums over n_tokens rows -> pair_score, head_score, pair_dist."""
    if not head_sum.is_cuda or head_sum.dtype != torch.float32 or head_sum.dim() != 3 or not head_sum.is_contiguous():
        raise ValueError("head_sum must be a contiguous float32 GPU tensor [B, L-1, Hq]")
    B, NP, Hq = head_sum.shape
    ps = torch.empty((B, NP), dtype=torch.float32, device=head_sum.device)
    hs = torch.empty((B, NP, Hq), dtype=torch.float32, device=head_sum.device)
    pd = torch.empty((B, NP), dtype=torch.float32, device=head_sum.device) if head_dist_sum is not None else None
    rc = lib().krul_pair_scores_from_sums(_dev_ptr(head_sum), _dev_ptr(head_dist_sum), B, NP + 1, Hq,
                                          float(n_tokens), _dev_ptr(ps), _dev_ptr(hs), _dev_ptr(pd),
                                          ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd}


def select_pairs(pair_score: torch.Tensor, n_select: int, eligible: torch.Tensor | None = None,
                 out_pairs: torch.Tensor | None = None, out_count: torch.Tensor | None = None):
    """krul_select_pairs on the current stream: (pairs [B,n_select] int32, count [B] int32)."""
    if not pair_score.is_cuda or pair_score.dtype != torch.float32 or not pair_score.is_contiguous():
        raise ValueError("pair_score must be a contiguous float32 GPU tensor")
    if pair_score.dim() == 1:
        pair_score = pair_score[None, :]
    B, NP = pair_score.shape
    L = NP + 1
    if eligible is not None:
        if not eligible.is_cuda or eligible.dtype != torch.uint8 or tuple(eligible.shape) != (B, L) \
                or not eligible.is_contiguous():
            raise ValueError("eligible must be a contiguous uint8 GPU tensor [B, n_layers]")
    if out_pairs is None:
        out_pairs = torch.empty((B, max(int(n_select), 0)), dtype=torch.int32, device=pair_score.device)
    if out_count is None:
        out_count = torch.empty((B,), dtype=torch.int32, device=pair_score.device)
    rc = lib().krul_select_pairs(_dev_ptr(pair_score), _dev_ptr(eligible), B, L, int(n_select),
                                 _dev_ptr(out_pairs), _dev_ptr(out_count), ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return out_pairs, out_count


def pair_similarity_select(q: torch.Tensor, k: torch.Tensor, n_select: int, eligible: torch.Tensor | None = None, *,
                           scale: float = 0.0, flags: int = 0, want_head_score: bool = True,
                           want_pair_dist: bool = True, workspace: torch.Tensor | None = None,
                           out: dict | None = None, events: tuple | None = None) -> dict:
    """krul_pair_similarity_select on the current stream: the outputs of pair_similarity plus
    pairs [B,n_select] int32 and count [B] int32 of select_pairs on its pair_score."""
    if not (q.is_cuda and k.is_cuda):
        raise ValueError("q and k must be GPU tensors (this library has no CPU path)")
    if not (q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous")
    shp = make_shape(q, k, scale, flags)
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    if eligible is not None:
        if not eligible.is_cuda or eligible.dtype != torch.uint8 or tuple(eligible.shape) != (B, L) \
                or not eligible.is_contiguous():
            raise ValueError("eligible must be a contiguous uint8 GPU tensor [B, n_layers]")
    need = workspace_bytes(shp)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    out = out or {}

    def buf(name, shape, dtype, wanted=True):
        t = out.get(name)
        return t if t is not None or not wanted else torch.empty(shape, dtype=dtype, device=q.device)
    ps = buf("pair_score", (B, L - 1), torch.float32)
    hs = buf("head_score", (B, L - 1, Hq), torch.float32, want_head_score)
    pd = buf("pair_dist", (B, L - 1), torch.float32, want_pair_dist)
    pairs = buf("pairs", (B, max(int(n_select), 0)), torch.int32)
    count = buf("count", (B,), torch.int32)
    ev = events or (None, None)
    rc = lib().krul_pair_similarity_select(
        ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), _dev_ptr(eligible), int(n_select), _dev_ptr(ps), _dev_ptr(hs),
        _dev_ptr(pd), _dev_ptr(pairs), _dev_ptr(count), _dev_ptr(workspace),
        workspace.numel() if workspace is not None else 0, ctypes.c_void_p(_stream_ptr()),
        ctypes.c_void_p(ev[0]), ctypes.c_void_p(ev[1]))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "head_score": hs, "pair_dist": pd, "pairs": pairs, "count": count, "workspace": workspace}


def all_pairs_workspace_bytes(shape: KrulShape, max_bytes: int = 0) -> int:
    return int(lib().krul_all_pairs_workspace(ctypes.byref(shape), int(max_bytes)))


def all_pairs_similarity(q: torch.Tensor, k: torch.Tensor, *, scale: float = 0.0, flags: int = 0,
                         want_pair_dist: bool = True, want_head_score: bool = False,
                         workspace: torch.Tensor | None = None, max_workspace_bytes: int = 0) -> dict:
    """krul_all_pairs_similarity on the current stream.  Returns device tensors pair_score [B,L,L],
    pair_dist [B,L,L] (or None), head_score [B,Hq,L,L] (or None) and the workspace used."""
    if not (q.is_cuda and k.is_cuda):
        raise ValueError("q and k must be GPU tensors (this library has no CPU path)")
    if not (q.is_contiguous() and k.is_contiguous()):
        raise ValueError("q and k must be contiguous")
    shp = make_shape(q, k, scale, flags)
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    if workspace is None:
        need = all_pairs_workspace_bytes(shp, max_workspace_bytes)
        if need == 0:   # let the library name the reason
            rc = lib().krul_all_pairs_similarity(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), None, None, None,
                                                 None, 0, None)
            raise KrulError(rc if rc != 0 else KRUL_EINVAL)
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ps = torch.empty((B, L, L), dtype=torch.float32, device=q.device)
    pd = torch.empty((B, L, L), dtype=torch.float32, device=q.device) if want_pair_dist else None
    hs = torch.empty((B, Hq, L, L), dtype=torch.float32, device=q.device) if want_head_score else None
    rc = lib().krul_all_pairs_similarity(ctypes.byref(shp), _dev_ptr(q), _dev_ptr(k), _dev_ptr(ps), _dev_ptr(pd),
                                         _dev_ptr(hs), _dev_ptr(workspace), workspace.numel(),
                                         ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "pair_dist": pd, "head_score": hs, "workspace": workspace}


def all_pairs_similarity_in_place(q: torch.Tensor, keys, *, scale: float = 0.0, flags: int = 0,
                                  want_pair_dist: bool = True, want_head_score: bool = False,
                                  workspace: torch.Tensor | None = None, max_workspace_bytes: int = 0) -> dict:
    """krul_all_pairs_similarity_in_place on the current stream; keys: a dense tensor, StridedKeys or PagedKeys."""
    shp, ks, keep = _keys(q, keys, scale, flags)
    B, L, Hq = shp.batch, shp.n_layers, shp.n_q_heads
    if workspace is None:
        need = all_pairs_workspace_bytes(shp, max_workspace_bytes)
        if need == 0:   # let the library name the reason
            rc = lib().krul_all_pairs_similarity_in_place(ctypes.byref(shp), _dev_ptr(q), ctypes.byref(ks), None, None,
                                                          None, None, 0, None)
            raise KrulError(rc if rc != 0 else KRUL_EINVAL)
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ps = torch.empty((B, L, L), dtype=torch.float32, device=q.device)
    pd = torch.empty((B, L, L), dtype=torch.float32, device=q.device) if want_pair_dist else None
    hs = torch.empty((B, Hq, L, L), dtype=torch.float32, device=q.device) if want_head_score else None
    rc = lib().krul_all_pairs_similarity_in_place(ctypes.byref(shp), _dev_ptr(q), ctypes.byref(ks), _dev_ptr(ps),
                                                  _dev_ptr(pd), _dev_ptr(hs), _dev_ptr(workspace), workspace.numel(),
                                                  ctypes.c_void_p(_stream_ptr()))
    del keep
    if rc != KRUL_OK:
        raise KrulError(rc)
    return {"pair_score": ps, "pair_dist": pd, "head_score": hs, "workspace": workspace}


def select_pairs_all(score: torch.Tensor, n_select: int, closer_is_smaller: bool,
                     eligible: torch.Tensor | None = None):
    """krul_select_pairs_all on the current stream: (pairs [B,n_select,2] int32 as (j, i), count [B] int32)."""
    if not score.is_cuda or score.dtype != torch.float32 or not score.is_contiguous():
        raise ValueError("score must be a contiguous float32 GPU tensor")
    if score.dim() == 2:
        score = score[None]
    B, L, L2 = score.shape
    if L != L2:
        raise ValueError("score must be [B, n_layers, n_layers]")
    if eligible is not None:
        if not eligible.is_cuda or eligible.dtype != torch.uint8 or tuple(eligible.shape) != (B, L) \
                or not eligible.is_contiguous():
            raise ValueError("eligible must be a contiguous uint8 GPU tensor [B, n_layers]")
    out_pairs = torch.empty((B, max(int(n_select), 0), 2), dtype=torch.int32, device=score.device)
    out_count = torch.empty((B,), dtype=torch.int32, device=score.device)
    rc = lib().krul_select_pairs_all(_dev_ptr(score), 1 if closer_is_smaller else 0, _dev_ptr(eligible), B, L,
                                     int(n_select), _dev_ptr(out_pairs), _dev_ptr(out_count),
                                     ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
    return out_pairs, out_count


def calibration_copy(src: torch.Tensor, dst: torch.Tensor):
    """krul_calibration_copy: plain copy kernel of known size (reference for traffic counters)."""
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("src and dst must be contiguous GPU tensors")
    n = src.numel() * src.element_size()
    if n != dst.numel() * dst.element_size():
        raise ValueError("src and dst must have the same size in bytes")
    rc = lib().krul_calibration_copy(_dev_ptr(src), _dev_ptr(dst), n, ctypes.c_void_p(_stream_ptr()))
    if rc != KRUL_OK:
        raise KrulError(rc)
