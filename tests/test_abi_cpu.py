"""Host-side checks of the C ABI that need no GPU: every function declared in
include/krul.h is exported by libkrul.so, host-only helpers compute what the header
says, and invalid arguments are rejected with the documented status before any GPU
work is attempted."""
import ctypes
import math
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kr():
    import paper_2507_08045_amd as kr_
    if not os.path.exists(kr_.binding.LIB_PATH):
        from paper_2507_08045_amd import build
        build.build()
    kr_.lib()
    return kr_


def declared_functions():
    text = open(os.path.join(ROOT, "include", "krul.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(krul_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(kr):
    names = declared_functions()
    assert {"krul_pair_similarity", "krul_select_pairs", "krul_pair_similarity_workspace",
            "krul_n_select_from_ratio", "krul_strerror", "krul_pair_similarity_timed",
            "krul_pair_similarity_ir", "krul_pair_similarity_ir_workspace",
            "krul_pair_similarity_accumulate", "krul_pair_scores_from_sums",
            "krul_pair_similarity_strided", "krul_all_pairs_similarity", "krul_all_pairs_workspace",
            "krul_select_pairs_all", "krul_pair_similarity_paged", "krul_pair_similarity_select", "krul_pair_similarity_accumulate_in_place",
            "krul_pair_similarity_ir_in_place", "krul_all_pairs_similarity_in_place"} <= set(names)
    lib = kr.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in krul.h but not exported"


def test_strerror_and_status_codes(kr):
    assert kr.strerror(0) == "ok"
    seen = {kr.strerror(c) for c in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6
    assert kr.strerror(-99) == "unknown status"


def test_n_select_from_ratio(kr):
    # Alg. 1 stops when the shared set holds N*r_l layers, two per pair
    assert kr.n_select_from_ratio(32, 0.5) == 8
    assert kr.n_select_from_ratio(80, 0.5) == 20
    assert kr.n_select_from_ratio(4, 0.5) == 1
    assert kr.n_select_from_ratio(6, 1.0) == 3
    assert kr.n_select_from_ratio(7, 1.0) == 3          # capped at N/2
    assert kr.n_select_from_ratio(32, 0.0) == 0
    assert kr.n_select_from_ratio(32, 0.3) == math.ceil(32 * 0.3 / 2)
    assert kr.n_select_from_ratio(1, 0.5) == 0


def shape(kr, B=1, L=4, Hq=4, Hkv=2, d=128, S=256, Tq=8, dtype=1, scale=0.0, flags=0):
    return kr.KrulShape(B, L, Hq, Hkv, d, S, Tq, dtype, scale, flags)


def test_workspace_query(kr):
    for cfg in [dict(), dict(dtype=0, d=64), dict(dtype=2), dict(dtype=2, d=72), dict(S=100000, Tq=1), dict(L=80, Hq=64, Hkv=8, Tq=256, S=16384, B=8)]:
        n = kr.workspace_bytes(shape(kr, **cfg))
        assert n > 0 and n % 256 == 0
    # the five benchmark configurations are all supported
    import workloads
    for name, (B, L, Hq, Hkv, d, S, Tq, dt, _) in workloads.CONFIGS.items():
        assert kr.workspace_bytes(shape(kr, B, L, Hq, Hkv, d, S, Tq, 0 if dt == "f32" else 1)) > 0, name
    bad = [dict(B=0), dict(L=1), dict(Hq=3, Hkv=2), dict(S=0), dict(Tq=0), dict(dtype=7), dict(d=100),
           dict(d=512), dict(scale=-1.0), dict(scale=float("nan")), dict(flags=2), dict(L=5000),
           dict(flags=1, S=4, Tq=8)]   # causal needs at least as many keys as rows
    for cfg in bad:
        assert kr.workspace_bytes(shape(kr, **cfg)) == 0, cfg
    assert kr.workspace_bytes(shape(kr, flags=kr.KRUL_FLAG_CAUSAL)) > 0
    assert kr.workspace_bytes_ir(shape(kr, flags=kr.KRUL_FLAG_CAUSAL)) > 0   # (rejected at the call: see below)


def call_sim(kr, shp, q=0x1000, k=0x2000, ps=0x3000, hs=None, pd=None, ws=0x10000, ws_bytes=1 << 40):
    vp = ctypes.c_void_p
    return kr.lib().krul_pair_similarity(ctypes.byref(shp), vp(q), vp(k), vp(ps), vp(hs), vp(pd), vp(ws),
                                         ctypes.c_size_t(ws_bytes), None)


def test_pair_similarity_rejects_bad_arguments_before_any_gpu_work(kr):
    ok = shape(kr)
    need = kr.workspace_bytes(ok)
    assert call_sim(kr, shape(kr, L=1)) == kr.KRUL_EINVAL
    assert call_sim(kr, shape(kr, Hq=3)) == kr.KRUL_EINVAL
    assert call_sim(kr, shape(kr, dtype=9)) == kr.KRUL_EDTYPE
    assert call_sim(kr, shape(kr, d=100)) == kr.KRUL_EUNSUPPORTED
    assert call_sim(kr, shape(kr, L=3000)) == kr.KRUL_EUNSUPPORTED
    assert call_sim(kr, ok, q=None) == kr.KRUL_EINVAL
    assert call_sim(kr, ok, k=None) == kr.KRUL_EINVAL
    assert call_sim(kr, ok, ps=None) == kr.KRUL_EINVAL
    assert call_sim(kr, ok, q=0x1008) == kr.KRUL_EINVAL            # 16-byte alignment
    assert call_sim(kr, ok, ps=0x3002) == kr.KRUL_EINVAL           # float alignment
    assert call_sim(kr, ok, ws=None) == kr.KRUL_EWORKSPACE
    assert call_sim(kr, ok, ws=0x10010) == kr.KRUL_EWORKSPACE      # 256-byte alignment
    assert call_sim(kr, ok, ws_bytes=need - 1) == kr.KRUL_EWORKSPACE
    assert kr.lib().krul_pair_similarity(None, None, None, None, None, None, None, 0, None) == kr.KRUL_EINVAL


def test_ir_entry_point_rejects_bad_arguments_before_any_gpu_work(kr):
    vp = ctypes.c_void_p
    ok = shape(kr)
    need = kr.workspace_bytes_ir(ok)
    assert need > kr.workspace_bytes(ok) and need % 256 == 0
    assert kr.workspace_bytes_ir(shape(kr, L=1)) == 0

    def call(shp, gamma=0.3, ps=0x3000, mass=0x4000, el=0x5000, ws=0x10000, ws_bytes=1 << 40):
        return kr.lib().krul_pair_similarity_ir(ctypes.byref(shp), vp(0x1000), vp(0x2000), ctypes.c_float(gamma),
                                                vp(ps), None, None, vp(mass), vp(el), vp(ws),
                                                ctypes.c_size_t(ws_bytes), None)
    assert call(shape(kr, Hq=3)) == kr.KRUL_EINVAL
    assert call(ok, gamma=-0.1) == kr.KRUL_EINVAL
    assert call(ok, gamma=float("nan")) == kr.KRUL_EINVAL
    assert call(ok, mass=None, el=None) == kr.KRUL_EINVAL          # nothing to write the test's result to
    assert call(ok, ps=None) == kr.KRUL_EINVAL
    assert call(ok, mass=0x4002) == kr.KRUL_EINVAL                 # float alignment
    assert call(ok, ws_bytes=need - 1) == kr.KRUL_EWORKSPACE
    assert call(ok, ws_bytes=kr.workspace_bytes(ok)) == kr.KRUL_EWORKSPACE   # the plain call's size is too small
    assert call(shape(kr, flags=kr.KRUL_FLAG_CAUSAL)) == kr.KRUL_EUNSUPPORTED  # the test is for whole-sequence attention


def test_strided_entry_point_rejects_bad_arguments_before_any_gpu_work(kr):
    vp = ctypes.c_void_p
    ok = shape(kr, B=2)

    def call(shp=ok, tab=0x2000, sb=1 << 20, sh=1 << 16, ss=128, lay=True, ws_bytes=1 << 40):
        kl = kr.KrulKLayout(tab, sb, sh, ss)
        return kr.lib().krul_pair_similarity_strided(ctypes.byref(shp), vp(0x1000), ctypes.byref(kl) if lay else None,
                                                     vp(0x3000), None, None, vp(0x10000), ctypes.c_size_t(ws_bytes),
                                                     None)
    assert call(lay=False) == kr.KRUL_EINVAL
    assert call(tab=None) == kr.KRUL_EINVAL
    assert call(tab=0x2004) == kr.KRUL_EINVAL          # the table holds 8-byte pointers
    assert call(sb=0) == kr.KRUL_EINVAL
    assert call(sh=-128) == kr.KRUL_EINVAL
    assert call(ss=64) == kr.KRUL_EINVAL               # keys would overlap
    assert call(ss=132) == kr.KRUL_EINVAL              # not a multiple of 8 elements
    assert call(ss=136, ws_bytes=16) == kr.KRUL_EWORKSPACE   # any multiple of 8 elements between keys will do
    assert call(ss=1 << 23) == kr.KRUL_EUNSUPPORTED    # 256 keys * 16 MiB: beyond the 32-bit key offsets
    assert call(shape(kr, B=2, flags=kr.KRUL_FLAG_GENERIC_KERNEL), ss=136, ws_bytes=16) == kr.KRUL_EWORKSPACE
    assert call(shape(kr, B=1), sb=0, ws_bytes=16) == kr.KRUL_EWORKSPACE   # one conversation: k_stride_b unused
    assert call(shape(kr, Hq=3)) == kr.KRUL_EINVAL
    assert call(ws_bytes=16) == kr.KRUL_EWORKSPACE


def test_paged_entry_point_rejects_bad_arguments_before_any_gpu_work(kr):
    vp = ctypes.c_void_p
    ok = shape(kr, B=2)           # S = 256

    def call(shp=ok, tab=0x2000, bt=0x4000, bs=16, mb=16, sp=1 << 14, sh=128, ss=256, pages=True, ws_bytes=1 << 40):
        kp = kr.KrulKPages(tab, bt, bs, mb, sp, sh, ss)
        return kr.lib().krul_pair_similarity_paged(ctypes.byref(shp), vp(0x1000), ctypes.byref(kp) if pages else None,
                                                   vp(0x3000), None, None, vp(0x10000), ctypes.c_size_t(ws_bytes), None)
    assert call(pages=False) == kr.KRUL_EINVAL
    assert call(tab=None) == kr.KRUL_EINVAL
    assert call(bt=None) == kr.KRUL_EINVAL
    assert call(bt=0x4002) == kr.KRUL_EINVAL            # int32 table
    assert call(bs=12) == kr.KRUL_EINVAL                # pages hold a power of two of keys ...
    assert call(bs=4) == kr.KRUL_EINVAL                 # ... at least 8
    assert call(mb=15) == kr.KRUL_EINVAL                # 256 keys need 16 pages of 16
    assert call(sp=0) == kr.KRUL_EINVAL
    assert call(ss=64) == kr.KRUL_EINVAL                # keys would overlap
    assert call(ss=136, ws_bytes=16) == kr.KRUL_EWORKSPACE    # any multiple of 8 elements between keys will do
    assert call(ss=1 << 27) == kr.KRUL_EUNSUPPORTED     # beyond the 32-bit offsets inside one copy
    assert call(shape(kr, B=2, flags=kr.KRUL_FLAG_GENERIC_KERNEL), ss=136, ws_bytes=16) == kr.KRUL_EWORKSPACE
    assert call(ws_bytes=16) == kr.KRUL_EWORKSPACE


def test_select_in_one_call_rejects_bad_arguments_before_any_gpu_work(kr):
    vp = ctypes.c_void_p
    ok = shape(kr)           # 4 layers

    def call(shp=ok, n_select=2, pairs=0x5000, count=0x6000, ps=0x3000, ws_bytes=1 << 40):
        return kr.lib().krul_pair_similarity_select(
            ctypes.byref(shp) if shp is not None else None, vp(0x1000), vp(0x2000), None, n_select, vp(ps), None, None,
            vp(pairs), vp(count), vp(0x10000), ctypes.c_size_t(ws_bytes), None, None, None)
    assert call(shp=None) == kr.KRUL_EINVAL
    assert call(n_select=-1) == kr.KRUL_EINVAL
    assert call(n_select=3) == kr.KRUL_EINVAL          # more pairs than 4 layers hold
    assert call(count=None) == kr.KRUL_EINVAL
    assert call(pairs=None) == kr.KRUL_EINVAL
    assert call(pairs=0x5002) == kr.KRUL_EINVAL
    assert call(ps=None) == kr.KRUL_EINVAL
    assert call(ws_bytes=16) == kr.KRUL_EWORKSPACE


def test_accumulate_entry_points_reject_bad_arguments(kr):
    vp = ctypes.c_void_p
    ok = shape(kr)
    L = kr.lib()
    assert L.krul_pair_similarity_accumulate(ctypes.byref(ok), vp(0x1000), vp(0x2000), None, None, vp(0x10000),
                                             ctypes.c_size_t(1 << 40), None) == kr.KRUL_EINVAL
    assert L.krul_pair_similarity_accumulate(ctypes.byref(ok), vp(0x1000), vp(0x2000), vp(0x3000), None, vp(0x10000),
                                             ctypes.c_size_t(16), None) == kr.KRUL_EWORKSPACE
    f = ctypes.c_float
    assert L.krul_pair_scores_from_sums(None, None, 1, 4, 4, f(8.0), vp(0x3000), None, None, None) == kr.KRUL_EINVAL
    assert L.krul_pair_scores_from_sums(vp(0x1000), None, 1, 4, 4, f(0.0), vp(0x3000), None, None, None) == kr.KRUL_EINVAL
    assert L.krul_pair_scores_from_sums(vp(0x1000), None, 1, 1, 4, f(8.0), vp(0x3000), None, None, None) == kr.KRUL_EINVAL
    assert L.krul_pair_scores_from_sums(vp(0x1000), None, 1, 4, 4, f(8.0), None, None, None, None) == kr.KRUL_EINVAL
    # a pair distance needs the distance sums
    assert L.krul_pair_scores_from_sums(vp(0x1000), None, 1, 4, 4, f(8.0), vp(0x3000), None, vp(0x4000), None) == kr.KRUL_EINVAL


def test_all_pairs_entry_points_reject_bad_arguments_before_any_gpu_work(kr):
    vp = ctypes.c_void_p
    ok = shape(kr)
    full = kr.all_pairs_workspace_bytes(ok)
    one = kr.all_pairs_workspace_bytes(ok, 1)
    assert 0 < one <= full and full % 256 == 0
    assert kr.all_pairs_workspace_bytes(shape(kr, L=129)) == 0          # at most 128 layers
    assert kr.all_pairs_workspace_bytes(shape(kr, Hq=3)) == 0
    assert kr.all_pairs_workspace_bytes(shape(kr, dtype=0, d=72)) > 0    # portable kernel
    # the batch grows with the budget, up to all rows
    big = shape(kr, B=2, L=32, Hq=32, Hkv=8, S=4096, Tq=64)
    sizes = [kr.all_pairs_workspace_bytes(big, m) for m in (1, 1 << 27, 1 << 29, 1 << 40)]
    assert sizes == sorted(sizes) and sizes[0] < sizes[-1] and sizes[1] <= 1 << 27 and sizes[2] <= 1 << 29

    def call(shp=ok, q=0x1000, k=0x2000, ps=0x3000, ws=0x10000, ws_bytes=1 << 40):
        return kr.lib().krul_all_pairs_similarity(ctypes.byref(shp), vp(q), vp(k), vp(ps), None, None, vp(ws),
                                                  ctypes.c_size_t(ws_bytes), None)
    assert call(shape(kr, L=1)) == kr.KRUL_EINVAL
    assert call(shape(kr, L=200)) == kr.KRUL_EUNSUPPORTED
    assert call(shape(kr, dtype=5)) == kr.KRUL_EDTYPE
    assert call(q=None) == kr.KRUL_EINVAL
    assert call(ps=None) == kr.KRUL_EINVAL
    assert call(k=0x2008) == kr.KRUL_EINVAL
    assert call(ws=None) == kr.KRUL_EWORKSPACE
    assert call(ws=0x10010) == kr.KRUL_EWORKSPACE
    assert call(ws_bytes=one - 1) == kr.KRUL_EWORKSPACE

    f = kr.lib().krul_select_pairs_all

    def sel(sc=0x1000, B=1, L=8, n=2, op=0x2000, oc=0x3000):
        return f(vp(sc), 1, None, B, L, n, vp(op), vp(oc), None)
    assert sel(sc=None) == kr.KRUL_EINVAL
    assert sel(oc=None) == kr.KRUL_EINVAL
    assert sel(op=None) == kr.KRUL_EINVAL
    assert sel(B=0) == kr.KRUL_EINVAL
    assert sel(L=1) == kr.KRUL_EINVAL
    assert sel(n=5) == kr.KRUL_EINVAL
    assert sel(L=5000, n=1) == kr.KRUL_EUNSUPPORTED
    assert sel(sc=0x1002) == kr.KRUL_EINVAL


def test_select_pairs_rejects_bad_arguments(kr):
    vp = ctypes.c_void_p
    f = kr.lib().krul_select_pairs
    good = dict(ps=vp(0x1000), el=None, B=1, L=8, n=2, op=vp(0x2000), oc=vp(0x3000))

    def call(**kw):
        a = {**good, **kw}
        return f(a["ps"], a["el"], a["B"], a["L"], a["n"], a["op"], a["oc"], None)
    assert call(ps=None) == kr.KRUL_EINVAL
    assert call(oc=None) == kr.KRUL_EINVAL
    assert call(op=None) == kr.KRUL_EINVAL
    assert call(B=0) == kr.KRUL_EINVAL
    assert call(L=1) == kr.KRUL_EINVAL
    assert call(n=-1) == kr.KRUL_EINVAL
    assert call(n=5) == kr.KRUL_EINVAL              # more pairs than N/2
    assert call(L=5000, n=1) == kr.KRUL_EUNSUPPORTED
    assert call(ps=vp(0x1002)) == kr.KRUL_EINVAL


def test_binding_refuses_cpu_tensors(kr):
    import torch
    q = torch.zeros((1, 2, 2, 2, 64), dtype=torch.bfloat16)
    k = torch.zeros((1, 2, 2, 4, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        kr.pair_similarity(q, k)
    with pytest.raises(ValueError):
        kr.select_pairs(torch.zeros((1, 3)), 1)


def test_plan_for_the_benchmark_shapes(kr):
    """krul_pair_similarity_plan is host logic: which kernel form and grid each benchmark shape gets."""
    import workloads

    def plan(name, **over):
        B, L, Hq, Hkv, d, S, Tq, dt, _ = workloads.CONFIGS[name]
        dtype = {"f32": kr.KRUL_F32, "bf16": kr.KRUL_BF16, "f16": kr.KRUL_F16}[dt]
        a = dict(B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, flags=0)
        a.update(over)
        return kr.plan(kr.KrulShape(a["B"], a["L"], a["Hq"], a["Hkv"], a["d"], a["S"], a["Tq"], dtype, 0.0, a["flags"]))

    assert plan("C1")["form"] == 0                                   # fp32: the portable kernel
    c2 = plan("C2")
    assert c2["form"] == 1 and c2["n_workgroups"] == 256 and c2["n_key_splits"] == 16
    assert plan("C3")["form"] == 2                                   # 64 rows per kv head: the 64 x 512 tile
    c4, c5 = plan("C4"), plan("C5")
    # many query rows: 256 x 256 tiles, four key splits per row tile (patches of 8 row tiles x 4 splits)
    assert c4["form"] == 8 and c4["n_key_splits"] == 4 and c4["n_workgroups"] == 8 * 32 * 4
    assert c5["form"] == 8 and c5["n_key_splits"] == 4 and c5["n_workgroups"] == 64 * 8 * 4
    assert plan("D1")["form"] in (3, 4) and plan("D2")["form"] in (3, 4) and plan("D3")["form"] == 5
    # a mask keeps the many-query shapes on the 128-row kernel; the single-split flag changes the grid, not the kernel
    assert plan("C4", flags=kr.KRUL_FLAG_CAUSAL)["form"] == 1
    one = plan("C4", flags=kr.KRUL_FLAG_SINGLE_SPLIT)
    assert one["form"] == 8 and one["n_key_splits"] == 1
    # the workspace covers whichever plan the call takes
    B, L, Hq, Hkv, d, S, Tq, _, _ = workloads.CONFIGS["C5"]
    sh = kr.KrulShape(B, L, Hq, Hkv, d, S, Tq, kr.KRUL_BF16, 0.0, 0)
    records = c5["n_workgroups"] * L * 256 * 16
    assert kr.workspace_bytes(sh) >= records


def test_static_entry_point_rejects_what_does_not_fit_before_any_gpu_work(kr):
    lib = kr.lib()
    import workloads
    B, L, Hq, Hkv, d, S, Tq, _, _ = workloads.CONFIGS["C5"]
    big = kr.KrulShape(B, L, Hq, Hkv, d, S, Tq, kr.KRUL_BF16, 0.0, 0)
    assert kr.workspace_bytes(big) > kr.KRUL_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(256)
    rc = lib.krul_pair_similarity_static(ctypes.byref(big), fake, fake, fake, None, None, None)
    assert rc == kr.KRUL_ESCRATCH
    bad = kr.KrulShape(1, 1, 8, 2, 128, 64, 4, kr.KRUL_BF16, 0.0, 0)      # one layer: no pair
    assert lib.krul_pair_similarity_static(ctypes.byref(bad), fake, fake, fake, None, None, None) == kr.KRUL_EINVAL


def test_calibration_entry_points_reject_bad_arguments(kr):
    lib = kr.lib()
    assert lib.krul_calibration_block(3, 7, 10, ctypes.c_void_p(256), None) == kr.KRUL_EINVAL     # row blocks: 1 or 2
    assert lib.krul_calibration_block(2, 7, 0, ctypes.c_void_p(256), None) == kr.KRUL_EINVAL      # no iterations
    assert lib.krul_calibration_block(2, 7, 10, None, None) == kr.KRUL_EINVAL                     # no output
