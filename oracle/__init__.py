"""fp64 CPU oracle for the Krul attention-similarity path -- TEST INFRASTRUCTURE.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It wraps ``krul_oracle.c`` (plain C, fp64, compiled here
with gcc) through ctypes and shares nothing with the GPU library: no header, no
kernel, no helper.  See the header of ``krul_oracle.c`` for what each function
computes and which passage of the paper (Sec. 2.1, Sec. 4.2 / Alg. 1, Sec. 5,
Sec. 7) it follows.

Inputs are numpy arrays: float32, float16, or uint16 holding bf16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "krul_oracle.c")
_LIB = os.path.join(_HERE, "libkrul_oracle.so")

F32, BF16, F16 = 0, 1, 2


class _Shape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_layers", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("n_hist", ctypes.c_int32),
        ("n_query", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_double), ("causal", ctypes.c_int32),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP, no fast-math so sums keep their order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.krul_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().krul_oracle_num_threads())


def _prep(q: np.ndarray, k: np.ndarray, scale, causal=False):
    if q.ndim != 5 or k.ndim != 5:
        raise ValueError("q must be [B,L,Hq,Tq,d] and k [B,L,Hkv,S,d]")
    if q.dtype != k.dtype:
        raise ValueError("q and k must share a dtype")
    if q.dtype == np.float32:
        dt = F32
    elif q.dtype == np.uint16:
        dt = BF16
    elif q.dtype == np.float16:
        dt = F16
    else:
        raise ValueError("dtype must be float32, float16 or uint16 (bf16 bits)")
    B, L, Hq, Tq, d = q.shape
    B2, L2, Hkv, S, d2 = k.shape
    if (B, L, d) != (B2, L2, d2):
        raise ValueError("q and k disagree on batch, layers or head_dim")
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    shp = _Shape(B, L, Hq, Hkv, d, S, Tq, dt, float(scale) if scale else 0.0, 1 if causal else 0)
    return q, k, shp


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def pair_similarity(q: np.ndarray, k: np.ndarray, scale=None, causal=False) -> dict:
    """All scores: dict with pair_score [B,L-1], head_score [B,L-1,Hq] (cosine) and
    pair_dist, head_dist (Euclidean), all float64.  causal: the Tq rows are the last Tq tokens of
    the S-token sequence and row t sees keys j <= S - Tq + t."""
    q, k, shp = _prep(q, k, scale, causal)
    B, NP, H = shp.batch, shp.n_layers - 1, shp.n_q_heads
    out = {
        "pair_score": np.empty((B, NP)), "head_score": np.empty((B, NP, H)),
        "pair_dist": np.empty((B, NP)), "head_dist": np.empty((B, NP, H)),
    }
    rc = _load().krul_oracle_pair_similarity(
        ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(out["pair_score"]), _ptr(out["head_score"]),
        _ptr(out["pair_dist"]), _ptr(out["head_dist"]))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def unit_scores(q: np.ndarray, k: np.ndarray, units, scale=None, causal=False):
    """Scores of chosen (b, l, h) units only: returns (head_cos[n], head_dist[n])."""
    q, k, shp = _prep(q, k, scale, causal)
    units = np.ascontiguousarray(np.asarray(units, dtype=np.int32).reshape(-1, 3))
    n = units.shape[0]
    hc, hd = np.empty(n), np.empty(n)
    rc = _load().krul_oracle_units(ctypes.byref(shp), _ptr(q), _ptr(k), ctypes.c_int(n),
                                   _ptr(units), _ptr(hc), _ptr(hd))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return hc, hd


def select_pairs(pair_score, n_select: int, eligible=None):
    """Greedy disjoint adjacent-pair choice (Alg. 1).  pair_score [B,L-1] -> (pairs
    [B,n_select] int32 padded with -1, count [B] int32)."""
    ps = np.ascontiguousarray(np.asarray(pair_score, dtype=np.float64))
    if ps.ndim == 1:
        ps = ps[None, :]
    B, NP = ps.shape
    L = NP + 1
    el = None
    if eligible is not None:
        el = np.ascontiguousarray(np.asarray(eligible, dtype=np.uint8).reshape(B, L))
    pairs = np.empty((B, max(n_select, 0)), dtype=np.int32)
    count = np.empty((B,), dtype=np.int32)
    rc = _load().krul_oracle_select_pairs(
        _ptr(ps), _ptr(el) if el is not None else None, ctypes.c_int(B), ctypes.c_int(L),
        ctypes.c_int(n_select), _ptr(pairs), _ptr(count))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return pairs, count


def ir_mass(q: np.ndarray, k: np.ndarray, gamma: float, scale=None):
    """Sec. 4.2 input-insensitive layer test: (mass [B,L] float64, eligible [B,L] uint8)."""
    q, k, shp = _prep(q, k, scale)
    B, L = shp.batch, shp.n_layers
    mass = np.empty((B, L))
    el = np.empty((B, L), dtype=np.uint8)
    rc = _load().krul_oracle_ir_mass(ctypes.byref(shp), _ptr(q), _ptr(k), ctypes.c_double(gamma),
                                     _ptr(mass), _ptr(el))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return mass, el


def all_pairs(q: np.ndarray, k: np.ndarray, scale=None, causal=False) -> dict:
    """Similarity of every two layers (Alg. 1 as printed): dict with pair_score, pair_dist [B,L,L]
    and head_score, head_dist [B,Hq,L,L], float64, symmetric, diagonal cos 1 / distance 0."""
    q, k, shp = _prep(q, k, scale, causal)
    B, L, H = shp.batch, shp.n_layers, shp.n_q_heads
    out = {
        "pair_score": np.empty((B, L, L)), "pair_dist": np.empty((B, L, L)),
        "head_score": np.empty((B, H, L, L)), "head_dist": np.empty((B, H, L, L)),
    }
    rc = _load().krul_oracle_all_pairs(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(out["pair_score"]),
                                       _ptr(out["pair_dist"]), _ptr(out["head_score"]), _ptr(out["head_dist"]))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def all_pairs_heads(q: np.ndarray, k: np.ndarray, heads, scale=None, causal=False):
    """The all-pairs matrices of chosen (b, h) heads only: (head_cos [n,L,L], head_dist [n,L,L])."""
    q, k, shp = _prep(q, k, scale, causal)
    heads = np.ascontiguousarray(np.asarray(heads, dtype=np.int32).reshape(-1, 2))
    n, L = heads.shape[0], shp.n_layers
    hc, hd = np.empty((n, L, L)), np.empty((n, L, L))
    rc = _load().krul_oracle_all_pairs_heads(ctypes.byref(shp), _ptr(q), _ptr(k), ctypes.c_int(n), _ptr(heads),
                                             _ptr(hc), _ptr(hd))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return hc, hd


def select_pairs_all(score, n_select: int, closer_is_smaller: bool, eligible=None):
    """Greedy disjoint choice over every two layers (Alg. 1).  score [B,L,L] (lower triangle read) ->
    (pairs [B,n_select,2] int32 as (j, i), j < i, padded with -1; count [B] int32)."""
    sc = np.ascontiguousarray(np.asarray(score, dtype=np.float64))
    if sc.ndim == 2:
        sc = sc[None]
    B, L, L2 = sc.shape
    if L != L2:
        raise ValueError("score must be [B,L,L]")
    el = None
    if eligible is not None:
        el = np.ascontiguousarray(np.asarray(eligible, dtype=np.uint8).reshape(B, L))
    pairs = np.empty((B, max(n_select, 0), 2), dtype=np.int32)
    count = np.empty((B,), dtype=np.int32)
    rc = _load().krul_oracle_select_pairs_all(
        _ptr(sc), ctypes.c_int(1 if closer_is_smaller else 0), _ptr(el) if el is not None else None,
        ctypes.c_int(B), ctypes.c_int(L), ctypes.c_int(n_select), _ptr(pairs), _ptr(count))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return pairs, count
