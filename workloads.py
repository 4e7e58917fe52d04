"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws random Q and K
tensors with the shapes and correlation structure of the five benchmark
configurations and rounds them to the storage type once.  Both the fp64 oracle and
the GPU library read the very same bits it returns.

The inputs stand in for the per-layer queries and keys a LLaMA / Qwen forward
pass would produce on multi-turn conversations (the paper's ShareGPT / LongBench
runs); no dataset item and no trained weight is involved.

Recipe (all configurations):
  layer 0:   Q_0, K_0 ~ N(0,1) i.i.d.
  layer l+1: K_{l+1} = rho_k * K_l + sqrt(1 - rho_k^2) * eps,  eps ~ N(0,1) fresh,
             Q_{l+1} = rho_q * Q_l + sqrt(1 - rho_q^2) * eps', rho_q = 0.95,
  so every layer keeps unit marginals and the logits of adjacent layers are
  correlated with r = rho_q * rho_k.  The recursion runs in float32 on unrounded
  values; each layer is rounded to the storage type (float32 kept, bf16
  round-to-nearest-even) when it is written out.
  Arrays: q [B, L, Hq, Tq, d], k [B, L, Hkv, S, d]; bf16 is returned as uint16
  bit patterns (view them as torch.bfloat16 on the device side).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 0x4B52554C  # "KRUL"

# name -> (B, L, Hq, Hkv, d, S, Tq, dtype, n_select)
CONFIGS = {
    "C1": (1, 4, 2, 2, 64, 256, 16, "f32", 1),
    "C2": (1, 32, 32, 8, 128, 4096, 64, "bf16", 8),
    "C3": (1, 32, 32, 8, 128, 32768, 16, "bf16", 8),
    "C4": (1, 32, 32, 8, 128, 8192, 2048, "bf16", 8),
    "C5": (8, 80, 64, 8, 128, 16384, 256, "bf16", 20),
    # decode steps (one query token per conversation; the token-wise scoring of Sec. 5) -- not among the
    # benchmark's five configurations, kept here so that their measurements can be repeated
    "D1": (8, 32, 32, 8, 128, 4096, 1, "bf16", 8),      # eight conversations, 4096 tokens each
    "D2": (1, 32, 32, 8, 128, 131072, 1, "bf16", 8),    # one long conversation
    "D3": (1, 32, 32, 8, 128, 4096, 1, "bf16", 8),      # one short conversation: too small to fill the chip
}
_CFG_ID = {"C1": 1, "C2": 2, "C3": 3, "C4": 4, "C5": 5, "D1": 6, "D2": 7, "D3": 8}


@dataclass
class Workload:
    name: str
    B: int
    L: int
    Hq: int
    Hkv: int
    d: int
    S: int
    Tq: int
    dtype: str            # "f32", "f16" or "bf16"
    n_select: int
    q: np.ndarray         # float32, float16, or uint16 bf16 bits
    k: np.ndarray
    rho_k: np.ndarray     # [B, L-1, Hkv] correlation used for each pair and kv head
    rho_q: float
    sinks: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.int64))

    @property
    def score_elems(self) -> int:
        return self.B * (self.L - 1) * self.Hq * self.Tq * self.S


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return x.astype(np.float32, copy=True)
    return x.astype(np.float16) if dtype == "f16" else f32_to_bf16_bits(x)


def make(name: str = "custom", *, B, L, Hq, Hkv, d, S, Tq, dtype="bf16", n_select=None,
         rho_k=0.8, rho_q=0.95, seed=BASE_SEED, sink_frac=0.0, sink_gain=4.0, progress=None) -> Workload:
    """Draw one workload.  rho_k: scalar, or an array broadcastable to [B, L-1, Hkv].
    progress: called with (conversation index, B) after each conversation is drawn (large workloads)."""
    rho = np.broadcast_to(np.asarray(rho_k, dtype=np.float32), (B, L - 1, Hkv)).copy()
    store_t = {"f32": np.float32, "f16": np.float16}.get(dtype, np.uint16)
    q = np.empty((B, L, Hq, Tq, d), dtype=store_t)
    k = np.empty((B, L, Hkv, S, d), dtype=store_t)
    rq, rk, re_q, re_k = _rng(seed, 1), _rng(seed, 2), _rng(seed, 3), _rng(seed, 4)
    sinks = np.zeros(0, dtype=np.int64)
    gain = None
    if sink_frac > 0.0:
        n_sink = max(1, int(round(sink_frac * S)))
        sinks = np.sort(_rng(seed, 5).choice(S, size=n_sink, replace=False))
        gain = np.ones((1, S, 1), dtype=np.float32)
        gain[0, sinks, 0] = sink_gain
    cq = np.float32(np.sqrt(1.0 - rho_q * rho_q))
    for b in range(B):
        qc = rq.standard_normal((Hq, Tq, d), dtype=np.float32)
        kc = rk.standard_normal((Hkv, S, d), dtype=np.float32)
        for l in range(L):
            if l > 0:
                r = rho[b, l - 1][:, None, None]
                kc = r * kc + np.sqrt(1.0 - r * r) * re_k.standard_normal((Hkv, S, d), dtype=np.float32)
                qc = np.float32(rho_q) * qc + cq * re_q.standard_normal((Hq, Tq, d), dtype=np.float32)
            q[b, l] = _store(qc, dtype)
            k[b, l] = _store(kc if gain is None else kc * gain, dtype)
        if progress is not None:
            progress(b, B)
    if n_select is None:
        n_select = max(1, L // 4)
    return Workload(name, B, L, Hq, Hkv, d, S, Tq, dtype, n_select, q, k, rho, rho_q, sinks)


def config(name: str, *, batch=None, seed=None, progress=None) -> Workload:
    """One of the benchmark configurations C1..C5, or of the decode-step shapes D1..D3 (full size unless batch
    is cut)."""
    B, L, Hq, Hkv, d, S, Tq, dtype, n_select = CONFIGS[name]
    if batch is not None:
        B = batch
    seed = BASE_SEED + _CFG_ID[name] if seed is None else seed
    rr = _rng(seed, 6)
    kw = {}
    if name == "C1":
        rho = 0.8                                   # K_{l+1} = 0.8 K_l + 0.6 noise
    elif name == "C4":
        rho = rr.uniform(0.5, 0.95, size=(B, L - 1, Hkv))   # varies per pair and per kv head
    else:
        rho = rr.uniform(0.5, 0.95, size=(B, L - 1, 1))     # one rho per pair
    if name in ("C3", "D2"):
        kw = dict(sink_frac=0.02, sink_gain=4.0)
    return make(name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, n_select=n_select,
                rho_k=rho, seed=seed, progress=progress, **kw)


def scaled(name: str, *, S=None, Tq=None, L=None, batch=None, seed=None) -> Workload:
    """A configuration with some extents cut down (same recipe), for quick parity cases."""
    B0, L0, Hq, Hkv, d, S0, Tq0, dtype, n_select = CONFIGS[name]
    B = batch or B0
    L = L or L0
    seed = BASE_SEED + _CFG_ID[name] if seed is None else seed
    rr = _rng(seed, 6)
    per_head = Hkv if name == "C4" else 1
    rho = 0.8 if name == "C1" else rr.uniform(0.5, 0.95, size=(B, L - 1, per_head))
    kw = dict(sink_frac=0.02, sink_gain=4.0) if name == "C3" else {}
    return make(name + "-cut", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S or S0, Tq=Tq or Tq0, dtype=dtype,
                n_select=max(1, L // 4), rho_k=rho, seed=seed, **kw)


def config_device(name: str, *, device="cuda", batch=None, seed=None, progress=None):
    """The same recipe drawn ON THE DEVICE with torch's seeded Philox generator, for configurations whose
    host draw takes minutes (C5: 22.5 GiB).  Returns (q, k, info): q [B, L, Hq, Tq, d] and k [B, L, Hkv, S, d]
    as device tensors of the storage type, info = dict(name, shape fields, n_select, rho_k [B, L-1, Hkv] numpy,
    rho_q, sinks).  The numbers differ from config()'s numpy draw (another generator), the recipe does not.
    progress: called with (conversation index, B) after each conversation is drawn."""
    import torch
    B, L, Hq, Hkv, d, S, Tq, dtype, n_select = CONFIGS[name]
    if batch is not None:
        B = batch
    seed = BASE_SEED + _CFG_ID[name] if seed is None else seed
    rr = _rng(seed, 6)
    if name == "C1":
        rho = np.full((B, L - 1, Hkv), 0.8)
    elif name == "C4":
        rho = rr.uniform(0.5, 0.95, size=(B, L - 1, Hkv))
    else:
        rho = np.broadcast_to(rr.uniform(0.5, 0.95, size=(B, L - 1, 1)), (B, L - 1, Hkv)).copy()
    rho = rho.astype(np.float32)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    q = torch.empty((B, L, Hq, Tq, d), dtype=tdt, device=device)
    k = torch.empty((B, L, Hkv, S, d), dtype=tdt, device=device)
    sinks = np.zeros(0, dtype=np.int64)
    gain = None
    if name in ("C3", "D2"):
        n_sink = max(1, int(round(0.02 * S)))
        sinks = np.sort(_rng(seed, 5).choice(S, size=n_sink, replace=False))
        gain = torch.ones((1, S, 1), dtype=torch.float32, device=device)
        gain[0, torch.from_numpy(sinks).to(device), 0] = 4.0
    rho_q = 0.95
    cq = float(np.sqrt(1.0 - rho_q * rho_q))
    rho_t = torch.from_numpy(rho).to(device)
    for b in range(B):
        qc = torch.randn((Hq, Tq, d), generator=g, device=device, dtype=torch.float32)
        kc = torch.randn((Hkv, S, d), generator=g, device=device, dtype=torch.float32)
        for l in range(L):
            if l > 0:
                r = rho_t[b, l - 1][:, None, None]
                kc = r * kc + torch.sqrt(1.0 - r * r) * torch.randn((Hkv, S, d), generator=g, device=device,
                                                                    dtype=torch.float32)
                qc = rho_q * qc + cq * torch.randn((Hq, Tq, d), generator=g, device=device, dtype=torch.float32)
            q[b, l] = qc.to(tdt)
            k[b, l] = (kc if gain is None else kc * gain).to(tdt)
        if progress is not None:
            progress(b, B)
    info = dict(name=name, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, S=S, Tq=Tq, dtype=dtype, n_select=n_select,
                rho_k=rho, rho_q=rho_q, sinks=sinks, score_elems=B * (L - 1) * Hq * Tq * S)
    return q, k, info


def units_to_host(q, k, units):
    """Copy the inputs of chosen (b, l, h) units -- query head h and its kv head, layers l and l+1 -- from device
    tensors to the host, as one small problem per unit: (q_units [n, 2, 1, Tq, d], k_units [n, 2, 1, S, d]),
    numpy arrays of the storage type's bits (bf16 as uint16).  Unit i is conversation i of that problem, with two
    layers and one head, so its one head score is the score of (b, l, h)."""
    import torch
    g = q.shape[2] // k.shape[2]
    qs = torch.stack([q[b, l:l + 2, h] for b, l, h in units])[:, :, None]
    ks = torch.stack([k[b, l:l + 2, h // g] for b, l, h in units])[:, :, None]

    def bits(t):
        t = t.contiguous().cpu()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()
    return bits(qs), bits(ks)
