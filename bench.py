#!/usr/bin/env python3
"""Benchmark of the cross-layer attention-similarity path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input already
resident in HBM: krul_pair_similarity (logits, online softmax sums, cross term, row
similarity, token-wise aggregation) followed by krul_select_pairs, on one stream.
Prints ONE JSON line.  Metric: layer-pair similarity throughput in Gscore-elems/s,
score-elems = B*(L-1)*Hq*Tq*S (one per pair of attention probabilities compared).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def algorithmic_bytes(w) -> int:
    """Every K and Q element once, plus the score outputs."""
    e = 4 if w.dtype == "f32" else 2
    return w.B * w.L * w.d * e * (w.Hkv * w.S + w.Hq * w.Tq) + 4 * w.B * (w.L - 1) * (w.Hq + 1)


def algorithmic_flops(w) -> int:
    """Each layer's logits once: 2*d flops per logit."""
    return 2 * w.d * w.B * w.L * w.Hq * w.Tq * w.S


def algorithmic_valu_ops(w, with_dist=False) -> int:
    """Vector-unit issue slots per logit, per lane: scale-and-shift fma, exp2 (two slots), the fma into the sum of
    squares and the fma into the cross term (+ one add into the plain sum when the distance is asked for)."""
    return (6 if with_dist else 5) * w.B * w.L * w.Hq * w.Tq * w.S


# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: lane operations per second of the vector units, one operation per
# lane and issue slot (the packed-fp32 forms, which would double it, are compiled out)
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def cpu_baseline(w, q, k, seconds_target=15.0):
    """The fp64 oracle, as it stands, on a bounded seeded sample of (conversation, pair, head) units -- all query
    rows and all keys of each -- copied back from the device tensors the GPU path read.  Work is linear in units,
    so the figure is the sample's own rate (score-elems of the sample / wall time)."""
    import numpy as np
    import oracle
    import workloads
    oracle.build()
    n_all = w.B * (w.L - 1) * w.Hq
    rng = np.random.default_rng(12345)
    threads = oracle.num_threads()

    def draw(n):
        idx = rng.choice(n_all, size=min(n, n_all), replace=False)
        return [(int(i // ((w.L - 1) * w.Hq)), int(i // w.Hq % (w.L - 1)), int(i % w.Hq)) for i in idx]

    def run(units):
        qs, ks = workloads.units_to_host(q, k, units)
        t0 = time.perf_counter()
        oracle.pair_similarity(qs, ks)
        return time.perf_counter() - t0

    # calibrate on one unit per thread, then size the sample for about seconds_target
    t_probe = run(draw(threads))
    n = int(min(n_all, max(threads, threads * (seconds_target / max(t_probe, 1e-3)))))
    n = min(max(threads, n // threads * threads), n_all, 4096)
    dt = run(draw(n))
    elems = n * w.Tq * w.S
    return {
        "value": elems / dt / 1e9, "unit": "Gscore-elems/s", "cores": threads, "kind": "oracle",
        "sample": f"{n} of {n_all} (conversation, pair, head) units of {w.name}, all rows and keys of each, "
                  f"{dt:.1f} s wall; the whole workload extrapolated from these n units: "
                  f"{dt * n_all / n:.0f} s",
    }


def all_pairs_bench(args, kr, torch, w, q, k, shp):
    """One step = krul_all_pairs_similarity (cosine and distance of every two layers) + krul_select_pairs_all
    on the distances.  The whole call is timed with events on the stream it runs on (torch's current one)."""
    ws = torch.empty(kr.all_pairs_workspace_bytes(shp), dtype=torch.uint8, device="cuda")

    def step():
        out = kr.all_pairs_similarity(q, k, flags=args.flags, workspace=ws)
        return kr.select_pairs_all(out["pair_dist"], w.n_select, True)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        pairs, _count = step()
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gpu_s = e0.elapsed_time(e1) * 1e-3 / args.steps
    in_bytes = (q.numel() + k.numel()) * q.element_size()
    out_bytes = 2 * w.B * w.L * w.L * 4
    weights_bytes = w.B * w.Hq * w.Tq * w.L * ((w.S + 31) // 32 * 32) * 2   # fp16 attention weights, written once, read once
    design_bytes = in_bytes + 2 * weights_bytes
    res = {
        "metric": "all-pairs layer similarity throughput", "value": w.score_elems / (dt / args.steps) / 1e9,
        "unit": "Gscore-elems/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} L={w.L} Hq/Hkv={w.Hq}/{w.Hkv} d={w.d} S={w.S} Tq={w.Tq} "
                               f"{w.dtype}, all {w.L * (w.L - 1) // 2} layer pairs, select {w.n_select}",
                   "score_elems": w.score_elems, "outputs": "pair_score_all+pair_dist_all", "workspace_bytes": ws.numel()},
        # against the algorithmic bytes (inputs once, outputs once); what this design moves on top of them -- the
        # fp16 attention weights out to HBM and back -- is given as design_traffic, and its ratio to the
        # algorithmic bytes says how far the path is from a fused one
        "roofline": {"bound": "hbm", "achieved": (in_bytes + out_bytes) / gpu_s / 1e9, "peak": 8000.0,
                     "unit": "GB/s", "frac": (in_bytes + out_bytes) / gpu_s / 1e9 / 8000.0, "traffic": None,
                     "kernel": "whole call (weights, scale, Gram, row, reduce kernels)", "kernel_us": gpu_s * 1e6,
                     "algorithmic_bytes": in_bytes + out_bytes, "design_traffic": design_bytes,
                     "design_traffic_over_algorithmic": design_bytes / (in_bytes + out_bytes),
                     "design_traffic_frac_of_peak": design_bytes / gpu_s / 1e9 / 8000.0},
        "selected_pairs": pairs.cpu().tolist()[0],
    }
    print(json.dumps(res))


def block_step_ns(kr, torch, rb, parts, iters=1500):
    """ns per 32 x 32 block of logits and SIMD of krul_calibration_block(rb, parts): two waves per SIMD, each
    2 * rb * iters blocks."""
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    for _ in range(2):
        kr.calibration_block(rb, parts, iters, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        kr.calibration_block(rb, parts, iters, out)
    e1.record()
    torch.cuda.synchronize()
    return round(e0.elapsed_time(e1) / 3 * 1e6 / (2 * 2 * rb * iters), 1)


def micro_bench(args, kr, torch):
    """The inner step of the similarity kernels with no memory traffic (krul_calibration_block): the floors
    'matrix cores alone', 'vector units alone', 'both from one instruction stream' per 32 x 32 block of logits,
    on one 8-wave workgroup per CU (two waves per SIMD).  Prints one JSON line."""
    res = {"metric": "block step of the similarity kernels, no memory traffic", "unit": "ns per 32x32 block of logits and SIMD",
           "blocks_per_wave": "2 * row_blocks * 1500", "waves_per_simd": 2, "results": {}}
    names = {1: "mfma", 2: "valu", 3: "mfma+valu", 5: "lds+mfma", 7: "lds+mfma+valu"}
    for rb in (1, 2):
        for parts in (1, 2, 3, 5, 7):
            res["results"][f"row_blocks={rb} {names[parts]}"] = block_step_ns(kr, torch, rb, parts)
    # the matrix cores' own time for a block: 8 MFMAs x 32 cycles at the clock the chain ran at
    res["note"] = ("a block is 8 MFMAs 32x32x16 (256 cycles of a SIMD's matrix core: 107 ns at 2.4 GHz) and the vector work "
                   "of 16 logits per lane")
    print(json.dumps(res))


class _Shape:
    """Extents and names of the workload being timed (the numbers live in the device tensors)."""
    def __init__(self, **kw):
        self.__dict__.update(kw)
        self.score_elems = self.B * (self.L - 1) * self.Hq * self.Tq * self.S


def load_inputs(name, torch, np):
    """(shape, [(q, k), ...]): the configuration's inputs on the device.  C5 (22.5 GiB) is drawn on the device;
    the others on the host, as the parity tests draw them.  Inputs smaller than twice the 256 MB last-level cache
    are held in two copies at different addresses and the steps alternate between them, so that no step finds
    the inputs of the step before it in that cache."""
    import workloads
    if name == "C5":
        q, k, info = workloads.config_device(
            name, progress=lambda b, n: print(f"bench.py: drew conversation {b + 1} of {n}", file=sys.stderr, flush=True))
        w = _Shape(**{f: info[f] for f in ("name", "B", "L", "Hq", "Hkv", "d", "S", "Tq", "dtype", "n_select")})
        return w, [(q, k)]
    ww = workloads.config(name)
    w = _Shape(**{f: getattr(ww, f) for f in ("name", "B", "L", "Hq", "Hkv", "d", "S", "Tq", "dtype", "n_select")})
    if ww.dtype == "f32":
        q, k = torch.from_numpy(ww.q).cuda(), torch.from_numpy(ww.k).cuda()
    else:
        q = torch.from_numpy(ww.q.view(np.int16)).cuda().view(torch.bfloat16)
        k = torch.from_numpy(ww.k.view(np.int16)).cuda().view(torch.bfloat16)
    sets = [(q, k)]
    if (q.numel() + k.numel()) * q.element_size() < 2 * 256e6:
        sets.append((q.clone(), k.clone()))
    return w, sets


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", choices=["C1", "C2", "C3", "C4", "C5", "D1", "D2", "D3"],
                    help="C5 (the default; the largest configuration that fits one GPU) draws its 22.5 GiB of inputs on "
                         "the device.  D1..D3 are decode-step shapes (one query token), not among the benchmark's "
                         "configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--with-dist", action="store_true",
                    help="also ask for the Euclidean distance by-product (pair_dist)")
    ap.add_argument("--two-calls", action="store_true",
                    help="score with krul_pair_similarity and select with krul_select_pairs, instead of the one "
                         "call that does both (krul_pair_similarity_select)")
    ap.add_argument("--all-pairs", action="store_true",
                    help="time the all-pairs reading instead (every two layers scored, then the greedy choice "
                         "over all of them); not the headline metric")
    ap.add_argument("--micro", action="store_true",
                    help="run the block-step calibration kernels instead (floors of the matrix cores, the vector units, "
                         "and both together for the similarity kernels' inner step); not the headline metric")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run the library's plain copy kernel on MIB MiB a few times (a known-size "
                         "reference for rocprofv3 traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus above 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2507_08045_amd as kr
    from paper_2507_08045_amd import hipevents

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.micro:
        micro_bench(args, kr, torch)
        return
    w, sets = load_inputs(args.config, torch, np)
    q, k = sets[0]
    torch.cuda.synchronize()
    print(f"bench.py: inputs of {w.name} on the device ({len(sets)} buffer set(s))", file=sys.stderr, flush=True)

    shp = kr.make_shape(q, k, 0.0, args.flags)
    if args.all_pairs:
        all_pairs_bench(args, kr, torch, w, q, k, shp)
        return
    ws = torch.empty(kr.workspace_bytes(shp), dtype=torch.uint8, device="cuda")
    out = {
        "pair_score": torch.empty((w.B, w.L - 1), dtype=torch.float32, device="cuda"),
        "head_score": torch.empty((w.B, w.L - 1, w.Hq), dtype=torch.float32, device="cuda"),
    }
    if args.with_dist:   # the Euclidean by-product costs one more running sum per logit
        out["pair_dist"] = torch.empty((w.B, w.L - 1), dtype=torch.float32, device="cuda")
    pairs = torch.empty((w.B, w.n_select), dtype=torch.int32, device="cuda")
    count = torch.empty((w.B,), dtype=torch.int32, device="cuda")
    K = args.steps
    # The similarity kernel is timed with HIP events (on the stream the library launches on) on a sample of
    # the timed steps: an event pair costs a few microseconds of stream time, which for a step of a hundred
    # microseconds would distort the step time it is measured within.
    EV_EVERY = 4 if K >= 16 else 1
    evs = [(hipevents.create(), hipevents.create()) if i % EV_EVERY == 0 else None for i in range(K)]

    out_sel = dict(out, pairs=pairs, count=count)

    def step(i, ev=None):
        qi, ki = sets[i % len(sets)]
        if args.two_calls:
            kr.pair_similarity(qi, ki, flags=args.flags, workspace=ws, out=out, events=ev,
                               want_pair_dist=args.with_dist)
            kr.select_pairs(out["pair_score"], w.n_select, out_pairs=pairs, out_count=count)
        else:   # the same two steps of Alg. 1 through the entry point that enqueues both
            kr.pair_similarity_select(qi, ki, w.n_select, flags=args.flags, workspace=ws, out=out_sel, events=ev,
                                      want_pair_dist=args.with_dist)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i, evs[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    if args.copy_calibration > 0:
        a = torch.empty(args.copy_calibration << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        b = torch.empty_like(a)
        for _ in range(5):
            kr.calibration_copy(a, b)
        torch.cuda.synchronize()

    evs = [e for e in evs if e is not None]
    kern_ms = [hipevents.elapsed_ms(a, b) for a, b in evs]
    for a, b in evs:
        hipevents.destroy(a)
        hipevents.destroy(b)
    kern_s = float(np.mean(kern_ms)) * 1e-3
    ms_per_step = dt / K * 1e3
    value = w.score_elems / (dt / K) / 1e9

    bytes_alg, flops_alg = algorithmic_bytes(w), algorithmic_flops(w)
    valu_alg = algorithmic_valu_ops(w, args.with_dist)
    # HBM bytes per launch by rocprofv3 counters: recorded by an earlier profiling run of this library (the file
    # names its command), not measured by this run
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
        traffic_src = f"profiles/traffic_{w.name}.json (recorded by a rocprofv3 --pmc run, not by this run)"
    kernel_name = "sim_generic_kernel" if args.flags & kr.KRUL_FLAG_GENERIC_KERNEL else kr.plan(shp)["kernel"]
    hbm = {"bound": "hbm", "achieved": bytes_alg / kern_s / 1e9, "peak": 8000.0, "unit": "GB/s",
           "frac": bytes_alg / kern_s / 1e9 / 8000.0, "algorithmic_bytes": bytes_alg}
    mfma = {"bound": "mfma", "achieved": flops_alg / kern_s / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
            "frac": flops_alg / kern_s / 1e12 / 2500.0, "algorithmic_flops": flops_alg}
    alu = {"bound": "alu", "achieved": valu_alg / kern_s / 1e12, "peak": VALU_PEAK_TOPS, "unit": "T lane-op/s",
           "frac": valu_alg / kern_s / 1e12 / VALU_PEAK_TOPS, "algorithmic_lane_ops": valu_alg}
    # What the method's own instruction mix allows, measured live: krul_calibration_block runs, per 32 x 32 block of
    # logits, the same MFMA chain, the same operand reads from LDS and the vector work of 16 logits per lane, with no
    # memory traffic, barriers or merges, on every SIMD of the chip.  The matrix and the vector instructions of a SIMD
    # overlap only in part, so this floor lies well above the MFMA roof's; reported beside the three plain roofs.
    mix = None
    if w.dtype == "bf16":
        rb = 2 if kr.plan(shp)["form"] == 8 else 1
        ns = block_step_ns(kr, torch, rb, 7)
        blocks_per_simd = w.B * w.L * w.Hq * w.Tq * w.S / 1024.0 / 1024.0
        mix = {"bound": "instruction mix (measured block step)", "ns_per_block_and_simd": ns, "row_blocks_per_wave": rb,
               "floor_us": blocks_per_simd * ns * 1e-3, "frac": blocks_per_simd * ns * 1e-9 / kern_s,
               "note": "floor = 32x32 blocks of logits per SIMD x the block step measured by krul_calibration_block "
                       "(MFMA chain + LDS operand reads + vector work, no memory traffic) in this run"}
    # The roof that binds this workload: the one whose floor time (algorithmic work / peak) is longest.  The matrix
    # cores bind the many-query configurations (C4, C5), the HBM stream of keys the few-query ones (C2, C3, D*);
    # the vector units' floor is reported beside them (matrix and vector instructions share a wave's issue slots).
    main_roof = dict(mfma if w.dtype == "bf16" and flops_alg / 2500e12 > bytes_alg / 8000e9 else hbm)
    main_roof.update({"traffic": traffic, "traffic_source": traffic_src, "kernel": kernel_name,
                      "kernel_us": kern_s * 1e6, "kernel_us_samples": len(kern_ms),
                      "floor_us": {"hbm": bytes_alg / 8000e9 * 1e6, "mfma": flops_alg / 2500e12 * 1e6,
                                   "alu": valu_alg / (VALU_PEAK_TOPS * 1e12) * 1e6}})
    res = {
        "metric": "layer-pair similarity throughput", "value": value, "unit": "Gscore-elems/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} L={w.L} Hq/Hkv={w.Hq}/{w.Hkv} d={w.d} S={w.S} Tq={w.Tq} "
                               f"{w.dtype}, select {w.n_select} pairs", "score_elems": w.score_elems,
                   "outputs": "pair_score+head_score" + ("+pair_dist" if args.with_dist else "") + "+pairs",
                   "calls": "krul_pair_similarity + krul_select_pairs" if args.two_calls else "krul_pair_similarity_select",
                   "input_buffer_sets": len(sets), "plan": kr.plan(shp)},
        "roofline": main_roof,
        "roofline_hbm": hbm, "roofline_mfma": mfma, "roofline_alu": alu, "roofline_instruction_mix": mix,
        "selected_pairs": pairs.cpu().tolist()[0],
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, q, k)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
