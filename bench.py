#!/usr/bin/env python3
"""Benchmark of the GlowQ group forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path (projection R = X B^T once per unit,
then Y_i = X dequant(W_q,i)^T + R A_i^T for every module, restore mask applied)
over one batch of seeded synthetic input that is already resident in HBM.  The
read-only operands are rotated over several distinct copies so that consecutive
steps do not find their weights in the 256 MB Infinity Cache.  The default
workload is the Llama-2-7B-shaped QKV group at one token (decode); others are
selectable with --workload.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16 / bf16 matrix throughput

# name -> (config id, T, bound)
WORKLOADS = {
    "cfg2_T1": (2, 1, "hbm"),
    "cfg2_T2": (2, 2, "hbm"),
    "cfg2_T4": (2, 4, "hbm"),
    "cfg2_T8": (2, 8, "hbm"),
    "cfg2_T16": (2, 16, "hbm"),
    "cfg3": (3, 2048, "mfma"),
    "cfg4": (4, 512, "mfma"),
    "cfg5_T1": (5, 1, "hbm"),
    "cfg5_T1024": (5, 1024, "mfma"),
    "cfg1": (1, 16, "hbm"),
    # calibration of the HBM traffic counters: a plain device copy of 256 MiB
    "copy256": (0, 0, "copy"),
}


def unit_cost(shape, T, r, G, restored):
    """Algorithmic bytes and flops of one unit: packed nibbles, (s, z) pairs, A and B
    only if restored, X, and Y in 16 bit; R stays on chip and is not counted."""
    rows, K = shape.rows, shape.d_in
    by = rows * K // 2 + rows * (K // G) * 4 + T * K * 2 + T * rows * 2
    fl = 2 * T * K * rows
    if restored and r > 0:
        by += rows * r * 2 + r * K * 2
        fl += 2 * T * r * K + 2 * T * r * rows
    return by, fl


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg2_T1", choices=sorted(WORKLOADS))
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="graph: the K timed steps are captured once into a HIP graph")
    ap.add_argument("--rot", type=int, default=None, help="distinct operand copies to rotate over")
    ap.add_argument("--layers", type=int, default=None, help="cfg5 only: layers to instantiate")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--restore", default="workload", choices=["workload", "none", "all"],
                    help="restore mask: the workload's own (default), no unit, or every unit "
                         "(to price the correction; the JSON line says how many units were restored)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collective is part of the path: units are independent and would be sharded "
              "whole, one process per GPU)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2603_25385_amd as G
    from glowq_inputs import CONFIGS, config_units, gen_direct_unit, gen_restore_mask

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    cfg_id, T, bound = WORKLOADS[args.workload]
    if bound == "copy":
        return copy_calibration(torch, args)
    cfg = CONFIGS[cfg_id]
    r, Gs, act = cfg["r"], cfg["G"], cfg["act"]
    shapes = config_units(cfg_id)
    if cfg_id == 5 and args.layers:
        shapes = shapes[:4 * args.layers]
    n_units = len(shapes)
    if "restore_fraction" in cfg:
        mask = gen_restore_mask(cfg["mask_seed"], len(config_units(cfg_id)),
                                cfg["restore_fraction"])[:n_units]
    else:
        mask = np.ones(n_units, np.uint8)
    if args.restore != "workload":
        mask = np.full(n_units, 1 if args.restore == "all" else 0, np.uint8)
    decode = bound == "hbm"
    steps = args.steps if args.steps is not None else (200 if decode else 20)
    warmup = args.warmup if args.warmup is not None else (20 if decode else 3)

    costs = [unit_cost(s, T, r, Gs, bool(f)) for s, f in zip(shapes, mask)]
    alg_bytes = sum(c[0] for c in costs)
    alg_flops = sum(c[1] for c in costs)
    ro_bytes = alg_bytes - sum(T * s.rows * 2 for s in shapes)       # read-only operands
    n_rot = args.rot if args.rot is not None else max(1, min(24, int(np.ceil(600e6 / ro_bytes))))

    act_code = {"f16": G.GLOWQ_F16, "bf16": G.GLOWQ_BF16}[act]
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[act]
    st = torch.cuda.current_stream().cuda_stream
    keep = []               # device buffers stay alive here
    host_unit0 = None       # host copy of unit 0 for the CPU baseline

    def build_rotation(rot):
        nonlocal host_unit0
        descs = []
        for ui, shape in enumerate(shapes):
            src = gen_direct_unit(cfg["seed"], ui, shape, T, r, Gs, act, device=dev)
            if rot == 0 and ui == 0 and not args.no_cpu_baseline:
                host_unit0 = dict(
                    X=src["X"].view(torch.int16).cpu().numpy().view(np.uint16),
                    B=src["B"].view(torch.int16).cpu().numpy().view(np.uint16),
                    act=act, G=Gs, r=r, d_in=shape.d_in, T=T,
                    modules=[dict(wq=m["wq"].cpu().numpy().view(np.uint32),
                                  scales=m["scales"].view(torch.int16).cpu().numpy().view(np.uint16),
                                  zeros=m["zeros"].view(torch.int16).cpu().numpy().view(np.uint16),
                                  A=m["A"].view(torch.int16).cpu().numpy().view(np.uint16))
                             for m in src["modules"]])
            mods = []
            for m in src["modules"]:
                nb = G.glowq_prepared_bytes(m["d_out"], shape.d_in, Gs)
                prep = torch.empty(nb, dtype=torch.uint8, device=dev)
                G.glowq_prepare_weights(m["wq"].data_ptr(), m["scales"].data_ptr(),
                                        m["zeros"].data_ptr(), m["d_out"], shape.d_in, Gs,
                                        prep.data_ptr(), st)
                Y = torch.empty((T, m["d_out"]), dtype=tdt, device=dev)
                keep.extend([prep, m["A"], Y])
                mods.append(G.make_module(prep.data_ptr(), m["A"].data_ptr(), Y.data_ptr(),
                                          m["d_out"], m["d_out"]))
            keep.extend([src["X"], src["B"]])
            descs.append(G.make_unit(src["X"].data_ptr(), src["B"].data_ptr(), mods, T,
                                     shape.d_in, r, Gs, act_code, act_code))
            torch.cuda.synchronize()      # canonical arrays of this unit can go now
        return descs

    rotations = []
    for rot in range(n_rot):
        descs = build_rotation(rot)
        keep.append(descs)
        rotations.append(G.pack_units(descs))
    cmask = G.pack_mask(mask.tolist())
    ws_bytes = G.glowq_workspace_bytes(rotations[0])
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    G.glowq_workspace_init(ws.data_ptr(), ws.numel(), st)
    torch.cuda.synchronize()

    def step(i):
        G.glowq_block_forward(rotations[i % n_rot], cmask, ws.data_ptr(), ws_bytes,
                              torch.cuda.current_stream().cuda_stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.mode == "graph":
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(steps):
                    step(i)
            graph.replay()               # one untimed replay
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev0.record(side)
            graph.replay()
            ev1.record(side)
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for i in range(steps):
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(ev_ms, 0.0) / steps
    wall_ms_per_step = wall * 1e3 / steps

    gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9
    tfs = alg_flops / (ms_per_step * 1e-3) / 1e12
    if decode:
        value, unit = gbs, "GB/s"
        roof = dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=gbs / HBM_PEAK_GBS)
    else:
        value, unit = tfs, "TFLOP/s"
        roof = dict(bound="mfma", achieved=tfs, peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=tfs / MFMA_PEAK_TFLOPS)
    roof["traffic"] = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            roof["traffic"] = json.load(f).get("hbm_bytes_per_step")
    roof["kernels_per_step"] = "see profiles/"

    out = {
        "metric": "grouped W4+low-rank forward: decode HBM GB/s & us/group; prefill TFLOP/s",
        "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": act, "data": "synthetic",
        "config": {"workload": f"{cfg['name']} T={T} r={r} G={Gs} ({args.workload})",
                   "units": n_units, "restored_units": int(mask.sum()), "rotating_copies": n_rot,
                   "launch": args.mode},
        "us_per_step": ms_per_step * 1e3,
        "wall_ms_per_step": wall_ms_per_step,
        "algorithmic_bytes": alg_bytes, "algorithmic_flops": alg_flops,
        "achieved_GBps": gbs, "achieved_TFLOPs": tfs,
        "roofline": roof,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host_unit0, shapes[0], T, r, Gs, decode)
    print(json.dumps(out))
    return 0


def copy_calibration(torch, args):
    """Plain device-to-device copy of 256 MiB (reads 256 MiB, writes 256 MiB per step):
    the known quantity against which the FETCH_SIZE / WRITE_SIZE counters are scaled."""
    n = 256 << 20
    steps = args.steps or 20
    srcs = [torch.empty(n, dtype=torch.uint8, device="cuda").fill_(i) for i in range(3)]
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    for i in range(3):
        dst.copy_(srcs[i])
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for i in range(steps):
        dst.copy_(srcs[i % 3])
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    print(json.dumps({"metric": "device copy (counter calibration)", "value": 2 * n / ms / 1e6,
                      "unit": "GB/s", "bytes_read_per_step": n, "bytes_written_per_step": n,
                      "steps": steps, "ms_per_step": ms}))
    return 0


def cpu_baseline(unit, shape, T, r, Gs, decode):
    """The oracle (naive C loops, float64) timed on this machine's host cores on a
    bounded sample of the same workload: unit 0, all tokens, a fixed number of
    output rows per module."""
    import numpy as np

    from oracle import naive

    rows_per_module = None if decode else max(8, int(2.0e10 // (2 * T * shape.d_in * len(shape.d_outs))))
    rows = None
    sampled = shape.rows
    if rows_per_module is not None:
        rng = np.random.default_rng(7)
        rows = [np.sort(rng.choice(o, size=min(o, rows_per_module), replace=False)).astype(np.int32)
                for o in shape.d_outs]
        sampled = int(sum(len(x) for x in rows))
    naive.load()
    naive.group_forward(unit, True, rows=rows)          # first touch of the operands
    # repeat the same sample until about ten seconds of CPU work have been timed
    reps, total = 0, 0.0
    while total < 10.0 and reps < 400:
        t0 = time.perf_counter()
        naive.group_forward(unit, True, rows=rows)
        total += time.perf_counter() - t0
        reps += 1
    dt = total / reps
    K = shape.d_in
    by = sampled * K // 2 + sampled * (K // Gs) * 4 + sampled * r * 2 + r * K * 2 + T * K * 2 \
        + T * sampled * 2
    fl = 2 * T * K * sampled + 2 * T * r * K + 2 * T * r * sampled
    if decode:
        val, unit_s = by / dt / 1e9, "GB/s"
    else:
        val, unit_s = fl / dt / 1e12, "TFLOP/s"
    return {"value": val, "unit": unit_s, "cores": naive.max_threads(), "kind": "oracle",
            "seconds": total,
            "sample": f"unit 0 ({shape.name}), {T} token(s), {sampled} of {shape.rows} output rows, "
                      f"{reps} repetitions, naive C loops in float64 with OpenMP"}


if __name__ == "__main__":
    sys.exit(main())
