#!/usr/bin/env python3
"""Benchmark of the GlowQ group forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path (projection R = X B^T once per unit,
then Y_i = X dequant(W_q,i)^T + R A_i^T for every module, restore mask applied)
over one batch of seeded synthetic input that is already resident in HBM.  The
read-only operands are rotated over several distinct copies so that consecutive
steps do not find their weights in the 256 MB Infinity Cache.

Without --workload the run times BOTH halves of the metric in one process: the
Llama-2-7B-shaped QKV group at one token (decode, HBM GB/s: the headline `value`)
and the Llama-2-7B-shaped gate/up group at 2048 tokens (prefill, TFLOP/s: the
`prefill` object of the same JSON line).  Every workload is timed as R replays of
K steps (median and minimum reported), once more on a single operand set that stays
cache resident (labelled `hot`), and is then checked: no unit may have dropped its
correction (status words) and unit 0's output must match the CPU oracle.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import platform
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16 / bf16 matrix throughput
REPLAYS = 5
TOL = 2e-3                     # max relative error of the outputs (fp32 accumulation)
ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8}

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
    # measured ceilings (no part of the method): one launch that only reads 24 MiB with
    # 128-bit loads, and a register-resident loop of 16x16x32 matrix instructions
    "stream24": (0, 0, "stream"),
    "mfma_f16": (0, 0, "mfma_probe"),
    "mfma_bf16": (0, 0, "mfma_probe"),
    "mfma_fp8fp4": (0, 0, "mfma_probe"),
    "mfma_fp4fp4": (0, 0, "mfma_probe"),
    "mfma_fp8fp4_32": (0, 0, "mfma_probe"),
    # offline side of GlowQ-S: the importance scores of the Llama-2-7B-shaped QKV unit
    "cfg2_scores": (2, 0, "scores"),
    # offline factorisation (Alg. 1) of a q/k/v group with d = 3072, r = 64, p = 16, q = 2:
    # the setting of the paper's timing table of the randomised SVD
    "factorize_d3072": (0, 0, "factorize"),
    # microscaling variant (MXFP4 weights, MXFP8 activations) on the shapes of workload 2
    "cfg2_T1_mx": (2, 1, "mx"),
    "cfg2_T16_mx": (2, 16, "mx"),
    "cfg3_mx": (3, 2048, "mx"),
}
METRIC = "grouped W4+low-rank forward: decode HBM GB/s & us/group; prefill TFLOP/s"


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


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return platform.processor() or "unknown"


def rel_err(y, y_ref):
    """max |y - y_ref| / max(|y_ref|, rms(y_ref))"""
    import numpy as np
    y, y_ref = np.asarray(y, np.float64), np.asarray(y_ref, np.float64)
    rms = float(np.sqrt(np.mean(y_ref ** 2))) or 1.0
    return float(np.max(np.abs(y - y_ref) / np.maximum(np.abs(y_ref), rms)))


def time_steps(torch, step, steps, mode, replays):
    """Event-timed milliseconds per step of `replays` runs of `steps` steps each."""
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out, wall = [], []
    if mode == "graph":
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(steps):
                    step(i)
            graph.replay()               # one untimed replay
            torch.cuda.synchronize()
            for _ in range(replays):
                t0 = time.perf_counter()
                ev0.record(side)
                graph.replay()
                ev1.record(side)
                torch.cuda.synchronize()
                wall.append((time.perf_counter() - t0) * 1e3 / steps)
                out.append(ev0.elapsed_time(ev1) / steps)
    else:
        for _ in range(replays):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev0.record()
            for i in range(steps):
                step(i)
            ev1.record()
            torch.cuda.synchronize()
            wall.append((time.perf_counter() - t0) * 1e3 / steps)
            out.append(ev0.elapsed_time(ev1) / steps)
    return out, wall


def run_workload(name, args, torch, want_cpu_baseline):
    import numpy as np

    import paper_2603_25385_amd as G
    from glowq_inputs import (CONFIGS, config_units, gen_direct_layerwise_B, gen_direct_unit,
                              gen_restore_mask)

    dev = "cuda"
    cfg_id, T, bound = WORKLOADS[name]
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
    if args.unit is not None:          # one unit of the block by itself
        shapes, mask, n_units = [shapes[args.unit]], mask[args.unit:args.unit + 1], 1
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
    host_unit0 = None       # host copy of unit 0, rotation 0, for the oracle
    y_unit0 = None          # its output buffers
    compare = args.compare and r > 0
    lw_B = []               # per rotation: device addresses of the per-module right factors

    def build_rotation(rot):
        nonlocal host_unit0, y_unit0
        descs, b_ptrs = [], []
        b16 = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
        for ui, shape in enumerate(shapes):
            src = gen_direct_unit(cfg["seed"], ui, shape, T, r, Gs, act, device=dev)
            if compare:
                own = gen_direct_layerwise_B(cfg["seed"] + 1000 * rot, ui, shape, r, act, device=dev)
                keep.extend(own)
                b_ptrs.extend(b.data_ptr() for b in own)
            if rot == 0 and ui == 0:
                host_unit0 = dict(
                    X=b16(src["X"]), B=b16(src["B"]), act=act, G=Gs, r=r, d_in=shape.d_in, T=T,
                    modules=[dict(wq=m["wq"].cpu().numpy().view(np.uint32), scales=b16(m["scales"]),
                                  zeros=b16(m["zeros"]), A=b16(m["A"])) for m in src["modules"]])
                if compare:
                    for m, b in zip(host_unit0["modules"], own):
                        m["B"] = b16(b)
            mods, ys = [], []
            for m in src["modules"]:
                nb = G.glowq_prepared_bytes(m["d_out"], shape.d_in, Gs)
                prep = torch.empty(nb, dtype=torch.uint8, device=dev)
                G.glowq_prepare_weights(m["wq"].data_ptr(), m["scales"].data_ptr(),
                                        m["zeros"].data_ptr(), m["d_out"], shape.d_in, Gs,
                                        prep.data_ptr(), st)
                Y = torch.empty((T, m["d_out"]), dtype=tdt, device=dev)
                keep.extend([prep, m["A"], Y])
                ys.append(Y)
                mods.append(G.make_module(prep.data_ptr(), m["A"].data_ptr(), Y.data_ptr(),
                                          m["d_out"], m["d_out"]))
            if rot == 0 and ui == 0:
                y_unit0 = ys
            keep.extend([src["X"], src["B"]])
            descs.append(G.make_unit(src["X"].data_ptr(), src["B"].data_ptr(), mods, T,
                                     shape.d_in, r, Gs, act_code, act_code))
            torch.cuda.synchronize()      # canonical arrays of this unit can go now
        if compare:
            lw_B.append(G.pack_pointers(b_ptrs))
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

    def step_hot(i):
        G.glowq_block_forward(rotations[0], cmask, ws.data_ptr(), ws_bytes,
                              torch.cuda.current_stream().cuda_stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ms, wall = time_steps(torch, step, steps, args.mode, REPLAYS)
    ms_hot, _ = time_steps(torch, step_hot, steps, args.mode, 2)
    ms_per_step = float(np.median(ms))

    # after the timed region: no unit dropped its correction, and unit 0 matches the oracle
    failed = torch.zeros(1, dtype=torch.int32, device=dev)
    G.glowq_workspace_status(rotations[0], ws.data_ptr(), ws_bytes, failed.data_ptr(), st)
    for ys in [y_unit0]:
        for y in ys:
            y.fill_(float("nan"))
    step_hot(0)
    torch.cuda.synchronize()
    n_failed = int(failed.item())
    parity = check_against_oracle(host_unit0, y_unit0, shapes[0], T, bool(mask[0]), decode, act)

    comparison = None
    if compare:
        comparison = run_comparison(torch, G, np, args, steps, rotations, lw_B, n_rot, n_units, cfg,
                                    ws, ws_bytes, host_unit0, y_unit0, shapes[0], T, decode, act)

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
    tpath = os.path.join(ROOT, "profiles", f"traffic_{name}.json")
    if os.path.exists(tpath) and args.unit is None and args.restore == "workload":
        with open(tpath) as f:
            roof["traffic"] = json.load(f).get("hbm_bytes_per_step")
    roof["traffic_source"] = f"profiles/{name}.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)"

    out = {
        "metric": METRIC, "value": value, "unit": unit, "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": act, "data": "synthetic",
        "config": {"workload": f"{cfg['name']} T={T} r={r} G={Gs} ({name})" +
                               (f", unit {args.unit} alone" if args.unit is not None else ""),
                   "units": n_units, "restored_units": int(mask.sum()), "rotating_copies": n_rot,
                   "launch": args.mode},
        "us_per_step": ms_per_step * 1e3,
        "timing": {"replays": REPLAYS, "us_per_step_median": ms_per_step * 1e3,
                   "us_per_step_min": min(ms) * 1e3, "us_per_step_max": max(ms) * 1e3,
                   "wall_us_per_step_median": float(np.median(wall)) * 1e3,
                   "hot_us_per_step": min(ms_hot) * 1e3,
                   "hot_note": "one operand set replayed: weights stay in the Infinity Cache; "
                               "not the figure of merit"},
        "algorithmic_bytes": alg_bytes, "algorithmic_flops": alg_flops,
        "achieved_GBps": gbs, "achieved_TFLOPs": tfs,
        "roofline": roof,
        "checks": {"units_that_dropped_their_correction": n_failed, "parity": parity},
    }
    if comparison is not None:
        out["comparison"] = comparison
        if not args.no_checks and not comparison["layerwise_parity"]["ok"]:
            raise SystemExit("bench.py: layer-wise output of unit 0 does not match the oracle: "
                             f"{comparison['layerwise_parity']}")
    if args.no_checks:
        pass
    elif n_failed:
        raise SystemExit(f"bench.py: {n_failed} unit(s) reported an expired in-kernel wait "
                         "(correction left out); the timing is void")
    if not args.no_checks and not parity["ok"]:
        raise SystemExit(f"bench.py: output of unit 0 does not match the oracle: {parity}")
    if want_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host_unit0, shapes[0], T, r, Gs, decode)
    return out


# Table 3 of the paper, average change against its Layerwise rows (LLaMA-2 7B and 13B, whole
# model, end to end on the authors' GPU): context for `comparison`, not a target
PAPER_TABLE3 = {"decode_ms_per_token_pct": {"GlowQ": -6.61, "GlowQ-S": -27.01},
                "prefill_ms_pct": {"GlowQ": -3.37, "GlowQ-S": -22.44}}


def run_comparison(torch, G, np, args, steps, rotations, lw_B, n_rot, n_units, cfg, ws, ws_bytes,
                   host_unit0, y_unit0, shape0, T, decode, act):
    """The same operands three ways (Sec. 4.3): layer-wise (a projection and a right factor
    per module), GlowQ (one per unit, every unit restored) and GlowQ-S (half of the units
    restored; a single-unit workload: its one unit not restored)."""
    from glowq_inputs import gen_restore_mask

    dev = "cuda"
    cur = lambda: torch.cuda.current_stream().cuda_stream
    lw_bytes = G.glowq_layerwise_workspace_bytes(rotations[0])
    lw_ws = torch.empty(lw_bytes, dtype=torch.uint8, device=dev)
    G.glowq_workspace_init(lw_ws.data_ptr(), lw_bytes, cur())
    if n_units > 1:
        half = gen_restore_mask(cfg.get("mask_seed", cfg["seed"]), n_units, 0.5)
    else:
        half = np.zeros(1, np.uint8)
    m_all, m_half = G.pack_mask([1] * n_units), G.pack_mask(half.tolist())

    def step_lw(i):
        G.glowq_layerwise_forward(rotations[i % n_rot], lw_B[i % n_rot], lw_ws.data_ptr(), lw_bytes, cur())

    def step_all(i):
        G.glowq_block_forward(rotations[i % n_rot], m_all, ws.data_ptr(), ws_bytes, cur())

    def step_half(i):
        G.glowq_block_forward(rotations[i % n_rot], m_half, ws.data_ptr(), ws_bytes, cur())

    res = {}
    for key, fn in (("layerwise", step_lw), ("glowq", step_all), ("glowq_s", step_half)):
        fn(0)
        torch.cuda.synchronize()
        ms, _ = time_steps(torch, fn, steps, args.mode, REPLAYS)
        res[key] = float(np.median(ms)) * 1e3
    # the layer-wise outputs of unit 0 against the oracle, module by module (each module is a
    # one-module unit with its own B)
    for y in y_unit0:
        y.fill_(float("nan"))
    G.glowq_layerwise_forward(rotations[0], lw_B[0], lw_ws.data_ptr(), lw_bytes, cur())
    torch.cuda.synchronize()
    worst, tol = 0.0, TOL + ULP[act]
    rows, sampled = sample_rows(shape0, T, decode)
    from oracle import naive
    naive.load()
    for i, (m, y) in enumerate(zip(host_unit0["modules"], y_unit0)):
        solo = dict(host_unit0, B=m["B"], modules=[m])
        (ref,) = naive.group_forward(solo, True, rows=None if rows is None else [rows[i]])
        got = y.double().cpu().numpy()
        if rows is not None:
            got = got[:, rows[i]]
        worst = max(worst, rel_err(got, ref) if np.isfinite(got).all() else float("inf"))
    pct = lambda a, b: 100.0 * (a - b) / b
    return {
        "us_per_step": res,
        "restored_units": {"layerwise": n_units, "glowq": n_units, "glowq_s": int(half.sum())},
        "glowq_vs_layerwise_pct": pct(res["glowq"], res["layerwise"]),
        "glowq_s_vs_layerwise_pct": pct(res["glowq_s"], res["layerwise"]),
        "layerwise_parity": {"max_rel_err": worst, "tolerance": tol, "ok": bool(worst <= tol),
                             "checked": f"unit 0 ({shape0.name}), {sampled} of {shape0.rows} output rows"},
        "paper_table3_avg_pct": PAPER_TABLE3,
        "note": "time of the linear layers of the workload only; the paper's table is whole-model "
                "latency on other hardware",
    }


def sample_rows(shape, T, decode):
    """Output rows the oracle computes: all of them for decode, a bounded seeded sample
    per module for prefill."""
    import numpy as np
    if decode:
        return None, shape.rows
    per = max(8, int(2.0e10 // (2 * T * shape.d_in * len(shape.d_outs))))
    rng = np.random.default_rng(7)
    rows = [np.sort(rng.choice(o, size=min(o, per), replace=False)).astype(np.int32)
            for o in shape.d_outs]
    return rows, int(sum(len(x) for x in rows))


def check_against_oracle(unit, ys, shape, T, restored, decode, act):
    """Unit 0 of rotation 0, computed once more after the timed loop, against the naive
    float64 oracle (all rows for decode, the sampled rows for prefill)."""
    import numpy as np

    from oracle import naive

    naive.load()
    rows, sampled = sample_rows(shape, T, decode)
    refs = naive.group_forward(unit, restored, rows=rows)
    worst = 0.0
    for i, (y, ref) in enumerate(zip(ys, refs)):
        got = y.double().cpu().numpy()
        if rows is not None:
            got = got[:, rows[i]]
        worst = max(worst, rel_err(got, ref) if np.isfinite(got).all() else float("inf"))
    tol = TOL + ULP[act]
    return {"max_rel_err": worst, "tolerance": tol, "ok": bool(worst <= tol),
            "checked": f"unit 0 ({shape.name}), {sampled} of {shape.rows} output rows, all tokens"}


def cpu_baseline(unit, shape, T, r, Gs, decode):
    """The oracle (naive C loops, float64) timed on this machine's host cores on a
    bounded sample of the same workload: unit 0, all tokens, a fixed number of
    output rows per module."""
    from oracle import naive

    rows, sampled = sample_rows(shape, T, decode)
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
            "cpu_model": cpu_model(), "seconds": total,
            "sample": f"unit 0 ({shape.name}), {T} token(s), {sampled} of {shape.rows} output rows, "
                      f"{reps} repetitions, naive C loops in float64 with OpenMP"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS),
                    help="one workload only (default: cfg2_T1 as the headline plus cfg3 as `prefill`)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="graph: the K timed steps are captured once into a HIP graph")
    ap.add_argument("--rot", type=int, default=None, help="distinct operand copies to rotate over")
    ap.add_argument("--layers", type=int, default=None, help="cfg5 only: layers to instantiate")
    ap.add_argument("--unit", type=int, default=None,
                    help="time one unit of the workload's block by itself (0 q/k/v, 1 o, 2 gate/up, "
                         "3 down), e.g. --workload cfg4 --unit 3: a long contraction on few tiles")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-checks", action="store_true",
                    help="report the status / parity checks but do not fail on them (tuning runs "
                         "of deliberately incomplete kernels only)")
    ap.add_argument("--compare", action=argparse.BooleanOptionalAction, default=None,
                    help="(default: on for the default run, off with --workload) also time the layer-wise mode (a right factor per module), GlowQ with "
                         "every unit restored and GlowQ-S with half of them, on the same operands")
    ap.add_argument("--restore", default="workload", choices=["workload", "none", "all"],
                    help="restore mask: the workload's own (default), no unit, or every unit "
                         "(to price the correction; the JSON line says how many units were restored)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collective is part of the path: units are independent and would be sharded "
              "whole, one process per GPU)", file=sys.stderr)
        return 2

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.compare is None:
        args.compare = args.workload is None
    if args.workload is not None:
        bound = WORKLOADS[args.workload][2]
        if bound == "copy":
            return copy_calibration(torch, args)
        if bound == "stream":
            return stream_ceiling(torch, args)
        if bound == "mfma_probe":
            kind = {"mfma_f16": 0, "mfma_bf16": 1, "mfma_fp8fp4": 2, "mfma_fp4fp4": 3, "mfma_fp8fp4_32": 4}[args.workload]
            return mfma_ceiling(torch, args, kind)
        if bound == "scores":
            return importance_scores(torch, args)
        if bound == "factorize":
            return factorize_unit(torch, args)
        if bound == "mx":
            return mx_workload(torch, args, args.workload)
        out = run_workload(args.workload, args, torch, not args.no_cpu_baseline)
        out["peaks"] = {"hbm_GBps": HBM_PEAK_GBS, "mfma_f16_bf16_TFLOPs": MFMA_PEAK_TFLOPS}
        print(json.dumps(out))
        return 0
    # default: both halves of the metric
    out = run_workload("cfg2_T1", args, torch, not args.no_cpu_baseline)
    pf = run_workload("cfg3", args, torch, False)
    out["prefill"] = {k: pf[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "dtype",
                                         "config", "timing", "algorithmic_bytes",
                                         "algorithmic_flops", "roofline", "checks", "comparison")
                      if k in pf}
    out["peaks"] = {"hbm_GBps": HBM_PEAK_GBS, "mfma_f16_bf16_TFLOPs": MFMA_PEAK_TFLOPS}
    print(json.dumps(out))
    return 0


def importance_scores(torch, args):
    """glowq_unit_importance (Sec. 3.3, Eqs. 10-11) on the QKV unit of workload 2: fp32
    weights, prepared weights and stored factors in, two float64 scores out; bound by the
    bytes of the fp32 weights.  Checked against the oracle on the first operand set."""
    import numpy as np

    import paper_2603_25385_amd as G
    from glowq_inputs import CONFIGS, config_units, gen_direct_unit
    from oracle import glowq_oracle as O

    cfg = CONFIGS[2]
    shape = config_units(2)[0]
    r, Gs, act = cfg["r"], cfg["G"], cfg["act"]
    steps = args.steps or 20
    st = torch.cuda.current_stream().cuda_stream
    act_code = {"f16": G.GLOWQ_F16, "bf16": G.GLOWQ_BF16}[act]
    sets, keep, host0 = [], [], None
    gen = torch.Generator(device="cuda")
    for rot in range(3):
        src = gen_direct_unit(cfg["seed"] + rot, 0, shape, 1, r, Gs, act, device="cuda")
        mods, Ws = [], []
        for i, m in enumerate(src["modules"]):
            nb = G.glowq_prepared_bytes(m["d_out"], shape.d_in, Gs)
            prep = torch.empty(nb, dtype=torch.uint8, device="cuda")
            G.glowq_prepare_weights(m["wq"].data_ptr(), m["scales"].data_ptr(), m["zeros"].data_ptr(),
                                    m["d_out"], shape.d_in, Gs, prep.data_ptr(), st)
            gen.manual_seed(1000 * rot + i)
            W = torch.randn(m["d_out"], shape.d_in, generator=gen, device="cuda") * 0.02
            keep.extend([prep, m["A"], W])
            Ws.append(W)
            mods.append(G.make_module(prep.data_ptr(), m["A"].data_ptr(), 0, m["d_out"], m["d_out"]))
        keep.append(src["B"])
        unit = G.make_unit(0, src["B"].data_ptr(), mods, 1, shape.d_in, r, Gs, act_code, act_code)
        sets.append((unit, G.pack_pointers([w.data_ptr() for w in Ws])))
        if rot == 0:
            b16 = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
            host0 = dict(W=[w.cpu().numpy() for w in Ws], B=b16(src["B"]),
                         modules=[dict(wq=m["wq"].cpu().numpy().view(np.uint32), scales=b16(m["scales"]),
                                       zeros=b16(m["zeros"]), A=b16(m["A"])) for m in src["modules"]])
        torch.cuda.synchronize()
    scratch = torch.empty(G.GLOWQ_IMPORTANCE_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    scores = torch.zeros(2, dtype=torch.float64, device="cuda")

    def step(i):
        u, w = sets[i % len(sets)]
        G.glowq_unit_importance(u, w, scratch.data_ptr(), scores.data_ptr(),
                                torch.cuda.current_stream().cuda_stream)

    for i in range(3):
        step(i)
    torch.cuda.synchronize()
    ms, _ = time_steps(torch, step, steps, args.mode, REPLAYS)
    med = float(np.median(ms))
    step(0)
    torch.cuda.synchronize()
    got = scores.cpu().numpy()
    What = [O.dequant(O.unpack_int4(m["wq"]), m["scales"], m["zeros"], Gs, act) for m in host0["modules"]]
    ner = O.importance_ner(host0["W"], What)
    energy = sum(float(np.sum((w.astype(np.float64) - wh) ** 2)) for w, wh in zip(host0["W"], What))
    ec = O.importance_ec_from_factors([m["A"] for m in host0["modules"]], host0["B"], act, energy)
    err = max(abs(got[0] - ner) / ner, abs(got[1] - ec) / ec)
    by = shape.rows * shape.d_in * 4 + shape.rows * shape.d_in // 2 + shape.rows * (shape.d_in // Gs) * 4 \
        + shape.rows * r * 2 + r * shape.d_in * 2
    gbs = by / (med * 1e-3) / 1e9
    out = {"metric": "importance scores of one unit (GlowQ-S, Eqs. 10-11): HBM GB/s", "value": gbs, "unit": "GB/s",
           "steps": steps, "ms_per_step": med, "us_per_step_min": min(ms) * 1e3, "dtype": "f64",
           "data": "synthetic", "config": {"workload": f"{cfg['name']} importance scores (cfg2_scores)",
                                           "launch": args.mode},
           "algorithmic_bytes": by,
           "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs / HBM_PEAK_GBS, "traffic": None},
           "checks": {"parity": {"max_rel_err": float(err), "tolerance": 1e-9, "ok": bool(err <= 1e-9),
                                 "scores": [float(got[0]), float(got[1])]}}}
    print(json.dumps(out))
    if not args.no_checks and err > 1e-9:
        raise SystemExit(f"bench.py: importance scores do not match the oracle: {out['checks']}")
    return 0


def mx_workload(torch, args, name):
    """glowq_mx_group_forward on the q/k/v unit of workload 2: MXFP4 weights (E2M1 codes, an
    E8M0 scale per 32 channels), activations quantised to MXFP8 inside the call, the 16-bit
    correction as in the W4A16 path.  Operands are random codes and scales of the recipe's
    magnitudes, rotated over enough copies to defeat the caches; the first copy's first
    module is checked against the oracle."""
    import numpy as np

    import paper_2603_25385_amd as G
    from glowq_inputs import CONFIGS, config_units
    from oracle import glowq_oracle as O
    from oracle import mx_oracle as MX

    cfg_id, T, _ = WORKLOADS[name]
    cfg = CONFIGS[cfg_id]
    shape = config_units(cfg_id)[0]
    r, act = cfg["r"], cfg["act"]
    d = shape.d_in
    decode = T <= 16
    steps = args.steps if args.steps is not None else (200 if decode else 20)
    warmup = args.warmup if args.warmup is not None else (20 if decode else 3)
    restored = args.restore != "none"
    by = shape.rows * d // 2 + shape.rows * (d // 32) + T * d * 2 + T * shape.rows * 2
    fl = 2 * T * d * shape.rows
    if restored:
        by += shape.rows * r * 2 + r * d * 2
        fl += 2 * T * r * d + 2 * T * r * shape.rows
    ro = by - T * shape.rows * 2
    n_rot = args.rot if args.rot is not None else max(1, min(24, int(np.ceil(600e6 / ro))))
    act_code = {"f16": G.GLOWQ_F16, "bf16": G.GLOWQ_BF16}[act]
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[act]
    st = torch.cuda.current_stream().cuda_stream
    gen = torch.Generator(device="cuda")
    keep, units, host0, y0 = [], [], None, None
    for rot in range(n_rot):
        gen.manual_seed(cfg["seed"] + 77 * rot)
        X = (torch.randn(T, d, generator=gen, device="cuda") * 1.0).to(tdt)
        B = (torch.randn(r, d, generator=gen, device="cuda") * 0.01).to(tdt)
        mods, ys = [], []
        for o in shape.d_outs:
            codes = torch.randint(-2 ** 31, 2 ** 31 - 1, (o, d // 8), generator=gen, device="cuda", dtype=torch.int64).to(torch.int32)
            scales = torch.randint(117, 123, (o, d // 32), generator=gen, device="cuda", dtype=torch.int64).to(torch.uint8)
            A = (torch.randn(o, r, generator=gen, device="cuda") * 0.01).to(tdt)
            prep = torch.empty(G.glowq_mx_prepared_bytes(o, d), dtype=torch.uint8, device="cuda")
            G.glowq_mx_prepare_weights(codes.data_ptr(), scales.data_ptr(), o, d, prep.data_ptr(), st)
            Y = torch.empty((T, o), dtype=tdt, device="cuda")
            keep += [prep, A, Y]
            ys.append(Y)
            mods.append(G.make_module(prep.data_ptr(), A.data_ptr(), Y.data_ptr(), o, o))
            if rot == 0 and host0 is None:
                b16 = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
                words = codes.cpu().numpy().view(np.uint32)
                host0 = dict(X=b16(X), B=b16(B), act=act, r=r, d_in=d, T=T,
                             modules=[dict(codes=O.unpack_int4(words), scales=scales.cpu().numpy(),
                                           A=b16(A), d_out=o)])
                y0 = Y
            torch.cuda.synchronize()
        keep += [X, B]
        units.append(G.make_unit(X.data_ptr(), B.data_ptr(), mods, T, d, r, 0, act_code, act_code))
    ws_bytes = G.glowq_mx_workspace_bytes(units[0])
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def step(i):
        G.glowq_mx_group_forward(units[i % n_rot], 1 if restored else 0, ws.data_ptr(), ws_bytes,
                                 torch.cuda.current_stream().cuda_stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ms, wall = time_steps(torch, step, steps, args.mode, REPLAYS)
    ms_hot, _ = time_steps(torch, lambda i: step(0), steps, args.mode, 2)
    med = float(np.median(ms))
    y0.fill_(float("nan"))
    step(0)
    torch.cuda.synchronize()
    ref = MX.mx_group_forward(host0, restored)[0]
    err = rel_err(y0.to(torch.float64).cpu().numpy(), ref)
    tol = TOL + ULP[act]
    gbs = by / (med * 1e-3) / 1e9
    tfs = fl / (med * 1e-3) / 1e12
    if decode:
        roof = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": gbs / HBM_PEAK_GBS, "traffic": None}
    else:
        roof = {"bound": "mfma", "achieved": tfs, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tfs / FP8_PEAK_TFLOPS, "traffic": None,
                "note": "fp8 x fp4 on the block-scaled instruction runs at the fp8 rate"}
    tpath = os.path.join(ROOT, "profiles", f"traffic_{name}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            roof["traffic"] = json.load(f).get("hbm_bytes_per_step")
    out = {"metric": METRIC + " (microscaling variant: MXFP4 weights, MXFP8 activations)",
           "value": gbs if decode else tfs,
           "unit": "GB/s" if decode else "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": med,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "mxfp4 x mxfp8 (fp32 accumulate)",
           "data": "synthetic",
           "config": {"workload": f"{cfg['name']} T={T} r={r} MXFP4/MXFP8 ({name})", "units": 1,
                      "restored_units": int(restored), "rotating_copies": n_rot, "launch": args.mode},
           "us_per_step": med * 1e3,
           "timing": {"replays": REPLAYS, "us_per_step_median": med * 1e3, "us_per_step_min": min(ms) * 1e3,
                      "us_per_step_max": max(ms) * 1e3, "wall_us_per_step_median": float(np.median(wall)) * 1e3,
                      "hot_us_per_step": min(ms_hot) * 1e3},
           "algorithmic_bytes": by, "algorithmic_flops": fl,
           "roofline": roof,
           "checks": {"parity": {"module": 0, "max_rel_err": err, "tolerance": tol, "ok": bool(err <= tol)}}}
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        MX.mx_group_forward(host0, restored)
        dt = time.perf_counter() - t0
        share = host0["modules"][0]["d_out"] / shape.rows
        cb = (by * share / dt / 1e9) if decode else (fl * share / dt / 1e12)
        out["cpu_baseline"] = {"value": cb, "unit": "GB/s" if decode else "TFLOP/s", "cores": os.cpu_count(), "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "module 0 of the unit (%d of %d rows), one pass, %.2f s" % (
                                   host0["modules"][0]["d_out"], shape.rows, dt)}
    print(json.dumps(out))
    if not args.no_checks and err > tol:
        raise SystemExit(f"bench.py: microscaling forward does not match the oracle: {out['checks']}")
    return 0


FP8_PEAK_TFLOPS = 5000.0       # MI355X dense fp8 matrix throughput
F64_PEAK_TFLOPS = 78.6         # MI355X float64, matrix or vector
# the paper's table of factorisation time (another machine; per-layer means, seconds)
PAPER_SVD_TIME = {"exact_svd_s_per_layer": 0.76, "randomized_svd_s_per_layer": 0.09}


def factorize_unit(torch, args):
    """One step = the whole offline chain of one unit on the GPU: quantise three modules
    (glowq_quantize_rtn), prepare them, factorise the stacked error (glowq_factorize_unit,
    Alg. 1 with r = 64, p = 16, q = 2).  Shapes: the q/k/v group at d = 3072.  The first
    operand set is checked against the oracle (codes bit-exact; singular values; stored
    factors after sign alignment)."""
    import numpy as np

    import paper_2603_25385_amd as G
    from glowq_inputs import UnitShape
    from oracle import glowq_oracle as O

    shape = UnitShape("qkv", 3072, (3072, 1024, 1024))
    d, m = shape.d_in, shape.rows
    r, p, q, Gs, act = 64, 16, 2, 128, "f16"
    l = r + p
    steps = args.steps or 5
    warmup = 2 if args.warmup is None else args.warmup
    gen = torch.Generator(device="cuda")
    sets = []
    for rot in range(2):
        Ws, bufs = [], []
        for i, o in enumerate(shape.d_outs):
            gen.manual_seed(4000 + 10 * rot + i)
            W = torch.randn(o, d, generator=gen, device="cuda") * 0.02
            Ws.append(W)
            bufs.append(dict(wq=torch.empty((o, d // 8), dtype=torch.int32, device="cuda"),
                             sc=torch.empty((o, d // Gs), dtype=torch.int16, device="cuda"),
                             zp=torch.empty((o, d // Gs), dtype=torch.int16, device="cuda"),
                             prep=torch.empty(G.glowq_prepared_bytes(o, d, Gs), dtype=torch.uint8, device="cuda"),
                             A=torch.empty((o, r), dtype=torch.int16, device="cuda")))
        gen.manual_seed(4900 + rot)
        Omega = torch.randn(d, l, generator=gen, device="cuda", dtype=torch.float64)
        B = torch.empty((r, d), dtype=torch.int16, device="cuda")
        sig = torch.empty(l, dtype=torch.float64, device="cuda")
        mods = [G.make_module(b["prep"].data_ptr(), 0, 0, o, o) for b, o in zip(bufs, shape.d_outs)]
        unit = G.make_unit(0, 0, mods, 1, d, 0, Gs, G.GLOWQ_F16, G.GLOWQ_F16)
        sets.append(dict(W=Ws, bufs=bufs, Omega=Omega, B=B, sig=sig, unit=unit,
                         Wp=G.pack_pointers([w.data_ptr() for w in Ws]),
                         Ap=G.pack_pointers([b["A"].data_ptr() for b in bufs])))
    nbytes = G.glowq_factorize_workspace_bytes(sets[0]["unit"], r, p)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def quantise(s, st):
        for W, b, o in zip(s["W"], s["bufs"], shape.d_outs):
            G.glowq_quantize_rtn(W.data_ptr(), o, d, Gs, b["wq"].data_ptr(), b["sc"].data_ptr(), b["zp"].data_ptr(), st)
            G.glowq_prepare_weights(b["wq"].data_ptr(), b["sc"].data_ptr(), b["zp"].data_ptr(), o, d, Gs,
                                    b["prep"].data_ptr(), st)

    def factorise(s, st):
        G.glowq_factorize_unit(s["unit"], s["Wp"], 0, r, p, q, s["Omega"].data_ptr(), ws.data_ptr(), nbytes,
                               s["Ap"], s["B"].data_ptr(), s["sig"].data_ptr(), st)

    def step(i):
        st = torch.cuda.current_stream().cuda_stream
        quantise(sets[i % 2], st)
        factorise(sets[i % 2], st)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ms, _ = time_steps(torch, step, steps, args.mode, REPLAYS)
    med = float(np.median(ms))
    # the quantiser alone, for the split of the step
    msq, _ = time_steps(torch, lambda i: quantise(sets[i % 2], torch.cuda.current_stream().cuda_stream),
                        steps, args.mode, 3)
    # ---- check of operand set 0 against the oracle
    step(0)
    torch.cuda.synchronize()
    s0 = sets[0]
    b16 = lambda t: t.cpu().numpy().view(np.uint16)
    W_host = [w.cpu().numpy() for w in s0["W"]]
    t0 = time.perf_counter()
    quant = [O.quantize_rtn(w, Gs) for w in W_host]
    codes_ok = all(np.array_equal(b["wq"].cpu().numpy().view(np.uint32), O.pack_int4(qv)) and
                   np.array_equal(b16(b["sc"]), sb) and np.array_equal(b16(b["zp"]), zb)
                   for b, (qv, sb, zb) in zip(s0["bufs"], quant))
    What = [O.dequant(qv, sb, zb, Gs, act) for qv, sb, zb in quant]
    E = O.stack_errors(W_host, What)
    t_quant = time.perf_counter() - t0
    Om = s0["Omega"].cpu().numpy()
    t0 = time.perf_counter()
    A_ref, B_ref = O.factors_alg1(E, r, p, q, Om, None, qr="householder")
    t_alg1 = time.perf_counter() - t0
    sig = s0["sig"].cpu().numpy()
    sig_err = float(np.max(np.abs(sig[:r] - np.sum(A_ref ** 2, axis=0)) / sig[:r]))
    B_gpu = O.bits_to_f64(b16(s0["B"]), act)
    sign = np.sign(np.sum(B_gpu * B_ref, axis=1))
    A_gpu_bits = np.concatenate([b16(b["A"]) for b in s0["bufs"]], axis=0)
    diff = max(float(np.mean(A_gpu_bits != O.f64_to_bits(A_ref * sign[None, :], act))),
               float(np.mean(b16(s0["B"]) != O.f64_to_bits(B_ref * sign[:, None], act))))
    ok = bool(codes_ok and sig_err <= 1e-9 and diff <= 1e-3)
    cpu = None
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        O.factors_svd(E, r)
        t_exact = time.perf_counter() - t0
        cpu = {"value": 1.0 / (t_quant + t_alg1), "unit": "units/s", "cores": os.cpu_count(), "kind": "oracle",
               "cpu_model": cpu_model(),
               "sample": "one unit: quantise + dequantise + stack (%.2f s), Alg. 1 with a Householder QR "
                         "reduction (%.2f s); for the paper's comparison, the exact SVD of the same "
                         "stack takes %.2f s" % (t_quant, t_alg1, t_exact),
               "alg1_s": t_alg1, "exact_svd_s": t_exact}
    fl = 2.0 * m * d * l * (2 * q + 2) + 2.0 * m * l * r
    tfl = fl / (med * 1e-3) / 1e12
    out = {"metric": "offline factorisation of one unit (quantise, prepare, Alg. 1): units/s", "value": 1e3 / med,
           "unit": "units/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": med,
           "ms_per_step_min": min(ms), "higher_is_better": True, "vs_baseline": None, "dtype": "f64",
           "data": "synthetic",
           "config": {"workload": "q/k/v group, d = 3072, rows 3072 + 1024 + 1024, G = 128, f16; r = 64, p = 16, "
                                  "q = 2 (factorize_d3072)", "launch": args.mode},
           "split_ms": {"quantise_and_prepare": float(np.median(msq)), "factorise": med - float(np.median(msq))},
           "algorithmic_flops": fl,
           "roofline": {"bound": "mfma", "achieved": tfl, "peak": F64_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": tfl / F64_PEAK_TFLOPS, "traffic": None,
                        "note": "flops of the float64 products only, over the time of the whole step"},
           "paper_other_machine": PAPER_SVD_TIME,
           "checks": {"parity": {"codes_bit_exact": bool(codes_ok), "sigma_max_rel_err": sig_err,
                                 "factor_bits_differing": diff, "ok": ok}}}
    if cpu:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))
    if not args.no_checks and not ok:
        raise SystemExit(f"bench.py: factorisation does not match the oracle: {out['checks']}")
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


def stream_ceiling(torch, args):
    """What ONE launch can read when it does nothing else: 24 MiB (the size of the headline
    workload's weight stream) per launch, 128-bit loads, rotated over 25 buffers (600 MiB)
    so that no launch finds its bytes in the Infinity Cache; and the same on one buffer."""
    import numpy as np

    import paper_2603_25385_amd as G

    n = 24 << 20
    steps = args.steps or 200
    bufs = [torch.empty(n, dtype=torch.uint8, device="cuda").fill_(i + 1) for i in range(25)]
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")

    def step(i):
        G.glowq_probe_stream_read(bufs[i % len(bufs)].data_ptr(), n, sink.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream)

    def step_hot(i):
        G.glowq_probe_stream_read(bufs[0].data_ptr(), n, sink.data_ptr(),
                                  torch.cuda.current_stream().cuda_stream)

    for i in range(25):
        step(i)
    torch.cuda.synchronize()
    ms, _ = time_steps(torch, step, steps, args.mode, REPLAYS)
    ms_hot, _ = time_steps(torch, step_hot, steps, args.mode, 2)
    med = float(np.median(ms))
    print(json.dumps({"metric": "one-launch streaming read of 24 MiB (measured ceiling)",
                      "value": n / med / 1e6, "unit": "GB/s", "steps": steps, "launch": args.mode,
                      "us_per_step_median": med * 1e3, "us_per_step_min": min(ms) * 1e3,
                      "hot_us_per_step": min(ms_hot) * 1e3, "bytes_per_step": n,
                      "frac_of_hbm_peak": n / med / 1e6 / HBM_PEAK_GBS}))
    return 0


def mfma_ceiling(torch, args, bf16):
    """What the matrix cores deliver on register-resident operands (16x16x32, two waves per
    SIMD on every compute unit): the clock-limited rate under a full-chip load."""
    import numpy as np

    import paper_2603_25385_amd as G

    steps = args.steps or 5
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    rows = []
    for wps in (1, 2, 4):
        iters = 40000 // wps
        flops = [0.0]

        def step(i):
            flops[0] = G.glowq_probe_mfma(iters, bf16, wps, sink.data_ptr(),
                                          torch.cuda.current_stream().cuda_stream)

        step(0)
        torch.cuda.synchronize()
        ms, _ = time_steps(torch, step, steps, "eager", REPLAYS)
        med = float(np.median(ms))
        rows.append({"waves_per_simd": wps, "TFLOPs": flops[0] / (med * 1e-3) / 1e12,
                     "ms_per_step_median": med, "ms_per_step_min": min(ms)})
    tf = max(r["TFLOPs"] for r in rows)
    name = ["16x16x32 f16", "16x16x32 bf16", "block-scaled 16x16x128 fp8 x fp4", "block-scaled 16x16x128 fp4 x fp4",
            "block-scaled 32x32x64 fp8 x fp4"][bf16]
    peak = [MFMA_PEAK_TFLOPS, MFMA_PEAK_TFLOPS, FP8_PEAK_TFLOPS, 2 * FP8_PEAK_TFLOPS, FP8_PEAK_TFLOPS][bf16]
    per_clock = [1024, 1024, 2048, 4096, 2048][bf16]        # flops per SIMD and clock at the published peak
    print(json.dumps({"metric": f"register-resident {name} matrix loop (measured ceiling)",
                      "value": tf, "unit": "TFLOP/s", "steps": steps, "by_occupancy": rows,
                      "frac_of_mfma_peak": tf / peak, "published_peak_TFLOPs": peak,
                      "implied_clock_GHz": tf * 1e12 / (256 * 4 * per_clock) / 1e9}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
