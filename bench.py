#!/usr/bin/env python3
"""Benchmark of the mini-sequence LM-head + cross-entropy path on one MI355X.

One "step" is one forward call plus one backward call (with logit
recomputation) over one batch of seeded synthetic input that is already
resident in HBM.  The workload is the long-sequence Llama3-8B-shaped
configuration the target is stated on (config 3: S=32768, d=4096, V=128256,
M=32).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]

`value` and `ms_per_step` come from the wall clock around the K timed steps (synchronised on both sides);
`step_ms` gives median / min / max of the individual steps from events recorded between them on the same stream.
The per-kernel figures (`kernels`, `roofline`) come from HIP events the library records around every launch on
the caller's stream INSIDE that timed region (so `value` includes their small cost; `--no-kernel-timing` leaves
them out).  `roofline.traffic` is read from profiles/pmc_traffic_per_launch.txt, the table the rocprofv3 counter
summaries in profiles/ cite.

`--path mlp` times the mini-sequence MLP block instead (forward + backward with recomputation of the
intermediates, Llama3-8B shape S=8192, d=4096, I=14336, chunk size C = d) and prints the same kind of line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published

# executed flop per step of each GEMM kernel kind, in units of S*d*V (a kind with no launches in a run is skipped)
GEMM_KINDS = {"fwd_gemm_lse": 2.0, "bwd_gemm_dlogits": 2.0, "bwd_gemm_dh": 2.0, "bwd_gemm_dw": 2.0, "bwd_gemm_dh_dw": 4.0}

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "pmc_traffic_per_launch.txt")


def pmc_traffic_bytes(path_name: str, config: int, schedule: str, kernel: str):
    """Bytes fetched + written beyond L2 per launch of `kernel`, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this command scaled by a copy of known size: a line `path config schedule kernel fetched_bytes written_bytes` of
    the table under profiles/ (schedule `-` = any).  None if the table has no such line."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                t = line.split("#")[0].split()
                if len(t) == 6 and t[0] == path_name and int(t[1]) == config and t[2] in (schedule, "-") and t[3] == kernel:
                    return float(t[4]) + float(t[5])
    except OSError:
        pass
    return None


def mfma_probe(mst, torch):
    """Empirical matrix-core rate of this chip with no data movement: a register-resident MFMA loop, all-zero
    operands and pseudo-random operands (the chip is power limited, so the two differ)."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    out = {}
    for name, scale in (("zero_operands", 0.0), ("random_operands", 1.0)):
        mst.mst_mfma_probe(512, 200, scale, sink, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        flop = mst.mst_mfma_probe(512, 6000, scale, sink, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        out[name + "_tflops"] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    out["what"] = "512 workgroups x 8 waves x 6000 x 16 v_mfma_f32_32x32x16_bf16 on register-resident operands"
    return out


def library_gemm_yardstick(torch, H, W, S, d, V, reps=5):
    """The path's contractions as unfused library GEMMs on the benchmark's own operands: logits = H W^T, then with the
    full S x V softmax materialised in bf16 (which the path never does), dH = G W and dW = G^T H.  Medians of `reps`
    launches each.  A plain head runs four of them per step (the logits twice when it recomputes) plus the softmax
    passes this figure leaves out."""
    Z = torch.empty((S, V), dtype=torch.bfloat16, device="cuda")
    oH = torch.empty((S, d), dtype=torch.bfloat16, device="cuda")
    oW = torch.empty((V, d), dtype=torch.bfloat16, device="cuda")

    def med(fn):
        fn()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))[reps // 2]

    res = {"logits": med(lambda: torch.matmul(H, W.t(), out=Z))}
    for r0 in range(0, S, 2048):                       # G = softmax(logits), in place, block by block
        Z[r0:r0 + 2048] = torch.softmax(Z[r0:r0 + 2048].float(), dim=1).to(torch.bfloat16)
    res["dH"] = med(lambda: torch.matmul(Z, W, out=oH))
    res["dW"] = med(lambda: torch.matmul(Z.t(), H, out=oW))
    flop = 2.0 * S * d * V
    return {"what": "torch.matmul bf16 (library GEMM), same H and W, G = bf16 softmax of the logits; median ms per GEMM",
            "ms": res, "tflops": {k: flop / (v * 1e-3) / 1e12 for k, v in res.items()},
            "four_gemms_ms": 2 * res["logits"] + res["dH"] + res["dW"]}


def cpu_baseline(inp, sample_rows: int):
    """The fp64 oracle as it stands, timed on the host cores on the first `sample_rows` tokens."""
    import numpy as np
    from oracle import lmhead_ce_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rows = np.arange(min(sample_rows, inp.cfg.S))
    H = inp.H_f64(rows)
    W = inp.W_f64()
    t0 = time.perf_counter()
    r = orc.lmhead_ce(H, W, inp.labels[rows], inp.ignore_index)
    dt = time.perf_counter() - t0
    flops = 6.0 * len(rows) * inp.cfg.d * inp.cfg.V       # forward + dH + dW, no recomputation
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": f"first {len(rows)} of {inp.cfg.S} tokens of the same workload, full V and d, fp64 numpy "
                  f"(loss+dH+dW = 6*S*d*V flop), {dt:.1f} s wall",
        "seconds": dt, "loss_on_sample": r["loss"],
    }


MLP_KINDS = ("gateup", "down", "da", "gateup_bwd", "dx", "dw")
# executed flop per step of each MLP kernel kind, in units of S*d*I
MLP_FLOP_UNITS = {"gateup": 4.0, "down": 2.0, "da": 2.0, "gateup_bwd": 4.0, "dx": 4.0, "dw": 6.0}

def mlp_cpu_baseline(inp, sample_rows: int):
    """The fp64 MLP oracle as it stands, timed on the host cores on the first `sample_rows` tokens."""
    import numpy as np
    from oracle import mlp_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rows = np.arange(min(sample_rows, inp.cfg.S))
    args = [inp.f64("X", rows), inp.f64("Wg"), inp.f64("Wu"), inp.f64("Wd"), inp.f64("dO", rows)]
    t0 = time.perf_counter()
    r = orc.mlp(*args)
    dt = time.perf_counter() - t0
    flops = 18.0 * len(rows) * inp.cfg.d * inp.cfg.I          # forward 6 + backward 12, no recomputation
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": f"first {len(rows)} of {inp.cfg.S} tokens of the same workload, full d and I, fp64 numpy "
                  f"(O, dX and the three weight gradients = 18*S*d*I flop), {dt:.1f} s wall",
        "seconds": dt, "checksum": float(np.abs(r["O"]).sum()),
    }


def main_mlp(args) -> int:
    import torch
    import mst_inputs as mi
    import paper_2407_15892_amd as mst
    from mst_inputs import to_device_bf16

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    mst.load_mlp_library()
    cfg = mi.MLP_CONFIGS[args.config]
    t0 = time.perf_counter()
    inp = mi.make_mlp_inputs(cfg)
    gen_s = time.perf_counter() - t0
    S, d, I, M = cfg.S, cfg.d, cfg.I, cfg.M
    X, Wg, Wu, Wd, dO = (to_device_bf16(getattr(inp, n + "_bits")) for n in ("X", "Wg", "Wu", "Wd", "dO"))
    fwd_bytes, bwd_bytes = mst.mst_mlp_workspace_bytes(S, d, I, M)
    ws = torch.empty(max(fwd_bytes, bwd_bytes), dtype=torch.uint8, device="cuda")
    O = torch.empty((S, d), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((S, d), dtype=torch.bfloat16, device="cuda")
    dWg = torch.empty((I, d), dtype=torch.float32, device="cuda")
    dWu = torch.empty((I, d), dtype=torch.float32, device="cuda")
    dWd = torch.empty((d, I), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def fwd():
        mst.mst_mlp_fwd(X, Wg, Wu, Wd, M, ws, O, stream)

    def bwd():
        mst.mst_mlp_bwd(X, Wg, Wu, Wd, dO, M, ws, dX, dWg, dWu, dWd, stream)

    if args.pmc_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    e[0].record(stream); fwd(); e[1].record(stream); bwd(); e[2].record(stream)
    torch.cuda.synchronize()
    fwd_ms, bwd_ms = e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])

    timing = not args.no_kernel_timing
    mst.mst_mlp_profile_enable(max(1, args.kernel_timing_every) if timing else 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fwd(); bwd()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kern = mst.mst_mlp_profile_collect() if timing else {}   # kind -> (ms of the timed launches, timed launches, all launches)
    mst.mst_mlp_profile_enable(0)

    ms_per_step = dt * 1e3 / args.steps
    f_exec = 22.0 * S * d * I          # forward 6, recomputation 4, dA 2, dX 4, weight gradients 6
    tflops = f_exec / (ms_per_step * 1e-3) / 1e12
    roofline, kernels = None, {}
    if kern:
        for k, (ms, n, issued) in kern.items():
            if n:
                fl = MLP_FLOP_UNITS[k] * S * d * I / (issued / args.steps)
                kernels[k] = {"launches": issued, "timed_launches": n, "avg_ms": ms / n,
                              "total_ms_per_step": ms / n * issued / args.steps, "tflops": fl / (ms / n * 1e-3) / 1e12}
        dom = max(MLP_KINDS, key=lambda k: kernels.get(k, {}).get("total_ms_per_step", 0.0))
        ms, n, issued = kern[dom]
        fl = MLP_FLOP_UNITS[dom] * S * d * I / (issued / args.steps)
        achieved = fl / (ms / n * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                    "traffic": pmc_traffic_bytes("mlp", args.config, "-", dom),
                    "flop_per_launch": fl, "avg_launch_ms": ms / n, "launches_per_step": issued / args.steps,
                    "timed_launches": n}
    out = {
        "metric": "MsT-MLP fwd+bwd TFLOP/s (22*S*d*I executed flop incl. recomputation)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"MLP config {cfg.index} {cfg.name}: S={S} d={d} I={I} M={M} (C={cfg.C}), bf16 X/weights/dO, "
                               f"fwd+bwd with recomputation of the intermediates", "S": S, "d": d, "I": I, "M": M},
        "frac_of_bf16_peak": tflops / PEAK_BF16_TFLOPS,
        "tflops_18SdI_convention": 18.0 * S * d * I / (ms_per_step * 1e-3) / 1e12,
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "peak_workspace_bytes": {"fwd": fwd_bytes, "bwd": bwd_bytes, "full_sequence_intermediate_bf16": S * I * 2},
        "checksum_O": float(O.float().abs().sum().item()),
        "roofline": roofline, "kernels": kernels, "input_generation_s": gen_s,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = mlp_cpu_baseline(inp, args.cpu_sample_rows)
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--path", choices=("lmhead", "mlp"), default="lmhead",
                    help="which block to time: the LM-head + cross-entropy (the headline metric) or the MLP")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None,
                    help="workload: LM-head configs 1-5 (default 3, the target configuration), MLP configs 1-4 (default 2)")
    ap.add_argument("--m", type=int, default=None,
                    help="LM-head path: override the number of mini-sequences M of the chosen configuration (sweeps)")
    ap.add_argument("--rows", type=int, default=None,
                    help="LM-head path: override the number of tokens S (same value distributions, own seed stream)")
    ap.add_argument("--operands", choices=("recipe", "zero"), default="recipe",
                    help="LM-head path: 'zero' replaces H and W by zeros on the device (same kernels, same traffic, the "
                         "matrix cores multiply zeros): a power probe, NOT a benchmark line")
    ap.add_argument("--cpu-sample-rows", type=int, default=4096)
    ap.add_argument("--bwd-schedule", choices=("auto", "pairs", "blocks", "blocks_fused"), default="auto",
                    help="order of the LM-head backward pass (default: the library's own choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="do not bracket kernels with events inside the timed region")
    ap.add_argument("--kernel-timing-every", type=int, default=5,
                    help="bracket every n-th launch of each kernel kind with events inside the timed region (default 5: "
                         "the launches of a kind repeat with period 8 or 32, so an odd stride visits every position; events "
                         "on every launch cost 0.4-0.7 %% of the step, on every third 0.1-0.25 %%)")
    ap.add_argument("--library-gemm", action="store_true",
                    help="LM-head path: after the timed region also time the path's three contractions as plain library "
                         "GEMMs (torch.matmul, bf16) on the same H and W and a materialised softmax: a yardstick for what "
                         "the chip sustains on these shapes and this data, not part of the step")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy, the known-size kernel the HBM counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2
    if args.config is None:
        args.config = 2 if args.path == "mlp" else 3
    if args.path == "mlp":
        return main_mlp(args)

    import numpy as np
    import torch
    import mst_inputs as mi
    import paper_2407_15892_amd as mst
    from mst_inputs import to_device_bf16

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    mst.load_library()
    mst.mst_set_bwd_schedule({"auto": mst.BWD_SCHEDULE_AUTO, "pairs": mst.BWD_SCHEDULE_PAIRS,
                              "blocks": mst.BWD_SCHEDULE_BLOCKS,
                              "blocks_fused": mst.BWD_SCHEDULE_BLOCKS_FUSED}[args.bwd_schedule])
    cfg = mi.CONFIGS[args.config]
    if args.m is not None or args.rows is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, S=args.rows or cfg.S, M=args.m or cfg.M,
                                  name=cfg.name + "-variant" + (f"-S{args.rows}" if args.rows else "") +
                                  (f"-M{args.m}" if args.m else ""))
    sched = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
    sched["schedule"] = {mst.BWD_SCHEDULE_PAIRS: "pairs", mst.BWD_SCHEDULE_BLOCKS: "blocks",
                         mst.BWD_SCHEDULE_BLOCKS_FUSED: "blocks_fused"}[sched["schedule"]]
    t0 = time.perf_counter()
    inp = mi.make_inputs(cfg)
    gen_s = time.perf_counter() - t0
    S, d, V, M = cfg.S, cfg.d, cfg.V, cfg.M

    H = to_device_bf16(inp.H_bits)
    W = to_device_bf16(inp.W_bits)
    if args.operands == "zero":
        H.zero_()
        W.zero_()
    labels = torch.from_numpy(inp.labels).cuda()
    fwd_bytes, bwd_bytes = mst.mst_workspace_bytes(S, d, V, M)
    ws = torch.empty(max(fwd_bytes, bwd_bytes), dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lse = torch.empty(S, dtype=torch.float32, device="cuda")
    nv = torch.zeros(1, dtype=torch.int64, device="cuda")
    dH = torch.empty((S, d), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((V, d), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        mst.mst_lmhead_ce_fwd(H, W, labels, inp.ignore_index, M, ws, loss, lse, nv, stream)
        mst.mst_lmhead_ce_bwd(H, W, labels, inp.ignore_index, M, 1.0, lse, nv, ws, dH, dW, stream)

    if args.pmc_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        b = torch.empty_like(a)
        b.copy_(a)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # separate forward / backward split (untimed for the headline, reported for information)
    e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    e[0].record(stream)
    mst.mst_lmhead_ce_fwd(H, W, labels, inp.ignore_index, M, ws, loss, lse, nv, stream)
    e[1].record(stream)
    mst.mst_lmhead_ce_bwd(H, W, labels, inp.ignore_index, M, 1.0, lse, nv, ws, dH, dW, stream)
    e[2].record(stream)
    torch.cuda.synchronize()
    fwd_ms, bwd_ms = e[0].elapsed_time(e[1]), e[1].elapsed_time(e[2])

    timing = not args.no_kernel_timing
    mst.mst_profile_enable(max(1, args.kernel_timing_every) if timing else 0)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(args.steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kern = mst.mst_profile_collect() if timing else {}      # kind -> (ms of the timed launches, timed launches, all launches)
    mst.mst_profile_enable(0)
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    ms_per_step = dt * 1e3 / args.steps
    f_exec = 8.0 * S * d * V                      # fwd GEMM + recompute + dH + dW
    tflops = f_exec / (ms_per_step * 1e-3) / 1e12

    # roofline of the dominant kernel (largest share of the timed region)
    roofline = None
    kernels = {}
    if kern:
        for k, (ms, n, issued) in kern.items():
            if n:
                kernels[k] = {"launches": issued, "timed_launches": n, "avg_ms": ms / n,
                              "total_ms_per_step": ms / n * issued / args.steps}
        # a GEMM kind executes GEMM_KINDS[kind] * S*d*V flop per step in total, split over its launches of that step
        def flop_per_launch(kind):
            return GEMM_KINDS[kind] * S * d * V / (kern[kind][2] / args.steps)
        dom = max(GEMM_KINDS, key=lambda k: kernels.get(k, {}).get("total_ms_per_step", 0.0))
        ms, n, issued = kern[dom]
        achieved = flop_per_launch(dom) / (ms / n * 1e-3) / 1e12
        traffic = None if (args.m or args.rows) else pmc_traffic_bytes("lmhead", args.config, sched["schedule"], dom)
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                    "flop_per_launch": flop_per_launch(dom), "avg_launch_ms": ms / n,
                    "launches_per_step": issued / args.steps, "timed_launches": n}
        if dom == "bwd_gemm_dw":
            # this kernel also moves dW through HBM: every row block writes it, every block after the first reads it
            # first; dlogits is read once, H once per vocabulary window
            passes = issued / args.steps
            n_rb, n_win = sched["row_blocks"], sched["windows"]
            alg_bytes = ((2 * n_rb - 1) * 4.0 * V * d + 2.0 * S * V + 2.0 * S * d * n_win) / passes
            roofline["hbm_side"] = {"algorithmic_bytes_per_launch": alg_bytes,
                                    "achieved_GBs": alg_bytes / (ms / n * 1e-3) / 1e9, "peak_GBs": PEAK_HBM_GBS,
                                    "frac": alg_bytes / (ms / n * 1e-3) / 1e9 / PEAK_HBM_GBS}
        for k in GEMM_KINDS:
            ms_k, n_k, _ = kern.get(k, (0.0, 0, 0))
            if n_k:
                kernels[k]["tflops"] = flop_per_launch(k) / (ms_k / n_k * 1e-3) / 1e12

    out = {
        "metric": "LM-head+CE fwd+bwd TFLOP/s (8*S*d*V executed flop incl. recomputation)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic" if args.operands == "recipe" else "all-zero H and W (power probe, not a benchmark line)",
        "step_ms": {"median": per_step[len(per_step) // 2] if len(per_step) % 2 else
                    0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2]),
                    "min": per_step[0], "max": per_step[-1], "n": len(per_step),
                    "what": "individual timed steps, events between steps on the launch stream"},
        "kernel_timing": (f"HIP events recorded by the library inside the timed region around every "
                          f"{max(1, args.kernel_timing_every)}-th launch of each kernel kind" if timing else "off"),
        "target": {"frac_of_bf16_peak": 0.60, "ms_per_step_at_target": f_exec / (0.60 * PEAK_BF16_TFLOPS * 1e12) * 1e3,
                   "gap_ms": ms_per_step - f_exec / (0.60 * PEAK_BF16_TFLOPS * 1e12) * 1e3},
        "config": {"workload": f"config {cfg.index} {cfg.name}: S={S} d={d} V={V} M={M} (C={cfg.C}), "
                               f"bf16 H/W, int32 labels, fwd+bwd with logit recomputation",
                   "S": S, "d": d, "V": V, "M": M},
        "frac_of_bf16_peak": tflops / PEAK_BF16_TFLOPS,
        "tflops_6SdV_convention": 6.0 * S * d * V / (ms_per_step * 1e-3) / 1e12,
        "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "peak_workspace_bytes": {"fwd": fwd_bytes, "bwd": bwd_bytes, "cap_one_fp32_logits_chunk": cfg.C * V * 4},
        "loss": float(loss.item()), "n_valid": int(nv.item()), "bwd_schedule": sched,
        "roofline": roofline, "kernels": kernels, "input_generation_s": gen_s,
    }
    out["empirical_mfma_peak"] = mfma_probe(mst, torch)
    if args.library_gemm:
        del ws, dW
        out["library_gemm"] = library_gemm_yardstick(torch, H, W, S, d, V)
    if not args.no_cpu_baseline and args.operands == "recipe":
        out["cpu_baseline"] = cpu_baseline(inp, args.cpu_sample_rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
