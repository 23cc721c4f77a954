#!/usr/bin/env python3
"""Benchmark of the CALS hot path on one MI355X.

A step is one round of the full algorithm (Alg. 3) over every model of the workload: three fused
MTTKRPs, the per-model Gram/Hadamard/Cholesky/normalise/fit updates, the fit read-back and the retire
decision; the last timed step retires all models (factor copy-out and bookkeeping included).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg2|cfg1|cfg5shape|cfg3shape]

`--workload cfgNjob` (N = 1..5) instead runs the configuration's whole job once as it is specified (queue, slots,
tolerances, iteration caps, non-negativity, line search) and reports models completed per second; --steps and
--warmup do not apply.  The default run appends, to the one JSON line: the whole jobs of configurations 1, 2, 3 and 5
under "jobs" (a job of under a quarter of a second is run twice and the second run reported); the fused MTTKRP alone
at each of those configurations' full width under "mttkrp_by_config"; a low-width point on the cfg4 tensor (16
columns: the bandwidth-bound regime, with its own roofline object against the HBM peak) under "low_width"; the order-4
workload (see below) under "order_n"; and the oracle's side of every figure under "cpu_baseline".  The fused MTTKRP
alone is always timed in steady state (steady_mttkrp: 100 ms of untimed calls, then at least 25 ms of timed ones).

`--workload sweepW1000` / `sweepW300` / `sweepWodd` time the fused MTTKRP alone, all three modes, over fused widths
1..1024 on the cfg4 tensor / a 300^3 tensor (the analogue of the paper's Fig. 1) / a 999 x 1001 x 997 tensor.  `--yardstick` prints the device's compute-unit
count and clock and its practical peaks (back-to-back fp64 MFMA; streaming read of a 4 GiB buffer).

`--workload mttkrpN` (N = 1..5) times the fused MTTKRP alone, all three modes, on configuration N's tensor at the width
its job starts with (cfg5: also at the full buffer width, 640); `mttkrp300` does so on a 300^3 tensor at width 420.
These are the launches whose counters profiles/short_modes_mttkrp.md holds.

`--workload splitscan` / `ridgescan` time the fused MTTKRP under forced plans (split counts on the cache-resident
short-mode shapes; row tiles per wavefront x split counts at widths 32-96 on 1000^3); `--workload kernelscan` times
the planner's choice against the tile kernel and the rows kernel forced over a grid of shapes and widths:
profiles/forced_plan_scans.md.

`--workload order4` / `order5` time the path on a tensor of order 4 (180^4) / 5 (60^5), 8.4 and 6.2 GB: the fused
MTTKRP alone per mode at several widths (contraction kernel by events, and the whole call including the explicit
partial Khatri-Rao products), and timed rounds of the 40-model, width-420 mix of cfg4.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP64_MFMA_TFLOPS = 78.6      # MI355X dense fp64 matrix peak (256 CUs x 128 flop/clk x 2.4 GHz)
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-jobs", action="store_true", help="skip the whole-job runs appended to the default line")
    ap.add_argument("--reuse", action="store_true",
                    help="two-step sweeps (CALS_CTX_REUSE): modes 2 and 3 from the tensor contracted with the mode-1 factors")
    ap.add_argument("--trace", action="store_true",
                    help="job workloads: time every round on the device (events) and report the MTTKRP rate over "
                         "tenths of the job's flops (the paper's efficiency-over-the-run measurement, Sec. 6)")
    ap.add_argument("--yardstick", action="store_true", help="device properties and practical peaks (MFMA-only, read)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain elementwise copy kernel of known size (counter calibration for rocprofv3 --pmc)")
    return ap.parse_args()


def workload(name: str):
    from workloads import get_config
    cid = {"cfg1": 1, "cfg2": 2, "cfg3shape": 3, "cfg4": 4, "cfg5shape": 5}[name]
    return get_config(cid)


def run_job(cid: int, T_dev=None, reuse: bool = False, trace: bool = False) -> dict:
    """One whole job of configuration `cid`, as specified: every model enqueued with its own tolerance, iteration
    cap and flags; rounds until the queue and the slots are empty.  Tensor resident in HBM before the clock starts."""
    import torch
    import paper_2010_04678_amd as P
    from workloads import get_config, make_models, make_tensor
    cfg = get_config(cid)
    models = make_models(cfg)
    if T_dev is None:
        T_dev = torch.from_numpy(make_tensor(cfg, threads=min(16, os.cpu_count() or 8))).to("cuda:0")
    ctx = P.Context(max_total_rank=cfg.max_total_rank, max_slots=cfg.max_slots,
                    flags=(P.CTX_REUSE if reuse else 0) | (P.CTX_TIMING if trace else 0))
    ctx.submit_tensor(T_dev)
    for m in models:
        ctx.enqueue_model(m["init"], m["tol"], m["max_iters"], m["flags"], m["ls_alpha"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = ctx.stats()
    res = ctx.poll_retired(len(models) + 1)
    assert len(res) == len(models)
    iters = sum(r.iters for r in res)
    profile = efficiency_profile(ctx.round_log(cap=1 << 20)) if trace else None
    ctx.close()
    out = job_summary(cfg, reuse, models, dt, st, iters)
    if profile is not None:
        out["efficiency_profile"] = profile
    return out


def efficiency_profile(log) -> list:
    """Rounds grouped into tenths of the job's algorithmic MTTKRP flops: device time, mean fused width and the rate
    flops / time of each tenth (time of whole rounds: MTTKRPs, updates, line search)."""
    total = sum(r[4] for r in log)
    out, acc, k = [], 0.0, 0
    for tenth in range(1, 11):
        fl = ms = w = 0.0
        n = 0
        while k < len(log) and (acc + log[k][4] <= total * tenth / 10.0 * (1 + 1e-12) or tenth == 10):
            acc += log[k][4]; fl += log[k][4]; ms += log[k][3]; w += log[k][2]; n += 1; k += 1
        if n:
            out.append({"upto_fraction_of_flops": tenth / 10.0, "rounds": n, "mean_width": w / n, "ms": ms,
                        "tflops": fl / (ms * 1e-3) * 1e-12 if ms > 0 else None})
    return out


def job_summary(cfg, reuse, models, dt, st, iters) -> dict:
    return {"workload": cfg.name + "_job", "two_step_sweeps": bool(reuse), "models": len(models), "seconds": dt, "ms": dt * 1e3, "models_per_s": len(models) / dt,
            "rounds": int(st.rounds), "ms_per_round": dt / max(1, st.rounds) * 1e3, "model_iterations": iters,
            "model_iterations_per_s": iters / dt, "mttkrp_gflops": st.mttkrp_flops / dt * 1e-9}


SWEEP_WIDTHS = [1, 2, 4, 8, 16, 32, 64, 128, 256, 420, 512, 1024]


STEADY_WARM_MS = 100.0     # launch time spent before a timed run of the fused MTTKRP alone
STEADY_MS = 25.0           # least launch time inside the timed run


def steady_mttkrp(ctx, mode: int, U, M, width: int, min_reps: int = 3, max_reps: int = 300):
    """Times cals_mttkrp(mode) in steady state: repeats the call untimed until STEADY_WARM_MS of launches have gone by,
    then times as many calls as fill STEADY_MS (at least min_reps).  A job keeps the GPU busy for its whole length, and
    a sub-millisecond launch sequence measured right after an idle stretch runs 10-17 % slower than the same launches
    some tens of milliseconds into continuous work.  Returns (contraction ms, reduction ms, host ms per call, timed
    calls, all calls)."""
    import torch
    n = mode - 1
    s0 = ctx.stats()
    ctx.mttkrp(mode, U, M, total_rank=width)
    torch.cuda.synchronize()
    s1 = ctx.stats()
    one = max(1e-3, s1.mttkrp_ms[n] - s0.mttkrp_ms[n] + s1.reduce_ms[n] - s0.reduce_ms[n])
    warm = min(8 * max_reps, int(STEADY_WARM_MS / one))
    for k in range(warm):
        ctx.mttkrp(mode, U, M, total_rank=width)
        if k % 64 == 63:
            ctx.stats()          # reads the launches' events back, so that the library reuses them
    reps = min(max_reps, max(min_reps, int(np.ceil(STEADY_MS / one))))
    torch.cuda.synchronize()
    s0 = ctx.stats()
    t0 = time.perf_counter()
    for _ in range(reps):
        ctx.mttkrp(mode, U, M, total_rank=width)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    s1 = ctx.stats()
    return ((s1.mttkrp_ms[n] - s0.mttkrp_ms[n]) / reps, (s1.reduce_ms[n] - s0.reduce_ms[n]) / reps,
            (t1 - t0) / reps * 1e3, reps, 1 + warm + reps)


def run_sweep(which: str, reps: int = 3) -> dict:
    """Fused MTTKRP alone over fused widths (columns of random factors), all three modes, on an HBM-resident tensor."""
    import torch
    import paper_2010_04678_amd as P
    from workloads import get_config, make_tensor
    if which == "sweepW1000":
        cfg = get_config(4)
        T = torch.from_numpy(make_tensor(cfg, threads=min(16, os.cpu_count() or 8))).to("cuda:0")
        dims = tuple(cfg.dims)
    else:
        # 300^3 (fits the last-level cache), or an 8 GB tensor with no dimension a multiple of 4 (the unaligned reads)
        dims = (300, 300, 300) if which == "sweepW300" else (999, 1001, 997)
        g = torch.Generator(device="cuda:0")
        g.manual_seed(300)
        T = torch.rand(dims[::-1], dtype=torch.float64, device="cuda:0", generator=g)
    I1, I2, I3 = dims
    ctx = P.Context(max_total_rank=max(SWEEP_WIDTHS), flags=P.CTX_TIMING)
    ctx.submit_tensor(T)
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7)
    rows = []
    for R in SWEEP_WIDTHS:
        ld = (R + 15) // 16 * 16
        U = [torch.rand((d, ld), dtype=torch.float64, device="cuda:0", generator=g) for d in dims]
        ms = []
        for mode in (1, 2, 3):
            M = torch.zeros((dims[mode - 1], ld), dtype=torch.float64, device="cuda:0")
            ms.append(steady_mttkrp(ctx, mode, U, M, R, min_reps=reps))
        flops = 2.0 * R * I1 * I2 * I3
        nbytes = 8.0 * I1 * I2 * I3 + 8.0 * R * (I1 + I2 + I3)
        rows.append({"width": R, "contraction_ms": [m[0] for m in ms], "reduce_ms": [m[1] for m in ms],
                     "tflops": [flops / (m[0] * 1e-3) * 1e-12 for m in ms],
                     "algorithmic_tb_per_s": [nbytes / (m[0] * 1e-3) * 1e-12 for m in ms],
                     "timed_calls": [m[3] for m in ms], "calls": [m[4] for m in ms]})
    ctx.close()
    return {"metric": "fused MTTKRP alone, widths 1..1024 (sweep W)", "workload": which, "dims": list(dims),
            "reps": "at least %d, and as many as fill %.0f ms after %.0f ms of untimed calls" % (reps, STEADY_MS, STEADY_WARM_MS), "peak_mfma_tflops": PEAK_FP64_MFMA_TFLOPS, "peak_hbm_gbs": PEAK_HBM_GBS, "rows": rows}


def mttkrp_alone(T_dev, dims, width: int, reps: int = 5) -> dict:
    """The fused MTTKRP alone (cals_mttkrp) at `width` columns of random factors on the resident tensor, all three
    modes: per mode the contraction and the split-K reduction from HIP events inside the library (launch stream)."""
    import torch
    import paper_2010_04678_amd as P
    ctx = P.Context(max_total_rank=width, flags=P.CTX_TIMING)
    ctx.submit_tensor(T_dev)
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7)
    ld = (width + 15) // 16 * 16
    U = [torch.rand((d, ld), dtype=torch.float64, device="cuda:0", generator=g) for d in dims]
    contraction, reduce, calls = [], [], []
    for mode in (1, 2, 3):
        M = torch.zeros((dims[mode - 1], ld), dtype=torch.float64, device="cuda:0")
        c, r, _, _, n = steady_mttkrp(ctx, mode, U, M, width, min_reps=reps)
        contraction.append(c)
        reduce.append(r)
        calls.append(n)
    st = ctx.stats()
    ctx.close()
    I1, I2, I3 = dims
    flops = 2.0 * width * I1 * I2 * I3
    nbytes = 8.0 * I1 * I2 * I3 + 8.0 * width * (I1 + I2 + I3)
    total = [c + r for c, r in zip(contraction, reduce)]
    return {"width": width, "contraction_ms": contraction, "reduce_ms": reduce,
            "tflops": [flops / (t * 1e-3) * 1e-12 for t in total],
            "frac_of_mfma_peak": [flops / (t * 1e-3) * 1e-12 / PEAK_FP64_MFMA_TFLOPS for t in total],
            "algorithmic_gb_per_s": [nbytes / (t * 1e-3) * 1e-9 for t in total],
            "rows_kernel_launches": int(st.mttkrp_rows_launches), "launches": int(sum(st.mttkrp_launches)), "calls": calls}



# Forced-plan scans (development knobs of the library, read from the environment when a context is created): the
# measurements the split planner and the row-tile choice were fitted to and checked against.
SCANS = {
    # tensors the last-level cache holds: split count against the planner's own choice (first row of each block)
    "splitscan": [((300, 300, 40), 630, [None], [None, 8, 10, 12, 16, 20, 24, 30, 32, 40, 50, 64, 100, 128, 150]),
                  ((300, 300, 300), 420, [None], [None, 32, 40, 48, 51, 56, 64]),
                  ((4000, 200, 50), 640, [None], [None, 3, 4, 6, 24, 48, 51, 64, 100, 102, 128, 152]),
                  ((200, 200, 200), 110, [None], [None, 63, 84, 125])],
    # the ridge on the cfg 4 shape: row tiles per wavefront x split count at widths around the ridge point
    "ridgescan": [((1000, 1000, 1000), w, [None, 4, 2], [None, 64, 128, 192, 256, 384]) for w in (32, 48, 64, 96)],
}


def run_scan(which: str) -> dict:
    import torch
    import paper_2010_04678_amd as P
    rows = []
    for dims, width, wms, splits in SCANS[which]:
        g = torch.Generator(device="cuda:0")
        g.manual_seed(1)
        T = torch.rand(dims[::-1], dtype=torch.float64, device="cuda:0", generator=g)
        ld = (width + 15) // 16 * 16
        U = [torch.rand((d, ld), dtype=torch.float64, device="cuda:0", generator=g) for d in dims]
        flops = 2.0 * width * dims[0] * dims[1] * dims[2]
        first = True
        for wm in wms:
            for sp in [None] + list(splits) if first else splits:     # the very first pass over a tensor is not reported
                env = {}
                if wm is not None or sp is not None:
                    env["CALS_MTTKRP_KERNEL"] = "1"            # forced plans are plans of the tile kernel
                if wm is not None:
                    env["CALS_MTTKRP_WM"] = str(wm)
                if sp is not None:
                    env["CALS_MTTKRP_SPLITS"] = str(sp)
                for k in [k for k in os.environ if k.startswith("CALS_MTTKRP_")]:
                    del os.environ[k]
                os.environ.update(env)
                ctx = P.Context(max_total_rank=width, flags=P.CTX_TIMING)
                for k in env:
                    del os.environ[k]
                ctx.submit_tensor(T)
                ms = []
                for mode in (1, 2, 3):
                    M = torch.zeros((dims[mode - 1], ld), dtype=torch.float64, device="cuda:0")
                    c, r, _, _, _ = steady_mttkrp(ctx, mode, U, M, width)
                    ms.append((c, r))
                st = ctx.stats()
                ctx.close()
                if first:
                    first = False
                    continue
                rows.append({"dims": list(dims), "width": width, "wm": wm, "splits": sp,
                             "contraction_ms": [m[0] for m in ms], "reduce_ms": [m[1] for m in ms],
                             "tflops": [flops / ((m[0] + m[1]) * 1e-3) * 1e-12 for m in ms],
                             "rows_kernel_launches": int(st.mttkrp_rows_launches)})
        del T
        torch.cuda.empty_cache()
    return {"metric": "fused MTTKRP alone under forced plans (contraction + reduction, steady state)", "workload": which,
            "peak_mfma_tflops": PEAK_FP64_MFMA_TFLOPS, "rows": rows}


# Planner's choice against each kernel forced (CALS_MTTKRP_KERNEL = 1 tile kernel, 2 rows kernel wherever it can
# run): the grid the rows kernel's selection rule was fitted to.  (dims, modes, widths)
KERNEL_SCAN_WIDTHS = [48, 64, 80, 96, 112, 128, 144, 160, 176, 192, 208, 224, 240, 256, 320, 420]
KERNEL_SCAN = [((200, 200, 200), [1, 2], KERNEL_SCAN_WIDTHS + [512, 640, 1024]), ((160, 160, 160), [1, 3], KERNEL_SCAN_WIDTHS),
               ((128, 300, 300), [1], KERNEL_SCAN_WIDTHS), ((4000, 200, 50), [2, 3], KERNEL_SCAN_WIDTHS + [512, 640]),
               ((100, 100, 100), [1, 3], KERNEL_SCAN_WIDTHS), ((64, 512, 512), [1], KERNEL_SCAN_WIDTHS),
               ((300, 300, 40), [1, 2, 3], [64, 128, 192, 256, 320, 420, 512, 630]), ((208, 64, 1000), [1], KERNEL_SCAN_WIDTHS),
               ((96, 400, 400), [1], KERNEL_SCAN_WIDTHS), ((300, 300, 300), [1, 2], [64, 128, 256, 420]),
               ((500, 500, 500), [1, 3], [64, 128, 256, 420]), ((180, 180, 2000), [1, 2], [64, 128, 256, 420]),
               ((1000, 1000, 1000), [1, 2, 3], [16, 32, 64, 128])]


def run_kernel_scan() -> dict:
    import torch
    import paper_2010_04678_amd as P
    rows = []
    for dims, modes, widths in KERNEL_SCAN:
        g = torch.Generator(device="cuda:0")
        g.manual_seed(1)
        T = torch.rand(dims[::-1], dtype=torch.float64, device="cuda:0", generator=g)
        flops1 = 2.0 * dims[0] * dims[1] * dims[2]
        first = True
        for width in widths:
            ld = (width + 15) // 16 * 16
            U = [torch.rand((d, ld), dtype=torch.float64, device="cuda:0", generator=g) for d in dims]
            rec = {"dims": list(dims), "width": width, "modes": modes}
            for name, forced in ([("warm", None)] if first else []) + [("planner", None), ("tile", "1"), ("rows", "2")]:
                for k in [k for k in os.environ if k.startswith("CALS_MTTKRP_")]:
                    del os.environ[k]
                if forced:
                    os.environ["CALS_MTTKRP_KERNEL"] = forced
                ctx = P.Context(max_total_rank=width, flags=P.CTX_TIMING)
                os.environ.pop("CALS_MTTKRP_KERNEL", None)
                ctx.submit_tensor(T)
                ms = []
                for mode in modes:
                    M = torch.zeros((dims[mode - 1], ld), dtype=torch.float64, device="cuda:0")
                    c, r, _, _, _ = steady_mttkrp(ctx, mode, U, M, width)
                    ms.append(c + r)
                st = ctx.stats()
                ctx.close()
                if name != "warm":
                    rec[name + "_ms"] = ms
                    rec[name + "_tflops"] = [flops1 * width / (m * 1e-3) * 1e-12 for m in ms]
                    if name == "planner":
                        rec["planner_rows_kernel_launches"] = int(st.mttkrp_rows_launches)
                        rec["planner_launches"] = int(sum(st.mttkrp_launches))
            first = False
            rows.append(rec)
        del T
        torch.cuda.empty_cache()
    return {"metric": "fused MTTKRP alone: the planner's choice against each kernel forced (contraction + reduction, steady state)",
            "workload": "kernelscan", "peak_mfma_tflops": PEAK_FP64_MFMA_TFLOPS, "rows": rows}


def settled_job(cid: int, T_dev, reuse: bool = False) -> dict:
    """run_job; a job shorter than a quarter of a second is run a second time and that run is reported (the first run of
    a few milliseconds also pays for loading the kernels it is the first to launch, which is no part of its rate)."""
    first = run_job(cid, T_dev=T_dev, reuse=reuse)
    if first["seconds"] >= 0.25:
        first["run"] = "first and only"
        return first
    second = run_job(cid, T_dev=T_dev, reuse=reuse)
    second["run"] = "second of two"
    second["first_run_ms"] = first["ms"]
    return second


def config_leg(cid: int) -> dict:
    """Configuration `cid` on its own tensor: the whole job as specified, and the fused MTTKRP alone at the width the
    job starts with (all models that fit the buffers side by side)."""
    import torch
    from workloads import get_config, make_models, make_tensor
    cfg = get_config(cid)
    T_dev = torch.from_numpy(make_tensor(cfg, threads=min(16, os.cpu_count() or 8))).to("cuda:0")
    models = make_models(cfg)
    width, n = 0, 0
    for m in models:
        if width + m["rank"] > cfg.max_total_rank or (cfg.max_slots and n >= cfg.max_slots):
            break
        width += m["rank"]
        n += 1
    out = {"job": settled_job(cid, T_dev), "mttkrp": dict(workload=cfg.name, dims=list(cfg.dims), **mttkrp_alone(T_dev, tuple(cfg.dims), width))}
    if cid == 5:      # the queue job also with two-step sweeps, and the fused MTTKRP at the full buffer width
        out["job_two_step"] = settled_job(cid, T_dev, reuse=True)
        out["mttkrp_full_buffer"] = dict(workload=cfg.name, dims=list(cfg.dims), **mttkrp_alone(T_dev, tuple(cfg.dims), cfg.max_total_rank))
    del T_dev
    torch.cuda.empty_cache()
    return out


ORDER_N = {"order4": (180,) * 4, "order5": (60,) * 5}

def run_order_n(which: str, steps: int, warmup: int, reps: int = 3) -> dict:
    """Tensors of order above 3: rank-15 Uniform[0,1) factors plus 1 % Gaussian noise, generated on the device
    (seeded); models as in cfg4 (ranks 1..20 twice, Uniform[0,1) starting points)."""
    import torch
    import paper_2010_04678_amd as P
    from workloads import get_config, low_rank_tensor_device, uniform_factors
    dims = ORDER_N[which]
    N = len(dims)
    dev = torch.device("cuda:0")
    T, _ = low_rank_tensor_device(dims, 15, 1000 + N, noise=0.01)
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    elems = float(np.prod(dims))
    cfg = get_config(4)
    ranks = list(cfg.ranks)
    rstar = sum(ranks)
    ctx = P.Context(max_total_rank=rstar, flags=P.CTX_TIMING)
    ctx.submit_tensor(T)
    rows = []
    for R in (16, 128, 256, rstar):
        ld = (R + 15) // 16 * 16
        U = [torch.rand((d, ld), dtype=torch.float64, device=dev, generator=g) for d in dims]
        kern, call = [], []
        for mode in range(1, N + 1):
            M = torch.zeros((dims[mode - 1], ld), dtype=torch.float64, device=dev)
            c, r, host_ms, _, _ = steady_mttkrp(ctx, mode, U, M, R, min_reps=reps)
            kern.append(c + r)
            call.append(host_ms)
        flops = 2.0 * R * elems
        nbytes = 8.0 * elems
        rows.append({"width": R, "kernel_ms": kern, "call_ms": call,
                     "kernel_tflops": [flops / (m * 1e-3) * 1e-12 for m in kern],
                     "call_tflops": [flops / (m * 1e-3) * 1e-12 for m in call],
                     "tensor_tb_per_s": [nbytes / (m * 1e-3) * 1e-12 for m in call]})
    ctx.close()
    # timed rounds of the whole path (plain, and with two-step sweeps: the tensor read twice instead of N times)
    def timed(flags):
        ctx = P.Context(max_total_rank=rstar, flags=flags)
        ctx.submit_tensor(T)
        for k, r in enumerate(ranks):
            ctx.enqueue_model(uniform_factors(dims, r, cfg.init_seeds[k]), tol=-1.0, max_iters=warmup + steps)
        ctx.iterate(warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.iterate(steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        res = ctx.poll_retired()
        assert len(res) == len(ranks) and all(r.iters == warmup + steps for r in res)
        ctx.close()
        return dt, res

    dt, res = timed(0)
    dt2, res2 = timed(P.CTX_REUSE)
    flops = 2.0 * N * rstar * elems * steps
    return {"metric": "fused MTTKRP fp64 GFLOP/s on an order-%d tensor; whole rounds" % N, "value": flops / dt * 1e-9,
            "unit": "GFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": which, "dims": list(dims), "models": len(ranks), "total_rank": rstar},
            "models_per_s": len(ranks) / dt, "fits": [round(r.fit, 6) for r in res[:4]],
            "two_step_sweeps": {"ms_per_step": dt2 / steps * 1e3, "models_per_s": len(ranks) / dt2,
                                "effective_gflops": flops / dt2 * 1e-9, "fits": [round(r.fit, 6) for r in res2[:4]]},
            "peak_mfma_tflops": PEAK_FP64_MFMA_TFLOPS, "mttkrp_alone": rows}


def run_yardstick() -> dict:
    import torch
    import paper_2010_04678_amd as P
    prop = torch.cuda.get_device_properties(0)
    buf = torch.ones(1 << 29, dtype=torch.float64, device="cuda:0")      # 4 GiB
    ctx = P.Context(max_total_rank=16)
    out = {"yardstick": True, "device": prop.name, "gcn_arch": getattr(prop, "gcnArchName", ""),
           "compute_units": int(ctx.yardstick(3)), "clock_mhz": ctx.yardstick(2),
           "hbm_gib": prop.total_memory / 2 ** 30,
           "mfma_f64_only_tflops": ctx.yardstick(0, reps=5),
           "read_4gib_gb_per_s": ctx.yardstick(1, buf, reps=10),
           "spec_mfma_f64_tflops": PEAK_FP64_MFMA_TFLOPS, "spec_hbm_gb_per_s": PEAK_HBM_GBS}
    ctx.close()
    return out


def cpu_baseline(cfg, T: np.ndarray, models) -> dict:
    """The oracle as it stands, timed on this host on a bounded sample: its fused MTTKRP of the workload's
    full width, all three modes, on the first slabs of the same tensor (sized for roughly 10-30 s)."""
    import oracle as O
    I1, I2, I3 = cfg.dims
    U = [np.hstack([m["init"][n] for m in models]) for n in range(3)]
    R = U[0].shape[1]
    # probe on a thin sample, then size the timed sample for ~15 s
    s0 = max(1, min(I3, int(2e9 / (2.0 * R * I1 * I2)) or 1))
    Ts = np.ascontiguousarray(T[:s0])
    Us = [U[0], U[1], U[2][:s0]]
    t = time.perf_counter()
    O.mttkrp(Ts, Us, 1)
    dt = time.perf_counter() - t
    rate = 2.0 * R * I1 * I2 * s0 / max(dt, 1e-9)
    slabs = int(max(1, min(I3, (15.0 * rate / 3.0) / (2.0 * R * I1 * I2))))
    Ts = np.ascontiguousarray(T[:slabs])
    Us = [U[0], U[1], U[2][:slabs]]
    t = time.perf_counter()
    for mode in (1, 2, 3):
        O.mttkrp(Ts, Us, mode)
    dt = time.perf_counter() - t
    flops = 3 * 2.0 * R * I1 * I2 * slabs
    out = {"value": flops / dt * 1e-9, "unit": "GFLOP/s", "cores": O.num_threads(), "kind": "oracle",
           "sample": "oracle fused MTTKRP, all 3 modes, width %d, first %d of %d slabs (i3) of the %s tensor, %.1f s"
                     % (R, slabs, I3, cfg.name, dt)}
    # the other half of the metric (models completed per second, ALS iterations per second): the oracle's whole jobs
    # of configurations 1 and 2, and this workload's rate extrapolated from the MTTKRP sample above (its sweeps are
    # MTTKRP to 99 %: the per-model steps are not in the sample)
    from workloads import get_config, make_models, make_tensor
    jobs = []
    for cid in (1, 2):
        c = get_config(cid)
        Tc = make_tensor(c)
        mc = make_models(c)
        t = time.perf_counter()
        ref = O.cals(Tc, mc, c.max_total_rank, c.max_slots)
        dj = time.perf_counter() - t
        its = int(sum(ref["iters"]))
        jobs.append({"workload": c.name + "_job", "models": len(mc), "seconds": dj, "models_per_s": len(mc) / dj,
                     "model_iterations_per_s": its / dj, "kind": "oracle, whole job"})
    sweep_s = dt * (I3 / float(slabs))                       # one sweep = three fused MTTKRPs over all slabs
    its = cfg.max_iters
    jobs.append({"workload": cfg.name, "models": len(models), "models_per_s": len(models) / (its * sweep_s),
                 "model_iterations_per_s": len(models) / sweep_s, "sweeps_per_s": 1.0 / sweep_s,
                 "kind": "oracle, extrapolated from the timed MTTKRP sample (%d of %d slabs, three modes) to %d sweeps"
                         % (slabs, I3, its)})
    out["jobs"] = jobs
    return out


def main() -> int:
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    import torch
    if args.calibrate_copy:
        n = 1 << 28                                    # 2 GiB read + 2 GiB written per launch
        a = torch.ones(n, dtype=torch.float64, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "read_bytes_per_launch": 8 * n, "write_bytes_per_launch": 8 * n,
                          "launches": 3}))
        return 0
    import paper_2010_04678_amd as P
    from workloads import make_models, make_tensor

    if args.yardstick:
        print(json.dumps(run_yardstick()))
        return 0
    if args.workload.startswith("sweepW"):
        print(json.dumps(run_sweep(args.workload)))
        return 0
    if args.workload in SCANS:
        print(json.dumps(run_scan(args.workload)))
        return 0
    if args.workload == "kernelscan":
        print(json.dumps(run_kernel_scan()))
        return 0
    if args.workload in ORDER_N:
        print(json.dumps(run_order_n(args.workload, min(args.steps, 10), args.warmup)))
        return 0
    if args.workload.startswith("mttkrp"):
        from workloads import get_config
        if args.workload == "mttkrp300":
            g = torch.Generator(device="cuda:0")
            g.manual_seed(300)
            T300 = torch.rand((300, 300, 300), dtype=torch.float64, device="cuda:0", generator=g)
            rows = [dict(workload="300cube", dims=[300, 300, 300], **mttkrp_alone(T300, (300, 300, 300), 420, reps=3))]
        else:
            cid = int(args.workload[6:])
            cfgm = get_config(cid)
            Tm = torch.from_numpy(make_tensor(cfgm, threads=min(16, os.cpu_count() or 8))).to("cuda:0")
            width, n = 0, 0
            for r in cfgm.ranks:
                if width + r > cfgm.max_total_rank or (cfgm.max_slots and n >= cfgm.max_slots):
                    break
                width += r
                n += 1
            widths = [width] + ([cfgm.max_total_rank] if cfgm.max_total_rank != width else [])
            rows = [dict(workload=cfgm.name, dims=list(cfgm.dims), **mttkrp_alone(Tm, tuple(cfgm.dims), w, reps=3)) for w in widths]
        print(json.dumps({"metric": "fused MTTKRP alone, all three modes", "workload": args.workload,
                          "peak_mfma_tflops": PEAK_FP64_MFMA_TFLOPS, "rows": rows}))
        return 0
    if args.workload.endswith("job"):
        job = run_job(int(args.workload[3]), reuse=args.reuse, trace=args.trace)
        print(json.dumps({"metric": "CP-ALS models completed/sec", "value": job["models_per_s"], "unit": "models/s",
                          "n_gpus": 1, "steps": job["rounds"], "warmup": 0, "ms_per_step": job["ms_per_round"],
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
                          "data": "synthetic", "config": {"workload": job["workload"]}, "job": job}))
        return 0
    cfg = workload(args.workload)
    K, W = args.steps, args.warmup
    I1, I2, I3 = cfg.dims
    t_gen = time.perf_counter()
    T = make_tensor(cfg, threads=min(16, os.cpu_count() or 8))
    models = make_models(cfg)
    # active set of the benchmark: the models that fit the buffers at once (all of them except for the queued cfg5)
    active, tot = [], 0
    for m in models:
        if tot + m["rank"] > cfg.max_total_rank or (cfg.max_slots and len(active) >= cfg.max_slots):
            break
        active.append(m)
        tot += m["rank"]
    t_gen = time.perf_counter() - t_gen

    dev = torch.device("cuda:0")
    Td = torch.from_numpy(T).to(dev)
    torch.cuda.synchronize()
    def timed_rounds(flags):
        ctx = P.Context(max_total_rank=cfg.max_total_rank, max_slots=cfg.max_slots, flags=flags)
        ctx.submit_tensor(Td)
        for m in active:
            ctx.enqueue_model(m["init"], tol=-1.0, max_iters=W + K)   # plain ALS steps; nobody leaves before the last step
        if W > 0:
            ctx.iterate(W)
        torch.cuda.synchronize()
        s0 = ctx.stats()
        t0 = time.perf_counter()
        ctx.iterate(K)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        s1 = ctx.stats()
        res = ctx.poll_retired()
        assert len(res) == len(active) and all(r.iters == W + K for r in res), "every model must finish in the last step"
        assert s1.rounds - s0.rounds == K
        ctx.close()
        return s0, s1, t0, t1

    s0, s1, t0, t1 = timed_rounds(P.CTX_TIMING | (P.CTX_REUSE if args.reuse else 0))

    dt = t1 - t0
    flops = s1.mttkrp_flops - s0.mttkrp_flops               # algorithmic: 2 * width * prod(I) per MTTKRP
    assert abs(flops - 6.0 * tot * I1 * I2 * I3 * K) <= 1e-6 * flops
    launches = sum(s1.mttkrp_launches) - sum(s0.mttkrp_launches)
    if args.reuse:
        launches = 2 * K      # per round: the mode-1 MTTKRP and the first-step contraction, 2 * width * prod(I) flops each
    kern_ms = sum(s1.mttkrp_ms) - sum(s0.mttkrp_ms)
    per_mode_ms = [(s1.mttkrp_ms[n] - s0.mttkrp_ms[n]) / max(1, s1.mttkrp_launches[n] - s0.mttkrp_launches[n])
                   for n in range(3)]   # with --reuse: [mode-1 MTTKRP, first-step contraction, 0]
    avg_ms = kern_ms / launches
    flops_per_launch = 2.0 * tot * I1 * I2 * I3
    bytes_per_launch = 8.0 * I1 * I2 * I3 + 8.0 * tot * (I1 + I2 + I3)   # tensor once + two factor panels + output
    ai = flops_per_launch / bytes_per_launch
    if ai >= PEAK_FP64_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        achieved = flops_per_launch / (avg_ms * 1e-3) * 1e-12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP64_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_FP64_MFMA_TFLOPS}
    else:
        achieved = bytes_per_launch / (avg_ms * 1e-3) * 1e-9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS}
    roof["traffic"] = None
    # HBM bytes per MTTKRP from the rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known
    # size); counters cannot be read from inside this process, so the figure of the committed summary is reported
    tfile = os.path.join(ROOT, "profiles", "traffic.txt")
    if os.path.exists(tfile):
        for ln in open(tfile):
            parts = ln.split()
            if len(parts) == 2 and parts[0] == cfg.name:
                roof["traffic"] = float(parts[1])
                roof["traffic_from"] = "profiles/traffic.txt (stored rocprofv3 FETCH_SIZE + WRITE_SIZE run of this workload; not measured in this run)"
    roof["kernel"] = "mttkrp_kernel (fused MTTKRP contraction)"
    roof["avg_launch_ms"] = avg_ms
    roof["per_mode_ms"] = per_mode_ms

    out = {
        "metric": "fused MTTKRP fp64 GFLOP/s (% roofline); CP-ALS models completed/sec",
        "value": flops / dt * 1e-9,
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": cfg.name, "dims": list(cfg.dims), "models": len(active), "total_rank": tot,
                   "iterations_timed": K},
        "sweeps_per_s": K / dt,
        "models_per_s": len(active) / dt,
        "model_iterations_per_s": len(active) * K / dt,
        "roofline": roof,
        "setup_s": {"generate": t_gen},
    }
    if args.reuse:
        out["config"]["two_step_sweeps"] = True
    if args.workload == "cfg4" and not args.no_jobs and not args.reuse:
        # the same timed rounds with two-step sweeps (one pass over the tensor fewer per sweep); flops stay algorithmic
        _, _, r0, r1 = timed_rounds(P.CTX_REUSE)
        out["two_step_sweeps"] = {"ms_per_step": (r1 - r0) / K * 1e3, "sweeps_per_s": K / (r1 - r0),
                                  "models_per_s": len(active) / (r1 - r0),
                                  "effective_gflops": flops / (r1 - r0) * 1e-9}
    if args.workload == "cfg4" and not args.no_jobs and not args.reuse:
        # the bandwidth-bound regime on the same (HBM-resident) tensor: 16 fused columns, all three modes
        lw = mttkrp_alone(Td, tuple(cfg.dims), 16)
        lw_bytes = 8.0 * I1 * I2 * I3 + 8.0 * 16 * (I1 + I2 + I3)
        lw_ms = sum(lw["contraction_ms"]) / 3.0
        out["low_width"] = {"workload": cfg.name, "width": 16, "per_mode": lw,
                            "roofline": {"bound": "hbm", "achieved": lw_bytes / (lw_ms * 1e-3) * 1e-9, "peak": PEAK_HBM_GBS,
                                         "unit": "GB/s", "frac": lw_bytes / (lw_ms * 1e-3) * 1e-9 / PEAK_HBM_GBS,
                                         "kernel": "mttkrp_kernel (contraction launches, mean of the three modes)",
                                         "avg_launch_ms": lw_ms}}
    del Td
    torch.cuda.empty_cache()
    if args.workload == "cfg4" and not args.no_jobs:
        if args.reuse:
            out["jobs"] = [run_job(5, reuse=True)]
        else:
            legs = {cid: config_leg(cid) for cid in (1, 2, 3, 5)}
            out["jobs"] = [legs[cid]["job"] for cid in (1, 2, 3, 5)] + [legs[5]["job_two_step"]]
            out["mttkrp_by_config"] = [legs[cid]["mttkrp"] for cid in (1, 2, 3, 5)] + [legs[5]["mttkrp_full_buffer"]]
    if args.workload == "cfg4" and not args.no_jobs and not args.reuse:
        # the same model mix on an order-4 tensor of the same size (180^4): whole rounds and the fused MTTKRP per mode
        try:
            o4 = run_order_n("order4", min(K, 10), W, reps=2)
            full = o4["mttkrp_alone"][-1]
            out["order_n"] = [{"workload": "order4", "dims": o4["config"]["dims"], "total_rank": o4["config"]["total_rank"],
                               "ms_per_step": o4["ms_per_step"], "gflops": o4["value"],
                               "mttkrp_ms_per_mode": full["kernel_ms"], "mttkrp_tflops_per_mode": full["kernel_tflops"]}]
        except Exception as e:          # a report line, not a reason to lose the main measurement
            out["order_n"] = [{"workload": "order4", "error": repr(e)}]
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, T, active)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
