#!/usr/bin/env python3
"""Writes tests/golden/cfg<N>_full.txt: what the CPU oracle obtains for a configuration run at FULL size, exactly as
specified (queue, slots, tolerances, iteration caps, non-negativity, line search).

Calls only oracle/ and workloads/ (never the GPU package).  The queue of the paper's full algorithm (Alg. 3: fill from
the queue front until the next model does not fit, advance every active model one iteration, remove the stopped ones
in slot order) is stepped here round by round over oracle.Model objects, so that the fit after every iteration of
every model is seen; `tests/test_oracle_pins.py` checks this loop against oracle.cals on small cases.

Per model the file holds rank, iterations, status, accepted line-search steps, fit and error (17 significant digits)
and two margins that say how close the model ever came to deciding differently:
  tol_margin  min over its stop tests of | |F - F_prev| - tol |        (in units of fit)
  ls_margin   min over its line-search decisions of |e_new - e| / ||T||^2
A model with a margin at rounding level (the fit formula cancels to about 1e-12) can legitimately take one iteration
more or less under another order of additions; the GPU test names such models and prints their margins.
For fixed-iteration configurations (negative tolerance) the per-iteration fits of a few sampled models and sampled
entries of their final factors are stored as well.

  python tests/golden/make_full_config_goldens.py --cfg 5 [--threads 8]
"""
from __future__ import annotations

import argparse
import hashlib
import math
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle as O                                                    # noqa: E402
from workloads import get_config, make_models, make_tensor           # noqa: E402


def input_hash(T: np.ndarray, models) -> str:
    """sha256 over the tensor's bytes and every starting factor's bytes (column-major), in order."""
    h = hashlib.sha256()
    flat = T.reshape(-1)
    step = 1 << 24
    for i in range(0, flat.size, step):
        h.update(flat[i:i + step].tobytes())
    for m in models:
        for u in m["init"]:
            h.update(np.asfortranarray(u).tobytes(order="F"))
    return h.hexdigest()


def lockstep(T, models, max_total_rank, max_slots, threads, only=None, progress=None):
    """Alg. 3 over oracle.Model objects.  `only`: when given, the ids of the models that are actually advanced (the
    others are skipped entirely: allowed only when every model runs a fixed number of iterations and all fit at once,
    so that nobody's schedule depends on anybody else).  Returns (per-model records, retirement order, rounds)."""
    normT2 = O.norm_sq(T)
    n = len(models)
    rec = [None] * n
    order, active, rtot, nxt, rounds = [], [], 0, 0, 0
    pool = ThreadPoolExecutor(max_workers=threads)

    def advance(entry):
        k, mdl, r = entry
        status = mdl.iterate()
        s = mdl.state(factors=False)
        tol = models[k]["tol"]
        if s["iters"] >= 2 and tol >= 0.0 and status != O.NUMERICAL:
            r["tol_margin"] = min(r["tol_margin"], abs(abs(s["fit"] - r["fit_prev"]) - tol))
        ea, en = mdl.last_ls_errors()
        if (models[k]["flags"] & O.FLAG_LINESEARCH) and s["iters"] >= 2 and not math.isnan(en):
            r["ls_margin"] = min(r["ls_margin"], abs(en - ea) / normT2)
        r["fit_prev"] = s["fit"]
        r["fits"].append(s["fit"])
        return status

    while nxt < n or active:
        while nxt < n:
            r = models[nxt]["rank"]
            if rtot + r > max_total_rank or (max_slots > 0 and len(active) >= max_slots):
                break
            m = models[nxt]
            mdl = None
            if only is None or nxt in only:
                mdl = O.Model(T, m["init"], m["tol"], m["max_iters"], m["flags"], m["ls_alpha"], normT2=normT2)
            active.append((nxt, mdl, dict(tol_margin=math.inf, ls_margin=math.inf, fit_prev=0.0, fits=[], left=m["max_iters"])))
            rtot += r
            nxt += 1
        live = [e for e in active if e[1] is not None]
        statuses = dict(zip([e[0] for e in live], pool.map(advance, live)))
        keep = []
        for e in active:
            k, mdl, r = e
            if mdl is None:
                r["left"] -= 1
                stopped = r["left"] == 0
            else:
                stopped = statuses[k] != O.RUNNING
            if stopped:
                order.append(k)
                rtot -= models[k]["rank"]
                if mdl is not None:
                    s = mdl.state(factors=True)
                    s.update(tol_margin=r["tol_margin"], ls_margin=r["ls_margin"], fits=r["fits"])
                    rec[k] = s
            else:
                keep.append(e)
        active = keep
        rounds += 1
        if progress:
            progress(rounds, len(order), rtot)
    pool.shutdown()
    return rec, order, rounds, normT2


def fmt(x: float) -> str:
    return "inf" if math.isinf(x) else "%.17g" % x


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfg", type=int, required=True)
    ap.add_argument("--threads", type=int, default=max(1, (os.cpu_count() or 8)))
    ap.add_argument("--sample", default="", help="fixed-iteration configurations: comma-separated model ids to follow")
    ap.add_argument("--entries", type=int, default=48, help="sampled factor entries stored per followed model and mode")
    ap.add_argument("--factors", action="store_true",
                    help="queue configurations: also store lambda and --entries sampled factor entries per mode of EVERY model")
    ap.add_argument("--out", default="")
    a = ap.parse_args()
    cfg = get_config(a.cfg)
    t0 = time.time()
    T = make_tensor(cfg, threads=a.threads)
    models = make_models(cfg)
    digest = input_hash(T, models)
    print("cfg %d: tensor and %d starts ready (%.0f s), sha256 %s" % (a.cfg, len(models), time.time() - t0, digest), flush=True)
    only = None
    if a.sample:
        assert cfg.tol < 0 and cfg.total_rank <= cfg.max_total_rank and cfg.max_slots == 0
        only = set(int(x) for x in a.sample.split(","))

    def progress(rounds, done, rtot):
        if rounds % 10 == 0 or done == len(models):
            print("  round %d: %d of %d models done, width %d, %.0f s" % (rounds, done, len(models), rtot, time.time() - t0), flush=True)

    rec, order, rounds, normT2 = lockstep(T, models, cfg.max_total_rank, cfg.max_slots, a.threads, only, progress)
    out = a.out or os.path.join(HERE, "cfg%d_full.txt" % a.cfg)
    rng = np.random.default_rng(7000 + a.cfg)
    with open(out, "w") as f:
        f.write("# Configuration %d at full size, as specified, run by the CPU oracle (lock-step queue of Alg. 3).\n" % a.cfg)
        f.write("# Written by tests/golden/make_full_config_goldens.py --cfg %d%s%s; calls only oracle/ and workloads/.\n"
                % (a.cfg, (" --sample " + a.sample) if a.sample else "", (" --factors --entries %d" % a.entries) if a.factors else ""))
        f.write("# model lines: id rank iters status ls_accepted fit error tol_margin ls_margin\n")
        f.write("input_sha256 %s\n" % digest)
        f.write("norm_sq %s\n" % fmt(normT2))
        f.write("rounds %d\n" % rounds)
        f.write("order %s\n" % " ".join(str(k) for k in order))
        for k, r in enumerate(rec):
            if r is None:
                continue
            f.write("model %d %d %d %d %d %s %s %s %s\n" % (k, models[k]["rank"], r["iters"], r["status"], r["ls_accepted"],
                                                           fmt(r["fit"]), fmt(r["err"]), fmt(r["tol_margin"]), fmt(r["ls_margin"])))
            if only is not None:
                f.write("fits %d %s\n" % (k, " ".join(fmt(x) for x in r["fits"])))
            if only is not None or a.factors:
                f.write("lambda %d %s\n" % (k, " ".join(fmt(x) for x in r["lam"])))
                for n, U in enumerate(r["U"]):
                    rows = rng.integers(0, U.shape[0], a.entries)
                    cols = rng.integers(0, U.shape[1], a.entries)
                    f.write("entries %d %d %s\n" % (k, n, " ".join("%d,%d,%s" % (i, c, fmt(U[i, c])) for i, c in zip(rows, cols))))
    print("wrote %s (%d rounds, %.0f s)" % (out, rounds, time.time() - t0), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
