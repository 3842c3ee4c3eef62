"""Runs the oracle's timeline trainer in child processes, one per "leg" (the fp64 reference and the
precision stand-ins of tests/precision_standins.py), so that the minutes-long oracle runs of the
full-size parity tests overlap.  The children are spawned (never forked: the parent holds a GPU
context), import only numpy and the oracle, and hand their parameters back through .npy files."""
from __future__ import annotations

import multiprocessing as mp
import os
import shutil
import tempfile
import time
from types import SimpleNamespace

import numpy as np


def _leg(args):
    name, N, leg, rule, T, seed, kw, threads, out_dir = args
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    for p in (os.path.dirname(here), here):
        if p not in sys.path:
            sys.path.insert(0, p)
    import conftest  # noqa: F401  (allocator setting)
    from threadpoolctl import threadpool_limits
    import cdp_workloads as wl
    from oracle import cdp_oracle as O
    import precision_standins as PS
    cfg = wl.get_config(name)
    if N is not None:
        cfg.N = N
    impl = {"fp64": None, "bf16": PS.Bf16Storage, "fp32": PS.Fp32Accumulation(seed + 1)}[leg]
    xs, ys = wl.make_data(cfg, T, seed)
    p0 = wl.init_params(cfg, seed)
    t0 = time.time()
    with threadpool_limits(limits=threads):
        r = O.train_schedule(cfg, p0, xs, ys, rule, keep_versions=False, stage_impl=impl, **kw)
    shapes = []
    for j, st in enumerate(r.params):
        for k, a in enumerate(st):
            np.save(os.path.join(out_dir, "%s_%d_%d.npy" % (leg, j, k)), np.asarray(a, dtype=np.float64))
        shapes.append(len(st))
    return leg, shapes, r.losses, r.trace, r.live_inputs, time.time() - t0


def run_legs(cfg, rule, T, seed, kw, legs, heartbeat=None):
    """{leg: SimpleNamespace(params, losses, trace, live_inputs, seconds)} for legs out of
    "fp64", "bf16", "fp32"; cfg must be wl.get_config(cfg.name) up to its N.  heartbeat(seconds) is
    called every 30 s while the children work."""
    cores = min(16, os.cpu_count() or 1)
    threads = max(1, cores // len(legs))
    out_dir = tempfile.mkdtemp(prefix="cdp_oracle_")
    try:
        jobs = [(cfg.name, cfg.N, leg, rule, T, seed, kw, threads, out_dir) for leg in legs]
        if len(legs) == 1:
            results = [_leg(jobs[0])]
        else:
            with mp.get_context("spawn").Pool(len(legs)) as pool:
                pending = pool.map_async(_leg, jobs)
                t0 = time.time()
                while not pending.ready():
                    pending.wait(30.0)
                    if heartbeat is not None and not pending.ready():
                        heartbeat(time.time() - t0)
                results = pending.get()
        out = {}
        for leg, shapes, losses, trace, live, secs in results:
            params = [[np.load(os.path.join(out_dir, "%s_%d_%d.npy" % (leg, j, k))) for k in range(n)] for j, n in enumerate(shapes)]
            out[leg] = SimpleNamespace(params=params, losses=losses, trace=trace, live_inputs=live, seconds=secs)
        return out
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)
