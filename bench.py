"""Benchmark of the OSSCAR layer solver on one MI355X.

One "step" is one pass of the whole hot path over one synthetic OPT-30B-shaped fc2 layer (cfg5: X is
262144 x 28672 bf16, W is 28672 x 7168 bf16, keep 14336 neurons, 5000 swaps): Gram accumulation over all
calibration rows, finalize (ridge, G = H W), magnitude support + state build, the local search, and the
final back-solve.  X and W are resident in HBM before the timed region starts.

Prints one JSON line.  `value` is seconds per layer (lower is better).  `roofline` describes the search's
bulk update of the tableau N (the kernel the layer time is dominated by), `roofline_gram` the bf16 MFMA
Gram kernel, and `cpu_baseline` the float64 oracle timed on this machine's host cores on a reduced layer of
the same recipe."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def gen_on_gpu(inp, torch, cfg, dev, rows_per=4096):
    X = torch.empty(cfg.n, cfg.d1, dtype=inp.torch_dtype(cfg.x_dtype), device=dev)
    for r0 in range(0, cfg.n, rows_per):
        nr = min(rows_per, cfg.n - r0)
        X[r0:r0 + nr] = inp.gen_X(cfg, r0, nr, device=dev)
    return X


def cpu_baseline(inp, cfg_full):
    """The oracle as it stands on a reduced layer (same recipe), projected to the full layer by work ratios."""
    import numpy as np
    from oracle import osscar_oracle as orc
    p, m, n, k, swaps = 4096, 1024, 16384, 2048, 24
    cfg = inp.scaled(cfg_full, p=p, m=m, n=n, k=k, swaps=swaps)
    X = inp.gen_X(cfg).double().numpy()
    W = inp.gen_W(cfg).double().numpy()
    t0 = time.perf_counter()
    H, G, c0, lam = orc.gram(X, W, cfg.lam_abs, cfg.lam_rel)
    t_gram = time.perf_counter() - t0
    K0 = orc.magnitude_support(W, cfg.p, cfg.q, cfg.k)
    t0 = time.perf_counter()
    orc.init_state(H, G, K0, cfg.q)
    t_init = time.perf_counter() - t0
    t0 = time.perf_counter()
    res = orc.local_search(H, G, c0, K0, cfg.p, cfg.q, swaps)
    t_search = time.perf_counter() - t0 - t_init          # local_search builds its own initial state
    t0 = time.perf_counter()
    orc.solve_support(H, G, c0, res.support, cfg.q)
    t_back = time.perf_counter() - t0
    f = cfg_full
    r_gram = (f.n * f.d1 ** 2) / (n * p ** 2)
    r_cube = ((f.k * f.q) / k) ** 3
    per_iter = t_search / max(res.iters, 1)
    projected = t_gram * r_gram + (t_init + t_back) * r_cube + per_iter * r_cube * f.swaps
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        pass
    return {"value": projected, "unit": "s", "cores": cores, "kind": "oracle",
            "sample": (f"float64 numpy oracle on the cfg5 recipe reduced to p={p}, m={m}, n={n}, k={k}, {res.iters} swap "
                       f"iterations: gram {t_gram:.2f}s, init {t_init:.2f}s, search {t_search:.2f}s, backsolve {t_back:.2f}s "
                       f"measured; projected to the full layer by work ratios (gram x{r_gram:.0f}, cubic phases x{r_cube:.0f}, "
                       f"{f.swaps} swaps)"),
            "measured_s": t_gram + t_init + t_search + t_back}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--swaps", type=int, default=None)
    ap.add_argument("--refresh-every", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one MI355X: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import osscar_inputs as inp
    import paper_2403_12983_amd as pkg

    cfg = inp.CONFIGS[a.config]
    swaps = cfg.swaps if a.swaps is None else a.swaps
    dev = "cuda:0"
    X = gen_on_gpu(inp, torch, cfg, dev)
    W = inp.gen_W(cfg, dev)
    s = pkg.Solver(cfg.d1, cfg.m, cfg.p, cfg.q, cfg.k, max(swaps, 1), X.dtype, W.dtype, dev)
    torch.cuda.synchronize()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    phases = {k: 0.0 for k in ("gram", "finalize", "init", "search", "backsolve")}
    upd_n = upd_z = 0.0
    info = {}

    def step(timed):
        nonlocal upd_n, upd_z
        ev[0].record()
        s.osscar_gram(X, False)
        ev[1].record()
        s.osscar_gram(None, True, W, cfg.lam_abs, cfg.lam_rel)
        ev[2].record()
        obj0 = s.osscar_init_support()
        ev[3].record()
        r = s.osscar_local_search(swaps, 0.0, 0, a.refresh_every)
        ev[4].record()
        What, support, obj = s.osscar_backsolve()
        ev[5].record()
        torch.cuda.synchronize()
        if timed:
            for i, k in enumerate(phases):
                phases[k] += ev[i].elapsed_time(ev[i + 1]) / 1e3
            tm = s.osscar_get_timers()
            upd_n += tm[5] / 1e3
            upd_z += tm[7] / 1e3
        info.update(obj0=obj0, obj=obj, iters=r["iters"], accepted=r["accepted"], tracked=r["obj_final"])

    for _ in range(a.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    K = max(a.steps, 1)
    for k in phases:
        phases[k] /= K
    upd_n /= K
    upd_z /= K
    t_layer = wall / K

    d1, m, n = cfg.d1, cfg.m, cfg.n
    bytes_n = 2 * 4 * (d1 * d1 // 2)           # read + write of the lower triangle of N (= P and V of the kept-set view)
    bytes_z = 2 * 4 * d1 * m                   # read + write of Z (= B and R)
    gram_flops = n * d1 * (d1 + 1)
    out = {
        "metric": "OPT-30B fc2 layer prune time", "value": t_layer, "unit": "s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": 1e3 * t_layer, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 inputs, f32 state, f64 accumulate", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: X {n}x{d1} {cfg.x_dtype}, W {d1}x{m} {cfg.w_dtype}, keep {cfg.k} of {cfg.p} groups "
                               f"(q={cfg.q}), {swaps} swaps, lambda = {cfg.lam_rel}*mean diag",
                   "refresh_every": a.refresh_every},
        "phases_s": phases,
        "swap_iterations": info["iters"], "accepted_swaps": info["accepted"],
        "swap_evals_per_s": info["iters"] * cfg.p / phases["search"] if phases["search"] > 0 else None,
        "ms_per_swap": 1e3 * phases["search"] / max(info["iters"], 1),
        "gram_tflops_syrk": gram_flops / phases["gram"] / 1e12,
        "gram_tflops_full_equiv": 2 * n * d1 * d1 / phases["gram"] / 1e12,
        "objective": {"initial": info["obj0"], "final": info["obj"], "tracked": info["tracked"]},
        "roofline": {"kernel": "update_N (bulk rank-2 update of the swept tableau, lower triangle)", "bound": "hbm",
                     "achieved": bytes_n / upd_n / 1e9 if upd_n > 0 else None, "peak": 8000.0, "unit": "GB/s",
                     "frac": bytes_n / upd_n / 1e9 / 8000.0 if upd_n > 0 else None, "traffic": None,
                     "bytes_per_launch": bytes_n, "ms_per_launch": 1e3 * upd_n},
        "roofline_update_Z": {"bound": "hbm", "achieved": bytes_z / upd_z / 1e9 if upd_z > 0 else None, "peak": 8000.0,
                              "unit": "GB/s", "frac": bytes_z / upd_z / 1e9 / 8000.0 if upd_z > 0 else None,
                              "bytes_per_launch": bytes_z, "ms_per_launch": 1e3 * upd_z},
        "roofline_gram": {"bound": "mfma", "achieved": gram_flops / phases["gram"] / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                          "frac": gram_flops / phases["gram"] / 1e12 / 2500.0,
                          "note": "algorithmic SYRK flops n*d1*(d1+1); the kernel issues about 2x that on diagonal tiles only"},
    }
    s.close()
    del X
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, inp.CONFIGS["cfg5"] if a.config == "cfg5" else cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
