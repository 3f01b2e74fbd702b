"""Benchmark of the OSSCAR layer solver on one MI355X.

One "step" is one pass of the whole hot path over one synthetic OPT-30B-shaped fc2 layer (cfg5: X is
262144 x 28672 bf16, W is 28672 x 7168 bf16, keep 14336 neurons, 5000 swaps): Gram accumulation over all
calibration rows, finalize (ridge, G = H W), magnitude support + state build, the local search, and the
final back-solve.  X and W are resident in HBM before the timed region starts.

Prints one JSON line.  `value` is seconds per layer (lower is better).  `roofline` describes the kernel the
layer time is dominated by, the float64-accumulating MFMA GEMM, on its largest launch (V = P H_{K,Kc}).
`roofline_gram` describes the bf16 MFMA Gram kernel, and `cpu_baseline` the float64 oracle timed on this
box's host cores on a reduced layer of the same recipe."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
GEMM_TRAFFIC_CFG5 = 40.53e9   # bytes; see profiles/gemm_f64acc_cfg5_pmc.md
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
    p, m, n, k, swaps = 4096, 1024, 16384, 2048, 48     # about 15 s of host work
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
    ap.add_argument("--init", choices=("magnitude", "greedy"), default="magnitude",
                    help="magnitude: the benchmark layer's recipe (magnitude support, then swaps); greedy: the nested "
                         "schedule of Algorithm 1 from the dense layer (t-hat groups pruned per iteration), then swaps")
    ap.add_argument("--t-hat", type=int, default=10)
    ap.add_argument("--block", type=int, default=1,
                    help="groups swapped per iteration (t-hat = 2 * block): swaps // block iterations of block moves")
    ap.add_argument("--no-lookahead", action="store_true",
                    help="search without the products computed ahead: every swap then makes one read-only pass over Z")
    ap.add_argument("--exact-in", action="store_true",
                    help="entering group by the exact gain of the pair (OSSCAR_SEARCH_EXACT_IN); runs on the in-place path")
    ap.add_argument("--rows", type=int, default=None,
                    help="calibration rows (default: the config's); a short X keeps counter-collection runs brief")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="end with one 1 GiB device-to-device copy, the known-size kernel that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one MI355X: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import osscar_inputs as inp
    import paper_2403_12983_amd as pkg

    cfg = inp.CONFIGS[a.config]
    if a.rows is not None:
        cfg = cfg.replace(n=a.rows)
    swaps = cfg.swaps if a.swaps is None else a.swaps
    dev = "cuda:0"
    X = gen_on_gpu(inp, torch, cfg, dev)
    W = inp.gen_W(cfg, dev)
    s = pkg.Solver(cfg.d1, cfg.m, cfg.p, cfg.q, cfg.k, max(swaps, 1), X.dtype, W.dtype, dev, from_dense=(a.init == "greedy"))
    torch.cuda.synchronize()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    phases = {k: 0.0 for k in ("gram", "finalize", "init", "search", "backsolve")}
    upd_n = upd_z = gemm_ms = gemm32_ms = flush_ms = 0.0
    info = {}

    def step(timed):
        nonlocal upd_n, upd_z, gemm_ms, gemm32_ms, flush_ms
        ev[0].record()
        s.osscar_gram(X, False)
        ev[1].record()
        s.osscar_gram(None, True, W, cfg.lam_abs, cfg.lam_rel)
        ev[2].record()
        obj0 = s.osscar_init_support() if a.init == "magnitude" else s.osscar_init_greedy(a.t_hat)[0]
        ev[3].record()
        fl = pkg.OSSCAR_SEARCH_NO_LOOKAHEAD if a.no_lookahead else 0
        if a.exact_in:
            fl |= pkg.OSSCAR_SEARCH_EXACT_IN
        if a.block > 1:
            r = s.osscar_block_search(swaps // a.block, a.block, 0.0, fl)
            r["iters"] = r["iters"] * a.block
        else:
            r = s.osscar_local_search(swaps, 0.0, fl, a.refresh_every)
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
            gemm_ms += tm[9]
            gemm32_ms += tm[10]
            flush_ms += tm[6]
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
    gemm_ms /= K
    gemm32_ms /= K
    flush_ms /= K
    t_layer = wall / K

    d1, m, n = cfg.d1, cfg.m, cfg.n
    gram_flops = n * d1 * (d1 + 1)
    lazy = (cfg.q == 1) and not a.exact_in
    # Per-swap state update of an in-place search (Proposition 4.1): read + write of P, V (= lower triangle of N) and B, R (= Z)
    bytes_swap_alg = 2 * 4 * (d1 * d1 // 2) + 2 * 4 * d1 * m
    ms_swap = 1e3 * phases["search"] / max(info["iters"], 1)
    # Dominant kernel of the layer: the float64-accumulating MFMA GEMM (the inverse's refinement, B, V, S, R, the look-ahead
    # products of the search, the back-solve's residual).  Its largest launch, V = P H_{K,Kc} in the state build, is timed by
    # HIP events on the library's stream (timer slot 9): 2 kr^2 cr flops on v_mfma_f64_16x16x4_f64.
    kr, cr = cfg.k * cfg.q, d1 - cfg.k * cfg.q
    n_inv = d1 if a.init == "greedy" else kr       # order of the matrix the support initialisation inverts
    g_flops = 2.0 * kr * kr * cr
    g_bytes = 4.0 * (kr * kr + 2 * kr * cr)                      # read P and H_{K,Kc} once, write V once
    # HBM bytes of that launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/gemm_f64acc_cfg5_pmc.md), cfg5 only
    g_traffic = GEMM_TRAFFIC_CFG5 if a.config == "cfg5" else None
    out = {
        "metric": "OPT-30B fc2 layer prune time", "value": t_layer, "unit": "s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": 1e3 * t_layer, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 inputs, f32 state, f64 accumulate", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: X {n}x{d1} {cfg.x_dtype}, W {d1}x{m} {cfg.w_dtype}, keep {cfg.k} of {cfg.p} groups "
                               f"(q={cfg.q}), {swaps} swaps, lambda = {cfg.lam_rel}*mean diag",
                   "refresh_every": a.refresh_every,
                   "search": (("delayed-update" + (", no look-ahead" if a.no_lookahead else "")) if lazy else "eager") +
                             (", exact entering rule" if a.exact_in else ""),
                   "init": a.init if a.init == "magnitude" else f"nested schedule from the dense layer, t_hat = {a.t_hat}",
                   "groups_per_move": a.block},
        "phases_s": phases,
        "swap_iterations": info["iters"], "accepted_swaps": info["accepted"],
        "swap_evals_per_s": info["iters"] * cfg.p / phases["search"] if phases["search"] > 0 else None,
        "ms_per_swap": ms_swap,
        "gram_tflops_syrk": gram_flops / phases["gram"] / 1e12,
        "gram_tflops_full_equiv": 2 * n * d1 * d1 / phases["gram"] / 1e12,
        "objective": {"initial": info["obj0"], "final": info["obj"], "tracked": info["tracked"]},
        "roofline": {"kernel": "gemm_f64acc_kernel<float>, launch V = P H_{K,Kc} (float32 operands, float64 MFMA accumulation)",
                     "bound": "mfma", "achieved": g_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else None, "peak": 78.6,
                     "unit": "TFLOP/s", "frac": g_flops / (gemm_ms * 1e-3) / 1e12 / 78.6 if gemm_ms > 0 else None,
                     "traffic": g_traffic, "flops_per_launch": g_flops, "algorithmic_bytes_per_launch": g_bytes,
                     "ms_per_launch": gemm_ms if gemm_ms > 0 else None},
        # The float32-accumulating MFMA GEMM (v_mfma_f32_32x32x2_f32: flushes of the search, sweeps of the inverse, small
        # corrections) takes about as long per layer as the float64-accumulating one; its largest launch is the lower triangle
        # of P (I - H_KK P) in the Newton-Schulz step: kr^3 flops (timer slot 10).
        "roofline_gemm_f32acc": {"kernel": "gemm_f32acc_kernel<false>, launch tril(P (I - H_KK P))", "bound": "mfma",
                                 "achieved": float(n_inv) ** 3 / (gemm32_ms * 1e-3) / 1e12 if gemm32_ms > 0 else None,
                                 "peak": 157.3, "unit": "TFLOP/s",
                                 "frac": float(n_inv) ** 3 / (gemm32_ms * 1e-3) / 1e12 / 157.3 if gemm32_ms > 0 else None,
                                 "ms_per_launch": gemm32_ms},
        "roofline_gram": {"kernel": "gram_packed_kernel (+ gram_pack_kernel, whole Gram phase)", "bound": "mfma",
                          "achieved": gram_flops / phases["gram"] / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                          "frac": gram_flops / phases["gram"] / 1e12 / 2500.0,
                          "note": "algorithmic SYRK flops n*d1*(d1+1); the kernel issues 2x that on diagonal tiles only"},
        "search_iteration": ({"note": "per swap: four small kernels (selection and pivot algebra; current pivot rows/columns and w from the "
                                      "products computed ahead; acceptance test and u; update of norms/diagonal/scores); every 64 swaps a flush by matrix "
                                      "products plus one look-ahead product Zc Z^T.  An eager in-place up/downdate of P, B, V, R would "
                                      "move bytes_per_swap_eager per swap",
                              "ms_per_swap": ms_swap, "accept_and_u_kernel_ms": 1e3 * upd_n, "iteration_kernels_ms": 1e3 * upd_z,
                              "flushes_total_ms": flush_ms, "bytes_per_swap_eager": bytes_swap_alg,
                              "eager_equivalent_GBps": bytes_swap_alg / ms_swap / 1e6} if lazy else
                             {"note": "in-place search: every swap is one rank-2q pass over the tableau (N: lower triangle, Z)",
                              "ms_per_swap": ms_swap, "update_N_ms": 1e3 * upd_n, "update_Z_ms": 1e3 * upd_z,
                              "bytes_per_swap": bytes_swap_alg,
                              "update_GBps": bytes_swap_alg / max(upd_n + upd_z, 1e-12) / 1e9}),
    }
    s.close()
    del X
    if a.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, inp.CONFIGS["cfg5"] if a.config == "cfg5" else cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
