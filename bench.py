"""Benchmark of the OSSCAR layer solver on one MI355X.

One "step" is one pass of the whole hot path over one synthetic OPT-30B-shaped fc2 layer (cfg5: X is
262144 x 28672 bf16, W is 28672 x 7168 bf16, keep 14336 neurons, 5000 swaps): Gram accumulation over all
calibration rows, finalize (ridge, G = H W), magnitude support + state build, the local search, and the
final back-solve.  X and W are resident in HBM before the timed region starts.

Prints one JSON line.  `value` is seconds per layer (lower is better).  `roofline` describes the kernel with the
largest share of the layer time, the bf16 MFMA Gram kernel: algorithmic SYRK flops of one launch (16384 calibration
rows) over the mean launch duration, measured by HIP events on the library's stream inside the timed steps.
`roofline_gemm_f64acc`, `roofline_gemm_int8` and `roofline_gemm_f32acc` give the three matrix-product kernels of the state
build and the back-solve: total algorithmic flops / total time over ALL their launches of the timed steps (the library
brackets every launch with HIP events on its own stream), and for the first its largest launch.  `cpu_baseline` is the
float64 oracle timed on this machine's host cores on a reduced layer of the same recipe: `value` is what the clock measured
on that reduced layer; the projection to the full layer is a separate, labelled key."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
# HBM-side bytes per launch on cfg5 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy
# (profiles/gemm_f64acc_cfg5_pmc.md: mean over the launches of one layer; profiles/gram_packed_cfg5_pmc.md: one chunk)
GEMM64_TRAFFIC_CFG5 = 2.99e7
GRAM_TRAFFIC_CFG5 = 93.9e9
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def gen_on_gpu(inp, torch, cfg, dev, rows_per=4096):
    X = torch.empty(cfg.n, cfg.d1, dtype=inp.torch_dtype(cfg.x_dtype), device=dev)
    for r0 in range(0, cfg.n, rows_per):
        nr = min(rows_per, cfg.n - r0)
        X[r0:r0 + nr] = inp.gen_X(cfg, r0, nr, device=dev)
    return X


def cpu_baseline(inp, cfg_full):
    """The oracle as it stands, timed on a reduced layer of the same recipe (the full layer would take the host days: one
    oracle iteration at d1 = 28672 is a minute of float64 matrix products, and there are 5000).  value = measured seconds."""
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
    measured = t_gram + t_init + t_search + t_back
    return {"value": measured, "unit": "s", "cores": cores, "kind": "oracle",
            "sample": (f"the float64 oracle (numpy with its BLAS / LAPACK, {cores} threads) on ONE reduced layer of the "
                       f"{cfg_full.name} recipe: p={p}, m={m}, n={n}, k={k}, {res.iters} swap iterations; measured gram {t_gram:.2f} s, "
                       f"state {t_init:.2f} s, search {t_search:.2f} s, final solve {t_back:.2f} s.  This is the whole-layer path on "
                       f"a layer with 1/{f.d1 // p} of the rows of W and {res.iters} of {f.swaps} swaps, not the full layer"),
            "reduced_layer": {"p": p, "m": m, "n": n, "k": k, "swaps": res.iters},
            "projected_full_layer_s": projected,
            "projection": (f"NOT measured: reduced-layer phases scaled by work ratios (gram x{r_gram:.0f}, cubic phases "
                           f"x{r_cube:.0f}, per-iteration cost x{r_cube:.0f} for {f.swaps} swaps)")}


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
    ap.add_argument("--eager", action="store_true",
                    help="in-place search (OSSCAR_SEARCH_EAGER): one rank-2 pass over the whole state per swap, the HBM-bound form")
    ap.add_argument("--gemm-table", default=None,
                    help="write the per-shape table of the general matrix-product launches of one layer (markdown) to this file")
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
    upd_n = upd_z = gemm_ms = gemm32_ms = flush_ms = gram_launch_ms = cand_ms = 0.0
    info = {}

    def step(timed):
        nonlocal upd_n, upd_z, gemm_ms, gemm32_ms, flush_ms, gram_launch_ms, cand_ms
        ev[0].record()
        s.osscar_gram(X, False)
        ev[1].record()
        s.osscar_gram(None, True, W, cfg.lam_abs, cfg.lam_rel)
        ev[2].record()
        obj0 = s.osscar_init_support() if a.init == "magnitude" else s.osscar_init_greedy(a.t_hat)[0]
        ev[3].record()
        fl = pkg.OSSCAR_SEARCH_NO_LOOKAHEAD if a.no_lookahead else 0
        if a.eager:
            fl |= pkg.OSSCAR_SEARCH_EAGER
        if a.exact_in:
            fl |= pkg.OSSCAR_SEARCH_EXACT_IN
        if a.block > 1:
            r = s.osscar_block_search(swaps // a.block, a.block, 0.0, fl)
            r["iters"] = r["iters"] * a.block
        else:
            r = s.osscar_local_search(swaps, 0.0, fl, a.refresh_every)
            info["counters"] = s.osscar_get_counters()
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
            gram_launch_ms += tm[13]
            cand_ms += tm[12]
        info.update(obj0=obj0, obj=obj, iters=r["iters"], accepted=r["accepted"], tracked=r["obj_final"])

    from paper_2403_12983_amd import binding as B
    for _ in range(a.warmup):
        step(False)
    torch.cuda.synchronize()
    B.gemm_log(True)            # two event records around every general matrix product of the timed steps
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
    gram_launch_ms /= K
    cand_ms /= K
    t_layer = wall / K

    log = B.gemm_log_read()     # every general matrix product of the timed steps: shape, kind, duration
    B.gemm_log(False)

    def weighted(rows):
        """time-weighted rate over launches: total flops / total time (lower-triangle launches count half the square)"""
        fl_ = sum(2.0 * r[0] * r[1] * r[2] * (0.5 if int(r[3]) & 4 else 1.0) for r in rows)
        ms_ = sum(r[4] for r in rows if r[4] > 0)
        return (fl_ / (ms_ * 1e-3) / 1e12 if ms_ > 0 else None), ms_, len(rows)
    w64, ms64, n64 = weighted([r for r in log if not int(r[3]) & 17])
    w32, ms32, n32 = weighted([r for r in log if int(r[3]) & 1])
    w8, ms8, n8 = weighted([r for r in log if int(r[3]) & 16])          # int8-digit products (packing included in the duration)
    ms64, ms32, ms8, n64, n32, n8 = ms64 / K, ms32 / K, ms8 / K, n64 / K, n32 / K, n8 / K          # per layer
    if a.gemm_table:
        groups = {}
        for r in log:
            key = (int(r[0]), int(r[1]), int(r[2]), int(r[3]))
            g = groups.setdefault(key, [0, 0.0])
            g[0] += 1
            g[1] += r[4]
        with open(a.gemm_table, "w") as f:
            f.write(f"launches of {K} layer(s); count and total ms are per layer\n\n")
            f.write("| M | N | K | accumulate | output | tiles | count | total ms | ms per launch | TFLOP/s | fraction of that pipe's peak |\n|---|---|---|---|---|---|---|---|---|---|---|\n")
            for (M_, N_, K_, kind), (cnt, ms_) in sorted(groups.items(), key=lambda kv: -kv[1][1]):
                fl_ = 2.0 * M_ * N_ * K_ * (0.5 if kind & 4 else 1.0) * cnt
                tf = fl_ / (ms_ * 1e-3) / 1e12 if ms_ > 0 else 0.0
                peak = 157.3 if kind & 1 else 78.6
                if kind & 16:       # fifteen int8 products per float product, against the 5.0 POP/s int8 peak
                    f.write(f"| {M_} | {N_} | {K_} | int8 digits | float32 | {'lower triangle' if kind & 4 else 'all'} | {cnt / K:g} | "
                            f"{ms_ / K:.3f} | {ms_ / cnt:.4f} | {tf:.1f} | {15 * tf / 5000.0:.3f} of the int8 peak |\n")
                    continue
                f.write(f"| {M_} | {N_} | {K_} | {'float32' if kind & 1 else 'float64'} | {'float64' if kind & 2 else 'float32'} | "
                        f"{'lower triangle' if kind & 4 else 'all'} | {cnt / K:g} | {ms_ / K:.3f} | {ms_ / cnt:.4f} | {tf:.1f} | {tf / peak:.3f} |\n")
            f.write(f"\nfloat64-accumulating kernel: {n64} launches, {ms64:.1f} ms, time-weighted {w64 or 0:.1f} TFLOP/s = {(w64 or 0) / 78.6:.3f} of 78.6\n")
            f.write(f"float32-accumulating kernel: {n32} launches, {ms32:.1f} ms, time-weighted {w32 or 0:.1f} TFLOP/s = {(w32 or 0) / 157.3:.3f} of 157.3\n")
            f.write(f"int8-digit products: {n8} launches, {ms8:.1f} ms, time-weighted {w8 or 0:.1f} TFLOP/s of float products = "
                    f"{15 * (w8 or 0) / 1000.0:.2f} POP/s on the int8 pipe = {15 * (w8 or 0) / 5000.0:.3f} of 5.0\n")

    d1, m, n = cfg.d1, cfg.m, cfg.n
    gram_flops = n * d1 * (d1 + 1)
    lazy = (cfg.q == 1) and not a.exact_in and not a.eager
    # Per-swap state update of an in-place search (Proposition 4.1): read + write of P, V (= lower triangle of N) and B, R (= Z)
    bytes_swap_alg = 2 * 4 * (d1 * d1 // 2) + 2 * 4 * d1 * m
    ms_swap = 1e3 * phases["search"] / max(info["iters"], 1)
    # Dominant kernel of the layer: the bf16 MFMA Gram kernel (Gram phase, G = H W, and the six-product forms of the state
    # build's products).  Unit of the roofline: one launch of the Gram phase = one chunk of up to 16384 calibration rows,
    # algorithmic SYRK flops rows * d1 * (d1 + 1) (the lower block triangle), duration = mean over the launches of the timed
    # steps, bracketed by HIP events on the library's stream (timer slot 13).
    kr, cr = cfg.k * cfg.q, d1 - cfg.k * cfg.q
    n_inv = d1 if a.init == "greedy" else kr       # order of the matrix the support initialisation inverts
    rows_per_launch = min(16384, n)
    gl_flops = float(rows_per_launch) * d1 * (d1 + 1)
    gl_bytes = 2.0 * rows_per_launch * d1 + 8.0 * d1 * (d1 + 1)       # the packed chunk read once; the float64 lower triangle read and written
    gram_traffic = GRAM_TRAFFIC_CFG5 if (a.config == "cfg5" and a.rows is None) else None
    # the inverse by the float64 sweep (timer slot 9): n / 128 rank-128 updates of the lower triangle, n^3 flops in all,
    # each reading and writing the 8-byte triangle once
    inv_flops = float(n_inv) ** 3
    inv_bytes = 2.0 * 8.0 * (n_inv * (n_inv + 128) / 2.0) * ((n_inv + 127) // 128)
    # mean algorithmic bytes of a float64-accumulating launch: A and B read once, C written once (float32; 8 bytes for a float64 output)
    rows64 = [r for r in log if not int(r[3]) & 17]
    big64 = None
    if rows64:
        rb_ = max(rows64, key=lambda r: r[0] * r[1] * r[2])
        same = [r for r in rows64 if (r[0], r[1], r[2], r[3]) == (rb_[0], rb_[1], rb_[2], rb_[3]) and r[4] > 0]
        fl_ = 2.0 * rb_[0] * rb_[1] * rb_[2] * (0.5 if int(rb_[3]) & 4 else 1.0)
        ms_ = sum(r[4] for r in same) / max(len(same), 1)
        big64 = {"what": f"{int(rb_[0])} x {int(rb_[1])} x {int(rb_[2])}", "flops": fl_,
                 "ms": ms_ if ms_ > 0 else None, "achieved": fl_ / (ms_ * 1e-3) / 1e12 if ms_ > 0 else None,
                 "frac": fl_ / (ms_ * 1e-3) / 1e12 / 78.6 if ms_ > 0 else None}
    alg64 = (sum(4.0 * (r[0] * r[2] + r[2] * r[1]) + (8.0 if int(r[3]) & 2 else 4.0) * r[0] * r[1] * (0.5 if int(r[3]) & 4 else 1.0)
                 for r in rows64) / len(rows64)) if rows64 else None
    out = {
        "metric": "OPT-30B fc2 layer prune time", "value": t_layer, "unit": "s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": 1e3 * t_layer, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
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
        # Largest share of the layer time: the bf16 MFMA Gram kernel.  Unit of the roofline: one launch = one chunk of up to 16384
        # calibration rows: algorithmic SYRK flops rows * d1 * (d1 + 1) (the lower block triangle) over the mean duration of the
        # launches of the timed steps, each bracketed by HIP events on the library's stream (timer slot 13).
        "roofline": {"kernel": "gram_packed_kernel (bf16 MFMA SYRK on the lower block triangle), one launch = one chunk of "
                               f"{rows_per_launch} calibration rows",
                     "bound": "mfma", "achieved": gl_flops / (gram_launch_ms * 1e-3) / 1e12 if gram_launch_ms > 0 else None,
                     "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": gl_flops / (gram_launch_ms * 1e-3) / 1e12 / 2500.0 if gram_launch_ms > 0 else None,
                     "traffic": gram_traffic, "flops_per_launch": gl_flops, "algorithmic_bytes_per_launch": gl_bytes,
                     "ms_per_launch": gram_launch_ms if gram_launch_ms > 0 else None},
        # The float64-accumulating product (the residuals that refine the inverse, the weights and the back-solve; small
        # products): mean algorithmic flops per launch (2 M N K) / mean launch duration over every launch of the timed steps.
        "roofline_gemm_f64acc": {"kernel": "float32 operands, float64 MFMA accumulation: gemm_f64acc_kernel (residuals, small shapes) and "
                                           f"thin_e_kernel (E = C0 M^-1 of every flush); {n64:g} launches per layer",
                                 "bound": "mfma", "achieved": w64, "peak": 78.6, "unit": "TFLOP/s", "frac": (w64 / 78.6) if w64 else None,
                                 "traffic": GEMM64_TRAFFIC_CFG5 if (a.config == "cfg5" and a.rows is None) else None,
                                 "launches_per_layer": n64, "ms_per_layer": ms64,
                                 "flops_per_launch": (w64 * 1e12 * ms64 * 1e-3 / n64) if (w64 and n64) else None,
                                 "ms_per_launch": (ms64 / n64) if n64 else None,
                                 "algorithmic_bytes_per_launch": alg64,
                                 "largest_launch": big64},
        # The inverse of H on the kept rows: blocked sweep on a float64 copy, n / 128 panels; the rank-128 update of the 8-byte
        # lower triangle (sweep_update64_kernel) is bound by the float64 matrix cores and by the read + write of the triangle
        # alike; the duration (timer slot 9) also contains the 128 x 128 pivot inverses, one workgroup each.
        "roofline_inverse_sweep": {"kernel": "spd_inverse_f64: sweep_update64_kernel + panel kernels, order "
                                             f"{n_inv}", "ms": gemm_ms if gemm_ms > 0 else None, "flops": inv_flops,
                                   "algorithmic_bytes": inv_bytes,
                                   "TFLOPs": inv_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else None,
                                   "frac_of_fp64_mfma_peak": inv_flops / (gemm_ms * 1e-3) / 1e12 / 78.6 if gemm_ms > 0 else None,
                                   "GBps": inv_bytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else None,
                                   "frac_of_hbm_peak": inv_bytes / (gemm_ms * 1e-3) / 1e9 / 8000.0 if gemm_ms > 0 else None},
        # The state-build products B, V, S, R on the int8 matrix cores: fifteen digit products per float product, so the pipe
        # runs 15 x the float rate; durations include the scaling and cutting of both operands.
        "roofline_gemm_int8": {"kernel": "i8_gemm_kernel (+ its packing kernels): float32 operands as five 7-bit digits, exact int32 sums; "
                                         f"{n8:g} launches per layer",
                               "bound": "mfma", "achieved": (15 * w8 / 1000.0) if w8 else None, "peak": 5.0, "unit": "POP/s",
                               "frac": (15 * w8 / 5000.0) if w8 else None, "float_equivalent_TFLOPs": w8,
                               "launches_per_layer": n8, "ms_per_layer": ms8},
        # The float32-accumulating MFMA GEMM (v_mfma_f32_32x32x2_f32): only the second route of the inverse and shapes that
        # the packed kernels do not take launch it; total flops / total time over its launches of the timed steps (none on cfg5).
        "roofline_gemm_f32acc": {"kernel": "gemm_f32acc_kernel (float32 MFMA accumulation)", "bound": "mfma", "peak": 157.3, "unit": "TFLOP/s",
                                 "achieved": w32, "frac": (w32 / 157.3) if w32 else None, "launches_per_layer": n32, "ms_per_layer": ms32},
        "state_build": {"candidate_side_products_ms": cand_ms, "inverse_correction_product_ms": gemm32_ms},
        "roofline_gram_phase": {"kernel": "gram_pack_kernel + gram_packed_kernel, the whole Gram phase (repacking included)",
                                "bound": "mfma", "achieved": gram_flops / phases["gram"] / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                                "frac": gram_flops / phases["gram"] / 1e12 / 2500.0,
                                "note": "algorithmic SYRK flops n*d1*(d1+1); the kernel issues 2x that on diagonal tiles only"},
        "search_iteration": ({"note": "per swap: four small kernels (selection and pivot algebra; current pivot rows/columns and w from the "
                                      "products computed ahead; acceptance test and u; update of norms/diagonal/scores); every 64 swaps a flush by matrix "
                                      "products plus one look-ahead product Zc Z^T.  An eager in-place up/downdate of P, B, V, R would "
                                      "move bytes_per_swap_eager per swap",
                              "ms_per_swap": ms_swap, "accept_and_u_kernel_ms": 1e3 * upd_n, "iteration_kernels_ms": 1e3 * upd_z,
                              "flushes_total_ms": flush_ms, "bytes_per_swap_eager": bytes_swap_alg,
                              "last_layer_counts": info.get("counters")} if lazy else
                             {"note": "in-place search: every swap is one rank-2q pass over the tableau (N: lower triangle, Z)",
                              "ms_per_swap": ms_swap, "update_N_ms": 1e3 * upd_n, "update_Z_ms": 1e3 * upd_z,
                              "bytes_per_swap": bytes_swap_alg,
                              "update_GBps": bytes_swap_alg / max(upd_n + upd_z, 1e-12) / 1e9,
                              "frac_of_hbm_peak": bytes_swap_alg / max(upd_n + upd_z, 1e-12) / 1e9 / 8000.0}),
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
