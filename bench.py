#!/usr/bin/env python3
"""Benchmark of the ELM-RNN fit hot path on one MI355X.

A "step" is one whole fit (weights from the seed -> hidden matrix H(Q) -> TSQR solve with
refinement) over one synthetic batch that is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg5] [--contraction fp32]
                    [--no-fast-mode] [--no-streamed] [--no-ceilings] [--no-cpu-baseline] [--no-configs]

The reported line is for --contraction (default fp32: float32 matrix instructions, the arithmetic the
configurations name).  Unless --no-fast-mode is given, the same K steps are then timed once more
in the library's other stage-1 mode (split16: the recurrent contraction as an fp16 hi/lo split on
fp16 matrix instructions, float32-equivalent accuracy) and reported under "fast_mode".  Unless
--no-streamed is given, the streamed fit (H produced and folded into the TSQR chunk by chunk, never
stored) is timed as well and reported under "streamed_fit".

Workload: the LSTM N = 4M, Q = 100, d = 8, L = 512, m = 2 configuration (the one the headline
metric is quoted on); other configurations can be selected for study with --config.  Unless
--no-configs is given, the default run also times the other four benchmark configurations (at most
three fits each) and reports them under "configs": per-stage times, samples/s, the roofline
fraction of stage 1 and of stage 2 (against both of its ceilings) and the oracle baseline.
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

import synthdata  # noqa: E402

GATES = {"elman": 1, "lstm": 4, "gru": 3, "elman_diag": 1, "fc_multilag": 1}
PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak (256 CUs x 256 flop/clk x 2.4 GHz)
PEAK_FP16_MFMA_TFLOPS = 2500.0    # MI355X dense fp16 matrix peak
PEAK_FP32_VECTOR_TFLOPS = 157.3   # MI355X fp32 vector peak (256 CUs x 4 SIMDs x 32 FMA lanes-equivalent x 2.4 GHz)

# Memory traffic of one hidden-matrix kernel launch, bytes, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs scaled by a copy kernel of known size (profiles/ holds the summaries these come from).  The
# counters sit at the L2 boundary: they include refills of the L2-resident weight operand from the
# Infinity Cache, which never reach HBM.
MEASURED_TRAFFIC_BYTES = {"cfg5": 923.4e9 + 9.2e9}   # profiles/hidden_kernel_cfg5_pmc.txt (L2-boundary traffic)
MEASURED_TRAFFIC_SPLIT_BYTES = {"cfg5": 1283.1e9 + 413.7e9}   # profiles/fit_cfg5_split16_kernel_trace_and_pmc.txt
TRAFFIC_SOURCE = ("profiles/hidden_kernel_cfg5_pmc.txt: stored rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE figure of the "
                  "same launch, not measured by this run")
TRAFFIC_SPLIT_SOURCE = ("profiles/fit_cfg5_split16_kernel_trace_and_pmc.txt: stored rocprofv3 --pmc figure, not "
                        "measured by this run")


_last_note = [0.0]


def note(msg: str) -> None:
    """Progress on stderr (stdout carries the one JSON line): at most one line per 20 s of wall time."""
    now = time.perf_counter()
    if now - _last_note[0] >= 20.0:
        _last_note[0] = now
        print(f"bench.py: {msg}", file=sys.stderr, flush=True)


def stage1_flops(cfg) -> float:
    """Algorithmic flops of one hidden-matrix launch: 2 Q kL (L + d) per sample for the dense cells,
    2 L (Q (Q - 1) / 2 + Q d) for the paper's diagonal multi-lag Elman, 2 L (L Q (Q - 1) / 2 + Q d) for
    its fully connected multi-lag cell."""
    if cfg.cell == "elman_diag":
        return 2.0 * cfg.L * (cfg.Q * (cfg.Q - 1) / 2 + cfg.Q * cfg.d) * cfg.N
    if cfg.cell == "fc_multilag":      # step t contracts (t - 1) L + d columns
        return 2.0 * cfg.L * (cfg.L * cfg.Q * (cfg.Q - 1) / 2 + cfg.Q * cfg.d) * cfg.N
    return 2.0 * cfg.Q * GATES[cfg.cell] * cfg.L * (cfg.L + cfg.d) * cfg.N


PEAK_HBM_GBS = 8000.0             # MI355X HBM3E


def stage2_work(cfg):
    """Algorithmic work of the solve on an N x n matrix, n = L + m: Householder flops 2 N n^2 - 2/3 n^3 and
    4 N n bytes (the rows of [H | T] read once)."""
    n = cfg.L + cfg.m
    return 2.0 * cfg.N * n * n - (2.0 / 3.0) * n ** 3, 4.0 * cfg.N * n


def stage2_roofline(cfg, solve_ms):
    """Stage 2 against both of its ceilings (the larger of the two times bounds it)."""
    flops, nbytes = stage2_work(cfg)
    tf = flops / (solve_ms * 1e-3) / 1e12
    gbs = nbytes / (solve_ms * 1e-3) / 1e9
    t_roof_ms = 1e3 * max(flops / (PEAK_FP32_MFMA_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9))
    return {"kernel": "TSQR fold kernels + back-solve + refinement (stage 2)", "solve_ms": solve_ms,
            "achieved_tflops": tf, "frac_of_fp32_mfma_peak": tf / PEAK_FP32_MFMA_TFLOPS,
            "achieved_gbs": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS,
            "roofline_ms": t_roof_ms, "frac_of_roofline": t_roof_ms / solve_ms}


def measure_config(elm, torch, cfg, steps: int, cpu_rows: int) -> dict:
    """One of the smaller benchmark configurations, float32 mode, materialised windows resident in HBM:
    a warm-up fit and `steps` timed ones, per-stage times from the library's events on the launch stream."""
    series = synthdata.make_series(cfg.N + cfg.Q, cfg.d, cfg.seed, cfg.ar_sigma).astype(np.float32)
    sd = torch.from_numpy(series).cuda()
    X = torch.as_strided(sd, (cfg.N, cfg.Q, cfg.d), (cfg.d, cfg.d, 1)).contiguous()
    T = sd[cfg.Q:cfg.Q + cfg.N, :cfg.m].contiguous()
    H = torch.empty((cfg.N, cfg.L), dtype=torch.float32, device="cuda")
    ws = torch.empty(elm.fit_workspace_bytes(cfg.N, cfg.L, cfg.m, False, cfg.cell, cfg.Q, cfg.d),
                     dtype=torch.uint8, device="cuda")
    kw = dict(w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius, forget_bias=cfg.forget_bias,
              zero_bias=cfg.zero_bias, workspace=ws, H_out=H)

    def one():
        res = elm.fit(cfg.cell, X, T, cfg.L, cfg.seed, **kw)
        st = res.stats
        res.model.close()
        return st

    one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats = [one() for _ in range(steps)]
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    hidden_ms = float(np.mean([s.t_hidden_ms for s in stats]))
    solve_ms = float(np.mean([s.t_solve_ms for s in stats]))
    tf = stage1_flops(cfg) / (hidden_ms * 1e-3) / 1e12
    out = {"workload": f"{cfg.name}: {cfg.cell} ELM-RNN fit, N={cfg.N}, Q={cfg.Q}, d={cfg.d}, L={cfg.L}, m={cfg.m}, "
                       "materialised windows resident in HBM",
           "dtype": "f32", "steps": steps, "value": cfg.N / dt, "unit": "samples/s", "ms_per_step": 1e3 * dt,
           "hidden_ms": hidden_ms, "solve_ms": solve_ms, "host_ms": 1e3 * dt - hidden_ms - solve_ms,
           "hidden_samples_per_s": cfg.N / (hidden_ms * 1e-3), "solve_samples_per_s": cfg.N / (solve_ms * 1e-3),
           "rmse": stats[-1].rmse, "ne_resid": stats[-1].ne_resid, "refine_iters": stats[-1].refine_iters,
           "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": tf / PEAK_FP32_MFMA_TFLOPS,
                        "kernel": "hidden_kernel (stage 1, fp32 MFMA 32x32x2)"},
           "stage2": stage2_roofline(cfg, solve_ms)}
    del X, T, H, ws
    if cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, cpu_rows)
    return out


def cpu_baseline(cfg, budget_rows: int):
    """The float64 oracle, as it stands, on a bounded row sample of the same workload."""
    from oracle import fit as ofit
    n = min(cfg.N, budget_rows)
    series = synthdata.make_series(n + cfg.Q, cfg.d, cfg.seed, cfg.ar_sigma).astype(np.float32)
    X, T = synthdata.make_windows(series, n, cfg.Q, cfg.m)
    t0 = time.perf_counter()
    ofit.fit(cfg.cell, X, T, cfg.L, cfg.seed, w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius,
             forget_bias=cfg.forget_bias, zero_bias=cfg.zero_bias)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    return {"value": n / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": f"numpy float64 oracle fit (H build + Householder solve) on the first {n} "
                      f"windows of {cfg.name} ({dt:.1f} s)"}


def run_sweep(elm, torch, steps: int) -> dict:
    """Study workloads beyond the benchmark configurations (the paper's scalability sweep over the hidden
    size, its longest-window dataset shape, and prediction on held-out windows), all synthetic."""
    import dataclasses
    rows = []

    def timed_fit(cfg, X, T, mode):
        H = torch.empty((cfg.N, cfg.L), dtype=torch.float32, device="cuda")
        ws = torch.empty(elm.fit_workspace_bytes(cfg.N, cfg.L, cfg.m, False, cfg.cell, cfg.Q, cfg.d), dtype=torch.uint8, device="cuda")
        kw = dict(w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius, forget_bias=cfg.forget_bias,
                  zero_bias=cfg.zero_bias, contraction=mode, workspace=ws, H_out=H, allow_rank_deficient=True)
        res = elm.fit(cfg.cell, X, T, cfg.L, cfg.seed, **kw)          # warm-up
        res.model.close()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            res = elm.fit(cfg.cell, X, T, cfg.L, cfg.seed, **kw)
            st = res.stats
            res.model.close()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        return {"cell": cfg.cell, "contraction": mode, "N": cfg.N, "Q": cfg.Q, "d": cfg.d, "L": cfg.L,
                "samples_per_s": cfg.N / dt, "ms_per_fit": 1e3 * dt, "hidden_ms": st.t_hidden_ms,
                "solve_ms": st.t_solve_ms, "rmse": st.rmse, "rank_deficient": st.rank_deficient}

    def windows(cfg):
        series = synthdata.make_series(cfg.N + cfg.Q, cfg.d, cfg.seed, cfg.ar_sigma).astype(np.float32)
        sd = torch.from_numpy(series).cuda()
        X = torch.as_strided(sd, (cfg.N, cfg.Q, cfg.d), (cfg.d, cfg.d, 1))      # zero-copy sliding windows
        T = sd[cfg.Q:cfg.Q + cfg.N, :cfg.m].contiguous()
        return X, T

    base = {"elman_diag": synthdata.get_config("paper_elman"),
            "elman": dataclasses.replace(synthdata.get_config("cfg2"), N=1_000_000, Q=50),
            "lstm": dataclasses.replace(synthdata.get_config("cfg3"), N=1_000_000, Q=50, d=1),
            "gru": dataclasses.replace(synthdata.get_config("cfg4"), N=1_000_000, Q=50, d=1, m=1)}
    for cell, b in base.items():
        X, T = windows(b)
        for L in (5, 10, 20, 50, 100):
            for mode in (("fp32",) if cell == "elman_diag" else ("fp32", "split16")):
                r = timed_fit(dataclasses.replace(b, L=L), X, T, mode)
                r["study"] = "hidden-size sweep"
                rows.append(r)
    # the paper's fully connected cell over the same hidden sizes at Q = 50: up to 20 units the history of a
    # window stays in LDS, beyond that every step is a launch over a device-resident history
    b = synthdata.get_config("paper_fc_q50")
    X, T = windows(b)
    for L in (5, 10, 20, 50, 100):
        c = dataclasses.replace(b, L=L)
        r = timed_fit(c, X, T, "fp32")
        r["study"] = "hidden-size sweep"
        r["stage1_tflops"] = stage1_flops(c) / (r["hidden_ms"] * 1e-3) / 1e12
        rows.append(r)
    for cell in ("elman", "lstm", "gru"):
        b = dataclasses.replace(base[cell], N=4500, Q=3197, L=50)
        X, T = windows(b)
        for mode in ("fp32", "split16"):
            r = timed_fit(b, X, T, mode)
            r["study"] = "long windows"
            rows.append(r)
    # the paper's own Elman cell on that shape (Q(Q-1)/2 lag terms per sample and neuron); its widest layer
    # there is 100 units.  The weight scale shrinks with sqrt(Q) so that the feedback sum keeps its size.
    for L in (50, 100):
        b = dataclasses.replace(base["elman_diag"], N=4500, Q=3197, L=L, w_scale=0.3 * (50 / 3197) ** 0.5)
        X, T = windows(b)
        r = timed_fit(b, X, T, "fp32")
        r["study"] = "long windows"
        r["stage1_tflops"] = 4500 * L * (3197 * 3196 + 2 * 3197) / (r["hidden_ms"] * 1e-3) / 1e12
        rows.append(r)
    # ... and its fully connected cell (L Q (Q - 1) / 2 lag products per sample and neuron: 1e11 flops per window
    # at 100 units; timed at 50): passes of 2,304 rows whose launches split the contraction over slices
    b = dataclasses.replace(synthdata.get_config("paper_fc_q50"), N=4500, Q=3197, d=1, L=50,
                            w_scale=0.05 * (50 / 3197) ** 0.5)
    X, T = windows(b)
    r = timed_fit(b, X, T, "fp32")
    r["study"] = "long windows"
    r["stage1_tflops"] = stage1_flops(b) / (r["hidden_ms"] * 1e-3) / 1e12
    rows.append(r)
    # fit on the first 80 % of the windows, predict the last 20 %
    cfg = synthdata.get_config("cfg3")
    X, T = windows(cfg)
    n_tr = int(0.8 * cfg.N)
    res = elm.fit(cfg.cell, X[:n_tr], T[:n_tr], cfg.L, cfg.seed, w_scale=cfg.w_scale, forget_bias=cfg.forget_bias)
    Y = elm.predict(res.model, X[n_tr:])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        Y = elm.predict(res.model, X[n_tr:])
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    test_rmse = float(torch.sqrt(torch.mean((Y.double() - T[n_tr:].double()) ** 2)))
    rows.append({"study": "held-out prediction", "cell": cfg.cell, "N_train": n_tr, "N_test": cfg.N - n_tr,
                 "Q": cfg.Q, "d": cfg.d, "L": cfg.L, "train_rmse": res.stats.rmse, "test_rmse": test_rmse,
                 "predict_samples_per_s": (cfg.N - n_tr) / dt})
    res.model.close()
    return {"metric": "ELM fit samples/sec (H build + TSQR solve) at 1 GPU, study workloads", "unit": "samples/s",
            "n_gpus": 1, "steps": steps, "data": "synthetic", "sweep": rows}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--contraction", default="fp32", choices=["fp32", "split16"],
                    help="stage-1 contraction mode of the reported line")
    ap.add_argument("--no-fast-mode", action="store_true", help="skip the extra split16 measurement")
    ap.add_argument("--no-streamed", action="store_true", help="skip the extra streamed-fit measurement")
    ap.add_argument("--streamed", action="store_true",
                    help="time the streamed fit as the main leg (profiling runs; implies --no-streamed)")
    ap.add_argument("--chunk-rows", type=int, default=0,
                    help="streamed fit: 0 = library default, -1 = in-kernel hand-off, > 0 = rows per chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the extra measurements of the four smaller benchmark configurations")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured-ceilings probe")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the oracle sample (0 = auto)")
    ap.add_argument("--n", type=int, default=0, help="override N (profiling runs only; the reported "
                                                     "workload string then names the reduced N)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line, time the study workloads: the hidden-size sweep "
                         "L = 5..100 (N = 1e6, Q = 50, d = 1) for every cell, the long-window shape "
                         "(N = 4500, Q = 3197), and a fit on 80 %% / predict on 20 %% split; prints one "
                         "JSON line with a \"sweep\" list")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates FETCH_SIZE / WRITE_SIZE "
                         "counters in rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU only (the fit path runs on a single GPU; rows are "
              "independent, so it would shard by row ranges with one exchange of R factors); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_1911_13252_amd as elm

    if args.sweep:
        print(json.dumps(run_sweep(elm, torch, args.steps)))
        return 0

    cfg = synthdata.get_config(args.config)
    if args.n > 0:
        import dataclasses
        cfg = dataclasses.replace(cfg, N=args.n)
    torch.cuda.set_device(0)
    series = synthdata.make_series(cfg.N + cfg.Q, cfg.d, cfg.seed, cfg.ar_sigma).astype(np.float32)
    sd = torch.from_numpy(series).cuda()
    X = torch.as_strided(sd, (cfg.N, cfg.Q, cfg.d), (cfg.d, cfg.d, 1)).contiguous()   # materialised windows
    T = sd[cfg.Q:cfg.Q + cfg.N, :cfg.m].contiguous()
    kw = dict(w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius, forget_bias=cfg.forget_bias,
              zero_bias=cfg.zero_bias)
    if args.streamed:
        args.no_streamed = True
        H = None
        ws = torch.empty(elm.fit_streamed_workspace_bytes(cfg.N, cfg.L, cfg.m, max(args.chunk_rows, 0), cfg.cell, cfg.Q, cfg.d),
                         dtype=torch.uint8, device="cuda")
    else:
        H = torch.empty((cfg.N, cfg.L), dtype=torch.float32, device="cuda")
        ws = torch.empty(elm.fit_workspace_bytes(cfg.N, cfg.L, cfg.m, False, cfg.cell, cfg.Q, cfg.d), dtype=torch.uint8, device="cuda")

    def step(mode=args.contraction):
        if args.streamed:
            res = elm.fit_streamed(cfg.cell, X, T, cfg.L, cfg.seed, contraction=mode, chunk_rows=args.chunk_rows,
                                   workspace=ws, **kw)
        else:
            res = elm.fit(cfg.cell, X, T, cfg.L, cfg.seed, contraction=mode, workspace=ws, H_out=H, **kw)
        st = res.stats
        res.model.close()
        return st

    def roofline(mode, hidden_ms):
        achieved = stage1_flops(cfg) / (hidden_ms * 1e-3) / 1e12
        if cfg.cell == "elman_diag":
            return {"bound": "alu", "achieved": achieved, "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_FP32_VECTOR_TFLOPS, "traffic": None,
                    "kernel": "diag_reg_kernel / diag_lds_kernel (stage 1, fp32 vector FMA; the build "
                              "disables packed fp32, which caps the rate at half the published peak)"}
        if mode == "fp32":
            r = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                 "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                 "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
                 "traffic_source": TRAFFIC_SOURCE if cfg.name in MEASURED_TRAFFIC_BYTES else None,
                 "kernel": "hidden_kernel (stage 1, fp32 MFMA 32x32x2)"}
            if cfg.cell == "fc_multilag" and (cfg.Q - 1) * cfg.L + cfg.d + 1 > 1272:
                r["kernel"] = "fc_step_kernel (stage 1, one launch per step, fp32 MFMA 32x32x2)"
            return r
        # three fp16 matrix instructions per algorithmic product (hi*hi, hi*lo, lo*hi): the
        # algorithmic rate can reach at most a third of the fp16 peak
        return {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP16_MFMA_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_FP16_MFMA_TFLOPS,
                "traffic": MEASURED_TRAFFIC_SPLIT_BYTES.get(cfg.name),
                "traffic_source": TRAFFIC_SPLIT_SOURCE if cfg.name in MEASURED_TRAFFIC_SPLIT_BYTES else None,
                "kernel": "hidden_split_kernel (stage 1, fp16 MFMA 32x32x16, 3 products per float32 product)",
                "issued_over_algorithmic": 3.0 * (16 * ((cfg.L + 15) // 16) + 32) / (cfg.L + cfg.d),
                "achieved_over_fp32_mfma_peak": achieved / PEAK_FP32_MFMA_TFLOPS}

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)            # 1 GiB read + 1 GiB written by one plain copy kernel
        torch.cuda.synchronize()
        del src, dst

    note(f"{cfg.name}: inputs resident, {args.warmup} warm-up and {args.steps} timed fits follow")
    for i in range(args.warmup):
        step()
        note(f"warm-up fit {i + 1}/{args.warmup} done")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stats, marks = [], [t0]
    for i in range(args.steps):
        stats.append(step())              # a fit synchronises its stream before it returns
        marks.append(time.perf_counter())
        note(f"timed fit {i + 1}/{args.steps} done")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step_ms = [1e3 * (b - a) for a, b in zip(marks[:-1], marks[1:])]

    ms_per_step = 1e3 * dt / args.steps
    hidden_ms = float(np.mean([s.t_hidden_ms for s in stats]))     # HIP events on the launch stream
    solve_ms = float(np.mean([s.t_solve_ms for s in stats]))
    out = {
        "metric": "ELM fit samples/sec (H build + TSQR solve) at 1 GPU",
        "value": cfg.N * args.steps / dt,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if args.contraction == "fp32" else "f32 (fp16 hi/lo split operands, f32 accumulate)",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.cell} ELM-RNN fit, N={cfg.N}, Q={cfg.Q}, d={cfg.d}, "
                               f"L={cfg.L}, m={cfg.m}, materialised windows resident in HBM",
                   "hidden_ms": hidden_ms, "solve_ms": solve_ms,
                   "host_ms": ms_per_step - hidden_ms - solve_ms,     # weights from the seed, packing, launches
                   "ms_per_step_min": min(per_step_ms), "ms_per_step_median": float(np.median(per_step_ms)),
                   "hidden_samples_per_s": cfg.N / (hidden_ms * 1e-3),
                   "solve_samples_per_s": cfg.N / (solve_ms * 1e-3),
                   "contraction": args.contraction, "streamed": bool(args.streamed),
                   "rmse": stats[-1].rmse,
                   "ne_resid": None if np.isnan(stats[-1].ne_resid) else stats[-1].ne_resid,
                   "refine_iters": stats[-1].refine_iters},
        "roofline": roofline(args.contraction, hidden_ms),
        "stage2": stage2_roofline(cfg, solve_ms),
    }
    if (not args.no_fast_mode and args.contraction == "fp32" and cfg.d <= 15
            and cfg.cell in ("elman", "lstm", "gru")):
        step("split16")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fstats = []
        for i in range(args.steps):
            fstats.append(step("split16"))
            note(f"split16 fit {i + 1}/{args.steps} done")
        torch.cuda.synchronize()
        fdt = time.perf_counter() - t0
        f_hidden = float(np.mean([s.t_hidden_ms for s in fstats]))
        f_solve = float(np.mean([s.t_solve_ms for s in fstats]))
        out["fast_mode"] = {"contraction": "split16", "value": cfg.N * args.steps / fdt, "unit": "samples/s",
                            "ms_per_step": 1e3 * fdt / args.steps, "hidden_ms": f_hidden, "solve_ms": f_solve,
                            "rmse": fstats[-1].rmse, "ne_resid": fstats[-1].ne_resid,
                            "roofline": roofline("split16", f_hidden)}
    if not args.no_streamed and args.contraction == "fp32":
        # the same fit with H produced and folded into the TSQR chunk by chunk (never stored)
        del H, ws
        sws = torch.empty(elm.fit_streamed_workspace_bytes(cfg.N, cfg.L, cfg.m, max(args.chunk_rows, 0), cfg.cell, cfg.Q, cfg.d),
                          dtype=torch.uint8, device="cuda")

        def sstep():
            res = elm.fit_streamed(cfg.cell, X, T, cfg.L, cfg.seed, workspace=sws, chunk_rows=args.chunk_rows, **kw)
            st = res.stats
            res.model.close()
            return st

        sstep()
        torch.cuda.synchronize()
        ssteps = min(args.steps, 2)
        t0 = time.perf_counter()
        sstats = []
        for i in range(ssteps):
            sstats.append(sstep())
            note(f"streamed fit {i + 1}/{ssteps} done")
        torch.cuda.synchronize()
        sdt = time.perf_counter() - t0
        out["streamed_fit"] = {"value": cfg.N * ssteps / sdt, "unit": "samples/s", "steps": ssteps,
                               "ms_per_step": 1e3 * sdt / ssteps,
                               "hidden_ms": float(np.mean([s.t_hidden_ms for s in sstats])),
                               "solve_ms": float(np.mean([s.t_solve_ms for s in sstats])),
                               "refine_iters": sstats[-1].refine_iters, "rmse": sstats[-1].rmse,
                               "workspace_bytes": sws.numel(),
                               "ordinary_fit_bytes": elm.fit_workspace_bytes(cfg.N, cfg.L, cfg.m, True, cfg.cell, cfg.Q, cfg.d)}
    if not args.no_ceilings:
        # what this device sustains: register-resident matrix-instruction loops and a streaming copy
        torch.cuda.empty_cache()
        c = elm.probe_ceilings()
        out["ceilings"] = c
        r = out["roofline"]
        if r.get("bound") == "mfma":
            r["frac_of_measured"] = r["achieved"] / (c["mfma_f32_tflops"] if r["peak"] == PEAK_FP32_MFMA_TFLOPS
                                                     else c["mfma_f16_tflops"])
        if "fast_mode" in out:
            out["fast_mode"]["roofline"]["frac_of_measured"] = out["fast_mode"]["roofline"]["achieved"] / c["mfma_f16_tflops"]
    cpu_rows = {"cfg1": 2000, "cfg2": 100_000, "cfg3": 50_000, "cfg4": 16_384, "cfg5": 8192,
                "paper_elman": 20_000, "paper_fc": 20_000, "paper_fc_q50": 20_000}
    if not args.no_configs and cfg.name == "cfg5" and args.n == 0 and not args.streamed:
        # the other four benchmark configurations (the headline fields above stay those of cfg5): at most
        # three timed fits each; the oracle on all rows of cfg1 / cfg2 and on a slice of cfg3 / cfg4
        del X, T
        if not args.no_streamed and args.contraction == "fp32":
            del sws
        torch.cuda.empty_cache()
        out["configs"] = []
        for n in ("cfg1", "cfg2", "cfg3", "cfg4"):
            note(f"{n}: fits and oracle baseline")
            out["configs"].append(measure_config(elm, torch, synthdata.get_config(n), min(args.steps, 3),
                                                 0 if args.no_cpu_baseline else cpu_rows[n]))
    if not args.no_cpu_baseline:
        note(f"{cfg.name}: oracle baseline on the host cores")
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_rows or cpu_rows[cfg.name])
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
