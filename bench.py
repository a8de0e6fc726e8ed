#!/usr/bin/env python3
"""Benchmark: WERSA attention forward + backward tokens/s on one MI355X at n = 131072.

One step = one wersa_forward + one wersa_backward (every step of the hot path) over the
synthetic long-sequence workload (configuration 4: B=1, H=8, n=131072, d=64, L=6, m=256, bf16),
with inputs resident in HBM.  Prints ONE JSON line with the whole-job throughput, the roofline
figure of the dominant kernel (HIP-event timing inside the timed region) and the float64 CPU
oracle timed on the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm": (8000.0, "GB/s"), "mfma_bf16": (2500.0, "TFLOP/s"), "fp32": (157.3, "TFLOP/s")}


# HBM bytes per launch (read + written) on configuration 4, from the rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/mfma_path_config4_hbm_traffic.md (FETCH_SIZE scaled by the factor 2.0 that
# a plain 1 GiB copy shows for this counter, WRITE_SIZE by 1.0).
MIB = 1024.0 * 1024.0
RANKING_STEPS = 20   # untimed steps with every launch bracketed, to rank the kernels
MEASURED_TRAFFIC_CONFIG4 = {
    "wersa_rows_fwd": (137.7 + 134.8) * MIB, "wersa_rows_bwd_q": (272.0 + 130.1) * MIB,
    "wersa_rows_bwd_k": (275.2 + 260.4) * MIB,   # with dV
    "wersa_phiT_contract": ((256.4 + 32.5) + (388.4 + 36.5)) / 2 * MIB,   # average of the two launches
    "wersa_qbar": 128.6 * MIB, "wersa_add_pooled": 256.1 * MIB,
}


def to_device(p, dtype, device="cuda:0"):
    """NumPy workload dict -> torch tensors on the GPU (storage dtype for the big tensors)."""
    import numpy as np
    import torch
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    t = {k: torch.from_numpy(p[k]).to(device).to(tdt) for k in ("Q", "K", "V", "dO", "Omega") if k in p}
    for k in ("Wg", "bg", "omega"):
        t[k] = torch.from_numpy(np.ascontiguousarray(p[k], dtype=np.float32)).to(device)
    t["sigma"] = torch.tensor([float(p["sigma"])], dtype=torch.float32, device=device)
    return t


def kernel_models(cfg):
    """Algorithmic work of ONE launch of each kernel: name -> (bound, peak key, work, unit scale).

    Contractions: flops = 2 n d m per slice per contraction; a fused kernel counts every
    contraction it performs.  Memory-bound kernels: the bytes the step must move (inputs read
    once, outputs written once), never the intermediate feature matrices."""
    sl = cfg["B"] * cfg["H"]
    n, d, m = cfg["n"], cfg["d"], cfg["m"]
    e = 2 if cfg["dtype"] == "bf16" else 4
    unit = 2.0 * n * d * m * sl          # one n x d x m contraction over all slices
    nd = float(n) * d * sl
    models = {
        # generic (float32 arithmetic) path
        # (float32 MFMA: v_mfma_f32_32x32x2_f32, dense float32 matrix peak)
        "gemm_features": ("mfma", "fp32", unit), "gemm_phiT": ("mfma", "fp32", unit),
        "gemm_rows": ("mfma", "fp32", unit),
        "haar_filter_kernel": ("hbm", "hbm", nd * (e + 4)),
        # fused MFMA path
        "wersa_qbar": ("hbm", "hbm", nd * e),
        "wersa_haar_stage": ("hbm", "hbm", nd * (e + 2)),       # head dimension 128: one tensor in (bf16), one out (fp16)
        "wersa_phiT_contract": ("mfma", "mfma_bf16", 2 * unit),  # projection + Phi^T Y
        "wersa_rows_fwd": ("mfma", "mfma_bf16", 2 * unit),       # projection + Phi S
        "wersa_rows_bwd_q": ("mfma", "mfma_bf16", 3 * unit),     # projection, dPhi, dX_F
        # projection, dPhi, dX_F; with head dimension 64, 256 features per pass and whole 64-row
        # blocks the kernel also forms dV = Phi dS (a fourth contraction) and no rows_bwd_v launch follows
        "wersa_rows_bwd_k": ("mfma", "mfma_bf16", (4 if (d == 64 and m % 256 == 0 and n % 64 == 0) else 3) * unit),
        "wersa_rows_bwd_v": ("mfma", "mfma_bf16", 2 * unit),     # projection, Phi dS
        "wersa_ln_prep": ("hbm", "hbm", 3 * nd * e),
        "wersa_add_pooled": ("hbm", "hbm", 2 * nd * e),
    }
    # attention block (configuration 5): hidden x hidden projections over all tokens.  Average
    # launch: forward and backward hold 6 NT launches worth 8 products (dX sums three), 4 TN launches.
    hidden, tokens = cfg["H"] * d, cfg["B"] * n
    gemm = 2.0 * tokens * hidden * hidden
    models["wersa_gemm_nt"] = ("mfma", "mfma_bf16", gemm * 8.0 / 6.0)
    models["wersa_gemm_tn"] = ("mfma", "mfma_bf16", gemm)
    return models


def cpu_baseline(cfg, p, budget_s=12.0):
    """Time the oracle (as it stands) slice by slice until the budget is spent."""
    import numpy as np
    from oracle import wersa_oracle as wo
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    done, t0 = 0, time.perf_counter()
    todo = [(b, h) for b in range(cfg["B"]) for h in range(cfg["H"])]
    for (b, h) in todo:
        wo.backward(p["Q"], p["K"], p["V"], p["Omega"], float(p["sigma"]), p["Wg"], p["bg"], p["omega"],
                    cfg["L"], p["dO"], slices=[(b, h)])
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    tokens = cfg["B"] * cfg["n"] * done / len(todo)
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {len(todo)} (batch, head) slices of the same workload, forward+backward, "
                      f"float64 NumPy, {dt:.1f} s"}


def cpu_baseline_block(cfg, p, budget_s=15.0):
    """Configuration 5: the oracle on the per-head part of the block (that head's three input
    projections, then the core forward and backward), slice by slice until the budget is spent.
    The output projection and the weight gradients are not in the sample."""
    import numpy as np
    from oracle import wersa_oracle as wo
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    d, H = cfg["d"], cfg["H"]
    done, t0 = 0, time.perf_counter()
    todo = [(b, h) for b in range(cfg["B"]) for h in range(H)]
    for (b, h) in todo:
        cols = slice(h * d, (h + 1) * d)
        Xb = np.asarray(p["X"][b], np.float64)
        Q, K, V = (Xb @ np.asarray(p[w][:, cols], np.float64) for w in ("WQ", "WK", "WV"))
        dA = np.asarray(p["dY"][b], np.float64) @ np.asarray(p["WO"][cols, :], np.float64).T
        wo.backward_slice(Q, K, V, np.asarray(p["Omega"], np.float64), float(p["sigma"]),
                          np.asarray(p["Wg"][h], np.float64), np.asarray(p["bg"][h], np.float64),
                          np.asarray(p["omega"], np.float64), cfg["L"], 1e-6, 1e-6, dA)
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    tokens = cfg["B"] * cfg["n"] * done / len(todo)
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {len(todo)} (batch, head) slices: that head's Q', K', V' and dA projections and "
                      f"the core forward+backward in float64 NumPy, {dt:.1f} s; output projection and weight "
                      "gradients not included"}


def run_block(args):
    """Configuration 5: the attention block (projections around the core), forward + backward."""
    import numpy as np
    import torch
    from paper_2507_08637_amd import binding, workloads

    cfg = dict(workloads.CONFIGS[5])
    B, H, n, d, L, m = (cfg[k] for k in ("B", "H", "n", "d", "L", "m"))
    p = workloads.make_block_inputs(B, H, n, d, L, m, seed_base=5000)
    dev = "cuda:0"
    bf = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16)
    t = {k: bf(p[k]) for k in ("X", "WQ", "WK", "WV", "WO", "Omega", "dY")}
    t.update({k: torch.from_numpy(np.ascontiguousarray(p[k], dtype=np.float32)).to(dev) for k in ("Wg", "bg", "omega")})
    t["sigma"] = torch.tensor([float(p["sigma"])], dtype=torch.float32, device=dev)
    desc = binding.make_block_desc(t["X"], H, L, m)
    lib = binding.load_library()
    import ctypes
    saved = torch.empty(lib.wersa_block_saved_bytes(ctypes.byref(desc)), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(lib.wersa_block_workspace_bytes(ctypes.byref(desc), 0), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(lib.wersa_block_workspace_bytes(ctypes.byref(desc), 1), dtype=torch.uint8, device=dev)
    y = torch.empty_like(t["X"])
    grads = None
    weights = (t["WQ"], t["WK"], t["WV"], t["WO"])
    params = (t["Omega"], t["sigma"], t["Wg"], t["bg"], t["omega"])

    def step():
        nonlocal grads
        binding.wersa_block_forward(t["X"], *weights, H, *params, L, y=y, saved=saved, workspace=ws_f)
        grads = binding.wersa_block_backward(t["X"], *weights, H, *params, t["dY"], saved, L, workspace=ws_b,
                                             grads=grads)

    core_desc = binding.WersaDesc(B, H, n, d, L, m, 1, 1e-6, 1e-6, n * H * d, d, H * d, 0)
    workload = (f"config5: attention block B={B} n={n} hidden={H * d} (H={H} d={d}) L={L} m={m} bf16 storage, "
                "N(0,1) inputs, forward+backward")
    return cfg, p, step, binding.wersa_path_name(core_desc), workload


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=4, help="workload configuration (1-4: the core; 5: the attention block)")
    ap.add_argument("--generic", action="store_true",
                    help="force the float32-arithmetic path (WERSA_FLAG_GENERIC_PATH) on configurations 1-4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time K replays (no event bracketing in the "
                         "timed region: the roofline then comes from the untimed survey steps)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference point for the "
                         "FETCH_SIZE / WRITE_SIZE counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2507_08637_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load_library()
    halves = None
    if args.config == 5:
        cfg, p, step, path, workload = run_block(args)
    else:
        cfg, p = workloads.make_config(args.config, backward=True)
        t = to_device(p, cfg["dtype"])
        L = cfg["L"]
        flags = binding.WERSA_FLAG_GENERIC_PATH if args.generic else 0
        desc = binding.make_desc(t["Q"], L, cfg["m"], flags=flags)
        saved, ws_f = binding.alloc_like(desc, t["Q"], 0)
        _, ws_b = binding.alloc_like(desc, t["Q"], 1)
        out = torch.empty_like(t["Q"])
        grads = None
        path = binding.wersa_path_name(desc)
        workload = (f"config{args.config}: B={cfg['B']} H={cfg['H']} n={cfg['n']} d={cfg['d']} "
                    f"L={cfg['L']} m={cfg['m']} {cfg['dtype']} storage, {cfg['flavour']} inputs, "
                    "forward+backward")

        def fwd():
            binding.wersa_forward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"], t["omega"], L,
                                  out=out, saved=saved, workspace=ws_f, flags=flags)

        def bwd():
            nonlocal grads
            grads = binding.wersa_backward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"],
                                           t["omega"], out, t["dO"], saved, L, workspace=ws_b, grads=grads,
                                           flags=flags)

        def step():
            fwd()
            bwd()
        halves = (fwd, bwd)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Untimed survey: a few steps with every launch bracketed, to rank the kernels.  The timed
    # region then brackets only the dominant one, so that the event records do not sit between
    # all the other launches of the step being timed.
    survey, dominant = {}, None
    if not args.no_events:
        binding.wersa_profile_enable(True)
        for _ in range(RANKING_STEPS):
            step()
        torch.cuda.synchronize()
        survey = binding.wersa_profile_collect()
        binding.wersa_profile_enable(False)
        dominant = max(survey, key=lambda k: survey[k][0])
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        prof = {dominant: (survey[dominant][0] * args.steps / RANKING_STEPS,
                           survey[dominant][1] * args.steps // RANKING_STEPS)} if dominant else {}
    else:
        binding.wersa_profile_enable(dominant is not None, only=dominant)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        prof = binding.wersa_profile_collect()
        binding.wersa_profile_enable(False)

    ms = (t1 - t0) * 1e3 / args.steps
    tokens = cfg["B"] * cfg["n"]

    # After the timed region: (a) K more steps with one event pair per step, for a median next to
    # the mean; (b) what this device sustains on a plain streaming copy and on a bare loop of matrix
    # instructions, measured now in this process; (c) a few steps each preceded by that 2 GiB copy,
    # every launch bracketed: the memory-bound stages with their inputs NOT resident in the 256 MB
    # last-level cache (in back-to-back steps the pooled-query pass finds part of Q there).
    median_ms, peaks, cold, haar_stage, split_ms = None, None, {}, None, None
    if not args.graph and not args.no_events:
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for a, b in evs:
            a.record()
            step()
            b.record()
        torch.cuda.synchronize()
        per = sorted(a.elapsed_time(b) for a, b in evs)
        median_ms = per[len(per) // 2]
        if halves:   # forward and backward on their own: three events per step
            ev3 = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(args.steps)]
            for a, b, c in ev3:
                a.record()
                halves[0]()
                b.record()
                halves[1]()
                c.record()
            torch.cuda.synchronize()
            fw = sorted(a.elapsed_time(b) for a, b, c in ev3)
            bw = sorted(b.elapsed_time(c) for a, b, c in ev3)
            split_ms = {"forward_ms_median": fw[len(fw) // 2], "backward_ms_median": bw[len(bw) // 2]}
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        peaks = {"hbm_copy_GBps": binding.wersa_peak_copy(dst, src, reps=10),
                 "mfma_bf16_TFLOPs": binding.wersa_peak_mfma(reps=3)}
        binding.wersa_profile_enable(True)
        for _ in range(3):
            dst.copy_(src)   # flushes the cache; asynchronous, so the step follows without a host wait
            step()
        torch.cuda.synchronize()
        cold = binding.wersa_profile_collect()
        # (d) the gated Haar filter as a stage of its own (steps 3, 5, 6 through the stage entry point), which
        # the fused step never launches at head dimension 64: on a 1 GiB bf16 tensor of the workload's
        # slice count, row length and depth (8 slices x 2^20 rows x 64 columns; larger than the cache)
        if cfg["dtype"] == "bf16" and args.config != 5 and cfg["L"] <= 6 and not args.generic:
            sl, dcol = cfg["B"] * cfg["H"], cfg["d"]
            rows = (1 << 29) // (sl * dcol)
            if rows <= (1 << 22) and sl * rows * dcol == (1 << 29):
                xs = src.view(torch.bfloat16).view(1, sl, rows, dcol)
                ys = dst.view(torch.bfloat16).view(1, sl, rows, dcol)
                filt = torch.rand(sl, cfg["L"] + 1, device="cuda")
                for _ in range(4):
                    binding.wersa_haar_filter(xs, filt, cfg["L"], out=ys)
                torch.cuda.synchronize()
                hs = binding.wersa_profile_collect().get("wersa_haar_filter_bf16")
                if hs:
                    haar_stage = {"kernel": "wersa_haar_filter_bf16", "bound": "hbm", "work_per_launch": float(2 << 30),
                                  "work_unit": "B", "avg_us": round(hs[0] / hs[1] * 1e3, 2),
                                  "input": f"1 GiB bf16 tensor ({sl} slices x {rows} rows x {dcol} columns, L={cfg['L']}), "
                                           "read once and written once; not a launch of the step"}
        binding.wersa_profile_enable(False)
        del src, dst
    rec = {
        "metric": "WERSA attention fwd+bwd tokens/s on 1 GPU at n=131072; % HBM/MFMA roofline"
                  if args.config != 5 else
                  "WERSA attention block fwd+bwd tokens/s on 1 GPU at n=65536 (hidden 2048); % MFMA roofline",
        "value": tokens / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if path == "generic" or cfg["dtype"] == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": workload, "path": path, "launch": "hip graph replay" if args.graph else "eager"},
    }
    roof = None
    if prof:
        models = kernel_models(cfg)
        name = max(prof, key=lambda k: prof[k][0])
        tot_ms, launches = prof[name]
        avg_ms = tot_ms / launches
        if name in models:
            bound, pk, work = models[name]
            peak, unit = PEAK[pk]
            achieved = work / (avg_ms * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
            traffic = MEASURED_TRAFFIC_CONFIG4.get(name) if args.config == 4 else None
            roof = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                    "frac": achieved / peak, "traffic": traffic,
                    "traffic_source": ("table in bench.py from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs under "
                                       "profiles/ (not measured in this run)") if traffic else None,
                    "kernel": name, "avg_launch_ms": avg_ms, "launches_per_step": launches / args.steps}
        # every kernel, from the untimed survey steps (all launches bracketed)
        rec["kernels_ms_per_step"] = {k: round(v[0] / RANKING_STEPS, 4) for k, v in
                                      sorted(survey.items(), key=lambda kv: -kv[1][0])}
        # per stage: algorithmic work of one launch, average launch time (survey steps), fraction of the
        # nominal peak and of the peak measured in this process; memory-bound stages also with cold inputs
        stages = []
        for k, (tot, cnt) in sorted(survey.items(), key=lambda kv: -kv[1][0]):
            if k not in models:
                continue
            bound, pk, work = models[k]
            peak, unit = PEAK[pk]
            us = tot / cnt * 1e3
            ach = work / (us * 1e-6) / (1e9 if unit == "GB/s" else 1e12)
            st = {"kernel": k, "bound": bound, "work_per_launch": work, "work_unit": "B" if bound == "hbm" else "flop",
                  "launches_per_step": cnt / RANKING_STEPS, "avg_us": round(us, 2), "achieved": round(ach, 1), "unit": unit,
                  "frac_nominal": round(ach / peak, 4)}
            if peaks:
                mp = peaks["hbm_copy_GBps"] if bound == "hbm" else (peaks["mfma_bf16_TFLOPs"] if pk == "mfma_bf16" else None)
                if mp and mp > 0:
                    st["frac_measured"] = round(ach / mp, 4)
            if bound == "hbm" and k in cold:
                cus = cold[k][0] / cold[k][1] * 1e3
                st["cold_avg_us"] = round(cus, 2)
                st["cold_frac_nominal"] = round(work / (cus * 1e-6) / 1e9 / peak, 4)
            stages.append(st)
        if haar_stage:
            ach = haar_stage["work_per_launch"] / (haar_stage["avg_us"] * 1e-6) / 1e9
            haar_stage.update({"achieved": round(ach, 1), "unit": "GB/s", "frac_nominal": round(ach / PEAK["hbm"][0], 4),
                               "frac_measured": round(ach / peaks["hbm_copy_GBps"], 4)})
            stages.append(haar_stage)
        rec["stages"] = stages
        rec["stages_note"] = ("avg_us: back-to-back steps (a stage may find part of its input in the 256 MB last-level "
                              "cache); cold_*: the step preceded by a 2 GiB streaming copy")
    rec["measured_peaks"] = peaks
    rec["ms_per_step_median"] = median_ms
    if split_ms:
        rec.update(split_ms)
    rec["roofline"] = roof
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline_block(cfg, p) if args.config == 5 else cpu_baseline(cfg, p)
    else:
        rec["cpu_baseline"] = None
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
