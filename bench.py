#!/usr/bin/env python3
"""Benchmark of the full-vocabulary KD loss forward+backward on one MI355X.

One step = one call of kd_loss_fwd_bwd (every kernel of the hot path) on one batch of
synthetic inputs already resident in HBM.  Prints ONE JSON line with tokens/s, the MFMA
roofline of the dominant kernel (timed live with HIP events through the library's
profiling hook) and the fp64 oracle timed on this host's cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
METRIC = "KD-loss fwd+bwd tokens/sec at V=151936; MFMA util vs bf16 peak"


def cpu_baseline(cfg, data, rows):
    """The fp64 oracle, as it stands, on the first `rows` tokens as a problem of its own."""
    import numpy as np
    from oracle import kd_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    sub = {k: data[k][:rows] for k in ("h_t", "h_s")}
    t0 = time.perf_counter()
    O.kd_loss_fwd_bwd(sub["h_t"], data["W_t"], sub["h_s"], data["W_s"], data["mask"][:rows], cfg.tau, cfg.kind,
                      cfg.beta, O.W_VH, row_block=min(rows, 256))
    dt = time.perf_counter() - t0
    return dict(value=rows / dt, unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"first {rows} of {cfg.T} tokens as a self-contained fwd+bwd problem, full V and H, "
                       f"numpy fp64, {dt:.1f} s wall")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="fkl_bf16")
    ap.add_argument("--cpu-rows", type=int, default=1024, help="tokens of the oracle sample (0 = skip)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "traffic.json"))
    ap.add_argument("--teacher-fp8", action="store_true",
                    help="optional mode, not the headline: teacher hidden states and head quantised to e4m3 "
                         "(one scale each) and the teacher logit tiles on the fp8 matrix pipe")
    ap.add_argument("--w-layout", choices=("vh", "hv"), default="vh",
                    help="storage order of the heads: vh = [V,H] (lm_head.weight order, the headline), hv = [H,V]")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (scale for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one worker's share of the data-parallel "
              "loss); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_01875_amd import inputs as I
    from paper_2603_01875_amd import kdloss as K

    torch.cuda.set_device(0)
    cfg = I.workload(args.workload)
    data = I.generate(cfg)
    dev = {k: I.to_device(data[k], cfg.dtype) for k in ("h_t", "W_t", "h_s", "W_s")}
    mask = torch.from_numpy(data["mask"]).cuda()
    T, V, H_t, H_s = cfg.T, cfg.V, cfg.H_t, cfg.H_s

    hv = args.w_layout == "hv"
    if hv:
        dev["W_t"] = dev["W_t"].t().contiguous()
        dev["W_s"] = dev["W_s"].t().contiguous()
    flags, t_scale = 0, 0.0
    if args.teacher_fp8:
        # quantise once (the head is frozen; hidden states would be quantised per batch by one more small kernel)
        s_h = float(dev["h_t"].abs().max().float().item()) / 448.0
        s_W = float(dev["W_t"].abs().max().float().item()) / 448.0
        dev["h_t"] = K.quantize_e4m3(dev["h_t"], s_h)
        dev["W_t"] = K.quantize_e4m3(dev["W_t"], s_W)
        flags, t_scale = K.FLAG_TEACHER_FP8, float(np.float32(s_h) * np.float32(s_W))
    p = K.make_params(T, H_t, H_s, V, cfg.kind, cfg.tau, cfg.beta, K.BF16, K.BF16, K.W_HV if hv else K.W_VH, False,
                      flags, t_scale)
    ws = K.alloc_workspace(p)
    vc, n_launch = K.kd_loss_plan_info(p)
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    ptl = torch.empty(T, dtype=torch.float32, device="cuda")
    gh = torch.empty((T, H_s), dtype=torch.bfloat16, device="cuda")
    gW = torch.empty((H_s, V) if hv else (V, H_s), dtype=torch.bfloat16, device="cuda")

    def step():
        K.kd_loss_fwd_bwd_raw(p, dev["h_t"], dev["W_t"], dev["h_s"], dev["W_s"], mask, loss, ptl, gh, gW, ws)

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                 # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps, bracketed by synchronisation; the dominant kernel
    # (logit tiles + online log-sum-exp, one launch per step) is bracketed by events inside it
    clk = K.ShaderClock().__enter__()      # shader clock seen by workgroup 0 of the last statistics kernel
    kt = K.KernelTimer(K.PROF_STATS, args.steps)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with kt:
        marks[0].record()
        for i in range(args.steps):
            step()
            marks[i + 1].record()          # per-step durations for the median / minimum (same stream)
        torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    stats_ms = kt.durations_ms()
    stats_avg = sum(stats_ms) / len(stats_ms)

    # the other kernel families, timed in one extra (untimed-region) step each
    fam = {}
    n_chunks = (V + vc - 1) // vc
    for name, which in (("grad", K.PROF_GRAD), ("gemm_grad_W", K.PROF_GEMM_GRAD_W),
                        ("gemm_grad_h", K.PROF_GEMM_GRAD_H), ("rows", K.PROF_ROWS)):
        if which == K.PROF_ROWS and cfg.kind < I.JSD:
            continue
        t = K.KernelTimer(which, n_chunks + 1)
        with t:
            step()
            torch.cuda.synchronize()
        fam[name] = sum(t.durations_ms())

    torch.cuda.synchronize()
    stats_ghz = clk.ghz()
    # the matrix pipe's own ceiling on this machine, measured right after the timed region (a few ms)
    probe = K.probe_mfma_rate()
    probe_ghz = clk.ghz()
    clk.__exit__()

    n_valid = int(data["mask"].sum())
    # masked tokens are compacted away on the device: the kernels work on the valid tokens, rounded up
    # to whole 256-token tiles; flop figures count exactly those rows
    T_comp = (n_valid + 255) // 256 * 256
    logit_flop = 2.0 * T_comp * V * (H_t + H_s)            # one pass over every computed logit, both heads
    passes = 3 if cfg.kind >= I.JSD else 2
    flop_alg = n_valid * V * (2.0 * H_t + 6.0 * H_s)
    flop_exec = passes * logit_flop + 4.0 * T_comp * V * H_s
    stats_tflops = logit_flop / (stats_avg * 1e-3) / 1e12
    # fp8 teacher: the student share of a launch runs against the bf16 peak, the teacher share against the
    # fp8 peak (5 PFLOP/s); the launch's peak is the flop-weighted harmonic mean of the two
    peak = (H_t + H_s) / (H_s / PEAK_BF16_TFLOPS + H_t / 5000.0) if args.teacher_fp8 else PEAK_BF16_TFLOPS

    traffic = None
    if os.path.exists(args.traffic_file) and not args.teacher_fp8:
        try:
            traffic = json.load(open(args.traffic_file)).get(args.workload, {}).get("stats_kernel_bytes")
        except Exception:
            traffic = None

    out = {
        "metric": METRIC, "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (teacher operands e4m3)" if args.teacher_fp8 else "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "H_t": H_t, "H_s": H_s, "V": V,
                   "kind": {0: "fkl", 1: "rkl", 2: "jsd", 3: "tvd", 4: "skew_fkl", 5: "skew_rkl"}[cfg.kind], "tau": cfg.tau, "beta": cfg.beta,
                   "valid_tokens": n_valid, "computed_token_rows": T_comp, "w_layout": args.w_layout.upper(), "teacher_fp8": bool(args.teacher_fp8), "vocab_chunk": vc, "launches_per_step": n_launch},
        "roofline": {"bound": "mfma", "kernel": "stats_kernel", "achieved": stats_tflops,
                     "peak": peak, "unit": "TFLOP/s", "frac": stats_tflops / peak,
                     "traffic": traffic, "launch_ms": stats_avg, "flop_per_launch": logit_flop,
                     "mfma_only_probe_tflops": probe,
                     "frac_of_probe": None if args.teacher_fp8 else stats_tflops / probe,
                     # the shader clock each of the two kernels ran at (cycles / 100 MHz ticks inside the kernel)
                     # and the share of the bf16 MFMA rate at THAT clock (256 CUs x 4 SIMDs x 1024 flop/clk)
                     "shader_clock_ghz": stats_ghz, "probe_shader_clock_ghz": probe_ghz,
                     "frac_at_shader_clock": None if args.teacher_fp8 else
                     stats_tflops / (1024 * 1024 * stats_ghz * 1e9 / 1e12)},
        "tflops_algorithmic": flop_alg / (ms_per_step * 1e-3) / 1e12,
        "tflops_executed": flop_exec / (ms_per_step * 1e-3) / 1e12,
        "mfma_frac_whole_step": (flop_exec / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS if not args.teacher_fp8 else
                                 (flop_exec - passes * 2.0 * T_comp * V * H_t / 2) / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS),
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "kernel_ms": dict(stats=stats_avg, **fam),
        "workspace_bytes": int(ws.numel()), "two_T_V_bytes": 2 * T * V,
        "loss": float(loss.item()),
    }
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, data, args.cpu_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
