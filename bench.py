#!/usr/bin/env python3
"""Benchmark of the full-vocabulary KD loss forward+backward on one MI355X.

One step = one call of kd_loss_fwd_bwd (every kernel of the hot path) on one batch of
synthetic inputs already resident in HBM.  Prints ONE JSON line with tokens/s, the MFMA
roofline of the dominant kernel (timed live with HIP events through the library's
profiling hook), the fp64 oracle timed on this host's cores on the same workload, the
other benchmark workloads timed for a few steps each (`other_workloads`), and what the
vendor GEMM reaches on the logit products of the same shape (a yardstick, not a target).
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
    """The fp64 oracle, as it stands, on the first `rows` tokens as a problem of its own (all of them by
    default: the headline workload takes it about half a minute on 16 host threads)."""
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
    what = "the whole workload" if rows >= cfg.T else f"first {rows} of {cfg.T} tokens as a self-contained problem"
    return dict(value=rows / dt, unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"{what}: one fwd+bwd, full V and H, numpy fp64, {dt:.1f} s wall")


def device_workload(name, seed=0):
    """One of the benchmark workloads with operands drawn on the device (same shapes, value scales and mask
    structure as inputs.generate, independent draws): the larger workloads would take the host generator
    the better part of a minute each."""
    import numpy as np
    import torch
    from paper_2603_01875_amd import inputs as I
    cfg = I.workload(name)
    g = torch.Generator(device="cuda").manual_seed(cfg.seed + seed)

    def hidden(H):
        x = torch.randn(cfg.T, H, device="cuda", generator=g)
        x = x / x.pow(2).mean(1, keepdim=True).sqrt()
        return x.to(torch.bfloat16)

    def head(H, std):
        out = torch.empty(cfg.V, H, device="cuda", dtype=torch.bfloat16)
        for v0 in range(0, cfg.V, 32768):                     # in slabs: bounds the fp32 temporary
            n = min(32768, cfg.V - v0)
            out[v0:v0 + n] = (torch.randn(n, H, device="cuda", generator=g) * std).to(torch.bfloat16)
        return out
    mask = I._mask(np.random.default_rng(cfg.seed), cfg)
    return cfg, dict(h_t=hidden(cfg.H_t), h_s=hidden(cfg.H_s), W_t=head(cfg.H_t, cfg.w_t_std),
                     W_s=head(cfg.H_s, cfg.w_s_std), mask=torch.from_numpy(mask).cuda()), int(mask.sum())


def time_other_workload(name, steps=3, warmup=1):
    """ms/step, tokens/s and the statistics kernel's rate for one of the other workloads."""
    import torch
    from paper_2603_01875_amd import inputs as I
    from paper_2603_01875_amd import kdloss as K
    cfg, d, n_valid = device_workload(name)
    T, V, H_t, H_s = cfg.T, cfg.V, cfg.H_t, cfg.H_s
    p = K.make_params(T, H_t, H_s, V, cfg.kind, cfg.tau, cfg.beta)
    ws = K.alloc_workspace(p)
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    gh = torch.empty((T, H_s), dtype=torch.bfloat16, device="cuda")
    gW = torch.empty((V, H_s), dtype=torch.bfloat16, device="cuda")
    mask = None if n_valid == T else d["mask"]

    def step():
        K.kd_loss_fwd_bwd_raw(p, d["h_t"], d["W_t"], d["h_s"], d["W_s"], mask, loss, None, gh, gW, ws)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    kt = K.KernelTimer(K.PROF_STATS, steps)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with kt:
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    stats_ms = sum(kt.durations_ms()) / steps
    T_comp = (n_valid + 255) // 256 * 256
    logit_flop = 2.0 * T_comp * V * (H_t + H_s)
    passes = 3 if cfg.kind >= I.JSD else 2
    flop_exec = passes * logit_flop + 4.0 * T_comp * V * H_s
    out = dict(T=T, H_t=H_t, H_s=H_s, V=V, kind={0: "fkl", 1: "rkl", 2: "jsd"}[cfg.kind], tau=cfg.tau, beta=cfg.beta,
               valid_tokens=n_valid, steps=steps, ms_per_step=ms, tokens_per_s=T / (ms * 1e-3),
               valid_tokens_per_s=n_valid / (ms * 1e-3), stats_kernel_ms=stats_ms,
               stats_kernel_tflops=logit_flop / (stats_ms * 1e-3) / 1e12,
               stats_kernel_frac=logit_flop / (stats_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
               tflops_executed=flop_exec / (ms * 1e-3) / 1e12, vocab_chunk=K.kd_loss_plan_info(p)[0],
               workspace_bytes=int(ws.numel()), two_T_V_bytes=2 * T * V, loss=float(loss.item()))
    del d, ws, gh, gW
    torch.cuda.empty_cache()
    return out


def vendor_gemm_yardstick(T_comp, V, H_t, H_s, reps=5):
    """TFLOP/s of the vendor GEMM (torch.matmul, i.e. hipBLASLt / rocBLAS) on the two logit products of the
    headline shape, writing the [T,V] result this library never forms.  A yardstick for what a tuned
    plain GEMM reaches on this GPU at this shape; not part of the method and not in the timed region."""
    import torch
    res = {}
    for name, H in (("teacher", H_t), ("student", H_s)):
        a = torch.randn(T_comp, H, device="cuda").to(torch.bfloat16)
        b = (torch.randn(V, H, device="cuda") * 0.02).to(torch.bfloat16)
        for _ in range(2):
            c = a @ b.t()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            c = a @ b.t()
        e1.record()
        torch.cuda.synchronize()
        res[name + "_ms"] = e0.elapsed_time(e1) / reps
        del a, b, c
    flop = 2.0 * T_comp * V * (H_t + H_s)
    total_ms = res["teacher_ms"] + res["student_ms"]
    res["both_products_tflops"] = flop / (total_ms * 1e-3) / 1e12
    res["teacher_tflops"] = 2.0 * T_comp * V * H_t / (res["teacher_ms"] * 1e-3) / 1e12
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="fkl_bf16")
    ap.add_argument("--cpu-rows", type=int, default=-1,
                    help="tokens of the oracle's timed run (-1 = the whole workload, 0 = skip)")
    ap.add_argument("--other-workloads", default="rkl_bf16,jsd_bf16,large_teacher,long_peaked",
                    help="comma-separated workloads timed for a few steps each after the headline measurement "
                         "(empty = none)")
    ap.add_argument("--no-vendor-gemm", action="store_true", help="skip the vendor-GEMM yardstick")
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

    # HBM-side traffic of one statistics launch: NOT measured in this run (it needs rocprofv3 --pmc); the value
    # stored with its command under profiles/ is passed through and labelled as such
    traffic, traffic_source = None, None
    if os.path.exists(args.traffic_file) and not args.teacher_fp8 and not hv:
        try:
            rec = json.load(open(args.traffic_file)).get(args.workload, {})
            traffic = rec.get("stats_kernel_bytes")
            traffic_source = "stored: " + rec.get("source", os.path.relpath(args.traffic_file, ROOT))
        except Exception:
            traffic = None

    logit_flop_valid = 2.0 * n_valid * V * (H_t + H_s)
    out = {
        "metric": METRIC, "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "valid_tokens_per_s": n_valid / (ms_per_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (teacher operands e4m3)" if args.teacher_fp8 else "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "H_t": H_t, "H_s": H_s, "V": V,
                   "kind": {0: "fkl", 1: "rkl", 2: "jsd", 3: "tvd", 4: "skew_fkl", 5: "skew_rkl"}[cfg.kind], "tau": cfg.tau, "beta": cfg.beta,
                   "valid_tokens": n_valid, "computed_token_rows": T_comp, "w_layout": args.w_layout.upper(), "teacher_fp8": bool(args.teacher_fp8), "vocab_chunk": vc, "launches_per_step": n_launch},
        "roofline": {"bound": "mfma", "kernel": "stats_kernel", "achieved": stats_tflops,
                     "peak": peak, "unit": "TFLOP/s", "frac": stats_tflops / peak,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "launch_ms": stats_avg, "flop_per_launch": logit_flop,
                     # the same launch counted on the valid token rows only (3528 of the 3584 computed)
                     "achieved_on_valid_rows": logit_flop_valid / (stats_avg * 1e-3) / 1e12,
                     "frac_on_valid_rows": logit_flop_valid / (stats_avg * 1e-3) / 1e12 / peak,
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
        "library": {"path": os.path.relpath(K._LIB_PATH, ROOT), "build": K.lib().kd_build_info().decode(),
                    "ablation": K.lib().kd_build_ablation()},
    }
    if out["library"]["ablation"]:
        out["data"] = "synthetic; ABLATION BUILD %d: a measurement build, its results are wrong by design" % \
            out["library"]["ablation"]
    # free the headline problem before the other workloads (the largest needs about 8 GB)
    del dev, gW, gh, ws
    torch.cuda.empty_cache()
    if not args.no_vendor_gemm and not args.teacher_fp8:
        out["roofline"]["vendor_gemm_same_shape"] = vendor_gemm_yardstick(T_comp, V, H_t, H_s)
    names = [n for n in args.other_workloads.split(",") if n and n != args.workload]
    if names:
        out["other_workloads"] = {n: time_other_workload(n) for n in names}
    rows = cfg.T if args.cpu_rows < 0 else min(args.cpu_rows, cfg.T)
    if rows > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, data, rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
