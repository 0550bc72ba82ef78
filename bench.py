"""Benchmark of the breadth-first training-step path on one MI355X.

A "step" is one pass of the whole hot path: forward and backward of the rank's N_loop stages
over N_mb micro-batches in breadth-first order, fp32 main-grad accumulation and the fused Adam
step per stage (bf_run_step with apply_optimizer = 1).  The default workload is the
52B-shaped rank share at S_mb = 1 (8 layers as 4 stages of 2, S_hidden 8192, 64 heads,
S_mlp 32768, S_seq 2048, N_mb 16, bf16 with fp32 main-grads), seeded synthetic inputs
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--no-cpu-baseline]

Protocol of the committed figures (App. E: 50 batches, the first 10 dropped): --warmup 10 --steps 40, which
are the defaults.  `value` is flops / wall-clock mean over the timed steps between device synchronisations;
the median and the minimum of the per-step device times (HIP events around each step) stand beside it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA: 256 CU x 2.4 GHz x 4096 flop/clk/CU
PEAK_HBM_GBS = 8000.0

# name: (N_layers, N_loop, S_hidden, N_heads, S_mlp, S_seq, S_mb, N_mb, dtype, ckpt)
WORKLOADS = {
    "c1": (4, 2, 256, 4, 1024, 128, 1, 4, "fp32", "none"),
    "c2": (6, 3, 2048, 16, 8192, 2048, 1, 8, "bf16", "none"),
    "c3": (8, 4, 8192, 64, 32768, 2048, 1, 16, "bf16", "none"),
    "c4": (8, 4, 8192, 64, 32768, 2048, 4, 4, "bf16", "none"),
    "c5": (16, 16, 6144, 48, 24576, 2048, 1, 32, "bf16", "layer"),
    "c3v": (8, 4, 8192, 64, 32768, 2048, 1, 16, "bf16", "none"),
    "bert": (8, 4, 8192, 64, 32768, 1024, 1, 16, "bf16", "none"),
}
# workloads that differ from the default causal stack without input / output layers
EXTRA = {"c3v": {"S_voc": 50304}, "bert": {"causal": 0}}
WORKLOAD_TEXT = {
    "c1": "tiny GPT stack fp32 (parity case)",
    "c2": "1.3B-shaped stack",
    "c3": "52B-shaped rank share, S_mb=1, N_mb=16",
    "c4": "52B-shaped rank share, S_mb=4, N_mb=4",
    "c5": "deep-loop stress case, N_loop=16, N_mb=32, per-layer checkpoints",
    "c3v": "c3 on token ids: embedding + 8 layers + final LayerNorm, 50304-way output projection and loss",
    "bert": "52B-shaped rank share as the paper measured it: bidirectional attention, S_seq=1024",
}


def time_steps(st, bf, schedule, N_loop, N_mb, S_mb, x, dy, y, dx, steps, warmup, timing):
    """x, dy, y, dx: activations in and out; or token ids, labels, per-micro-batch loss, None for the
    step with input and output layers."""
    import torch
    if dx is None:
        run = lambda tm: st.bf_run_lm_step(schedule, N_loop, N_mb, S_mb, x, dy, y, apply_optimizer=1, timing=tm)
    else:
        run = lambda tm: st.bf_run_step(schedule, N_loop, N_mb, S_mb, x, dy, y, dx, apply_optimizer=1, timing=tm)
    for _ in range(warmup):
        run(0)
    torch.cuda.synchronize()
    reports = []
    t0 = time.perf_counter()
    for _ in range(steps):
        reports.append(run(timing))
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps, reports


def cpu_baseline(w, causal=True):
    """The CPU oracle, as it stands, timed on the host cores on a reduced shape of the same workload: the same
    S_hidden / N_heads / S_seq / S_mb (so the same products), 2 layers as 2 stages, one micro-batch, forward +
    backward in breadth-first order.  The rate is flops of the sample / its time; what the whole step would take
    at that rate is an extrapolation by the exact flop ratio, and labelled so."""
    import numpy as np

    import bf_inputs
    from oracle import formulas as F
    from oracle import stack as K
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, dtype, _ = w
    lyr_s, loop_s, mb_s = min(2, Lyr), min(2, Lyr), 1
    params = bf_inputs.make_params(1, lyr_s, h, f, bf16=dtype == "bf16")
    p64 = [{k: v.astype(np.float64) for k, v in p.items()} for p in params]
    del params
    x, dy = bf_inputs.make_batch(1, mb_s, S_mb, S_seq, h, bf16=dtype == "bf16")
    t0 = time.perf_counter()
    K.run_step(p64, x.astype(np.float64), dy.astype(np.float64), K.SCHED_BF, loop_s, a, causal=causal)
    dt = time.perf_counter() - t0
    per_layer_mb = 3.0 * float(F.fwd_flops_layer_mb(h, S_seq, S_mb)) if f == 4 * h else None
    flops = per_layer_mb * lyr_s * mb_s
    ratio = (Lyr * N_mb) / float(lyr_s * mb_s)
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": flops / dt / 1e12, "unit": "model TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d layers as %d stages x %d micro-batch of the workload's %d x %d (same S_hidden / N_heads / S_seq / "
                      "S_mb), forward+backward, %.1f s; fp64 numpy" % (lyr_s, loop_s, mb_s, Lyr, N_mb, dt),
            "extrapolated": True, "flop_ratio_step_to_sample": ratio, "extrapolated_step_s": dt * ratio}


def power_check(bf, h):
    """One weight-gradient-shaped product (h x h over 2 h tokens) timed on normally distributed and on
    all-zero operands.  The kernel, the shape and the launch are the same, only the switching activity
    differs: the gap between the two rates is what the socket power limit takes."""
    import torch
    M, N, Kd = h, h, 2 * h
    out = {"product": "weight-gradient layout, %d x %d x %d, bf16 operands, fp32 result" % (M, N, Kd)}
    C = torch.empty(M, N, device="cuda:0", dtype=torch.float32)
    for name in ("randn", "zeros"):
        mk = (lambda *sh: torch.randn(*sh, device="cuda:0").bfloat16()) if name == "randn" else \
             (lambda *sh: torch.zeros(*sh, device="cuda:0", dtype=torch.bfloat16))
        A, B = mk(Kd, M), mk(Kd, N)
        run = lambda: bf.bf_op_gemm(bf.BF_BF16, 0, bf.BF_TN, bf.BF_EPI_ACCUM, M, N, Kd, A, B, C, None, None, None, 0)
        for _ in range(3):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            run()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_tflops"] = 2.0 * M * N * Kd * 20 / (e0.elapsed_time(e1) * 1e9)
        del A, B
    return out


T_START = time.time()


def note(msg):
    """A progress line on stderr (stdout carries the one JSON line): a run of some minutes should not look hung."""
    print("bench.py [%5.0f s] %s" % (time.time() - T_START, msg), file=sys.stderr, flush=True)


def step_stats(reports):
    """Median, minimum and maximum of the per-step device times (events around each step on its stream)."""
    ms = sorted(rp.gpu_ms for rp in reports if rp.timed)
    if not ms:
        return None
    n = len(ms)
    return {"median": 0.5 * (ms[(n - 1) // 2] + ms[n // 2]), "min": ms[0], "max": ms[-1], "n": n}


def other_workload(bf, name, steps=3, warmup=1, mb_chains=1):
    """One of the other configurations, BF and DF, a few timed steps after one warm-up: model and executed
    TFLOP/s, step time, peak checkpoints and activation bytes.  The stack is built and freed here.
    mb_chains = 2: the BF step with its micro-batches on two streams (DF is then left out: it runs as one chain)."""
    import torch
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, dtype, ckpt = WORKLOADS[name]
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16,
                         ckpt_mode=bf.BF_CKPT_LAYER if ckpt == "layer" else bf.BF_CKPT_NONE, lr=1e-5, queue_depth=0,
                         fuse_wgrad=1, N_loop_min=N_loop, mb_chains=mb_chains, **EXTRA.get(name, {}))
    st = bf.Stack(cfg, device="cuda:0")
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x221105953)
    shape = (N_mb, S_mb, S_seq, h)
    x = torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    dy = torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    out = {"workload": "%s: %s" % (name, WORKLOAD_TEXT[name]), "N_layers": Lyr, "N_loop": N_loop, "S_hidden": h, "S_mb": S_mb,
           "N_mb": N_mb, "ckpt": ckpt, "steps": steps, "warmup": warmup, "workspace_bytes": int(bf.bf_workspace_bytes(cfg))}
    for tag, sched in (("bf", bf.BF_SCHED_BF), ("df", bf.BF_SCHED_DF)):
        if mb_chains == 2 and tag == "df":
            continue
        sec, reps = time_steps(st, bf, sched, N_loop, N_mb, S_mb, x, dy, y, dx, steps, warmup, 1)
        rp = reps[-1]
        out[tag] = {"mb_chains": int(rp.mb_chains), "ms_per_step": sec * 1e3, "gpu_ms": step_stats(reps), "model_tflops": rp.flops_model / sec / 1e12,
                    "frac_bf16_mfma_peak": rp.flops_model / sec / 1e12 / PEAK_BF16_TFLOPS,
                    "executed_tflops": rp.flops_executed / sec / 1e12,
                    "executed_frac_bf16_mfma_peak": rp.flops_executed / sec / 1e12 / PEAK_BF16_TFLOPS,
                    "tokens_per_s": N_mb * S_mb * S_seq / sec,
                    "peak_ckpt_count": rp.peak_ckpt_count, "peak_ckpt_bytes": rp.peak_ckpt_bytes,
                    "peak_act_bytes": rp.peak_act_bytes, "fused_wgrad_bytes": rp.fused_wgrad_bytes}
    st.close()
    del st, x, dy, y, dx
    torch.cuda.empty_cache()
    return out


def sweep(bf, w, extra, which):
    """The workload in both orders over the micro-batch count (1 .. N_mb, powers of two) or over the
    loop count (the divisors of N_layers): one-GPU counterparts of the paper's sweeps of Fig. 5 and
    Fig. 6.  Untimed launches (timing 0), optimizer on, wall clock between device synchronisations."""
    import torch
    Lyr, N_loop0, h, a, f, S_seq, S_mb, N_mb0, dtype, ckpt = w
    b16 = dtype == "bf16"
    td = torch.bfloat16 if b16 else torch.float32
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x221105953)
    X = torch.randn((N_mb0, S_mb, S_seq, h), generator=gen, device="cuda:0", dtype=torch.float32).to(td)
    DY = torch.randn((N_mb0, S_mb, S_seq, h), generator=gen, device="cuda:0", dtype=torch.float32).to(td)
    if which == "N_mb":
        points = [(N_loop0, n) for n in (1, 2, 4, 8, 16, 32, 64) if n <= N_mb0]
    else:
        points = [(n, N_mb0) for n in range(1, Lyr + 1) if Lyr % n == 0]
    out, st, made_for = [], None, None
    for N_loop, N_mb in points:
        if made_for != N_loop:
            if st is not None:
                st.close()
                del st
                torch.cuda.empty_cache()
            cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb0, S_mb, dtype=bf.BF_BF16 if b16 else bf.BF_FP32,
                                 ckpt_mode=bf.BF_CKPT_LAYER if ckpt == "layer" else bf.BF_CKPT_NONE, lr=1e-5, queue_depth=0,
                                 fuse_wgrad=1, N_loop_min=N_loop, **extra)
            st, made_for = bf.Stack(cfg, device="cuda:0"), N_loop
        x, dy = X[:N_mb].contiguous(), DY[:N_mb].contiguous()
        y, dx = torch.empty_like(x), torch.empty_like(x)
        p = {"N_loop": N_loop, "N_mb": N_mb, "workspace_bytes": int(bf.bf_workspace_bytes(cfg))}
        for name, sched in (("bf", bf.BF_SCHED_BF), ("df", bf.BF_SCHED_DF)):
            sec, reps = time_steps(st, bf, sched, N_loop, N_mb, S_mb, x, dy, y, dx, 3 if N_mb >= 4 else 8, 1, 0)
            p[name] = {"ms_per_step": sec * 1e3, "model_tflops": reps[-1].flops_model / sec / 1e12}
        out.append(p)
    st.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-df", action="store_true")
    ap.add_argument("--no-fuse-wgrad", action="store_true",
                    help="accumulate weight gradients per micro-batch in BF order too (default: one product per stage)")
    ap.add_argument("--no-dp-fs", action="store_true",
                    help="skip the fully-sharded (dp_fs = 1) BF and DF steps reported under \"dp_fs\"")
    ap.add_argument("--no-power-check", action="store_true",
                    help="skip the product timed on random and on zero operands reported under \"power_check\"")
    ap.add_argument("--sweep", choices=["N_mb", "N_loop"],
                    help="instead of the benchmark line: both orders over the micro-batch count or the loop count")
    ap.add_argument("--mb-chains", type=int, default=1, choices=[1, 2],
                    help="2: the micro-batches of the BF step on two streams (stacks without S_voc; the dp_fs steps are skipped)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the c2 / c4 / c5 steps (BF and DF) reported under \"other_workloads\" of the default workload")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one pipeline rank's share of the step); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2211_05953_amd as bf
    bf.load()   # no fallback: a missing library is an error
    w = WORKLOADS[args.workload]
    if args.mb_chains == 2 and EXTRA.get(args.workload, {}).get("S_voc"):
        print("bench.py: --mb-chains 2 runs the stack on activations (workloads without S_voc)", file=sys.stderr)
        sys.exit(2)
    Lyr, N_loop, h, a, f, S_seq, S_mb, N_mb, dtype, ckpt = w
    b16 = dtype == "bf16"
    cfg = bf.make_config(h, a, f, S_seq, Lyr, N_mb, S_mb, dtype=bf.BF_BF16 if b16 else bf.BF_FP32,
                         ckpt_mode=bf.BF_CKPT_LAYER if ckpt == "layer" else bf.BF_CKPT_NONE, lr=1e-5, queue_depth=0,
                         fuse_wgrad=0 if args.no_fuse_wgrad else 1, N_loop_min=N_loop, mb_chains=args.mb_chains,
                         **EXTRA.get(args.workload, {}))
    S_voc = cfg.S_voc
    torch.cuda.set_device(0)
    if args.sweep:
        if S_voc:
            print("bench.py: --sweep runs the stack on activations (workloads without S_voc)", file=sys.stderr)
            sys.exit(2)
        print(json.dumps({"sweep": args.sweep, "workload": "%s: %s" % (args.workload, WORKLOAD_TEXT[args.workload]),
                          "unit": "model TFLOP/s", "data": "synthetic",
                          "points": sweep(bf, w, EXTRA.get(args.workload, {}), args.sweep)}))
        return
    # A 1 GiB device copy of known traffic (1 GiB read, 1 GiB written) opens every run: a rocprofv3 --pmc
    # collection of this command scales its FETCH_SIZE / WRITE_SIZE readings by what they read for it.
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    torch.cuda.empty_cache()
    st = bf.Stack(cfg, device="cuda:0")
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0x221105953)
    td = torch.bfloat16 if b16 else torch.float32
    shape = (N_mb, S_mb, S_seq, h)
    if S_voc:
        # token ids with a Zipf-like law (a few frequent tokens, a long tail), labels = next token
        wz = 1.0 / torch.arange(1, S_voc + 1, device="cuda:0", dtype=torch.float64) ** 1.1
        stream = torch.multinomial(wz / wz.sum(), N_mb * S_mb * (S_seq + 1), replacement=True, generator=gen)
        stream = stream.to(torch.int32).reshape(N_mb, S_mb, S_seq + 1)
        x, dy = stream[..., :-1].contiguous(), stream[..., 1:].contiguous()
        y, dx = torch.zeros(N_mb, device="cuda:0"), None
    else:
        x = torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32).to(td)
        dy = torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32).to(td)
        y, dx = torch.empty_like(x), torch.empty_like(x)

    # The timed region: the step as it runs in production (Adam of a stage as soon as its gradient is
    # final), with HIP events around the weight-gradient products only, the
    # class with the most time (timing 3: 64 events per step at C3 instead of 2000 and more).
    note("%s: breadth-first, %d warm-up + %d timed steps" % (args.workload, args.warmup, args.steps))
    sec_bf, rep_bf = time_steps(st, bf, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, x, dy, y, dx, args.steps, args.warmup, 3)
    r = rep_bf[-1]
    note("breadth-first: %.1f ms per step" % (sec_bf * 1e3))
    out_df = None
    if not args.no_df:
        # the other order under the same protocol, at a quarter of the steps (its time is not the headline)
        k_df, w_df = max(3, args.steps // 4), max(1, args.warmup // 4)
        sec_df, rep_df = time_steps(st, bf, bf.BF_SCHED_DF, N_loop, N_mb, S_mb, x, dy, y, dx, k_df, w_df, 1)
        note("depth-first: %.1f ms per step" % (sec_df * 1e3))
        rd = rep_df[-1]
        out_df = {"ms_per_step": sec_df * 1e3, "steps": k_df, "warmup": w_df, "gpu_ms": step_stats(rep_df),
                  "model_tflops": rd.flops_model / sec_df / 1e12,
                  "peak_ckpt_count": rd.peak_ckpt_count, "peak_ckpt_bytes": rd.peak_ckpt_bytes,
                  "peak_act_bytes": rd.peak_act_bytes}
    # one plain-timed BF step (no per-launch events at all), and two fully instrumented ones (events around
    # every launch, Adam in line on the main stream so that nothing is timed together with it) for the
    # other classes
    sec_plain, _ = time_steps(st, bf, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, x, dy, y, dx, 1, 0, 1)
    sec_instr, rep_instr = time_steps(st, bf, bf.BF_SCHED_BF, N_loop, N_mb, S_mb, x, dy, y, dx, 2, 0, 2)
    note("instrumented steps done")

    def classes(reps):
        out = {}
        for i, name in enumerate(bf.binding.KERNEL_CLASSES):
            ms = sum(rp.kernel_ms[i] for rp in reps) / len(reps)
            n = sum(rp.kernel_launches[i] for rp in reps) / len(reps)
            fl = sum(rp.kernel_flops[i] for rp in reps) / len(reps)
            by = sum(rp.kernel_bytes[i] for rp in reps) / len(reps)
            if n:
                out[name] = {"ms_per_step": ms, "launches": n, "avg_launch_ms": ms / n,
                             "tflops": fl / ms / 1e9 if fl else None, "gbs": by / ms / 1e6 if by else None}
        return out
    kern = classes(rep_instr)          # every class, from the instrumented steps
    kern.update(classes(rep_bf))       # the weight-gradient products, from the timed region itself
    # the dominant kernel: one instantiation, the fused weight-gradient product (the forward class is
    # three instantiations of similar total)
    dom = "gemm_wgrad" if "gemm_wgrad" in kern else max((k for k in kern if k.startswith("gemm")), key=lambda k: kern[k]["ms_per_step"])
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kern[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": kern[dom]["tflops"] / PEAK_BF16_TFLOPS, "traffic": None,
                "flops_per_launch": kern[dom]["tflops"] * 1e9 * kern[dom]["avg_launch_ms"],
                "avg_launch_ms": kern[dom]["avg_launch_ms"]}
    # HBM-side bytes per launch of that kernel.  `traffic` is not measured in this run: it is read from
    # profiles/traffic.json, which holds what two rocprofv3 --pmc collections (FETCH_SIZE, WRITE_SIZE, scaled by
    # the opening copy's readings) gave for this command.  The algorithmic bytes (every operand read once,
    # the result written once) stand beside it.
    roofline["traffic_algorithmic"] = sum(rp.kernel_bytes[bf.binding.KERNEL_CLASSES.index(dom)] for rp in rep_bf) / \
        max(1, sum(rp.kernel_launches[bf.binding.KERNEL_CLASSES.index(dom)] for rp in rep_bf))
    roofline["traffic_source"] = None
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        t = json.load(open(traffic_file)).get(args.workload, {}).get(dom)
        if t:
            roofline["traffic"] = t
            roofline["traffic_source"] = "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, " \
                                         "a committed constant, not measured in this run)"

    value = r.flops_model / sec_bf / 1e12
    line = {
        "metric": "model TFLOP/s per training step at S_mb=1, BF order (3x forward flops, full attention)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_bf * 1e3, "gpu_ms": step_stats(rep_bf),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: %s" % (args.workload, WORKLOAD_TEXT[args.workload]), "N_layers": Lyr, "N_loop": N_loop,
                   "S_hidden": h, "N_heads": a, "S_mlp": f, "S_seq": S_seq, "S_mb": S_mb, "N_mb": N_mb,
                   "schedule": "BF", "ckpt": ckpt, "causal": int(cfg.causal), "S_voc": int(S_voc), "fuse_wgrad": not args.no_fuse_wgrad, "mb_chains": int(r.mb_chains), "tokens_per_step": N_mb * S_mb * S_seq},
        "frac_bf16_mfma_peak": value / PEAK_BF16_TFLOPS,
        "paper_eq_tflops": r.flops_paper / sec_bf / 1e12,
        "executed_tflops": r.flops_executed / sec_bf / 1e12,
        "tokens_per_s": N_mb * S_mb * S_seq / sec_bf,
        "bf": {"peak_ckpt_count": r.peak_ckpt_count, "peak_ckpt_bytes": r.peak_ckpt_bytes,
               "peak_act_bytes": r.peak_act_bytes, "fused_wgrad_bytes": r.fused_wgrad_bytes,
               "state_bytes": r.state_bytes, "adam_ms": r.adam_ms,
               "ms_per_step_without_launch_events": sec_plain * 1e3,
               "ms_per_step_with_events_on_every_launch": sec_instr * 1e3},
        "df": out_df,
        "kernels": kern,
        "roofline": roofline,
    }
    st.close()
    del st
    torch.cuda.empty_cache()
    if b16 and not args.no_dp_fs and args.mb_chains == 1:
        # the same step with the bf16 weights rebuilt per interval of use into a two-stage double buffer
        # (Sec. 3.1, App. D.1): BF rebuilds a stage twice per step, DF twice per micro-batch
        cfg.dp_fs = 1
        fs = bf.Stack(cfg, device="cuda:0")
        out_fs = {}
        for name, sched, k in (("bf", bf.BF_SCHED_BF, min(args.steps, 3)), ("df", bf.BF_SCHED_DF, min(args.steps, 2))):
            if name == "df" and args.no_df:
                continue
            # timed as it runs (reconstruction on the side stream under the compute of the other half);
            # one instrumented step afterwards for the time the reconstruction kernels take by themselves
            sec, _ = time_steps(fs, bf, sched, N_loop, N_mb, S_mb, x, dy, y, dx, k, 1, 1)
            _, reps = time_steps(fs, bf, sched, N_loop, N_mb, S_mb, x, dy, y, dx, 1, 0, 2)
            rp = reps[-1]
            i = bf.binding.KERNEL_CLASSES.index("reconstruct")
            out_fs[name] = {"ms_per_step": sec * 1e3, "model_tflops": rp.flops_model / sec / 1e12,
                            "n_weight_intervals": rp.n_weight_intervals, "n_reconstruct": rp.n_reconstruct,
                            "reconstruct_bytes": rp.reconstruct_bytes, "reconstruct_ms": rp.kernel_ms[i],
                            "weight_buffer_bytes": rp.weight_buffer_bytes, "state_bytes": rp.state_bytes}
        line["dp_fs"] = out_fs
        note("fully sharded steps done")
        fs.close()
        del fs
    del x, dy, y, dx
    torch.cuda.empty_cache()
    if args.workload == "c3" and not args.no_other_workloads:
        line["other_workloads"] = {}
        for name in ("c2", "c4", "c5"):
            line["other_workloads"][name] = other_workload(bf, name)
            note("%s done" % name)
        # the small stack and the 6144-wide one (192 tiles on 256 compute units in five of its eight products per
        # layer) again with two micro-batches in flight: their kernels do not fill the chip one at a time
        line["other_workloads"]["c2_two_chains"] = other_workload(bf, "c2", mb_chains=2)
        line["other_workloads"]["c5_two_chains"] = other_workload(bf, "c5", mb_chains=2)
        note("c2 and c5 with two chains done")
    if b16 and not args.no_power_check and h % 256 == 0:
        line["power_check"] = power_check(bf, h)
        note("power check done")
    if not args.no_cpu_baseline:
        note("CPU oracle on the reduced sample (about half a minute)")
        line["cpu_baseline"] = cpu_baseline(w, causal=bool(EXTRA.get(args.workload, {}).get("causal", 1)))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
