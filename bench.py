#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: mtnlg_stage_step (forward + backward of one GPU's
tensor-parallel slice of a 3-layer pipeline stage) at MT-NLG's per-GPU shapes.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Prints ONE JSON line.  `value` is model TFLOP/s of the whole step (3x forward, attention counted on
the causal half), inputs resident in HBM.  `roofline` is for the dominant kernel class (the bf16 MFMA
GEMMs), timed live with HIP events on the launch stream during the timed steps.  `cpu_baseline` is the
fp64 oracle timed on the host cores on a bounded sample (a causal prefix of one layer).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0     # MI355X HBM3E


def measured_peaks(x, reps=5):
    """What the chip sustains in this process, on this data, before the timed steps: (a) a loop of nothing but bf16
    matrix-core instructions (mtnlg_calibrate_mfma) on operands drawn like the workload's activations, long enough
    (about 20 ms a launch) for the clock to settle under the power limit; (b) a plain streaming copy of 1 GiB
    (mtnlg_calibrate_copy).  Both are timed with events on the launch stream."""
    import torch

    import paper_2201_11990_amd as M

    wgs, iters = 256 * 4, 3000
    n = M.mtnlg_calibrate_mfma_operand_bytes(wgs) // 2
    ops = x.reshape(-1)
    ops = ops[:n].contiguous() if ops.numel() >= n else torch.randn(n, device=x.device).bfloat16()
    out = torch.empty(wgs * 512, device=x.device)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=x.device).fill_(1)
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_mfma = timed(lambda: M.mtnlg_calibrate_mfma(wgs, iters, ops, out))
    zeros = torch.zeros_like(ops)   # the same loop on zeros: what the matrix pipes do when the data toggles nothing
    ms_zero = timed(lambda: M.mtnlg_calibrate_mfma(wgs, iters, zeros, out))
    ms_copy = timed(lambda: M.mtnlg_calibrate_copy(dst, src))
    fl = M.mtnlg_calibrate_mfma_flops(wgs, iters)
    return {"mfma_tflops": fl / (ms_mfma * 1e-3) / 1e12, "mfma_ms": ms_mfma,
            "mfma_tflops_zeros": fl / (ms_zero * 1e-3) / 1e12,
            "copy_gbps": 2 * (1 << 30) / (ms_copy * 1e-3) / 1e9, "copy_ms": ms_copy}


def gemm_flops_per_step(wl):
    """FLOPs of one stage step that run in each GEMM kernel class (forward NT, dgrad NN, wgrad TN)."""
    T, h, p, F = wl.tokens, wl.hidden, wl.proj, wl.ffn
    per_layer = 2 * T * (h * 3 * p + p * h + h * F + F * h)
    fwd_passes = 2 if wl.recompute else 1  # a recomputed forward reruns QKV, proj, FC1 (not FC2)
    nt = per_layer + (fwd_passes - 1) * (per_layer - 2 * T * F * h) * (wl.n_layers - 1) / wl.n_layers
    return {"gemm_nt": wl.n_layers * nt, "gemm_nn": wl.n_layers * per_layer, "gemm_tn": wl.n_layers * per_layer}


def cpu_baseline(wl, weights0, x, prefix):
    """Time the oracle (as it stands) on layer 0 restricted to the first `prefix` tokens: by causality
    that is exactly the `prefix`-token problem with the full-width weights."""
    import numpy as np
    import torch

    import oracle
    from paper_2201_11990_amd import flops

    dims = oracle.Dims(wl.hidden, wl.heads, wl.head_dim, wl.ffn, prefix, wl.micro_batch)
    w = {k: v.detach().to("cpu", torch.float64).numpy() for k, v in weights0.items()}
    xs = x[:, :prefix].detach().to("cpu", torch.float64).numpy().reshape(-1, wl.hidden)
    dy = np.random.default_rng(0).standard_normal(xs.shape)
    t0 = time.perf_counter()
    _, saved = oracle.layer_fwd(dims, w, xs)
    oracle.layer_bwd(dims, w, xs, saved, dy)
    dt = time.perf_counter() - t0
    fl = 3 * flops.layer_forward_flops(wl.hidden, wl.heads, wl.head_dim, wl.ffn, prefix, wl.micro_batch)
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 oracle, layer 0 fwd+bwd on the first {prefix} tokens (causal prefix, full-width "
                      f"weights), {fl / 1e9:.1f} GFLOP in {dt:.1f} s"}


def lm_head_bench(wl, vocab_local=6400, reps=10):
    """mtnlg_lm_head_step at the slice's shape: T tokens, hidden h, 6400 rows of the tied embedding (GPT-2's
    vocabulary padded to 51200, one of 8 slices; the paper gives no vocabulary size).  FLOPs = the three GEMMs
    (logits, dgrad, wgrad), 6 T V h."""
    import torch

    import paper_2201_11990_amd as M
    from paper_2201_11990_amd import binding as B

    T, h = wl.tokens, wl.hidden
    dev = "cuda"
    x = torch.randn((T, h), device=dev).bfloat16()
    gamma, beta = torch.ones(h, device=dev).bfloat16(), torch.zeros(h, device=dev).bfloat16()
    E = (torch.randn((vocab_local, h), device=dev) * 0.004).bfloat16()
    targets = torch.randint(0, vocab_local, (T,), device=dev, dtype=torch.int32)
    desc = B.head_desc(h, vocab_local, 0, wl.seq, wl.micro_batch, "bf16")
    ws = torch.empty(M.mtnlg_lm_head_workspace(desc), dtype=torch.uint8, device=dev)
    loss = torch.empty(T, device=dev)
    dx, dg, db, dE = torch.empty_like(x), torch.empty_like(gamma), torch.empty_like(beta), torch.empty_like(E)

    def step():
        M.mtnlg_lm_head_step(desc, x, gamma, beta, E, targets, None, loss, dx, dg, db, dE, ws)

    step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    fl = 6.0 * T * vocab_local * h
    return {"tokens": T, "hidden": h, "vocab_local": vocab_local, "ms": round(ms, 3),
            "achieved": round(fl / (ms * 1e-3) / 1e12, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "bound": "mfma",
            "mean_loss": round(float(loss.mean()), 4)}


def optimizer_step_bench(weights, reps=3):
    """Adam step over every parameter of the stage: one squared-norm pass over the fp32 gradients (4 B read per
    parameter), then the fused update (16 B read, 14 B written per parameter: fp32 weight and both moments in
    place, bf16 weight out).  Reports achieved HBM bandwidth on those algorithmic bytes."""
    import torch

    import paper_2201_11990_amd as M

    tensors = [t for w in weights for t in w.values()]
    n = sum(t.numel() for t in tensors)
    state = [(t.float().contiguous(), torch.zeros(t.shape, device=t.device), torch.zeros(t.shape, device=t.device),
              torch.randn(t.shape, device=t.device) * 1e-3) for t in tensors]
    ws = torch.empty(M.mtnlg_grad_sqnorm_workspace(), dtype=torch.uint8, device=tensors[0].device)
    sq = torch.zeros(1, device=tensors[0].device)

    def step(t):
        for i, (_, _, _, g) in enumerate(state):
            M.mtnlg_grad_sqnorm(g, ws, sq, accumulate=i > 0)
        for w16, (p, m, v, g) in zip(tensors, state):
            M.mtnlg_adam_step(p, m, v, g, w16, sq, lr=5e-5, step=t, weight_decay=0.1 if w16.dim() > 1 else 0.0)

    step(1)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for r in range(reps):
        step(2 + r)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    gbs = n * 34 / (ms * 1e-3) / 1e9
    return {"parameters": n, "ms": round(ms, 3), "bytes_per_parameter": 34, "achieved": round(gbs, 1), "peak": 8000.0,
            "unit": "GB/s", "frac": round(gbs / 8000.0, 4), "bound": "hbm"}


# kernel symbol of each GEMM class in the rocprofv3 summaries: gemm_stream_kernel<BM, BN, A transposed, B transposed, ...>
CLASS_SYMBOL = {"gemm_nt": r"gemm_stream_kernel<\d+, \d+, false, false", "gemm_nn": r"gemm_stream_kernel<\d+, \d+, false, true",
                "gemm_tn": r"gemm_stream_kernel<\d+, \d+, true, true"}


def counter_traffic(cls):
    """HBM-side bytes per launch of a GEMM class (FETCH_SIZE + WRITE_SIZE, each scaled by a copy kernel of
    known size) from the committed summary of the two rocprofv3 --pmc runs of this benchmark; None when the
    summary is missing.  Counters cannot be read from inside the timed run."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "stage_step_mtnlg_tp8_hbm_traffic.txt")
    try:
        line = [l for l in open(path) if l.startswith("TRAFFIC_TABLE ")][0]
        table = json.loads(line[len("TRAFFIC_TABLE "):])
    except (OSError, IndexError, ValueError):
        return None
    import re
    rows = [v for k, v in table.items() if re.match(CLASS_SYMBOL[cls], k)]
    n = sum(r["launches"] for r in rows)
    return int(sum(r["launches"] * r["bytes_per_launch"] for r in rows) / n) if n else None



def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="mtnlg_tp8_stage")
    ap.add_argument("--cpu-prefix", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="before the timed steps, run one plain streaming copy of BYTES (mtnlg_calibrate_copy: a kernel "
                         "of known size to calibrate FETCH_SIZE / WRITE_SIZE counters against)")
    ap.add_argument("--micro-batches", type=int, default=1, metavar="K",
                    help="a step = K micro-batches through mtnlg_stage_step_accumulate with fp32 gradient buffers "
                         "(gradient accumulation); default 1 = the plain step the metric is quoted on")
    ap.add_argument("--lm-head", action="store_true",
                    help="also time the last stage's extras (final LayerNorm, tied output projection on a 6400-row "
                         "vocabulary slice, cross-entropy, and back) and add an `lm_head_step` object to the line")
    ap.add_argument("--optimizer-step", action="store_true",
                    help="also time the Adam step (squared gradient norm + fused update) over all parameters of the "
                         "stage and add an `optimizer_step` object (HBM roofline) to the line")
    ap.add_argument("--no-measured-peak", action="store_true",
                    help="skip the matrix-core-only loop and the 1 GiB copy that measure what the chip sustains")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the HIP-event bracketing of kernels (roofline.achieved becomes null)")
    ap.add_argument("--kernel-timing-every", type=int, default=4, metavar="N",
                    help="bracket the kernels of every N-th timed step with HIP events (the events cost 0.6 %% of a "
                         "step); 1 = every step")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2201_11990_amd as M
    from paper_2201_11990_amd import flops
    from paper_2201_11990_amd.inputs import WORKLOADS, make_activations, make_layer_params
    from paper_2201_11990_amd.runner import StageRunner

    wl = WORKLOADS[args.workload]
    if wl.dtype != "bf16":
        print("bench.py: benchmark workloads are bf16", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = "cuda"
    weights = [make_layer_params(wl, l, seed=0, device=dev) for l in range(wl.n_layers)]
    x, dy = make_activations(wl, seed=0, device=dev)
    if args.micro_batches > 1:
        from paper_2201_11990_amd import binding as B
        run = StageRunner(wl, weights, flags=B.WGRAD_FP32, device=dev)
        xs = torch.stack([make_activations(wl, seed=m, device=dev)[0] for m in range(args.micro_batches)])
        dys = torch.stack([make_activations(wl, seed=m, device=dev)[1] for m in range(args.micro_batches)])

        def one_step():
            run.step_accumulate(xs, dys)
    else:
        run = StageRunner(wl, weights, device=dev)

        def one_step():
            run.step(x, dy)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    peaks = None if args.no_measured_peak else measured_peaks(x)
    if peaks is not None:   # the probe leaves the chip hot and clocked down: let one untimed step pass
        one_step()
        torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(args.copy_calibration, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        M.mtnlg_calibrate_copy(dst, src)   # calibrate_copy_kernel in the profiler's listing
        torch.cuda.synchronize()
        del src, dst
    every = max(1, args.kernel_timing_every)
    sampled = [i for i in range(args.steps) if i % every == 0]
    if not args.no_kernel_timing:
        M.mtnlg_profile_enable(True)
        M.mtnlg_profile_pause(True)
    # one event after every step (on the stream the steps run on) gives the spread over the steps; the
    # headline time stays the wall clock around all of them
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        timed_kernels = not args.no_kernel_timing and i % every == 0
        if timed_kernels:
            M.mtnlg_profile_pause(False)
        one_step()
        if timed_kernels:
            M.mtnlg_profile_pause(True)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    prof = None
    if not args.no_kernel_timing:
        prof = M.mtnlg_profile_read()
        M.mtnlg_profile_enable(False)

    ms = dt / args.steps * 1e3
    model = flops.step_model_flops(wl, "causal") * args.micro_batches
    value = model / (ms * 1e-3) / 1e12
    out = {
        "metric": "model TFLOP/s per GPU, MT-NLG TP=8-slice layer fwd+bwd; % of bf16 MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "ms_per_step_median": round(per_step[len(per_step) // 2], 4),
        "ms_per_step_min": round(per_step[0], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "hidden": wl.hidden, "heads_local": wl.heads, "head_dim": wl.head_dim,
                   "ffn_local": wl.ffn, "seq": wl.seq, "micro_batch": wl.micro_batch, "n_layers": wl.n_layers,
                   "tp_size": wl.tp_size, "recompute": wl.recompute, "micro_batches_per_step": args.micro_batches,
                   "parallelism": "one GPU's TP slice, no collectives"},
        "pct_of_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "model_tflops_paper_convention": round(args.micro_batches * flops.step_model_flops(wl, "full") / (ms * 1e-3) / 1e12, 2),
        "hardware_tflops": round(args.micro_batches * flops.step_hardware_flops(wl, "causal") / (ms * 1e-3) / 1e12, 2),
    }
    if prof is not None:
        gf = {k: v * args.micro_batches for k, v in gemm_flops_per_step(wl).items()}
        nsamp = len(sampled)   # steps whose kernels were bracketed
        classes = {}
        for k, (n, tms) in prof.items():
            if n:
                classes[k] = {"launches_per_step": n / nsamp, "ms_per_step": round(tms / nsamp, 4)}
        dom = max(("gemm_nt", "gemm_nn", "gemm_tn"), key=lambda k: prof[k][1])
        g_ms = sum(prof[k][1] for k in gf) / nsamp
        for k in gf:
            classes[k]["tflops"] = round(gf[k] / (prof[k][1] / nsamp * 1e-3) / 1e12, 1)
        ach = gf[dom] / (prof[dom][1] / nsamp * 1e-3) / 1e12
        # the counter summary was taken on the default workload only
        traffic = counter_traffic(dom) if wl.name == "mtnlg_tp8_stage" and args.micro_batches == 1 else None
        out["roofline"] = {"bound": "mfma", "kernel": dom, "achieved": round(ach, 1), "peak": PEAK_BF16_TFLOPS,
                           "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                           "traffic_source": "profiles/stage_step_mtnlg_tp8_hbm_traffic.txt (two rocprofv3 --pmc runs "
                                             "of this command; counters cannot be read inside the timed run)",
                           "all_gemm_tflops": round(sum(gf.values()) / (g_ms * 1e-3) / 1e12, 1),
                           "gemm_share_of_step": round(g_ms / ms, 3),
                           "kernel_timed_steps": nsamp}
        if peaks is not None:
            # the same fractions against what a loop of nothing but matrix-core instructions sustains here
            out["roofline"]["measured_peak"] = round(peaks["mfma_tflops"], 1)
            out["roofline"]["measured_peak_zero_operands"] = round(peaks["mfma_tflops_zeros"], 1)
            out["roofline"]["frac_of_measured"] = round(ach / peaks["mfma_tflops"], 4)
            out["pct_of_measured_mfma_loop"] = round(100 * value / peaks["mfma_tflops"], 2)
        # bandwidth-bound classes: achieved GB/s on their algorithmic bytes against the HBM peak
        per_launch = flops.hbm_bytes_per_launch(wl)
        for k, nbytes in per_launch.items():
            if k in classes and prof[k][1] > 0:
                gbps = prof[k][0] * nbytes / (prof[k][1] * 1e-3) / 1e9
                classes[k].update({"bound": "hbm", "bytes_per_launch": int(nbytes), "gbps": round(gbps, 1),
                                   "frac_hbm": round(gbps / PEAK_HBM_GBPS, 4)})
        out["kernel_classes"] = classes
        if peaks is not None:
            out["hbm_copy_1gib"] = {"ms": round(peaks["copy_ms"], 4), "gbps": round(peaks["copy_gbps"], 1),
                                    "frac_hbm": round(peaks["copy_gbps"] / PEAK_HBM_GBPS, 4)}
    else:
        out["roofline"] = {"bound": "mfma", "achieved": None, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                           "frac": None, "traffic": None}
    if args.lm_head:
        out["lm_head_step"] = lm_head_bench(wl)
    if args.optimizer_step:
        del run
        out["optimizer_step"] = optimizer_step_bench(weights)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, weights[0], x, args.cpu_prefix)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
