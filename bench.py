#!/usr/bin/env python3
"""Benchmark of the AdLoCo hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
  adloco_grad_stats   GPT-2-small-shaped workload: 12 blocks x {768->2304, 768->768, 768->3072,
                      3072->768}, B = 32, T = 512, bf16 a ~ N(0,1), delta ~ N(0,1e-2):
                      Gram kernel (per-sample norms), gradient-sum GEMM, reductions
  adloco_norm_test    ||sum_i g_i||^2, norm test, batch rule, SwitchMode (eta = 0.3)
  adloco_check_merge  host
  adloco_outer_step   M = 4 instances x 124M fp32 parameters, Nesterov (lr 0.7, mu 0.9), in place
  adloco_merge        S = 4 instances, weights = requested batches, in place
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

DT = None                    # element type code / torch dtype of a and delta, set from --dtype
TDT = None
PEAK_BF16_MFMA = 2.5e15     # dense bf16 MFMA flop/s, MI355X
PEAK_HBM = 8.0e12           # bytes/s
TILE = 128                  # T-tile edge of the Gram kernel (executed-flop accounting)


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=3)
    p.add_argument("--gram-variant", type=int, default=None)
    p.add_argument("--wgrad-variant", type=int, default=None)
    p.add_argument("--stream-blocks-per-cu", type=int, default=None)
    p.add_argument("--stats-variant", default="tile", choices=["tile", "gram"],
                   help="route of the statistics in the timed step: per-sample gradient tiles fused "
                        "with the gradient sum (default), or Gram kernel + gradient-sum GEMM")
    p.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                   help="storage type of activations and output gradients (both run the same "
                        "kernels; the metric is quoted on bf16)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--cpu-blocks", type=int, default=12,
                   help="transformer blocks (of 12) the CPU oracle is timed on")
    p.add_argument("--grad-provided", action="store_true",
                   help="caller supplies the gradient sum (skips the gradient-sum GEMM)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run three plain 1 GiB device copies (untimed) so that a counter "
                        "profile of this command holds a kernel of known traffic")
    p.add_argument("--config", type=int, default=2, choices=[2, 4, 5],
                   help="2 (default, the benchmark workload): GPT-2-small statistics + 124M x 4 outer "
                        "step; 4: transformer blocks of the Llama-1B-shaped workload (statistics only); "
                        "5: blocks of the 350M round + its M = 8 outer step and merge")
    p.add_argument("--blocks", type=int, default=None,
                   help="transformer blocks of --config 4 / 5 to hold in memory (default 2)")
    p.add_argument("--no-next-rows", action="store_true",
                   help="skip the extra leg that times the bias / gain / embedding blocks")
    p.add_argument("--only", default="all", choices=["all", "stats", "outer"],
                   help="time only one half (diagnostics; the JSON line says so)")
    return p.parse_args()


def gram_flops(shapes, B, T):
    """(symmetric-half algorithmic, full, executed by the tile-pair kernel) flops per launch."""
    dsum = sum(di + do for _, di, do in shapes)
    nt = -(-T // TILE)
    # 128 x 128 tile pairs: nt(nt-1)/2 off the diagonal, nt on it, where one of the four 64 x 64
    # wave tiles mirrors another and is not computed and the two on the diagonal leave out one of
    # their four 32 x 32 blocks: (0.75 + 0.75 + 1 + 0) / 4 of a pair
    pairs = nt * (nt - 1) / 2 + 0.625 * nt
    sym = B * T * (T + 1) * dsum
    full = 2 * B * T * T * dsum
    executed = 0
    for _, di, do in shapes:
        kp = -(-di // 64) * 64 + -(-do // 64) * 64      # k-chunks of 64 are zero padded
        executed += B * pairs * 2 * TILE * TILE * kp
    return sym, full, int(executed)


def cpu_baseline(synth, orc, shapes, B, T, N, M, blocks):
    """The oracle, as it stands, on a bounded sample of the same workload: `blocks` of the 12
    transformer blocks (all samples), and the outer step + merge on N/4 parameters."""
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    n_blocks = len(shapes) // 4
    t_stats = 0.0
    for b in range(blocks):
        layers = synth.grad_stats_inputs(2, linears=range(4 * b, 4 * b + 4), B=B, T=T)
        t0 = time.perf_counter()
        st = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=False)
        orc.norm_test(st["S1"], st["S2"], B, 0.3, B, 32)
        t_stats += time.perf_counter() - t0
        del layers, st
    n_s = N // 4
    theta, insts, mom = synth.outer_inputs(3, N=n_s, M=M)
    t0 = time.perf_counter()
    orc.outer_step(theta, insts, mom, 0.7, 0.9, True)
    orc.merge(insts, [32.0 + k for k in range(M)])
    t_outer = time.perf_counter() - t0
    t_est = t_stats * n_blocks / blocks + 4 * t_outer
    return dict(value=B * T / t_est, unit="tokens/s", cores=int(cores), kind="oracle",
                sample=(f"{blocks} of {n_blocks} blocks ({4 * blocks} linears, all {B} samples, "
                        f"T={T}) took {t_stats:.2f} s; outer step + merge on N/4 = {n_s} params "
                        f"took {t_outer:.2f} s; step time scaled linearly to {n_blocks} blocks "
                        f"and N params: {t_est:.1f} s"),
                grad_stats_tokens_per_s=B * T / (t_stats * n_blocks / blocks),
                outer_merge_GBps=((4 * (M + 2) + 8 + 4 * (M + 1)) * n_s) / t_outer / 1e9)


def vector_table_leg(torch, synth, A, ctx, layers, B, T, dev, steps):
    """Extra leg (not part of `value`): per-sample norms of the GPT-2-small blocks that are not
    linear weights -- the four linear biases of each block (their delta is the linear layer's),
    two LayerNorm gains and biases per block plus the final one, token and position embeddings.
    Returns the group's kernel time and its algorithmic HBM bytes (every delta / x element once
    per block that uses it, 2 bytes each; ids 4 bytes)."""
    d, V = 768, 50257
    blocks, nbytes = [], 0
    for l in layers:                                   # biases
        blocks.append(dict(kind="vector", x=None, delta=l["delta"],
                           grad_sum=torch.zeros(l["d_out"], device=dev)))
        nbytes += 2 * B * T * l["d_out"]
    for j in range(25):                                # LayerNorm gains and biases
        x = synth.device_normal(7000 + 2 * j, (B, T, d), 1.0, TDT, dev)
        dl = synth.device_normal(7001 + 2 * j, (B, T, d), 1e-2, TDT, dev)
        blocks.append(dict(kind="vector", x=x, delta=dl, grad_sum=torch.zeros(d, device=dev)))
        blocks.append(dict(kind="vector", x=None, delta=dl, grad_sum=torch.zeros(d, device=dev)))
        nbytes += 3 * 2 * B * T * d
    ids = torch.from_numpy(synth.token_ids(7100, B, T, V)).to(dev)
    pos = torch.arange(T, dtype=torch.int32, device=dev).repeat(B, 1).contiguous()
    de = synth.device_normal(7101, (B, T, d), 1e-2, TDT, dev)
    blocks.append(dict(kind="embed", ids=ids, vocab=V, delta=de, grad_sum=None))
    blocks.append(dict(kind="embed", ids=pos, vocab=T, delta=de, grad_sum=None))
    nbytes += 2 * (2 * B * T * d + 4 * B * T)
    descs = A.make_layer_descs(blocks, B, T, DT)
    ps = torch.zeros(B, dtype=torch.float32, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev)
    for _ in range(2):
        A.adloco_grad_stats(ctx, blocks, B, T, DT, ps, None, acc, 0, descs=descs)
    torch.cuda.synchronize()
    ctx.profile_read("vector_table")
    for _ in range(steps):
        A.adloco_grad_stats(ctx, blocks, B, T, DT, ps, None, acc, 0, descs=descs)
    torch.cuda.synchronize()
    ms, n = ctx.profile_read("vector_table")
    ms = ms / n if n else None
    # the whole parameter list of the model in one call (linear weights + these blocks): the
    # vector / table kernels run on a second stream next to the tile-statistics kernel
    both = list(layers) + blocks
    for l in layers:
        l["provided"] = False
    d_both = A.make_layer_descs(both, B, T, DT)
    combined = {}
    for overlap in (1, 0):
        ctx.set_tuning("overlap_aux", overlap)
        for _ in range(2):
            A.adloco_grad_stats(ctx, both, B, T, DT, ps, None, acc, 0, descs=d_both)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            A.adloco_grad_stats(ctx, both, B, T, DT, ps, None, acc, 0, descs=d_both)
        torch.cuda.synchronize()
        combined["overlapped" if overlap else "serial"] = (time.perf_counter() - t0) / steps * 1e3
    ctx.set_tuning("overlap_aux", 1)
    for k in ("vector_table", "tile_stats", "gram", "wgrad", "finalize", "sqnorm"):
        ctx.profile_read(k)
    return dict(bound="hbm", kernel="vector_rowsum_kernel + embed_rows_kernel (+ small reductions)",
                all_blocks_of_the_model_ms=combined,
                blocks=len(blocks), avg_kernel_ms=ms, bytes_algorithmic=nbytes,
                achieved=(nbytes / (ms * 1e-3) / 1e9) if ms else None, peak=PEAK_HBM / 1e9, unit="GB/s",
                frac=(nbytes / (ms * 1e-3) / PEAK_HBM) if ms else None, traffic=None)


def inner_products_leg(torch, A, ctx, layers, B, T, dev, steps):
    """Extra leg (not part of `value`): c_i = <g_i, G> of every sample against the gradient sums
    the timed step left in place (Section 3.3.2's tests).  Each 256 x 256 tile of each per-sample
    gradient is one T-deep bf16 contraction: 2 * d_in * d_out * T flop per (block, sample)."""
    flops = sum(2.0 * l["d_in"] * l["d_out"] * T * B for l in layers)
    descs = A.make_layer_descs(layers, B, T, DT)
    c = torch.zeros(B, dtype=torch.float32, device=dev)
    acc = torch.zeros(4, dtype=torch.float64, device=dev)
    for _ in range(2):
        A.adloco_inner_products(ctx, layers, B, T, DT, c, None, acc, 0, descs=descs)
    torch.cuda.synchronize()
    ctx.profile_read("inner_products")
    for _ in range(steps):
        A.adloco_inner_products(ctx, layers, B, T, DT, c, None, acc, 0, descs=descs)
    torch.cuda.synchronize()
    ms, n = ctx.profile_read("inner_products")
    ms = ms / n if n else None
    return dict(bound="mfma", kernel="ip_tile_kernel (+ small reductions)", blocks=len(layers),
                avg_kernel_ms=ms, flops_algorithmic=flops,
                achieved=(flops / (ms * 1e-3) / 1e12) if ms else None, peak=PEAK_BF16_MFMA / 1e12,
                unit="TFLOP/s", frac=(flops / (ms * 1e-3) / PEAK_BF16_MFMA) if ms else None, traffic=None)


def inner_step_leg(torch, synth, A, ctx, N, dev, steps):
    """Extra leg (not part of `value`): the workers' fused AdamW step on N parameters; reads
    theta, m, v, grad and writes theta, m, v: 28 bytes per parameter."""
    th = synth.device_normal(7200, (N,), 0.02, torch.float32, dev)
    m = synth.device_normal(7201, (N,), 1e-3, torch.float32, dev)
    v = synth.device_normal(7202, (N,), 1e-3, torch.float32, dev).square_()
    g = synth.device_normal(7203, (N,), 16.0, torch.float32, dev)
    for k in range(2):
        A.adloco_inner_step(ctx, th, m, v, g, step=k + 1, lr=4e-4, weight_decay=0.1, grad_scale=1.0 / 32)
    torch.cuda.synchronize()
    ctx.profile_read("inner_step")
    for k in range(steps):
        A.adloco_inner_step(ctx, th, m, v, g, step=k + 3, lr=4e-4, weight_decay=0.1, grad_scale=1.0 / 32)
    torch.cuda.synchronize()
    ms, n = ctx.profile_read("inner_step")
    ms = ms / n if n else None
    nbytes = 28 * N
    return dict(bound="hbm", kernel="inner_step_vec_kernel", N=N, avg_kernel_ms=ms,
                bytes_algorithmic=nbytes, achieved=(nbytes / (ms * 1e-3) / 1e9) if ms else None,
                peak=PEAK_HBM / 1e9, unit="GB/s", frac=(nbytes / (ms * 1e-3) / PEAK_HBM) if ms else None,
                traffic=None)


def measured_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs of this command, scaled as stated there); {} when the file is absent."""
    path = os.path.join(ROOT, "profiles", "bench_gpt2small_hbm_traffic.md")
    out = {}
    try:
        with open(path) as f:
            for ln in f:
                parts = [p.strip() for p in ln.split("|")]
                if len(parts) >= 5 and parts[1] in ("tile_stats", "gram", "wgrad", "outer_step", "merge",
                                                     "sqnorm", "vector_table", "inner_step",
                                                     "inner_products"):
                    out[parts[1]] = float(parts[2]) + float(parts[3])
    except OSError:
        pass
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures the one-GPU hot path only: --gpus must be 1 "
              "(this build has no multi-GPU path)", file=sys.stderr)
        sys.exit(2)
    import torch

    import adloco_synth as synth
    import paper_2508_18182_amd as A

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    global DT, TDT
    DT, TDT = {"bf16": (A.ADLOCO_BF16, torch.bfloat16), "f16": (A.ADLOCO_F16, torch.float16)}[args.dtype]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    ctx = A.Context(0)
    if args.gram_variant is not None:
        ctx.set_tuning("gram_variant", args.gram_variant)
    if args.wgrad_variant is not None:
        ctx.set_tuning("wgrad_variant", args.wgrad_variant)
    if args.stream_blocks_per_cu is not None:
        ctx.set_tuning("stream_blocks_per_cu", args.stream_blocks_per_cu)
    ctx.set_tuning("stats_variant", 1 if args.stats_variant == "tile" else 0)
    ctx.set_tuning("profile", 1)

    cfg = synth.CONFIGS[args.config]
    B, T, eta = cfg["B"], cfg["T"], cfg["eta"]
    shapes = synth.linear_shapes(args.config)
    linears = None
    if args.config != 2:
        per_block = len(cfg["block"])
        linears = range(per_block * (args.blocks or 2))
        shapes = shapes[:len(linears)]
        args.no_next_rows = True
        args.no_cpu_baseline = True
        if args.config == 4 and args.only == "all":
            args.only = "stats"
    ocfg = synth.CONFIGS[5 if args.config == 5 else 3]["outer"]
    N, M = ocfg["N"], ocfg["M"]
    workload = {2: "GPT-2-small-shaped grad stats (48 linears, B=32, T=512, " + args.dtype + ") + norm test + "
                   "outer step and merge (M=4 x 124M fp32)",
                4: f"Llama-1B-shaped grad stats, {len(shapes)} linears of {len(shapes) // 7} blocks "
                   f"(B=64, T=1024, bf16, q/k/v and gate/up share their input) + norm test",
                5: f"350M-round grad stats, {len(shapes)} linears of {len(shapes) // 4} blocks (B=32, "
                   f"T=1024, bf16) + norm test + outer step and merge (M=8 x 350M fp32)"}[args.config]

    # ---- inputs, resident in HBM
    layers = synth.device_grad_stats_inputs(args.config, dev, linears=linears, share=args.config == 4,
                                            dtype=args.dtype)
    for l in layers:
        l["grad_sum"] = torch.zeros(l["d_out"], l["d_in"], dtype=torch.float32, device=dev)
        l["provided"] = bool(args.grad_provided)
    descs = A.binding.make_layer_descs(layers, B, T, DT)
    per_sample = torch.zeros(B, dtype=torch.float32, device=dev)
    per_layer = torch.zeros(len(layers), B, dtype=torch.float32, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev)
    theta, insts, mom = (synth.device_outer_inputs(5 if args.config == 5 else 3, dev)
                         if args.only in ("all", "outer") else (None, None, None))
    if args.grad_provided:
        # the caller's own weight gradient: any values do; computed once, outside the timed region
        for l in layers:
            l["provided"] = False
        d2 = A.binding.make_layer_descs(layers, B, T, DT)
        A.adloco_grad_stats(ctx, layers, B, T, DT, per_sample, per_layer, acc, 0,
                            descs=d2)
        for l in layers:
            l["provided"] = True
    torch.cuda.synchronize()

    b_req = [B] * M
    last = {}

    def step():
        if args.only in ("all", "stats"):
            A.adloco_grad_stats(ctx, layers, B, T, DT, per_sample, per_layer, acc, 0,
                                descs=descs)
            res = A.adloco_norm_test(ctx, None, acc, eta, B, 32, 2, 256, descs=descs)
            last.update(res)
            b_req[0] = res["b_req"]
        if args.only in ("all", "outer"):
            A.adloco_check_merge(b_req, M)
            A.adloco_outer_step(ctx, theta, insts, mom, ocfg["lr"], ocfg["mu"], True)
            A.adloco_merge(ctx, insts, [float(b + k) for k, b in enumerate(b_req)])

    # PyTorch's plain device copy of 1 GiB, for scale (a read + write stream on this machine)
    copy_GBps = None
    if args.only in ("all", "outer") and args.config == 2:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_GBps = 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    PROF = ("tile_stats", "gram", "wgrad", "finalize", "sqnorm", "outer_step", "merge")
    for k in PROF:
        ctx.profile_read(k)                      # drop warm-up events
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    kern = {}
    for k in PROF:
        ms, n = ctx.profile_read(k)
        kern[k] = dict(avg_ms=(ms / n) if n else None, launches=n)

    # the other route to the same statistics: Gram kernel + gradient-sum GEMM (what runs when a
    # block does not qualify for the tile form, or with stats_variant = 0); timed apart, not part
    # of `value` unless --stats-variant gram made it the step's route
    alt_ms = None
    if args.only in ("all", "stats") and args.stats_variant == "tile" and not args.grad_provided:
        ctx.set_tuning("stats_variant", 0)

        def stats_gram():
            A.adloco_grad_stats(ctx, layers, B, T, DT, per_sample, per_layer, acc, 0,
                                descs=descs)
        for _ in range(2):
            stats_gram()
        torch.cuda.synchronize()
        for k in ("gram", "wgrad", "finalize", "sqnorm"):
            ctx.profile_read(k)
        t1 = time.perf_counter()
        for _ in range(args.steps):
            stats_gram()
        torch.cuda.synchronize()
        alt_ms = (time.perf_counter() - t1) / args.steps * 1e3
        for k in ("gram", "wgrad"):
            ms, n = ctx.profile_read(k)
            kern[k] = dict(avg_ms=(ms / n) if n else None, launches=n)
        for k in ("finalize", "sqnorm"):
            ctx.profile_read(k)
        ctx.set_tuning("stats_variant", 1)

    # the same statistics with the gradient sum supplied by the caller (the training framework's
    # own weight gradient): Gram kernel + reductions + norm test only
    provided_ms = None
    if args.only in ("all", "stats") and not args.grad_provided:
        for l in layers:
            l["provided"] = True
        d_prov = A.binding.make_layer_descs(layers, B, T, DT)

        def stats_provided():
            A.adloco_grad_stats(ctx, layers, B, T, DT, per_sample, per_layer, acc, 0,
                                descs=d_prov)
            A.adloco_norm_test(ctx, None, acc, eta, B, 32, 2, 256, descs=d_prov)
        for _ in range(2):
            stats_provided()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            stats_provided()
        torch.cuda.synchronize()
        provided_ms = (time.perf_counter() - t1) / args.steps * 1e3
        ms, n = ctx.profile_read("gram")
        if kern["gram"]["avg_ms"] is None and n:
            kern["gram"] = dict(avg_ms=ms / n, launches=n)
        for k in ("finalize", "sqnorm"):
            ctx.profile_read(k)

    sym, full, executed = gram_flops(shapes, B, T)
    wgrad_flops = sum(2 * B * T * di * do for _, di, do in shapes)
    outer_bytes = (4 * (M + 2) + 8) * N
    merge_bytes = 4 * (M + 1) * N
    sq_bytes = 4 * sum(di * do for _, di, do in shapes)

    # the committed counter summary belongs to the default workload and its bf16 kernels only
    traffic = measured_traffic() if (args.config == 2 and args.dtype == "bf16") else {}

    def roof(name, bound, work, ms, peak, unit, scale, **extra):
        if not ms:
            return None
        a = work / (ms * 1e-3) / scale
        return dict(bound=bound, achieved=a, peak=peak / scale, unit=unit, frac=a / (peak / scale),
                    traffic=traffic.get(name), avg_kernel_ms=ms, **extra)

    r_gram = roof("gram", "mfma", sym, kern["gram"]["avg_ms"], PEAK_BF16_MFMA, "TFLOP/s", 1e12,
                  kernel="gram_bf16_dual_kernel<false>", flops_algorithmic_symmetric=sym, flops_full=full,
                  flops_executed=executed,
                  frac_executed=(executed / (kern["gram"]["avg_ms"] * 1e-3) / PEAK_BF16_MFMA)
                  if kern["gram"]["avg_ms"] else None)
    r_wgrad = roof("wgrad", "mfma", wgrad_flops, kern["wgrad"]["avg_ms"], PEAK_BF16_MFMA, "TFLOP/s", 1e12,
                   kernel="wgrad_bf16_x_kernel<false>", flops_algorithmic=wgrad_flops)
    r_tile = roof("tile_stats", "mfma", wgrad_flops, kern["tile_stats"]["avg_ms"], PEAK_BF16_MFMA, "TFLOP/s",
                  1e12, kernel="ip_tile_kernel<1, true, false> (+ split-tile and per-sample reductions)",
                  flops_algorithmic=wgrad_flops)
    r_outer = roof("outer_step", "hbm", outer_bytes, kern["outer_step"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                   kernel="outer_step_vec_kernel", bytes_algorithmic=outer_bytes)
    r_merge = roof("merge", "hbm", merge_bytes, kern["merge"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                   kernel="merge_vec_kernel", bytes_algorithmic=merge_bytes)
    r_sq = roof("sqnorm", "hbm", sq_bytes, kern["sqnorm"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                kernel="sqnorm_partial_kernel", bytes_algorithmic=sq_bytes)
    roofs = dict(tile_stats=r_tile, gram=r_gram, wgrad=r_wgrad, outer_step=r_outer, merge=r_merge,
                 sqnorm=r_sq)
    # kernels of the timed step (the other route's kernels were timed apart)
    in_step = ("tile_stats", "finalize", "sqnorm", "outer_step", "merge") if kern["tile_stats"]["avg_ms"] \
        else ("gram", "wgrad", "finalize", "sqnorm", "outer_step", "merge")
    timed = {k: kern[k]["avg_ms"] for k in in_step if kern[k]["avg_ms"]}
    dominant = max(timed, key=timed.get) if timed else None
    stats_ms = sum(kern[k]["avg_ms"] or 0.0 for k in in_step if k not in ("outer_step", "merge"))

    out = {
        "metric": "grad-stats tokens/s (MFMA util) + outer-step GB/s (frac HBM peak), 1 GPU",
        "value": B * T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": workload,
                   "blocks_held": (len(shapes) // len(cfg["block"])), "blocks_of_model": cfg["n_blocks"],
                   "B": B, "T": T, "n_linears": len(shapes), "M": M, "N": N, "eta": eta,
                   "grad_sum": "caller-provided" if args.grad_provided else "computed by the library",
                   "stats_route": args.stats_variant,
                   "timed_part": args.only},
        "roofline": (dict(roofs[dominant], dominant_kernel=dominant)
                     if dominant in roofs and roofs[dominant] else None),
        "kernels": {"avg_ms": {k: v["avg_ms"] for k, v in kern.items()},
                    "tile_stats": r_tile, "gram": r_gram, "wgrad": r_wgrad, "outer_step": r_outer,
                    "merge": r_merge, "sqnorm": r_sq,
                    "in_timed_step": list(in_step)},
        "grad_stats_ms_gram_plus_gradient_sum_route": alt_ms,
        "grad_stats_tokens_per_s": (B * T / (stats_ms * 1e-3)) if stats_ms else None,
        "grad_stats_tokens_per_s_gradient_supplied": (B * T / (provided_ms * 1e-3)) if provided_ms else None,
        "outer_step_GBps": r_outer["achieved"] if r_outer else None,
        "merge_GBps": r_merge["achieved"] if r_merge else None,
        "norm_test": {k: last.get(k) for k in ("stat", "b_req", "test_passed", "accumulate")},
        "hbm_copy_reference": ({"GBps": copy_GBps, "how": "PyTorch device copy of 1 GiB fp32 (read + write bytes), for scale",
                              "outer_step_vs_copy": (r_outer["achieved"] / copy_GBps) if r_outer else None,
                              "merge_vs_copy": (r_merge["achieved"] / copy_GBps) if r_merge else None}
                             if copy_GBps else None),
    }
    if not args.no_next_rows:
        out["next_rows"] = {}
        if args.only in ("all", "stats"):
            out["next_rows"]["vector_table"] = vector_table_leg(torch, synth, A, ctx, layers, B, T, dev,
                                                                args.steps)
            out["next_rows"]["inner_products"] = inner_products_leg(torch, A, ctx, layers, B, T, dev,
                                                                    args.steps)
        if args.only in ("all", "outer"):
            del insts, mom
            torch.cuda.empty_cache()
            out["next_rows"]["inner_step"] = inner_step_leg(torch, synth, A, ctx, N, dev, args.steps)
        for k, v in out["next_rows"].items():
            v["traffic"] = traffic.get(k)
    if not args.no_cpu_baseline:
        from oracle import adloco_oracle as orc
        out["cpu_baseline"] = cpu_baseline(synth, orc, shapes, B, T, N, M, max(1, min(12, args.cpu_blocks)))
    else:
        out["cpu_baseline"] = None
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
