#!/usr/bin/env python3
"""Benchmark of the AdLoCo hot path on one MI355X.  Prints ONE JSON line.

Timed region (the "steps"): the full AdLoCo round of the largest single-GPU workload,
  24 blocks x {1024->3072, 1024->1024, 1024->4096, 4096->1024} (350M-parameter model), T = 1024, bf16,
  micro-batch cap b_max = 32, ceiling b_cap = 256, eta = 0.3, M = 8 instances x 350M fp32 parameters.
One step = one pass of the whole path over one (accumulated) batch; the batch schedule 32, 64, 128, 256
samples = 1, 2, 4, 8 micro-batches of 32 repeats every four steps:
  adloco_grad_stats   per micro-batch, ADLOCO_ACCUMULATE from the second on; the gradient sum is the
                      caller's (a training framework's backward pass already holds it), so the
                      per-sample norms come from the Gram contractions
  adloco_norm_test    ||sum_i g_i||^2, norm test, batch rule, SwitchMode
  adloco_check_merge  host
  adloco_outer_step   pseudo-gradient average over the 8 instances, Nesterov (lr 0.7, mu 0.9), in place
  adloco_merge        all 8 instances, weights = the requested batches the schedule produced
`value` = tokens of the timed steps / time of their statistics part (grad_stats + norm_test, HIP events
on the stream); the outer step and merge handle no tokens and are reported in GB/s.  Inputs are resident
in HBM before the timed region; every micro-batch has its own tensors, so the pointers change from call
to call as they do in training.

Further legs (each timed apart, all in the same JSON line): the same round with the gradient sum formed
by the library; the Llama-1B-shaped statistics on all 22 blocks (B = 64, T = 1024); the GPT-2-small
statistics + 124M x 4 outer step and merge, also with rotating buffer sets; the LDS-fed MFMA ceiling;
bias / gain / embedding blocks, inner products, fused AdamW step; the CPU oracle on a bounded slice.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15     # dense bf16 / fp16 MFMA flop/s, MI355X
PEAK_HBM = 8.0e12           # bytes/s
METRIC = "grad-stats tokens/s (MFMA util) + outer-step GB/s (frac HBM peak), 1 GPU"
B_SCHEDULE = (32, 64, 128, 256)        # effective batch of the four outer steps of the schedule
STAT_TARGETS = (63.5, 127.5, 255.0, 400.0)     # where the input recipe puts the norm-test statistic


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=8)
    p.add_argument("--warmup", type=int, default=4)
    p.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                   help="storage type of activations and output gradients (same kernels; the metric is "
                        "quoted on bf16)")
    p.add_argument("--blocks", type=int, default=None,
                   help="transformer blocks of the round to hold (default: all 24)")
    p.add_argument("--llama-blocks", type=int, default=None,
                   help="transformer blocks of the Llama-1B-shaped leg (default: all 22)")
    p.add_argument("--legs", default="all",
                   help="comma-separated subset of: self,llama,gpt2,probe,next,cpu (default all); "
                        "'none' runs the timed region only")
    p.add_argument("--gram-variant", type=int, default=None)
    p.add_argument("--gram-job-order", type=int, default=None)
    p.add_argument("--stream-blocks-per-cu", type=int, default=None)
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run three plain 1 GiB device copies (untimed) so that a counter profile of "
                        "this command holds a kernel of known traffic")
    return p.parse_args()


# ------------------------------------------------------------------------------------------------
# work accounting
# ------------------------------------------------------------------------------------------------

def gram_flops(shapes, B, T, shared=()):
    """(algorithmic = symmetric half, full, executed) flops of the Gram contractions of B samples, per
    linear layer as the method states them.  Executed: 128 x 128 tile pairs (p <= q), a pair on the
    diagonal computes 10 of its 16 blocks of 32 x 32; `shared` names the linears (by the last part of
    their name) that read the activation tensor of the linear before them in the block: the kernel
    forms A A^T once for such a group, so their d_in is not contracted again."""
    dsum = sum(di + do for _, di, do in shapes)
    dexec = sum((0 if nm.split(".")[-1] in shared else di) + do for nm, di, do in shapes)
    nt = -(-T // 128)
    blocks = 16 * nt * (nt - 1) / 2 + 10 * nt
    return B * T * (T + 1) * dsum, 2 * B * T * T * dsum, B * blocks * 2 * 32 * 32 * dexec


def source_hash():
    """sha256 over the kernel sources: a counter summary under profiles/ is only quoted for the build
    it was taken from."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2508_18182_amd", "csrc")
    for fn in sorted(os.listdir(d)):
        with open(os.path.join(d, fn), "rb") as f:
            h.update(fn.encode())
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(name):
    """HBM bytes per launch of kernel `name` from the rocprofv3 counter summary committed under
    profiles/ -- only if that summary carries the hash of the kernel sources of this build."""
    path = os.path.join(ROOT, "profiles", "bench_adloco350m_hbm_traffic.md")
    try:
        txt = open(path).read()
    except OSError:
        return None, "no counter summary under profiles/"
    stamp = [ln.split(":", 1)[1].strip() for ln in txt.splitlines() if ln.startswith("kernel_source_sha256:")]
    if not stamp or stamp[0] != source_hash():
        return None, "the counter summary under profiles/ belongs to other kernel sources: not quoted"
    for ln in txt.splitlines():
        parts = [p.strip() for p in ln.split("|")]
        if len(parts) >= 5 and parts[1] == name:
            return float(parts[2]) + float(parts[3]), "profiles/bench_adloco350m_hbm_traffic.md (same kernel sources)"
    return None, "kernel not in the counter summary"


def roof(bound, work, ms, peak, unit, scale, **extra):
    if not ms:
        return None
    a = work / (ms * 1e-3) / scale
    return dict(bound=bound, achieved=a, peak=peak / scale, unit=unit, frac=a / (peak / scale),
                avg_kernel_ms=ms, **extra)


class Timer:
    """HIP events on torch's current stream, which is the stream the library launches on."""
    def __init__(self, torch):
        self.torch, self.pairs = torch, []

    def span(self):
        e0 = self.torch.cuda.Event(enable_timing=True)
        e1 = self.torch.cuda.Event(enable_timing=True)
        self.pairs.append((e0, e1))
        return e0, e1

    def total_ms(self):
        self.torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in self.pairs)


def drop_profile(ctx, names):
    for k in names:
        ctx.profile_read(k)


def read_profile(ctx, names):
    out = {}
    for k in names:
        ms, n = ctx.profile_read(k)
        out[k] = dict(avg_ms=(ms / n) if n else None, launches=n)
    return out


PROF = ("tile_stats", "gram", "wgrad", "finalize", "sqnorm", "outer_step", "merge")


# ------------------------------------------------------------------------------------------------
# the round (timed region and its self-contained twin)
# ------------------------------------------------------------------------------------------------

def build_round(torch, synth, A, ctx, args, dev, DT):
    cfg = synth.CONFIGS[5]
    T, eta, b_max, b_cap = cfg["T"], cfg["eta"], cfg["b_max"], cfg["b_cap"]
    n_blocks = args.blocks or cfg["n_blocks"]
    linears = range(4 * n_blocks)
    shapes = synth.linear_shapes(5)[:4 * n_blocks]
    per_set_bytes = sum(2 * b_max * T * (di + do) for _, di, do in shapes)
    free, _ = torch.cuda.mem_get_info()
    ocfg = cfg["outer"]
    N, M = ocfg["N"], ocfg["M"]
    fixed = (M + 2) * 4 * N + 5 * 4 * sum(di * do for _, di, do in shapes) + (6 << 30)
    n_sets = 8 if free - fixed > 8 * per_set_bytes else 4
    while n_blocks > 1 and free - fixed < n_sets * per_set_bytes:
        # a card with less free memory than four sets of the whole model: hold fewer transformer blocks
        # (config.workload says how many)
        n_blocks -= 1
        linears = range(4 * n_blocks)
        shapes = synth.linear_shapes(5)[:4 * n_blocks]
        per_set_bytes = sum(2 * b_max * T * (di + do) for _, di, do in shapes)
    rhos_sched = synth.round_rho_schedule(eta, B_SCHEDULE, STAT_TARGETS)
    # which sets each outer step of the schedule accumulates, and the correlation they are drawn with:
    # step 0 -> set 0, step 1 -> sets 1, 2, step 2 -> sets 3..6, step 3 -> all eight (set 7 with its own)
    if n_sets == 8:
        plan = [[0], [1, 2], [3, 4, 5, 6], [7, 0, 1, 2, 3, 4, 5, 6]]
        rho_of_set = [rhos_sched[0], rhos_sched[1], rhos_sched[1], rhos_sched[2], rhos_sched[2],
                      rhos_sched[2], rhos_sched[2], rhos_sched[3]]
    else:   # not enough free memory for eight sets: four, each used twice in the largest batch
        plan = [[0], [1, 2], [3, 0, 1, 2], [3, 0, 1, 2, 3, 0, 1, 2]]
        rho_of_set = [rhos_sched[0], rhos_sched[1], rhos_sched[1], rhos_sched[2]]
    sets = synth.device_round_micro_batches(5, dev, rho_of_set, linears=linears, dtype=args.dtype)
    # one set of gradient-sum buffers per outer step of the schedule (the "caller's" weight gradients)
    grads = [[torch.zeros(do, di, dtype=torch.float32, device=dev) for _, di, do in shapes] for _ in plan]
    theta, insts, mom = synth.device_outer_inputs(5, dev)
    st = dict(cfg=cfg, T=T, eta=eta, b_max=b_max, b_cap=b_cap, shapes=shapes, n_blocks=n_blocks, plan=plan,
              sets=sets, grads=grads, theta=theta, insts=insts, mom=mom, N=N, M=M, ocfg=ocfg, n_sets=n_sets,
              rho_of_set=rho_of_set, per_set_bytes=per_set_bytes,
              per_sample=torch.zeros(b_max, dtype=torch.float32, device=dev),
              acc=torch.zeros(2, dtype=torch.float64, device=dev))

    def descs(provided):
        out = {}
        for r, ids in enumerate(plan):
            for s in set(ids):
                layers = [dict(a=l["a"], delta=l["delta"], grad_sum=g, provided=provided)
                          for l, g in zip(sets[s], grads[r])]
                out[(r, s)] = A.make_layer_descs(layers, b_max, T, DT)
        return out
    st["descs_provided"], st["descs_own"] = descs(True), descs(False)
    return st


def round_stats(A, ctx, st, r, DT, provided):
    """The statistics of outer step r of the schedule: its micro-batches, then the norm test."""
    d = st["descs_provided"] if provided else st["descs_own"]
    for j, s in enumerate(st["plan"][r]):
        A.adloco_grad_stats(ctx, None, st["b_max"], st["T"], DT, st["per_sample"], None, st["acc"],
                            A.ADLOCO_ACCUMULATE if j else 0, descs=d[(r, s)])
    b = st["b_max"] * len(st["plan"][r])
    return A.adloco_norm_test(ctx, None, st["acc"], st["eta"], b, st["b_max"], 2, st["b_cap"],
                              descs=d[(r, st["plan"][r][0])])


# ------------------------------------------------------------------------------------------------
# legs
# ------------------------------------------------------------------------------------------------

def llama_leg(torch, synth, A, ctx, args, dev, DT):
    """Llama-1B-shaped statistics, all blocks resident: 7 linears per block, q / k / v and gate / up read
    one activation tensor each, B = 64, T = 1024."""
    cfg = synth.CONFIGS[4]
    B, T, eta = cfg["B"], cfg["T"], cfg["eta"]
    n_blocks = args.llama_blocks or cfg["n_blocks"]
    linears = range(7 * n_blocks)
    shapes = synth.linear_shapes(4)[:7 * n_blocks]
    layers = synth.device_grad_stats_inputs(4, dev, linears=linears, share=True, dtype=args.dtype)
    for l in layers:
        l["grad_sum"] = torch.zeros(l["d_out"], l["d_in"], dtype=torch.float32, device=dev)
    ps = torch.zeros(B, dtype=torch.float32, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev)
    own = A.make_layer_descs([dict(l, provided=False) for l in layers], B, T, DT)
    prov = A.make_layer_descs([dict(l, provided=True) for l in layers], B, T, DT)
    out = {}
    for name, d, reps in (("self_contained", own, 3), ("gradient_supplied", prov, 5)):
        def run():
            A.adloco_grad_stats(ctx, None, B, T, DT, ps, None, acc, 0, descs=d)
            return A.adloco_norm_test(ctx, None, acc, eta, B, 32, 2, 0, descs=d)
        run()
        torch.cuda.synchronize()
        drop_profile(ctx, PROF)
        t0 = time.perf_counter()
        for _ in range(reps):
            res = run()
        torch.cuda.synchronize()
        out[name] = dict(ms=(time.perf_counter() - t0) / reps * 1e3, kernels=read_profile(ctx, PROF),
                         norm_test={k: res[k] for k in ("stat", "b_req", "test_passed", "accumulate")})
    # k, v read q's activation tensor, up reads gate's: A A^T is formed once per group (T % 128 = 0)
    sym, full, executed = gram_flops(shapes, B, T, shared=("k", "v", "up"))
    wflops = sum(2.0 * B * T * di * do for _, di, do in shapes)
    g_ms = out["gradient_supplied"]["kernels"]["gram"]["avg_ms"]
    t_ms = out["self_contained"]["kernels"]["tile_stats"]["avg_ms"]
    return dict(workload=f"Llama-1B-shaped grad stats, all {n_blocks} blocks = {len(shapes)} linears "
                         f"(q/k/v and gate/up share their input), B={B}, T={T}, {args.dtype}",
                tokens=B * T,
                gradient_supplied=dict(ms=out["gradient_supplied"]["ms"], tokens_per_s=B * T / (out["gradient_supplied"]["ms"] * 1e-3),
                                       norm_test=out["gradient_supplied"]["norm_test"]),
                self_contained=dict(ms=out["self_contained"]["ms"], tokens_per_s=B * T / (out["self_contained"]["ms"] * 1e-3),
                                    norm_test=out["self_contained"]["norm_test"]),
                gram=roof("mfma", sym, g_ms, PEAK_BF16_MFMA, "TFLOP/s", 1e12, kernel="gram_bf16_dual_kernel",
                          flops_algorithmic_symmetric=sym, flops_full=full, flops_executed=executed,
                          frac_executed=(executed / (g_ms * 1e-3) / PEAK_BF16_MFMA) if g_ms else None,
                          note="`frac` counts the symmetric-half flops of every linear; the kernel forms A A^T once "
                               "for q/k/v and once for gate/up, so it executes fewer: `frac_executed` is the MFMA "
                               "utilisation"),
                tile_stats=roof("mfma", wflops, t_ms, PEAK_BF16_MFMA, "TFLOP/s", 1e12,
                                kernel="ip_tile_kernel<1, true> (norms and gradient sum in one pass)",
                                flops_algorithmic=wflops))


def gpt2_leg(torch, synth, A, ctx, args, dev, DT, TDT):
    """GPT-2-small statistics (48 linears, B = 32, T = 512) + 124M x 4 outer step and merge.  The
    statistics are timed with one fixed set of buffers and with three sets taken in turn."""
    cfg = synth.CONFIGS[2]
    B, T, eta = cfg["B"], cfg["T"], cfg["eta"]
    shapes = synth.linear_shapes(2)
    base = synth.device_grad_stats_inputs(2, dev, dtype=args.dtype)
    sets = [base]
    for k in (1, 2):     # two more sets of the same shapes (other values, other addresses)
        sets.append([dict(l, a=torch.roll(l["a"], k, 0).contiguous(), delta=torch.roll(l["delta"], k, 0).contiguous())
                     for l in base])
    for s in sets:
        for l in s:
            l["grad_sum"] = torch.zeros(l["d_out"], l["d_in"], dtype=torch.float32, device=dev)
    ps = torch.zeros(B, dtype=torch.float32, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev)
    d_own = [A.make_layer_descs([dict(l, provided=False) for l in s], B, T, DT) for s in sets]
    d_prov = [A.make_layer_descs([dict(l, provided=True) for l in s], B, T, DT) for s in sets]
    reps = 12

    def timed(dl):
        def run(i):
            d = dl[i % len(dl)]
            A.adloco_grad_stats(ctx, None, B, T, DT, ps, None, acc, 0, descs=d)
            return A.adloco_norm_test(ctx, None, acc, eta, B, 32, 2, 256, descs=d)
        for i in range(3):
            run(i)
        torch.cuda.synchronize()
        drop_profile(ctx, PROF)
        b0 = ctx.table_builds()
        t0 = time.perf_counter()
        for i in range(reps):
            run(i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        rebuilt[0] += ctx.table_builds() - b0
        return ms, read_profile(ctx, PROF)

    rebuilt = [0]
    own_fixed_ms, own_k = timed(d_own[:1])
    own_rot_ms, _ = timed(d_own)
    prov_fixed_ms, prov_k = timed(d_prov[:1])
    prov_rot_ms, _ = timed(d_prov)
    sym, full, executed = gram_flops(shapes, B, T)
    wflops = sum(2.0 * B * T * di * do for _, di, do in shapes)
    # outer step + merge, M = 4 x 124M
    ocfg = synth.CONFIGS[3]["outer"]
    N, M = ocfg["N"], ocfg["M"]
    theta, insts, mom = synth.device_outer_inputs(3, dev)
    for _ in range(3):
        A.adloco_outer_step(ctx, theta, insts, mom, ocfg["lr"], ocfg["mu"], True)
        A.adloco_merge(ctx, insts, [32.0 + k for k in range(M)])
    torch.cuda.synchronize()
    drop_profile(ctx, PROF)
    for _ in range(20):
        A.adloco_outer_step(ctx, theta, insts, mom, ocfg["lr"], ocfg["mu"], True)
        A.adloco_merge(ctx, insts, [32.0 + k for k in range(M)])
    torch.cuda.synchronize()
    k = read_profile(ctx, PROF)
    g_ms, t_ms = prov_k["gram"]["avg_ms"], own_k["tile_stats"]["avg_ms"]
    out = dict(workload=f"GPT-2-small-shaped grad stats (48 linears, B={B}, T={T}, {args.dtype}) + outer step "
                        f"and merge (M={M} x {N // 10**6}M fp32)",
               tokens=B * T,
               gradient_supplied=dict(ms=prov_fixed_ms, tokens_per_s=B * T / (prov_fixed_ms * 1e-3),
                                      ms_three_buffer_sets_in_turn=prov_rot_ms),
               self_contained=dict(ms=own_fixed_ms, tokens_per_s=B * T / (own_fixed_ms * 1e-3),
                                   ms_three_buffer_sets_in_turn=own_rot_ms),
               rotation_overhead=dict(self_contained=own_rot_ms / own_fixed_ms - 1.0,
                                      gradient_supplied=prov_rot_ms / prov_fixed_ms - 1.0,
                                      tables_rebuilt_while_timing=rebuilt[0]),
               gram=roof("mfma", sym, g_ms, PEAK_BF16_MFMA, "TFLOP/s", 1e12, kernel="gram_bf16_dual_kernel",
                         flops_algorithmic_symmetric=sym, flops_full=full, flops_executed=executed,
                         frac_executed=(executed / (g_ms * 1e-3) / PEAK_BF16_MFMA) if g_ms else None),
               tile_stats=roof("mfma", wflops, t_ms, PEAK_BF16_MFMA, "TFLOP/s", 1e12,
                               kernel="ip_tile_kernel<1, true>", flops_algorithmic=wflops),
               outer_step=roof("hbm", (4 * (M + 2) + 8) * N, k["outer_step"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                               kernel="outer_step_vec_kernel", bytes_algorithmic=(4 * (M + 2) + 8) * N),
               merge=roof("hbm", 4 * (M + 1) * N, k["merge"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                          kernel="merge_vec_kernel", bytes_algorithmic=4 * (M + 1) * N))
    del theta, insts, mom
    return out, sets[0], (B, T)


def vector_table_leg(torch, synth, A, ctx, layers, B, T, dev, DT, TDT, steps):
    """Per-sample norms of the GPT-2-small blocks that are not linear weights: four linear biases per
    block (their delta is the linear layer's), two LayerNorm gains and biases per block plus the final
    one, token and position embeddings.  Algorithmic HBM bytes: every distinct delta / x tensor once,
    2 bytes per element; ids 4 bytes."""
    d, V = 768, 50257
    blocks, nbytes = [], 0
    for l in layers:                                   # biases
        blocks.append(dict(kind="vector", x=None, delta=l["delta"], grad_sum=torch.zeros(l["d_out"], device=dev)))
        nbytes += 2 * B * T * l["d_out"]
    for j in range(25):                                # LayerNorm gains and biases: x and delta once each
        x = synth.device_normal(7000 + 2 * j, (B, T, d), 1.0, TDT, dev)
        dl = synth.device_normal(7001 + 2 * j, (B, T, d), 1e-2, TDT, dev)
        blocks.append(dict(kind="vector", x=x, delta=dl, grad_sum=torch.zeros(d, device=dev)))
        blocks.append(dict(kind="vector", x=None, delta=dl, grad_sum=torch.zeros(d, device=dev)))
        nbytes += 2 * 2 * B * T * d
    ids = torch.from_numpy(synth.token_ids(7100, B, T, V)).to(dev)
    pos = torch.arange(T, dtype=torch.int32, device=dev).repeat(B, 1).contiguous()
    de = synth.device_normal(7101, (B, T, d), 1e-2, TDT, dev)
    blocks.append(dict(kind="embed", ids=ids, vocab=V, delta=de, grad_sum=None))
    blocks.append(dict(kind="embed", ids=pos, vocab=T, delta=de, grad_sum=None))
    nbytes += 2 * B * T * d + 2 * 4 * B * T
    descs = A.make_layer_descs(blocks, B, T, DT)
    ps = torch.zeros(B, dtype=torch.float32, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev)
    for _ in range(2):
        A.adloco_grad_stats(ctx, None, B, T, DT, ps, None, acc, 0, descs=descs)
    torch.cuda.synchronize()
    ctx.profile_read("vector_table")
    for _ in range(steps):
        A.adloco_grad_stats(ctx, None, B, T, DT, ps, None, acc, 0, descs=descs)
    torch.cuda.synchronize()
    ms, n = ctx.profile_read("vector_table")
    ms = ms / n if n else None
    drop_profile(ctx, PROF)
    return dict(bound="hbm", kernel="vector_rowsum_kernel + embed_rows_kernel (+ small reductions)",
                blocks=len(blocks), avg_kernel_ms=ms, bytes_algorithmic=nbytes,
                achieved=(nbytes / (ms * 1e-3) / 1e9) if ms else None, peak=PEAK_HBM / 1e9, unit="GB/s",
                frac=(nbytes / (ms * 1e-3) / PEAK_HBM) if ms else None)


def inner_products_leg(torch, A, ctx, layers, B, T, dev, DT, steps):
    """c_i = <g_i, G> of every sample against the gradient sums in place (Section 3.3.2's tests): per
    (block, sample) one T-deep bf16 contraction of 2 d_in d_out T flop."""
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
                unit="TFLOP/s", frac=(flops / (ms * 1e-3) / PEAK_BF16_MFMA) if ms else None)


def inner_step_leg(torch, synth, A, ctx, N, dev, steps):
    """The workers' fused AdamW step on N parameters: reads theta, m, v, grad and writes theta, m, v,
    28 bytes per parameter."""
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
    return roof("hbm", 28 * N, ms, PEAK_HBM, "GB/s", 1e9, kernel="inner_step_vec_kernel", N=N,
                bytes_algorithmic=28 * N)


def drift_leg(torch, synth, A, ctx, dev, steps):
    """The outer step and merge of the round (M = 8 x 350M) on instance drifts stored in bf16: the
    outer step reads 8 + 2 M and writes 8 bytes per parameter, the merge reads 4 + 2 (S - 1) and writes
    4, packing one instance reads 8 and writes 2."""
    o = synth.CONFIGS[5]["outer"]
    N, M = o["N"], o["M"]
    theta = synth.device_normal(9305, (N,), o["std_theta"], torch.float32, dev)
    mom = synth.device_normal(9355, (N,), o["std_mom"], torch.float32, dev)
    inst = theta - synth.device_normal(9405, (N,), o["std_delta"], torch.float32, dev)
    drifts = [torch.empty(N, dtype=torch.bfloat16, device=dev) for _ in range(M)]
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}

    def timed(fn, nbytes, kernel):
        for _ in range(2):
            fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return roof("hbm", nbytes, e0.elapsed_time(e1) / steps, PEAK_HBM, "GB/s", 1e9, kernel=kernel,
                    bytes_algorithmic=nbytes)
    out["pack_drift"] = timed(lambda: A.adloco_pack_drift(ctx, theta, inst, drifts[0]), 10 * N,
                              "pack_drift_vec_kernel")
    for d in drifts[1:]:
        d.copy_(drifts[0])
    out["outer_step_drift"] = timed(lambda: A.adloco_outer_step_drift(ctx, theta, drifts, mom, o["lr"], o["mu"], True),
                                    (16 + 2 * M) * N, "outer_step_drift_vec_kernel")
    out["merge_drift"] = timed(lambda: A.adloco_merge_drift(ctx, theta, drifts[1:], 64.0, [32.0 + k for k in range(M - 1)]),
                               (8 + 2 * (M - 1)) * N, "merge_drift_vec_kernel")
    out["bytes_vs_fp32_instances"] = dict(outer_step=(16 + 2 * M) / (16 + 4 * M), merge=(8 + 2 * (M - 1)) / (4 * (M + 1)))
    return out


def cpu_baseline(synth, orc, cfg, n_blocks, N, M):
    """The oracle as it stands on a bounded slice of the timed workload: the four linears of 4 of the
    24 transformer blocks on one whole micro-batch of 32 samples (per-sample norms, gradient sum, norm
    test), and the outer step + merge on N / 8 parameters."""
    import numpy as np
    cores = len(os.sched_getaffinity(0))
    T, B, ns, nb = cfg["T"], cfg["b_max"], cfg["b_max"], 4
    t_stats = 0.0
    for b in range(nb):
        layers = synth.grad_stats_inputs(5, linears=range(4 * b, 4 * b + 4), B=ns, T=T)
        t0 = time.perf_counter()
        st = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=False)
        orc.norm_test(st["S1"], st["S2"], ns, cfg["eta"], ns, B)
        t_stats += time.perf_counter() - t0
        del layers, st
    t_stats /= nb
    n_s = N // 8
    theta, insts, mom = synth.outer_inputs(5, N=n_s, M=M)
    t0 = time.perf_counter()
    orc.outer_step(theta, insts, mom, 0.7, 0.9, True)
    orc.merge(insts, [32.0 + k for k in range(M)])
    t_outer = time.perf_counter() - t0
    tok_s = ns * T / (t_stats * n_blocks)
    nbytes = ((4 * (M + 2) + 8) + 4 * (M + 1)) * n_s
    return dict(value=tok_s, unit="tokens/s", cores=cores, kind="oracle",
                sample=(f"statistics: the 4 linears of each of {nb} of {n_blocks} blocks on {ns} samples x {T} tokens took "
                        f"{t_stats:.2f} s per block (explicit per-sample gradients, numpy fp64: the matrix products run on "
                        f"the BLAS thread pool of up to {cores} cores, squares and sums on one); tokens/s = "
                        f"{ns * T} tokens / ({t_stats:.2f} s x {n_blocks} blocks), a linear extrapolation to the "
                        f"whole model; outer step + merge on N/8 = {n_s} parameters, M = {M}: {t_outer:.2f} s, "
                        f"single-threaded numpy"),
                outer_merge_GBps=nbytes / t_outer / 1e9)


# ------------------------------------------------------------------------------------------------

def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures the one-GPU hot path only: --gpus must be 1 (this build has no multi-GPU "
              "path)", file=sys.stderr)
        sys.exit(2)
    import torch

    import adloco_synth as synth
    import paper_2508_18182_amd as A

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    DT, TDT = {"bf16": (A.ADLOCO_BF16, torch.bfloat16), "f16": (A.ADLOCO_F16, torch.float16)}[args.dtype]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    legs = set("self,llama,gpt2,probe,next,cpu".split(",")) if args.legs == "all" else \
        (set() if args.legs == "none" else set(args.legs.split(",")))
    ctx = A.Context(0)
    if args.gram_variant is not None:
        ctx.set_tuning("gram_variant", args.gram_variant)
    if args.gram_job_order is not None:
        ctx.set_tuning("gram_job_order", args.gram_job_order)
    if args.stream_blocks_per_cu is not None:
        ctx.set_tuning("stream_blocks_per_cu", args.stream_blocks_per_cu)
    ctx.set_tuning("profile", 1)

    st = build_round(torch, synth, A, ctx, args, dev, DT)
    T, M, N, ocfg, plan = st["T"], st["M"], st["N"], st["ocfg"], st["plan"]
    # the caller's gradient sums, formed once outside the timed region (by the library itself)
    reqs = []
    for r in range(len(plan)):
        res = round_stats(A, ctx, st, r, DT, provided=False)
        reqs.append(int(res["b_req"]))
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    b_req = [reqs[k % len(reqs)] + k // len(reqs) for k in range(M)]   # the M instances' requests
    tm_stats, tm_outer = Timer(torch), Timer(torch)
    last = {}

    def step(i, timed):
        r = i % len(plan)
        if timed:
            e0, e1 = tm_stats.span()
            e0.record()
        res = round_stats(A, ctx, st, r, DT, provided=True)
        if timed:
            e1.record()
        b_req[r] = int(res["b_req"])
        last[r] = {k: res[k] for k in ("stat", "b_req", "test_passed", "accumulate", "accum_steps")}
        A.adloco_check_merge(b_req, M)
        if timed:
            e0, e1 = tm_outer.span()
            e0.record()
        A.adloco_outer_step(ctx, st["theta"], st["insts"], st["mom"], ocfg["lr"], ocfg["mu"], True)
        A.adloco_merge(ctx, st["insts"], [float(b) for b in b_req])
        if timed:
            e1.record()

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    drop_profile(ctx, PROF)
    builds0 = ctx.table_builds()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    kern = read_profile(ctx, PROF)
    stats_ms, outer_ms = tm_stats.total_ms(), tm_outer.total_ms()
    tokens = sum(st["b_max"] * len(plan[i % len(plan)]) * T for i in range(args.steps))
    rebuilt = ctx.table_builds() - builds0

    shapes = st["shapes"]
    sym, full, executed = gram_flops(shapes, st["b_max"], T)       # per launch = per micro-batch
    g_ms = kern["gram"]["avg_ms"]
    traffic, traffic_note = measured_traffic("gram")
    r_gram = roof("mfma", sym, g_ms, PEAK_BF16_MFMA, "TFLOP/s", 1e12, kernel="gram_bf16_dual_kernel",
                  launches=kern["gram"]["launches"], units_per_launch=f"{st['b_max']} samples x {T} tokens x {len(shapes)} linears",
                  flops_algorithmic_symmetric=sym, flops_full=full, flops_executed=executed,
                  frac_executed=(executed / (g_ms * 1e-3) / PEAK_BF16_MFMA) if g_ms else None,
                  traffic=traffic, traffic_source=traffic_note)
    outer_bytes, merge_bytes = (4 * (M + 2) + 8) * N, 4 * (M + 1) * N
    sq_bytes = 4 * sum(di * do for _, di, do in shapes)
    r_outer = roof("hbm", outer_bytes, kern["outer_step"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                   kernel="outer_step_vec_kernel", bytes_algorithmic=outer_bytes)
    r_merge = roof("hbm", merge_bytes, kern["merge"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                   kernel="merge_vec_kernel", bytes_algorithmic=merge_bytes)
    r_sq = roof("hbm", sq_bytes, kern["sqnorm"]["avg_ms"], PEAK_HBM, "GB/s", 1e9,
                kernel="sqnorm_partial_kernel", bytes_algorithmic=sq_bytes)

    out = {
        "metric": METRIC,
        "value": tokens / (stats_ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "value_is": ("grad-stats tokens/s with the gradient sum supplied by the caller: tokens of the timed "
                     "steps / HIP-event time of their adloco_grad_stats + adloco_norm_test calls; the outer "
                     "step and merge of the same steps handle no tokens and are given in GB/s"),
        "config": {"workload": (f"full AdLoCo round on one GPU: M={M} instances of a 350M-parameter model "
                                f"({st['n_blocks']} of 24 blocks resident = {len(shapes)} linears, d=1024, MLP 4096, "
                                f"T={T}, {args.dtype}), batch schedule {list(B_SCHEDULE)} samples = 1, 2, 4, 8 "
                                f"accumulated micro-batches of {st['b_max']}, norm test eta={st['eta']}, b_cap "
                                f"{st['b_cap']}, then outer step (Nesterov, lr 0.7, mu 0.9) and merge of all {M}"),
                   "micro_batch_sets_resident": st["n_sets"], "bytes_per_micro_batch": st["per_set_bytes"],
                   "rho_of_set": st["rho_of_set"], "M": M, "N": N,
                   "grad_sum": "caller-supplied in the timed region (formed once by the library beforehand)",
                   "tokens_in_timed_steps": tokens},
        "stats_ms_in_timed_steps": stats_ms, "outer_merge_ms_in_timed_steps": outer_ms,
        "tables_rebuilt_in_timed_steps": rebuilt,
        "outer_step_GBps": r_outer["achieved"] if r_outer else None,
        "merge_GBps": r_merge["achieved"] if r_merge else None,
        "roofline": dict(r_gram, dominant_kernel="gram") if r_gram else None,
        "kernels": {"avg_ms": {k: v["avg_ms"] for k, v in kern.items()},
                    "launches": {k: v["launches"] for k, v in kern.items()},
                    "gram": r_gram, "outer_step": r_outer, "merge": r_merge, "sqnorm": r_sq},
        "norm_test_by_schedule_step": [last.get(r) for r in range(len(plan))],
        "requested_batches_from_the_setup_pass": reqs,
    }

    # ---- the same round with the gradient sum formed by the library (per-sample gradient tiles)
    if "self" in legs:
        for r in range(len(plan)):
            round_stats(A, ctx, st, r, DT, provided=False)
        torch.cuda.synchronize()
        drop_profile(ctx, PROF)
        tm = Timer(torch)
        n_pass = 2
        for _ in range(n_pass):
            for r in range(len(plan)):
                e0, e1 = tm.span()
                e0.record()
                round_stats(A, ctx, st, r, DT, provided=False)
                e1.record()
        ms = tm.total_ms()
        k = read_profile(ctx, PROF)
        wflops = sum(2.0 * st["b_max"] * T * di * do for _, di, do in shapes)
        out["self_contained"] = dict(
            what="the same batch schedule with grad_sum formed by the library: norms and gradient sum from "
                 "one pass over per-sample gradient tiles",
            tokens_per_s=n_pass * sum(st["b_max"] * len(p) * T for p in plan) / (ms * 1e-3),
            tile_stats=roof("mfma", wflops, k["tile_stats"]["avg_ms"], PEAK_BF16_MFMA, "TFLOP/s", 1e12,
                            kernel="ip_tile_kernel<1, true>", flops_algorithmic=wflops,
                            launches=k["tile_stats"]["launches"]))
    # free the round before the other legs
    for key in ("sets", "grads", "theta", "insts", "mom", "descs_provided", "descs_own"):
        st[key] = None
    torch.cuda.empty_cache()

    if "llama" in legs:
        out["llama_1b"] = llama_leg(torch, synth, A, ctx, args, dev, DT)
        torch.cuda.empty_cache()
    gpt2_layers = None
    if "gpt2" in legs or "next" in legs:
        out["gpt2_small_plus_outer_124m"], gpt2_layers, (B2, T2) = gpt2_leg(torch, synth, A, ctx, args, dev, DT, TDT)
    if "probe" in legs:
        probes = {}
        for v, name in ((0, "wave_tile_64x64"), (1, "wave_tile_128x64")):
            ms, fl = ctx.probe_mfma_lds(v, 8192)
            probes[name] = dict(ms=ms, TFLOPs=fl / (ms * 1e-3) / 1e12, frac_of_peak=fl / (ms * 1e-3) / PEAK_BF16_MFMA)
        out["lds_fed_mfma_ceiling"] = dict(
            what="32x32x16 bf16 MFMAs on fragments read from LDS, nothing else running (no global loads, no "
                 "barriers): what the chip sustains at the clock it holds under that load",
            **probes)
        if r_gram:
            best = max(p["frac_of_peak"] for p in probes.values())
            out["roofline"]["frac_executed_of_lds_fed_ceiling"] = r_gram["frac_executed"] / best
    if "next" in legs and gpt2_layers is not None:
        nr = {}
        nr["vector_table"] = vector_table_leg(torch, synth, A, ctx, gpt2_layers, B2, T2, dev, DT, TDT, 10)
        nr["inner_products"] = inner_products_leg(torch, A, ctx, gpt2_layers, B2, T2, dev, DT, 10)
        gpt2_layers = None
        torch.cuda.empty_cache()
        nr["inner_step"] = inner_step_leg(torch, synth, A, ctx, 124_000_000, dev, 10)
        torch.cuda.empty_cache()
        nr["bf16_drift_M8_350M"] = drift_leg(torch, synth, A, ctx, dev, 10)
        out["next_rows"] = nr
    if "cpu" in legs:
        from oracle import adloco_oracle as orc
        out["cpu_baseline"] = cpu_baseline(synth, orc, st["cfg"], 24, N, M)
    else:
        out["cpu_baseline"] = None
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
