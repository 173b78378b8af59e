"""Seeded synthetic inputs for the AdLoCo hot path (shapes only; no method arithmetic).

This module is the one piece shared by the CPU oracle's tests and the HIP path's tests
and benchmark.  It draws Gaussian activations `a`, output-gradients `delta` and flat
parameter vectors with the shapes of the five workloads, and converts fp32 values to
bf16 bit patterns.  Nothing here computes a gradient, a norm, a statistic or an update.

The paper trains MicroLlama on C4 (Section 6.1); neither is available, so seeded
Gaussian tensors with transformer-shaped linear layers stand in for the activations
and output gradients of a real backward pass.

Seeds: grad-stats tensors use  1000*config + 10*linear_index + {0: a, 1: delta};
outer-step tensors use 9000 + config (+ instance index offsets documented below).
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------------------
# Workload shapes
# --------------------------------------------------------------------------------------

def _gpt2_small_layer():
    return [("attn.qkv", 768, 2304), ("attn.proj", 768, 768),
            ("mlp.fc", 768, 3072), ("mlp.proj", 3072, 768)]


def _llama_1b_layer():
    return [("q", 2048, 2048), ("k", 2048, 2048), ("v", 2048, 2048), ("o", 2048, 2048),
            ("gate", 2048, 5632), ("up", 2048, 5632), ("down", 5632, 2048)]


def _m350_layer():
    return [("attn.qkv", 1024, 3072), ("attn.proj", 1024, 1024),
            ("mlp.fc", 1024, 4096), ("mlp.proj", 4096, 1024)]


CONFIGS = {
    # config id -> description of the workload
    1: dict(name="tiny", n_blocks=1, block=[("lin", 64, 32)], B=8, T=16, dtype="f32",
            std_a=1.0, std_delta=1.0, eta=0.5,
            outer=dict(M=2, N=10_000, std_theta=0.02, std_delta=1e-3, std_mom=0.0,
                       lr=0.7, mu=0.9)),
    2: dict(name="gpt2-small", n_blocks=12, block=_gpt2_small_layer(), B=32, T=512,
            dtype="bf16", std_a=1.0, std_delta=1e-2, eta=0.3),
    3: dict(name="outer-124M", outer=dict(M=4, N=124_000_000, std_theta=0.02,
                                          std_delta=1e-3, std_mom=1e-4, lr=0.7, mu=0.9)),
    4: dict(name="llama-1b", n_blocks=22, block=_llama_1b_layer(), B=64, T=1024,
            dtype="bf16", std_a=1.0, std_delta=1e-2, eta=0.3),
    5: dict(name="round-350M", n_blocks=24, block=_m350_layer(), B=32, T=1024,
            dtype="bf16", std_a=1.0, std_delta=1e-2, eta=0.3, b_max=32, b_cap=256,
            n_switch=2,
            outer=dict(M=8, N=350_000_000, std_theta=0.02, std_delta=1e-3, std_mom=1e-4,
                       lr=0.7, mu=0.9)),
}


def linear_shapes(config: int):
    """[(name, d_in, d_out)] for every linear of the workload, block by block."""
    c = CONFIGS[config]
    out = []
    for b in range(c["n_blocks"]):
        for (nm, di, do) in c["block"]:
            out.append((f"h{b}.{nm}", di, do))
    return out


def tensor_seed(config: int, linear_index: int, which: int) -> int:
    """which: 0 = activations a, 1 = output gradients delta."""
    return 1000 * config + 10 * linear_index + which


# --------------------------------------------------------------------------------------
# Host (numpy) generators
# --------------------------------------------------------------------------------------

def normal_f32(seed: int, shape, std: float = 1.0) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 draws in the storage type of a workload: "f32" as is, "bf16" as uint16 bit patterns
    (round to nearest even), "f16" as numpy float16."""
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    return f32_to_bf16_bits(x)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32 (a format conversion)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def grad_stats_inputs(config: int, linears=None, B=None, T=None, dtype=None, rho=0.0,
                      seed_offset=0):
    """Host tensors for the grad-stats half.

    Returns a list of dicts {name, d_in, d_out, a, delta}; a is [B,T,d_in], delta is
    [B,T,d_out]; fp32 arrays for dtype 'f32', uint16 bf16 bit patterns for 'bf16'.
    `linears` selects linear indices (default all).  `rho` in [0,1) mixes a component
    shared by all samples into every sample (x_i = rho*x0 + sqrt(1-rho^2)*eps_i) so that the
    batch gradient does not vanish against the noise; rho = 0 is the pure-noise case.
    """
    c = CONFIGS[config]
    B = c["B"] if B is None else B
    T = c["T"] if T is None else T
    dtype = c["dtype"] if dtype is None else dtype
    shapes = linear_shapes(config)
    idx = range(len(shapes)) if linears is None else linears
    out = []
    for li in idx:
        nm, di, do = shapes[li]
        tensors = {}
        for which, (key, d, std) in enumerate((("a", di, c["std_a"]),
                                               ("delta", do, c["std_delta"]))):
            seed = tensor_seed(config, li, which) + seed_offset
            if rho == 0.0:
                x = normal_f32(seed, (B, T, d), std)
            else:
                eps = normal_f32(seed, (B + 1, T, d), std)
                x = (np.float32(rho) * eps[:1]
                     + np.float32(np.sqrt(1.0 - rho * rho)) * eps[1:])
            tensors[key] = to_dtype(x, dtype)
        out.append(dict(name=nm, d_in=di, d_out=do, a=tensors["a"], delta=tensors["delta"]))
    return out


def custom_grad_stats_inputs(seed: int, shapes, B: int, T: int, dtype: str,
                             std_a=1.0, std_delta=1e-2, rho=0.0):
    """Same recipe for an arbitrary list of (d_in, d_out) (edge-case and ragged shapes)."""
    out = []
    for li, (di, do) in enumerate(shapes):
        tensors = {}
        for which, (key, d, std) in enumerate((("a", di, std_a), ("delta", do, std_delta))):
            s = seed + 10 * li + which
            if rho == 0.0:
                x = normal_f32(s, (B, T, d), std)
            else:
                eps = normal_f32(s, (B + 1, T, d), std)
                x = (np.float32(rho) * eps[:1]
                     + np.float32(np.sqrt(1.0 - rho * rho)) * eps[1:])
            tensors[key] = to_dtype(x, dtype)
        out.append(dict(name=f"lin{li}", d_in=di, d_out=do, a=tensors["a"],
                        delta=tensors["delta"]))
    return out


def token_ids(seed: int, B: int, T: int, vocab: int, zipf: float = 1.1) -> np.ndarray:
    """int32 [B, T] token ids with a Zipf-like frequency profile (rank r drawn with weight
    1 / r^zipf, then mapped through a fixed permutation of the vocabulary), the repeat
    structure of natural-language token streams: a few ids occur many times per sample, most
    at most once.  zipf = 0 is uniform."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = 1.0 / np.arange(1, vocab + 1, dtype=np.float64) ** zipf
    w /= w.sum()
    ranks = rng.choice(vocab, size=(B, T), p=w)
    return rng.permutation(vocab)[ranks].astype(np.int32)


def vector_table_inputs(seed: int, B: int, T: int, dtype: str, vectors=(), tables=(),
                        std_delta: float = 1e-2, rho: float = 0.0):
    """Host tensors for blocks that are not linear weights.
    vectors: list of (d, has_x): a gain (has_x: x ~ N(0,1), the normalised input) or a bias.
    tables: list of (vocab, d): token ids (Zipf-like) and delta.
    Returns dicts {kind, d, delta, x | ids, vocab}; fp32 arrays or uint16 bf16 bit patterns."""
    def draw(sd, d, std):
        if rho == 0.0:
            v = normal_f32(sd, (B, T, d), std)
        else:
            eps = normal_f32(sd, (B + 1, T, d), std)
            v = np.float32(rho) * eps[:1] + np.float32(np.sqrt(1.0 - rho * rho)) * eps[1:]
        return to_dtype(v, dtype)
    out = []
    for j, (d, has_x) in enumerate(vectors):
        e = dict(kind="vector", d=d, delta=draw(seed + 10 * j + 1, d, std_delta), x=None)
        if has_x:
            e["x"] = draw(seed + 10 * j, d, 1.0)
        out.append(e)
    for j, (vocab, d) in enumerate(tables):
        out.append(dict(kind="embed", d=d, vocab=vocab, ids=token_ids(seed + 5000 + j, B, T, vocab),
                        delta=draw(seed + 5000 + 10 * j + 1, d, std_delta)))
    return out


def outer_inputs(config: int, N=None, M=None, seed_offset=0):
    """theta_outer [N], list of M instance vectors theta_k = theta_outer - Delta_k, momentum [N].

    Seeds: theta_outer 9000+config, Delta_k 9100+config+10*k, momentum 9050+config.
    """
    o = CONFIGS[config]["outer"]
    N = o["N"] if N is None else N
    M = o["M"] if M is None else M
    base = 9000 + config + seed_offset
    theta = normal_f32(base, (N,), o["std_theta"])
    insts = [theta - normal_f32(base + 100 + 10 * k, (N,), o["std_delta"]) for k in range(M)]
    if o["std_mom"] > 0:
        mom = normal_f32(base + 50, (N,), o["std_mom"])
    else:
        mom = np.zeros((N,), dtype=np.float32)
    return theta, insts, mom


# --------------------------------------------------------------------------------------
# Device (torch) generators for the full-size workloads: drawn on the GPU from a seeded
# generator because 10^9..10^10 host normals would take minutes.  Tests copy back only
# the slices the oracle checks.
# --------------------------------------------------------------------------------------

def device_normal(seed: int, shape, std: float, dtype, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.empty(shape, dtype=torch.float32, device=device)
    x.normal_(0.0, std, generator=g)
    return x if dtype == torch.float32 else x.to(dtype)


def device_grad_stats_inputs(config: int, device, linears=None, B=None, T=None, rho=0.0,
                             share=False, dtype=None):
    """Device tensors (torch) with the recipe of grad_stats_inputs; bf16 or fp32 per config,
    or the storage type named by dtype ("f32" / "bf16" / "f16").

    share=True reuses one activation tensor for linears of a block that read the same
    input (q/k/v and gate/up in the Llama-shaped workload), as a real model would.
    """
    import torch
    c = CONFIGS[config]
    B = c["B"] if B is None else B
    T = c["T"] if T is None else T
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype or c["dtype"]]
    shapes = linear_shapes(config)
    idx = list(range(len(shapes))) if linears is None else list(linears)
    out = []
    shared = {}
    for li in idx:
        nm, di, do = shapes[li]
        tensors = {}
        for which, (key, d, std) in enumerate((("a", di, c["std_a"]),
                                               ("delta", do, c["std_delta"]))):
            seed = tensor_seed(config, li, which)
            blk, leaf = nm.split(".", 1)
            group = {"q": "qkv", "k": "qkv", "v": "qkv", "gate": "gu", "up": "gu"}.get(leaf)
            if share and key == "a" and group is not None and (blk, group) in shared:
                tensors[key] = shared[(blk, group)]
                continue
            if rho == 0.0:
                x = device_normal(seed, (B, T, d), std, torch.float32, device)
            else:
                eps = device_normal(seed, (B + 1, T, d), std, torch.float32, device)
                x = rho * eps[:1] + float(np.sqrt(1.0 - rho * rho)) * eps[1:]
                del eps
            x = x.to(tdt).contiguous()
            tensors[key] = x
            if share and key == "a" and group is not None:
                shared[(blk, group)] = x
        out.append(dict(name=nm, d_in=di, d_out=do, a=tensors["a"], delta=tensors["delta"]))
    return out


def round_rho_schedule(eta: float, b_schedule, stat_targets):
    """Correlation rho of each outer step's batches such that, for samples x_i = rho x0 + sqrt(1 -
    rho^2) eps_i in both operands of every block (x0 shared by the whole batch), the norm-test
    statistic of a batch of b samples lands near the target: with r = rho^4 the share of the
    squared gradient that the samples have in common, stat ~ (1 - r) / (eta^2 (r + (1 - r) / b)).
    Input recipe only: nothing here is computed from gradients."""
    out = []
    for b, s in zip(b_schedule, stat_targets):
        e = eta * eta * s
        r = (1.0 - e / b) / (1.0 + e * (1.0 - 1.0 / b))
        out.append(float(max(r, 0.0) ** 0.25))
    return out


def device_round_micro_batches(config: int, device, rhos, linears=None, B=None, T=None, dtype=None):
    """Micro-batches of one trainer's accumulated batches, on the device: set s holds, for every
    linear, a [B, T, d_in] and delta [B, T, d_out] with samples x_i = rhos[s] x0 + sqrt(1 -
    rhos[s]^2) eps_i.  x0 (one [1, T, d] tensor per operand and linear, seed = tensor_seed) is common
    to all sets, so that micro-batches accumulated into one batch share their mean; eps has seed
    tensor_seed + 100000 (set + 1).  Returns sets[s] = list of dicts {name, d_in, d_out, a, delta}."""
    import torch
    c = CONFIGS[config]
    B = c["B"] if B is None else B
    T = c["T"] if T is None else T
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype or c["dtype"]]
    shapes = linear_shapes(config)
    idx = list(range(len(shapes))) if linears is None else list(linears)
    sets = [[] for _ in rhos]
    for li in idx:
        nm, di, do = shapes[li]
        per_set = [dict(name=nm, d_in=di, d_out=do) for _ in rhos]
        for which, (key, d, std) in enumerate((("a", di, c["std_a"]), ("delta", do, c["std_delta"]))):
            seed = tensor_seed(config, li, which)
            x0 = device_normal(seed, (1, T, d), std, torch.float32, device)
            for s, rho in enumerate(rhos):
                eps = device_normal(seed + 100000 * (s + 1), (B, T, d), std, torch.float32, device)
                eps.mul_(float(np.sqrt(1.0 - rho * rho))).add_(x0, alpha=float(rho))
                per_set[s][key] = eps.to(tdt).contiguous()
                del eps
            del x0
        for s in range(len(rhos)):
            sets[s].append(per_set[s])
    return sets


def device_outer_inputs(config: int, device, N=None, M=None):
    import torch
    o = CONFIGS[config]["outer"]
    N = o["N"] if N is None else N
    M = o["M"] if M is None else M
    base = 9000 + config
    theta = device_normal(base, (N,), o["std_theta"], torch.float32, device)
    insts = []
    for k in range(M):
        d = device_normal(base + 100 + 10 * k, (N,), o["std_delta"], torch.float32, device)
        insts.append(theta - d)
        del d
    if o["std_mom"] > 0:
        mom = device_normal(base + 50, (N,), o["std_mom"], torch.float32, device)
    else:
        mom = torch.zeros((N,), dtype=torch.float32, device=device)
    return theta, insts, mom


# --------------------------------------------------------------------------------------
# One outer step of Algorithm 3 on tiny blocks: the stand-in for the model (sampling and
# backward pass are outside the hot path) and the trainers' initial state.
# --------------------------------------------------------------------------------------

def round_batch_fn(shapes, T, vec=False):
    """batch_fn(uid, worker, inner_step, micro_step, b, theta) -> blocks for b samples: one (a, delta)
    pair per (d_in, d_out) in `shapes` (fp32; a component shared by the samples of a call keeps the
    batch gradient away from zero), plus the bias vector of the last linear layer when `vec`.
    Every (uid, worker, inner_step, micro_step, block) has its own seed, so that a driver which
    asks for the wrong batch gets different numbers."""
    def fn(uid, worker, h, s, b, theta):
        out = []
        for l, (di, do) in enumerate(shapes):
            r = np.random.Generator(np.random.PCG64(100000 * uid + 1000 * worker + 100 * h + 10 * s + l))
            shared = r.standard_normal((1, T, di + do))
            x = 0.6 * shared + 0.8 * r.standard_normal((b, T, di + do))
            out.append((x[:, :, :di].astype(np.float32), (0.1 * x[:, :, di:]).astype(np.float32)))
        if vec:
            out.append(("rowsum", None, out[-1][1]))
        return out
    return fn


def round_trainers(k, M, N, b_reqs, seed=77, stale_workers=False):
    """k trainers with M workers each over N flat fp32 parameters.  With `stale_workers` the
    workers start from parameters, AdamW moments and step counts of their own, as they would after
    earlier outer steps: only then does a driver that forgets the worker reset show."""
    r = np.random.Generator(np.random.PCG64(seed))
    ts = []
    for i in range(k):
        th = (0.02 * r.standard_normal(N)).astype(np.float32)
        mom = (1e-3 * r.standard_normal(N)).astype(np.float32) if stale_workers else np.zeros(N, np.float32)
        ws = []
        for _ in range(M):
            if stale_workers:
                ws.append(dict(theta=(0.02 * r.standard_normal(N)).astype(np.float32),
                               exp_avg=(1e-3 * r.standard_normal(N)).astype(np.float32),
                               exp_avg_sq=(1e-6 * r.standard_normal(N) ** 2).astype(np.float32),
                               step=int(r.integers(1, 5))))
            else:
                ws.append(dict(theta=th.copy(), exp_avg=np.zeros(N, np.float32),
                               exp_avg_sq=np.zeros(N, np.float32), step=0))
        ts.append(dict(uid=i, theta_outer=th, momentum=mom, b_req=b_reqs[i], workers=ws))
    return ts
