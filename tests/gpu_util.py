"""Helpers shared by the GPU parity tests: move seeded host inputs to the GPU and run the
HIP path through the C-ABI binding.  No arithmetic of the method lives here."""
import numpy as np
import torch

import paper_2508_18182_amd as A

DEV = "cuda:0"


def to_dev(x: np.ndarray):
    """fp32 / fp16 array -> tensor of that type; uint16 bf16 bit patterns -> bf16 tensor (same bits)."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def code_of(name: str) -> int:
    """"f32" / "bf16" / "f16" -> the library's element type code."""
    return {"f32": A.ADLOCO_F32, "bf16": A.ADLOCO_BF16, "f16": A.ADLOCO_F16}[name]


def dtype_code(x: np.ndarray) -> int:
    if x.dtype == np.float16:
        return A.ADLOCO_F16
    return A.ADLOCO_BF16 if x.dtype == np.uint16 else A.ADLOCO_F32


def new_acc():
    return torch.zeros(2, dtype=torch.float64, device=DEV)


def read_acc(acc):
    h = acc.cpu()
    return float(h[0]), int(h.view(torch.int64)[1])


def run_grad_stats(ctx, host_layers, flags=0, acc=None, grad_sums=None, provided=False):
    """host_layers: list of dicts from adloco_synth (numpy).  Returns dict of GPU results
    copied back to the host."""
    B, T = host_layers[0]["a"].shape[:2]
    dt = dtype_code(host_layers[0]["a"])
    layers = []
    for i, l in enumerate(host_layers):
        a, d = to_dev(l["a"]), to_dev(l["delta"])
        if grad_sums is not None:
            g = grad_sums[i]
        else:
            g = torch.full((l["d_out"], l["d_in"]), float("nan"), dtype=torch.float32, device=DEV)
        layers.append(dict(a=a, delta=d, grad_sum=g, provided=provided))
    ps = torch.full((B,), float("nan"), dtype=torch.float32, device=DEV)
    pl = torch.full((len(layers), B), float("nan"), dtype=torch.float32, device=DEV)
    acc = new_acc() if acc is None else acc
    A.adloco_grad_stats(ctx, layers, B, T, dt, ps, pl, acc, flags)
    torch.cuda.synchronize()
    S1, n = read_acc(acc)
    return dict(per_sample=ps.cpu().numpy(), per_layer=pl.cpu().numpy(), S1=S1, n_samples=n,
                acc=acc, layers=layers, G=[l["grad_sum"].cpu().numpy() for l in layers])


def rel_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-300)))
