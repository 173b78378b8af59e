"""GPU parity of the fused inner optimizer step (AdamW as Algorithm 3's InnerOpt) against the CPU
oracle: 1e-6 relative to the operand scale, as for the outer step."""
import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 1e-6


@pytest.fixture(scope="module")
def ctx():
    import paper_2508_18182_amd as A
    c = A.Context(0)
    yield c
    c.close()


def _inputs(seed, N):
    theta = synth.normal_f32(seed, (N,), 0.02)
    m = synth.normal_f32(seed + 1, (N,), 1e-3)
    v = np.abs(synth.normal_f32(seed + 2, (N,), 1e-3)) ** 2
    g = synth.normal_f32(seed + 3, (N,), 0.5)
    return theta, m, v.astype(np.float32), g


def _close(got, want, *scales):
    scale = np.maximum.reduce([np.abs(want)] + [np.abs(s) for s in scales])
    return np.all(np.abs(got.astype(np.float64) - want) <= TOL * scale + 1e-300)


@pytest.mark.parametrize("N", [1, 3, 4, 255, 256, 1000, 10_001, 1_000_003])
def test_inner_step_sizes(ctx, N):
    import torch
    import paper_2508_18182_amd as A
    theta, m, v, g = _inputs(4000 + N % 97, N)
    d = [torch.from_numpy(x.copy()).cuda() for x in (theta, m, v, g)]
    A.adloco_inner_step(ctx, d[0], d[1], d[2], d[3], step=3, lr=4e-4, weight_decay=0.1, grad_scale=1.0 / 32)
    torch.cuda.synchronize()
    o = orc.inner_step(theta, m, v, g, 3, 4e-4, weight_decay=0.1, grad_scale=1.0 / 32)
    assert _close(d[0].cpu().numpy(), o["theta_f64"], theta)
    assert _close(d[1].cpu().numpy(), o["exp_avg_f64"], m)
    assert _close(d[2].cpu().numpy(), o["exp_avg_sq_f64"], v)
    np.testing.assert_array_equal(d[3].cpu().numpy(), g)          # the gradient is only read


def test_inner_step_sequence_and_unaligned(ctx):
    # five consecutive steps from a zero state, on views that start 4 bytes off a 16-byte boundary
    import torch
    import paper_2508_18182_amd as A
    N = 5003
    theta = synth.normal_f32(4100, (N,), 0.02)
    bufs = [torch.zeros(N + 1, device="cuda") for _ in range(4)]
    th, m, v, g = [b[1:] for b in bufs]
    th.copy_(torch.from_numpy(theta))
    x64, m64, v64 = theta.astype(np.float64), np.zeros(N), np.zeros(N)
    xs, ms, vs = theta, np.zeros(N, np.float32), np.zeros(N, np.float32)
    for step in range(1, 6):
        gh = synth.normal_f32(4100 + step, (N,), 1.0)
        g.copy_(torch.from_numpy(gh))
        A.adloco_inner_step(ctx, th, m, v, g, step=step, lr=1e-3, beta1=0.8, beta2=0.95, eps=1e-6,
                            weight_decay=0.05, grad_scale=0.5, N=N)
        torch.cuda.synchronize()
        # the oracle steps from the GPU's fp32 state: one rounding per step on either side
        o = orc.inner_step(xs, ms, vs, gh, step, 1e-3, 0.8, 0.95, 1e-6, 0.05, 0.5)
        assert _close(th.cpu().numpy(), o["theta_f64"], xs), step
        assert _close(m.cpu().numpy(), o["exp_avg_f64"], ms, 0.5 * gh * 0.2), step
        assert _close(v.cpu().numpy(), o["exp_avg_sq_f64"], vs), step
        xs, ms, vs = th.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()


def test_inner_step_closed_forms_on_gpu(ctx):
    import torch
    import paper_2508_18182_amd as A
    N = 4096
    theta = synth.normal_f32(4200, (N,), 1.0)
    g = synth.normal_f32(4201, (N,), 1.0) + np.float32(0.01)
    z = lambda: torch.zeros(N, device="cuda")
    th, m, v = torch.from_numpy(theta.copy()).cuda(), z(), z()
    # zero gradient, zero state: pure decoupled decay
    A.adloco_inner_step(ctx, th, m, v, z(), step=1, lr=1e-2, weight_decay=0.1)
    torch.cuda.synchronize()
    want = theta.astype(np.float64) * (1 - 1e-3)
    assert np.max(np.abs(th.cpu().numpy() - want) / np.abs(want)) < 1e-6
    assert float(m.abs().max()) == 0.0 and float(v.abs().max()) == 0.0
    # first step without decay: theta - lr * g / (|g| + eps)
    th, m, v = torch.from_numpy(theta.copy()).cuda(), z(), z()
    A.adloco_inner_step(ctx, th, m, v, torch.from_numpy(g).cuda(), step=1, lr=1e-2, weight_decay=0.0)
    torch.cuda.synchronize()
    g64 = g.astype(np.float64)
    want = theta - 1e-2 * g64 / (np.abs(g64) + 1e-8)
    assert np.max(np.abs(th.cpu().numpy() - want)) < 1e-6 * np.max(np.abs(theta))


def test_inner_step_errors(ctx):
    import torch
    import paper_2508_18182_amd as A
    t = [torch.zeros(16, device="cuda") for _ in range(4)]
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_step(ctx, t[0], t[1], t[2], t[3], step=0, lr=1e-3)          # steps count from 1
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_step(ctx, t[0], t[1], t[2], t[3], step=1, lr=1e-3, beta1=1.0)
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_step(ctx, t[0], t[1], t[0], t[3], step=1, lr=1e-3)          # aliasing
    A.adloco_inner_step(ctx, t[0], t[1], t[2], t[3], step=1, lr=1e-3, N=0)          # no-op


def test_inner_step_124m_sampled(ctx):
    # the size bench.py times: 124M parameters, checked on 5e5 random elements
    import torch
    import paper_2508_18182_amd as A
    N = 124_000_000
    dev = "cuda:0"
    th = synth.device_normal(4300, (N,), 0.02, torch.float32, dev)
    m = synth.device_normal(4301, (N,), 1e-3, torch.float32, dev)
    v = synth.device_normal(4302, (N,), 1e-3, torch.float32, dev).square_()
    g = synth.device_normal(4303, (N,), 0.5 * 32, torch.float32, dev)
    idx = torch.from_numpy(np.random.Generator(np.random.PCG64(4304)).integers(0, N, 500_000)).to(dev)
    idx[:4] = torch.tensor([0, 1, N - 2, N - 1], device=dev)
    before = [t[idx].cpu().numpy() for t in (th, m, v, g)]
    A.adloco_inner_step(ctx, th, m, v, g, step=7, lr=4e-4, weight_decay=0.1, grad_scale=1.0 / 32)
    torch.cuda.synchronize()
    o = orc.inner_step(*before, 7, 4e-4, weight_decay=0.1, grad_scale=1.0 / 32)
    assert _close(th[idx].cpu().numpy(), o["theta_f64"], before[0])
    assert _close(m[idx].cpu().numpy(), o["exp_avg_f64"], before[1])
    assert _close(v[idx].cpu().numpy(), o["exp_avg_sq_f64"], before[2])
