"""The outer step and the merge on instance drifts stored in bf16 (pack, outer step, merge) against
the oracle: the stored codes bit for bit, the updates within 1e-6 of the operand scale -- both sides
read the same bf16 codes, so the bf16 rounding of the drift is not part of the comparison; how far
it moves the result from the fp32 outer step is checked against its bound (2^-8 of the drifts)."""
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


def _bits(t):
    import torch
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def _from_bits(b, dev="cuda:0"):
    import torch
    return torch.from_numpy(b.view(np.int16).copy()).to(dev).view(torch.bfloat16)


@pytest.mark.parametrize("N,off", [(1, 0), (7, 0), (8, 0), (1000, 0), (100_003, 0), (4099, 1), (4099, 3)])
def test_pack_drift_codes_are_bit_exact(ctx, N, off):
    import torch
    import paper_2508_18182_amd as A
    r = np.random.Generator(np.random.PCG64(500 + N + off))
    th = (0.02 * r.standard_normal(N + off)).astype(np.float32)
    xm = th - (1e-3 * r.standard_normal(N + off) * np.exp(r.uniform(-8, 2, N + off))).astype(np.float32)
    if N > 20:                                      # special values: equal, huge, tiny, inf, nan
        xm[3] = th[3]
        th[5], xm[5] = np.float32(3e38), np.float32(-3e38)
        th[6], xm[6] = np.float32(1e-40), np.float32(0.0)
        th[9], xm[9] = np.float32(np.inf), np.float32(1.0)
        th[11] = np.float32(np.nan)
        # exact ties of the bf16 rounding
        th[13], xm[13] = np.float32(1.0 + 2.0 ** -8), np.float32(0.0)
        th[14], xm[14] = np.float32(1.0 + 3 * 2.0 ** -8), np.float32(0.0)
    d_th, d_xm = torch.from_numpy(th).cuda()[off:], torch.from_numpy(xm).cuda()[off:]   # off: unaligned views
    out = torch.zeros(N + off, dtype=torch.bfloat16, device="cuda:0")[off:]
    A.adloco_pack_drift(ctx, d_th, d_xm, out, N=N)
    torch.cuda.synchronize()
    with np.errstate(all="ignore"):
        want = orc.pack_drift(th[off:], xm[off:])
    got = _bits(out)
    nan = np.isnan(orc.widen(want))
    np.testing.assert_array_equal(got[~nan], want[~nan])
    assert np.all(np.isnan(orc.widen(got[nan])))


@pytest.mark.parametrize("M", [1, 2, 3, 4, 8, 16])
@pytest.mark.parametrize("N,off", [(5, 0), (4096, 0), (100_003, 0), (100_003, 1)])
def test_outer_step_drift(ctx, M, N, off):
    import torch
    import paper_2508_18182_amd as A
    theta, insts, mom = synth.outer_inputs(1, N=N + off, M=M, seed_offset=7 * M)
    mom = synth.normal_f32(600 + M, (N + off,), 1e-4)
    bits = [orc.pack_drift(theta, x) for x in insts]
    d_theta = torch.from_numpy(theta).cuda()[off:]
    d_mom = torch.from_numpy(mom).cuda()[off:]
    d_drift = [_from_bits(b)[off:] for b in bits]
    pg = torch.zeros(N + off, device="cuda:0")[off:]
    A.adloco_outer_step_drift(ctx, d_theta, d_drift, d_mom, 0.7, 0.9, True, 0, pg, N=N)
    torch.cuda.synchronize()
    ref = orc.outer_step_drift(theta[off:], [b[off:] for b in bits], mom[off:], 0.7, 0.9, True)
    scale = np.maximum(np.abs(theta[off:].astype(np.float64)), np.abs(ref["theta_outer_f64"]))
    got = d_theta.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref["theta_outer_f64"]) <= TOL * scale)
    np.testing.assert_allclose(d_mom.cpu().numpy(), ref["momentum"], rtol=TOL, atol=1e-30)
    np.testing.assert_allclose(pg.cpu().numpy(), ref["pseudo_grad"], rtol=TOL, atol=1e-30)
    for t, b in zip(d_drift, bits):
        np.testing.assert_array_equal(_bits(t), b[off:])             # drifts untouched without the reset
    # distance from the fp32 outer step: the bf16 rounding of the drifts, at most 2^-8 of their mean size
    full = orc.outer_step(theta[off:], [x[off:] for x in insts], mom[off:], 0.7, 0.9, True)
    bound = 2.0 ** -8 * np.mean([np.abs(theta[off:].astype(np.float64) - x[off:]) for x in insts], axis=0)
    assert np.all(np.abs(pg.cpu().numpy() - full["pseudo_grad_f64"]) <= bound + 1e-9)


def test_outer_step_drift_modes_and_errors(ctx):
    import torch
    import paper_2508_18182_amd as A
    N, M = 10_000, 3
    theta, insts, mom = synth.outer_inputs(1, N=N, M=M)
    bits = [orc.pack_drift(theta, x) for x in insts]
    for nesterov, mu, use_mom in ((False, 0.9, True), (True, 0.0, False), (True, 0.5, True)):
        d_theta = torch.from_numpy(theta).cuda()
        d_mom = torch.from_numpy(mom).cuda() if use_mom else None
        d_drift = [_from_bits(b) for b in bits]
        A.adloco_outer_step_drift(ctx, d_theta, d_drift, d_mom, 0.3, mu, nesterov, A.ADLOCO_BROADCAST)
        torch.cuda.synchronize()
        ref = orc.outer_step_drift(theta, bits, mom if use_mom else None, 0.3, mu, nesterov, broadcast=True)
        np.testing.assert_allclose(d_theta.cpu().numpy(), ref["theta_outer"], rtol=TOL, atol=1e-9)
        for t in d_drift:
            assert not _bits(t).any()                                  # the reset leaves zero drifts
    th = torch.zeros(64, device="cuda:0")
    d = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(A.AdlocoError):
        A.adloco_outer_step_drift(ctx, th, [d], None, 0.7, 0.9)       # mu without a buffer
    with pytest.raises(A.AdlocoError) as e:
        A.adloco_outer_step_drift(ctx, th, [d] * 17, None, 0.7, 0.0)
    assert e.value.code == 2
    with pytest.raises(A.AdlocoError):                                 # written drifts overlap
        A.adloco_outer_step_drift(ctx, th[:32], [d[:32], d[16:48]], None, 0.7, 0.0, True, A.ADLOCO_BROADCAST)
    with pytest.raises(TypeError):
        A.adloco_outer_step_drift(ctx, th, [th], None, 0.7, 0.0)      # fp32 where bf16 is expected
    A.adloco_outer_step_drift(ctx, th, [d], None, 0.7, 0.0, N=0)      # N = 0: no-op


@pytest.mark.parametrize("S", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("N,off", [(9, 0), (100_003, 0), (65_537, 1)])
def test_merge_drift(ctx, S, N, off):
    import torch
    import paper_2508_18182_amd as A
    r = np.random.Generator(np.random.PCG64(700 + S))
    xr = (0.02 * r.standard_normal(N + off)).astype(np.float32)
    others = [xr - (1e-3 * r.standard_normal(N + off)).astype(np.float32) for _ in range(S - 1)]
    bits = [orc.pack_drift(xr, x) for x in others]
    w_rep, w_o = 40.0, [float(v) for v in r.integers(1, 40, size=S - 1)]
    d_x = torch.from_numpy(xr).cuda()[off:]
    d_drift = [_from_bits(b)[off:] for b in bits]
    A.adloco_merge_drift(ctx, d_x, d_drift, w_rep, w_o, N=N)
    torch.cuda.synchronize()
    ref = orc.merge_drift(xr[off:], [b[off:] for b in bits], w_rep, w_o)
    got = d_x.cpu().numpy().astype(np.float64)
    if S == 1:
        np.testing.assert_array_equal(d_x.cpu().numpy(), xr[off:])    # singleton: bit-identical
    # relative to the operand scale: the representative, the result and the drifts that enter it
    scale = np.maximum.reduce([np.abs(xr[off:].astype(np.float64)), np.abs(ref["x_merge_f64"])] +
                              [np.abs(orc.widen(b[off:])) for b in bits])
    assert np.all(np.abs(got - ref["x_merge_f64"]) <= TOL * scale)
    # and it is the merge of the reconstructed trainers
    full = orc.merge([xr[off:].astype(np.float64)] + [xr[off:].astype(np.float64) - orc.widen(b[off:]) for b in bits],
                     [w_rep] + w_o)
    np.testing.assert_allclose(ref["x_merge_f64"], full["x_merge_f64"], rtol=0, atol=1e-16)


def test_round_trip_124m_sampled(ctx):
    # workload 3 at full size: pack the four instances' drifts, outer step from them, sampled elements
    import torch
    import paper_2508_18182_amd as A
    o = synth.CONFIGS[3]["outer"]
    N, M = o["N"] + 1, o["M"]
    theta, insts, mom = synth.device_outer_inputs(3, "cuda:0", N=N)
    r = np.random.Generator(np.random.PCG64(801))
    idx = np.concatenate([np.arange(0, 1024), np.arange(N - 1024, N), r.integers(0, N, 300_000)]).astype(np.int64)
    tidx = torch.from_numpy(idx).cuda()
    h_theta, h_mom = theta[tidx].cpu().numpy(), mom[tidx].cpu().numpy()
    h_inst = [x[tidx].cpu().numpy() for x in insts]
    drifts = [torch.empty(N, dtype=torch.bfloat16, device="cuda:0") for _ in range(M)]
    for x, d in zip(insts, drifts):
        A.adloco_pack_drift(ctx, theta, x, d)
    torch.cuda.synchronize()
    want_bits = [orc.pack_drift(h_theta, x) for x in h_inst]
    for d, wb in zip(drifts, want_bits):
        np.testing.assert_array_equal(_bits(d[tidx]), wb)
    A.adloco_outer_step_drift(ctx, theta, drifts, mom, o["lr"], o["mu"], True)
    torch.cuda.synchronize()
    ref = orc.outer_step_drift(h_theta, want_bits, h_mom, o["lr"], o["mu"], True)
    got = theta[tidx].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref["theta_outer_f64"]) <= TOL * np.maximum(np.abs(h_theta), np.abs(got)))
    np.testing.assert_allclose(mom[tidx].cpu().numpy(), ref["momentum"], rtol=TOL, atol=0)
