"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Tolerances (stated by the workload definition): relative 1e-4 for norms of
fp32 inputs, 2e-3 for norms of bf16 inputs, 1e-6 relative element-wise for the fp32 outer
step and merge (relative to the operand scale), identical decisions unless the statistic lies
within 1e-3 (relative) of a cut."""
import math

import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-3
TOL_OUTER = 1e-6


# Every test runs twice: with the per-sample norms taken from the per-sample gradient tiles on
# their way into the gradient sum (the default where the blocks qualify), and with the Gram and
# gradient-sum kernels.
@pytest.fixture(scope="module", params=[1, 0], ids=["tile_stats", "gram"])
def ctx(request):
    import paper_2508_18182_amd as A
    c = A.Context(0)
    c.set_tuning("stats_variant", request.param)
    yield c
    c.close()


def _check_grad_stats(ctx, host_layers, tol, wgrad_variant=None):
    from gpu_util import run_grad_stats, rel_err
    if wgrad_variant is not None:
        ctx.set_tuning("wgrad_variant", wgrad_variant)
    got = run_grad_stats(ctx, host_layers)
    want = orc.grad_stats([(l["a"], l["delta"]) for l in host_layers], two_pass=False)
    B = want["B"]
    assert got["n_samples"] == B
    assert rel_err(got["per_layer"], want["n_layer_sample"]) < tol
    assert rel_err(got["per_sample"], want["n_sample"]) < tol
    assert rel_err(got["S1"], want["S1"]) < tol
    for l, (g, w) in enumerate(zip(got["G"], want["G"])):
        scale = float(np.sqrt(np.mean(w * w))) + 1e-300
        err = float(np.max(np.abs(g.astype(np.float64) - w))) / scale
        assert err < 1e-4, (l, err)
    return got, want


# ------------------------------------------------------------------ grad stats

def test_tiny_config_fp32(ctx):
    # workload 1: one 64->32 linear, B=8, T=16, fp32
    layers = synth.grad_stats_inputs(1)
    got, want = _check_grad_stats(ctx, layers, TOL_F32)
    import paper_2508_18182_amd as A
    res = A.adloco_norm_test(ctx, got["layers"], got["acc"], 0.5, 8, 32)
    # the oracle's own variance: the second pass over the explicit per-sample gradients
    want2 = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=True)
    ref = orc.norm_test(want2["S1"], want2["S2"], 8, 0.5, 8, 32, V=want2["V"])
    assert res["S2"] == pytest.approx(want["S2"], rel=TOL_F32)
    assert res["stat"] == pytest.approx(ref["stat"], rel=1e-3)
    for k in ("b_req", "test_passed", "accumulate", "accum_steps", "b_micro"):
        assert res[k] == ref[k], k


@pytest.mark.parametrize("B,T,shapes", [
    (3, 70, [(40, 24), (17, 9), (64, 64)]),       # ragged tiles, odd dims
    (1, 1, [(5, 3)]),                               # single sample, single token
    (2, 33, [(1, 1), (1, 7), (6, 1)]),              # degenerate widths
])
def test_fp32_shapes(ctx, B, T, shapes):
    layers = synth.custom_grad_stats_inputs(500 + B + T, shapes, B, T, "f32", std_delta=0.3, rho=0.4)
    _check_grad_stats(ctx, layers, TOL_F32)


@pytest.mark.parametrize("variant", [0, 1])
def test_bf16_gpt2_block_mid(ctx, variant):
    # one GPT-2-small block, B=8, T=320: 2.5 T-tiles, all fast-path shapes
    shapes = [(768, 2304), (768, 768), (768, 3072), (3072, 768)]
    layers = synth.custom_grad_stats_inputs(600, shapes, 8, 320, "bf16", rho=0.3)
    _check_grad_stats(ctx, layers, TOL_BF16, wgrad_variant=variant)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("B,T,shapes", [
    (5, 133, [(100, 52), (72, 200), (8, 8), (136, 264)]),   # ragged T tile, guarded loads
    (2, 128, [(64, 64)]),                                    # exactly one tile
    (3, 129, [(256, 128)]),                                  # one row into the second tile
    (1, 1, [(8, 16)]),                                       # one token
    (4, 257, [(7, 5), (1, 1), (9, 130)]),                    # odd widths: 2-byte path
    (9, 40, [(128, 384)]),                                   # B not a multiple of the XCD count
    (4, 64, [(8, 16), (264, 520), (256, 256)]),              # 256-tile gradient kernel: clamped edges
    (2, 512, [(64, 320), (320, 64)]),                        # four T tiles, many k-chunks
    (3, 384, [(128, 64)]),                                   # three T tiles: a single-pair job
])
def test_bf16_ragged_and_edges(ctx, variant, B, T, shapes):
    layers = synth.custom_grad_stats_inputs(700 + B + T, shapes, B, T, "bf16", std_delta=0.05,
                                            rho=0.5)
    _check_grad_stats(ctx, layers, TOL_BF16, wgrad_variant=variant)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("B,T,shapes", [
    (5, 133, [(100, 52), (72, 200), (8, 8), (136, 264)]),   # ragged T tile, guarded loads
    (4, 257, [(7, 5), (1, 1), (9, 130)]),                    # odd widths: 2-byte path
    (4, 64, [(8, 16), (264, 520), (256, 256)]),              # 256-tile gradient kernel
    (2, 512, [(64, 320), (320, 64)]),                        # four T tiles, many k-chunks
])
def test_fp16_shapes(ctx, variant, B, T, shapes):
    # fp16 inputs (the mixed-precision setting of Section 6): same kernels, the other MFMA
    layers = synth.custom_grad_stats_inputs(750 + B + T, shapes, B, T, "f16", std_delta=0.05,
                                            rho=0.5)
    _check_grad_stats(ctx, layers, TOL_BF16, wgrad_variant=variant)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("T", [1, 64, 127, 128, 129, 255, 256, 257, 384, 500, 640])
def test_gram_symmetry_shortcuts_at_ragged_T(dtype, T):
    # the dual-tile Gram kernel (widths multiples of 64) leaves out the mirrored parts of the tile
    # pairs on the diagonal: every position of the sequence end relative to the 128-row blocks,
    # the 64-row wave tiles and the 32-row MFMA blocks
    import paper_2508_18182_amd as A
    c = A.Context(0)
    try:
        c.set_tuning("stats_variant", 0)
        layers = synth.custom_grad_stats_inputs(770 + T, [(64, 128), (192, 64)], 3, T, dtype, std_delta=0.05,
                                                rho=0.5)
        _check_grad_stats(c, layers, TOL_BF16)
    finally:
        c.close()


def test_bf16_strided_rows(ctx):
    # a and delta as column slices of wider buffers (fused qkv-style storage)
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import to_dev, new_acc, read_acc, rel_err, DEV
    B, T = 4, 200
    wide = synth.custom_grad_stats_inputs(800, [(256, 384)], B, T, "bf16", rho=0.3)[0]
    a_w, d_w = to_dev(wide["a"]), to_dev(wide["delta"])
    cuts = [((0, 128), (0, 128)), ((128, 256), (128, 384)), ((64, 192), (8, 72))]
    layers, host = [], []
    for (a0, a1), (d0, d1) in cuts:
        layers.append(dict(a=a_w[:, :, a0:a1], delta=d_w[:, :, d0:d1],
                           grad_sum=torch.zeros(d1 - d0, a1 - a0, device=DEV)))
        host.append((np.ascontiguousarray(wide["a"][:, :, a0:a1]),
                     np.ascontiguousarray(wide["delta"][:, :, d0:d1])))
    ps = torch.zeros(B, device=DEV)
    pl = torch.zeros(len(cuts), B, device=DEV)
    acc = new_acc()
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, pl, acc)
    torch.cuda.synchronize()
    want = orc.grad_stats(host, two_pass=False)
    assert rel_err(pl.cpu().numpy(), want["n_layer_sample"]) < TOL_BF16
    assert rel_err(read_acc(acc)[0], want["S1"]) < TOL_BF16
    for l, w in zip(layers, want["G"]):
        g = l["grad_sum"].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(g - w)) / np.sqrt(np.mean(w * w)) < 1e-4


def test_micro_batch_accumulation_matches_concatenation(ctx):
    # switch mode: S1, n_samples and grad_sum carried over three micro-batches; the oracle
    # simply concatenates the micro-batches (Algorithm 3, accumulate branch)
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import run_grad_stats, rel_err, DEV
    shapes = [(128, 192), (96, 64)]
    mbs = [synth.custom_grad_stats_inputs(900 + 100 * m, shapes, 4, 150, "bf16", rho=0.6)
           for m in range(3)]
    grad_sums = [torch.full((do, di), float("nan"), device=DEV) for di, do in shapes]
    acc = None
    for m, mb in enumerate(mbs):
        out = run_grad_stats(ctx, mb, flags=A.ADLOCO_ACCUMULATE if m else 0, acc=acc,
                             grad_sums=grad_sums)
        acc = out["acc"]
    want = orc.grad_stats(orc.concat_micro_batches(
        [[(l["a"], l["delta"]) for l in mb] for mb in mbs]), two_pass=True)
    assert out["n_samples"] == 12
    assert rel_err(out["S1"], want["S1"]) < TOL_BF16
    res = A.adloco_norm_test(ctx, out["layers"], acc, 0.3, 12, 4, 2, 256)
    assert res["S2"] == pytest.approx(want["S2"], rel=TOL_BF16)
    ref = orc.norm_test(want["S1"], want["S2"], 12, 0.3, 12, 4, 2, 256, V=want["V"])
    assert res["variance"] == pytest.approx(ref["variance"], rel=TOL_BF16 * 2)
    _same_decisions(res, ref, eta=0.3, b_cur=12, b_max=4, n_switch=2, b_cap=256)


NEAR_CUT = {"n": 0, "total": 0, "cases": []}


def _same_decisions(res, ref, **oracle_kw):
    """Identical decisions unless the statistic lies within 1e-3 (relative) of a cut (an integer,
    where the ceiling jumps, or b_cur, where the test flips).  On such a boundary case the GPU
    must still decide consistently with its own statistic, which must be within 1e-3 of the
    oracle's."""
    stat = ref["stat"]
    assert res["stat"] == pytest.approx(stat, rel=1e-3)
    # the cuts that can change a decision: b_cur (the test flips there), and the integers next to the
    # statistic unless both neighbours give the same request anyway (below b_cur, or above the ceiling)
    cap = oracle_kw.get("b_cap", 0) or float("inf")
    req = [min(cap, max(ref["b_cur"], c, 1)) for c in (math.floor(stat), math.ceil(stat))]
    cuts = [ref["b_cur"]] + ([math.floor(stat), math.ceil(stat)] if req[0] != req[1] else [])
    near = any(c > 0 and abs(stat - c) <= 1e-3 * c for c in cuts)
    NEAR_CUT["total"] += 1
    if near:
        NEAR_CUT["n"] += 1
        NEAR_CUT["cases"].append((round(stat, 4), dict(oracle_kw)))
        ref = orc.norm_test(res["S1"], res["S2"], res["n_samples"], **oracle_kw)
    for k in ("b_req", "test_passed", "accumulate", "accum_steps", "b_micro", "stat_undefined"):
        assert res[k] == ref[k], (k, res, ref)


@pytest.mark.parametrize("rho,eta,b_cur,b_max,cap", [
    (0.0, 0.31, 8, 32, 0), (0.5, 0.3, 8, 32, 256), (0.9, 0.3, 8, 4, 0), (0.7, 0.8, 8, 2, 64)])
def test_norm_test_decisions(ctx, rho, eta, b_cur, b_max, cap):
    import paper_2508_18182_amd as A
    from gpu_util import run_grad_stats
    shapes = [(128, 256), (256, 64)]
    layers = synth.custom_grad_stats_inputs(1000 + int(rho * 10), shapes, 8, 140, "bf16", rho=rho)
    got = run_grad_stats(ctx, layers)
    want = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=True)
    for flags, kw in ((0, {}), (A.ADLOCO_BIASED_VAR, dict(biased_var=True)),
                      (A.ADLOCO_ALLOW_SHRINK, dict(allow_shrink=True))):
        res = A.adloco_norm_test(ctx, got["layers"], got["acc"], eta, b_cur, b_max, 2, cap, flags)
        ref = orc.norm_test(want["S1"], want["S2"], 8, eta, b_cur, b_max, 2, cap,
                            V=want["V"], **kw)
        assert res["S1"] == pytest.approx(want["S1"], rel=TOL_BF16)
        assert res["S2"] == pytest.approx(want["S2"], rel=TOL_BF16)
        assert res["batch_grad_sqnorm"] == pytest.approx(want["batch_grad_sqnorm"], rel=TOL_BF16)
        _same_decisions(res, ref, eta=eta, b_cur=b_cur, b_max=b_max, n_switch=2, b_cap=cap, **kw)


def test_grad_provided_skips_gradient_sum(ctx):
    import torch
    from gpu_util import run_grad_stats, rel_err, DEV
    shapes = [(64, 128)]
    layers = synth.custom_grad_stats_inputs(1100, shapes, 4, 130, "bf16")
    marker = torch.full((128, 64), 7.0, device=DEV)
    got = run_grad_stats(ctx, layers, grad_sums=[marker], provided=True)
    assert torch.all(marker == 7.0)                      # untouched
    want = orc.grad_stats([(layers[0]["a"], layers[0]["delta"])], two_pass=False)
    assert rel_err(got["per_sample"], want["n_sample"]) < TOL_BF16


def test_repeatable_bitwise(ctx):
    from gpu_util import run_grad_stats
    layers = synth.custom_grad_stats_inputs(1200, [(256, 512), (512, 256)], 6, 300, "bf16", rho=0.2)
    r1, r2 = run_grad_stats(ctx, layers), run_grad_stats(ctx, layers)
    np.testing.assert_array_equal(r1["per_layer"], r2["per_layer"])
    assert r1["S1"] == r2["S1"]
    for g1, g2 in zip(r1["G"], r2["G"]):
        np.testing.assert_array_equal(g1, g2)


# ------------------------------------------------------------------ outer step and merge

def _outer_parity(ctx, theta, insts, mom, lr, mu, nesterov, broadcast, want_pg=True, offset=0):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    N = theta.size

    def dev(x):
        # offset > 0 gives a pointer that is not 16-byte aligned (scalar path)
        buf = torch.zeros(N + offset, device=DEV)
        buf[offset:] = torch.from_numpy(x)
        return buf[offset:]
    th, ms = dev(theta), [dev(x) for x in insts]
    mo = dev(mom) if mom is not None else None
    pg = torch.zeros(N, device=DEV) if want_pg else None
    A.adloco_outer_step(ctx, th, ms, mo, lr, mu, nesterov, A.ADLOCO_BROADCAST if broadcast else 0, pg)
    torch.cuda.synchronize()
    ref = orc.outer_step(theta, insts, mom, lr, mu, nesterov, broadcast)
    scale = np.maximum.reduce([np.abs(theta.astype(np.float64))] +
                              [np.abs(x.astype(np.float64)) for x in insts])

    def ok(got, want64, extra=None):
        s = np.maximum(scale, np.abs(want64))
        if extra is not None:
            s = np.maximum(s, extra)
        assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - want64) <= TOL_OUTER * s)
    ok(th, ref["theta_outer_f64"])
    if mo is not None:
        # the momentum buffer lives at the scale of Delta, far below theta: compare to fp32 rounding
        np.testing.assert_allclose(mo.cpu().numpy(), ref["momentum"], rtol=TOL_OUTER, atol=0)
    if want_pg:
        np.testing.assert_allclose(pg.cpu().numpy(), ref["pseudo_grad"], rtol=TOL_OUTER, atol=0)
    for k, m in enumerate(ms):
        if broadcast:
            assert torch.equal(m, th)
        else:
            np.testing.assert_array_equal(m.cpu().numpy(), insts[k])
    return th, mo


def test_outer_step_tiny_config(ctx):
    theta, insts, mom = synth.outer_inputs(1)
    _outer_parity(ctx, theta, insts, mom, 0.7, 0.9, True, False)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 16])
@pytest.mark.parametrize("N", [1, 3, 4, 1023, 100_003])
def test_outer_step_sizes(ctx, M, N):
    theta, insts, mom = synth.outer_inputs(3, N=N, M=M)
    _outer_parity(ctx, theta, insts, mom, 0.7, 0.9, True, False)


@pytest.mark.parametrize("nesterov,broadcast,mu,with_mom,offset", [
    (True, True, 0.9, True, 0), (False, False, 0.9, True, 0), (True, False, 0.0, False, 0),
    (False, True, 0.0, True, 0), (True, True, 0.9, True, 1), (True, False, 0.5, True, 3)])
def test_outer_step_modes(ctx, nesterov, broadcast, mu, with_mom, offset):
    theta, insts, mom = synth.outer_inputs(3, N=70_001, M=4)
    _outer_parity(ctx, theta, insts, mom if with_mom else None, 0.7, mu, nesterov, broadcast,
                  want_pg=not broadcast, offset=offset)


def test_outer_step_invariants_on_gpu(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    theta, insts, mom = synth.outer_inputs(3, N=50_000, M=4)
    # M = 1, lr = 1, mu = 0 returns the inner model (to fp32 rounding of theta - (theta - x))
    th = torch.from_numpy(theta).to(DEV)
    x = torch.from_numpy(insts[0]).to(DEV)
    A.adloco_outer_step(ctx, th, [x], None, 1.0, 0.0, True)
    np.testing.assert_allclose(th.cpu().numpy(), insts[0], rtol=1e-6, atol=0)
    # instance order does not matter beyond the tolerance
    outs = []
    for perm in ([0, 1, 2, 3], [3, 1, 0, 2]):
        th = torch.from_numpy(theta).to(DEV)
        mo = torch.from_numpy(mom).to(DEV)
        A.adloco_outer_step(ctx, th, [torch.from_numpy(insts[p]).to(DEV) for p in perm], mo, 0.7, 0.9)
        outs.append(th.cpu().numpy().astype(np.float64))
    assert np.all(np.abs(outs[0] - outs[1]) <= TOL_OUTER * np.abs(theta))


@pytest.mark.parametrize("S", [1, 2, 4, 7, 16])
@pytest.mark.parametrize("N,offset", [(5, 0), (100_003, 0), (4096, 2)])
def test_merge(ctx, S, N, offset):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    _, xs, _ = synth.outer_inputs(3, N=N, M=S, seed_offset=S)
    r = np.random.Generator(np.random.PCG64(S * 31 + N))
    w = [int(v) for v in r.integers(1, 300, size=S)]
    bufs = []
    for x in xs:
        b = torch.zeros(N + offset, device=DEV)
        b[offset:] = torch.from_numpy(x)
        bufs.append(b[offset:])
    rep = A.adloco_merge(ctx, bufs, w)
    torch.cuda.synchronize()
    ref = orc.merge(xs, w)
    assert rep == ref["rep"]
    scale = np.max(np.abs(np.stack(xs)), axis=0).astype(np.float64)
    got = bufs[rep].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref["x_merge_f64"]) <= TOL_OUTER * scale)
    for j in range(S):
        if j != rep:
            np.testing.assert_array_equal(bufs[j].cpu().numpy(), xs[j])   # untouched, bit for bit
    if S == 1:
        np.testing.assert_array_equal(bufs[0].cpu().numpy(), xs[0])


def test_merge_explicit_rep_and_ties(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    _, xs, _ = synth.outer_inputs(3, N=1000, M=3)
    bufs = [torch.from_numpy(x).to(DEV) for x in xs]
    assert A.adloco_merge(ctx, bufs, [4, 9, 9]) == 1        # first of the tied maxima
    bufs = [torch.from_numpy(x).to(DEV) for x in xs]
    assert A.adloco_merge(ctx, bufs, [4, 9, 9], rep=0) == 0
    ref = orc.merge(xs, [4, 9, 9], rep=0)
    np.testing.assert_allclose(bufs[0].cpu().numpy(), ref["x_merge"], rtol=1e-6, atol=1e-9)


# ------------------------------------------------------------------ error paths (host checks)

def test_argument_errors(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc
    th = torch.zeros(16, device=DEV)
    with pytest.raises(A.AdlocoError) as e:
        A.adloco_outer_step(ctx, th, [torch.zeros(16, device=DEV)] * 17, None, 0.7, 0.0)
    assert e.value.code == 2
    with pytest.raises(A.AdlocoError):
        A.adloco_outer_step(ctx, th, [th], None, 0.7, 0.0)          # aliasing
    with pytest.raises(A.AdlocoError):
        A.adloco_outer_step(ctx, th, [torch.zeros(16, device=DEV)], None, 0.7, 0.9)  # mu without buffer
    with pytest.raises(A.AdlocoError):
        A.adloco_merge(ctx, [th, torch.zeros(16, device=DEV)], [1.0, 0.0])  # zero weight
    with pytest.raises(A.AdlocoError):
        A.adloco_merge(ctx, [th, th], [1.0, 2.0])                           # same vector twice
    # N = 0 is a no-op
    A.adloco_outer_step(ctx, th, [torch.zeros(16, device=DEV)], None, 0.7, 0.0, N=0)
    assert torch.all(th == 0)
    # empty accumulator -> ESTATE
    g = torch.zeros(4, 4, device=DEV)
    with pytest.raises(A.AdlocoError) as e:
        A.adloco_norm_test(ctx, [dict(grad_sum=g)], new_acc(), 0.3, 1, 32)
    assert e.value.code == 5
    with pytest.raises(ValueError):
        A.adloco_grad_stats(ctx, [dict(a=torch.zeros(2, 3, 4, device=DEV),
                                       delta=torch.zeros(2, 3, 4, device=DEV))], 2, 3,
                            A.ADLOCO_BF16, torch.zeros(2, device=DEV), None, new_acc())


def test_zz_boundary_cases_are_rare():
    # runs after the decision tests of this module: at most one seeded case in ten may sit on a cut
    assert NEAR_CUT["total"] == 0 or NEAR_CUT["n"] * 10 <= NEAR_CUT["total"], NEAR_CUT


@pytest.mark.parametrize("T", [128, 256, 200])
def test_layers_sharing_their_activation_tensor(ctx, T):
    # q / k / v of a transformer block read one activation tensor, gate / up another: the Gram kernel
    # forms A A^T once per such group (T a multiple of the tile edge) or falls back to one layer at a
    # time (ragged T); the result must not depend on which
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import to_dev, new_acc, read_acc, rel_err, DEV
    B = 3
    shapes = [(128, 192), (128, 192), (128, 192), (192, 128), (128, 64), (128, 64)]
    host = synth.custom_grad_stats_inputs(7300 + T, shapes, B, T, "bf16", std_delta=0.1, rho=0.4)
    for l in (1, 2):
        host[l]["a"] = host[0]["a"]          # q, k, v
    host[5]["a"] = host[4]["a"]              # gate, up
    want = orc.grad_stats([(l["a"], l["delta"]) for l in host], two_pass=False)
    dev_a = {id(l["a"]): to_dev(l["a"]) for l in host}
    for provided in (False, True):
        layers = [dict(a=dev_a[id(l["a"])], delta=to_dev(l["delta"]), provided=provided,
                       grad_sum=torch.from_numpy(np.asarray(G, np.float32)).to(DEV) if provided else
                       torch.full((l["d_out"], l["d_in"]), float("nan"), device=DEV))
                  for l, G in zip(host, want["G"])]
        assert layers[0]["a"].data_ptr() == layers[2]["a"].data_ptr()
        ps = torch.zeros(B, device=DEV)
        pl = torch.zeros(len(layers), B, device=DEV)
        acc = new_acc()
        A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, pl, acc, 0)
        torch.cuda.synchronize()
        assert rel_err(pl.cpu().numpy(), want["n_layer_sample"]) < TOL_BF16
        assert rel_err(ps.cpu().numpy(), want["n_sample"]) < TOL_BF16
        assert rel_err(read_acc(acc)[0], want["S1"]) < TOL_BF16
