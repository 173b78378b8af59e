"""GPU parity at the full workload sizes, in the launch configuration bench.py times.

The explicit oracle costs 10^12..10^14 flop on these shapes, so it is evaluated on sampled
outputs (single (layer, sample) norms, single rows of the gradient sum, random elements of the
parameter vectors) whose inputs are copied back from the GPU, plus properties that hold at any
size.  Inputs are drawn on the device from seeded generators (adloco_synth)."""
import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

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


def _bits(t):
    """bf16 device tensor -> uint16 bit patterns on the host."""
    import torch
    return t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def _run_stats(ctx, layers, B, T, flags=0, acc=None):
    import torch
    import paper_2508_18182_amd as A
    dev = layers[0]["a"].device
    for l in layers:
        if "grad_sum" not in l:
            l["grad_sum"] = torch.full((l["d_out"], l["d_in"]), float("nan"), device=dev)
    ps = torch.zeros(B, device=dev)
    pl = torch.zeros(len(layers), B, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev) if acc is None else acc
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, pl, acc, flags)
    torch.cuda.synchronize()
    return ps, pl, acc


def _check_sampled_norms(layers, pl, picks):
    for (l, i) in picks:
        g = orc.per_sample_gradient(_bits(layers[l]["a"][i]), _bits(layers[l]["delta"][i]))
        want = float(np.sum(g * g))
        got = float(pl[l, i])
        assert abs(got - want) <= TOL_BF16 * want, (l, i, got, want)


def _check_grad_rows(layer, rows):
    """rows of grad_sum = sum over all tokens of delta[token, e] * a[token, :]."""
    a = orc.widen(_bits(layer["a"].reshape(-1, layer["d_in"])))
    G = layer["grad_sum"]
    for e in rows:
        col = orc.widen(_bits(layer["delta"].reshape(-1, layer["d_out"])[:, e]))
        want = col @ a
        got = G[e].cpu().numpy().astype(np.float64)
        scale = float(np.sqrt(np.mean(want * want)))
        assert np.max(np.abs(got - want)) <= 1e-4 * scale, (e, np.max(np.abs(got - want)), scale)


def test_gpt2_small_full_workload(ctx):
    # workload 2: 48 linears, B = 32, T = 512, bf16; exactly what bench.py launches
    import torch
    import paper_2508_18182_amd as A
    B, T, eta = 32, 512, 0.3
    layers = synth.device_grad_stats_inputs(2, "cuda:0")
    assert len(layers) == 48
    ps, pl, acc = _run_stats(ctx, layers, B, T)
    # sampled per-(layer, sample) norms against explicit per-sample gradients
    _check_sampled_norms(layers, pl, [(0, 0), (1, 31), (2, 7), (3, 16), (45, 3), (47, 30)])
    # sampled rows of the gradient sum (first and last tile of a wide and a tall layer)
    _check_grad_rows(layers[0], [0, 1151, 2303])
    _check_grad_rows(layers[47], [5, 767])
    # properties that hold at any size
    plh, psh = pl.cpu().numpy().astype(np.float64), ps.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(plh.sum(axis=0), psh, rtol=1e-6)
    S1 = float(acc.cpu()[0])
    assert int(acc.cpu().view(torch.int64)[1]) == B
    assert S1 == pytest.approx(psh.sum(), rel=1e-6)
    res = A.adloco_norm_test(ctx, layers, acc, eta, B, 32, 2, 256)
    S2_host = sum(float((l["grad_sum"].double() ** 2).sum()) for l in layers)
    assert res["S2"] == pytest.approx(S2_host, rel=1e-9)
    assert res["S1"] == S1 and res["n_samples"] == B
    # iid zero-mean inputs: stat -> B / eta^2 = 355.6 (closed form), so the batch must grow to the cap
    assert res["stat"] == pytest.approx(B / eta ** 2, rel=0.05)
    ref = orc.norm_test(res["S1"], res["S2"], B, eta, B, 32, 2, 256)
    for k in ("b_req", "test_passed", "accumulate", "accum_steps", "b_micro"):
        assert res[k] == ref[k]
    assert res["b_req"] == 256 and res["accumulate"] == 1 and res["accum_steps"] == 8


def test_llama_1b_block_shared_activations(ctx):
    # workload 4, one block: q,k,v,o 2048->2048, gate,up 2048->5632, down 5632->2048, B = 64,
    # T = 1024; q/k/v and gate/up read the same activation tensor
    layers = synth.device_grad_stats_inputs(4, "cuda:0", linears=range(7), share=True)
    assert layers[0]["a"].data_ptr() == layers[1]["a"].data_ptr() == layers[2]["a"].data_ptr()
    assert layers[4]["a"].data_ptr() == layers[5]["a"].data_ptr()
    ps, pl, acc = _run_stats(ctx, layers, 64, 1024)
    _check_sampled_norms(layers, pl, [(0, 0), (2, 63), (3, 17), (5, 40), (6, 9)])
    _check_grad_rows(layers[1], [0, 2047])
    plh, psh = pl.cpu().numpy().astype(np.float64), ps.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(plh.sum(axis=0), psh, rtol=1e-6)
    assert float(acc.cpu()[0]) == pytest.approx(psh.sum(), rel=1e-6)


def test_round_350m_style_accumulation(ctx):
    # workload 5 in miniature (same T = 1024 and micro-batch cap 32, narrower layers so that the
    # oracle finishes): requested batch 64 > 2 * 32 -> two accumulated micro-batches
    import torch
    import paper_2508_18182_amd as A
    shapes = [(256, 768), (256, 256), (256, 1024), (1024, 256)]
    B, T, eta = 32, 1024, 0.3
    mbs = [synth.custom_grad_stats_inputs(5000 + 100 * m, shapes, B, T, "bf16", rho=0.35)
           for m in range(2)]
    from gpu_util import to_dev
    grad_sums = [torch.full((do, di), float("nan"), device="cuda:0") for di, do in shapes]
    acc = None
    for m, mb in enumerate(mbs):
        layers = [dict(a=to_dev(l["a"]), delta=to_dev(l["delta"]), d_in=l["d_in"], d_out=l["d_out"],
                       grad_sum=g) for l, g in zip(mb, grad_sums)]
        ps, pl, acc = _run_stats(ctx, layers, B, T, A.ADLOCO_ACCUMULATE if m else 0, acc)
    want = orc.grad_stats(orc.concat_micro_batches(
        [[(l["a"], l["delta"]) for l in mb] for mb in mbs]), two_pass=True)
    res = A.adloco_norm_test(ctx, layers, acc, eta, 64, 32, 2, 256)
    assert res["n_samples"] == 64
    assert res["S1"] == pytest.approx(want["S1"], rel=TOL_BF16)
    assert res["S2"] == pytest.approx(want["S2"], rel=TOL_BF16)
    ref = orc.norm_test(want["S1"], want["S2"], 64, eta, 64, 32, 2, 256, V=want["V"])
    assert res["stat"] == pytest.approx(ref["stat"], rel=1e-3)
    near = any(abs(ref["stat"] - c) <= 1e-3 * c for c in (np.floor(ref["stat"]), np.ceil(ref["stat"]), 64) if c > 0)
    if not near:
        for k in ("b_req", "test_passed", "accumulate", "accum_steps", "b_micro"):
            assert res[k] == ref[k], k


def _sample_idx(N, n, seed):
    r = np.random.Generator(np.random.PCG64(seed))
    idx = np.concatenate([np.arange(0, 1024), np.arange(N - 1024, N),
                          r.integers(0, N, size=n)]).astype(np.int64)
    return idx


@pytest.mark.parametrize("N", [124_000_000, 124_000_001])
def test_outer_step_and_merge_124m(ctx, N):
    # workload 3: M = 4 instances x 124M fp32 parameters, in place; N + 1 exercises the tail
    import torch
    import paper_2508_18182_amd as A
    o = synth.CONFIGS[3]["outer"]
    theta, insts, mom = synth.device_outer_inputs(3, "cuda:0", N=N)
    idx = _sample_idx(N, 500_000, 77)
    tidx = torch.from_numpy(idx).to("cuda:0")
    h_theta = theta[tidx].cpu().numpy()
    h_inst = [x[tidx].cpu().numpy() for x in insts]
    h_mom = mom[tidx].cpu().numpy()
    A.adloco_outer_step(ctx, theta, insts, mom, o["lr"], o["mu"], True)
    torch.cuda.synchronize()
    ref = orc.outer_step(h_theta, h_inst, h_mom, o["lr"], o["mu"], True)
    scale = np.maximum.reduce([np.abs(h_theta.astype(np.float64))] +
                              [np.abs(x.astype(np.float64)) for x in h_inst])
    got = theta[tidx].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref["theta_outer_f64"]) <= TOL_OUTER * np.maximum(scale, np.abs(got)))
    np.testing.assert_allclose(mom[tidx].cpu().numpy(), ref["momentum"], rtol=TOL_OUTER, atol=0)
    for x, hx in zip(insts, h_inst):
        np.testing.assert_array_equal(x[tidx].cpu().numpy(), hx)       # instances untouched
    # merge of the four instances, weights = requested batches
    w = [32, 64, 256, 128]
    rep = A.adloco_merge(ctx, insts, w)
    torch.cuda.synchronize()
    m = orc.merge(h_inst, w)
    assert rep == m["rep"] == 2
    got = insts[rep][tidx].cpu().numpy().astype(np.float64)
    mscale = np.max(np.abs(np.stack(h_inst)), axis=0).astype(np.float64)
    assert np.all(np.abs(got - m["x_merge_f64"]) <= TOL_OUTER * mscale)
    for j in range(4):
        if j != rep:
            np.testing.assert_array_equal(insts[j][tidx].cpu().numpy(), h_inst[j])
    # convexity holds everywhere: min <= merged <= max over the instances (checked on the device)
    others = torch.stack([insts[j] for j in range(4) if j != rep])
    # the representative was overwritten; bound it by the other three and its own old samples
    lo = torch.minimum(others.min(dim=0).values[tidx], torch.from_numpy(h_inst[rep]).to("cuda:0"))
    hi = torch.maximum(others.max(dim=0).values[tidx], torch.from_numpy(h_inst[rep]).to("cuda:0"))
    mg = insts[rep][tidx]
    assert bool(torch.all(mg >= lo - 1e-7) & torch.all(mg <= hi + 1e-7))


def test_outer_step_broadcast_350m_m8(ctx):
    # workload 5's outer half: M = 8 instances x 350M parameters with the worker reset
    import torch
    import paper_2508_18182_amd as A
    o = synth.CONFIGS[5]["outer"]
    N = o["N"]
    theta, insts, mom = synth.device_outer_inputs(5, "cuda:0")
    idx = _sample_idx(N, 300_000, 78)
    tidx = torch.from_numpy(idx).to("cuda:0")
    h_theta = theta[tidx].cpu().numpy()
    h_inst = [x[tidx].cpu().numpy() for x in insts]
    h_mom = mom[tidx].cpu().numpy()
    pg = torch.empty(N, device="cuda:0")
    A.adloco_outer_step(ctx, theta, insts, mom, o["lr"], o["mu"], True, A.ADLOCO_BROADCAST, pg)
    torch.cuda.synchronize()
    ref = orc.outer_step(h_theta, h_inst, h_mom, o["lr"], o["mu"], True, broadcast=True)
    scale = np.maximum.reduce([np.abs(h_theta.astype(np.float64))] +
                              [np.abs(x.astype(np.float64)) for x in h_inst])
    got = theta[tidx].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref["theta_outer_f64"]) <= TOL_OUTER * np.maximum(scale, np.abs(got)))
    np.testing.assert_allclose(pg[tidx].cpu().numpy(), ref["pseudo_grad"], rtol=TOL_OUTER, atol=0)
    for x in insts:
        assert torch.equal(x, theta)                                    # reset everywhere


def test_round_350m_real_widths_eight_micro_batches(ctx):
    # workload 5 at its real widths: one transformer block {1024->3072, 1024->1024, 1024->4096,
    # 4096->1024}, T = 1024, micro-batch cap 32, the batch grown to 256 samples = 8 accumulated
    # micro-batches with their own tensors (as bench.py holds them), then the M = 8 x 350M outer step
    # and the merge of all 8 instances weighted by the requested batches.
    import torch
    import paper_2508_18182_amd as A
    cfg = synth.CONFIGS[5]
    T, b_max, eta, b_cap = cfg["T"], cfg["b_max"], cfg["eta"], cfg["b_cap"]
    rho = synth.round_rho_schedule(eta, [256], [180.0])[0]
    sets = synth.device_round_micro_batches(5, "cuda:0", [rho] * 8, linears=range(4))
    shapes = [(l["d_in"], l["d_out"]) for l in sets[0]]
    assert shapes == [(1024, 3072), (1024, 1024), (1024, 4096), (4096, 1024)]
    grad_sums = [torch.full((do, di), float("nan"), device="cuda:0") for di, do in shapes]
    acc = torch.zeros(2, dtype=torch.float64, device="cuda:0")
    per_set, S1_running, checkpoints = [], 0.0, {}
    for m, mb in enumerate(sets):
        layers = [dict(l, grad_sum=g) for l, g in zip(mb, grad_sums)]
        ps, pl, acc = _run_stats(ctx, layers, b_max, T, A.ADLOCO_ACCUMULATE if m else 0, acc)
        per_set.append((ps.cpu().numpy().astype(np.float64), pl.clone()))
        S1_running += float(per_set[-1][0].sum())
        # the running accumulator after 1, 2, 4 and 8 micro-batches
        if m + 1 in (1, 2, 4, 8):
            assert int(acc.cpu().view(torch.int64)[1]) == b_max * (m + 1)
            assert float(acc.cpu()[0]) == pytest.approx(S1_running, rel=1e-6)
            res = A.adloco_norm_test(ctx, layers, acc, eta, b_max * (m + 1), b_max, 2, b_cap)
            S2_host = sum(float((g.double() ** 2).sum()) for g in grad_sums)
            assert res["S2"] == pytest.approx(S2_host, rel=1e-9)
            ref = orc.norm_test(res["S1"], res["S2"], b_max * (m + 1), eta, b_max * (m + 1), b_max, 2, b_cap)
            assert res["stat"] == pytest.approx(ref["stat"], rel=1e-9)
            for k in ("b_req", "test_passed", "accumulate", "accum_steps", "b_micro"):
                assert res[k] == ref[k], (m, k)
            checkpoints[m + 1] = res
    # sampled per-(layer, sample) norms of several micro-batches against explicit per-sample gradients
    for m, picks in ((0, [(0, 0), (3, 31)]), (3, [(1, 7)]), (7, [(2, 19), (3, 2)])):
        _check_sampled_norms(sets[m], per_set[m][1], picks)
    for ps, pl in per_set:
        np.testing.assert_allclose(pl.cpu().numpy().astype(np.float64).sum(axis=0), ps, rtol=1e-6)
    # sampled rows of the accumulated gradient sum: all 256 samples of the 1024->1024 layer
    a_all = np.concatenate([orc.widen(_bits(mb[1]["a"].reshape(-1, 1024))) for mb in sets])
    for e in (0, 517, 1023):
        col = np.concatenate([orc.widen(_bits(mb[1]["delta"].reshape(-1, 1024)[:, e])) for mb in sets])
        want = col @ a_all
        got = grad_sums[1][e].cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - want)) <= 1e-4 * float(np.sqrt(np.mean(want * want))), e
    del a_all
    # the statistic sits where the input recipe puts it (common component rho in every sample)
    assert checkpoints[8]["stat"] == pytest.approx(180.0, rel=0.1)
    assert checkpoints[8]["n_samples"] == 256 and checkpoints[8]["accumulate"] == 1
    sets = None
    torch.cuda.empty_cache()
    # ---- the outer half: 8 instances x 350M, then the merge of all 8 weighted by requested batches
    o = cfg["outer"]
    N = o["N"]
    theta, insts, mom = synth.device_outer_inputs(5, "cuda:0")
    idx = _sample_idx(N, 300_000, 79)
    tidx = torch.from_numpy(idx).to("cuda:0")
    h_theta, h_mom = theta[tidx].cpu().numpy(), mom[tidx].cpu().numpy()
    h_inst = [x[tidx].cpu().numpy() for x in insts]
    A.adloco_outer_step(ctx, theta, insts, mom, o["lr"], o["mu"], True)
    torch.cuda.synchronize()
    ref = orc.outer_step(h_theta, h_inst, h_mom, o["lr"], o["mu"], True)
    scale = np.maximum.reduce([np.abs(h_theta.astype(np.float64))] + [np.abs(x.astype(np.float64)) for x in h_inst])
    got = theta[tidx].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref["theta_outer_f64"]) <= TOL_OUTER * np.maximum(scale, np.abs(got)))
    np.testing.assert_allclose(mom[tidx].cpu().numpy(), ref["momentum"], rtol=TOL_OUTER, atol=0)
    w = [checkpoints[c]["b_req"] for c in (1, 2, 4, 8)] + [checkpoints[c]["b_req"] + 1 for c in (1, 2, 4, 8)]
    assert A.adloco_check_merge(w, 8) == list(np.argsort(np.array(w), kind="stable"))
    rep = A.adloco_merge(ctx, insts, w)
    torch.cuda.synchronize()
    m = orc.merge(h_inst, w)
    assert rep == m["rep"]
    got = insts[rep][tidx].cpu().numpy().astype(np.float64)
    mscale = np.max(np.abs(np.stack(h_inst)), axis=0).astype(np.float64)
    assert np.all(np.abs(got - m["x_merge_f64"]) <= TOL_OUTER * mscale)
    for j in range(8):
        if j != rep:
            np.testing.assert_array_equal(insts[j][tidx].cpu().numpy(), h_inst[j])
