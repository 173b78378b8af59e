"""What a training loop does to the statistics entry points: every call comes with other tensors
(fresh activations and output gradients, another worker's gradient buffers) but the same shapes.
After the first call on a list of shapes the library must not rebuild a table, and every call must
use the pointers it was given -- also when a graph captured on one set of buffers is replayed
between eager calls on another.  Checked against the oracle and against the call's own first result.
Also here: ADLOCO_SUM_ONLY (gradient sums without statistics) and the range checks on aliasing."""
import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

SHAPES = [(256, 512), (512, 256), (256, 256)]
B, T = 4, 64


@pytest.fixture(scope="module")
def ctx():
    import paper_2508_18182_amd as A
    c = A.Context(0)
    yield c
    c.close()


def _buffer_set(seed):
    import torch
    from gpu_util import to_dev, DEV
    host = synth.custom_grad_stats_inputs(seed, SHAPES, B, T, "bf16", std_delta=0.1, rho=0.3)
    dev = [dict(a=to_dev(e["a"]), delta=to_dev(e["delta"]),
                grad_sum=torch.full((e["d_out"], e["d_in"]), float("nan"), device=DEV)) for e in host]
    return host, dev


def _call(ctx, dev, flags=0, provided=False, with_test=True):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc, read_acc
    ps = torch.full((B,), float("nan"), device=DEV)
    pl = torch.full((len(dev), B), float("nan"), device=DEV)
    acc = new_acc()
    layers = [dict(l, provided=provided) for l in dev]
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, pl, acc, flags)
    nt = A.adloco_norm_test(ctx, layers, acc, 0.3, B, 32) if with_test else None
    torch.cuda.synchronize()
    return dict(ps=ps.cpu().numpy(), pl=pl.cpu().numpy(), S1=read_acc(acc)[0], nt=nt,
                G=[l["grad_sum"].cpu().numpy().copy() for l in dev])


@pytest.mark.parametrize("variant", [1, 0], ids=["tile_stats", "gram"])
def test_rotating_buffer_sets(ctx, variant):
    ctx.set_tuning("stats_variant", variant)
    try:
        sets = [_buffer_set(8800 + 10 * i) for i in range(3)]
        first = [_call(ctx, dev) for _, dev in sets]
        builds = ctx.table_builds()
        for host, r in zip(sets, first):
            want = orc.grad_stats([(e["a"], e["delta"]) for e in host[0]], two_pass=False)
            np.testing.assert_allclose(r["ps"], want["n_sample"], rtol=2e-3)
            np.testing.assert_allclose(r["S1"], want["S1"], rtol=2e-3)
            np.testing.assert_allclose(r["nt"]["S2"], want["S2"], rtol=2e-3)
            for G, Gw in zip(r["G"], want["G"]):
                assert np.max(np.abs(G - Gw)) <= 1e-4 * np.sqrt(np.mean(np.square(Gw)))
        # the three sets differ, so a call that used stale pointers would show
        assert not np.allclose(first[0]["ps"], first[1]["ps"], rtol=1e-3)
        for rnd in range(3):
            for i in (2, 0, 1):
                for l in sets[i][1]:
                    l["grad_sum"].fill_(float("nan"))
                r = _call(ctx, sets[i][1])
                np.testing.assert_array_equal(r["ps"], first[i]["ps"])
                np.testing.assert_array_equal(r["pl"], first[i]["pl"])
                assert r["S1"] == first[i]["S1"] and r["nt"]["S2"] == first[i]["nt"]["S2"]
                for G, G0 in zip(r["G"], first[i]["G"]):
                    np.testing.assert_array_equal(G, G0)
        # same shapes, other addresses: nothing was rebuilt
        assert ctx.table_builds() == builds
        # the gradient supplied by the caller: only grad_sum pointers matter to the norm test
        r = _call(ctx, sets[1][1], provided=True)
        np.testing.assert_allclose(r["ps"], first[1]["ps"], rtol=1e-5)
        assert r["nt"]["S2"] == first[1]["nt"]["S2"]
    finally:
        ctx.set_tuning("stats_variant", 1)


def test_graph_captured_on_one_buffer_set_survives_eager_calls_on_another():
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc
    ctx = A.Context(0)
    (_, dev_a), (_, dev_b), (_, dev_c) = [_buffer_set(8900 + 10 * i) for i in range(3)]
    want_a, want_b, want_c = _call(ctx, dev_a, with_test=False), _call(ctx, dev_b, with_test=False), \
        _call(ctx, dev_c, with_test=False)
    ps = torch.zeros(B, device=DEV)
    pl = torch.zeros(len(dev_b), B, device=DEV)
    acc = new_acc()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):                       # eager once on the capture stream, on set A
        A.adloco_grad_stats(ctx, dev_a, B, T, A.ADLOCO_BF16, ps, pl, acc, 0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):              # captured on set B
        A.adloco_grad_stats(ctx, dev_b, B, T, A.ADLOCO_BF16, ps, pl, acc, 0)
    for rep in range(3):
        other, want_other = (dev_a, want_a) if rep % 2 == 0 else (dev_c, want_c)
        r = _call(ctx, other, with_test=False)       # eager calls on another set in between
        np.testing.assert_array_equal(r["ps"], want_other["ps"])
        for l in dev_b:
            l["grad_sum"].fill_(float("nan"))
        ps.fill_(-1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(ps.cpu().numpy(), want_b["ps"])
        np.testing.assert_array_equal(pl.cpu().numpy(), want_b["pl"])
        for l, G0 in zip(dev_b, want_b["G"]):
            np.testing.assert_array_equal(l["grad_sum"].cpu().numpy(), G0)
        r = _call(ctx, other, with_test=False)       # and the eager path still sees its own pointers
        np.testing.assert_array_equal(r["ps"], want_other["ps"])
        for G, G0 in zip(r["G"], want_other["G"]):
            np.testing.assert_array_equal(G, G0)
    ctx.close()


def test_sum_only_forms_the_gradient_sums_and_nothing_else(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    host, dev = _buffer_set(9000)
    full = _call(ctx, dev, with_test=False)
    for l in dev:
        l["grad_sum"].fill_(float("nan"))
    A.adloco_grad_stats(ctx, dev, B, T, A.ADLOCO_BF16, None, None, None, A.ADLOCO_SUM_ONLY)
    torch.cuda.synchronize()
    for l, G0 in zip(dev, full["G"]):
        G = l["grad_sum"].cpu().numpy()
        assert np.max(np.abs(G - G0)) <= 1e-5 * np.sqrt(np.mean(np.square(G0)))
    # accumulating on top: twice the sum
    A.adloco_grad_stats(ctx, dev, B, T, A.ADLOCO_BF16, None, None, None,
                        A.ADLOCO_SUM_ONLY | A.ADLOCO_ACCUMULATE)
    torch.cuda.synchronize()
    for l, G0 in zip(dev, full["G"]):
        G = l["grad_sum"].cpu().numpy()
        assert np.max(np.abs(G - 2 * G0)) <= 2e-5 * np.sqrt(np.mean(np.square(G0)))
    # outputs that are passed are left alone
    ps = torch.full((B,), 7.0, device=DEV)
    acc = torch.full((2,), 3.0, dtype=torch.float64, device=DEV)
    A.adloco_grad_stats(ctx, dev, B, T, A.ADLOCO_BF16, ps, None, acc, A.ADLOCO_SUM_ONLY)
    torch.cuda.synchronize()
    assert torch.all(ps == 7.0) and torch.all(acc == 3.0)
    # fp32 inputs and a bias block take the same flag
    h32 = synth.custom_grad_stats_inputs(9001, [(24, 16)], 3, 5, "f32", std_delta=0.1)
    a, d = torch.from_numpy(h32[0]["a"]).to(DEV), torch.from_numpy(h32[0]["delta"]).to(DEV)
    layers = [dict(a=a, delta=d, grad_sum=torch.zeros(16, 24, device=DEV)),
              dict(kind="vector", x=None, delta=d, grad_sum=torch.zeros(16, device=DEV))]
    A.adloco_grad_stats(ctx, layers, 3, 5, A.ADLOCO_F32, None, None, None, A.ADLOCO_SUM_ONLY)
    torch.cuda.synchronize()
    want = orc.grad_stats([(h32[0]["a"], h32[0]["delta"]), ("rowsum", None, h32[0]["delta"])], two_pass=False)
    np.testing.assert_allclose(layers[0]["grad_sum"].cpu().numpy(), want["G"][0], rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(layers[1]["grad_sum"].cpu().numpy(), np.asarray(want["G"][1]).reshape(-1),
                               rtol=1e-4, atol=1e-6)


def test_overlapping_ranges_are_refused(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    buf = torch.zeros(64, device=DEV)
    th, inst = buf[:32], buf[16:48]                  # overlap in 16 floats, distinct pointers
    with pytest.raises(A.AdlocoError):
        A.adloco_outer_step(ctx, th, [inst], None, 0.7, 0.0)
    with pytest.raises(A.AdlocoError):               # momentum overlapping theta_outer
        A.adloco_outer_step(ctx, th, [torch.zeros(32, device=DEV)], buf[8:40], 0.7, 0.9)
    with pytest.raises(A.AdlocoError):               # two written instances overlap
        A.adloco_outer_step(ctx, torch.zeros(32, device=DEV), [buf[:32], buf[31:63]], None, 0.7, 0.0,
                            flags=A.ADLOCO_BROADCAST)
    with pytest.raises(A.AdlocoError):
        A.adloco_merge(ctx, [buf[:32], buf[16:48]], [1.0, 2.0])
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_step(ctx, buf[:16], buf[8:24], torch.zeros(16, device=DEV),
                            torch.zeros(16, device=DEV), step=1, lr=1e-3)
    # adjacent, not overlapping: fine
    A.adloco_merge(ctx, [buf[:32], buf[32:64]], [1.0, 2.0])
    # an instance that is only read may be given twice (it simply counts twice in the mean)
    x = torch.ones(32, device=DEV)
    A.adloco_outer_step(ctx, torch.zeros(32, device=DEV), [x, x], None, 1.0, 0.0)
    torch.cuda.synchronize()
