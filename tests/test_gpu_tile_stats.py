"""GPU parity of the route of adloco_grad_stats that takes the per-sample norms from the 256 x 128
tiles of the per-sample gradients on their way into the gradient sum (aligned bf16 blocks,
T % 32 == 0, gradient sum formed by the library), against the CPU oracle and against the Gram
route: tiles on the edge of a layer, entries split along the samples (few tiles) and whole entries
(more than 32 tiles on an XCD), accumulation over micro-batches, bitwise repeatability."""
import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3


@pytest.fixture(scope="module")
def ctx():
    import paper_2508_18182_amd as A
    c = A.Context(0)
    yield c
    c.close()


def _check(ctx, layers, flags=0, acc=None, grad_sums=None):
    from gpu_util import run_grad_stats, rel_err
    got = run_grad_stats(ctx, layers, flags=flags, acc=acc, grad_sums=grad_sums)
    return got


def _compare(got, want):
    from gpu_util import rel_err
    assert rel_err(got["per_layer"], want["n_layer_sample"]) < TOL_BF16
    assert rel_err(got["per_sample"], want["n_sample"]) < TOL_BF16
    assert rel_err(got["S1"], want["S1"]) < TOL_BF16
    for l, (g, w) in enumerate(zip(got["G"], want["G"])):
        scale = float(np.sqrt(np.mean(w * w))) + 1e-300
        assert float(np.max(np.abs(g.astype(np.float64) - w))) / scale < 1e-4, l


@pytest.mark.parametrize("B,T,shapes", [
    (5, 32, [(72, 264)]),                  # one chunk per sample, both edges ragged
    (1, 64, [(256, 128)]),                 # exactly one tile, one sample
    (7, 96, [(320, 520), (8, 8)]),         # three chunks per sample, a tiny block
    (40, 32, [(128, 256)]),                # more samples than pieces: uneven sample runs
    (3, 160, [(136, 72), (264, 8), (16, 392)]),
])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_tile_route_small(ctx, dtype, B, T, shapes):
    layers = synth.custom_grad_stats_inputs(6000 + B + T, shapes, B, T, dtype, std_delta=0.2, rho=0.4)
    want = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=False)
    ctx.set_tuning("stats_variant", 1)
    got = _check(ctx, layers)
    assert got["n_samples"] == B
    _compare(got, want)
    # the Gram route agrees to rounding, and the route itself repeats bit for bit
    again = _check(ctx, layers)
    assert np.array_equal(again["per_layer"], got["per_layer"])
    for g0, g1 in zip(got["G"], again["G"]):
        assert np.array_equal(g0, g1)
    ctx.set_tuning("stats_variant", 0)
    gram = _check(ctx, layers)
    ctx.set_tuning("stats_variant", 1)
    assert np.max(np.abs(gram["per_layer"] - got["per_layer"]) / got["per_layer"]) < 1e-4


def test_tile_route_whole_and_split_entries(ctx):
    # 288 tiles: every XCD holds 36, one full round of whole entries and four entries split along
    # the three samples; the second layer straddles two XCDs
    B, T = 3, 32
    shapes = [(2048, 2048), (2048, 2048), (2048, 264)]
    layers = synth.custom_grad_stats_inputs(6100, shapes, B, T, "bf16", std_delta=0.05, rho=0.3)
    want = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=False)
    ctx.set_tuning("stats_variant", 1)
    got = _check(ctx, layers)
    _compare(got, want)


def test_tile_route_extreme_aspect_ratios(ctx):
    # one tile row of 32 tile columns, one tile column of 16 tile rows, and a 5 x 9 grid: the blocks in
    # which the tiles of a layer are ordered are cut off by the layer's edge in every way
    B, T = 2, 32
    shapes = [(4096, 8), (8, 4096), (1160, 1288)]
    layers = synth.custom_grad_stats_inputs(6300, shapes, B, T, "bf16", std_delta=0.05, rho=0.3)
    want = orc.grad_stats([(l["a"], l["delta"]) for l in layers], two_pass=False)
    ctx.set_tuning("stats_variant", 1)
    got = _check(ctx, layers)
    _compare(got, want)
    ctx.set_tuning("stats_variant", 0)       # the gradient-sum GEMM orders its 256 x 256 tiles the same way
    _compare(_check(ctx, layers), want)
    ctx.set_tuning("stats_variant", 1)


def test_tile_route_accumulates_over_micro_batches(ctx):
    # switch mode: S1, n and the gradient sums continue over three micro-batches; whole and split
    # entries both add to what is there
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc
    B, T = 2, 64
    shapes = [(1024, 2048), (520, 136)]
    mbs = [synth.custom_grad_stats_inputs(6200 + 10 * k, shapes, B, T, "bf16", std_delta=0.1, rho=0.3)
           for k in range(3)]
    want = orc.grad_stats(orc.concat_micro_batches([[(l["a"], l["delta"]) for l in mb] for mb in mbs]),
                          two_pass=False)
    ctx.set_tuning("stats_variant", 1)
    gs = [torch.full((do, di), float("nan"), device=DEV) for di, do in shapes]
    acc = new_acc()
    per_layer = []
    for k, mb in enumerate(mbs):
        got = _check(ctx, mb, flags=A.ADLOCO_ACCUMULATE if k else 0, acc=acc, grad_sums=gs)
        per_layer.append(got["per_layer"])
    from gpu_util import rel_err
    assert got["n_samples"] == 3 * B
    assert rel_err(np.concatenate(per_layer, axis=1), want["n_layer_sample"]) < TOL_BF16
    assert rel_err(got["S1"], want["S1"]) < TOL_BF16
    for l, w in enumerate(want["G"]):
        g = gs[l].cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - w))) / (float(np.sqrt(np.mean(w * w))) + 1e-300) < 1e-4
