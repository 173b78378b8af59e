"""GPU parity of the vector (bias / gain) and embedding-table blocks of the per-sample gradient:
the HIP path through the C ABI against the CPU oracle on the same seeded inputs.  Tolerances as
for the linear weights: 1e-4 relative for fp32 inputs, 2e-3 for bf16 inputs."""
import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-3, "f16": 2e-3}


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


def _oracle_entry(e):
    kind = e.get("kind", "linear")
    if kind == "vector":
        return ("rowsum", e["x"], e["delta"])
    if kind == "embed":
        return ("embed", e["ids"], e["delta"])
    return (e["a"], e["delta"])


def _run(ctx, entries, B, T, dtype, flags=0, acc=None, grad_sums=None, table_grads=None):
    """entries: host dicts (linear dicts from synth.custom_grad_stats_inputs carry no 'kind')."""
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import to_dev, new_acc, read_acc, code_of, DEV
    layers = []
    on_dev = {}

    def to_dev(x, _up=to_dev):
        # one device tensor per host array: a bias that names its linear layer's delta passes the
        # same pointer, as a framework would
        if id(x) not in on_dev:
            on_dev[id(x)] = _up(x)
        return on_dev[id(x)]

    for i, e in enumerate(entries):
        kind = e.get("kind", "linear")
        if kind == "linear":
            g = grad_sums[i] if grad_sums else torch.full((e["d_out"], e["d_in"]), float("nan"), device=DEV)
            layers.append(dict(a=to_dev(e["a"]), delta=to_dev(e["delta"]), grad_sum=g))
        elif kind == "vector":
            g = grad_sums[i] if grad_sums else torch.full((e["d"],), float("nan"), device=DEV)
            layers.append(dict(kind="vector", x=None if e["x"] is None else to_dev(e["x"]),
                               delta=to_dev(e["delta"]), grad_sum=g))
        else:
            g = table_grads[i] if table_grads else None
            layers.append(dict(kind="embed", ids=torch.from_numpy(e["ids"]).to(DEV), vocab=e["vocab"],
                               delta=to_dev(e["delta"]), grad_sum=g))
    ps = torch.full((B,), float("nan"), dtype=torch.float32, device=DEV)
    pl = torch.full((len(layers), B), float("nan"), dtype=torch.float32, device=DEV)
    acc = new_acc() if acc is None else acc
    A.adloco_grad_stats(ctx, layers, B, T, code_of(dtype), ps, pl,
                        acc, flags)
    torch.cuda.synchronize()
    S1, n = read_acc(acc)
    return dict(per_sample=ps.cpu().numpy(), per_layer=pl.cpu().numpy(), S1=S1, n_samples=n, acc=acc,
                layers=layers)


def _check(ctx, entries, B, T, dtype):
    from gpu_util import rel_err
    got = _run(ctx, entries, B, T, dtype)
    want = orc.grad_stats([_oracle_entry(e) for e in entries], two_pass=False)
    tol = TOL[dtype]
    assert got["n_samples"] == B
    assert rel_err(got["per_layer"], want["n_layer_sample"]) < tol
    assert rel_err(got["per_sample"], want["n_sample"]) < tol
    assert rel_err(got["S1"], want["S1"]) < tol
    for l, e in enumerate(entries):
        if e.get("kind", "linear") == "embed":
            continue
        g = got["layers"][l]["grad_sum"].cpu().numpy().astype(np.float64)
        w = want["G"][l]
        scale = float(np.sqrt(np.mean(w * w))) + 1e-300
        assert float(np.max(np.abs(g - w))) / scale < 1e-4, l
    return got, want


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("B,T,vectors,tables", [
    (3, 37, [(40, True), (40, False), (7, True), (1, False)], [(11, 24), (50, 5)]),   # odd widths
    (2, 1, [(8, True)], [(4, 8)]),                                                     # one token
    (5, 130, [(768, True), (768, False), (2304, False)], [(1000, 768), (130, 768)]),   # slabs, ragged T
    (1, 64, [(256, False), (520, True)], [(3, 264)]),                                  # B = 1, few ids
])
def test_vector_table_blocks(ctx, dtype, B, T, vectors, tables):
    entries = synth.vector_table_inputs(3000 + B + T, B, T, dtype, vectors, tables, std_delta=0.3, rho=0.4)
    _check(ctx, entries, B, T, dtype)


def test_mixed_with_linear_layers_and_norm_test(ctx):
    # a transformer block's worth: linear weights with their biases, two norm layers, token and
    # position embeddings; then the norm test over all of them
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    B, T, d, V = 6, 192, 128, 300
    lin = synth.custom_grad_stats_inputs(3100, [(d, 3 * d), (d, d), (d, 4 * d), (4 * d, d)], B, T, "bf16",
                                         std_delta=0.05, rho=0.5)
    aux = synth.vector_table_inputs(3200, B, T, "bf16", [(d, True), (d, False), (d, True), (d, False)],
                                    [(V, d)], std_delta=0.05, rho=0.5)
    # biases reuse the deltas of their linear layers; position embedding: ids = 0..T-1
    entries = list(lin)
    for l in lin:
        entries.append(dict(kind="vector", d=l["d_out"], x=None, delta=l["delta"]))
    entries += aux
    pos = dict(kind="embed", d=d, vocab=T, ids=np.tile(np.arange(T, dtype=np.int32), (B, 1)),
               delta=aux[-1]["delta"])
    entries.append(pos)
    want = orc.grad_stats([_oracle_entry(e) for e in entries], two_pass=True)
    # the caller maintains the table gradients: scatter the oracle's rows into [V, d]
    table_grads = {}
    for l, e in enumerate(entries):
        if e.get("kind") == "embed":
            g = np.zeros((e["vocab"], e["d"]), dtype=np.float32)
            g[want["embed_rows"][l]] = want["G"][l].astype(np.float32)
            table_grads[l] = torch.from_numpy(g).to(DEV)
    got = _run(ctx, entries, B, T, "bf16", table_grads=table_grads)
    from gpu_util import rel_err
    assert rel_err(got["per_layer"], want["n_layer_sample"]) < 2e-3
    assert rel_err(got["S1"], want["S1"]) < 2e-3
    # position embedding: all ids distinct -> sum_t ||delta_t||^2 ; the identity V = S1 - S2/B
    res = A.adloco_norm_test(ctx, got["layers"], got["acc"], 0.3, B, 32)
    assert res["S2"] == pytest.approx(want["S2"], rel=2e-3)
    assert res["variance"] == pytest.approx(want["V"] / (B - 1), rel=2e-3)
    ref = orc.norm_test(want["S1"], want["S2"], B, 0.3, B, 32)
    assert res["stat"] == pytest.approx(ref["stat"], rel=3e-3)


def test_vector_accumulation_over_micro_batches(ctx):
    # switch mode: two micro-batches accumulate S1, n and the vectors' gradient sums
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc, rel_err
    B, T = 4, 50
    mbs = [synth.vector_table_inputs(3300 + 100 * k, B, T, "bf16", [(96, True), (96, False)], [(40, 96)],
                                     std_delta=0.2, rho=0.3) for k in range(2)]
    gs = [torch.zeros(96, device=DEV), torch.zeros(96, device=DEV), None]
    acc = new_acc()
    _run(ctx, mbs[0], B, T, "bf16", acc=acc, grad_sums=gs)
    got = _run(ctx, mbs[1], B, T, "bf16", flags=A.ADLOCO_ACCUMULATE, acc=acc, grad_sums=gs)
    want = orc.grad_stats(orc.concat_micro_batches([[_oracle_entry(e) for e in mb] for mb in mbs]),
                          two_pass=False)
    assert got["n_samples"] == 2 * B
    assert rel_err(got["S1"], want["S1"]) < 2e-3
    for l in range(2):
        w = want["G"][l]
        g = gs[l].cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - w))) / (float(np.sqrt(np.mean(w * w))) + 1e-300) < 1e-4


def _with_biases(lin, extra=()):
    """linear entries followed by one bias per linear layer on the same delta array."""
    return list(lin) + [dict(kind="vector", d=l["d_out"], x=None, delta=l["delta"]) for l in lin] + list(extra)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("B,T,shapes", [
    (5, 64, [(72, 264), (128, 256), (320, 520), (8, 8)]),     # ragged tile rows, several tile columns
    (40, 32, [(128, 256)]),                                   # one tile split along the samples
    (3, 96, [(264, 72), (16, 392)]),
])
def test_biases_on_their_linear_layers_delta(ctx, dtype, B, T, shapes):
    # every linear layer with a bias on the same delta tensor (one pointer, as a framework passes it)
    lin = synth.custom_grad_stats_inputs(3500 + B + T, shapes, B, T, dtype, std_delta=0.2, rho=0.4)
    own = synth.vector_table_inputs(3550 + B, B, T, dtype, [(shapes[0][1], False), (64, True)], [],
                                    std_delta=0.2, rho=0.4)    # a bias with a delta of its own, a gain
    _check(ctx, _with_biases(lin, own), B, T, dtype)


def test_biases_with_whole_and_split_tile_entries_accumulate(ctx):
    # 288 tiles: whole entries and entries split along the samples; two micro-batches accumulate
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc, rel_err
    B, T = 3, 32
    shapes = [(2048, 2048), (2048, 2048), (2048, 264)]
    mbs = [_with_biases(synth.custom_grad_stats_inputs(3600 + 50 * k, shapes, B, T, "bf16", std_delta=0.05,
                                                       rho=0.3)) for k in range(2)]
    gs = [torch.zeros(do, di, device=DEV) for di, do in shapes] + [torch.zeros(do, device=DEV) for _, do in shapes]
    acc = new_acc()
    first = _run(ctx, mbs[0], B, T, "bf16", acc=acc, grad_sums=gs)
    got = _run(ctx, mbs[1], B, T, "bf16", flags=A.ADLOCO_ACCUMULATE, acc=acc, grad_sums=gs)
    want = orc.grad_stats(orc.concat_micro_batches([[_oracle_entry(e) for e in mb] for mb in mbs]),
                          two_pass=False)
    assert got["n_samples"] == 2 * B
    per_layer = np.concatenate([first["per_layer"], got["per_layer"]], axis=1)
    assert rel_err(per_layer, want["n_layer_sample"]) < 2e-3
    assert rel_err(got["S1"], want["S1"]) < 2e-3
    for l, w in enumerate(want["G"]):
        g = gs[l].cpu().numpy().astype(np.float64)
        assert float(np.max(np.abs(g - w))) / (float(np.sqrt(np.mean(w * w))) + 1e-300) < 1e-4, l


def test_strided_bias_of_fused_projection(ctx):
    # the bias of one third of a fused qkv projection: delta is a column slice of a wider buffer
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import to_dev, new_acc, read_acc, rel_err, DEV
    B, T = 3, 70
    wide = synth.vector_table_inputs(3400, B, T, "bf16", [(384, False)], [], std_delta=0.3)[0]
    d_w = to_dev(wide["delta"])
    cuts = [(0, 128), (128, 384), (72, 200)]
    layers = [dict(kind="vector", x=None, delta=d_w[:, :, c0:c1], grad_sum=torch.zeros(c1 - c0, device=DEV))
              for c0, c1 in cuts]
    ps = torch.zeros(B, device=DEV)
    pl = torch.zeros(len(cuts), B, device=DEV)
    acc = new_acc()
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, pl, acc)
    torch.cuda.synchronize()
    want = orc.grad_stats([("rowsum", None, wide["delta"][:, :, c0:c1]) for c0, c1 in cuts], two_pass=False)
    assert rel_err(pl.cpu().numpy(), want["n_layer_sample"]) < 2e-3


def test_vector_table_errors(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc
    B, T, d = 2, 8, 16
    delta = torch.zeros(B, T, d, dtype=torch.bfloat16, device=DEV)
    ps = torch.zeros(B, device=DEV)
    descs = A.make_layer_descs([dict(kind="vector", x=None, delta=delta, grad_sum=torch.zeros(d, device=DEV))],
                               B, T, A.ADLOCO_BF16)
    descs[0].d_in = 3                                   # a vector block must have d_in = 1
    with pytest.raises(A.AdlocoError):
        A.adloco_grad_stats(ctx, None, B, T, A.ADLOCO_BF16, ps, None, new_acc(), descs=descs)
    ids = torch.zeros(B, T, dtype=torch.int32, device=DEV)
    descs = A.make_layer_descs([dict(kind="embed", ids=ids, vocab=5, delta=delta)], B, T, A.ADLOCO_BF16)
    descs[0].flags = A.ADLOCO_KIND_EMBED                # table gradient not provided
    with pytest.raises(A.AdlocoError):
        A.adloco_grad_stats(ctx, None, B, T, A.ADLOCO_BF16, ps, None, new_acc(), descs=descs)
    descs = A.make_layer_descs([dict(kind="vector", x=None, delta=delta, grad_sum=torch.zeros(d, device=DEV))],
                               B, T, A.ADLOCO_BF16)
    descs[0].flags = 0x30                               # unknown kind
    with pytest.raises(A.AdlocoError):
        A.adloco_grad_stats(ctx, None, B, T, A.ADLOCO_BF16, ps, None, new_acc(), descs=descs)


def test_fullsize_gpt2_vector_table_blocks(ctx):
    # the launch of bench.py's extra leg: 100 blocks (48 biases, 25 norm gains + biases, token
    # and position embeddings), B = 32, T = 512, drawn on the device; sampled blocks are copied
    # back and checked in full against the oracle
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, rel_err
    B, T, d, V = 32, 512, 768, 50257

    def bits(t):
        return t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)

    blocks = []
    for j, do in enumerate([2304, 768, 3072, 768] * 12):
        dl = synth.device_normal(8000 + j, (B, T, do), 1e-2, torch.bfloat16, DEV)
        blocks.append(dict(kind="vector", x=None, delta=dl, grad_sum=torch.zeros(do, device=DEV)))
    for j in range(25):
        x = synth.device_normal(8100 + 2 * j, (B, T, d), 1.0, torch.bfloat16, DEV)
        dl = synth.device_normal(8101 + 2 * j, (B, T, d), 1e-2, torch.bfloat16, DEV)
        blocks.append(dict(kind="vector", x=x, delta=dl, grad_sum=torch.zeros(d, device=DEV)))
        blocks.append(dict(kind="vector", x=None, delta=dl, grad_sum=torch.zeros(d, device=DEV)))
    ids = torch.from_numpy(synth.token_ids(8200, B, T, V)).to(DEV)
    pos = torch.arange(T, dtype=torch.int32, device=DEV).repeat(B, 1).contiguous()
    de = synth.device_normal(8201, (B, T, d), 1e-2, torch.bfloat16, DEV)
    blocks.append(dict(kind="embed", ids=ids, vocab=V, delta=de, grad_sum=None))
    blocks.append(dict(kind="embed", ids=pos, vocab=T, delta=de, grad_sum=None))
    assert len(blocks) == 100
    ps = torch.zeros(B, device=DEV)
    pl = torch.zeros(len(blocks), B, device=DEV)
    acc = torch.zeros(2, dtype=torch.float64, device=DEV)
    A.adloco_grad_stats(ctx, blocks, B, T, A.ADLOCO_BF16, ps, pl, acc)
    torch.cuda.synchronize()
    pl_h = pl.cpu().numpy()
    for l in (0, 2, 47, 48, 49, 96, 97, 98, 99):
        b = blocks[l]
        if b["kind"] == "vector":
            entry = ("rowsum", None if b["x"] is None else bits(b["x"]), bits(b["delta"]))
        else:
            entry = ("embed", b["ids"].cpu().numpy(), bits(b["delta"]))
        want = orc.grad_stats([entry], two_pass=False)
        assert rel_err(pl_h[l], want["n_layer_sample"][0]) < 2e-3, l
        if b["kind"] == "vector":
            w = want["G"][0]
            g = b["grad_sum"].cpu().numpy().astype(np.float64)
            assert float(np.max(np.abs(g - w))) / (float(np.sqrt(np.mean(w * w))) + 1e-300) < 1e-4, l
    # size-free properties: totals add up; the position table (all ids distinct) gives the sum
    # of squared entries of delta; repeated ids make the token table differ from it
    np.testing.assert_allclose(ps.cpu().numpy(), pl_h.sum(axis=0), rtol=1e-5)
    S1 = float(acc.cpu()[0])
    assert S1 == pytest.approx(float(pl_h.astype(np.float64).sum()), rel=1e-5)
    sq = (de.float() ** 2).sum(dim=(1, 2)).cpu().numpy()
    np.testing.assert_allclose(pl_h[99], sq, rtol=2e-3)
    assert np.all(np.abs(pl_h[98] - sq) > 1e-6 * sq)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("order", ["gain_first", "bias_first", "two_layers"])
def test_gain_and_bias_of_one_normalisation_layer_share_their_delta(ctx, dtype, order):
    # the gain (x = normalised input) and the bias (x = 1) of a normalisation layer are given the
    # same delta tensor: the library forms both in one pass over it, in either order of the list, and
    # keeps them apart from a second layer's pair and from a bias that has no partner
    B, T, d = 3, 37, 300
    aux = synth.vector_table_inputs(6100, B, T, dtype, [(d, True), (d, True), (d, False)], [], std_delta=0.1, rho=0.3)
    g1, g2, lone = aux
    b1 = dict(kind="vector", d=d, x=None, delta=g1["delta"])
    b2 = dict(kind="vector", d=d, x=None, delta=g2["delta"])
    entries = {"gain_first": [g1, b1, lone], "bias_first": [b1, lone, g1],
               "two_layers": [g1, b1, b2, g2, lone]}[order]
    _check(ctx, entries, B, T, dtype)       # norms and the gradient sums of every block
