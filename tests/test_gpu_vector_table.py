"""GPU parity of the vector (bias / gain) and embedding-table blocks of the per-sample gradient:
the HIP path through the C ABI against the CPU oracle on the same seeded inputs.  Tolerances as
for the linear weights: 1e-4 relative for fp32 inputs, 2e-3 for bf16 inputs."""
import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-3}


@pytest.fixture(scope="module")
def ctx():
    import paper_2508_18182_amd as A
    c = A.Context(0)
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
    from gpu_util import to_dev, new_acc, read_acc, DEV
    layers = []
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
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16 if dtype == "bf16" else A.ADLOCO_F32, ps, pl,
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


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
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
