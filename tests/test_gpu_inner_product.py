"""GPU parity of the inner products c_i = <g_i, G> and of the inner-product and augmented
inner-product tests (Section 3.3.2): the HIP path through the C ABI against the CPU oracle on
the same seeded inputs.

Tolerance: c_i is a sum of products of per-sample gradient entries and entries of G, both held
in fp32 on the GPU, so its error is measured against sqrt(||g_i||^2 ||G||^2) (Cauchy-Schwarz
bound of |c_i|): 1e-4 of it for fp32 inputs, 2e-3 for bf16 inputs, the bars of the norms.  The
decisions are compared unless a statistic lies within 1e-3 (relative) of an integer cut."""
import math

import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-3, "f16": 2e-3}


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


def _device_layers(entries, want_G=None, embed_rows=None):
    """Device descriptors; embedding tables get the caller-kept [V, d] gradient scattered from the
    oracle's rows (the library reads it, it never writes a table gradient)."""
    import torch
    from gpu_util import to_dev, DEV
    layers = []
    for l, e in enumerate(entries):
        kind = e.get("kind", "linear")
        if kind == "linear":
            layers.append(dict(a=to_dev(e["a"]), delta=to_dev(e["delta"]),
                               grad_sum=torch.zeros(e["d_out"], e["d_in"], device=DEV)))
        elif kind == "vector":
            layers.append(dict(kind="vector", x=None if e["x"] is None else to_dev(e["x"]),
                               delta=to_dev(e["delta"]), grad_sum=torch.zeros(e["d"], device=DEV)))
        else:
            g = np.zeros((e["vocab"], e["d"]), dtype=np.float32)
            g[embed_rows[l]] = want_G[l].astype(np.float32)
            layers.append(dict(kind="embed", ids=torch.from_numpy(e["ids"]).to(DEV), vocab=e["vocab"],
                               delta=to_dev(e["delta"]), grad_sum=torch.from_numpy(g).to(DEV)))
    return layers


def _new_ip_acc():
    import torch
    return torch.full((4,), float("nan"), dtype=torch.float64, device="cuda:0")


def _read_ip_acc(t):
    import torch
    h = t.cpu()
    return float(h[0]), float(h[1]), int(h.view(torch.int64)[2])


def _close(got, want, n_sample, S2, tol):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    scale = np.sqrt(np.asarray(n_sample, np.float64) * S2) + 1e-300
    return float(np.max(np.abs(got - want) / scale)) < tol


def _compare_decisions(got, want):
    for tag in ("ip", "aug"):
        s = want["stat_" + tag]
        if math.isinf(s) or abs(s - round(s)) <= 1e-3 * max(abs(s), 1.0):
            continue
        if tag == "aug":
            s_ip = want["stat_ip"]
            if abs(s_ip - round(s_ip)) <= 1e-3 * max(abs(s_ip), 1.0):
                continue
        assert got["b_req_" + tag] == want["b_req_" + tag], (tag, got, want)
        sw = want["switch_" + tag]
        assert (got["accumulate_" + tag], got["accum_steps_" + tag], got["b_micro_" + tag]) == \
            (sw["accumulate"], sw["accum_steps"], sw["b_micro"])


def _run_case(ctx, micro_batches, B, T, dtype, vartheta=0.01, nu=0.3, b_cur=None, b_max=32):
    """micro_batches: list of entry lists (same blocks).  Statistics and G accumulate over all of
    them first; then the inner products of every micro-batch against the complete G."""
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import new_acc, read_acc, DEV
    from gpu_util import code_of
    code = code_of(dtype)
    tol = TOL[dtype]
    oracle_mbs = [[_oracle_entry(e) for e in mb] for mb in micro_batches]
    whole = orc.concat_micro_batches(oracle_mbs) if len(oracle_mbs) > 1 else oracle_mbs[0]
    want = orc.grad_stats(whole, two_pass=True)
    dev_mbs = [_device_layers(mb, want["G"], want.get("embed_rows")) for mb in micro_batches]
    for layers in dev_mbs[1:]:                     # one gradient buffer per block, shared
        for l, d in enumerate(layers):
            d["grad_sum"] = dev_mbs[0][l]["grad_sum"]
    acc = new_acc()
    ps = [torch.zeros(B, device=DEV) for _ in dev_mbs]
    for k, layers in enumerate(dev_mbs):
        A.adloco_grad_stats(ctx, layers, B, T, code, ps[k], None, acc, A.ADLOCO_ACCUMULATE if k else 0)
    ip_acc = _new_ip_acc()
    c_got, sq_got = [], []
    for k, layers in enumerate(dev_mbs):
        c = torch.full((B,), float("nan"), device=DEV)
        sq = torch.full((B,), float("nan"), device=DEV)
        A.adloco_inner_products(ctx, layers, B, T, code, c, sq, ip_acc, A.ADLOCO_ACCUMULATE if k else 0)
        c_got.append(c)
        sq_got.append(sq)
    torch.cuda.synchronize()
    n_total = B * len(dev_mbs)
    c_got = np.concatenate([c.cpu().numpy() for c in c_got]).astype(np.float64)
    sq_got = np.concatenate([s.cpu().numpy() for s in sq_got]).astype(np.float64)
    c_want = np.concatenate([orc.inner_products(mb, G=want["G"], embed_rows=want.get("embed_rows"))
                             for mb in oracle_mbs])
    assert _close(c_got, c_want, want["n_sample"], want["S2"], tol)
    # the explicit per-sample norms are a second route to the Gram result
    assert np.max(np.abs(sq_got - want["n_sample"]) / want["n_sample"]) < tol
    s_ip, s_ip2, n = _read_ip_acc(ip_acc)
    assert n == n_total
    assert s_ip == pytest.approx(float(c_got.sum()), rel=1e-6)
    assert s_ip2 == pytest.approx(float((c_got * c_got).sum()), rel=1e-6)
    assert s_ip == pytest.approx(want["S2"], rel=10 * tol)         # sum_i <g_i, G> = ||G||^2
    b_cur = n_total if b_cur is None else b_cur
    res = A.adloco_inner_product_test(ctx, dev_mbs[0], acc, ip_acc, vartheta, nu, b_cur, b_max)
    ref = orc.inner_product_test(want["n_sample"], c_want, want["S2"], vartheta, nu, b_cur, b_max)
    assert res["n_samples"] == n_total and res["stat_undefined"] == ref["stat_undefined"]
    if n_total >= 2:
        # variances are differences of close numbers: their error scales with the terms
        terms_ip = float(np.sum((c_want / n_total) ** 2)) / (n_total - 1)
        assert abs(res["var_ip"] - ref["var_ip"]) <= 4 * tol * terms_ip
        assert abs(res["var_aug"] - ref["var_aug"]) <= 4 * tol * want["S1"] / (n_total - 1)
        if abs(res["var_ip"] - ref["var_ip"]) <= 1e-3 * ref["var_ip"] and \
                abs(res["var_aug"] - ref["var_aug"]) <= 1e-3 * ref["var_aug"]:
            _compare_decisions(res, ref)
    return res, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("B,T,shapes", [
    (3, 5, [(3, 2), (1, 4)]),                          # tiny
    (4, 37, [(40, 24), (17, 33), (8, 8)]),             # odd widths, ragged T: plain path
    (2, 1, [(16, 8)]),                                 # one token
    (1, 32, [(64, 64)]),                               # B = 1: both tests undefined
])
def test_inner_products_small_linear(ctx, dtype, B, T, shapes):
    entries = synth.custom_grad_stats_inputs(5000 + B + T, shapes, B, T, dtype, std_delta=0.3, rho=0.5)
    _run_case(ctx, [entries], B, T, dtype)


@pytest.mark.parametrize("B,T,shapes", [
    (5, 64, [(256, 512), (64, 128), (768, 256)]),      # whole tiles and a small one
    (3, 32, [(320, 136), (8, 264)]),                   # one chunk; ragged tile edges
    (4, 96, [(512, 256), (256, 776)]),                 # three chunks (pipeline tail)
    (2, 256, [(768, 768)]),                            # deeper pipeline
])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_inner_products_tile_path_16bit(ctx, dtype, B, T, shapes):
    entries = synth.custom_grad_stats_inputs(5100 + B + T, shapes, B, T, dtype, std_delta=0.1, rho=0.5)
    _run_case(ctx, [entries], B, T, dtype)


def test_inner_products_mixed_paths_and_kinds(ctx):
    # tile path (aligned), plain path (odd width), bias / gain vectors and two tables in one call
    B, T, d = 6, 64, 128
    lin = synth.custom_grad_stats_inputs(5200, [(d, 3 * d), (d, d), (d + 4, 52)], B, T, "bf16",
                                         std_delta=0.05, rho=0.5)
    aux = synth.vector_table_inputs(5201, B, T, "bf16", [(d, True), (d, False), (3 * d, False)],
                                    [(300, d), (20, 40)], std_delta=0.05, rho=0.5)
    _run_case(ctx, [list(lin) + list(aux)], B, T, "bf16")


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_inner_products_over_micro_batches(ctx, dtype):
    # switch mode: G and S1 accumulate over three micro-batches, then the inner products of each
    B, T = 4, 64
    shapes = [(128, 256), (72, 40)]
    mbs = []
    for k in range(3):
        lin = synth.custom_grad_stats_inputs(5300 + 10 * k, shapes, B, T, dtype, std_delta=0.1, rho=0.4)
        aux = synth.vector_table_inputs(5305 + 10 * k, B, T, dtype, [(256, True), (40, False)], [(50, 72)],
                                        std_delta=0.1, rho=0.4)
        mbs.append(list(lin) + list(aux))
    res, ref = _run_case(ctx, mbs, B, T, dtype, vartheta=0.05, nu=0.3, b_cur=4, b_max=8)
    assert res["n_samples"] == 12


def test_inner_products_strong_common_direction_and_pure_noise(ctx):
    # nearly identical per-sample gradients: tiny variances; independent ones: large requests
    B, T = 8, 64
    for seed, rho in ((5400, 0.95), (5401, 0.0)):
        entries = synth.custom_grad_stats_inputs(seed, [(256, 256)], B, T, "bf16", std_delta=0.1, rho=rho)
        _run_case(ctx, [entries], B, T, "bf16", vartheta=0.2, nu=1.0, b_cur=1, b_max=16)


def test_inner_products_errors(ctx):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV, new_acc
    B, T, d = 2, 32, 16
    a = torch.zeros(B, T, d, dtype=torch.bfloat16, device=DEV)
    layers = [dict(a=a, delta=a, grad_sum=torch.zeros(d, d, device=DEV))]
    c = torch.zeros(B, device=DEV)
    ip_acc = _new_ip_acc()
    descs = A.make_layer_descs(layers, B, T, A.ADLOCO_BF16)
    descs[0].grad_sum = None                            # G is read here: it has to be there
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_products(ctx, None, B, T, A.ADLOCO_BF16, c, None, ip_acc, descs=descs)
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_products(ctx, layers, B, T, A.ADLOCO_BF16, c, None, ip_acc, flags=0x80)
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_products(ctx, None, 0, T, A.ADLOCO_BF16, c, None, ip_acc,
                                descs=A.make_layer_descs(layers, B, T, A.ADLOCO_BF16))
    # sample counts of the two accumulators must agree
    acc = new_acc()
    ps = torch.zeros(B, device=DEV)
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, None, acc)
    A.adloco_inner_products(ctx, layers, B, T, A.ADLOCO_BF16, c, None, ip_acc)
    A.adloco_inner_products(ctx, layers, B, T, A.ADLOCO_BF16, c, None, ip_acc, flags=A.ADLOCO_ACCUMULATE)
    with pytest.raises(A.AdlocoError):
        A.adloco_inner_product_test(ctx, layers, acc, ip_acc, 0.01, 0.3, B, 32)
    # all-zero gradients: zero variances, both requests stay at b_cur
    A.adloco_inner_products(ctx, layers, B, T, A.ADLOCO_BF16, c, None, ip_acc)
    res = A.adloco_inner_product_test(ctx, layers, acc, ip_acc, 0.01, 0.3, 5, 32)
    assert res["b_req_ip"] == 5 and res["b_req_aug"] == 5 and res["var_ip"] == 0.0


def _bits(t):
    import torch
    return t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def test_inner_products_gpt2_small_full_workload(ctx):
    # workload 2 in the launch bench.py times: 48 linears, B = 32, T = 512, bf16, drawn on the
    # device.  Properties over all blocks; sampled c_i against the oracle on a four-block call.
    import torch
    import paper_2508_18182_amd as A
    B, T = 32, 512
    layers = synth.device_grad_stats_inputs(2, "cuda:0")
    dev = layers[0]["a"].device
    for l in layers:
        l["grad_sum"] = torch.zeros(l["d_out"], l["d_in"], device=dev)
    ps = torch.zeros(B, device=dev)
    acc = torch.zeros(2, dtype=torch.float64, device=dev)
    A.adloco_grad_stats(ctx, layers, B, T, A.ADLOCO_BF16, ps, None, acc)
    c = torch.zeros(B, device=dev)
    sq = torch.zeros(B, device=dev)
    ip_acc = _new_ip_acc()
    A.adloco_inner_products(ctx, layers, B, T, A.ADLOCO_BF16, c, sq, ip_acc)
    torch.cuda.synchronize()
    res = A.adloco_inner_product_test(ctx, layers, acc, ip_acc, 0.01, 0.3, B, 32)
    s_ip, s_ip2, n = _read_ip_acc(ip_acc)
    assert n == B
    assert s_ip == pytest.approx(res["S2"], rel=1e-3)               # sum_i <g_i, G> = ||G||^2
    assert torch.max(torch.abs(sq - ps) / ps).item() < TOL["bf16"]  # explicit norms = Gram norms
    cd = c.double()
    # Cauchy-Schwarz, and the sample variance re-derived from the returned c_i
    assert bool(torch.all(cd * cd <= ps.double() * res["S2"] * (1 + 1e-3)))
    ip = (cd / B).cpu().numpy()
    assert res["var_ip"] == pytest.approx(float(np.var(ip, ddof=1)), rel=1e-4)
    # sampled: four blocks of different shapes (one block's four linears), three samples
    sub = [dict(l) for l in layers[4:8]]
    c4 = torch.zeros(B, device=dev)
    A.adloco_inner_products(ctx, sub, B, T, A.ADLOCO_BF16, c4, None, ip_acc)
    torch.cuda.synchronize()
    G = [l["grad_sum"].cpu().numpy().astype(np.float64) for l in sub]
    S2_sub = float(sum(np.sum(g * g) for g in G))
    for i in (0, 13, 31):
        want, n_i = 0.0, 0.0
        for l, g in zip(sub, G):
            gi = orc.per_sample_gradient(_bits(l["a"][i]), _bits(l["delta"][i]))
            want += float(np.sum(gi * g))
            n_i += float(np.sum(gi * gi))
        assert abs(float(c4[i]) - want) <= TOL["bf16"] * math.sqrt(n_i * S2_sub), (i, float(c4[i]), want)
