"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the
oracle's own formulas (hand-worked fixtures, closed forms, brute force, library routines
reached by another route).  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

import adloco_synth as synth
from oracle import adloco_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLD, name)) as f:
        for ln in f:
            ln = ln.rstrip("\n")
            if ln.strip() and not ln.lstrip().startswith("#"):
                yield ln


def _ints(s):
    s = s.strip()
    return [int(v) for v in s.split(",")] if s else []


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ------------------------------------------------------------------ per-sample norms

def test_gram_hand_cases():
    # g = sum_t delta_t a_t^T, norms worked by hand (tests/golden/gram_hand_cases.txt)
    n = 0
    for ln in _lines("gram_hand_cases.txt"):
        lhs, want = ln.split("->")
        dims, a, d = lhs.split(";")
        T, di, do = [int(v) for v in dims.split()]
        a = np.array([float(v) for v in a.split(",")], dtype=np.float32).reshape(1, T, di)
        d = np.array([float(v) for v in d.split(",")], dtype=np.float32).reshape(1, T, do)
        st = orc.grad_stats([(a, d)])
        assert st["n_sample"][0] == pytest.approx(float(want), abs=1e-12)
        n += 1
    assert n >= 6


def test_T1_closed_form():
    # one token: g = delta a^T  =>  ||g||^2 = ||a||^2 ||delta||^2
    r = _rng(1)
    a = r.standard_normal((5, 1, 7)).astype(np.float32)
    d = r.standard_normal((5, 1, 3)).astype(np.float32)
    st = orc.grad_stats([(a, d)])
    want = (a.astype(np.float64) ** 2).sum(axis=(1, 2)) * (d.astype(np.float64) ** 2).sum(axis=(1, 2))
    np.testing.assert_allclose(st["n_sample"], want, rtol=1e-13)


def test_T2_closed_form():
    # two tokens: ||a1||^2||d1||^2 + ||a2||^2||d2||^2 + 2 (a1.a2)(d1.d2)
    r = _rng(2)
    a = r.standard_normal((4, 2, 6))
    d = r.standard_normal((4, 2, 5))
    st = orc.grad_stats([(a, d)])
    for i in range(4):
        a1, a2, d1, d2 = a[i, 0], a[i, 1], d[i, 0], d[i, 1]
        want = (a1 @ a1) * (d1 @ d1) + (a2 @ a2) * (d2 @ d2) + 2 * (a1 @ a2) * (d1 @ d2)
        assert st["n_sample"][i] == pytest.approx(want, rel=1e-12)


def test_orthonormal_tokens():
    # orthonormal activation rows: ||sum_t delta_t a_t^T||^2 = sum_t ||delta_t||^2
    r = _rng(3)
    T, di, do = 6, 9, 4
    q, _ = np.linalg.qr(r.standard_normal((di, di)))
    a = q[:T][None]                       # [1,T,di] orthonormal rows
    d = r.standard_normal((1, T, do))
    st = orc.grad_stats([(a, d)])
    assert st["n_sample"][0] == pytest.approx((d ** 2).sum(), rel=1e-12)


def test_constant_tokens():
    # every token has the same activation: g = (sum_t delta_t) a^T
    r = _rng(4)
    T, di, do = 5, 8, 3
    a0 = r.standard_normal(di)
    a = np.broadcast_to(a0, (1, T, di)).copy()
    d = r.standard_normal((1, T, do))
    st = orc.grad_stats([(a, d)])
    want = (a0 @ a0) * (d[0].sum(axis=0) ** 2).sum()
    assert st["n_sample"][0] == pytest.approx(want, rel=1e-12)


def test_token_permutation_and_rotation_invariance():
    r = _rng(5)
    B, T, di, do = 3, 7, 6, 5
    a = r.standard_normal((B, T, di))
    d = r.standard_normal((B, T, do))
    base = orc.grad_stats([(a, d)])
    perm = r.permutation(T)
    st = orc.grad_stats([(a[:, perm], d[:, perm])])
    np.testing.assert_allclose(st["n_sample"], base["n_sample"], rtol=1e-12)
    assert st["S2"] == pytest.approx(base["S2"], rel=1e-12)
    Q, _ = np.linalg.qr(r.standard_normal((di, di)))
    R, _ = np.linalg.qr(r.standard_normal((do, do)))
    st = orc.grad_stats([(a @ Q, d @ R)])
    np.testing.assert_allclose(st["n_sample"], base["n_sample"], rtol=1e-11)
    assert st["S2"] == pytest.approx(base["S2"], rel=1e-11)
    # permuting tokens of a only (not delta) must change the result: guards a dropped pairing
    st = orc.grad_stats([(a[:, perm], d)])
    assert not np.allclose(st["n_sample"], base["n_sample"], rtol=1e-6)


def test_brute_force_tiny_config():
    # Config 1 element by element with python loops, no matmul: G[e][c] = sum_t delta[t][e]*a[t][c]
    inp = synth.grad_stats_inputs(1)[0]
    a, d = inp["a"], inp["delta"]
    B, T, di = a.shape
    do = d.shape[2]
    st = orc.grad_stats([(a, d)])
    tot = [[0.0] * di for _ in range(do)]
    for i in range(B):
        n = 0.0
        for e in range(do):
            for c in range(di):
                s = 0.0
                for t in range(T):
                    s += float(d[i, t, e]) * float(a[i, t, c])
                n += s * s
                tot[e][c] += s
        assert st["n_sample"][i] == pytest.approx(n, rel=1e-12)
    S2 = sum(v * v for row in tot for v in row)
    assert st["S2"] == pytest.approx(S2, rel=1e-12)
    assert st["batch_grad_sqnorm"] == pytest.approx(S2 / B ** 2, rel=1e-12)
    np.testing.assert_allclose(st["G"][0], np.array(tot), rtol=1e-11, atol=1e-12)


def test_autograd_linear_layer():
    # library route: per-sample weight gradient of a bias-free linear layer y = a W^T with
    # loss sum <delta, y> is delta^T a
    import torch
    r = _rng(6)
    B, T, di, do = 4, 5, 6, 3
    a = r.standard_normal((B, T, di))
    d = r.standard_normal((B, T, do))
    st = orc.grad_stats([(a, d)])
    W = torch.zeros(do, di, dtype=torch.float64, requires_grad=True)
    tot = torch.zeros(do, di, dtype=torch.float64)
    for i in range(B):
        y = torch.from_numpy(a[i]) @ W.T
        (g,) = torch.autograd.grad((torch.from_numpy(d[i]) * y).sum(), W)
        assert st["n_sample"][i] == pytest.approx(float((g ** 2).sum()), rel=1e-12)
        np.testing.assert_allclose(orc.per_sample_gradient(a[i], d[i]), g.numpy(), rtol=1e-12,
                                   atol=1e-14)
        tot += g
    assert st["S2"] == pytest.approx(float((tot ** 2).sum()), rel=1e-12)


def test_vector_table_hand_cases():
    # tests/golden/vector_table_hand_cases.txt: bias, gain and embedding blocks by hand
    n = 0
    for ln in _lines("vector_table_hand_cases.txt"):
        lhs, want = ln.split("->")
        head, x, d = lhs.split(";")
        kind, T, dim = head.split()
        T, dim = int(T), int(dim)
        delta = np.array([float(v) for v in d.split(",")], dtype=np.float32).reshape(1, T, dim)
        if kind == "bias":
            entry = ("rowsum", None, delta)
        elif kind == "gain":
            entry = ("rowsum", np.array([float(v) for v in x.split(",")], dtype=np.float32).reshape(1, T, dim), delta)
        else:
            entry = ("embed", np.array(_ints(x), dtype=np.int32).reshape(1, T), delta)
        st = orc.grad_stats([entry])
        assert st["n_sample"][0] == pytest.approx(float(want), abs=1e-12)
        n += 1
    assert n >= 7


def test_autograd_bias_gain_embedding():
    # library route: per-sample gradients of a linear bias, a LayerNorm gain and bias and an
    # embedding table by torch.autograd, with loss sum <delta, y> per sample
    import torch
    r = _rng(61)
    B, T, di, do, V = 3, 6, 5, 4, 7
    a = r.standard_normal((B, T, di))
    d_lin = r.standard_normal((B, T, do))
    x = r.standard_normal((B, T, do))
    d_ln = r.standard_normal((B, T, do))
    ids = r.integers(0, V, size=(B, T))
    d_emb = r.standard_normal((B, T, do))
    lin = torch.nn.Linear(di, do, bias=True).double()
    ln = torch.nn.LayerNorm(do).double()
    with torch.no_grad():
        ln.weight.copy_(torch.from_numpy(r.standard_normal(do)))
        ln.bias.copy_(torch.from_numpy(r.standard_normal(do)))
    emb = torch.nn.Embedding(V, do).double()
    xhat = torch.nn.functional.layer_norm(torch.from_numpy(x), (do,)).numpy()   # no affine part
    entries = [(a, d_lin), ("rowsum", None, d_lin), ("rowsum", xhat, d_ln), ("rowsum", None, d_ln),
               ("embed", ids, d_emb)]
    st = orc.grad_stats(entries)
    params = [lin.weight, lin.bias, ln.weight, ln.bias, emb.weight]
    tot = [torch.zeros_like(p) for p in params]
    for i in range(B):
        loss = (torch.from_numpy(d_lin[i]) * lin(torch.from_numpy(a[i]))).sum() \
            + (torch.from_numpy(d_ln[i]) * ln(torch.from_numpy(x[i]))).sum() \
            + (torch.from_numpy(d_emb[i]) * emb(torch.from_numpy(ids[i]))).sum()
        grads = torch.autograd.grad(loss, params)
        for l, g in enumerate(grads):
            assert st["n_layer_sample"][l, i] == pytest.approx(float((g ** 2).sum()), rel=1e-12)
            tot[l] += g
    for l in range(4):
        np.testing.assert_allclose(st["G"][l], tot[l].detach().numpy(), rtol=1e-12, atol=1e-13)
    rows = st["embed_rows"][4]
    dense = np.zeros((V, do))
    dense[rows] = st["G"][4]
    np.testing.assert_allclose(dense, tot[4].detach().numpy(), rtol=1e-12, atol=1e-13)
    assert st["S2"] == pytest.approx(sum(float((t ** 2).sum()) for t in tot), rel=1e-12)


def test_vector_table_closed_forms_and_invariance():
    r = _rng(62)
    B, T, d = 4, 9, 6
    delta = r.standard_normal((B, T, d))
    x = r.standard_normal((B, T, d))
    # one-token samples: ||delta * x||^2
    st1 = orc.grad_stats([("rowsum", x[:, :1], delta[:, :1])])
    np.testing.assert_allclose(st1["n_sample"], ((delta[:, 0] * x[:, 0]) ** 2).sum(axis=1), rtol=1e-13)
    # embedding: distinct ids -> sum_t ||delta_t||^2 ; equal ids -> ||sum_t delta_t||^2
    ids_distinct = np.stack([r.permutation(50)[:T] for _ in range(B)])
    st2 = orc.grad_stats([("embed", ids_distinct, delta)])
    np.testing.assert_allclose(st2["n_sample"], (delta ** 2).sum(axis=(1, 2)), rtol=1e-13)
    st3 = orc.grad_stats([("embed", np.full((B, T), 3), delta)])
    np.testing.assert_allclose(st3["n_sample"], (delta.sum(axis=1) ** 2).sum(axis=1), rtol=1e-13)
    # an embedding whose ids are all equal is a bias: same norms, same gradient sum
    stb = orc.grad_stats([("rowsum", None, delta)])
    np.testing.assert_allclose(st3["n_sample"], stb["n_sample"], rtol=1e-13)
    np.testing.assert_allclose(st3["G"][0][0], stb["G"][0], rtol=1e-13)
    # token order inside a sample does not matter
    ids = r.integers(0, 5, size=(B, T))
    perm = r.permutation(T)
    base = orc.grad_stats([("rowsum", x, delta), ("embed", ids, delta)])
    shuf = orc.grad_stats([("rowsum", x[:, perm], delta[:, perm]), ("embed", ids[:, perm], delta[:, perm])])
    np.testing.assert_allclose(base["n_layer_sample"], shuf["n_layer_sample"], rtol=1e-12)
    # two-pass variance identity over a mixed list of blocks
    mixed = orc.grad_stats([(x, delta), ("rowsum", x, delta), ("rowsum", None, delta), ("embed", ids, delta)])
    assert mixed["V"] == pytest.approx(mixed["S1"] - mixed["S2"] / B, rel=1e-11)


def test_transposed_operand_detected():
    # d_in != d_out: the gradient is [d_out, d_in]; its sum over samples must match einsum
    r = _rng(7)
    a = r.standard_normal((3, 4, 5))
    d = r.standard_normal((3, 4, 2))
    st = orc.grad_stats([(a, d)])
    G = np.einsum("ite,itc->ec", d, a)
    assert st["G"][0].shape == (2, 5)
    np.testing.assert_allclose(st["G"][0], G, rtol=1e-12, atol=1e-14)


def test_layers_concatenate():
    # g_i is the concatenation over layers: norms add across layers
    r = _rng(8)
    l1 = (r.standard_normal((3, 4, 5)), r.standard_normal((3, 4, 2)))
    l2 = (r.standard_normal((3, 4, 3)), r.standard_normal((3, 4, 6)))
    s1, s2, s12 = orc.grad_stats([l1]), orc.grad_stats([l2]), orc.grad_stats([l1, l2])
    np.testing.assert_allclose(s12["n_sample"], s1["n_sample"] + s2["n_sample"], rtol=1e-13)
    assert s12["S2"] == pytest.approx(s1["S2"] + s2["S2"], rel=1e-13)
    assert s12["V"] == pytest.approx(s1["V"] + s2["V"], rel=1e-12)
    np.testing.assert_allclose(s12["n_layer_sample"][1], s2["n_sample"], rtol=1e-13)


def test_bf16_widening_is_exact():
    x = synth.normal_f32(11, (1000,), 1.0)
    bits = synth.f32_to_bf16_bits(x)
    import torch
    t = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(bits, t.view(torch.int16).numpy().view(np.uint16))
    np.testing.assert_array_equal(orc.widen(bits), t.to(torch.float64).numpy())


def test_fp16_widening_is_exact():
    # fp16 storage (the mixed-precision setting of Section 6): values decoded from their bit fields
    # (sign, 5-bit exponent with bias 15, 10-bit fraction; subnormals scale by 2^-24)
    x = synth.to_dtype(synth.normal_f32(12, (2000,), 1e-2), "f16")
    x[:4] = np.array([6e-8, -3e-5, 65504.0, -0.0], dtype=np.float16)
    u = x.view(np.uint16).astype(np.int64)
    sign = np.where(u >> 15, -1.0, 1.0)
    e, f = (u >> 10) & 31, u & 1023
    want = sign * np.where(e == 0, f * 2.0 ** -24, (1024 + f) * 2.0 ** (e - 25.0))
    np.testing.assert_array_equal(orc.widen(x), want)
    import torch
    np.testing.assert_array_equal(synth.to_dtype(synth.normal_f32(13, (500,), 1.0), "f16"),
                                  torch.from_numpy(synth.normal_f32(13, (500,), 1.0)).to(torch.float16).numpy())


# ------------------------------------------------------------------ S2, variance, identity

def test_identical_samples():
    r = _rng(9)
    a1 = r.standard_normal((1, 4, 5))
    d1 = r.standard_normal((1, 4, 3))
    B = 6
    a, d = np.repeat(a1, B, axis=0), np.repeat(d1, B, axis=0)
    st = orc.grad_stats([(a, d)])
    n1 = orc.grad_stats([(a1, d1)])["n_sample"][0]
    assert st["S2"] == pytest.approx(B * B * n1, rel=1e-12)
    assert st["V"] == pytest.approx(0.0, abs=1e-20 * n1 + 1e-22)
    res = orc.norm_test(st["S1"], st["S2"], B, 0.3, b_cur=B, b_max=32, V=st["V"])
    assert res["stat"] == pytest.approx(0.0, abs=1e-12) and res["b_req"] == B


def test_sample_permutation_invariance():
    r = _rng(10)
    a = r.standard_normal((5, 3, 4))
    d = r.standard_normal((5, 3, 2))
    p = r.permutation(5)
    s0, s1 = orc.grad_stats([(a, d)]), orc.grad_stats([(a[p], d[p])])
    assert s1["S1"] == pytest.approx(s0["S1"], rel=1e-13)
    assert s1["S2"] == pytest.approx(s0["S2"], rel=1e-12)
    assert s1["V"] == pytest.approx(s0["V"], rel=1e-12)
    np.testing.assert_allclose(s1["n_sample"], s0["n_sample"][p], rtol=1e-13)


@pytest.mark.parametrize("seed,rho", [(20, 0.0), (21, 0.6), (22, 0.95)])
def test_variance_identity_and_numpy_var(seed, rho):
    # sum ||g_i - gbar||^2 = sum ||g_i||^2 - B ||gbar||^2, and the two-pass value equals numpy's
    # var(ddof=1) summed over coordinates of the stacked per-sample gradients
    layers = synth.custom_grad_stats_inputs(seed, [(6, 4), (5, 7)], B=7, T=5, dtype="f32",
                                            std_a=1.0, std_delta=1.0, rho=rho)
    lay = [(l["a"], l["delta"]) for l in layers]
    st = orc.grad_stats(lay)
    B = 7
    assert st["V"] == pytest.approx(st["S1"] - st["S2"] / B, rel=1e-10)
    assert st["V"] == pytest.approx(st["S1"] - B * st["batch_grad_sqnorm"], rel=1e-10)
    flat = np.stack([np.concatenate([orc.per_sample_gradient(a[i], d[i]).ravel() for a, d in lay])
                     for i in range(B)])
    assert orc.variance(st["V"], B) == pytest.approx(flat.var(axis=0, ddof=1).sum(), rel=1e-11)
    assert orc.variance(st["V"], B, biased=True) == pytest.approx(flat.var(axis=0).sum(), rel=1e-11)
    assert st["batch_grad_sqnorm"] == pytest.approx((flat.mean(axis=0) ** 2).sum(), rel=1e-11)


def test_iid_noise_expectation():
    # iid zero-mean inputs: E||g_i||^2 = T d_in d_out s_a^2 s_d^2 and stat -> B/eta^2
    B, T, di, do = 16, 12, 48, 40
    layers = synth.custom_grad_stats_inputs(30, [(di, do)], B=B, T=T, dtype="f32",
                                            std_a=1.0, std_delta=0.5)
    st = orc.grad_stats([(layers[0]["a"], layers[0]["delta"])])
    assert st["S1"] / B == pytest.approx(T * di * do * 0.25, rel=0.1)
    res = orc.norm_test(st["S1"], st["S2"], B, 0.5, b_cur=B, b_max=8, V=st["V"])
    assert res["stat"] == pytest.approx(B / 0.25, rel=0.25)
    assert res["test_passed"] == 0 and res["accumulate"] == 1


def test_micro_batch_concatenation():
    layers = synth.custom_grad_stats_inputs(40, [(6, 4)], B=6, T=3, dtype="f32", std_delta=1.0,
                                            rho=0.5)
    a, d = layers[0]["a"], layers[0]["delta"]
    whole = orc.grad_stats([(a, d)])
    cat = orc.concat_micro_batches([[(a[:2], d[:2])], [(a[2:4], d[2:4])], [(a[4:], d[4:])]])
    st = orc.grad_stats(cat)
    assert st["S1"] == whole["S1"] and st["S2"] == whole["S2"] and st["B"] == 6


# ------------------------------------------------------------------ decisions

def test_norm_test_hand_cases():
    n = 0
    for ln in _lines("norm_test_hand_cases.txt"):
        lhs, rhs = ln.split("->")
        S1, S2, B, eta, b_cur, biased, shrink, cap = lhs.split()
        var, stat, b_req, passed = rhs.split()
        res = orc.norm_test(float(S1), float(S2), int(B), float(eta), int(b_cur), b_max=1 << 40,
                            b_cap=int(cap), biased_var=bool(int(biased)),
                            allow_shrink=bool(int(shrink)))
        assert res["variance"] == pytest.approx(float(var), rel=1e-12)
        if math.isinf(float(stat)):
            assert math.isinf(res["stat"])
        else:
            assert res["stat"] == pytest.approx(float(stat), rel=1e-12)
        assert res["b_req"] == int(b_req), ln
        assert res["test_passed"] == int(passed), ln
        n += 1
    assert n >= 10


def test_norm_test_explicit_vectors():
    # the hand case again, but through explicit gradients realised as a T=1 linear layer
    # with d_in = 1: g_i = delta_i * a_i with a_i = 1  ->  g_i = delta_i in R^2
    g = np.array([[1, 0], [0, 1], [1, 1], [2, 2]], dtype=np.float64)
    a = np.ones((4, 1, 1))
    d = g.reshape(4, 1, 2)
    st = orc.grad_stats([(a, d)])
    assert (st["S1"], st["S2"], st["V"]) == (12.0, 32.0, 4.0)
    res = orc.norm_test(st["S1"], st["S2"], 4, 0.5, b_cur=2, b_max=64, V=st["V"])
    assert res["variance"] == pytest.approx(4 / 3) and res["b_req"] == 3
    assert res["test_passed"] == 0


def test_eq4_equivalence_and_monotone():
    # eq. 4 rearranged: pass <=> b_cur >= sigma^2/(eta^2 ||g||^2); requested batch never shrinks
    r = _rng(50)
    for _ in range(200):
        B = int(r.integers(2, 40))
        S2 = float(r.uniform(0.1, 10.0)) * B
        S1 = S2 / B + float(r.uniform(0.0, 50.0))
        eta = float(r.uniform(0.05, 0.95))
        b_cur = int(r.integers(1, 300))
        res = orc.norm_test(S1, S2, B, eta, b_cur, b_max=32)
        sigma2 = (S1 - S2 / B) / (B - 1)
        g2 = S2 / B ** 2
        # E||g_k - grad F||^2 ~ sigma^2 / b  <= eta^2 ||grad F||^2
        assert res["test_passed"] == int(sigma2 / b_cur <= eta * eta * g2 * (1 + 1e-15))
        assert res["b_req"] >= b_cur
        assert res["b_req"] >= math.ceil(res["stat"]) or res["b_req"] == b_cur
        raw = orc.norm_test(S1, S2, B, eta, b_cur, b_max=32, allow_shrink=True)
        assert raw["b_req"] == max(1, math.ceil(sigma2 / (eta * eta * g2)))


def test_single_sample_and_zero_gradient_conventions():
    res = orc.norm_test(5.0, 5.0, 1, 0.3, b_cur=1, b_max=32)
    assert res["stat_undefined"] == 1 and res["b_req"] == 2 and res["test_passed"] == 0
    res = orc.norm_test(2.0, 0.0, 2, 0.3, b_cur=2, b_max=32, b_cap=0)
    assert math.isinf(res["stat"]) and res["b_req"] == orc.INT64_MAX and res["accumulate"] == 1
    res = orc.norm_test(0.0, 0.0, 4, 0.3, b_cur=4, b_max=32)
    assert res["stat"] == 0.0 and res["b_req"] == 4 and res["test_passed"] == 1


def test_switch_mode_cases():
    n = 0
    for ln in _lines("switch_mode_cases.txt"):
        lhs, rhs = ln.split("->")
        b_req, b_max, nsw = [int(v) for v in lhs.split()]
        acc, steps, micro = [int(v) for v in rhs.split()]
        got = orc.switch_mode(b_req, b_max, nsw)
        assert (got["accumulate"], got["accum_steps"], got["b_micro"]) == (acc, steps, micro), ln
        # the micro-batches always cover the requested batch when accumulating
        if acc:
            assert steps * micro >= b_req > (steps - 1) * micro
        n += 1
    assert n >= 12


def test_check_merge_cases():
    n = 0
    for ln in _lines("check_merge_cases.txt"):
        b, w, want = ln.split(";")
        assert orc.check_merge(_ints(b), int(w)) == _ints(want), ln
        n += 1
    assert n >= 12


# ------------------------------------------------------------------ outer step

def _outer_case(seed=60, N=257, M=3):
    r = _rng(seed)
    th = (0.02 * r.standard_normal(N)).astype(np.float32)
    ins = [(th - (1e-3 * r.standard_normal(N)).astype(np.float32)) for _ in range(M)]
    mom = (1e-4 * r.standard_normal(N)).astype(np.float32)
    return th, ins, mom


def test_inner_product_hand_cases():
    n = 0
    for ln in _lines("inner_product_hand_cases.txt"):
        lhs, want = ln.split("->")
        rows, vth, nu = lhs.split(";")
        g = np.array([[float(v) for v in r.split(",")] for r in rows.split("|")])
        B = len(g)
        G = g.sum(axis=0)
        c = g @ G
        n_s = (g ** 2).sum(axis=1)
        S2 = float(G @ G)
        w = [float(v) for v in want.split()]
        for rows_arg in (None, g):
            res = orc.inner_product_test(n_s, c, S2, float(vth), float(nu), B, 64, g_rows=rows_arg)
            assert res["var_ip"] == pytest.approx(w[0], abs=1e-12)
            assert res["var_aug"] == pytest.approx(w[1], abs=1e-12)
            assert res["stat_ip"] == pytest.approx(w[2], abs=1e-12)
            assert res["stat_aug"] == pytest.approx(w[3], abs=1e-12)
        n += 1
    assert n >= 3


def test_inner_products_identities():
    r = _rng(80)
    B, T = 5, 4
    a = r.standard_normal((B, T, 6))
    d = r.standard_normal((B, T, 3))
    ids = r.integers(0, 4, size=(B, T))
    blocks = [(a, d), ("rowsum", None, d), ("rowsum", d * 0.5, d), ("embed", ids, d)]
    st = orc.grad_stats(blocks, two_pass=False)
    c = orc.inner_products(blocks)
    rows = orc.explicit_sample_gradients(blocks)
    G = rows.sum(axis=0)
    # c_i is the dot product of the explicit rows with their sum; the c_i add up to ||G||^2 = S2;
    # the rows reproduce the per-sample norms
    np.testing.assert_allclose(c, rows @ G, rtol=1e-12)
    assert c.sum() == pytest.approx(st["S2"], rel=1e-12)
    np.testing.assert_allclose((rows ** 2).sum(axis=1), st["n_sample"], rtol=1e-12)
    # numpy's var over <g_i, g_k>, and the residual vectors against the scalar form
    res_s = orc.inner_product_test(st["n_sample"], c, st["S2"], 0.3, 0.3, B, 64)
    res_v = orc.inner_product_test(st["n_sample"], c, st["S2"], 0.3, 0.3, B, 64, g_rows=rows)
    assert res_s["var_ip"] == pytest.approx(np.var(rows @ (G / B), ddof=1), rel=1e-12)
    assert res_s["var_aug"] == pytest.approx(res_v["var_aug"], rel=1e-10)
    gk = G / B
    resid = rows - np.outer((rows @ gk) / (gk @ gk), gk)
    np.testing.assert_allclose(resid.mean(axis=0), 0.0, atol=1e-12)      # residuals average to zero
    np.testing.assert_allclose(resid @ gk, 0.0, atol=1e-10)              # and are orthogonal to g_k
    assert res_s["var_aug"] == pytest.approx(np.var(resid, axis=0, ddof=1).sum(), rel=1e-10)
    # an accumulated batch: c against the sum over both halves
    half = [tuple(x[:2] if isinstance(x, np.ndarray) else x for x in e) for e in blocks]
    c_half = orc.inner_products(half, G=st["G"], embed_rows=st["embed_rows"])
    np.testing.assert_allclose(c_half, c[:2], rtol=1e-12)
    # ... also when a micro-batch touches fewer table rows than the whole batch
    ids2 = np.array([[0, 0, 1, 1], [5, 5, 2, 2], [7, 3, 3, 3], [1, 1, 1, 1], [6, 6, 6, 0]])
    blocks2 = [(a, d), ("embed", ids2, d)]
    st2 = orc.grad_stats(blocks2, two_pass=False)
    c2 = orc.inner_products(blocks2)
    np.testing.assert_allclose(c2, orc.explicit_sample_gradients(blocks2) @
                               orc.explicit_sample_gradients(blocks2).sum(axis=0), rtol=1e-12)
    tail = [(a[3:], d[3:]), ("embed", ids2[3:], d[3:])]
    np.testing.assert_allclose(orc.inner_products(tail, G=st2["G"], embed_rows=st2["embed_rows"]),
                               c2[3:], rtol=1e-12)


def test_inner_product_special_cases():
    # collinear gradients g_i = s_i * u: residuals vanish, var_aug = 0; <g_i,g_k> = s_i * mean(s)
    u = np.array([3.0, 4.0])
    sc = np.array([1.0, 2.0, 4.0, 5.0])
    g = np.outer(sc, u)
    G = g.sum(axis=0)
    res = orc.inner_product_test((g ** 2).sum(axis=1), g @ G, float(G @ G), 0.5, 0.3, 4, 64, g_rows=g)
    assert res["var_aug"] == pytest.approx(0.0, abs=1e-12)
    assert res["var_ip"] == pytest.approx(np.var(sc * sc.mean() * 25.0, ddof=1), rel=1e-12)
    # identical samples: both variances vanish, requested batches stay at b_cur
    g = np.tile(u, (3, 1))
    G = g.sum(axis=0)
    res = orc.inner_product_test((g ** 2).sum(axis=1), g @ G, float(G @ G), 0.01, 0.3, 7, 64)
    assert res["stat_ip"] == 0.0 and res["stat_aug"] == pytest.approx(0.0, abs=1e-12)
    assert res["b_req_ip"] == 7 and res["b_req_aug"] == 7
    # gradients that cancel (g_k = 0): nothing to project on, the residuals are the g_i; both
    # statistics are unbounded, the requests go to the ceiling
    g = np.array([[1.0, 2.0], [-1.0, -2.0], [2.0, -1.0], [-2.0, 1.0]])
    for rows_arg in (None, g):
        res = orc.inner_product_test((g ** 2).sum(axis=1), g @ g.sum(axis=0), 0.0, 0.01, 0.3, 4, 64,
                                     b_cap=1000, g_rows=rows_arg)
        assert res["var_aug"] == pytest.approx(20.0 / 3.0, rel=1e-12)
        assert res["var_ip"] == 0.0 and res["stat_ip"] == 0.0 and math.isinf(res["stat_aug"])
        assert res["b_req_ip"] == 4 and res["b_req_aug"] == 1000
    # the augmented request is never below the inner-product request; scaling all gradients by s
    # leaves both statistics unchanged
    r = _rng(81)
    g = r.standard_normal((6, 5))
    G = g.sum(axis=0)
    a = orc.inner_product_test((g ** 2).sum(axis=1), g @ G, float(G @ G), 0.2, 0.3, 2, 64)
    g2 = 7.0 * g
    G2 = g2.sum(axis=0)
    b = orc.inner_product_test((g2 ** 2).sum(axis=1), g2 @ G2, float(G2 @ G2), 0.2, 0.3, 2, 64)
    assert a["b_req_aug"] >= a["b_req_ip"]
    assert a["stat_ip"] == pytest.approx(b["stat_ip"], rel=1e-12)
    assert a["stat_aug"] == pytest.approx(b["stat_aug"], rel=1e-12)
    # one sample: undefined, ask for two
    one = orc.inner_product_test([1.0], [1.0], 1.0, 0.2, 0.3, 1, 64)
    assert one["stat_undefined"] == 1 and one["b_req_ip"] == 2 and one["b_req_aug"] == 2


def test_inner_step_matches_torch_adamw():
    # library route: several steps of torch.optim.AdamW in float64
    import torch
    r = _rng(70)
    N = 257
    theta = r.standard_normal(N).astype(np.float32)
    m = np.zeros(N, dtype=np.float32)
    v = np.zeros(N, dtype=np.float32)
    p = torch.tensor(theta.astype(np.float64), requires_grad=True)
    opt = torch.optim.AdamW([p], lr=4e-4, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.1)
    x64, m64, v64 = theta.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    for step in range(1, 6):
        g = r.standard_normal(N).astype(np.float32) * 3
        p.grad = torch.tensor(0.25 * g.astype(np.float64))
        opt.step()
        o = orc.inner_step(x64, m64, v64, g, step, 4e-4, grad_scale=0.25)
        x64, m64, v64 = o["theta_f64"], o["exp_avg_f64"], o["exp_avg_sq_f64"]
        np.testing.assert_allclose(x64, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_inner_step_closed_forms():
    r = _rng(71)
    N = 64
    theta = r.standard_normal(N).astype(np.float32)
    g = (r.standard_normal(N) + 0.1).astype(np.float32)
    z = np.zeros(N, dtype=np.float32)
    # first step from a zero state without decay: m_hat = g, v_hat = g^2 -> lr * g / (|g| + eps)
    o = orc.inner_step(theta, z, z, g, 1, 1e-2, weight_decay=0.0, eps=1e-8)
    g64 = g.astype(np.float64)
    np.testing.assert_allclose(o["theta_f64"], theta - 1e-2 * g64 / (np.abs(g64) + 1e-8), rtol=1e-12)
    # zero gradient and zero state: pure decoupled decay x (1 - lr * wd)
    o = orc.inner_step(theta, z, z, z, 3, 1e-2, weight_decay=0.1)
    np.testing.assert_allclose(o["theta_f64"], theta.astype(np.float64) * (1 - 1e-3), rtol=1e-15)
    # the update is odd in the gradient and invariant to its scale on the first step (eps -> 0)
    a = orc.inner_step(z, z, z, g, 1, 1e-2, weight_decay=0.0, eps=0.0)
    b = orc.inner_step(z, z, z, -7.0 * g, 1, 1e-2, weight_decay=0.0, eps=0.0)
    np.testing.assert_allclose(a["theta_f64"], -b["theta_f64"], rtol=1e-12)
    # grad_scale multiplies the gradient
    c = orc.inner_step(theta, z, z, g, 2, 1e-3, grad_scale=0.5)
    d = orc.inner_step(theta, z, z, (0.5 * g64).astype(np.float64), 2, 1e-3)
    np.testing.assert_allclose(c["theta_f64"], d["theta_f64"], rtol=1e-13)


def test_outer_m1_lr1_mu0_returns_inner_model():
    th, ins, _ = _outer_case(M=1)
    out = orc.outer_step(th, ins, None, lr=1.0, mu=0.0)
    np.testing.assert_array_equal(out["theta_outer"], ins[0])


def test_outer_mu0_lr1_is_localsgd_average():
    # Section 3.1 (LocalSGD): synchronisation replaces the model by the mean over workers
    th, ins, mom = _outer_case(M=4)
    out = orc.outer_step(th, ins, mom, lr=1.0, mu=0.0, nesterov=False)
    want = np.mean(np.stack([i.astype(np.float64) for i in ins]), axis=0)
    np.testing.assert_allclose(out["theta_outer_f64"], want, rtol=1e-13, atol=1e-18)
    out2 = orc.outer_step(th, ins, mom, lr=1.0, mu=0.0, nesterov=True)
    np.testing.assert_allclose(out2["theta_outer_f64"], want, rtol=1e-13, atol=1e-18)


def test_outer_fixed_points():
    th, ins, mom = _outer_case(M=3)
    same = [th.copy() for _ in range(3)]
    out = orc.outer_step(th, same, np.zeros_like(th), lr=0.7, mu=0.9)
    np.testing.assert_array_equal(out["theta_outer"], th)
    np.testing.assert_array_equal(out["momentum"], np.zeros_like(th))
    out = orc.outer_step(th, same, mom, lr=0.7, mu=0.9)
    want = th.astype(np.float64) - 0.7 * 0.81 * mom.astype(np.float64)
    np.testing.assert_allclose(out["theta_outer_f64"], want, rtol=1e-13)
    out = orc.outer_step(th, same, mom, lr=0.7, mu=0.9, nesterov=False)
    want = th.astype(np.float64) - 0.7 * 0.9 * mom.astype(np.float64)
    np.testing.assert_allclose(out["theta_outer_f64"], want, rtol=1e-13)


def test_outer_instance_order_invariance():
    th, ins, mom = _outer_case(M=4)
    base = orc.outer_step(th, ins, mom, lr=0.7, mu=0.9)
    for perm in itertools.permutations(range(4)):
        out = orc.outer_step(th, [ins[p] for p in perm], mom, lr=0.7, mu=0.9)
        np.testing.assert_allclose(out["theta_outer_f64"], base["theta_outer_f64"], rtol=1e-13,
                                   atol=1e-18)
        np.testing.assert_allclose(out["momentum_f64"], base["momentum_f64"], rtol=1e-12, atol=1e-20)


def test_outer_sign_and_scale():
    # instances moved by -d from theta (theta_k = theta - d): the outer model must move the same way
    th = np.zeros(4, dtype=np.float32)
    d = np.array([1.0, -2.0, 0.5, 0.0], dtype=np.float32)
    out = orc.outer_step(th, [th - d, th - d], np.zeros(4, np.float32), lr=0.5, mu=0.0)
    np.testing.assert_allclose(out["pseudo_grad"], d)
    np.testing.assert_allclose(out["theta_outer"], -0.5 * d)


@pytest.mark.parametrize("nesterov", [True, False])
def test_outer_matches_torch_sgd(nesterov):
    # library route: torch.optim.SGD fed grad = Delta, two consecutive steps so that the second
    # starts from a non-zero momentum buffer
    import torch
    th, ins, _ = _outer_case(seed=61, N=100, M=3)
    p = torch.nn.Parameter(torch.from_numpy(th.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=0.7, momentum=0.9, nesterov=nesterov)
    x = th.astype(np.float64)
    buf = np.zeros_like(x)
    r = _rng(62)
    for step in range(2):
        cur = [x - 1e-3 * r.standard_normal(100) for _ in range(3)]
        p.grad = torch.from_numpy(np.mean([x - c for c in cur], axis=0))
        opt.step()
        out = orc.outer_step(x, cur, buf, lr=0.7, mu=0.9, nesterov=nesterov)
        x, buf = out["theta_outer_f64"], out["momentum_f64"]
        np.testing.assert_allclose(x, p.detach().numpy(), rtol=1e-12, atol=1e-16)


def test_outer_broadcast():
    th, ins, mom = _outer_case(M=2)
    out = orc.outer_step(th, ins, mom, lr=0.7, mu=0.9, broadcast=True)
    for t in out["thetas"]:
        np.testing.assert_array_equal(t, out["theta_outer"])


# ------------------------------------------------------------------ merge

def test_merge_properties():
    r = _rng(70)
    xs = [r.standard_normal(101).astype(np.float32) for _ in range(4)]
    eq = orc.merge(xs, [5, 5, 5, 5])
    np.testing.assert_allclose(eq["x_merge_f64"], np.mean([x.astype(np.float64) for x in xs], axis=0),
                               rtol=1e-13, atol=1e-17)
    assert eq["rep"] == 0                                   # ties -> lowest index
    one = orc.merge(xs[:1], [7])
    np.testing.assert_array_equal(one["x_merge"], xs[0])    # singleton = identity
    w = [3, 9, 1, 9]
    m = orc.merge(xs, w)
    assert m["rep"] == 1                                    # argmax, first of the ties
    m2 = orc.merge(xs, [10 * v for v in w])
    np.testing.assert_allclose(m2["x_merge_f64"], m["x_merge_f64"], rtol=1e-13, atol=1e-17)
    lo, hi = np.min(xs, axis=0), np.max(xs, axis=0)
    assert np.all(m["x_merge_f64"] >= lo - 1e-12) and np.all(m["x_merge_f64"] <= hi + 1e-12)
    # hand value: weights 1 and 3 on values 0 and 4 -> 3
    h = orc.merge([np.zeros(2, np.float32), np.full(2, 4, np.float32)], [1, 3])
    np.testing.assert_array_equal(h["x_merge"], np.full(2, 3, np.float32))
    assert h["rep"] == 1


# ------------------------------------------------------------------ one round of Algorithm 3

def _round_batch_fn(shapes, T):
    def fn(uid, worker, h, s, b, theta):
        out = []
        for l, (di, do) in enumerate(shapes):
            seed = 100000 * uid + 1000 * worker + 100 * h + 10 * s + l
            r = _rng(seed)
            shared = r.standard_normal((1, T, di + do))
            x = 0.6 * shared + 0.8 * r.standard_normal((b, T, di + do))
            out.append((x[:, :, :di].astype(np.float32), (0.1 * x[:, :, di:]).astype(np.float32)))
        return out
    return fn


def _round_trainers(k, M, N, b_reqs):
    r = _rng(77)
    ts = []
    for i in range(k):
        th = (0.02 * r.standard_normal(N)).astype(np.float32)
        ts.append(dict(uid=i, theta_outer=th, momentum=np.zeros(N, np.float32), b_req=b_reqs[i],
                       workers=[dict(theta=th.copy(), exp_avg=np.zeros(N, np.float32),
                                     exp_avg_sq=np.zeros(N, np.float32), step=0) for _ in range(M)]))
    return ts


_ROUND_CFG = dict(inner_steps=2, b_max=4, n_switch=2, b_cap=64, eta=0.5, merge_w=0, lr_inner=1e-3,
                  beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1, lr_outer=0.7, mu_outer=0.9,
                  nesterov=1)


def test_round_reduces_to_its_parts():
    # one trainer, one worker, one inner step, no merge: the round is grad_stats -> norm test ->
    # AdamW step -> outer step on the same batch, each pinned separately above
    shapes, T = [(5, 3), (3, 2)], 4
    N = sum(a * b for a, b in shapes)
    fn = _round_batch_fn(shapes, T)
    ts = _round_trainers(1, 1, N, [3])
    th0 = ts[0]["theta_outer"].copy()
    cfg = dict(_ROUND_CFG, inner_steps=1)
    rep = orc.round_step(ts, cfg, fn)
    blocks = fn(0, 0, 0, 0, 3, th0)
    st = orc.grad_stats(blocks, two_pass=False)
    g = np.concatenate([G.reshape(-1) for G in st["G"]])
    o = orc.inner_step(th0, np.zeros(N, np.float32), np.zeros(N, np.float32), g, 1, 1e-3, grad_scale=1 / 3)
    out = orc.outer_step(th0, [o["theta"]], np.zeros(N, np.float32), 0.7, 0.9, True)
    np.testing.assert_array_equal(ts[0]["theta_outer"], out["theta_outer"])
    nt = orc.norm_test(st["S1"], st["S2"], 3, 0.5, 3, 4, 2, 64)
    assert ts[0]["b_req"] == nt["b_req"] and rep[0]["accumulate"] == 0 and rep[0]["b_micro"] == 3


def test_round_merge_switch_and_bookkeeping():
    shapes, T = [(6, 4)], 3
    N = 24
    fn = _round_batch_fn(shapes, T)
    ts = _round_trainers(3, 2, N, [2, 9, 3])
    before = [t["theta_outer"].copy() for t in ts]
    rep = orc.round_step(ts, dict(_ROUND_CFG, merge_w=2), fn)
    # CheckMerge picks the two smallest requests (trainers 0 and 2); the representative is the one
    # with the larger request (trainer 2); trainer 1 (b_req 9 > 2 * 4) accumulates 3 micro-batches of 4
    assert [t["uid"] for t in ts] == [1, 2]
    assert rep[0]["accumulate"] == 1 and rep[0]["accum_steps"] == 3 and rep[0]["b_micro"] == 4
    assert rep[1]["accumulate"] == 0 and rep[1]["b_micro"] == 3 and rep[1]["merged_from"] == 1
    assert all(w["step"] == 2 for t in ts for w in t["workers"])
    # requested batches never shrink (monotone reading) and respect the ceiling
    assert ts[0]["b_req"] >= 9 and ts[1]["b_req"] >= 3 and max(t["b_req"] for t in ts) <= 64
    # with lr_inner = 0 and no decay the workers do not move: Delta = 0 and, from a zero
    # momentum, the outer model of an unmerged trainer is unchanged
    ts2 = _round_trainers(3, 2, N, [2, 9, 3])
    orc.round_step(ts2, dict(_ROUND_CFG, lr_inner=0.0, weight_decay=0.0), fn)
    for t, b in zip(ts2, before):
        np.testing.assert_array_equal(t["theta_outer"], b)


# ------------------------------------------------------------------ round_step against a case sequenced by hand

_CASE_SHAPES, _CASE_T = [(3, 2), (2, 2)], 2
_CASE_N = sum(a * b for a, b in _CASE_SHAPES)
_CASE_CFG = dict(inner_steps=2, b_max=2, n_switch=2, b_cap=64, eta=0.5, merge_w=2, lr_inner=1e-3,
                 beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1, lr_outer=0.7, mu_outer=0.9,
                 nesterov=1)


def _round_case_expected():
    want = dict(test={}, worker={}, switch={}, theta_outer={}, momentum={})
    for ln in open(os.path.join(GOLD, "round_step_case.txt")):
        f = ln.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "remaining_uids":
            want["uids"] = [int(v) for v in f[1:]]
        elif f[0] == "merged_from":
            want["merged_from"] = [int(v) for v in f[1:]]
        elif f[0] == "test":
            want["test"][int(f[1])] = dict(b_cur=int(f[3]), stat=float(f[5]), passed=int(f[7]), b_next=int(f[9]))
        elif f[0] == "worker":
            want["worker"][(int(f[1]), int(f[2]))] = (int(f[4]), np.array([float(v) for v in f[6:]]))
        elif f[0] == "switch":
            want["switch"][int(f[1])] = (int(f[3]), int(f[5]), int(f[7]))
        else:
            want[f[0]][int(f[1])] = np.array([float(v) for v in f[2:]])
    return want


def _round_case_check(round_fn):
    """Runs round_fn on the case of tests/golden/round_step_case.txt and compares everything the
    fixture holds.  Raises AssertionError on the first difference."""
    import adloco_synth as synth
    fn = synth.round_batch_fn(_CASE_SHAPES, _CASE_T)
    ts = synth.round_trainers(3, 2, _CASE_N, [3, 5, 2], stale_workers=True)
    rep = round_fn(ts, dict(_CASE_CFG), fn)
    want = _round_case_expected()
    assert [t["uid"] for t in ts] == want["uids"]
    assert [r["merged_from"] for r in rep] == want["merged_from"]
    for t, r in zip(ts, rep):
        u = t["uid"]
        assert (r["accumulate"], r["accum_steps"], r["b_micro"]) == want["switch"][u]
        w = want["test"][u]
        assert r["test"]["b_cur"] == w["b_cur"] and r["test"]["test_passed"] == w["passed"]
        np.testing.assert_allclose(r["test"]["stat"], w["stat"], rtol=1e-9)
        assert t["b_req"] == w["b_next"]
        for m, wk in enumerate(t["workers"]):
            step, theta = want["worker"][(u, m)]
            assert wk["step"] == step
            np.testing.assert_allclose(wk["theta"], theta, rtol=2e-6, atol=1e-9)
        np.testing.assert_allclose(t["theta_outer"], want["theta_outer"][u], rtol=2e-6, atol=1e-9)
        np.testing.assert_allclose(t["momentum"], want["momentum"][u], rtol=2e-6, atol=1e-10)


def test_round_step_matches_the_case_sequenced_by_hand():
    # 3 trainers x 2 workers, H = 2, a merge, one trainer cut to b_max, one accumulating 3 x 2:
    # expected values from tests/golden/make_round_step_case.py, which never calls round_step
    _round_case_check(orc.round_step)


_ROUND_MUTATIONS = [
    # (what goes wrong, text of round_step, replacement)
    ("gradient scale without the accumulation count",
     'grad_scale=1.0 / (sm["accum_steps"] * sm["b_micro"])', 'grad_scale=1.0 / sm["b_micro"]'),
    ("norm test on another worker's batch", "if m == 0 and h == 0:", "if m == 1 and h == 0:"),
    ("norm test on the second inner step's batch", "if m == 0 and h == 0:", "if m == 0 and h == 1:"),
    ("workers not reset to the trainer's model",
     'w["theta"] = np.array(t["theta_outer"], dtype=np.float32, copy=True)', 'w["theta"] = w["theta"]'),
    ("norm test told the requested instead of the actual batch size",
     'cfg["eta"], int(st["B"]), cfg["b_max"]', 'cfg["eta"], int(t["b_req"]), cfg["b_max"]'),
    ("next request may shrink", 'b_next = max(int(t["b_req"]), int(nt["b_req"]))', 'b_next = int(nt["b_req"]) - 8'),
    ("one micro-batch too few", 'for s in range(sm["accum_steps"])]', 'for s in range(max(1, sm["accum_steps"] - 1))]'),
    ("step count not advanced", 'w["step"] += 1', 'w["step"] += 0'),
    ("merge weights ignored", '[trainers[j]["b_req"] for j in sel])', '[1 for j in sel])'),
    ("outer step over the first worker only", '[w["theta"] for w in t["workers"]]', '[t["workers"][0]["theta"]]'),
]


@pytest.mark.parametrize("what,old,new", _ROUND_MUTATIONS, ids=[m[0] for m in _ROUND_MUTATIONS])
def test_round_step_case_catches_planted_mistakes(what, old, new):
    # the case above must fail as soon as round_step is wrong in one of the ways a driver of
    # Algorithm 3 plausibly is: the mistake is planted in a copy of the oracle's own source
    import inspect
    src = inspect.getsource(orc.round_step)
    assert src.count(old) == 1, f"mutation target not found: {old}"
    ns = dict(vars(orc))
    exec(compile(src.replace(old, new), "<mutated round_step>", "exec"), ns)
    with pytest.raises(AssertionError):
        _round_case_check(ns["round_step"])


# ------------------------------------------------------------------ drifts stored in bf16

def test_bf16_rounding_is_nearest_even_and_matches_torch():
    import torch
    # hand cases on the bit pattern: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1);
    # 1 + 3 * 2^-8 is a tie -> even (1 + 2^-6); just above a tie rounds up; exact values stay
    one = np.float32(1.0)
    cases = [(one + np.float32(2.0 ** -8), 0x3F80), (one + np.float32(3 * 2.0 ** -8), 0x3F82),
             (one + np.float32(2.0 ** -8 + 2.0 ** -20), 0x3F81), (np.float32(-0.5), 0xBF00),
             (np.float32(0.0), 0x0000), (np.float32(3.0e38), 0x7F62), (np.float32(np.inf), 0x7F80)]
    for x, want in cases:
        assert int(orc.round_to_bf16_bits(np.array([x]))[0]) == want, (x, hex(want))
    assert np.isnan(orc.widen(orc.round_to_bf16_bits(np.array([np.nan], np.float32)))[0])
    # library pin: torch's own fp32 -> bf16 conversion on two million values of every size
    r = _rng(4401)
    x = (r.standard_normal(2_000_000) * np.exp(r.uniform(-30, 30, 2_000_000))).astype(np.float32)
    tb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(orc.round_to_bf16_bits(x), tb)


def test_pack_drift_hand_values_and_error_bound():
    th = np.array([1.0, 0.02, -0.5, 3.0], np.float32)
    xm = np.array([0.99609375, 0.02, -0.75, 1.0], np.float32)      # drifts 2^-8, 0, 0.25, 2: exact in bf16
    np.testing.assert_array_equal(orc.widen(orc.pack_drift(th, xm)), [2.0 ** -8, 0.0, 0.25, 2.0])
    r = _rng(4402)
    th = (0.02 * r.standard_normal(100_000)).astype(np.float32)
    xm = th - (1e-3 * r.standard_normal(100_000)).astype(np.float32)
    d = orc.widen(orc.pack_drift(th, xm))
    exact = th.astype(np.float64) - xm.astype(np.float64)
    # one fp32 subtraction (2^-24 of the operands) and one bf16 rounding (half an ulp of 8 significant bits: 2^-8 of the drift)
    assert np.all(np.abs(d - exact) <= 2.0 ** -8 * np.abs(exact) + 2.0 ** -23 * np.abs(th))


def test_outer_step_drift_is_outer_step_on_the_stored_drifts():
    r = _rng(4403)
    N, M = 5000, 3
    th = (0.02 * r.standard_normal(N)).astype(np.float32)
    mom = (1e-4 * r.standard_normal(N)).astype(np.float32)
    insts = [th - (1e-3 * r.standard_normal(N)).astype(np.float32) for _ in range(M)]
    bits = [orc.pack_drift(th, x) for x in insts]
    got = orc.outer_step_drift(th, bits, mom, 0.7, 0.9, True)
    # the plain outer step on instances that sit exactly at theta - stored drift (fp64 inputs)
    ref = orc.outer_step(th, [th.astype(np.float64) - orc.widen(b) for b in bits], mom, 0.7, 0.9, True)
    np.testing.assert_allclose(got["theta_outer_f64"], ref["theta_outer_f64"], rtol=0, atol=1e-18)
    np.testing.assert_allclose(got["momentum_f64"], ref["momentum_f64"], rtol=1e-13, atol=1e-20)
    # against the unquantised step: the pseudo-gradient moves by at most 2^-8 of the mean |drift|
    full = orc.outer_step(th, insts, mom, 0.7, 0.9, True)
    bound = 2.0 ** -8 * np.mean([np.abs(th.astype(np.float64) - x) for x in insts], axis=0) + 1e-9
    assert np.all(np.abs(got["pseudo_grad_f64"] - full["pseudo_grad_f64"]) <= bound)
    # hand value: drifts 0.25 and 0.75, zero momentum, lr 1, mu 0 -> theta - 0.5
    h = orc.outer_step_drift(np.array([2.0], np.float32),
                             [orc.round_to_bf16_bits(np.array([0.25], np.float32)),
                              orc.round_to_bf16_bits(np.array([0.75], np.float32))], None, 1.0, 0.0, False)
    assert float(h["theta_outer"][0]) == 1.5 and float(h["pseudo_grad"][0]) == 0.5
    z = orc.outer_step_drift(th, bits, mom, 0.7, 0.9, True, broadcast=True)
    assert all(not b.any() for b in z["drifts"])


def test_merge_drift_is_merge_on_the_stored_drifts():
    r = _rng(4404)
    N = 4000
    xr = (0.02 * r.standard_normal(N)).astype(np.float32)
    others = [xr - (1e-3 * r.standard_normal(N)).astype(np.float32) for _ in range(3)]
    bits = [orc.pack_drift(xr, x) for x in others]
    got = orc.merge_drift(xr, bits, 9.0, [3.0, 5.0, 1.0])
    ref = orc.merge([xr.astype(np.float64)] + [xr.astype(np.float64) - orc.widen(b) for b in bits],
                    [9.0, 3.0, 5.0, 1.0])
    assert ref["rep"] == 0
    np.testing.assert_allclose(got["x_merge_f64"], ref["x_merge_f64"], rtol=0, atol=1e-17)
    # hand value: representative 4 (weight 1), one other at 0 (drift 4, weight 3) -> 1
    h = orc.merge_drift(np.array([4.0], np.float32), [orc.round_to_bf16_bits(np.array([4.0], np.float32))], 1.0, [3.0])
    assert float(h["x_merge"][0]) == 1.0
