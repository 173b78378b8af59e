"""One outer step of Algorithm 3 through the native driver (adloco_round) against the oracle's
round on the same seeded batches: merge, switch mode with accumulation, norm test, AdamW inner
steps and the Nesterov outer step in sequence."""
import numpy as np
import pytest

from oracle import adloco_oracle as orc

pytestmark = pytest.mark.gpu

CFG = dict(inner_steps=2, b_max=4, n_switch=2, b_cap=64, eta=0.5, merge_w=2, lr_inner=1e-3, beta1=0.9,
           beta2=0.999, eps=1e-8, weight_decay=0.1, lr_outer=0.7, mu_outer=0.9, nesterov=1)


@pytest.fixture(scope="module")
def ctx():
    import paper_2508_18182_amd as A
    c = A.Context(0)
    yield c
    c.close()


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _host_batch(shapes, vec_d, T):
    """Seeded stand-in for the model: blocks (linear weights, then one bias vector) for b samples."""
    def fn(uid, worker, h, s, b, theta):
        out = []
        for l, (di, do) in enumerate(shapes):
            r = _rng(100000 * uid + 1000 * worker + 100 * h + 10 * s + l)
            shared = r.standard_normal((1, T, di + do))
            x = 0.6 * shared + 0.8 * r.standard_normal((b, T, di + do))
            out.append((x[:, :, :di].astype(np.float32), (0.1 * x[:, :, di:]).astype(np.float32)))
        if vec_d:
            out.append(("rowsum", None, out[-1][1]))      # the bias of the last linear layer
        return out
    return fn


def _make_trainers(k, M, N, b_reqs, seed=77):
    r = _rng(seed)
    ts = []
    for i in range(k):
        th = (0.02 * r.standard_normal(N)).astype(np.float32)
        ts.append(dict(uid=i, theta_outer=th, momentum=np.zeros(N, np.float32), b_req=b_reqs[i],
                       workers=[dict(theta=th.copy(), exp_avg=np.zeros(N, np.float32),
                                     exp_avg_sq=np.zeros(N, np.float32), step=0) for _ in range(M)]))
    return ts


def _to_gpu(ts, N, b_max):
    import torch
    dev = "cuda:0"
    out = []
    for t in ts:
        g = dict(uid=t["uid"], b_req=t["b_req"], theta_outer=torch.from_numpy(t["theta_outer"].copy()).to(dev),
                 momentum=torch.from_numpy(t["momentum"].copy()).to(dev),
                 acc=torch.zeros(2, dtype=torch.float64, device=dev),
                 per_sample_sqnorm=torch.zeros(b_max, device=dev), workers=[])
        for w in t["workers"]:
            g["workers"].append(dict(theta=torch.from_numpy(w["theta"].copy()).to(dev),
                                     exp_avg=torch.zeros(N, device=dev), exp_avg_sq=torch.zeros(N, device=dev),
                                     grad=torch.zeros(N, device=dev), step=0))
        out.append(g)
    return out


def _close(got, want, scale, tol):
    return float(np.max(np.abs(got.astype(np.float64) - want.astype(np.float64)))) <= tol * scale


@pytest.mark.parametrize("rounds", [1, 2])
def test_round_matches_oracle(ctx, rounds):
    import torch
    import paper_2508_18182_amd as A
    shapes, vec_d, T = [(24, 16), (16, 8)], 8, 6
    N = sum(a * b for a, b in shapes) + vec_d
    host_fn = _host_batch(shapes, vec_d, T)
    want = _make_trainers(3, 2, N, [2, 9, 3])
    got = _to_gpu(want, N, CFG["b_max"])
    blocks = [dict(d_in=a, d_out=b) for a, b in shapes] + [dict(kind="vector", d_out=vec_d)]

    def gpu_fn(uid, worker, h, s, b, theta_ptr):
        out = []
        for e in host_fn(uid, worker, h, s, b, None):
            if isinstance(e[0], str):
                out.append(dict(x=None, delta=torch.from_numpy(e[2]).cuda()))
            else:
                out.append(dict(a=torch.from_numpy(e[0]).cuda(), delta=torch.from_numpy(e[1]).cuda()))
        return out

    cfg = dict(CFG, T=T, dtype=A.ADLOCO_F32)
    for _ in range(rounds):
        rep_w = orc.round_step(want, CFG, host_fn)
        rep_g = A.adloco_round(ctx, cfg, got, blocks, gpu_fn)
        torch.cuda.synchronize()
        assert [t["uid"] for t in got] == [t["uid"] for t in want]
        for rw, rg in zip(rep_w, rep_g):
            for key in ("b_req_used", "b_micro", "accum_steps", "accumulate", "merged_from"):
                assert rg[key] == rw[key], key
            assert rg["test"]["stat"] == pytest.approx(rw["test"]["stat"], rel=1e-3)
            assert rg["test"]["b_req"] == rw["test"]["b_req"]
    assert len(got) == len(want) == (2 if rounds == 1 else 1)
    for tg, tw in zip(got, want):
        assert tg["b_req"] == tw["b_req"]
        scale = float(np.max(np.abs(tw["theta_outer"])))
        assert _close(tg["theta_outer"].cpu().numpy(), tw["theta_outer"], scale, 2e-5)
        assert _close(tg["momentum"].cpu().numpy(), tw["momentum"], float(np.max(np.abs(tw["momentum"]))) + 1e-30, 2e-4)
        for wg, ww in zip(tg["workers"], tw["workers"]):
            assert wg["step"] == ww["step"]
            assert _close(wg["theta"].cpu().numpy(), ww["theta"], scale, 2e-5)
            assert _close(wg["exp_avg"].cpu().numpy(), ww["exp_avg"], float(np.max(np.abs(ww["exp_avg"]))), 1e-4)


def test_round_errors(ctx):
    import torch
    import paper_2508_18182_amd as A
    N = 24
    ts = _to_gpu(_make_trainers(1, 1, N, [3]), N, 4)
    blocks = [dict(d_in=6, d_out=4)]
    cfg = dict(CFG, T=3, dtype=A.ADLOCO_F32, merge_w=0)

    def failing(uid, worker, h, s, b, theta_ptr):
        raise RuntimeError("no data")

    with pytest.raises(RuntimeError):
        A.adloco_round(ctx, cfg, ts, blocks, failing)
    with pytest.raises(A.AdlocoError):                       # H must be at least 1
        A.adloco_round(ctx, dict(cfg, inner_steps=0), ts, blocks, lambda *a: [])
    ts[0]["b_req"] = 0
    with pytest.raises(A.AdlocoError):                       # a trainer without a requested batch
        A.adloco_round(ctx, cfg, ts, blocks, lambda *a: [])
