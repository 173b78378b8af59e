"""Writes tests/golden/round_step_case.txt: the expected result of one outer step of Algorithm 3
on a tiny case, worked out WITHOUT the oracle's round_step.

Only element functions of the oracle that are pinned on their own are called (check_merge, merge,
switch_mode, grad_stats, norm_test, inner_step, outer_step), in a sequence written out for this one
case: trainer by trainer, the accumulated batch formed by ADDING the micro-batches' gradient sums and
sample-norm sums (Algorithm 3's "g <- g + grad L") rather than by concatenating them.

Case: 3 trainers x 2 workers, H = 2 inner steps, b_max = 2, n = 2, merge_w = 2, requests (3, 5, 2).
  * CheckMerge picks the two smallest requests, trainers 2 and 0; the representative is trainer 0
    (larger request), whose outer model becomes (3 x_0 + 2 x_2) / 5; trainer 2 is dropped.
  * trainer 0 (request 3 <= n b_max = 4) does not accumulate, its batch is cut to b_max = 2 samples;
    trainer 1 (request 5 > 4) accumulates ceil(5 / 2) = 3 micro-batches of 2.
  * every worker starts from its trainer's (merged) outer model, keeps its own AdamW moments and
    step count, and takes 2 inner steps with gradient = sum / (accum * b_micro);
  * the norm test reads the first inner step's batch of worker 0, with b_cur = the samples in it;
    the next request is max(previous request, result);
  * Delta = mean over the 2 workers of (x_T - x_m), Nesterov outer step.

Run from the repository root:  python tests/golden/make_round_step_case.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import adloco_synth as synth                      # noqa: E402
from oracle import adloco_oracle as orc           # noqa: E402

SHAPES, T = [(3, 2), (2, 2)], 2
N = sum(a * b for a, b in SHAPES)
CFG = dict(inner_steps=2, b_max=2, n_switch=2, b_cap=64, eta=0.5, merge_w=2, lr_inner=1e-3, beta1=0.9,
           beta2=0.999, eps=1e-8, weight_decay=0.1, lr_outer=0.7, mu_outer=0.9, nesterov=1)
B_REQ = [3, 5, 2]


def accumulated(fn, uid, worker, h, accum, b_micro, theta):
    """Sum of the micro-batches' gradient sums and of their sample-norm sums."""
    G, S1 = None, 0.0
    for s in range(accum):
        st = orc.grad_stats(fn(uid, worker, h, s, b_micro, theta), two_pass=False)
        g = np.concatenate([np.asarray(x, np.float64).reshape(-1) for x in st["G"]])
        G = g if G is None else G + g
        S1 += st["S1"]
    return G, S1


def main():
    fn = synth.round_batch_fn(SHAPES, T)
    ts = synth.round_trainers(3, 2, N, B_REQ, stale_workers=True)
    # --- merge
    sel = orc.check_merge(B_REQ, CFG["merge_w"])
    assert sel == [2, 0], sel
    x_merged = orc.merge([ts[2]["theta_outer"], ts[0]["theta_outer"]], [2, 3])
    assert x_merged["rep"] == 1
    outer = {0: x_merged["x_merge"], 1: ts[1]["theta_outer"]}
    lines = ["# one outer step of Algorithm 3 (3 trainers x 2 workers, H = 2, b_max = 2, requests 3, 5, 2);",
             "# written by tests/golden/make_round_step_case.py from the oracle's element functions only",
             "remaining_uids 0 1", "merged_from 1 0"]
    for uid, accum, b_micro in ((0, 1, 2), (1, 3, 2)):
        sm = orc.switch_mode(B_REQ[uid], CFG["b_max"], CFG["n_switch"])
        assert (sm["accum_steps"], sm["b_micro"]) == (accum, b_micro)
        x_T = np.asarray(outer[uid], np.float32)
        finals = []
        for m in (0, 1):
            w = ts[uid]["workers"][m]
            th, ea, es, step = x_T.copy(), w["exp_avg"], w["exp_avg_sq"], w["step"]
            for h in (0, 1):
                G, S1 = accumulated(fn, uid, m, h, accum, b_micro, th)
                if m == 0 and h == 0:
                    n = accum * b_micro
                    nt = orc.norm_test(S1, float(np.dot(G, G)), n, CFG["eta"], n, CFG["b_max"],
                                       CFG["n_switch"], CFG["b_cap"])
                    lines.append(f"test {uid} b_cur {n} stat {nt['stat']!r} passed {nt['test_passed']} "
                                 f"b_req_next {max(B_REQ[uid], nt['b_req'])}")
                step += 1
                o = orc.inner_step(th, ea, es, G, step, CFG["lr_inner"], CFG["beta1"], CFG["beta2"],
                                   CFG["eps"], CFG["weight_decay"], grad_scale=1.0 / (accum * b_micro))
                th, ea, es = o["theta"], o["exp_avg"], o["exp_avg_sq"]
            finals.append(th)
            lines.append(f"worker {uid} {m} step {step} theta " + " ".join(repr(float(v)) for v in th))
        o = orc.outer_step(x_T, finals, ts[uid]["momentum"], CFG["lr_outer"], CFG["mu_outer"], True)
        lines.append(f"switch {uid} accumulate {sm['accumulate']} accum_steps {accum} b_micro {b_micro}")
        lines.append(f"theta_outer {uid} " + " ".join(repr(float(v)) for v in o["theta_outer"]))
        lines.append(f"momentum {uid} " + " ".join(repr(float(v)) for v in o["momentum"]))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "round_step_case.txt")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
