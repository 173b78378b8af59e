"""adloco_norm_test_noalloc (the entry point that allocates nothing: partial sums and block table in
a fixed device array of the library) against adloco_norm_test on the same gradient buffers, through
the C ABI: two calls in a row, the second on a smaller list, then the size limits."""
import numpy as np
import pytest

import adloco_synth as synth

pytestmark = pytest.mark.gpu


def _case(ctx, seed, shapes, B, eta):
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    layers = []
    for l, (d_out, d_in) in enumerate(shapes):
        g = synth.normal_f32(seed + l, (d_out, d_in) if d_in > 0 else (d_out,), 0.05)
        layers.append(dict(grad_sum=torch.from_numpy(g).to(DEV), **({"kind": "vector"} if d_in == 0 else {})))
    acc = torch.zeros(2, dtype=torch.float64, device=DEV)
    S2 = sum(float(np.sum(np.square(l["grad_sum"].double().cpu().numpy()))) for l in layers)
    acc[0] = 1.7 * S2 / B + 3.0                       # some S1 > S2 / B
    acc.view(torch.int64)[1] = B
    torch.cuda.synchronize()
    want = A.adloco_norm_test(ctx, layers, acc, eta, B, 32, 2, 4096)
    got = A.adloco_norm_test_noalloc(ctx, layers, acc, eta, B, 32, 2, 4096)
    assert got == want, (got, want)                   # same kernels, same order of summation
    np.testing.assert_allclose(got["S2"], S2, rtol=1e-12)
    return got


def test_no_alloc_norm_test_matches_norm_test():
    import torch
    import paper_2508_18182_amd as A
    from gpu_util import DEV
    ctx = A.Context(0)
    # a list of 70 blocks (two table chunks), some unaligned in size, one bias vector, 3.3 M entries
    big = [(257, 129), (64, 0)] + [(192 + 8 * l, 256) for l in range(68)]
    r1 = _case(ctx, 4100, big, 24, 0.3)
    # the second call is smaller: whatever the first one left in the array must not be read
    r2 = _case(ctx, 4200, [(31, 17), (8, 0)], 5, 0.5)
    assert r2["S2"] < r1["S2"] * 1e-2
    r3 = _case(ctx, 4100, big, 24, 0.3)
    assert r3 == r1
    # limits: more blocks than the fixed table, more entries than the fixed partial sums
    g = torch.zeros(4, 4, device=DEV)
    acc = torch.zeros(2, dtype=torch.float64, device=DEV)
    acc.view(torch.int64)[1] = 4
    with pytest.raises(A.AdlocoError) as e:
        A.adloco_norm_test_noalloc(ctx, [dict(grad_sum=g)] * 513, acc, 0.3, 4, 32)
    assert e.value.code == 2 and "512" in str(e.value)
    descs = (A.LinearDesc * 3)()
    for d in descs:                                   # 3 x 2^30 entries: never touched, the call refuses first
        d.grad_sum, d.d_in, d.d_out = g.data_ptr(), 1 << 15, 1 << 15
    with pytest.raises(A.AdlocoError) as e:
        A.adloco_norm_test_noalloc(ctx, None, acc, 0.3, 4, 32, descs=descs)
    assert e.value.code == 2 and "partial" in str(e.value)
    # an empty accumulator is a state error, as in adloco_norm_test
    acc.zero_()
    with pytest.raises(A.AdlocoError) as e:
        A.adloco_norm_test_noalloc(ctx, [dict(grad_sum=g)], acc, 0.3, 4, 32)
    assert e.value.code == 5
    ctx.close()
