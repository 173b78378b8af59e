"""CPU oracle for the AdLoCo data-parallel hot path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  The HIP library never calls it and shares no code, table or constant with it.

Everything is written as the plain definition, in fp64 (numpy), with no blocking, fusion
or reordering: per-sample gradients are materialised explicitly as d_out x d_in matrices
(one library matmul per sample, `delta_i.T @ a_i`), norms are sums of squared entries,
the variance is the two-pass mean-of-squared-deviations, and the outer step and the merge
are element-wise formulas.  The Gram identity that the GPU path uses is deliberately NOT
used here.

Notation (paper, Section 2.1 and Section 3.3.1): a batch B_k of b_k samples; per-sample
gradient grad f(x_k; xi_i) =: g_i; mini-batch gradient g_k = (1/b_k) sum_i g_i (eq. 1).
For one linear layer with weight W [d_out, d_in], sample i with activations
a_i [T, d_in] and output gradients delta_i [T, d_out] has g_i = delta_i^T a_i.

Pins (tests/test_oracle_pins.py): hand closed forms for T = 1, 2; orthonormal / constant
token rows; permutation and rotation invariance; element-by-element brute force; torch
autograd of a bias-free linear layer, and of a linear bias, a LayerNorm gain and bias and an
embedding table for the vector and table blocks (plus their one-token / all-distinct /
all-equal-id closed forms); numpy's var(ddof=1) over the stacked per-sample
gradients; iid-noise expectation B/eta^2; for the inner-product tests hand-worked vectors,
sum_i <g_i, G> = ||G||^2, numpy's var, the explicit residual vectors against the scalar form and
the collinear / orthogonal special cases; torch.optim.AdamW and the first-step / zero-gradient
closed forms for the inner step; LocalSGD averaging (Section 3.1) and
torch.optim.SGD(nesterov=True) for the outer step; convexity / identity cases for the
merge; Algorithm 1's branches enumerated by hand; for round_step (one outer step of Algorithm 3)
a case of 3 trainers x 2 workers x 2 inner steps with a merge, a batch cut to b_max and an
accumulated batch, sequenced by a separate script from the element functions above
(tests/golden/make_round_step_case.py), which ten planted mistakes in round_step each fail.

Parity unpinned (the paper fixes none of these; they are readings documented in the
design notes): the 1/(B-1) normalisation of the variance, the B = 1 convention, the
monotone clamp b_req >= b_cur and the optional ceiling b_cap; in round_step the reading of the
listing itself (which batch feeds the norm test, H inner steps in the accumulate branch).
"""
from __future__ import annotations

import math

import numpy as np

INT64_MAX = (1 << 63) - 1


# --------------------------------------------------------------------------------------
# Input widening (exact; the oracle sees the very bits the GPU sees)
# --------------------------------------------------------------------------------------

def widen(x) -> np.ndarray:
    """fp32 / fp16 array, or uint16 array of bf16 bit patterns  ->  fp64, exactly."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float16, np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported input dtype {x.dtype}")


# --------------------------------------------------------------------------------------
# Gradient statistics (eq. 1; variance of Section 3.3.1)
# --------------------------------------------------------------------------------------

def per_sample_gradient(a_i, delta_i) -> np.ndarray:
    """g_i = sum_t delta_{i,t} a_{i,t}^T  as an explicit [d_out, d_in] fp64 matrix."""
    a_i = widen(a_i)
    delta_i = widen(delta_i)
    assert a_i.ndim == 2 and delta_i.ndim == 2 and a_i.shape[0] == delta_i.shape[0]
    return delta_i.T @ a_i


def per_sample_gradient_rowsum(x_i, delta_i) -> np.ndarray:
    """Per-sample gradient of a parameter vector p [d] that enters the layer element-wise,
    y_t = p * x_t (+ ...): g_i = sum_t delta_{i,t} * x_{i,t}, an explicit [d] fp64 vector.
    x_i = None stands for x = 1, the bias of a linear or normalisation layer (g_i =
    sum_t delta_{i,t}); otherwise x_i is the normalised input of a normalisation layer and p
    its gain.  These are further blocks of the grad f(x_k; xi_i) that eq. 1 averages."""
    delta_i = widen(delta_i)
    if x_i is None:
        return delta_i.sum(axis=0)
    x_i = widen(x_i)
    assert x_i.shape == delta_i.shape
    return (delta_i * x_i).sum(axis=0)


def per_sample_gradient_embedding(ids_i, delta_i, rows) -> np.ndarray:
    """Per-sample gradient of an embedding table E [V, d] (y_t = E[id_t]): row v of g_i is the
    sum of delta_{i,t} over the tokens with id_t = v.  Returned explicitly for the table rows
    listed in `rows` (sorted ids; every other row of g_i is zero): [len(rows), d] fp64."""
    delta_i = widen(delta_i)
    ids_i = np.asarray(ids_i)
    g = np.zeros((len(rows), delta_i.shape[1]), dtype=np.float64)
    pos = np.searchsorted(rows, ids_i)
    assert np.all(rows[pos] == ids_i)
    for t in range(delta_i.shape[0]):        # plain loop: one token adds one row
        g[pos[t]] += delta_i[t]
    return g


def _layer_kind(entry):
    """(a, delta) is a linear layer; ("rowsum", x | None, delta) a bias / gain vector;
    ("embed", ids, delta) an embedding table."""
    if isinstance(entry[0], str):
        return entry[0]
    return "linear"


def _entry_sample_gradient(entry, i, rows=None):
    kind = _layer_kind(entry)
    if kind == "linear":
        return per_sample_gradient(np.asarray(entry[0])[i], np.asarray(entry[1])[i])
    if kind == "rowsum":
        x = None if entry[1] is None else np.asarray(entry[1])[i]
        return per_sample_gradient_rowsum(x, np.asarray(entry[2])[i])
    if kind == "embed":
        return per_sample_gradient_embedding(np.asarray(entry[1])[i], np.asarray(entry[2])[i], rows)
    raise ValueError(kind)


def grad_stats(layers, two_pass: bool = True) -> dict:
    """Statistics of the per-sample gradients of a list of parameter blocks.

    layers: list of (a [B,T,d_in], delta [B,T,d_out]) for linear weights, ("rowsum", x | None,
    delta [B,T,d]) for bias / gain vectors, ("embed", ids [B,T] int, delta [B,T,d]) for
    embedding tables, all sharing B and T.  For an embedding table G holds only the rows whose
    id occurs in the batch (`embed_rows[l]`, sorted); all other rows are zero.
    Returns
      n_layer_sample [L,B]  ||g_i^l||_F^2
      n_sample       [B]    ||g_i||^2 = sum_l ||g_i^l||^2   (g_i = concatenation over layers)
      S1                    sum_i ||g_i||^2
      G              list   sum_i g_i^l   (B times the mini-batch gradient of eq. 1)
      S2                    ||sum_i g_i||^2
      batch_grad_sqnorm     ||g_k||^2 = S2 / B^2            (eq. 1)
      V                     sum_i ||g_i - g_k||^2, by a second explicit pass (two_pass only)
    """
    L = len(layers)
    B = int(np.asarray(layers[0][-1]).shape[0])
    n_ls = np.zeros((L, B), dtype=np.float64)
    G = []
    embed_rows = {}
    for l, entry in enumerate(layers):
        assert np.asarray(entry[-1]).shape[0] == B
        rows = None
        if _layer_kind(entry) == "embed":
            rows = embed_rows[l] = np.unique(np.asarray(entry[1]))
        Gl = None
        for i in range(B):
            g = _entry_sample_gradient(entry, i, rows)
            n_ls[l, i] = np.sum(g * g)
            Gl = g.copy() if Gl is None else Gl + g
        G.append(Gl)
    n_s = n_ls.sum(axis=0)
    S1 = float(n_s.sum())
    S2 = float(sum(np.sum(Gl * Gl) for Gl in G))
    out = dict(n_layer_sample=n_ls, n_sample=n_s, S1=S1, G=G, S2=S2, B=B, embed_rows=embed_rows,
               batch_grad_sqnorm=S2 / (B * B) if B > 0 else float("nan"))
    if two_pass:
        V = 0.0
        for l, entry in enumerate(layers):
            gbar = G[l] / B
            for i in range(B):
                dev = _entry_sample_gradient(entry, i, embed_rows.get(l)) - gbar
                V += float(np.sum(dev * dev))
        out["V"] = V
    return out


def concat_micro_batches(micro_batches):
    """Switch mode (Algorithm 3, accumulate branch): the effective batch is the union of the
    micro-batches.  micro_batches: list over micro-batches of layer lists [(a, delta), ...].
    Returns one layer list over the concatenated samples."""
    L = len(micro_batches[0])
    out = []
    for l in range(L):
        first = micro_batches[0][l]
        parts = []
        for j in range(len(first)):
            if isinstance(first[j], str) or first[j] is None:
                parts.append(first[j])
            else:
                parts.append(np.concatenate([np.asarray(mb[l][j]) for mb in micro_batches], axis=0))
        out.append(tuple(parts))
    return out


# --------------------------------------------------------------------------------------
# Norm test, batch rule, switch mode (Section 3.3.1; Section 4.2; Algorithm 3)
# --------------------------------------------------------------------------------------

def variance(V: float, B: int, biased: bool = False) -> float:
    """sigma^2_{B_k}: trace of the sample covariance of the per-sample gradients.
    V = sum_i ||g_i - g_k||^2.  Unbiased 1/(B-1) by default (a reading; parity unpinned)."""
    if biased:
        return V / B
    return V / (B - 1)


def switch_mode(b_req: int, b_max: int, n_switch: int = 2) -> dict:
    """SwitchMode (Section 4.2; Algorithm 3): gradient accumulation only when the requested
    batch exceeds n * max_batch; then accum = ceil(b_req / b_max) micro-batches of b_max;
    otherwise a single micro-batch of min(b_req, b_max)."""
    if b_req > n_switch * b_max:
        return dict(accumulate=1, accum_steps=-(-b_req // b_max), b_micro=b_max)
    return dict(accumulate=0, accum_steps=1, b_micro=min(b_req, b_max))


def norm_test(S1: float, S2: float, B: int, eta: float, b_cur: int, b_max: int,
              n_switch: int = 2, b_cap: int = 0, biased_var: bool = False,
              allow_shrink: bool = False, V: float | None = None) -> dict:
    """Approximate norm test (eq. 4) and the batch rule b_{k+1} = ceil(sigma^2 /
    (eta^2 ||grad F_B||^2)) of Section 3.3.1, followed by SwitchMode.

    If V (two-pass sum of squared deviations) is given it defines sigma^2; otherwise
    sigma^2 comes from S1 - S2/B.  The test passes when b_cur >= sigma^2/(eta^2 ||g_k||^2),
    the rearranged form of eq. 4.
    """
    res = dict(S1=S1, S2=S2, b_cur=int(b_cur), stat_undefined=0)
    gnorm2 = S2 / (float(B) * float(B)) if B > 0 else float("nan")
    res["batch_grad_sqnorm"] = gnorm2
    ceiling = b_cap if b_cap > 0 else INT64_MAX
    if B < 2 and not biased_var or B < 1:
        # one sample: the sample variance is 0/0 -> ask for two samples so it becomes defined
        res.update(variance=float("nan"), stat=float("nan"), stat_undefined=1, test_passed=0)
        b_req = min(ceiling, max(int(b_cur), 2))
    else:
        dev = V if V is not None else max(S1 - S2 / B, 0.0)
        sigma2 = variance(dev, B, biased_var)
        res["variance"] = sigma2
        if gnorm2 > 0.0:
            stat = sigma2 / (eta * eta * gnorm2)
        else:
            stat = float("inf") if sigma2 > 0.0 else 0.0
        res["stat"] = stat
        res["test_passed"] = 1 if stat <= b_cur else 0
        if math.isinf(stat) or stat >= float(ceiling):
            b_raw = ceiling
        else:
            b_raw = int(math.ceil(stat))
        b_req = b_raw if allow_shrink else max(int(b_cur), b_raw)
        b_req = min(ceiling, max(b_req, 1))
    res["b_req"] = int(b_req)
    res.update(switch_mode(int(b_req), int(b_max), int(n_switch)))
    return res


# --------------------------------------------------------------------------------------
# Inner-product test and augmented inner-product test (Section 3.3.2)
# --------------------------------------------------------------------------------------

def inner_products(layers, G=None, embed_rows=None) -> np.ndarray:
    """c_i = <g_i, G> for every sample, with G = sum_j g_j the gradient sum of the batch
    (B times eq. 1's g_k) unless another list G of per-block sums is given (an accumulated batch:
    G over all micro-batches; embed_rows then names, per embedding block, the table rows that the
    rows of its G stand for, as grad_stats returns them).  Per-sample gradients are formed
    explicitly, block by block."""
    B = int(np.asarray(layers[0][-1]).shape[0])
    rows = {l: np.unique(np.asarray(e[1])) for l, e in enumerate(layers) if _layer_kind(e) == "embed"}
    if embed_rows is not None:
        rows = {l: np.asarray(embed_rows[l]) for l in rows}
    if G is None:
        G = grad_stats(layers, two_pass=False)["G"]
    c = np.zeros(B, dtype=np.float64)
    for l, entry in enumerate(layers):
        for i in range(B):
            g = _entry_sample_gradient(entry, i, rows.get(l))
            c[i] += float(np.sum(g * G[l]))
    return c


def explicit_sample_gradients(layers) -> np.ndarray:
    """All per-sample gradients as rows of one [B, P] fp64 matrix (blocks concatenated; for an
    embedding table only the rows whose id occurs in the batch).  Small shapes only."""
    B = int(np.asarray(layers[0][-1]).shape[0])
    rows = {l: np.unique(np.asarray(e[1])) for l, e in enumerate(layers) if _layer_kind(e) == "embed"}
    out = []
    for i in range(B):
        out.append(np.concatenate([_entry_sample_gradient(e, i, rows.get(l)).reshape(-1)
                                   for l, e in enumerate(layers)]))
    return np.stack(out)


def inner_product_test(n_sample, c, S2: float, vartheta: float, nu: float, b_cur: int, b_max: int,
                       n_switch: int = 2, b_cap: int = 0, g_rows=None) -> dict:
    """Section 3.3.2.  With g_k = G / B the batch gradient, c_i = <g_i, G>:
      inner-product test:  b_ip  = ceil( Var_i(<g_i, g_k>) / (vartheta^2 ||g_k||^4) )
      augmented test:      b_aug = ceil( max{ b_ip, Var_i(g_i - (<g_i, g_k>/||g_k||^2) g_k)
                                                    / (nu^2 ||g_k||^2) } )
    Var_i is the sample variance over the batch with the 1/(B-1) normalisation (for a vector:
    the trace of the sample covariance), the convention of the norm test.  If g_rows (the explicit
    [B, P] matrix of per-sample gradients) is given, the augmented variance is formed from the
    explicit residual vectors; otherwise from the scalars, sum_i (||g_i||^2 - <g_i,g_k>^2 /
    ||g_k||^2) / (B-1), which is the same number because the residuals average to zero.
    Where g_k = 0 the projection has no direction: the residual is then g_i itself (and both
    statistics are +inf unless their variance is zero too, as in the norm test).
    Followed by the monotone clamp, ceiling and SwitchMode of the norm test."""
    c = np.asarray(c, dtype=np.float64)
    n_sample = np.asarray(n_sample, dtype=np.float64)
    B = len(c)
    ceiling = b_cap if b_cap > 0 else INT64_MAX
    res = dict(S2=S2, b_cur=int(b_cur), stat_undefined=0)
    gk2 = S2 / (float(B) * float(B))
    res["batch_grad_sqnorm"] = gk2
    if B < 2:
        res.update(var_ip=float("nan"), stat_ip=float("nan"), var_aug=float("nan"),
                   stat_aug=float("nan"), stat_undefined=1)
        b_ip = b_aug = min(ceiling, max(int(b_cur), 2))
    else:
        ip = c / B                                     # <g_i, g_k>
        var_ip = float(np.sum((ip - ip.mean()) ** 2) / (B - 1))
        # g_k = 0: the component along g_k is taken to be zero, the residual is g_i itself
        coef = ip / gk2 if gk2 > 0 else np.zeros_like(ip)
        if g_rows is not None:
            gk = g_rows.sum(axis=0) / B
            resid = g_rows - np.outer(coef, gk)
            var_aug = float(np.sum((resid - resid.mean(axis=0)) ** 2) / (B - 1))
        else:
            var_aug = float(np.sum(n_sample - ip * coef) / (B - 1))
        res.update(var_ip=var_ip, var_aug=var_aug)

        def ratio(num, den):
            if den > 0.0:
                return num / den
            return float("inf") if num > 0.0 else 0.0

        stat_ip = ratio(var_ip, vartheta * vartheta * gk2 * gk2)
        stat_aug = ratio(var_aug, nu * nu * gk2)
        res.update(stat_ip=stat_ip, stat_aug=stat_aug)

        def to_batch(stat):
            if math.isinf(stat) or stat >= float(ceiling):
                return ceiling
            return int(math.ceil(stat))

        b_ip_raw = to_batch(stat_ip)
        b_aug_raw = to_batch(max(float(b_ip_raw), stat_aug))
        b_ip = min(ceiling, max(int(b_cur), b_ip_raw, 1))
        b_aug = min(ceiling, max(int(b_cur), b_aug_raw, 1))
    res["b_req_ip"] = int(b_ip)
    res["b_req_aug"] = int(b_aug)
    res["switch_ip"] = switch_mode(int(b_ip), int(b_max), int(n_switch))
    res["switch_aug"] = switch_mode(int(b_aug), int(b_max), int(n_switch))
    return res


# --------------------------------------------------------------------------------------
# Inner step (Algorithm 3, the InnerOpt lines; Section 6.1 names AdamW, lr 4e-4, decay 0.1)
# --------------------------------------------------------------------------------------

def inner_step(theta, exp_avg, exp_avg_sq, grad, step: int, lr: float, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.1,
               grad_scale: float = 1.0) -> dict:
    """x_m <- InnerOpt(x_m, g) with InnerOpt = AdamW (decoupled weight decay), step = 1, 2, ...:
        g = grad_scale * grad            (grad is a sum over samples; 1/b gives eq. 1's g_k)
        x <- x - lr * weight_decay * x
        m <- beta1 m + (1 - beta1) g ;   v <- beta2 v + (1 - beta2) g^2
        x <- x - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
    fp64 arithmetic on the fp32 inputs, rounded to fp32 once.  beta1, beta2, eps are not given
    by the paper; the defaults are the customary ones."""
    x = widen(theta)
    m = widen(exp_avg)
    v = widen(exp_avg_sq)
    g = grad_scale * widen(grad)
    x = x - lr * weight_decay * x
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    x = x - lr * m_hat / (np.sqrt(v_hat) + eps)
    return dict(theta=x.astype(np.float32), exp_avg=m.astype(np.float32),
                exp_avg_sq=v.astype(np.float32), theta_f64=x, exp_avg_f64=m, exp_avg_sq_f64=v)


# --------------------------------------------------------------------------------------
# Outer step (Algorithm 3, pseudo-gradient and OuterOpt lines; worker reset line)
# --------------------------------------------------------------------------------------

def outer_step(theta_outer, thetas, momentum, lr: float, mu: float, nesterov: bool = True,
               broadcast: bool = False) -> dict:
    """Delta = (1/M) sum_m (x^{(t-1)} - x_m^{(t,H)});  x <- OuterOpt(x, Delta) with OuterOpt
    = SGD with (Nesterov) momentum:  buf <- mu*buf + Delta;  step = Delta + mu*buf (Nesterov)
    or buf (heavy ball);  x <- x - lr*step.  mu = 0 is plain SGD.  fp64 arithmetic on the
    fp32 inputs, rounded to fp32 once at the end.  broadcast: every instance is reset to the
    new outer parameters (start of the next round)."""
    x = widen(theta_outer)
    M = len(thetas)
    delta = np.zeros_like(x)
    for th in thetas:
        delta += x - widen(th)
    delta /= M
    buf = widen(momentum) if momentum is not None else np.zeros_like(x)
    buf = mu * buf + delta
    step = delta + mu * buf if nesterov else buf
    x_new = x - lr * step
    out = dict(theta_outer=x_new.astype(np.float32), momentum=buf.astype(np.float32),
               pseudo_grad=delta.astype(np.float32), theta_outer_f64=x_new,
               momentum_f64=buf, pseudo_grad_f64=delta)
    if broadcast:
        out["thetas"] = [x_new.astype(np.float32) for _ in range(M)]
    return out


# --------------------------------------------------------------------------------------
# The same outer step and merge with the instances' DRIFTS stored in bf16 (the quantity
# Algorithm 3 averages, x^{(t-1)} - x_m^{(t,H)}, is what travels; outer model and momentum
# stay fp32).  Halves the bytes an instance contributes; the drift, not the parameter,
# carries the rounding error: at most 2^-8 relative to the drift itself.
# --------------------------------------------------------------------------------------

def round_to_bf16_bits(x32) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even, written out on the bit
    pattern: keep the upper 16 bits, add one if the dropped half is above one half, or exactly one
    half and the kept part is odd.  NaN stays NaN (quiet bit set)."""
    u = np.ascontiguousarray(np.asarray(x32, dtype=np.float32)).view(np.uint32)
    upper = u >> np.uint32(16)
    lower = u & np.uint32(0xFFFF)
    up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    out = (upper + up.astype(np.uint32)).astype(np.uint32)
    nan = np.isnan(np.asarray(x32, dtype=np.float32))
    out = np.where(nan, upper | np.uint32(0x40), out)
    return out.astype(np.uint16)


def pack_drift(theta_outer, theta_m) -> np.ndarray:
    """d_m = x^{(t-1)} - x_m^{(t,H)} (Algorithm 3, the summand of Delta) as stored: the fp32
    difference of the two fp32 vectors, rounded to bf16.  Both roundings are the format's own
    (IEEE fp32 subtraction, then nearest-even to 8 significant bits): the stored code is decided in
    fp32 on both sides of a comparison."""
    a = np.asarray(theta_outer, dtype=np.float32)
    b = np.asarray(theta_m, dtype=np.float32)
    return round_to_bf16_bits(a - b)


def outer_step_drift(theta_outer, drift_bits, momentum, lr: float, mu: float, nesterov: bool = True,
                     broadcast: bool = False) -> dict:
    """Algorithm 3's Delta and OuterOpt from stored drifts: Delta = (1/M) sum_m d_m with d_m the
    bf16 values as stored (widened exactly), then the update of outer_step, fp64, rounded once.
    broadcast: the worker reset x_m <- x leaves every drift at zero."""
    x = widen(theta_outer)
    M = len(drift_bits)
    delta = np.zeros_like(x)
    for d in drift_bits:
        delta += widen(np.asarray(d, dtype=np.uint16))
    delta /= M
    buf = widen(momentum) if momentum is not None else np.zeros_like(x)
    buf = mu * buf + delta
    step = delta + mu * buf if nesterov else buf
    x_new = x - lr * step
    out = dict(theta_outer=x_new.astype(np.float32), momentum=buf.astype(np.float32),
               pseudo_grad=delta.astype(np.float32), theta_outer_f64=x_new, momentum_f64=buf,
               pseudo_grad_f64=delta)
    if broadcast:
        out["drifts"] = [np.zeros(x.shape, dtype=np.uint16) for _ in range(M)]
    return out


def merge_drift(x_rep, drift_bits, w_rep: float, w_others) -> dict:
    """DoMerge (Algorithm 2) when the other trainers are known by their stored drifts from the
    representative, d_j = x_r - x_j (bf16): x_merge = sum_j b_j x_j / sum_j b_j = x_r - sum_{j != r}
    b_j d_j / sum_j b_j, fp64, rounded once."""
    x = widen(x_rep)
    wsum = float(w_rep) + float(sum(float(w) for w in w_others))
    s = np.zeros_like(x)
    for d, w in zip(drift_bits, w_others):
        s += float(w) * widen(np.asarray(d, dtype=np.uint16))
    xm = x - s / wsum
    return dict(x_merge=xm.astype(np.float32), x_merge_f64=xm)


# --------------------------------------------------------------------------------------
# Trainer merge (Section 4.1.1; Algorithms 1 and 2)
# --------------------------------------------------------------------------------------

def check_merge(b_req, w: int):
    """CheckMerge (Algorithm 1): nothing when w = 0 or at most one trainer; otherwise the w
    trainers with the smallest requested batch when w <= k, else nothing.  Ties keep the
    lower index first (stable sort)."""
    k = len(b_req)
    if w == 0 or k <= 1:
        return []
    order = sorted(range(k), key=lambda i: b_req[i])
    if w <= k:
        return order[:w]
    return []


def merge(xs, weights, rep: int = -1) -> dict:
    """DoMerge (Algorithm 2): x_merge = sum_j b_j x_j / sum_j b_j; the representative
    r = argmax b_j (lowest index on ties) receives x_merge; the others are left as they are
    (the caller drops them)."""
    S = len(xs)
    assert S == len(weights) and S >= 1
    w = np.asarray(weights, dtype=np.float64)
    wsum = float(w.sum())
    acc = np.zeros_like(widen(xs[0]))
    for j in range(S):
        acc += w[j] * widen(xs[j])
    acc /= wsum
    if rep < 0:
        rep = int(np.argmax(w))        # first maximal element
    return dict(rep=rep, x_merge=acc.astype(np.float32), x_merge_f64=acc)


# --------------------------------------------------------------------------------------
# One outer step of Algorithm 3 for k trainers (host loop; the model is a callback)
# --------------------------------------------------------------------------------------

def round_step(trainers, cfg: dict, batch_fn) -> list:
    """Algorithm 3, one outer step t, in the listing's order.

    trainers: list of dicts {theta_outer [N], momentum [N], b_req, uid, workers: [{theta, exp_avg,
    exp_avg_sq, step}]} (numpy fp32 vectors); modified in place; merged-away trainers are
    removed from the list.  cfg: T-independent scalars {inner_steps, b_max, n_switch, b_cap, eta,
    merge_w, lr_inner, beta1, beta2, eps, weight_decay, lr_outer, mu_outer, nesterov}.
    batch_fn(uid, worker, inner_step, micro_step, b, theta) -> list of blocks in grad_stats'
    entry format (linear weights and vectors only), b samples each.
    The flat parameter vector is the concatenation of the blocks in list order (a linear weight
    row-major [d_out, d_in]).  Readings as in the design notes: the switch decision is per trainer,
    the accumulate branch runs the same number of inner steps, each over its accumulated
    micro-batches, and the norm test runs on the first inner step's batch of worker 0 with b_cur =
    the samples that batch held; the next request is never below the previous one.
    Returns one report dict per remaining trainer."""
    # CheckMerge / DoMerge (Algorithms 1 and 2)
    if len(trainers) > 1 and cfg["merge_w"] > 0:
        sel = check_merge([t["b_req"] for t in trainers], cfg["merge_w"])
        if sel:
            mg = merge([trainers[j]["theta_outer"] for j in sel], [trainers[j]["b_req"] for j in sel])
            keep = sel[mg["rep"]]
            trainers[keep]["theta_outer"] = mg["x_merge"]
            trainers[keep]["merged_from"] = len(sel) - 1
            for j in sorted((j for j in sel if j != keep), reverse=True):
                del trainers[j]
    reports = []
    for t in trainers:
        sm = switch_mode(int(t["b_req"]), cfg["b_max"], cfg["n_switch"])
        rep = dict(b_req_used=int(t["b_req"]), merged_from=t.pop("merged_from", 0), **sm)
        b_next = t["b_req"]
        for m, w in enumerate(t["workers"]):
            w["theta"] = np.array(t["theta_outer"], dtype=np.float32, copy=True)
            for h in range(cfg["inner_steps"]):
                micro = [batch_fn(t["uid"], m, h, s, sm["b_micro"], w["theta"])
                         for s in range(sm["accum_steps"])]
                blocks = concat_micro_batches(micro)
                st = grad_stats(blocks, two_pass=False)
                if m == 0 and h == 0:
                    # eq. 4 compares with the size of the batch the statistics come from, which
                    # SwitchMode may have cut to b_max (Section 4.2); the previous request stays
                    # the floor of the next one (b_{k+1} >= b_k)
                    nt = norm_test(st["S1"], st["S2"], st["B"], cfg["eta"], int(st["B"]), cfg["b_max"],
                                   cfg["n_switch"], cfg["b_cap"])
                    rep["test"] = nt
                    b_next = max(int(t["b_req"]), int(nt["b_req"]))
                g = np.concatenate([np.asarray(G).reshape(-1) for G in st["G"]])
                w["step"] += 1
                o = inner_step(w["theta"], w["exp_avg"], w["exp_avg_sq"], g, w["step"], cfg["lr_inner"],
                               cfg["beta1"], cfg["beta2"], cfg["eps"], cfg["weight_decay"],
                               grad_scale=1.0 / (sm["accum_steps"] * sm["b_micro"]))
                w["theta"], w["exp_avg"], w["exp_avg_sq"] = o["theta"], o["exp_avg"], o["exp_avg_sq"]
        t["b_req"] = b_next
        reports.append(rep)
    for t in trainers:
        o = outer_step(t["theta_outer"], [w["theta"] for w in t["workers"]], t["momentum"],
                       cfg["lr_outer"], cfg["mu_outer"], bool(cfg["nesterov"]))
        t["theta_outer"], t["momentum"] = o["theta_outer"], o["momentum"]
    return reports
