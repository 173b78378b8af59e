"""ctypes binding of libadloco.so: argument marshalling only.

Function names and argument order follow include/adloco.h.  Tensors are torch tensors on
the GPU (PyTorch-ROCm owns device memory and streams); nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("ADLOCO_LIBRARY_PATH") or os.path.join(_PKG, "libadloco.so")

ADLOCO_F32, ADLOCO_BF16, ADLOCO_F16 = 0, 1, 2
ADLOCO_ACCUMULATE = 0x1
ADLOCO_SUM_ONLY = 0x2
ADLOCO_GRAD_PROVIDED = 0x1
ADLOCO_KIND_LINEAR, ADLOCO_KIND_VECTOR, ADLOCO_KIND_EMBED = 0x00, 0x10, 0x20
ADLOCO_BROADCAST = 0x1
ADLOCO_BIASED_VAR = 0x1
ADLOCO_ALLOW_SHRINK = 0x2
ADLOCO_MAX_INSTANCES = 16

_ERR_NAMES = {1: "ADLOCO_EINVAL", 2: "ADLOCO_EUNSUPPORTED", 3: "ADLOCO_ENOMEM", 4: "ADLOCO_EHIP",
              5: "ADLOCO_ESTATE"}


class AdlocoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


class LinearDesc(C.Structure):
    _fields_ = [("a", C.c_void_p), ("delta", C.c_void_p), ("d_in", C.c_int32),
                ("d_out", C.c_int32), ("a_row_stride", C.c_int64),
                ("delta_row_stride", C.c_int64), ("grad_sum", C.c_void_p),
                ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class StatsAcc(C.Structure):
    _fields_ = [("sum_sample_sqnorm", C.c_double), ("n_samples", C.c_int64)]


class NormTestResult(C.Structure):
    _fields_ = [("S1", C.c_double), ("S2", C.c_double), ("batch_grad_sqnorm", C.c_double),
                ("variance", C.c_double), ("stat", C.c_double), ("n_samples", C.c_int64),
                ("b_cur", C.c_int64), ("b_req", C.c_int64), ("b_micro", C.c_int64),
                ("accum_steps", C.c_int64), ("test_passed", C.c_int32),
                ("accumulate", C.c_int32), ("stat_undefined", C.c_int32),
                ("reserved", C.c_int32)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_}


class IpAcc(C.Structure):
    _fields_ = [("sum_ip", C.c_double), ("sum_ip_sq", C.c_double), ("n_samples", C.c_int64),
                ("reserved", C.c_int64)]


class IpTestResult(C.Structure):
    _fields_ = [("S1", C.c_double), ("S2", C.c_double), ("batch_grad_sqnorm", C.c_double),
                ("var_ip", C.c_double), ("stat_ip", C.c_double), ("var_aug", C.c_double),
                ("stat_aug", C.c_double), ("n_samples", C.c_int64), ("b_cur", C.c_int64),
                ("b_req_ip", C.c_int64), ("b_req_aug", C.c_int64), ("b_micro_ip", C.c_int64),
                ("accum_steps_ip", C.c_int64), ("b_micro_aug", C.c_int64),
                ("accum_steps_aug", C.c_int64), ("accumulate_ip", C.c_int32),
                ("accumulate_aug", C.c_int32), ("stat_undefined", C.c_int32),
                ("reserved", C.c_int32)]

    def as_dict(self) -> dict:
        return {k: getattr(self, k) for k, _ in self._fields_}


class Worker(C.Structure):
    _fields_ = [("theta", C.c_void_p), ("exp_avg", C.c_void_p), ("exp_avg_sq", C.c_void_p),
                ("grad", C.c_void_p), ("step", C.c_int64)]


class Trainer(C.Structure):
    _fields_ = [("theta_outer", C.c_void_p), ("momentum", C.c_void_p), ("workers", C.POINTER(Worker)),
                ("n_workers", C.c_int32), ("reserved", C.c_int32), ("b_req", C.c_int64),
                ("acc", C.c_void_p), ("per_sample_sqnorm", C.c_void_p), ("user", C.c_void_p)]


class RoundConfig(C.Structure):
    _fields_ = [("T", C.c_int32), ("dtype", C.c_int32), ("inner_steps", C.c_int32),
                ("n_switch", C.c_int32), ("merge_w", C.c_int32), ("nesterov", C.c_int32),
                ("b_max", C.c_int64), ("b_cap", C.c_int64), ("eta", C.c_double),
                ("lr_inner", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("lr_outer", C.c_double),
                ("mu_outer", C.c_double)]


class RoundReport(C.Structure):
    _fields_ = [("b_req_used", C.c_int64), ("b_micro", C.c_int64), ("accum_steps", C.c_int64),
                ("accumulate", C.c_int32), ("merged_from", C.c_int32), ("test", NormTestResult)]


BATCH_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_void_p,
                       C.POINTER(LinearDesc), C.c_int32, C.c_void_p)

_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libadloco.so; there is no fallback path: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2508_18182_amd.build` "
            "(or __graft_entry__.build()); the HIP library is the only implementation")
    # PyTorch ships its own HIP runtime (same soname as the system one).  It has to be the one
    # already loaded when libadloco.so resolves libamdhip64, otherwise the process ends up with
    # two runtimes and the second one to initialise sees no GPU.
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, u32, dbl, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_double, C.c_size_t
    lib.adloco_version.restype = C.c_int
    lib.adloco_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.adloco_destroy.argtypes = [vp]
    lib.adloco_last_error.argtypes = [vp]
    lib.adloco_last_error.restype = C.c_char_p
    lib.adloco_set_tuning.argtypes = [vp, C.c_char_p, C.c_int]
    lib.adloco_profile_read.argtypes = [vp, C.c_char_p, C.POINTER(dbl), C.POINTER(C.c_int)]
    lib.adloco_profile_read.restype = C.c_int
    lib.adloco_table_builds.argtypes = [vp]
    lib.adloco_probe_mfma_lds.argtypes = [vp, C.c_int, C.c_int, C.POINTER(dbl), C.POINTER(dbl)]
    lib.adloco_probe_mfma_lds.restype = C.c_int
    lib.adloco_table_builds.restype = C.c_int
    lib.adloco_grad_stats.argtypes = [vp, C.POINTER(LinearDesc), C.c_int, C.c_int, C.c_int, C.c_int,
                                      vp, vp, vp, u32, vp]
    lib.adloco_norm_test.argtypes = [vp, C.POINTER(LinearDesc), C.c_int, vp, dbl, i64, i64, i32,
                                     i64, u32, C.POINTER(NormTestResult), vp]
    lib.adloco_norm_test_noalloc.argtypes = lib.adloco_norm_test.argtypes
    lib.adloco_norm_test_decide.argtypes = [dbl, dbl, i64, dbl, i64, i64, i32, i64, u32,
                                            C.POINTER(NormTestResult)]
    lib.adloco_switch_mode.argtypes = [i64, i64, i32, C.POINTER(i32), C.POINTER(i64),
                                       C.POINTER(i64)]
    lib.adloco_outer_step.argtypes = [vp, vp, C.POINTER(vp), C.c_int, sz, vp, dbl, dbl,
                                      C.c_int, u32, vp, vp]
    lib.adloco_merge.argtypes = [vp, C.POINTER(vp), C.POINTER(dbl), C.c_int, sz, C.c_int,
                                 C.POINTER(C.c_int), vp]
    lib.adloco_inner_step.argtypes = [vp, vp, vp, vp, vp, sz, dbl, dbl, dbl, dbl, dbl, dbl, i64, vp]
    lib.adloco_pack_drift.argtypes = [vp, vp, vp, vp, sz, vp]
    lib.adloco_outer_step_drift.argtypes = [vp, vp, C.POINTER(vp), C.c_int, sz, vp, dbl, dbl, C.c_int, u32, vp, vp]
    lib.adloco_merge_drift.argtypes = [vp, vp, C.POINTER(vp), dbl, C.POINTER(dbl), C.c_int, sz, vp]
    lib.adloco_round.argtypes = [vp, C.POINTER(RoundConfig), C.POINTER(Trainer), C.POINTER(C.c_int),
                                 C.POINTER(LinearDesc), C.c_int, sz, BATCH_FN, C.POINTER(RoundReport), vp]
    lib.adloco_inner_products.argtypes = [vp, C.POINTER(LinearDesc), C.c_int, C.c_int, C.c_int,
                                          C.c_int, vp, vp, vp, u32, vp]
    lib.adloco_inner_product_test.argtypes = [vp, C.POINTER(LinearDesc), C.c_int, vp, vp, dbl, dbl,
                                              i64, i64, i32, i64, C.POINTER(IpTestResult), vp]
    lib.adloco_inner_product_decide.argtypes = [dbl, dbl, dbl, dbl, i64, dbl, dbl, i64, i64, i32,
                                                i64, C.POINTER(IpTestResult)]
    lib.adloco_check_merge.argtypes = [C.POINTER(i64), C.c_int, C.c_int, C.POINTER(C.c_int),
                                       C.POINTER(C.c_int)]
    for name in ("adloco_create", "adloco_destroy", "adloco_set_tuning", "adloco_grad_stats",
                 "adloco_norm_test", "adloco_norm_test_noalloc", "adloco_norm_test_decide", "adloco_switch_mode",
                 "adloco_outer_step", "adloco_merge", "adloco_check_merge", "adloco_inner_step", "adloco_round",
                 "adloco_inner_products", "adloco_inner_product_test", "adloco_inner_product_decide",
                 "adloco_pack_drift", "adloco_outer_step_drift", "adloco_merge_drift"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def adloco_version() -> int:
    return load_library().adloco_version()


class Context:
    """Owner of an adloco_ctx (scratch memory on one device)."""

    def __init__(self, device: int = 0):
        lib = load_library()
        h = C.c_void_p()
        rc = lib.adloco_create(C.byref(h), int(device))
        if rc != 0:
            raise AdlocoError(rc, lib.adloco_last_error(None).decode())
        self._h = h
        self.device = int(device)

    def close(self):
        if getattr(self, "_h", None):
            load_library().adloco_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def set_tuning(self, name: str, value: int):
        self._check(load_library().adloco_set_tuning(self._h, name.encode(), int(value)))

    def table_builds(self) -> int:
        """Number of times this context has (re)built its shape-dependent tables (measurement aid)."""
        return int(load_library().adloco_table_builds(self._h))

    def probe_mfma_lds(self, variant: int, ksteps: int = 4096):
        """(ms, flops) of the LDS-fed MFMA loop (measurement aid, see adloco_internal.h)."""
        ms, fl = C.c_double(), C.c_double()
        self._check(load_library().adloco_probe_mfma_lds(self._h, variant, ksteps, C.byref(ms), C.byref(fl)))
        return ms.value, fl.value

    def profile_read(self, kernel: str):
        """(total milliseconds, launches) of the named kernel since the last read."""
        ms, n = C.c_double(0.0), C.c_int(0)
        self._check(load_library().adloco_profile_read(self._h, kernel.encode(), C.byref(ms),
                                                       C.byref(n)))
        return ms.value, n.value

    def _check(self, rc: int):
        if rc != 0:
            raise AdlocoError(rc, load_library().adloco_last_error(self._h).decode())


def _stream_ptr(stream) -> C.c_void_p:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dev_ptr(t, dtype=None, numel=None, name="tensor") -> C.c_void_p:
    """Device address of a contiguous CUDA/HIP tensor after shape and dtype checks."""
    if t is None:
        return C.c_void_p(None)
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} has {t.numel()} elements, needs {numel}")
    return C.c_void_p(t.data_ptr())


def make_layer_descs(layers: Sequence[dict], B: int, T: int, dtype: int):
    """layers: dicts with a [B,T,d_in], delta [B,T,d_out], optional grad_sum [d_out,d_in] fp32,
    optional provided=True.  Token rows may be strided views (last dim contiguous).
    kind="vector": a bias / gain block, delta [B,T,d], optional x [B,T,d], grad_sum [d].
    kind="embed": an embedding table, ids int32 [B,T], delta [B,T,d], vocab=V, grad_sum [V,d]
    (maintained by the caller)."""
    import torch
    tdt = {ADLOCO_BF16: torch.bfloat16, ADLOCO_F16: torch.float16}.get(dtype, torch.float32)
    arr = (LinearDesc * len(layers))()

    def check_rows(i, nm, t):
        if not t.is_cuda or t.dtype != tdt or t.dim() != 3 or t.shape[0] != B or t.shape[1] != T:
            raise ValueError(f"layer {i}: {nm} must be a GPU {tdt} tensor [B={B},T={T},d], got "
                             f"{tuple(t.shape)} {t.dtype}")
        if t.stride(2) != 1 or t.stride(0) != T * t.stride(1):
            raise ValueError(f"layer {i}: {nm} needs unit stride in d and samples T rows apart")

    for i, l in enumerate(layers):
        kind = l.get("kind", "linear")
        d = l["delta"]
        check_rows(i, "delta", d)
        g = l.get("grad_sum")
        flags = ADLOCO_GRAD_PROVIDED if l.get("provided") else 0
        if kind == "linear":
            a = l["a"]
            check_rows(i, "a", a)
            a_ptr, a_stride, d_in, gshape = a.data_ptr(), a.stride(1), a.shape[2], (d.shape[2], a.shape[2])
        elif kind == "vector":
            x = l.get("x")
            if x is not None:
                check_rows(i, "x", x)
                if x.shape[2] != d.shape[2]:
                    raise ValueError(f"layer {i}: x and delta differ in width")
            a_ptr, a_stride = (x.data_ptr(), x.stride(1)) if x is not None else (None, 0)
            d_in, gshape = 1, (d.shape[2],)
            flags |= ADLOCO_KIND_VECTOR
        elif kind == "embed":
            ids = l["ids"]
            if (not ids.is_cuda or ids.dtype != torch.int32 or not ids.is_contiguous()
                    or tuple(ids.shape) != (B, T)):
                raise ValueError(f"layer {i}: ids must be a contiguous GPU int32 tensor [B, T]")
            a_ptr, a_stride, d_in, gshape = ids.data_ptr(), 0, int(l["vocab"]), (int(l["vocab"]), d.shape[2])
            flags |= ADLOCO_KIND_EMBED | ADLOCO_GRAD_PROVIDED
        else:
            raise ValueError(f"layer {i}: unknown kind {kind!r}")
        if g is not None:
            if (not g.is_cuda or g.dtype != torch.float32 or not g.is_contiguous()
                    or tuple(g.shape) != gshape):
                raise ValueError(f"layer {i}: grad_sum must be contiguous fp32 {gshape} on the GPU")
        arr[i].a = a_ptr
        arr[i].delta = d.data_ptr()
        arr[i].d_in = d_in
        arr[i].d_out = d.shape[2]
        arr[i].a_row_stride = a_stride
        arr[i].delta_row_stride = d.stride(1)
        arr[i].grad_sum = g.data_ptr() if g is not None else None
        arr[i].flags = flags
        arr[i].reserved = 0
    return arr


def adloco_grad_stats(ctx: Context, layers: Sequence[dict], B: int, T: int, dtype: int,
                      per_sample_sqnorm, per_layer_sample_sqnorm, acc, flags: int = 0,
                      stream=None, descs=None):
    """acc: GPU tensor of 16 bytes (e.g. torch.zeros(2, dtype=torch.float64)) holding an
    adloco_stats_acc.  descs: a LinearDesc array from make_layer_descs to skip re-marshalling."""
    import torch
    arr = descs if descs is not None else make_layer_descs(layers, B, T, dtype)
    n = len(arr)
    ps = _dev_ptr(per_sample_sqnorm, torch.float32, B, "per_sample_sqnorm")
    pl = _dev_ptr(per_layer_sample_sqnorm, torch.float32, n * B, "per_layer_sample_sqnorm")
    if acc is None and (flags & ADLOCO_SUM_ONLY):
        acc_ptr = C.c_void_p(None)
    elif acc is None or not acc.is_cuda or acc.numel() * acc.element_size() < 16:
        raise ValueError("acc must be a GPU tensor of at least 16 bytes")
    else:
        acc_ptr = C.c_void_p(acc.data_ptr())
    ctx._check(load_library().adloco_grad_stats(ctx._h, arr, n, B, T, dtype, ps, pl, acc_ptr, flags,
                                                _stream_ptr(stream)))


def _grad_sum_descs(layers):
    """Descriptors that carry only grad_sum, its shape and the block kind."""
    arr = (LinearDesc * len(layers))()
    for i, l in enumerate(layers):
        g = l["grad_sum"]
        _dev_ptr(g, None, None, f"layer {i} grad_sum")
        arr[i].grad_sum = g.data_ptr()
        kind = l.get("kind", "linear")
        if kind == "vector":
            arr[i].d_out, arr[i].d_in = g.shape[0], 1
            arr[i].flags = ADLOCO_KIND_VECTOR | (ADLOCO_GRAD_PROVIDED if l.get("provided") else 0)
        elif kind == "embed":
            arr[i].d_in, arr[i].d_out = g.shape
            arr[i].flags = ADLOCO_KIND_EMBED | ADLOCO_GRAD_PROVIDED
        else:
            arr[i].d_out, arr[i].d_in = g.shape
            arr[i].flags = ADLOCO_GRAD_PROVIDED if l.get("provided") else 0
    return arr


def adloco_inner_products(ctx: Context, layers: Sequence[dict], B: int, T: int, dtype: int,
                          per_sample_ip, per_sample_sqnorm, acc, flags: int = 0, stream=None,
                          descs=None):
    """c_i = <g_i, G> of one micro-batch against the (complete) grad_sum buffers.  acc: GPU tensor
    of 32 bytes (e.g. torch.zeros(4, dtype=torch.float64)) holding an adloco_ip_acc."""
    import torch
    arr = descs if descs is not None else make_layer_descs(layers, B, T, dtype)
    ip = _dev_ptr(per_sample_ip, torch.float32, B, "per_sample_ip")
    sq = _dev_ptr(per_sample_sqnorm, torch.float32, B, "per_sample_sqnorm")
    if acc is None or not acc.is_cuda or acc.numel() * acc.element_size() < 32:
        raise ValueError("acc must be a GPU tensor of at least 32 bytes")
    ctx._check(load_library().adloco_inner_products(ctx._h, arr, len(arr), B, T, dtype, ip, sq,
                                                    C.c_void_p(acc.data_ptr()), flags,
                                                    _stream_ptr(stream)))


def adloco_inner_product_test(ctx: Context, layers, acc, ip_acc, vartheta: float, nu: float,
                              b_cur: int, b_max: int, n_switch: int = 2, b_cap: int = 0,
                              stream=None, descs=None) -> dict:
    arr = descs if descs is not None else _grad_sum_descs(layers)
    res = IpTestResult()
    ctx._check(load_library().adloco_inner_product_test(
        ctx._h, arr, len(arr), C.c_void_p(acc.data_ptr()), C.c_void_p(ip_acc.data_ptr()), vartheta,
        nu, b_cur, b_max, n_switch, b_cap, C.byref(res), _stream_ptr(stream)))
    return res.as_dict()


def adloco_inner_product_decide(S1: float, S2: float, sum_ip: float, sum_ip_sq: float,
                                n_samples: int, vartheta: float, nu: float, b_cur: int, b_max: int,
                                n_switch: int = 2, b_cap: int = 0) -> dict:
    res = IpTestResult()
    rc = load_library().adloco_inner_product_decide(S1, S2, sum_ip, sum_ip_sq, n_samples, vartheta,
                                                    nu, b_cur, b_max, n_switch, b_cap, C.byref(res))
    if rc != 0:
        raise AdlocoError(rc, "adloco_inner_product_decide rejected its arguments")
    return res.as_dict()


def adloco_norm_test(ctx: Context, layers, acc, eta: float, b_cur: int, b_max: int,
                     n_switch: int = 2, b_cap: int = 0, flags: int = 0, stream=None,
                     descs=None) -> dict:
    """layers: dicts with grad_sum (and d_in/d_out taken from its shape), or descs."""
    arr = descs if descs is not None else _grad_sum_descs(layers)
    res = NormTestResult()
    ctx._check(load_library().adloco_norm_test(ctx._h, arr, len(arr), C.c_void_p(acc.data_ptr()),
                                               eta, b_cur, b_max, n_switch, b_cap, flags,
                                               C.byref(res), _stream_ptr(stream)))
    return res.as_dict()


def adloco_norm_test_noalloc(ctx: Context, layers, acc, eta: float, b_cur: int, b_max: int,
                             n_switch: int = 2, b_cap: int = 0, flags: int = 0, stream=None,
                             descs=None) -> dict:
    """adloco_norm_test through the entry point that allocates nothing (fixed device array)."""
    arr = descs if descs is not None else _grad_sum_descs(layers)
    res = NormTestResult()
    ctx._check(load_library().adloco_norm_test_noalloc(ctx._h, arr, len(arr), C.c_void_p(acc.data_ptr()),
                                                       eta, b_cur, b_max, n_switch, b_cap, flags,
                                                       C.byref(res), _stream_ptr(stream)))
    return res.as_dict()


def adloco_norm_test_decide(S1: float, S2: float, n_samples: int, eta: float, b_cur: int,
                            b_max: int, n_switch: int = 2, b_cap: int = 0, flags: int = 0) -> dict:
    res = NormTestResult()
    rc = load_library().adloco_norm_test_decide(S1, S2, n_samples, eta, b_cur, b_max, n_switch,
                                                b_cap, flags, C.byref(res))
    if rc != 0:
        raise AdlocoError(rc, "adloco_norm_test_decide rejected its arguments")
    return res.as_dict()


def adloco_switch_mode(b_req: int, b_max: int, n_switch: int = 2) -> dict:
    acc, steps, micro = C.c_int32(), C.c_int64(), C.c_int64()
    rc = load_library().adloco_switch_mode(b_req, b_max, n_switch, C.byref(acc), C.byref(steps),
                                           C.byref(micro))
    if rc != 0:
        raise AdlocoError(rc, "adloco_switch_mode rejected its arguments")
    return dict(accumulate=acc.value, accum_steps=steps.value, b_micro=micro.value)


def _ptr_array(tensors, N: int, name: str):
    import torch
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _dev_ptr(t, torch.float32, N, f"{name}[{i}]").value
    return arr


def adloco_outer_step(ctx: Context, theta_outer, theta_inst, momentum, lr: float, mu: float,
                      nesterov: bool = True, flags: int = 0, pseudo_grad_out=None, stream=None,
                      N: Optional[int] = None):
    import torch
    N = theta_outer.numel() if N is None else N
    th = _dev_ptr(theta_outer, torch.float32, N, "theta_outer")
    mom = _dev_ptr(momentum, torch.float32, N, "momentum")
    pg = _dev_ptr(pseudo_grad_out, torch.float32, N, "pseudo_grad_out")
    arr = _ptr_array(theta_inst, N, "theta_inst")
    ctx._check(load_library().adloco_outer_step(ctx._h, th, arr, len(theta_inst), N, mom, lr, mu,
                                                1 if nesterov else 0, flags, pg,
                                                _stream_ptr(stream)))


def adloco_inner_step(ctx: Context, theta, exp_avg, exp_avg_sq, grad, step: int, lr: float,
                      beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                      weight_decay: float = 0.1, grad_scale: float = 1.0, stream=None,
                      N: Optional[int] = None):
    import torch
    N = theta.numel() if N is None else N
    ptrs = [_dev_ptr(t, torch.float32, N, nm) for nm, t in
            (("theta", theta), ("exp_avg", exp_avg), ("exp_avg_sq", exp_avg_sq), ("grad", grad))]
    ctx._check(load_library().adloco_inner_step(ctx._h, *ptrs, N, grad_scale, lr, beta1, beta2, eps,
                                                weight_decay, int(step), _stream_ptr(stream)))


def adloco_merge(ctx: Context, x, weights, rep: int = -1, stream=None,
                 N: Optional[int] = None) -> int:
    N = x[0].numel() if N is None else N
    arr = _ptr_array(x, N, "x")
    w = (C.c_double * len(weights))(*[float(v) for v in weights])
    if len(weights) != len(x):
        raise ValueError("one weight per vector")
    r = C.c_int(-1)
    ctx._check(load_library().adloco_merge(ctx._h, arr, w, len(x), N, rep, C.byref(r),
                                           _stream_ptr(stream)))
    return r.value


def _bf16_ptr(t, N, name):
    """Device address of a contiguous bf16 (or int16 / uint16 bit pattern) tensor of >= N elements."""
    import torch
    if t is None or not t.is_cuda or t.dtype not in (torch.bfloat16, torch.int16, torch.uint16):
        raise TypeError(f"{name} must be a GPU bf16 tensor")
    if not t.is_contiguous() or t.numel() < N:
        raise ValueError(f"{name} must be contiguous with at least {N} elements")
    return C.c_void_p(t.data_ptr())


def adloco_pack_drift(ctx: Context, theta_outer, theta_m, drift_out, stream=None, N: Optional[int] = None):
    """drift_out (bf16 [N]) = bf16(theta_outer - theta_m)."""
    import torch
    N = theta_outer.numel() if N is None else N
    ctx._check(load_library().adloco_pack_drift(
        ctx._h, _dev_ptr(theta_outer, torch.float32, N, "theta_outer"),
        _dev_ptr(theta_m, torch.float32, N, "theta_m"), _bf16_ptr(drift_out, N, "drift_out"), N,
        _stream_ptr(stream)))


def adloco_outer_step_drift(ctx: Context, theta_outer, drifts, momentum, lr: float, mu: float,
                            nesterov: bool = True, flags: int = 0, pseudo_grad_out=None, stream=None,
                            N: Optional[int] = None):
    """adloco_outer_step on M instance drifts stored in bf16."""
    import torch
    N = theta_outer.numel() if N is None else N
    arr = (C.c_void_p * len(drifts))()
    for i, t in enumerate(drifts):
        arr[i] = _bf16_ptr(t, N, f"drifts[{i}]").value
    ctx._check(load_library().adloco_outer_step_drift(
        ctx._h, _dev_ptr(theta_outer, torch.float32, N, "theta_outer"), arr, len(drifts), N,
        _dev_ptr(momentum, torch.float32, N, "momentum"), lr, mu, 1 if nesterov else 0, flags,
        _dev_ptr(pseudo_grad_out, torch.float32, N, "pseudo_grad_out"), _stream_ptr(stream)))


def adloco_merge_drift(ctx: Context, x_rep, drifts, w_rep: float, w_others, stream=None,
                       N: Optional[int] = None):
    """x_rep <- x_rep - sum_j w_j d_j / (w_rep + sum_j w_j), d_j bf16 drifts of the other trainers."""
    import torch
    N = x_rep.numel() if N is None else N
    if len(w_others) != len(drifts):
        raise ValueError("one weight per drift")
    arr = (C.c_void_p * max(len(drifts), 1))()
    for i, t in enumerate(drifts):
        arr[i] = _bf16_ptr(t, N, f"drifts[{i}]").value
    w = (C.c_double * max(len(w_others), 1))(*[float(v) for v in w_others])
    ctx._check(load_library().adloco_merge_drift(ctx._h, _dev_ptr(x_rep, torch.float32, N, "x_rep"), arr,
                                                 float(w_rep), w, len(drifts), N, _stream_ptr(stream)))


def adloco_check_merge(b_req: Sequence[int], w: int):
    k = len(b_req)
    arr = (C.c_int64 * max(k, 1))(*[int(v) for v in b_req])
    sel = (C.c_int * max(w, 1))()
    n = C.c_int(0)
    rc = load_library().adloco_check_merge(arr, k, w, sel, C.byref(n))
    if rc != 0:
        raise AdlocoError(rc, "adloco_check_merge rejected its arguments")
    return [sel[i] for i in range(n.value)]


def adloco_round(ctx: Context, cfg: dict, trainers: Sequence[dict], blocks: Sequence[dict], batch_fn,
                 stream=None):
    """One outer step of Algorithm 3 (include/adloco.h: adloco_round).

    trainers: dicts {theta_outer, momentum, b_req, acc, per_sample_sqnorm, uid, workers: [{theta,
    exp_avg, exp_avg_sq, grad, step}]} of GPU tensors; updated in place (b_req, step); the list is
    reordered / shortened like the C array when trainers merge.
    blocks: template of the parameter blocks: dicts {d_in, d_out, kind ("linear" | "vector")}.
    batch_fn(uid, worker, inner_step, micro_step, b, theta_ptr) -> list of dicts {a | x, delta}
    (GPU tensors [b, T, .]) in block order; the tensors are kept alive until the round returns.
    Returns the reports of the remaining trainers."""
    import torch
    lib = load_library()
    n_layers = len(blocks)
    tmpl = (LinearDesc * n_layers)()
    N = 0
    for l, b in enumerate(blocks):
        kind = b.get("kind", "linear")
        tmpl[l].d_in = 1 if kind == "vector" else b["d_in"]
        tmpl[l].d_out = b["d_out"]
        tmpl[l].flags = ADLOCO_KIND_VECTOR if kind == "vector" else 0
        N += tmpl[l].d_in * tmpl[l].d_out
    k = len(trainers)
    arr = (Trainer * k)()
    worker_arrays = []
    for i, t in enumerate(trainers):
        wa = (Worker * len(t["workers"]))()
        for m, w in enumerate(t["workers"]):
            wa[m].theta = _dev_ptr(w["theta"], torch.float32, N, "worker theta").value
            wa[m].exp_avg = _dev_ptr(w["exp_avg"], torch.float32, N, "exp_avg").value
            wa[m].exp_avg_sq = _dev_ptr(w["exp_avg_sq"], torch.float32, N, "exp_avg_sq").value
            wa[m].grad = _dev_ptr(w["grad"], torch.float32, N, "grad").value
            wa[m].step = int(w["step"])
        worker_arrays.append(wa)
        arr[i].theta_outer = _dev_ptr(t["theta_outer"], torch.float32, N, "theta_outer").value
        arr[i].momentum = _dev_ptr(t["momentum"], torch.float32, N, "momentum").value
        arr[i].workers = wa
        arr[i].n_workers = len(t["workers"])
        arr[i].b_req = int(t["b_req"])
        arr[i].acc = t["acc"].data_ptr()
        arr[i].per_sample_sqnorm = t["per_sample_sqnorm"].data_ptr()
        arr[i].user = i
    c = RoundConfig()
    for name, _ in RoundConfig._fields_:
        setattr(c, name, cfg[name])
    keep_alive = []
    errors = []

    def trampoline(user, worker, inner_step, micro_step, b, theta, layers, n, stream_ptr):
        try:
            t = trainers[int(user or 0)]
            got = batch_fn(t["uid"], worker, inner_step, micro_step, int(b), theta)
            keep_alive.append(got)
            for l in range(n):
                e = got[l]
                d = e["delta"]
                layers[l].delta = d.data_ptr()
                layers[l].delta_row_stride = d.stride(1)
                x = e.get("a") if "a" in e else e.get("x")
                if x is not None:
                    layers[l].a = x.data_ptr()
                    layers[l].a_row_stride = x.stride(1)
            return 0
        except Exception as exc:      # an exception must not cross the C frame
            errors.append(exc)
            return 1

    cb = BATCH_FN(trampoline)
    kk = C.c_int(k)
    reports = (RoundReport * k)()
    rc = lib.adloco_round(ctx._h, C.byref(c), arr, C.byref(kk), tmpl, n_layers, N, cb, reports,
                          _stream_ptr(stream))
    if errors:
        raise errors[0]
    ctx._check(rc)
    order = [int(arr[i].user or 0) for i in range(k)]
    new_list = [trainers[j] for j in order]
    for i, t in enumerate(new_list):
        t["b_req"] = int(arr[i].b_req)
        for m, w in enumerate(t["workers"]):
            w["step"] = int(arr[i].workers[m].step)
    trainers[:] = new_list[:kk.value]
    out = []
    for i in range(kk.value):
        r = reports[i]
        out.append(dict(b_req_used=r.b_req_used, b_micro=r.b_micro, accum_steps=r.accum_steps,
                        accumulate=r.accumulate, merged_from=r.merged_from, test=r.test.as_dict()))
    return out
