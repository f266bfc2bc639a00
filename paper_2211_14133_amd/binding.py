"""ctypes binding of the C ABI in include/kfac.h: argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used as device memory; every arithmetic
step runs in the HIP library.  There is no fallback: if the library is missing
or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

from . import build as _build

KFAC_OK = 0
KFAC_F32 = 0
KFAC_BF16 = 1
KFAC_F32_BF16X3 = 2
KFAC_F32_F16X2 = 3

_i64 = ctypes.c_int64
_f32 = ctypes.c_float
_vp = ctypes.c_void_p
_sz = ctypes.c_size_t
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int64)


class CurvatureItem(ctypes.Structure):
    _fields_ = [("x", _vp), ("n_tokens", _i64), ("d", _i64), ("ldx", _i64), ("factor", _vp), ("ldf", _i64)]


class InvertItem(ctypes.Structure):
    _fields_ = [("factor", _vp), ("d", _i64), ("ldf", _i64), ("inv", _vp), ("ldi", _i64), ("info_dev", _vp)]


class PreconditionItem(ctypes.Structure):
    _fields_ = [("b_inv", _vp), ("d_out", _i64), ("ldb", _i64), ("a_inv", _vp), ("d_in", _i64), ("lda", _i64),
                ("grad", _vp), ("ldg", _i64), ("out", _vp), ("ldo", _i64)]


#: every symbol include/kfac.h declares, with its ctypes signature
SIGNATURES = {
    "kfac_curvature": (ctypes.c_int, [_vp, ctypes.c_int, _i64, _i64, _i64, _f32, _f32, _vp, _i64, _vp, _sz, _vp]),
    "kfac_curvature_workspace": (_sz, [_i64, _i64, ctypes.c_int]),
    "kfac_curvature_grouped": (ctypes.c_int, [ctypes.POINTER(CurvatureItem), _i64, ctypes.c_int, _f32, _f32, _vp, _sz, _vp]),
    "kfac_curvature_grouped_workspace": (_sz, [ctypes.POINTER(CurvatureItem), _i64, ctypes.c_int]),
    "kfac_invert": (ctypes.c_int, [_vp, _i64, _i64, _f32, _vp, _i64, _vp, _vp, _sz, _vp]),
    "kfac_invert_workspace": (_sz, [_i64]),
    "kfac_invert_batched": (ctypes.c_int, [ctypes.POINTER(InvertItem), _i64, _f32, _vp, _sz, _vp]),
    "kfac_invert_batched_workspace": (_sz, [ctypes.POINTER(InvertItem), _i64]),
    "kfac_invert_noalloc": (ctypes.c_int, [_vp, _i64, _i64, _f32, _vp, _i64, _vp, _vp]),
    "kfac_invert_noalloc_max_d": (_i64, []),
    "kfac_precondition": (ctypes.c_int, [_vp, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _sz, _vp]),
    "kfac_precondition_workspace": (_sz, [_i64, _i64]),
    "kfac_precondition_grouped": (ctypes.c_int, [ctypes.POINTER(PreconditionItem), _i64, _vp, _sz, _vp]),
    "kfac_precondition_grouped_workspace": (_sz, [ctypes.POINTER(PreconditionItem), _i64]),
    "kfac_precondition_grouped_f16x2": (ctypes.c_int, [ctypes.POINTER(PreconditionItem), _i64, _vp, _sz, _vp]),
    "kfac_precondition_grouped_f16x2_workspace": (_sz, [ctypes.POINTER(PreconditionItem), _i64]),
    "kfac_precondition_f16x2_prepare": (ctypes.c_int, [ctypes.POINTER(PreconditionItem), _i64, _vp, _sz, _vp]),
    "kfac_precondition_f16x2_prepared_bytes": (_sz, [ctypes.POINTER(PreconditionItem), _i64]),
    "kfac_precondition_grouped_f16x2_prepared": (ctypes.c_int, [ctypes.POINTER(PreconditionItem), _i64, _vp, _sz, _vp, _sz, _vp]),
    "kfac_precondition_grouped_f16x2_prepared_workspace": (_sz, [ctypes.POINTER(PreconditionItem), _i64]),
    "kfac_invert_plan_create": (ctypes.c_int, [ctypes.POINTER(InvertItem), _i64, _f32, _vp, _sz, ctypes.POINTER(_vp)]),
    "kfac_invert_plan_steps": (_i64, [_vp]),
    "kfac_invert_plan_position": (_i64, [_vp]),
    "kfac_invert_plan_step_flops": (ctypes.c_double, [_vp, _i64]),
    "kfac_invert_plan_step_label": (ctypes.c_char_p, [_vp, _i64]),
    "kfac_invert_plan_run": (ctypes.c_int, [_vp, _i64, _vp]),
    "kfac_invert_plan_reset": (ctypes.c_int, [_vp]),
    "kfac_invert_plan_destroy": (None, [_vp]),
    "kfac_assign_work": (ctypes.c_int, [_i64, _dp, _dp, ctypes.c_double, _i64, _ip, _dp, _dp, _ip, _ip, _ip, _ip, _dp, _ip]),
    "kfac_gpipe_stage": (ctypes.c_int, [_i64, _i64, _i64, ctypes.c_double, ctypes.c_double, _dp, _dp, _dp, _dp, _ip, _dp]),
    "kfac_perf_model": (ctypes.c_int, [ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double, _i64,
                                       ctypes.c_double, ctypes.c_double, ctypes.c_double, _dp]),
    "kfac_mfma_probe": (ctypes.c_int, [ctypes.c_int, _i64, _vp, _dp, _vp]),
    "kfac_mfma_probe_data": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, _i64, _vp, _dp, _vp]),
    "kfac_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "kfac_version": (ctypes.c_int, []),
}

_lib = None


class KfacError(RuntimeError):
    pass


def library_path():
    return _build.LIB


def load():
    """Load the HIP library (built in-tree).  Raises if it is not there."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise KfacError("HIP library %s is missing: run paper_2211_14133_amd/build.py (there is no CPU fallback)" % path)
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(status):
    if status != KFAC_OK:
        raise KfacError("kfac call failed: %s" % load().kfac_status_string(status).decode())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t, split_bf16=False):
    """split_bf16: False, True / "bf16x3" (three bfloat16 terms) or "f16x2" (two float16 terms)."""
    if t.dtype == torch.float32:
        if not split_bf16:
            return KFAC_F32
        return KFAC_F32_F16X2 if split_bf16 == "f16x2" else KFAC_F32_BF16X3
    if split_bf16:
        raise KfacError("the split modes are for float32 input (got %s)" % t.dtype)
    if t.dtype == torch.bfloat16:
        return KFAC_BF16
    raise KfacError("unsupported activation dtype %s" % t.dtype)


def _need_f32_matrix(t, name):
    if not (t.is_cuda and t.dtype == torch.float32 and t.dim() == 2 and t.stride(1) == 1):
        raise KfacError("%s must be a 2-D float32 device tensor with unit column stride" % name)


def _workspace(nbytes, like, workspace, stream=None):
    if nbytes == 0:
        return None, 0, None
    if workspace is None:
        # A temporary buffer comes from torch's caching allocator, which only knows about the stream that is
        # current now: tell it which stream the kernels will run on, so the memory is not handed out again
        # while they are still queued there.
        workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=like.device)
        if stream is not None:
            workspace.record_stream(stream)
    ptr = (workspace.data_ptr() + 255) // 256 * 256
    avail = workspace.numel() * workspace.element_size() - (ptr - workspace.data_ptr())
    return ctypes.c_void_p(ptr), avail, workspace


def _curv_items(xs, factors):
    arr = (CurvatureItem * len(xs))()
    for i, (x, f) in enumerate(zip(xs, factors)):
        if not (x.is_cuda and x.dim() == 2 and x.stride(1) == 1):
            raise KfacError("x must be a 2-D device tensor [tokens, d] with unit column stride")
        _need_f32_matrix(f, "factor")
        if f.shape[0] != x.shape[1] or f.shape[1] != x.shape[1]:
            raise KfacError("factor must be [d, d] for x [tokens, d]")
        if x.dtype != xs[0].dtype:
            raise KfacError("all inputs of a grouped curvature call must have the same dtype (got %s and %s)"
                            % (xs[0].dtype, x.dtype))
        arr[i] = CurvatureItem(x.data_ptr(), x.shape[0], x.shape[1], x.stride(0), f.data_ptr(), f.stride(0))
    return arr


def kfac_curvature(x, factor, alpha, beta, workspace=None, stream=None, split_bf16=False):
    """factor = beta * factor + alpha * x^T x  (one factor, one micro-batch).

    split_bf16: float32 input computed as KFAC_F32_BF16X3 (three bfloat16 terms per value, bf16 MFMA)."""
    lib = load()
    _curv_items([x], [factor])
    dt = _dtype_code(x, split_bf16)
    need = lib.kfac_curvature_workspace(x.shape[0], x.shape[1], dt)
    ws, nbytes, keep = _workspace(need, x, workspace, stream)
    _check(lib.kfac_curvature(ctypes.c_void_p(x.data_ptr()), dt, x.shape[0], x.shape[1], x.stride(0),
                              alpha, beta, ctypes.c_void_p(factor.data_ptr()), factor.stride(0),
                              ws, nbytes, _stream(stream)))
    return factor


def kfac_curvature_grouped_workspace(xs, factors, split_bf16=False):
    arr = _curv_items(xs, factors)
    return int(load().kfac_curvature_grouped_workspace(arr, len(xs), _dtype_code(xs[0], split_bf16)))


def kfac_curvature_grouped(xs, factors, alpha, beta, workspace=None, stream=None, split_bf16=False):
    """Many independent curvature items with a common alpha / beta."""
    lib = load()
    arr = _curv_items(xs, factors)
    dt = _dtype_code(xs[0], split_bf16)
    need = lib.kfac_curvature_grouped_workspace(arr, len(xs), dt)
    ws, nbytes, keep = _workspace(need, xs[0], workspace, stream)
    _check(lib.kfac_curvature_grouped(arr, len(xs), dt, alpha, beta, ws, nbytes, _stream(stream)))
    return factors


def _inv_items(factors, invs, infos):
    arr = (InvertItem * len(factors))()
    for i, (f, v) in enumerate(zip(factors, invs)):
        _need_f32_matrix(f, "factor")
        _need_f32_matrix(v, "inv")
        if f.shape[0] != f.shape[1] or v.shape != f.shape:
            raise KfacError("factor and inv must be square and of equal shape")
        arr[i] = InvertItem(f.data_ptr(), f.shape[0], f.stride(0), v.data_ptr(), v.stride(0),
                            infos.data_ptr() + 4 * i)
    return arr


def kfac_invert(factor, damping, inv, info=None, workspace=None, stream=None):
    """inv = (factor + damping I)^-1; returns the device int32 status tensor."""
    lib = load()
    if info is None:
        info = torch.zeros(1, dtype=torch.int32, device=factor.device)
    _inv_items([factor], [inv], info)
    need = lib.kfac_invert_workspace(factor.shape[0])
    ws, nbytes, keep = _workspace(need, factor, workspace, stream)
    _check(lib.kfac_invert(ctypes.c_void_p(factor.data_ptr()), factor.shape[0], factor.stride(0), damping,
                           ctypes.c_void_p(inv.data_ptr()), inv.stride(0), ctypes.c_void_p(info.data_ptr()),
                           ws, nbytes, _stream(stream)))
    return info


def kfac_invert_noalloc(factor, damping, inv, info, stream=None):
    """kfac_invert with the library's built-in scratch array (d <= 2048): nothing is allocated, here or there."""
    _inv_items([factor], [inv], info)
    _check(load().kfac_invert_noalloc(ctypes.c_void_p(factor.data_ptr()), factor.shape[0], factor.stride(0), damping,
                                      ctypes.c_void_p(inv.data_ptr()), inv.stride(0), ctypes.c_void_p(info.data_ptr()),
                                      _stream(stream)))
    return info


def kfac_invert_batched_workspace(factors, invs):
    infos = torch.zeros(len(factors), dtype=torch.int32, device=factors[0].device)
    arr = _inv_items(factors, invs, infos)
    return int(load().kfac_invert_batched_workspace(arr, len(factors)))


def kfac_invert_batched(factors, damping, invs, infos=None, workspace=None, stream=None):
    """All inversions of a stage advanced together; returns the int32 status tensor [count]."""
    lib = load()
    if infos is None:
        infos = torch.zeros(len(factors), dtype=torch.int32, device=factors[0].device)
    arr = _inv_items(factors, invs, infos)
    need = lib.kfac_invert_batched_workspace(arr, len(factors))
    ws, nbytes, keep = _workspace(need, factors[0], workspace, stream)
    _check(lib.kfac_invert_batched(arr, len(factors), damping, ws, nbytes, _stream(stream)))
    return infos


def _prec_items(b_invs, a_invs, grads, outs):
    arr = (PreconditionItem * len(grads))()
    for i, (b, a, g, o) in enumerate(zip(b_invs, a_invs, grads, outs)):
        for t, nm in ((b, "b_inv"), (a, "a_inv"), (g, "grad"), (o, "out")):
            _need_f32_matrix(t, nm)
        d_out, d_in = g.shape
        if b.shape != (d_out, d_out) or a.shape != (d_in, d_in) or o.shape != g.shape:
            raise KfacError("shape mismatch: grad [d_out, d_in], b_inv [d_out, d_out], a_inv [d_in, d_in]")
        arr[i] = PreconditionItem(b.data_ptr(), d_out, b.stride(0), a.data_ptr(), d_in, a.stride(0),
                                  g.data_ptr(), g.stride(0), o.data_ptr(), o.stride(0))
    return arr


def kfac_precondition(b_inv, a_inv, grad, out, workspace=None, stream=None):
    """out = b_inv @ grad @ a_inv for one layer."""
    lib = load()
    _prec_items([b_inv], [a_inv], [grad], [out])
    d_out, d_in = grad.shape
    need = lib.kfac_precondition_workspace(d_out, d_in)
    ws, nbytes, keep = _workspace(need, grad, workspace, stream)
    _check(lib.kfac_precondition(ctypes.c_void_p(b_inv.data_ptr()), d_out, b_inv.stride(0),
                                 ctypes.c_void_p(a_inv.data_ptr()), d_in, a_inv.stride(0),
                                 ctypes.c_void_p(grad.data_ptr()), grad.stride(0),
                                 ctypes.c_void_p(out.data_ptr()), out.stride(0), ws, nbytes, _stream(stream)))
    return out


def kfac_precondition_grouped_workspace(b_invs, a_invs, grads, outs, f16x2=False):
    arr = _prec_items(b_invs, a_invs, grads, outs)
    lib = load()
    query = lib.kfac_precondition_grouped_f16x2_workspace if f16x2 else lib.kfac_precondition_grouped_workspace
    return int(query(arr, len(grads)))


def kfac_precondition_grouped(b_invs, a_invs, grads, outs, workspace=None, stream=None, f16x2=False):
    """All layers of a stage in two launches (f16x2: operands as two float16 terms on the f16 MFMA)."""
    lib = load()
    arr = _prec_items(b_invs, a_invs, grads, outs)
    query = lib.kfac_precondition_grouped_f16x2_workspace if f16x2 else lib.kfac_precondition_grouped_workspace
    run = lib.kfac_precondition_grouped_f16x2 if f16x2 else lib.kfac_precondition_grouped
    need = query(arr, len(grads))
    ws, nbytes, keep = _workspace(need, grads[0], workspace, stream)
    _check(run(arr, len(grads), ws, nbytes, _stream(stream)))
    return outs


class PreparedInverses:
    """The float16 planes of the inverses of a stage, made once per refresh; `precondition` then applies them to
    any number of gradients (kfac_precondition_f16x2_prepare / kfac_precondition_grouped_f16x2_prepared)."""

    def __init__(self, b_invs, a_invs, stream=None):
        lib = load()
        self._invs = (list(b_invs), list(a_invs))
        arr = (PreconditionItem * len(b_invs))()
        for i, (b, a) in enumerate(zip(b_invs, a_invs)):
            _need_f32_matrix(b, "b_inv")
            _need_f32_matrix(a, "a_inv")
            if b.shape[0] != b.shape[1] or a.shape[0] != a.shape[1]:
                raise KfacError("the inverses must be square")
            arr[i] = PreconditionItem(b.data_ptr(), b.shape[0], b.stride(0), a.data_ptr(), a.shape[0], a.stride(0),
                                      0, a.shape[0], 0, a.shape[0])  # gradient and output are not looked at
        need = lib.kfac_precondition_f16x2_prepared_bytes(arr, len(b_invs))
        self._ptr, self._bytes, self._buf = _workspace(need, b_invs[0], None, stream)
        _check(lib.kfac_precondition_f16x2_prepare(arr, len(b_invs), self._ptr, self._bytes, _stream(stream)))

    def precondition(self, grads, outs, workspace=None, stream=None):
        lib = load()
        arr = _prec_items(self._invs[0], self._invs[1], grads, outs)
        need = lib.kfac_precondition_grouped_f16x2_prepared_workspace(arr, len(grads))
        ws, nbytes, keep = _workspace(need, grads[0], workspace, stream)
        _check(lib.kfac_precondition_grouped_f16x2_prepared(arr, len(grads), self._ptr, self._bytes, ws, nbytes,
                                                            _stream(stream)))
        return outs


class InvertPlan:
    """Chunked form of kfac_invert_batched: the launch sequence is recorded once and run piecewise."""

    def __init__(self, factors, damping, invs, infos=None, workspace=None):
        lib = load()
        if infos is None:
            infos = torch.zeros(len(factors), dtype=torch.int32, device=factors[0].device)
        self.infos = infos
        self._keep = (list(factors), list(invs), infos)
        arr = _inv_items(factors, invs, infos)
        need = lib.kfac_invert_batched_workspace(arr, len(factors))
        ws, nbytes, self._ws = _workspace(need, factors[0], workspace)  # kept for the plan's lifetime
        handle = ctypes.c_void_p()
        _check(lib.kfac_invert_plan_create(arr, len(factors), damping, ws, nbytes, ctypes.byref(handle)))
        self._h = handle

    @property
    def steps(self):
        return int(load().kfac_invert_plan_steps(self._h))

    @property
    def position(self):
        return int(load().kfac_invert_plan_position(self._h))

    def step_flops(self, i):
        return float(load().kfac_invert_plan_step_flops(self._h, i))

    def step_label(self, i):
        label = load().kfac_invert_plan_step_label(self._h, i)
        return None if label is None else label.decode()

    def run(self, n_steps, stream=None):
        _check(load().kfac_invert_plan_run(self._h, n_steps, _stream(stream)))

    def reset(self):
        _check(load().kfac_invert_plan_reset(self._h))

    def close(self):
        if self._h is not None:
            load().kfac_invert_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _darr(values):
    return (ctypes.c_double * max(1, len(values)))(*[float(v) for v in values])


def _iarr(values):
    return (ctypes.c_int64 * max(1, len(values)))(*[int(v) for v in values])


def kfac_assign_work(bubble_start, bubble_length, step_period, chunk_times, release, deps):
    """Greedy assignment of work chunks to pipeline bubbles (host only).

    chunk_times: per work, the list of its chunk durations; release: per work; deps: per work, ids of
    earlier works it waits for.  Returns (per work: list of (step, bubble, start)), steps_needed.
    """
    lib = load()
    n_works = len(chunk_times)
    counts = [len(c) for c in chunk_times]
    flat = [t for c in chunk_times for t in c]
    dep_begin, dep_ids = [0], []
    for d in deps:
        dep_ids += list(d)
        dep_begin.append(len(dep_ids))
    n = len(flat)
    out_step, out_bubble, out_start = _iarr([0] * n), _iarr([0] * n), _darr([0.0] * n)
    needed = ctypes.c_int64(0)
    _check(lib.kfac_assign_work(len(bubble_start), _darr(bubble_start), _darr(bubble_length), float(step_period),
                                n_works, _iarr(counts), _darr(flat), _darr(release), _iarr(dep_begin), _iarr(dep_ids),
                                out_step, out_bubble, out_start, ctypes.cast(ctypes.byref(needed), _ip)))
    res, k = [], 0
    for c in counts:
        res.append([(int(out_step[k + i]), int(out_bubble[k + i]), float(out_start[k + i])) for i in range(c)])
        k += c
    return res, int(needed.value)


def kfac_gpipe_stage(stage, depth, n_micro, t_f, t_b):
    """One GPipe step seen from `stage`: release times, bubbles and the step length (host only)."""
    fwd, bwd = _darr([0.0] * n_micro), _darr([0.0] * n_micro)
    bs, bl = _darr([0.0] * 3), _darr([0.0] * 3)
    nb, t_step = ctypes.c_int64(0), ctypes.c_double(0.0)
    _check(load().kfac_gpipe_stage(stage, depth, n_micro, float(t_f), float(t_b), fwd, bwd, bs, bl,
                                   ctypes.cast(ctypes.byref(nb), _ip), ctypes.cast(ctypes.byref(t_step), _dp)))
    return {"forward_end": [fwd[m] for m in range(n_micro)], "backward_end": [bwd[m] for m in range(n_micro)],
            "bubbles": [(bs[i], bl[i]) for i in range(nb.value)], "t_step": t_step.value}


def kfac_perf_model(c_f, c_b, t_f, t_b, n_micro, t_curv, t_inv, t_prec):
    """Closed forms of the paper's performance model; returns a dict."""
    out = _darr([0.0] * 5)
    _check(load().kfac_perf_model(c_f, c_b, t_f, t_b, n_micro, t_curv, t_inv, t_prec, out))
    return {"t_pipe": out[0], "t_bubble": out[1], "t_kfac": out[2], "ratio": out[3], "t_step": out[4]}


def kfac_mfma_probe(dtype, iters, sink, stream=None, random_operands=False):
    """Enqueue the register-only MFMA loop; returns the flops it performs (time it with events)."""
    flops = ctypes.c_double(0.0)
    _check(load().kfac_mfma_probe_data(int(dtype), int(bool(random_operands)), int(iters),
                                       ctypes.c_void_p(sink.data_ptr()), ctypes.byref(flops), _stream(stream)))
    return flops.value
