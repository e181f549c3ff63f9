"""Thin ctypes binding of libcast.so: the same entry points as ``include/cast.h``, taking
torch tensors that already live on the GPU.  Argument marshalling only: every step of the
method runs inside the library's HIP kernels.  A missing library is an error; there is no
CPU path."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CAST_LIBRARY") or os.path.join(_HERE, "libcast.so")   # override: A/B experiments only

CAST_F32, CAST_BF16 = 0, 1
FLAG_V_FROM_GRAD = 1
FLAG_MU_BF16 = 4
FLAG_V_BF16 = 8
RULE_ADAMS, RULE_ADAMW_L1, RULE_ADAM_L1, RULE_ADDITIVE, RULE_MASKED_FROZEN = range(5)

EXPORTS = ["cast_status_str", "cast_sizes", "cast_nm_select", "cast_adams_step", "cast_weight_scale",
           "cast_weight_scale_grad", "cast_nm_project_compress", "cast_mask_stats", "cast_hbm_copy_probe",
           "cast_debug_div_by_uniform", "cast_adams_multi_workspace_bytes", "cast_adams_step_multi",
           "cast_adams_step_emit", "cast_adams_multi_launches", "cast_debug_plan", "cast_adams_step_multi_noalloc",
           "cast_hbm_stream_probe", "cast_nm_select_multi", "cast_weight_scale_multi", "cast_nm_project_compress_multi",
           "cast_mask_stats_multi", "cast_mask_stats_multi_workspace_bytes", "cast_weight_scale_grad_multi"]


class CastError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_str(status)})")
        self.status = status


class _Tensor(C.Structure):
    _fields_ = [("w", C.c_void_p), ("grad", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("mask_bits", C.c_void_p), ("scale", C.c_void_p), ("scale_grad", C.c_void_p),
                ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("compute_copy", C.c_void_p), ("copy_scale", C.c_void_p),
                ("initial_mask_bits", C.c_void_p), ("refresh_stats", C.c_void_p)]


class _Matrix(C.Structure):
    _fields_ = [("w", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64), ("scale", C.c_void_p),
                ("mask_bits", C.c_void_p), ("out", C.c_void_p), ("meta", C.c_void_p), ("mask_status", C.c_void_p)]


class _StatsMatrix(C.Structure):
    _fields_ = [("w", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64), ("mask_bits", C.c_void_p),
                ("other_bits", C.c_void_p), ("stats", C.c_void_p)]


class _ScaleGradMatrix(C.Structure):
    _fields_ = [("w", C.c_void_p), ("grad_scaled", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("scale_grad", C.c_void_p)]


class _Config(C.Structure):
    _fields_ = [("n_keep", C.c_int32), ("m_group", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("lambda_", C.c_float), ("alpha", C.c_float),
                ("bias_corr1", C.c_float), ("bias_corr2", C.c_float), ("refresh_mask", C.c_int32),
                ("scale_segments", C.c_int32), ("grad_dtype", C.c_int32), ("flags", C.c_uint32), ("rule", C.c_int32),
                ("sr_seed", C.c_uint32)]


@dataclass
class AdamsConfig:
    """Mirror of ``cast_adams_config`` (inputs of one iteration of Algorithm 1)."""
    n_keep: int = 2
    m_group: int = 4
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    lambda_: float = 2e-6
    alpha: float = 0.0
    bias_corr1: float = 1.0
    bias_corr2: float = 1.0
    refresh_mask: int = 1
    scale_segments: int = 0
    grad_dtype: int = CAST_F32
    flags: int = 0
    rule: int = 0
    sr_seed: int = 0        # seed of the stochastic rounding of a bf16 second moment; another one every iteration

    def c_struct(self) -> _Config:
        return _Config(self.n_keep, self.m_group, self.lr, self.beta1, self.beta2, self.eps, self.lambda_,
                       self.alpha, self.bias_corr1, self.bias_corr2, self.refresh_mask, self.scale_segments,
                       self.grad_dtype, self.flags, self.rule, self.sr_seed & 0xFFFFFFFF)


_lib = None


def load():
    """Load libcast.so (built in place by ``python -m paper_2509_25996_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_25996_amd.build` "
                                "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    i64, vp, ci = C.c_int64, C.c_void_p, C.c_int
    L.cast_status_str.argtypes = [C.c_int32]
    L.cast_status_str.restype = C.c_char_p
    L.cast_sizes.argtypes = [i64, i64, ci, ci, ci, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    L.cast_nm_select.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp]
    L.cast_adams_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, C.POINTER(_Config), vp]
    L.cast_adams_step_emit.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, C.POINTER(_Config), vp]
    L.cast_weight_scale.argtypes = [vp, vp, i64, i64, i64, ci, vp, ci, vp]
    L.cast_weight_scale_grad.argtypes = [vp, vp, ci, i64, i64, i64, ci, vp, vp]
    L.cast_nm_project_compress.argtypes = [vp, vp, ci, vp, i64, i64, i64, ci, ci, vp, ci, vp, vp]
    L.cast_mask_stats.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, vp]
    L.cast_hbm_copy_probe.argtypes = [vp, vp, C.c_size_t, vp]
    L.cast_debug_div_by_uniform.argtypes = [vp, C.c_float, vp, i64]
    L.cast_adams_multi_workspace_bytes.argtypes = [C.POINTER(_Tensor), ci, C.POINTER(_Config)]
    L.cast_adams_multi_workspace_bytes.restype = C.c_size_t
    L.cast_adams_step_multi.argtypes = [C.POINTER(_Tensor), ci, C.POINTER(_Config), vp, C.c_size_t, vp]
    L.cast_adams_step_multi_noalloc.argtypes = [C.POINTER(_Tensor), ci, C.POINTER(_Config), vp]
    L.cast_nm_select_multi.argtypes = [C.POINTER(_Matrix), ci, ci, ci, vp]
    L.cast_weight_scale_multi.argtypes = [C.POINTER(_Matrix), ci, ci, ci, vp]
    L.cast_nm_project_compress_multi.argtypes = [C.POINTER(_Matrix), ci, ci, ci, ci, ci, vp]
    L.cast_weight_scale_grad_multi.argtypes = [C.POINTER(_ScaleGradMatrix), ci, ci, ci, vp]
    L.cast_mask_stats_multi.argtypes = [C.POINTER(_StatsMatrix), ci, vp, C.c_size_t, vp]
    L.cast_mask_stats_multi_workspace_bytes.argtypes = [C.POINTER(_StatsMatrix), ci]
    L.cast_mask_stats_multi_workspace_bytes.restype = C.c_size_t
    L.cast_hbm_stream_probe.argtypes = [C.POINTER(_Tensor), ci, ci, ci, C.c_uint32, vp, C.c_size_t, vp]
    L.cast_debug_plan.argtypes = [i64, i64, i64, ci, ci, i64, ci, C.POINTER(i64), C.POINTER(i64)]
    L.cast_adams_multi_launches.argtypes = [C.POINTER(_Tensor), ci, C.POINTER(_Config), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    for name in EXPORTS:
        if name not in ("cast_status_str", "cast_adams_multi_workspace_bytes", "cast_mask_stats_multi_workspace_bytes"):
            getattr(L, name).restype = C.c_int32
    _lib = L
    return L


def status_str(status: int) -> str:
    return load().cast_status_str(status).decode()


def _check(status: int, what: str):
    if status != 0:
        raise CastError(status, what)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CAST_F32
    if t.dtype == torch.bfloat16:
        return CAST_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous and on the GPU")


def _ld(w, *same):
    """Row stride of a [rows, cols] weight/moment tensor whose rows are contiguous; dense tensors
    give ld == cols, row-interleaved state (see interleaved_state) gives ld == 3 * cols."""
    if not w.is_cuda or w.dim() != 2:
        raise ValueError("w, m, v must be 2-D GPU tensors with contiguous rows")
    if w.numel() == 0:
        return w.shape[1]
    if w.shape[1] > 1 and w.stride(1) != 1:
        raise ValueError("w, m, v must be 2-D GPU tensors with contiguous rows")
    ld = w.stride(0) if w.shape[0] > 1 else max(w.stride(0), w.shape[1])
    ld = max(ld, w.shape[1])
    for t in same:
        # a first moment kept in bf16: dense if w is, else the byte pitch of w (twice its row stride in entries)
        want = w.stride(0) if t.dtype == torch.float32 else (w.shape[1] if ld == w.shape[1] else 2 * ld)
        if t.shape != w.shape or (t.shape[0] > 1 and t.stride(0) != want) or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("w, m and v must share one shape and one row stride")
    return ld


def _mu_flag(cfg, m, v=None) -> None:
    """Sets or clears CAST_FLAG_MU_BF16 and CAST_FLAG_V_BF16 according to the dtypes of the moments."""
    for t in (m, v):
        if t is not None and t.dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("m and v must be float32 or bfloat16")
    cfg.flags = (cfg.flags & ~(FLAG_MU_BF16 | FLAG_V_BF16)) | (FLAG_MU_BF16 if m.dtype == torch.bfloat16 else 0) \
        | (FLAG_V_BF16 if v is not None and v.dtype == torch.bfloat16 else 0)


def interleaved_state(w0: torch.Tensor, mu_bf16: bool = False, v_bf16: bool = False):
    """Allocate w, m, v of one matrix interleaved row by row in one buffer [rows, 3, cols] (row
    stride 3*cols for each of the three views).  w is initialised from w0, m and v are zero.
    mu_bf16: m is bfloat16 and a row of the buffer is cols fp32, cols bf16, cols fp32 (10 * cols bytes);
    with v_bf16 on top v is bfloat16 as well (8 * cols bytes a row)."""
    rows, cols = w0.shape
    if v_bf16 and not mu_bf16:
        raise ValueError("v_bf16 comes with mu_bf16")
    if mu_bf16:
        if cols % 8:
            raise ValueError("cols must be a multiple of 8")
        raw = torch.zeros((rows, (8 if v_bf16 else 10) * cols), dtype=torch.uint8, device=w0.device)
        w = raw[:, :4 * cols].view(torch.float32)
        m = raw[:, 4 * cols:6 * cols].view(torch.bfloat16)
        v = raw[:, 6 * cols:].view(torch.bfloat16 if v_bf16 else torch.float32)
        w.copy_(w0)
        return w, m, v
    state = torch.zeros((rows, 3, cols), dtype=torch.float32, device=w0.device)
    state[:, 0, :].copy_(w0)
    return state[:, 0, :], state[:, 1, :], state[:, 2, :]


def cast_sizes(rows: int, cols: int, n_keep: int, m_group: int, value_dtype: int = CAST_F32):
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(load().cast_sizes(rows, cols, n_keep, m_group, value_dtype, C.byref(a), C.byref(b), C.byref(c)), "cast_sizes")
    return a.value, b.value, c.value


def alloc_mask(rows: int, cols: int, device="cuda:0") -> torch.Tensor:
    """int32 tensor [rows, ceil(cols/32)] holding the uint32 mask words."""
    return torch.zeros((rows, (cols + 31) // 32), dtype=torch.int32, device=device)


def cast_nm_select(w: torch.Tensor, n_keep: int, m_group: int, mask_bits: torch.Tensor, stream=None):
    _dev(mask_bits)
    rows, cols = w.shape
    _check(load().cast_nm_select(_ptr(w), rows, cols, _ld(w), n_keep, m_group, _ptr(mask_bits), _stream(stream)),
           "cast_nm_select")


class MatrixList:
    """Descriptors of a list of matrices for the once-per-run list calls (cast_nm_select_multi,
    cast_weight_scale_multi, cast_nm_project_compress_multi), marshalled once.  Each item is a dict with w and,
    as the call needs them, scale, mask, out (the scaled weights or the packed values), meta, mask_status (an int32
    tensor of one word that counts the invalid groups of a stored mask) (tensors)."""

    def __init__(self, items):
        self.items = list(items)     # keeps the tensors alive
        n = len(self.items)
        self.array = (_Matrix * max(n, 1))()
        self.count = n
        self.out_dtype = None
        segments = set()
        for k, x in enumerate(self.items):
            w = x["w"]
            sc, mk, out, meta, status = x.get("scale"), x.get("mask"), x.get("out"), x.get("meta"), x.get("mask_status")
            _dev(sc, mk, out, meta, status)
            if out is not None:
                dt = _dtype_code(out)
                if self.out_dtype not in (None, dt):
                    raise ValueError("all outputs of a list must have one dtype")
                self.out_dtype = dt
            if sc is not None and w.numel():
                segments.add(sc.shape[1])
            self.array[k] = _Matrix(w.data_ptr(), w.shape[0], w.shape[1], _ld(w), None if sc is None else sc.data_ptr(),
                                    None if mk is None else mk.data_ptr(), None if out is None else out.data_ptr(),
                                    None if meta is None else meta.data_ptr(), None if status is None else status.data_ptr())
        if len(segments) > 1:
            raise ValueError("all matrices of a list must have the same number of scaling segments")
        self.segments = segments.pop() if segments else 0


def cast_nm_select_multi(matrices: MatrixList, n_keep: int, m_group: int, stream=None):
    _check(load().cast_nm_select_multi(matrices.array, matrices.count, n_keep, m_group, _stream(stream)), "cast_nm_select_multi")


def cast_weight_scale_multi(matrices: MatrixList, stream=None):
    _check(load().cast_weight_scale_multi(matrices.array, matrices.count, matrices.segments, matrices.out_dtype or CAST_F32,
                                          _stream(stream)), "cast_weight_scale_multi")


def cast_nm_project_compress_multi(matrices: MatrixList, n_keep: int, m_group: int, stream=None):
    _check(load().cast_nm_project_compress_multi(matrices.array, matrices.count, matrices.segments, n_keep, m_group,
                                                 matrices.out_dtype or CAST_F32, _stream(stream)),
           "cast_nm_project_compress_multi")


def cast_adams_step(w, grad, m, v, mask_bits, cfg: AdamsConfig, scale=None, scale_grad=None, stream=None):
    _dev(grad, mask_bits, scale, scale_grad)
    rows, cols = w.shape
    cfg.grad_dtype = _dtype_code(grad)
    _mu_flag(cfg, m, v)
    cs = cfg.c_struct()
    _check(load().cast_adams_step(_ptr(w), _ptr(grad), _ptr(m), _ptr(v), _ptr(mask_bits), _ptr(scale), _ptr(scale_grad),
                                  rows, cols, _ld(w, m, v), C.byref(cs), _stream(stream)), "cast_adams_step")


def cast_adams_step_emit(w, grad, m, v, mask_bits, cfg: AdamsConfig, compute_copy, copy_scale=None, scale=None,
                         scale_grad=None, stream=None):
    """cast_adams_step that also writes bf16(copy_scale * w_new) (or bf16(w_new)) into compute_copy."""
    _dev(grad, mask_bits, scale, scale_grad, compute_copy, copy_scale)
    if compute_copy.dtype != torch.bfloat16:
        raise TypeError("compute_copy must be bfloat16")
    rows, cols = w.shape
    cfg.grad_dtype = _dtype_code(grad)
    _mu_flag(cfg, m, v)
    cs = cfg.c_struct()
    _check(load().cast_adams_step_emit(_ptr(w), _ptr(grad), _ptr(m), _ptr(v), _ptr(mask_bits), _ptr(scale), _ptr(scale_grad),
                                       _ptr(copy_scale), _ptr(compute_copy), rows, cols, _ld(w, m, v), C.byref(cs),
                                       _stream(stream)), "cast_adams_step_emit")


def cast_adams_multi_workspace_bytes(array, count: int, cfg: "AdamsConfig") -> int:
    cs = cfg.c_struct()
    return load().cast_adams_multi_workspace_bytes(array, count, C.byref(cs))


def alloc_refresh_stats(device="cuda:0") -> "torch.Tensor":
    """Device storage of one cast_refresh_stats (two uint64 counts, two doubles)."""
    return torch.zeros(4, dtype=torch.int64, device=device)


def read_refresh_stats(t: "torch.Tensor") -> dict:
    """A cast_refresh_stats written by a refresh step, as Python numbers (synchronises)."""
    h = t.cpu()
    norms = h[2:].view(torch.float64)
    return {"flips_prev": int(h[0]), "flips_init": int(h[1]), "l1_kept": float(norms[0]), "l1_all": float(norms[1])}


class TensorList:
    """The descriptors of a list of matrices for cast_adams_step_multi, marshalled once, plus the
    device workspace the call needs.  Each item is a dict with w, grad, m, v, mask and optionally
    scale, scale_grad, compute_copy, copy_scale, initial_mask, refresh_stats (tensors)."""

    def __init__(self, items, device="cuda:0"):
        self.items = list(items)     # keeps the tensors alive
        n = len(self.items)
        self.array = (_Tensor * max(n, 1))()
        self.grad_dtype = None
        self.mu_dtype = None
        for k, x in enumerate(self.items):
            w, m, v = x["w"], x["m"], x["v"]
            if self.mu_dtype not in (None, (m.dtype, v.dtype)):
                raise ValueError("the moments of a list must have the same dtypes in every matrix")
            self.mu_dtype = (m.dtype, v.dtype)
            _dev(x["grad"], x["mask"], x.get("scale"), x.get("scale_grad"))
            dt = _dtype_code(x["grad"])
            if self.grad_dtype not in (None, dt):
                raise ValueError("all gradients of a list must have one dtype")
            self.grad_dtype = dt
            sc, sg = x.get("scale"), x.get("scale_grad")
            cp, cps = x.get("compute_copy"), x.get("copy_scale")
            im, rs = x.get("initial_mask"), x.get("refresh_stats")
            _dev(cp, cps, im, rs)
            if rs is not None and (rs.dtype != torch.int64 or rs.numel() != 4):
                raise TypeError("refresh_stats must come from alloc_refresh_stats()")
            if cp is not None and cp.dtype != torch.bfloat16:
                raise TypeError("compute_copy must be bfloat16")
            self.array[k] = _Tensor(w.data_ptr(), x["grad"].data_ptr(), m.data_ptr(), v.data_ptr(), x["mask"].data_ptr(),
                                    None if sc is None else sc.data_ptr(), None if sg is None else sg.data_ptr(),
                                    w.shape[0], w.shape[1], _ld(w, m, v),
                                    None if cp is None else cp.data_ptr(), None if cps is None else cps.data_ptr(),
                                    None if im is None else im.data_ptr(), None if rs is None else rs.data_ptr())
        self.count = n
        # the workspace depends on the shapes and on the number of scaling segments
        segments = {0 if x.get("scale") is None else x["scale"].shape[1] for x in self.items if x["w"].numel()}
        if len(segments) > 1:
            raise ValueError("all matrices of a list must have the same number of scaling segments")
        probe = AdamsConfig(scale_segments=segments.pop() if segments else 0)
        need = max(16, cast_adams_multi_workspace_bytes(self.array, n, probe))
        self.workspace = torch.empty(need, dtype=torch.uint8, device=device)


def cast_adams_step_multi(tensors: TensorList, cfg: AdamsConfig, stream=None):
    if tensors.count:
        cfg.grad_dtype = tensors.grad_dtype
        _mu_flag(cfg, tensors.items[0]["m"], tensors.items[0]["v"])
    cs = cfg.c_struct()
    _check(load().cast_adams_step_multi(tensors.array, tensors.count, C.byref(cs), _ptr(tensors.workspace),
                                        tensors.workspace.numel(), _stream(stream)), "cast_adams_step_multi")


def cast_adams_step_multi_noalloc(tensors: TensorList, cfg: AdamsConfig, stream=None):
    """cast_adams_step_multi on the library's built-in workspace (the list's own workspace is not used)."""
    if tensors.count:
        cfg.grad_dtype = tensors.grad_dtype
        _mu_flag(cfg, tensors.items[0]["m"], tensors.items[0]["v"])
    cs = cfg.c_struct()
    _check(load().cast_adams_step_multi_noalloc(tensors.array, tensors.count, C.byref(cs), _stream(stream)),
           "cast_adams_step_multi_noalloc")


def cast_adams_multi_launches(tensors: TensorList, cfg: AdamsConfig):
    """(launches of the step kernel, other launches) one cast_adams_step_multi call makes for this list."""
    if tensors.count:
        cfg.grad_dtype = tensors.grad_dtype
        _mu_flag(cfg, tensors.items[0]["m"], tensors.items[0]["v"])
    cs = cfg.c_struct()
    a, b = C.c_int32(0), C.c_int32(0)
    _check(load().cast_adams_multi_launches(tensors.array, tensors.count, C.byref(cs), C.byref(a), C.byref(b)),
           "cast_adams_multi_launches")
    return a.value, b.value


def cast_weight_scale(w, scale, out, stream=None):
    _dev(scale, out)
    rows, cols = w.shape
    _check(load().cast_weight_scale(_ptr(w), _ptr(scale), rows, cols, _ld(w), scale.shape[1], _ptr(out),
                                    _dtype_code(out), _stream(stream)), "cast_weight_scale")


def cast_weight_scale_grad(w, grad_scaled, n_segments: int, scale_grad, stream=None):
    _dev(grad_scaled, scale_grad)
    rows, cols = w.shape
    _check(load().cast_weight_scale_grad(_ptr(w), _ptr(grad_scaled), _dtype_code(grad_scaled), rows, cols, _ld(w),
                                         n_segments, _ptr(scale_grad), _stream(stream)), "cast_weight_scale_grad")


class ScaleGradList:
    """Descriptors for cast_weight_scale_grad_multi, marshalled once.  Each item is a dict with w, grad (dL/dW_scale,
    dense, one dtype for the whole list) and scale_grad (fp32 [rows, n]: n is the same for the whole list)."""

    def __init__(self, items):
        self.items = list(items)
        n = len(self.items)
        self.array = (_ScaleGradMatrix * max(n, 1))()
        self.count = n
        self.grad_dtype, self.segments = None, None
        for k, x in enumerate(self.items):
            w, g, sg = x["w"], x["grad"], x["scale_grad"]
            _dev(g, sg)
            if self.grad_dtype not in (None, _dtype_code(g)):
                raise ValueError("all gradients of a list must have one dtype")
            if self.segments not in (None, sg.shape[1]):
                raise ValueError("all matrices of a list must have the same number of scaling segments")
            self.grad_dtype, self.segments = _dtype_code(g), sg.shape[1]
            self.array[k] = _ScaleGradMatrix(w.data_ptr(), g.data_ptr(), w.shape[0], w.shape[1], _ld(w), sg.data_ptr())


def cast_weight_scale_grad_multi(matrices: ScaleGradList, stream=None):
    _check(load().cast_weight_scale_grad_multi(matrices.array, matrices.count, matrices.grad_dtype or CAST_F32,
                                               matrices.segments or 1, _stream(stream)), "cast_weight_scale_grad_multi")


def cast_nm_project_compress(w, n_keep: int, m_group: int, values, meta, scale=None, mask_bits=None, stream=None):
    _dev(values, meta, scale, mask_bits)
    rows, cols = w.shape
    n_seg = 0 if scale is None else scale.shape[1]
    _check(load().cast_nm_project_compress(_ptr(w), _ptr(scale), n_seg, _ptr(mask_bits), rows, cols, _ld(w), n_keep, m_group,
                                           _ptr(values), _dtype_code(values), _ptr(meta), _stream(stream)),
           "cast_nm_project_compress")


def cast_mask_stats(w, mask_bits, other_bits, flips, l1, stream=None):
    """flips: int64 tensor [1]; l1: float64 tensor [2]; both accumulated into."""
    _dev(mask_bits, other_bits, flips, l1)
    rows, cols = w.shape
    _check(load().cast_mask_stats(_ptr(w), _ptr(mask_bits), _ptr(other_bits), rows, cols, _ld(w), _ptr(flips), _ptr(l1),
                                  _stream(stream)), "cast_mask_stats")


class StatsList:
    """Descriptors for cast_mask_stats_multi, marshalled once, with the workspace the call needs.  Each item is a dict
    with w, mask, optionally other (the mask flips are counted against) and stats (from alloc_refresh_stats())."""

    def __init__(self, items, device="cuda:0"):
        self.items = list(items)
        n = len(self.items)
        self.array = (_StatsMatrix * max(n, 1))()
        self.count = n
        for k, x in enumerate(self.items):
            w, mk, other, st = x["w"], x["mask"], x.get("other"), x["stats"]
            _dev(mk, other, st)
            if st.dtype != torch.int64 or st.numel() != 4:
                raise TypeError("stats must come from alloc_refresh_stats()")
            self.array[k] = _StatsMatrix(w.data_ptr(), w.shape[0], w.shape[1], _ld(w), mk.data_ptr(),
                                         None if other is None else other.data_ptr(), st.data_ptr())
        need = load().cast_mask_stats_multi_workspace_bytes(self.array, n)
        self.workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=device)


def cast_mask_stats_multi(matrices: StatsList, stream=None):
    _check(load().cast_mask_stats_multi(matrices.array, matrices.count, _ptr(matrices.workspace), matrices.workspace.numel(),
                                        _stream(stream)), "cast_mask_stats_multi")


def cast_hbm_copy_probe(dst, src, stream=None):
    _dev(dst, src)
    _check(load().cast_hbm_copy_probe(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)),
           "cast_hbm_copy_probe")


def cast_hbm_stream_probe(tensors: TensorList, scale_segments: int, stream=None):
    """The list call's launches with next to no arithmetic (bandwidth ceiling of its access pattern), for the
    gradient and moment dtypes of the list.  Overwrites w, m, v and scale_grad of every matrix of the list."""
    flags = 0
    if tensors.count:
        m, v = tensors.items[0]["m"], tensors.items[0]["v"]
        flags = (FLAG_MU_BF16 if m.dtype == torch.bfloat16 else 0) | (FLAG_V_BF16 if v.dtype == torch.bfloat16 else 0)
    _check(load().cast_hbm_stream_probe(tensors.array, tensors.count, scale_segments,
                                        CAST_BF16 if tensors.grad_dtype is None else tensors.grad_dtype, flags,
                                        _ptr(tensors.workspace), tensors.workspace.numel(), _stream(stream)),
           "cast_hbm_stream_probe")


def cast_debug_div_by_uniform(x, y: float):
    """Host-side: numpy fp32 array x divided by y through the kernels' own division routine."""
    import numpy as np
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty_like(x)
    _check(load().cast_debug_div_by_uniform(x.ctypes.data_as(C.c_void_p), y, out.ctypes.data_as(C.c_void_p), x.size),
           "cast_debug_div_by_uniform")
    return out


def iteration_config(t: int, total_steps: int, mask_period: int = 10, **kw) -> AdamsConfig:
    """Scalars of iteration t of Algorithm 1's loop (t = 0 .. T-1): alpha_t = t/T, mask
    refresh when t mod T_1 == 0, and bias corrections with exponent t + 1 (the printed
    1 - beta^t is zero at t = 0)."""
    cfg = AdamsConfig(**kw)
    b1 = C.c_float(cfg.beta1).value
    b2 = C.c_float(cfg.beta2).value
    cfg.alpha = t / total_steps
    cfg.bias_corr1 = 1.0 - b1 ** (t + 1)
    cfg.bias_corr2 = 1.0 - b2 ** (t + 1)
    cfg.refresh_mask = int(t % mask_period == 0)
    cfg.sr_seed = t
    return cfg
