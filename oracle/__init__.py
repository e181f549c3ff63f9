"""CPU oracle for the AdamS / N:M hot path of CAST (arXiv 2509.25996).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library and its Python binding never do.

The arithmetic lives in ``cast_oracle.c`` (plain C, one loop per element); this module
compiles it with gcc and marshals numpy arrays.  ``bruteforce.py`` holds the exhaustive
C(M, N) mask search used to pin the selection rule.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cast_oracle.c")
# CAST_ORACLE_LIB: load this library instead of building cast_oracle.c (the pins' own test uses it to
# run them against deliberately broken builds of the oracle)
_OVERRIDE = os.environ.get("CAST_ORACLE_LIB")
_LIB = _OVERRIDE or os.path.join(_HERE, "liboracle.so")
_lib = None


def compile_source(src: str, out: str) -> None:
    """gcc with the flags the oracle is defined under: no fast-math, no FMA contraction, so that every C
    operation is one IEEE-754 operation of its declared type."""
    cmd = ["gcc", "-std=c99", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", out, src, "-lm"]
    subprocess.run(cmd, check=True)


def build(force: bool = False) -> str:
    """Compile the oracle (unless CAST_ORACLE_LIB names a library to use instead)."""
    if _OVERRIDE:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("n_keep", C.c_int32), ("m_group", C.c_int32), ("lr", C.c_float),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("lambda_", C.c_float), ("alpha", C.c_float), ("bias_corr1", C.c_float),
                ("bias_corr2", C.c_float), ("refresh_mask", C.c_int32),
                ("scale_segments", C.c_int32), ("v_from_grad", C.c_int32), ("rule", C.c_int32),
                ("mu_bf16", C.c_int32), ("v_bf16", C.c_int32), ("sr_seed", C.c_uint32)]


# update rules (the enum of cast_oracle.c)
RULE_ADAMS, RULE_ADAMW_L1, RULE_ADAM_L1, RULE_ADDITIVE, RULE_MASKED_FROZEN = range(5)


@dataclass
class AdamsCfg:
    """Inputs of Algorithm 1 for one iteration, as fp32 scalars."""
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
    v_from_grad: int = 0
    rule: int = 0
    mu_bf16: int = 0        # first moment kept in bf16 between iterations (storage variant, not in the paper)
    v_bf16: int = 0         # second moment kept in bf16 too, stochastically rounded with bits drawn from sr_seed
    sr_seed: int = 0

    def c_struct(self) -> _Cfg:
        return _Cfg(self.n_keep, self.m_group, self.lr, self.beta1, self.beta2, self.eps,
                    self.lambda_, self.alpha, self.bias_corr1, self.bias_corr2,
                    self.refresh_mask, self.scale_segments, self.v_from_grad, self.rule, self.mu_bf16,
                    self.v_bf16, self.sr_seed & 0xFFFFFFFF)


def iteration_scalars(t: int, total_steps: int, beta1: float, beta2: float):
    """alpha_t and the two bias corrections for iteration t of Algorithm 1's loop
    (t = 0 .. T-1).  The printed 1 - beta^t is zero at t = 0, so the exponent used is
    t + 1, the only reading under which the first iteration is defined.  beta is taken at
    the fp32 value the step receives."""
    b1 = float(np.float32(beta1))
    b2 = float(np.float32(beta2))
    alpha = np.float32(t / total_steps)
    bc1 = np.float32(1.0 - b1 ** (t + 1))
    bc2 = np.float32(1.0 - b2 ** (t + 1))
    return float(alpha), float(bc1), float(bc2)


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i64, vp = C.c_int64, C.c_void_p
        L.oracle_nm_select.argtypes = [vp, i64, i64, C.c_int, C.c_int, vp]
        L.oracle_pack_mask_bits.argtypes = [vp, i64, i64, vp]
        L.oracle_pack_mask_bits.restype = None
        L.oracle_unpack_mask_bits.argtypes = [vp, i64, i64, vp]
        L.oracle_unpack_mask_bits.restype = None
        for f in (L.oracle_adams_step_f64, L.oracle_adams_step_f32):
            f.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, C.POINTER(_Cfg), C.c_int]
        L.oracle_adams_elements_state64.argtypes = [vp, vp, vp, vp, vp, i64] + [C.c_double] * 8 + [C.c_int, C.c_int]
        L.oracle_weight_scale.argtypes = [vp, vp, i64, i64, C.c_int, vp]
        L.oracle_weight_scale_grad.argtypes = [vp, vp, i64, i64, C.c_int, vp]
        L.oracle_meta_field_bits.argtypes = [C.c_int, C.c_int]
        L.oracle_project_compress.argtypes = [vp, vp, C.c_int, vp, i64, i64, C.c_int, C.c_int, vp, vp]
        L.oracle_bf16_rne_array.argtypes = [vp, i64, vp]
        L.oracle_bf16_rne_array.restype = None
        L.oracle_mask_stats.argtypes = [vp, vp, vp, i64, vp, vp, vp]
        L.oracle_bf16_stochastic.argtypes = [C.c_float, C.c_uint32]
        L.oracle_bf16_stochastic.restype = C.c_uint16
        L.oracle_sr_bits.argtypes = [C.c_uint32, C.c_uint64]
        L.oracle_sr_bits.restype = C.c_uint32
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def nm_select(w: np.ndarray, n_keep: int, m_group: int) -> np.ndarray:
    """Eq. 6 mask of a [rows, cols] fp32 matrix as a uint8 array of 0/1."""
    w = _f32(w)
    rows, cols = w.shape
    keep = np.zeros((rows, cols), np.uint8)
    rc = lib().oracle_nm_select(_p(w), rows, cols, n_keep, m_group, _p(keep))
    if rc:
        raise ValueError("oracle_nm_select: bad shape or N:M")
    return keep


def mask_words_per_row(cols: int) -> int:
    return (cols + 31) // 32


def pack_mask_bits(keep: np.ndarray) -> np.ndarray:
    keep = np.ascontiguousarray(keep, np.uint8)
    rows, cols = keep.shape
    words = np.zeros((rows, mask_words_per_row(cols)), np.uint32)
    lib().oracle_pack_mask_bits(_p(keep), rows, cols, _p(words))
    return words


def unpack_mask_bits(words: np.ndarray, cols: int) -> np.ndarray:
    words = np.ascontiguousarray(words, np.uint32)
    rows = words.shape[0]
    keep = np.zeros((rows, cols), np.uint8)
    lib().oracle_unpack_mask_bits(_p(words), rows, cols, _p(keep))
    return keep


def adams_step(w, grad, mu, v, keep, cfg: AdamsCfg, A=None, want_gA=True, arithmetic="f64",
               nthreads: int = 1):
    """One iteration of Algorithm 1 over one matrix, IN PLACE on w, mu, v (and keep when
    cfg.refresh_mask).  ``arithmetic`` is "f64" (the definition, state rounded to fp32 on
    store) or "f32" (one fp32 rounding per operation).  Returns dL/dA (float64 [rows, n])
    when A is given, else None."""
    for a in (w, grad, mu, v):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    assert keep.dtype == np.uint8 and keep.flags.c_contiguous and keep.shape == w.shape
    rows, cols = w.shape
    gA = None
    if A is not None:
        A = _f32(A)
        assert A.shape == (rows, cfg.scale_segments)
        if want_gA:
            gA = np.zeros((rows, cfg.scale_segments), np.float64)
    fn = {"f64": lib().oracle_adams_step_f64, "f32": lib().oracle_adams_step_f32}[arithmetic]
    cs = cfg.c_struct()
    rc = fn(_p(w), _p(grad), _p(mu), _p(v), _p(keep), _p(A), _p(gA), rows, cols, C.byref(cs), nthreads)
    if rc:
        raise ValueError("oracle_adams_step: bad shape or configuration")
    return gA


def adams_elements_state64(theta, grad, mu, v, m_bits, *, lr, beta1, beta2, eps, lambda_, alpha,
                           bias_corr1, bias_corr2, v_from_grad=0, rule=0):
    """Algorithm 1's per-parameter body on flat float64 arrays, in place."""
    for a in (theta, grad, mu, v):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    assert m_bits.dtype == np.uint8
    lib().oracle_adams_elements_state64(_p(theta), _p(grad), _p(mu), _p(v), _p(m_bits), theta.size,
                                        lr, beta1, beta2, eps, lambda_, alpha, bias_corr1,
                                        bias_corr2, v_from_grad, rule)


def weight_scale(w, A):
    w, A = _f32(w), _f32(A)
    rows, cols = w.shape
    out = np.empty_like(w)
    if lib().oracle_weight_scale(_p(w), _p(A), rows, cols, A.shape[1], _p(out)):
        raise ValueError("oracle_weight_scale: n must divide cols")
    return out


def weight_scale_grad(w, grad_scaled, n):
    w, grad_scaled = _f32(w), _f32(grad_scaled)
    rows, cols = w.shape
    gA = np.zeros((rows, n), np.float64)
    if lib().oracle_weight_scale_grad(_p(w), _p(grad_scaled), rows, cols, n, _p(gA)):
        raise ValueError("oracle_weight_scale_grad: n must divide cols")
    return gA


def meta_field_bits(n_keep: int, m_group: int) -> int:
    return lib().oracle_meta_field_bits(n_keep, m_group)


def meta_words_per_row(cols: int, n_keep: int, m_group: int) -> int:
    f = meta_field_bits(n_keep, m_group)
    groups, gpw = cols // m_group, 32 // f
    return (groups + gpw - 1) // gpw


def project_compress(w, n_keep, m_group, A=None, keep=None):
    """Hard N:M prune + fold of A + pack.  Returns (values fp32 [rows, cols*N/M],
    meta uint32 [rows, meta_words_per_row])."""
    w = _f32(w)
    rows, cols = w.shape
    n = 0
    if A is not None:
        A = _f32(A)
        n = A.shape[1]
    if keep is not None:
        keep = np.ascontiguousarray(keep, np.uint8)
    values = np.zeros((rows, cols // m_group * n_keep), np.float32)
    meta = np.zeros((rows, meta_words_per_row(cols, n_keep, m_group)), np.uint32)
    rc = lib().oracle_project_compress(_p(w), _p(A), n, _p(keep), rows, cols, n_keep, m_group,
                                       _p(values), _p(meta))
    if rc:
        raise ValueError(f"oracle_project_compress failed ({rc})")
    return values, meta


def bf16_stochastic(x: float, r16: int) -> int:
    """bf16 bit pattern of the fp32 value x rounded stochastically with the 16 random bits r16."""
    return int(lib().oracle_bf16_stochastic(float(np.float32(x)), r16 & 0xFFFF))


def sr_bits(seed: int, index: int) -> int:
    """The 16 rounding bits of matrix entry `index` (row * cols + col) under `seed`."""
    return int(lib().oracle_sr_bits(seed & 0xFFFFFFFF, index))


def bf16_rne(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    x = _f32(x)
    out = np.empty(x.shape, np.uint16)
    lib().oracle_bf16_rne_array(_p(x), x.size, _p(out))
    return out


def mask_stats(w, keep, keep_other=None):
    """(flips vs keep_other, ||W*M||_1, ||W||_1) for one matrix."""
    w = _f32(w)
    keep = np.ascontiguousarray(keep, np.uint8)
    if keep_other is not None:
        keep_other = np.ascontiguousarray(keep_other, np.uint8)
    flips = C.c_int64(0)
    a, b = C.c_double(0), C.c_double(0)
    lib().oracle_mask_stats(_p(w), _p(keep), _p(keep_other), w.size, C.byref(flips), C.byref(a), C.byref(b))
    return flips.value, a.value, b.value
