"""Helpers of the GPU parity tests: move arrays, run an N-step trajectory on both sides."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from fp32_bound import Fp32Drift
from paper_2509_25996_amd import binding as B

DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)) if isinstance(a, np.ndarray) else a
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV).contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def words(t: torch.Tensor) -> np.ndarray:
    """int32 device tensor of uint32 words -> numpy uint32."""
    return host(t).view(np.uint32)


def same_bits(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Elementwise: identical fp32 bit patterns, any NaN matching any NaN."""
    a = np.ascontiguousarray(a, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    return (a.view(np.uint32) == b.view(np.uint32)) | (np.isnan(a) & np.isnan(b))


def assert_same_bits(got, ref, what=""):
    ok = same_bits(got, ref)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {ok.size} entries differ; first at {i}: "
                             f"got {got[i]!r} ({got[i].view(np.uint32):#x}) ref {ref[i]!r} ({ref[i].view(np.uint32):#x})")


def max_rel_err(got, ref):
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    d = np.abs(got - ref)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(d == 0, 0.0, d / np.abs(ref))
    return float(np.nanmax(r)) if r.size else 0.0


def oracle_cfg(cfg: B.AdamsConfig) -> oracle.AdamsCfg:
    """The same fp32 scalars for the oracle (field by field; no arithmetic)."""
    return oracle.AdamsCfg(n_keep=cfg.n_keep, m_group=cfg.m_group, lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2,
                           eps=cfg.eps, lambda_=cfg.lambda_, alpha=cfg.alpha, bias_corr1=cfg.bias_corr1,
                           bias_corr2=cfg.bias_corr2, refresh_mask=cfg.refresh_mask,
                           scale_segments=cfg.scale_segments, v_from_grad=int(bool(cfg.flags & B.FLAG_V_FROM_GRAD)),
                           rule=cfg.rule, mu_bf16=int(bool(cfg.flags & B.FLAG_MU_BF16)),
                           v_bf16=int(bool(cfg.flags & B.FLAG_V_BF16)), sr_seed=cfg.sr_seed)


class GpuState:
    """w, mu, v, mask (and optionally A, dL/dA) of one matrix on the GPU."""

    def __init__(self, w: np.ndarray, n_segments: int = 0, interleaved: bool = False, mu_bf16: bool = False,
                 v_bf16: bool = False):
        rows, cols = w.shape
        if interleaved:      # w, mu, v row-interleaved in one buffer: row stride 3 * cols (2.5 * cols with a bf16 mu, 2 * cols with both)
            self.w, self.m, self.v = B.interleaved_state(dev(w), mu_bf16=mu_bf16, v_bf16=v_bf16)
        else:
            self.w = dev(w)
            self.m = torch.zeros_like(self.w, dtype=torch.bfloat16 if mu_bf16 else torch.float32)
            self.v = torch.zeros_like(self.w, dtype=torch.bfloat16 if v_bf16 else torch.float32)
        self.mask = B.alloc_mask(rows, cols, DEV)
        self.scale_grad = torch.zeros((rows, n_segments), dtype=torch.float32, device=DEV) if n_segments else None

    def step(self, grad: torch.Tensor, cfg: B.AdamsConfig, scale=None):
        B.cast_adams_step(self.w, grad, self.m, self.v, self.mask, cfg, scale=scale,
                          scale_grad=self.scale_grad if scale is not None else None)


class OracleState:
    def __init__(self, w: np.ndarray, arithmetic: str):
        self.w = w.copy()
        self.m = np.zeros_like(w)
        self.v = np.zeros_like(w)
        self.keep = np.zeros(w.shape, np.uint8)
        self.arith = arithmetic
        # running maximum magnitude of every entry: the scale rounding errors are measured against
        self.scale = [np.abs(w).astype(np.float64), np.zeros(w.shape), np.zeros(w.shape)]
        # the double run also carries the derived bound on how far an fp32 run may have drifted from it (unscaled steps)
        self.drift = Fp32Drift(w.shape) if arithmetic == "f64" else None

    def step(self, grad_f32: np.ndarray, cfg: oracle.AdamsCfg, A=None, nthreads=8):
        entering = [x.copy() for x in (self.w, self.m, self.v)] if self.drift is not None and A is None else None
        gA = oracle.adams_step(self.w, grad_f32, self.m, self.v, self.keep, cfg, A=A, arithmetic=self.arith,
                               nthreads=nthreads)
        if entering is not None:
            self.drift.advance(*entering, grad_f32, self.keep, **self.drift.scalars(cfg))
        for i, x in enumerate((self.w, self.m, self.v)):
            np.maximum(self.scale[i], np.abs(x), out=self.scale[i])
        return gA


def stepped_in_pieces(segment_entries: int) -> bool:
    """Whether the list call steps row segments of this length in pieces (more than 8 chunks of 256 entries, 16
    chunks excepted), so that dL/dA is summed per piece first."""
    chunks = -(-segment_entries // 256)
    return chunks > 8 and chunks != 16
