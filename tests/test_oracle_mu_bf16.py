"""Pins for the oracle's storage variant that keeps the first moment in bf16 between iterations (not in
the paper: Algorithm 1 says nothing about how the moments are stored).  Its definition: the new mu is
rounded to nearest-even bf16 when stored, everything computed in the same iteration uses the unrounded
value.  The rounding itself is pinned against the tensor library's conversion."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import AdamsCfg
from paper_2509_25996_amd import synth


def _bf16_round(x: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def _cfg(t, total, **kw):
    alpha, bc1, bc2 = O.iteration_scalars(t, total, 0.9, 0.999)
    return AdamsCfg(lr=1e-3, lambda_=1e-3, alpha=alpha, bias_corr1=bc1, bias_corr2=bc2, **kw)


@pytest.mark.parametrize("arithmetic", ["f32", "f64"])
@pytest.mark.parametrize("nseg", [0, 2])
def test_one_step_from_a_bf16_moment_differs_only_in_what_is_stored(arithmetic, nseg):
    rows, cols = 12, 64
    w0 = synth.weights(31, 0, rows, cols)
    g = synth.grads_f32(31, 0, 0, rows, cols)
    mu0 = _bf16_round(synth.grads_f32(31, 0, 1, rows, cols))
    v0 = np.abs(synth.grads_f32(31, 0, 2, rows, cols)) * np.float32(1e-3)
    A = (1 + 0.1 * np.random.default_rng(0).standard_normal((rows, nseg))).astype(np.float32) if nseg else None
    out = {}
    for flag in (0, 1):
        w, mu, v = w0.copy(), mu0.copy(), v0.copy()
        keep = np.zeros((rows, cols), np.uint8)
        gA = O.adams_step(w, g, mu, v, keep, _cfg(4, 10, scale_segments=nseg, mu_bf16=flag), A=A, arithmetic=arithmetic)
        out[flag] = (w, mu, v, keep, gA)
    for k in (0, 2, 3):      # w, v and the mask: the same bits
        assert out[0][k].tobytes() == out[1][k].tobytes()
    if nseg:
        assert out[0][4].tobytes() == out[1][4].tobytes()
    assert out[1][1].tobytes() == _bf16_round(out[0][1]).tobytes()      # mu: the library's rounding of the fp32 result
    assert (out[1][1] != out[0][1]).any()


def test_stored_moment_is_always_bf16_and_follows_the_rounded_recurrence():
    # constant gradient, nothing masked (N = M is not allowed, so the decay is switched off with lambda = 0):
    # mu_t = bf16(b1 * mu_{t-1} + (1 - b1) * g) with fp32 products and sum, rounded by the library
    rows, cols, steps = 4, 32, 12
    g = synth.grads_f32(32, 0, 0, rows, cols)
    w, mu, v = synth.weights(32, 0, rows, cols), np.zeros((rows, cols), np.float32), np.zeros((rows, cols), np.float32)
    keep = np.zeros((rows, cols), np.uint8)
    want = np.zeros((rows, cols), np.float32)
    b1, c1 = np.float32(0.9), np.float32(1.0) - np.float32(0.9)
    for t in range(steps):
        cfg = _cfg(t, steps, mu_bf16=1)
        cfg.lambda_ = 0.0
        O.adams_step(w, g, mu, v, keep, cfg, arithmetic="f32")
        want = _bf16_round(b1 * want + c1 * g)
        assert mu.tobytes() == want.tobytes(), t
        assert (mu.view(np.uint32) & 0xFFFF == 0).all()


def test_bf16_moment_stays_close_to_the_fp32_one():
    # rounding error of one store is 2^-9 relative; with beta1 = 0.9 the accumulated error stays below
    # 2^-9 / (1 - beta1) of the largest moment seen
    rows, cols, steps = 16, 128, 30
    state = {}
    for flag in (0, 1):
        w, mu, v = synth.weights(33, 0, rows, cols), np.zeros((rows, cols), np.float32), np.zeros((rows, cols), np.float32)
        keep = np.zeros((rows, cols), np.uint8)
        for t in range(steps):
            O.adams_step(w, synth.grads_f32(33, 0, t, rows, cols), mu, v, keep, _cfg(t, steps, mu_bf16=flag, refresh_mask=int(t % 10 == 0)),
                         arithmetic="f32")
        state[flag] = (w, mu, v)
    scale = np.abs(state[0][1]).max()
    assert np.abs(state[0][1] - state[1][1]).max() <= 2.0 ** -9 / 0.1 * scale
    # the weights: single entries may part ways (a mask refresh that falls the other way), the bulk does not
    assert np.abs(state[0][0] - state[1][0]).mean() <= 1e-3 * 30 * 0.05      # a few percent of the total movement lr * steps


def test_frozen_entries_keep_their_bf16_moment():
    rows, cols = 4, 16
    w = synth.weights(34, 0, rows, cols)
    mu0 = _bf16_round(synth.grads_f32(34, 0, 1, rows, cols))
    mu, v = mu0.copy(), np.zeros((rows, cols), np.float32)
    keep = O.nm_select(w, 2, 4)
    cfg = _cfg(3, 10, mu_bf16=1, refresh_mask=0, rule=O.RULE_MASKED_FROZEN)
    O.adams_step(w, synth.grads_f32(34, 0, 0, rows, cols), mu, v, keep, cfg, arithmetic="f32")
    assert (mu[keep == 0] == mu0[keep == 0]).all() and (mu[keep == 1] != mu0[keep == 1]).any()
