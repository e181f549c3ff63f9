"""Pins for the oracle's comparison update rules: Eq. 9 (decay after the adaptive step), Eq. 10
(decay inside the gradient), additive decay on the momentum (Sec. 4.1.2) and sparsity-aware
fine-tuning (Sec. 6.7).  Each is checked against a library Adam, a closed form, or an invariant."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import AdamsCfg

B1, B2, EPS = 0.9, 0.999, 1e-8


def _bc(k):
    return 1.0 - B1 ** k, 1.0 - B2 ** k


def _adam(theta0, lr):
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    return p, torch.optim.Adam([p], lr=lr, betas=(B1, B2), eps=EPS, weight_decay=0.0)


def _step(oracle, th, g, mu, v, m_bits, k, rule, lr=1e-4, lam=1e-3, alpha=1.0):
    bc1, bc2 = _bc(k)
    oracle.adams_elements_state64(th, g.copy(), mu, v, m_bits, lr=lr, beta1=B1, beta2=B2, eps=EPS, lambda_=lam,
                                  alpha=alpha, bias_corr1=bc1, bias_corr2=bc2, rule=rule)


def test_eq9_is_library_adam_plus_a_sign_step_on_masked_entries(oracle):
    # Eq. 9: the moments never see the decay, so they are the library's; each step moves the
    # weight by the library's own step and, where the mask bit is 0, by -lr*alpha*lambda*Sign(w_prev)
    rng = np.random.default_rng(10)
    n, steps, lr, lam, alpha = 96, 12, 1e-4, 1e-3, 0.7
    theta0 = rng.standard_normal(n) * 0.02
    grads = [rng.standard_normal(n) * 1e-3 for _ in range(steps)]
    m_bits = (rng.random(n) < 0.5).astype(np.uint8)
    p, opt = _adam(theta0, lr)
    th, mu, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for k, g in enumerate(grads, 1):
        lib_before = p.detach().numpy().copy()
        p.grad = torch.tensor(g)
        opt.step()
        lib_step = p.detach().numpy() - lib_before
        prev = th.copy()
        _step(oracle, th, g, mu, v, m_bits, k, O.RULE_ADAMW_L1, lr=lr, lam=lam, alpha=alpha)
        np.testing.assert_allclose(mu, opt.state[p]["exp_avg"].numpy(), rtol=1e-13)
        np.testing.assert_allclose(v, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-13)
        expect = prev + lib_step - np.where(m_bits == 0, lr * alpha * lam * np.sign(prev), 0.0)
        np.testing.assert_allclose(th, expect, rtol=0, atol=1e-17)


def test_eq10_is_library_adam_fed_the_decayed_gradient(oracle):
    rng = np.random.default_rng(11)
    n, steps, lr, lam, alpha = 96, 12, 1e-4, 2e-3, 1.0
    theta0 = rng.standard_normal(n) * 0.002        # small weights: several cross zero and flip the decay's sign
    grads = [rng.standard_normal(n) * 1e-3 for _ in range(steps)]
    m_bits = (rng.random(n) < 0.5).astype(np.uint8)
    p, opt = _adam(theta0, lr)
    th, mu, v = theta0.copy(), np.zeros(n), np.zeros(n)
    crossed = 0
    for k, g in enumerate(grads, 1):
        w_prev = p.detach().numpy().copy()
        p.grad = torch.tensor(g + np.where(m_bits == 0, alpha * lam * np.sign(w_prev), 0.0))
        opt.step()
        _step(oracle, th, g, mu, v, m_bits, k, O.RULE_ADAM_L1, lr=lr, lam=lam, alpha=alpha)
        crossed += int((np.sign(th) != np.sign(w_prev)).sum())
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-16)
        np.testing.assert_allclose(mu, opt.state[p]["exp_avg"].numpy(), rtol=1e-12, atol=1e-20)
        np.testing.assert_allclose(v, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-12)
    assert crossed > 0


def test_additive_decay_closed_forms(oracle):
    # first step from a zero state: mu1 = (1-b1) g, mu~ = mu1 + alpha*lambda*s, v1 = (1-b2) mu~^2,
    # so w1 = w0 - lr * mu~ / ((1-b1) (|mu~| + eps)); the proportional rule has (1-alpha) mu1 instead of mu1
    g = np.array([1e-3, -2e-3, 5e-4, 0.0, -1e-6])
    w0 = np.array([0.02, -0.01, -0.03, 0.5, 0.0])
    lam, alpha, lr = 3e-3, 0.25, 1e-4
    for rule, keep_frac in ((O.RULE_ADDITIVE, 1.0), (O.RULE_ADAMS, 1.0 - alpha)):
        th, mu, v = w0.copy(), np.zeros(5), np.zeros(5)
        _step(oracle, th, g, mu, v, np.zeros(5, np.uint8), 1, rule, lr=lr, lam=lam, alpha=alpha)
        mt = keep_frac * (1 - B1) * g + alpha * lam * np.sign(w0)
        np.testing.assert_allclose(th, w0 - lr * mt / ((1 - B1) * (np.abs(mt) + EPS)), rtol=1e-12, atol=0)
        np.testing.assert_allclose(mu, (1 - B1) * g, rtol=1e-15)
    # with lambda = 0 nothing is added: masked entries move exactly like kept ones (not so under Eq. 7,
    # whose (1 - alpha) factor attenuates them)
    rng = np.random.default_rng(12)
    n = 64
    theta0, g1 = rng.standard_normal(n) * 0.02, rng.standard_normal(n) * 1e-3
    res = []
    for bits in (np.zeros(n, np.uint8), np.ones(n, np.uint8)):
        th, mu, v = theta0.copy(), np.abs(rng.standard_normal(n)) * 0 + 1e-4, np.full(n, 1e-7)
        _step(oracle, th, g1, mu, v, bits, 5, O.RULE_ADDITIVE, lam=0.0, alpha=0.6)
        res.append((th.copy(), mu.copy(), v.copy()))
    for a, b in zip(*res):
        assert (a == b).all()


def test_additive_pure_decay_matches_proportional_when_momentum_is_zero(oracle):
    # g = 0 from a zero state: mu stays 0, so (1-alpha)*mu vanishes and both rules follow
    # w_k = w_{k-1} - lr*s*a / ((1-b1^k)(a+eps)), a = alpha*lambda
    lam, alpha, lr = 1e-3, 0.5, 1e-4
    w0 = np.array([0.02, -0.015, 0.0, 0.05])
    a = alpha * lam
    for rule in (O.RULE_ADDITIVE, O.RULE_ADAMS):
        th, mu, v = w0.copy(), np.zeros(4), np.zeros(4)
        expect = w0.copy()
        for k in range(1, 15):
            _step(oracle, th, np.zeros(4), mu, v, np.zeros(4, np.uint8), k, rule, lr=lr, lam=lam, alpha=alpha)
            expect = expect - lr * np.sign(expect) * a / (_bc(k)[0] * (a + EPS))
            np.testing.assert_allclose(th, expect, rtol=1e-12, atol=1e-18)


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_frozen_rule_touches_only_kept_entries(oracle, arith):
    rng = np.random.default_rng(13)
    rows, cols = 6, 64
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    g = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    mu = (rng.standard_normal((rows, cols)) * 1e-4).astype(np.float32)
    v = (rng.random((rows, cols)) * 1e-7).astype(np.float32)
    keep = oracle.nm_select(w, 2, 4)
    runs = {}
    for rule in (O.RULE_MASKED_FROZEN, O.RULE_ADAMS):
        s = [x.copy() for x in (w, mu, v)]
        cfg = AdamsCfg(lr=1e-3, lambda_=1e-3, alpha=0.5, bias_corr1=0.3, bias_corr2=0.01, refresh_mask=0, rule=rule)
        oracle.adams_step(s[0], g, s[1], s[2], keep.copy(), cfg, arithmetic=arith)
        runs[rule] = s
    fr, ad = runs[O.RULE_MASKED_FROZEN], runs[O.RULE_ADAMS]
    masked, kept = keep == 0, keep == 1
    for got, before, other in zip(fr, (w, mu, v), ad):
        assert (got[masked] == before[masked]).all()           # not updated at all
        assert (got[kept] == other[kept]).all()                # Eq. 8 with mu~ = mu
    assert (fr[0][kept] != w[kept]).any()


@pytest.mark.parametrize("rule", [O.RULE_ADAMW_L1, O.RULE_ADAM_L1, O.RULE_ADDITIVE, O.RULE_MASKED_FROZEN])
def test_rules_fp32_arithmetic_close_to_double(oracle, rule):
    # the per-operation fp32 variant of every rule follows the double one (a wrong operand or a
    # dropped term in either shows up as an error far above fp32 rounding)
    rng = np.random.default_rng(20 + rule)
    rows, cols = 8, 128
    w0 = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    state = {a: [w0.copy(), np.zeros_like(w0), np.zeros_like(w0), np.zeros(w0.shape, np.uint8)] for a in ("f64", "f32")}
    for k in range(1, 9):
        g = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
        bc1, bc2 = _bc(k)
        for a, (w, mu, v, keep) in state.items():
            cfg = AdamsCfg(lr=1e-4, lambda_=2e-6, alpha=k / 8, bias_corr1=bc1, bias_corr2=bc2, refresh_mask=int(k == 1),
                           rule=rule)
            oracle.adams_step(w, g, mu, v, keep, cfg, arithmetic=a)
    (w64, m64, v64, k64), (w32, m32, v32, k32) = state["f64"], state["f32"]
    assert (k64 == k32).all()
    assert np.abs(w64.astype(np.float64) - w32).max() <= 1e-6 * np.abs(w64).max()
    assert np.abs(m64.astype(np.float64) - m32).max() <= 1e-6 * np.abs(m64).max()
    assert np.abs(v64.astype(np.float64) - v32).max() <= 1e-6 * np.abs(v64).max()


def test_unknown_rule_is_rejected(oracle):
    w = np.zeros((1, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.adams_step(w, w.copy(), w.copy(), w.copy(), np.zeros((1, 4), np.uint8), AdamsCfg(rule=9))
