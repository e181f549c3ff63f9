"""Pins for the oracle's AdamS iteration (Algorithm 1, Eq. 7, Eq. 8).

Each test checks the oracle against something that is not the oracle: a library Adam,
a closed form worked out by hand from Eq. 8, or an invariant the paper states."""
import numpy as np
import pytest
import torch

from fp32_bound import Fp32Drift
from oracle import AdamsCfg, iteration_scalars

B1, B2, EPS = 0.9, 0.999, 1e-8


def _bc(k):
    return 1.0 - B1 ** k, 1.0 - B2 ** k


def _library_adam(theta0, grads, lr):
    """torch.optim.Adam in float64: returns per-step (theta, exp_avg, exp_avg_sq)."""
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=lr, betas=(B1, B2), eps=EPS, weight_decay=0.0)
    out = []
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        st = opt.state[p]
        out.append((p.detach().numpy().copy(), st["exp_avg"].numpy().copy(), st["exp_avg_sq"].numpy().copy()))
    return out


def test_first_moment_is_library_adam_exp_avg_even_with_decay(oracle):
    # Algorithm 1 stores mu_t, not the decayed mu~_t: its recursion is Adam's (Eq. 8, first line)
    rng = np.random.default_rng(0)
    n, steps = 64, 12
    theta0 = rng.standard_normal(n) * 0.02
    grads = [rng.standard_normal(n) * 1e-3 for _ in range(steps)]
    ref = _library_adam(theta0, grads, 1e-4)
    th, mu, v = theta0.copy(), np.zeros(n), np.zeros(n)
    m_bits = (rng.random(n) < 0.5).astype(np.uint8)
    for k, g in enumerate(grads, 1):
        bc1, bc2 = _bc(k)
        oracle.adams_elements_state64(th, g.copy(), mu, v, m_bits, lr=1e-4, beta1=B1, beta2=B2, eps=EPS,
                                      lambda_=1e-3, alpha=k / steps, bias_corr1=bc1, bias_corr2=bc2)
        np.testing.assert_allclose(mu, ref[k - 1][1], rtol=1e-13, atol=0)


def test_textbook_form_equals_library_adam(oracle):
    # alpha = 0 and the second moment fed g^2 (Eq. 9 with lambda = 0) is plain Adam
    rng = np.random.default_rng(1)
    n, steps = 128, 10
    theta0 = rng.standard_normal(n) * 0.02
    grads = [rng.standard_normal(n) * 1e-3 for _ in range(steps)]
    ref = _library_adam(theta0, grads, 1e-4)
    th, mu, v = theta0.copy(), np.zeros(n), np.zeros(n)
    m_bits = (rng.random(n) < 0.5).astype(np.uint8)
    for k, g in enumerate(grads, 1):
        bc1, bc2 = _bc(k)
        oracle.adams_elements_state64(th, g.copy(), mu, v, m_bits, lr=1e-4, beta1=B1, beta2=B2, eps=EPS,
                                      lambda_=1e-3, alpha=0.0, bias_corr1=bc1, bias_corr2=bc2, v_from_grad=1)
        np.testing.assert_allclose(th, ref[k - 1][0], rtol=1e-12, atol=0)
        np.testing.assert_allclose(mu, ref[k - 1][1], rtol=1e-12, atol=0)
        np.testing.assert_allclose(v, ref[k - 1][2], rtol=1e-12, atol=0)


def test_paper_form_alpha0_is_adam_with_v_fed_by_momentum(oracle):
    # Eq. 8 at alpha = 0: v accumulates mu_t^2.  Independent check through the library Adam:
    # its exp_avg_sq recursion applied to the sequence mu_t (fed as "gradients") gives v_t.
    rng = np.random.default_rng(2)
    n, steps = 32, 8
    theta0 = rng.standard_normal(n) * 0.02
    grads = [rng.standard_normal(n) * 1e-3 for _ in range(steps)]
    mus = [m for (_, m, _) in _library_adam(theta0, grads, 1e-4)]
    v_ref = [s for (_, _, s) in _library_adam(theta0, mus, 1e-4)]
    th, mu, v = theta0.copy(), np.zeros(n), np.zeros(n)
    keep_all = np.ones(n, np.uint8)
    for k, g in enumerate(grads, 1):
        bc1, bc2 = _bc(k)
        prev = th.copy()
        oracle.adams_elements_state64(th, g.copy(), mu, v, keep_all, lr=1e-4, beta1=B1, beta2=B2, eps=EPS,
                                      lambda_=5e-4, alpha=0.0, bias_corr1=bc1, bias_corr2=bc2)
        np.testing.assert_allclose(v, v_ref[k - 1], rtol=1e-12, atol=0)
        expect = prev - 1e-4 * (mus[k - 1] / bc1) / (np.sqrt(v_ref[k - 1] / bc2) + EPS)
        np.testing.assert_allclose(th, expect, rtol=1e-13, atol=0)


def test_first_step_closed_forms(oracle):
    # zero state, alpha = 0:  paper form  w1 = w0 - lr*g / ((1-b1)|g| + eps);  textbook form  w1 = w0 - lr*g/(|g|+eps)
    g = np.array([1e-3, -2e-3, 5e-4, 0.0, -1e-6])
    w0 = np.array([0.02, -0.01, 0.03, 0.5, -0.25])
    for vfg, denom in ((0, (1 - B1) * np.abs(g) + EPS), (1, np.abs(g) + EPS)):
        th, mu, v = w0.copy(), np.zeros(5), np.zeros(5)
        oracle.adams_elements_state64(th, g.copy(), mu, v, np.zeros(5, np.uint8), lr=1e-4, beta1=B1, beta2=B2,
                                      eps=EPS, lambda_=1.0, alpha=0.0, bias_corr1=1 - B1, bias_corr2=1 - B2,
                                      v_from_grad=vfg)
        np.testing.assert_allclose(th, w0 - 1e-4 * g / denom, rtol=1e-12, atol=0)


def test_masked_entries_closed_form_pure_decay(oracle):
    # g = 0, alpha = 1, zero state: mu = 0, mu~ = lambda*sign(w), v_k = (1-b2^k) lambda^2, v^ = lambda^2,
    # so w_k = w_{k-1} - lr * sign(w) * lambda / ((1-b1^k)(lambda+eps)); kept entries never move.
    lam, lr = 1e-3, 1e-4
    w0 = np.array([0.02, -0.015, 0.01, -0.03, 0.0, 0.05])
    m_bits = np.array([0, 0, 1, 1, 0, 0], np.uint8)
    th, mu, v = w0.copy(), np.zeros(6), np.zeros(6)
    expect = w0.copy()
    for k in range(1, 21):
        bc1, bc2 = _bc(k)
        oracle.adams_elements_state64(th, np.zeros(6), mu, v, m_bits, lr=lr, beta1=B1, beta2=B2, eps=EPS,
                                      lambda_=lam, alpha=1.0, bias_corr1=bc1, bias_corr2=bc2)
        expect = np.where(m_bits == 0, expect - lr * np.sign(expect) * lam / (bc1 * (lam + EPS)), expect)
        np.testing.assert_allclose(th, expect, rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(v, np.where(m_bits == 0, bc2 * lam * lam, 0.0) * (w0 != 0), rtol=1e-12, atol=0)
        assert (mu == 0).all()
    assert (th[m_bits == 1] == w0[m_bits == 1]).all()      # kept: bit for bit unchanged
    assert th[4] == 0.0                                      # Sign(0) = 0: an exact zero stays
    assert abs(th[0]) < abs(w0[0]) and abs(th[1]) < abs(w0[1])  # decay points toward zero for both signs


def test_alpha_one_lambda_zero_freezes_masked(oracle):
    # (1 - alpha) also attenuates the momentum of masked entries: at alpha = 1, lambda = 0 they stop moving
    rng = np.random.default_rng(3)
    n = 16
    th0 = rng.standard_normal(n)
    th, mu, v = th0.copy(), rng.standard_normal(n) * 1e-3, np.abs(rng.standard_normal(n)) * 1e-6
    v0 = v.copy()
    m_bits = np.zeros(n, np.uint8)
    oracle.adams_elements_state64(th, rng.standard_normal(n), mu, v, m_bits, lr=1e-2, beta1=B1, beta2=B2, eps=EPS,
                                  lambda_=0.0, alpha=1.0, bias_corr1=0.5, bias_corr2=0.5)
    assert (th == th0).all()
    np.testing.assert_allclose(v, B2 * v0, rtol=1e-15)


def _random_state(rng, rows, cols):
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    g = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    mu = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    v = (np.abs(rng.standard_normal((rows, cols))) * 1e-6).astype(np.float32)
    return w, g, mu, v


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_kept_entries_receive_no_decay(oracle, arith):
    # Algorithm 1: m = 1  =>  mu~ = mu.  Kept outputs are bit-identical with and without decay.
    rng = np.random.default_rng(4)
    w, g, mu, v = _random_state(rng, 8, 64)
    keep = oracle.nm_select(w, 2, 4)
    outs = []
    for lam, alpha in ((1e-3, 0.7), (0.0, 0.0)):
        a, b, c = w.copy(), mu.copy(), v.copy()
        cfg = AdamsCfg(lambda_=lam, alpha=alpha, bias_corr1=0.5, bias_corr2=0.1, refresh_mask=0)
        oracle.adams_step(a, g, b, c, keep.copy(), cfg, arithmetic=arith)
        outs.append((a, b, c))
    k = keep.astype(bool)
    for x, y in zip(outs[0], outs[1]):
        assert (x[k].view(np.uint32) == y[k].view(np.uint32)).all()
    assert (outs[0][0][~k] != outs[1][0][~k]).any()          # and masked ones do differ
    assert (outs[0][1].view(np.uint32) == outs[1][1].view(np.uint32)).all()  # stored mu never sees decay


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_exact_zero_masked_weight_stays_zero(oracle, arith):
    # Sign(0) = 0 for both zeros: with no gradient and no momentum a masked zero receives no decay and stays
    # put under full decay strength, while its nonzero neighbours move toward zero
    w = np.array([[0.0, -0.0, 0.5, -0.5, 0.0, -0.0, 0.25, -0.25]], np.float32)
    keep = np.array([[0, 0, 1, 1, 0, 0, 0, 0]], np.uint8)
    a, mu, v = w.copy(), np.zeros_like(w), np.zeros_like(w)
    cfg = AdamsCfg(lr=1e-2, lambda_=1e-3, alpha=1.0, bias_corr1=0.1, bias_corr2=0.001, refresh_mask=0)
    oracle.adams_step(a, np.zeros_like(w), mu, v, keep, cfg, arithmetic=arith)
    assert (a[0, [0, 1, 4, 5]] == 0.0).all() and (v[0, [0, 1, 4, 5]] == 0.0).all()
    assert (a[0, 2:4] == w[0, 2:4]).all()                            # kept, no gradient: untouched
    assert 0 < a[0, 6] < 0.25 and -0.25 < a[0, 7] < 0               # masked and nonzero: toward zero


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_alpha_zero_ignores_the_mask(oracle, arith):
    rng = np.random.default_rng(5)
    w, g, mu, v = _random_state(rng, 4, 32)
    res = []
    for keep in (np.ones_like(w, dtype=np.uint8), np.zeros_like(w, dtype=np.uint8)):
        a, b, c = w.copy(), mu.copy(), v.copy()
        cfg = AdamsCfg(lambda_=1e-3, alpha=0.0, bias_corr1=0.3, bias_corr2=0.01, refresh_mask=0)
        oracle.adams_step(a, g, b, c, keep, cfg, arithmetic=arith)
        res.append((a, b, c))
    for x, y in zip(*res):
        assert (x.view(np.uint32) == y.view(np.uint32)).all()


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_matrix_step_agrees_with_elementwise_double_state(oracle, arith):
    # the matrix-level function (fp32 storage) against the flat double-state body pinned above
    rng = np.random.default_rng(6)
    w, g, mu, v = _random_state(rng, 6, 48)
    keep = oracle.nm_select(w, 2, 4)
    cfg = AdamsCfg(lr=1e-4, lambda_=1e-3, alpha=0.4, bias_corr1=0.65, bias_corr2=0.004, refresh_mask=0)
    th, m1, v1 = (x.astype(np.float64).ravel().copy() for x in (w, mu, v))
    f = lambda x: float(np.float32(x))
    oracle.adams_elements_state64(th, g.astype(np.float64).ravel(), m1, v1, keep.ravel(), lr=f(1e-4), beta1=f(B1),
                                  beta2=f(B2), eps=f(EPS), lambda_=f(1e-3), alpha=f(0.4), bias_corr1=f(0.65),
                                  bias_corr2=f(0.004))
    a, b, c = w.copy(), mu.copy(), v.copy()
    oracle.adams_step(a, g, b, c, keep.copy(), cfg, arithmetic=arith)
    tol = 0 if arith == "f64" else 1e-6
    for got, ref in ((a, th), (c, v1)):
        ref32 = ref.astype(np.float32).reshape(got.shape)
        if arith == "f64":
            assert (got.view(np.uint32) == ref32.view(np.uint32)).all()
        else:
            np.testing.assert_allclose(got, ref32, rtol=tol, atol=0)
    # mu may cancel: bound the error by the size of its terms instead of its value
    err = np.abs(b.astype(np.float64).ravel() - m1)
    assert (err <= 2e-7 * (np.abs(mu).ravel() + np.abs(g).ravel())).all()


@pytest.mark.parametrize("lr", [1e-4, 1e-2])
@pytest.mark.parametrize("lam", [2e-6, 1e-3])
def test_fp32_arithmetic_stays_within_its_derived_bound_of_double_over_10_steps(oracle, lam, lr):
    # fp32-per-operation against double arithmetic on the same fp32 storage: after every iteration every entry of
    # w, mu, v lies within the bound that tests/fp32_bound.py derives from the roundings of Eq. 7-8, operation by
    # operation, entry by entry (including the entries whose decayed momentum cancels while v is still small,
    # where mu^/sqrt(v^) turns rounding noise into up to 2*sqrt(bc2/(1-beta2))/bc1 steps of size lr).
    # Besides that the tolerance the workload states (1e-6 after 10 steps) is asserted at the paper's lambda
    # (Table 11), measured against each entry's running maximum magnitude: a masked weight driven through zero,
    # or a momentum that cancels, keeps the absolute error of its earlier, larger self, so a relative error
    # against the current value is unbounded for any fp32 implementation.
    rng = np.random.default_rng(7)
    rows, cols, steps = 32, 256, 10
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    st = {a: (w.copy(), np.zeros_like(w), np.zeros_like(w), np.zeros(w.shape, np.uint8)) for a in ("f64", "f32")}
    scale = [np.abs(w).astype(np.float64), np.zeros(w.shape), np.zeros(w.shape)]
    drift = Fp32Drift(w.shape)
    for t in range(steps):
        g = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
        alpha, bc1, bc2 = iteration_scalars(t, steps, B1, B2)
        cfg = AdamsCfg(lr=lr, lambda_=lam, alpha=alpha, bias_corr1=bc1, bias_corr2=bc2, refresh_mask=int(t % 5 == 0))
        entering = [x.copy() for x in st["f64"][:3]]
        for a in st:
            wa, ma, va, ka = st[a]
            oracle.adams_step(wa, g, ma, va, ka, cfg, arithmetic=a)
        assert (st["f64"][3] == st["f32"][3]).all()
        drift.advance(*entering, g, st["f64"][3], **drift.scalars(cfg))
        for i, bound in enumerate((drift.E_w, drift.E_mu, drift.E_v)):
            err = np.abs(st["f32"][i].astype(np.float64) - st["f64"][i])
            assert (err <= bound).all(), (t, i, float((err / np.maximum(bound, 1e-300)).max()))
            scale[i] = np.maximum(scale[i], np.abs(st["f64"][i]))
    if lam == 2e-6 and lr == 1e-4:
        for i, bound in enumerate((drift.E_w, drift.E_mu, drift.E_v)):
            err = np.abs(st["f32"][i].astype(np.float64) - st["f64"][i])
            assert (err <= 1e-6 * scale[i]).all(), (i, (err / scale[i]).max())
            # the bound is worst-case (every rounding in the same direction for 10 iterations) but not vacuous:
            # it stays within about ten stated tolerances of every entry's magnitude
            assert (bound <= 1e-5 * scale[i]).all(), (i, (bound / scale[i]).max())
    # and the naive per-value relative error does blow up on the cancelling entries, which is why it is not used
    rel_w = np.abs(st["f32"][0].astype(np.float64) - st["f64"][0]) / np.abs(st["f64"][0])
    assert rel_w.max() > 1e-6


def test_refresh_uses_weights_before_the_update(oracle):
    # a large step reorders the magnitudes; the stored mask must be that of the incoming weights
    w = np.array([[1.0, 0.9, 0.5, 0.1]], np.float32)
    g = np.array([[10.0, 0.0, -10.0, 0.0]], np.float32)
    keep = np.zeros((1, 4), np.uint8)
    a, mu, v = w.copy(), np.zeros_like(w), np.zeros_like(w)
    cfg = AdamsCfg(lr=0.8, lambda_=0.0, alpha=0.0, bias_corr1=0.1, bias_corr2=0.001, refresh_mask=1)
    oracle.adams_step(a, g, mu, v, keep, cfg)
    assert keep.tolist() == [[1, 1, 0, 0]]
    assert (oracle.nm_select(a, 2, 4) != keep).any()         # the updated weights would give another mask


def test_masked_weights_end_near_zero_under_the_ramp(oracle):
    # Sec. 4.1 / Appendix "Mask Learning": with alpha ramped to 1 masked weights are driven to
    # (an O(lr) band around) zero and the kept-mass ratio S_t goes to 1.
    rng = np.random.default_rng(8)
    rows, cols, steps, lr, lam = 16, 64, 1500, 1e-3, 1e-3
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    mu, v, keep = np.zeros_like(w), np.zeros_like(w), np.zeros(w.shape, np.uint8)
    for t in range(steps):
        g = (rng.standard_normal((rows, cols)) * 1e-4).astype(np.float32)
        alpha, bc1, bc2 = iteration_scalars(t, steps, B1, B2)
        cfg = AdamsCfg(lr=lr, lambda_=lam, alpha=alpha, bias_corr1=bc1, bias_corr2=bc2, refresh_mask=int(t % 10 == 0))
        oracle.adams_step(w, g, mu, v, keep, cfg, arithmetic="f32")
    masked = np.abs(w[keep == 0])
    assert masked.max() <= 4 * lr, masked.max()
    _, kept_l1, total_l1 = oracle.mask_stats(w, keep)
    assert kept_l1 / total_l1 > 0.97


def test_iteration_scalars_reading():
    a, bc1, bc2 = iteration_scalars(0, 100, B1, B2)
    assert a == 0.0
    assert bc1 == float(np.float32(1 - float(np.float32(B1))))
    a, _, _ = iteration_scalars(50, 100, B1, B2)
    assert a == 0.5
