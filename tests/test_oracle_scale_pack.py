"""Pins for the oracle's weight scaling (Eq. 11, Eq. 12), hard prune + fold + pack, bf16
rounding and the mask statistics of the appendix "Mask Learning"."""
import numpy as np
import pytest
import torch

from oracle import AdamsCfg

NM = [(1, 2), (2, 4), (1, 4), (3, 4), (4, 8), (2, 8), (7, 8)]


# ---------------------------------------------------------------- Eq. 12
def test_scale_is_the_reshape_of_eq12(oracle):
    # independent statement of Eq. 12: reshape (R, C) -> (R*n, C/n), multiply row i by a~_i, reshape back
    rng = np.random.default_rng(0)
    for rows, cols, n in [(4, 16, 2), (3, 24, 4), (5, 8, 1), (2, 12, 3)]:
        w = rng.standard_normal((rows, cols)).astype(np.float32)
        A = (1 + 0.1 * rng.standard_normal((rows, n))).astype(np.float32)
        expect = (w.reshape(rows * n, cols // n) * A.reshape(rows * n, 1)).reshape(rows, cols)
        assert (oracle.weight_scale(w, A).view(np.uint32) == expect.view(np.uint32)).all()
    # n = 1 is Eq. 11: Diag(A) W
    w = rng.standard_normal((6, 10)).astype(np.float32)
    A = rng.standard_normal((6, 1)).astype(np.float32)
    assert (oracle.weight_scale(w, A) == (np.diag(A[:, 0]) @ w).astype(np.float32)).all()


def test_scale_grad_by_finite_differences(oracle):
    # L(A) = 1/2 || Diag(A~) W~ - Y ||^2 ; dL/dW_scale = W_scale - Y ; check dL/dA numerically
    rng = np.random.default_rng(1)
    rows, cols, n = 3, 16, 2
    w = rng.standard_normal((rows, cols)).astype(np.float32)
    y = rng.standard_normal((rows, cols)).astype(np.float32)
    A = (1 + 0.2 * rng.standard_normal((rows, n))).astype(np.float32)

    def loss(Aq):
        ws = (w.astype(np.float64).reshape(rows * n, -1) * Aq.reshape(rows * n, 1)).reshape(rows, cols)
        return 0.5 * ((ws - y) ** 2).sum()

    G = (oracle.weight_scale(w, A).astype(np.float64) - y).astype(np.float32)
    gA = oracle.weight_scale_grad(w, G, n)
    h = 1e-3
    for r in range(rows):
        for s in range(n):
            Ap, Am = A.astype(np.float64).copy(), A.astype(np.float64).copy()
            Ap[r, s] += h
            Am[r, s] -= h
            fd = (loss(Ap) - loss(Am)) / (2 * h)   # exact for a quadratic up to rounding
            assert abs(fd - gA[r, s]) <= 1e-5 * max(1.0, abs(fd))


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_step_with_unit_scale_is_the_unscaled_step(oracle, arith):
    # A initialised to 1 (Algorithm 2) makes Eq. 12 the identity
    rng = np.random.default_rng(2)
    rows, cols = 6, 64
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    g = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    mu = (rng.standard_normal((rows, cols)) * 1e-4).astype(np.float32)
    v = (np.abs(rng.standard_normal((rows, cols))) * 1e-7).astype(np.float32)
    res = []
    for n in (0, 2):
        a, b, c, k = w.copy(), mu.copy(), v.copy(), np.zeros(w.shape, np.uint8)
        cfg = AdamsCfg(lambda_=1e-3, alpha=0.3, bias_corr1=0.5, bias_corr2=0.02, refresh_mask=1, scale_segments=n)
        A = np.ones((rows, n), np.float32) if n else None
        gA = oracle.adams_step(a, g, b, c, k, cfg, A=A, arithmetic=arith)
        res.append((a, b, c, k))
    for x, y in zip(*res):
        assert (x.view(np.uint8) == y.view(np.uint8)).all()
    assert np.allclose(gA, oracle.weight_scale_grad(w, g, 2), rtol=1e-15)


@pytest.mark.parametrize("arith", ["f64", "f32"])
def test_step_chain_rule_power_of_two_scale(oracle, arith):
    # dL/dW = a * dL/dW_scale: with a = 2 or 1/4 (exact in binary) the scaled step equals the
    # unscaled step on a gradient multiplied by the same factor beforehand, bit for bit
    rng = np.random.default_rng(3)
    rows, cols, n = 4, 32, 2
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    g = (rng.standard_normal((rows, cols)) * 1e-3).astype(np.float32)
    A = np.array([[2.0, 0.25]] * rows, np.float32)
    g_pre = g.copy()
    g_pre[:, : cols // 2] *= 2.0
    g_pre[:, cols // 2:] *= 0.25
    res = []
    for grad, scale, nseg in ((g, A, n), (g_pre, None, 0)):
        a, b, c, k = w.copy(), np.zeros_like(w), np.zeros_like(w), np.zeros(w.shape, np.uint8)
        cfg = AdamsCfg(lambda_=1e-3, alpha=0.5, bias_corr1=0.1, bias_corr2=0.001, refresh_mask=1, scale_segments=nseg)
        oracle.adams_step(a, grad, b, c, k, cfg, A=scale, arithmetic=arith)
        res.append((a, b, c, k))
    for x, y in zip(*res):
        assert (x.view(np.uint8) == y.view(np.uint8)).all()
    # dL/dA of the scaled step is the sum over the incoming gradient times the raw weight (the function pinned
    # by finite differences above), whatever A is: not times the scaled weight, not times the chained gradient
    a, b, c, k = w.copy(), np.zeros_like(w), np.zeros_like(w), np.zeros(w.shape, np.uint8)
    cfg = AdamsCfg(lambda_=1e-3, alpha=0.5, bias_corr1=0.1, bias_corr2=0.001, refresh_mask=1, scale_segments=n)
    gA = oracle.adams_step(a, g, b, c, k, cfg, A=A, arithmetic=arith)
    assert np.allclose(gA, oracle.weight_scale_grad(w, g, n), rtol=1e-14, atol=0)


def test_mask_is_taken_from_unscaled_weights(oracle):
    # a scale that differs between segments cannot move an entry across groups, but rounding
    # could create ties; the mask is defined on the raw weights
    w = np.array([[1.0, 1.0000001, 0.5, 0.25, 3.0, 2.0, 1.0, 0.0]], np.float32)
    A = np.array([[1e-30, 1.0]], np.float32)
    cfg = AdamsCfg(refresh_mask=1, scale_segments=2, alpha=0.0)
    keep = np.zeros(w.shape, np.uint8)
    oracle.adams_step(w.copy(), np.zeros_like(w), np.zeros_like(w), np.zeros_like(w), keep, cfg, A=A)
    assert (keep == oracle.nm_select(w, 2, 4)).all()


# ---------------------------------------------------------------- prune + fold + pack
def _decode(values, meta, cols, n, m):
    """Independent decoder of the packed layout (written from its description, not from the
    oracle's packer): rebuilds the dense pruned matrix and the mask."""
    b = {2: 1, 4: 2, 8: 3}[m]
    f = 1
    while f < n * b:
        f *= 2
    gpw = 32 // f
    rows = values.shape[0]
    dense = np.zeros((rows, cols), np.float32)
    keep = np.zeros((rows, cols), np.uint8)
    used = np.zeros_like(meta)
    for r in range(rows):
        for i in range(cols // m):
            word = int(meta[r, i // gpw])
            shift = (i % gpw) * f
            field = (word >> shift) & ((1 << f) - 1)
            used[r, i // gpw] |= np.uint32(((1 << (n * b)) - 1) << shift)
            prev = -1
            for q in range(n):
                j = (field >> (q * b)) & ((1 << b) - 1)
                assert j > prev, "indices must ascend inside a group"
                prev = j
                dense[r, i * m + j] = values[r, i * n + q]
                keep[r, i * m + j] = 1
    assert ((meta & ~used) == 0).all(), "padding bits must be zero"
    return dense, keep


@pytest.mark.parametrize("n,m", NM)
def test_pack_roundtrip_is_the_masked_matrix(oracle, n, m):
    rng = np.random.default_rng(10 * n + m)
    rows, cols = 5, 24 * m
    w = np.round(rng.standard_normal((rows, cols)) * 3).astype(np.float32) / 4  # ties and zeros
    values, meta = oracle.project_compress(w, n, m)
    assert values.shape == (rows, cols // m * n)
    dense, keep = _decode(values, meta, cols, n, m)
    assert (keep.reshape(rows, -1, m).sum(-1) == n).all()           # Eq. 4
    ref_keep = oracle.nm_select(w, n, m)
    assert (keep == ref_keep).all()
    assert (dense.view(np.uint32) == (w * ref_keep).view(np.uint32)).all() or \
        np.array_equal(dense, np.where(ref_keep == 1, w, np.float32(0)))   # W (.) M, Eq. 1


def test_pack_2of4_field_values_by_hand(oracle):
    # 2:4: b = 2 bits per index, field = 4 bits, 8 groups per word, first kept index in the low bits
    w = np.zeros((1, 32), np.float32)
    kept = [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3), (0, 1), (2, 3)]
    for i, (a, b) in enumerate(kept):
        w[0, 4 * i + a] = 1.0 + i
        w[0, 4 * i + b] = -(2.0 + i)
    values, meta = oracle.project_compress(w, 2, 4)
    word = 0
    for i, (a, b) in enumerate(kept):
        word |= (a | (b << 2)) << (4 * i)
    assert meta.tolist() == [[word]]
    assert values[0].tolist() == [x for i in range(8) for x in (1.0 + i, -(2.0 + i))]
    # 4:8: b = 3, 12 bits padded to 16, two groups per word
    w8 = np.zeros((1, 16), np.float32)
    w8[0, [1, 2, 5, 7]] = [1, 2, 3, 4]
    w8[0, [8, 9, 10, 15]] = [5, 6, 7, 8]
    values, meta = oracle.project_compress(w8, 4, 8)
    f0 = 1 | (2 << 3) | (5 << 6) | (7 << 9)
    f1 = 0 | (1 << 3) | (2 << 6) | (7 << 9)
    assert meta.tolist() == [[f0 | (f1 << 16)]]
    assert values[0].tolist() == [1, 2, 3, 4, 5, 6, 7, 8]
    # 1:2: one bit per group, 32 groups per word
    w2 = np.array([[1.0, 0.5] * 3 + [0.5, 1.0] * 2], np.float32)
    values, meta = oracle.project_compress(w2, 1, 2)
    assert meta.tolist() == [[0b11000]]
    assert values[0].tolist() == [1.0] * 5


def test_pack_folds_the_scale_and_keeps_the_pattern(oracle):
    # Sec. 4.2: scaling is elementwise, so the pattern is that of the raw weights and the fold is exact
    rng = np.random.default_rng(4)
    rows, cols, n = 6, 64, 2
    w = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    A = (1 + 0.3 * rng.standard_normal((rows, n))).astype(np.float32)
    values, meta = oracle.project_compress(w, 2, 4, A=A)
    dense, keep = _decode(values, meta, cols, 2, 4)
    assert (keep == oracle.nm_select(w, 2, 4)).all()
    expect = oracle.weight_scale(w, A) * keep
    assert np.array_equal(dense, expect)
    assert (np.count_nonzero(dense.reshape(rows, -1, 4), axis=-1) <= 2).all()


def test_pack_with_a_given_mask_is_algorithm1_literal(oracle):
    # Algorithm 1's last loop multiplies by the last refreshed mask, which need not be the top-N of the final weights
    w = np.array([[0.1, 0.9, 0.8, 0.2]], np.float32)
    keep = np.array([[1, 0, 0, 1]], np.uint8)
    values, meta = oracle.project_compress(w, 2, 4, keep=keep)
    assert values.tolist() == [[np.float32(0.1), np.float32(0.2)]]
    assert meta.tolist() == [[0 | (3 << 2)]]
    with pytest.raises(ValueError):
        oracle.project_compress(w, 2, 4, keep=np.array([[1, 1, 1, 0]], np.uint8))


def test_bf16_rounding_is_the_library_conversion(oracle):
    rng = np.random.default_rng(5)
    x = rng.standard_normal(20000).astype(np.float32) * np.float32(0.02)
    bits = rng.integers(0, 2 ** 32, 20000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, 3.3895314e38, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8],
                       np.float32)
    allx = np.concatenate([x, bits.view(np.float32), special])
    ref = torch.from_numpy(allx.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.bf16_rne(allx)
    nan = np.isnan(allx)
    assert (got[~nan] == ref[~nan]).all()
    assert (got[nan] == 0x7FC0).all()


# ---------------------------------------------------------------- appendix statistics
def test_mask_stats_against_numpy(oracle):
    rng = np.random.default_rng(6)
    w = rng.standard_normal((8, 64)).astype(np.float32)
    k0 = oracle.nm_select(w, 2, 4)
    w2 = w + 0.5 * rng.standard_normal(w.shape).astype(np.float32)
    k1 = oracle.nm_select(w2, 2, 4)
    flips, kept, total = oracle.mask_stats(w2, k1, k0)
    assert flips == int(np.abs(k1.astype(int) - k0.astype(int)).sum())      # ||M_t - M_{t-1}||_0
    assert np.isclose(kept, np.abs(w2.astype(np.float64) * k1).sum(), rtol=1e-12)
    assert np.isclose(total, np.abs(w2.astype(np.float64)).sum(), rtol=1e-12)
    assert flips % 2 == 0   # within a group the number of ones is fixed, so changes come in pairs
