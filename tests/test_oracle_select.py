"""Pins for the oracle's mask selection (Eq. 4, Eq. 6): none of these re-uses the oracle's
own rank formula; they are brute force, printed values, invariants and special cases."""
import os

import numpy as np
import pytest

from oracle import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
NM = [(1, 2), (2, 4), (1, 4), (3, 4), (4, 8), (2, 8), (1, 8), (7, 8)]


def test_paper_worked_example_1_of_2(oracle):
    # Sec. 5.1 prints which entry of each pair is masked under 1:2
    rows = []
    with open(os.path.join(GOLDEN, "select_1of2_example.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            lhs, rhs = line.split("->")
            rows.append(([float(x) for x in lhs.split()], [int(x) for x in rhs.split()]))
    assert len(rows) == 2
    for vals, expect in rows:
        keep = oracle.nm_select(np.array([vals], np.float32), 1, 2)
        assert keep.tolist() == [expect]


@pytest.mark.parametrize("n,m", NM)
def test_matches_exhaustive_search_with_ties(oracle, n, m):
    rng = np.random.default_rng(100 * n + m)
    # few distinct magnitudes, both signs, some zeros: ties inside most groups
    w = rng.integers(-3, 4, size=(6, 8 * m)).astype(np.float32) * np.float32(0.25)
    assert (oracle.nm_select(w, n, m) == bruteforce.best_mask(w, n, m)).all()


@pytest.mark.parametrize("n,m", NM)
def test_matches_exhaustive_search_distinct(oracle, n, m):
    rng = np.random.default_rng(7 * n + m)
    w = (rng.standard_normal((5, 6 * m)) * 0.02).astype(np.float32)
    assert (oracle.nm_select(w, n, m) == bruteforce.best_mask(w, n, m)).all()


@pytest.mark.parametrize("n,m", NM)
def test_exactly_n_per_group(oracle, n, m):
    rng = np.random.default_rng(3)
    w = (rng.standard_normal((16, 16 * m))).astype(np.float32)
    w[rng.random(w.shape) < 0.3] = 0.0
    keep = oracle.nm_select(w, n, m)
    assert (keep.reshape(16, -1, m).sum(-1) == n).all()
    assert set(np.unique(keep)) <= {0, 1}


@pytest.mark.parametrize("n,m", NM)
def test_all_equal_group_keeps_lowest_indices(oracle, n, m):
    for val in (0.0, -0.0, 0.5, -0.5):
        w = np.full((1, m), val, np.float32)
        assert oracle.nm_select(w, n, m)[0].tolist() == [1] * n + [0] * (m - n)


def test_sign_and_power_of_two_scale_invariance(oracle):
    rng = np.random.default_rng(11)
    w = rng.standard_normal((8, 64)).astype(np.float32)
    w = np.round(w * 4) / 4  # ties
    w = w.astype(np.float32)
    ref = oracle.nm_select(w, 2, 4)
    flips = np.where(rng.random(w.shape) < 0.5, -1.0, 1.0).astype(np.float32)
    assert (oracle.nm_select(-w, 2, 4) == ref).all()
    assert (oracle.nm_select(np.abs(w), 2, 4) == ref).all()
    assert (oracle.nm_select(w * flips, 2, 4) == ref).all()
    assert (oracle.nm_select(w * np.float32(2.0 ** -10), 2, 4) == ref).all()
    assert (oracle.nm_select(w * np.float32(2.0 ** 7), 2, 4) == ref).all()


def test_distinct_magnitudes_mask_is_the_top_n_set(oracle):
    # with no ties the answer does not depend on any tie rule: it is the top-N set (a sort)
    rng = np.random.default_rng(5)
    w = rng.standard_normal((32, 64)).astype(np.float32)
    for n, m in [(2, 4), (4, 8)]:
        g = np.abs(w).reshape(32, -1, m)
        order = np.argsort(-g, axis=-1, kind="stable")
        expect = np.zeros_like(g, dtype=np.uint8)
        np.put_along_axis(expect, order[..., :n], 1, axis=-1)
        assert (oracle.nm_select(w, n, m).reshape(g.shape) == expect).all()


def test_special_values_total_order(oracle):
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    den = np.float32(1e-45)  # smallest denormal
    cases = [
        ([0.0, -0.0, den, 0.0], [0, 0, 1, 0], 1),      # a denormal beats zeros
        ([den, 2 * den, 0.0, -den], [1, 1, 0, 0], 2),  # denormals are ordered; tie -> lower index
        ([1e30, -inf, 3.0, 2.0], [1, 1, 0, 0], 2),     # inf above finite
        ([inf, nan, -inf, 1.0], [1, 1, 0, 0], 2),      # NaN above inf; equal infs -> lower index
        ([1.0, 2.0, nan, 3.0], [0, 0, 1, 1], 2),       # a NaN is never pruned silently
    ]
    for vals, expect, n in cases:
        keep = oracle.nm_select(np.array([vals], np.float32), n, 4)
        assert keep[0].tolist() == expect, vals


def test_bad_shapes_rejected(oracle):
    w = np.zeros((2, 6), np.float32)
    with pytest.raises(ValueError):
        oracle.nm_select(w, 2, 4)   # 6 % 4 != 0
    with pytest.raises(ValueError):
        oracle.nm_select(np.zeros((2, 8), np.float32), 4, 4)  # N must be < M


def test_mask_bit_words_layout(oracle):
    # one bit per parameter (the 1/32 optimizer-state overhead of the Remark in Sec. 4.1)
    rng = np.random.default_rng(2)
    for cols in (4, 32, 36, 100):
        keep = (rng.random((3, cols)) < 0.5).astype(np.uint8)
        words = oracle.pack_mask_bits(keep)
        assert words.shape == (3, (cols + 31) // 32) and words.dtype == np.uint32
        # independent decode: numpy's bit unpacking of the little-endian bytes
        bits = np.unpackbits(words.view(np.uint8).reshape(3, -1), axis=1, bitorder="little")
        assert (bits[:, :cols] == keep).all()
        assert (bits[:, cols:] == 0).all()
        assert (oracle.unpack_mask_bits(words, cols) == keep).all()
    assert oracle.pack_mask_bits(np.ones((1, 4096), np.uint8)).nbytes * 32 == 4096 * 4
