"""Exhaustive N:M projection, used only to pin the oracle's selection rule.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The N:M constraint (Eq. 4) admits C(M, N) masks per group.  The magnitude mask of Eq. 6 is
the one that retains the most L1 mass (equivalently the Euclidean projection of the group
onto the N:M set).  This module finds it by trying every mask with exact rational
arithmetic; when several masks retain the same mass it returns the one whose sorted index
tuple is lexicographically smallest, which is what "lower index wins" means for a set.
"""
from __future__ import annotations

from fractions import Fraction
from itertools import combinations

import numpy as np


def best_mask_group(values, n_keep: int):
    """values: M finite floats.  Returns the kept index tuple."""
    mags = [abs(Fraction(float(x))) for x in values]
    best, best_mass = None, None
    for idx in combinations(range(len(mags)), n_keep):  # lexicographic order
        mass = sum(mags[i] for i in idx)
        if best_mass is None or mass > best_mass:  # strict: the first maximiser is kept
            best, best_mass = idx, mass
    return best


def best_mask(w: np.ndarray, n_keep: int, m_group: int) -> np.ndarray:
    rows, cols = w.shape
    keep = np.zeros((rows, cols), np.uint8)
    for r in range(rows):
        for i in range(cols // m_group):
            idx = best_mask_group(w[r, i * m_group:(i + 1) * m_group], n_keep)
            for j in idx:
                keep[r, i * m_group + j] = 1
    return keep
