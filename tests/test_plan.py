"""Host-side check of how the step kernels cover a matrix: cast_debug_plan runs the kernels' own
span arithmetic on the host.  For every shape tried, every entry must be covered exactly once, no
span may leave its row (or the matrix), spans must start on mask words, and the chunks of a span
must be dealt to exactly the wavefronts that cooperate on it: an error here would be an
out-of-bounds access or a missed entry on the GPU."""
import ctypes as C

import numpy as np
import pytest

from paper_2509_25996_amd import binding as B

CHUNK = 256


@pytest.fixture(scope="module")
def lib():
    return B.load()


def _plan(lib, rows, cols, ld, nseg, split, block=0, wave=0):
    plan, span = (C.c_int64 * 5)(), (C.c_int64 * 5)()
    rc = lib.cast_debug_plan(rows, cols, ld, nseg, int(split), block, wave, plan, span)
    assert rc == 0, rc
    return list(plan), list(span)


def _check_span(rows, cols, ld, nseg, plan, span):
    state, dense, length, index, sub = span
    vec, grid, block_waves, P, pieces = plan
    assert 0 <= sub < P <= block_waves <= 16
    if length == 0:
        return
    assert dense % 32 == 0 and length % 32 == 0 and length > 0
    assert dense + length <= rows * cols
    r, c = divmod(dense, cols)
    if ld != cols or nseg:
        assert c + length <= cols, "a span leaves its row"
        assert state == r * ld + c
    else:
        assert state == dense
    if nseg:
        seg_len = cols // nseg
        assert c // seg_len == (c + length - 1) // seg_len, "a span lies in two scale segments"
        if pieces == 1:
            assert length == seg_len and index == r * nseg + c // seg_len
        else:
            assert length <= 8 * CHUNK and index // pieces == r * nseg + c // seg_len


SMALL = [(1, 32), (3, 64), (2, 256), (5, 512), (4, 1024), (3, 1280 + 64), (2, 2560), (2, 4096), (1, 4096 + 32), (2, 5504),
         (1, 8768), (1, 11008), (2, 6912), (1, 16384), (1, 262144 + 32), (7, 96),
         (2, 5120), (2, 13824), (1, 4608), (1, 6656), (1, 14336), (3, 6144), (1, 7424), (1, 28672)]


# split = 2, 3: the plan of the selection and pack kernels (spans on multiples of 32 / 64 columns), which has no
# scaling segments
@pytest.mark.parametrize("rows,cols", SMALL)
@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("nseg,split", [(n, s) for s in (False, True) for n in (0, 1, 2)] + [(0, 2), (0, 3)])
def test_every_entry_is_covered_exactly_once(lib, rows, cols, nseg, interleaved, split):
    if nseg and (cols % nseg or (cols // nseg) % 4):
        pytest.skip("segments must be whole groups")
    _covered_exactly_once(lib, rows, cols, nseg, interleaved, split)


def test_random_shapes_are_covered_exactly_once(lib):
    """The same over 300 seeded random shapes: any multiple of 32 columns up to 16384, any segment count that
    divides them into whole groups, every plan kind."""
    rng = np.random.default_rng(20250928)
    done = 0
    while done < 300:
        cols = 32 * int(rng.integers(1, 513))
        rows = int(rng.integers(1, 5))
        split = [False, True, 2, 3][int(rng.integers(0, 4))]
        nseg = 0 if split in (2, 3) else int(rng.choice([0, 1, 2, 3, 4, 6, 8]))
        if nseg and (cols % nseg or (cols // nseg) % 4):
            continue
        _covered_exactly_once(lib, rows, cols, nseg, bool(rng.integers(0, 2)), split)
        done += 1


def _covered_exactly_once(lib, rows, cols, nseg, interleaved, split):
    ld = 3 * cols if interleaved else cols
    plan, _ = _plan(lib, rows, cols, ld, nseg, split)
    vec, grid, block_waves, P, pieces = plan
    if nseg and (cols // nseg) % 32:
        assert not vec
    if not vec:
        return
    assert pieces == 1 or (split is True and nseg)
    if split == 3 and cols % 64 == 0:
        assert all(_plan(lib, rows, cols, ld, nseg, split, b, 0)[1][1] % 64 == 0 for b in range(grid))
    covered = np.zeros(rows * cols, np.int32)
    seen_spans = {}
    for block in range(grid):
        for wave in range(block_waves):
            _, span = _plan(lib, rows, cols, ld, nseg, split, block, wave)
            _check_span(rows, cols, ld, nseg, plan, span)
            state, dense, length, index, sub = span
            if length == 0:
                continue
            seen_spans.setdefault(index, (dense, length, set()))
            assert seen_spans[index][:2] == (dense, length)
            assert sub not in seen_spans[index][2], "two wavefronts with the same place in a span"
            seen_spans[index][2].add(sub)
            for first in range(sub * CHUNK, length, P * CHUNK):       # the chunks this wavefront walks
                covered[dense + first:dense + min(first + CHUNK, length)] += 1
    assert (covered == 1).all(), (int((covered == 0).sum()), int((covered > 1).sum()))
    for dense, length, subs in seen_spans.values():
        assert subs == set(range(P)), "a span without all of its cooperating wavefronts"


@pytest.mark.parametrize("rows,cols", [(4096, 4096), (11008, 4096), (4096, 11008), (5120, 5120), (13824, 5120), (5120, 13824),
                                       (768, 768), (3072, 768), (768, 3072), (4096, 14336), (28672, 8192), (8192, 28672)])
@pytest.mark.parametrize("nseg,interleaved,split", [(2, True, True), (2, False, False), (0, True, False), (0, False, False),
                                                    (0, True, 2), (0, False, 2), (0, True, 3)])
def test_benchmark_shapes_stay_in_bounds(lib, rows, cols, nseg, interleaved, split):
    ld = 3 * cols if interleaved else cols
    plan, _ = _plan(lib, rows, cols, ld, nseg, split)
    vec, grid, block_waves, P, pieces = plan
    assert vec and grid >= 1
    rng = np.random.default_rng(rows + cols)
    blocks = sorted(set([0, 1, grid - 2, grid - 1] + list(rng.integers(0, grid, 60))))
    total = 0
    for block in blocks:
        if block < 0:
            continue
        for wave in range(block_waves):
            _, span = _plan(lib, rows, cols, ld, nseg, split, int(block), wave)
            _check_span(rows, cols, ld, nseg, plan, span)
            total += span[2]
    assert total > 0
    # the last workgroup ends exactly at the end of the matrix
    ends = [s[1] + s[2] for s in (_plan(lib, rows, cols, ld, nseg, split, grid - 1, w)[1] for w in range(block_waves)) if s[2]]
    assert max(ends) == rows * cols
    # past the grid nothing is handed out
    assert _plan(lib, rows, cols, ld, nseg, split, grid, 0)[1][2] == 0
