"""cast_adams_step_multi_noalloc (the list call on the library's built-in workspace, for callers that
cannot allocate) against cast_adams_step_multi on a caller's workspace: two calls in a row through the
raw C ABI, the second with a smaller list, every output byte equal."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, host

pytestmark = pytest.mark.gpu

# row segments of 2560 and 5504 entries are stepped in pieces (their dL/dA sums pass through the workspace),
# the 64 x 512 matrices share a launch, 5 x 72 runs on the scalar kernels; statistics slots for all of them
BIG = [(48, 5120), (64, 512), (64, 512), (16, 11008), (64, 512), (5, 72), (40, 4096)]
SMALL = [(16, 11008), (64, 512), (24, 5120)]


def _state(shapes, seed, n):
    items = []
    for i, (r, c) in enumerate(shapes):
        w, m, v = B.interleaved_state(torch.from_numpy(synth.weights(seed, i, r, c)).to(DEV)) if c % 8 == 0 and i % 2 == 0 else \
            (torch.from_numpy(synth.weights(seed, i, r, c)).to(DEV), torch.zeros((r, c), device=DEV), torch.zeros((r, c), device=DEV))
        A = torch.from_numpy((1 + 0.1 * np.random.default_rng(seed * 100 + i).standard_normal((r, n))).astype(np.float32)).to(DEV)
        mask = B.alloc_mask(r, c, DEV)
        items.append(dict(w=w, m=m, v=v, mask=mask, grad=synth.grads_bf16(seed, i, 0, r, c).to(DEV), scale=A,
                          scale_grad=torch.full((r, n), 7.0, device=DEV), initial_mask=torch.zeros_like(mask),
                          refresh_stats=B.alloc_refresh_stats(DEV)))
    return items


def _run(shapes, seed, noalloc: bool):
    """Three steps (refresh with statistics, non-refresh, refresh) through the raw entry points."""
    lib = B.load()
    n = 2
    items = _state(shapes, seed, n)
    tl = B.TensorList(items, DEV)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for t in range(3):
        cfg = B.iteration_config(t, 4, mask_period=2, lr=1e-3, lambda_=1e-3, scale_segments=n, grad_dtype=B.CAST_BF16)
        for i, x in enumerate(items):
            x["grad"].copy_(synth.grads_bf16(seed, i, t, *shapes[i]).to(DEV))
        cs = cfg.c_struct()
        if noalloc:
            rc = lib.cast_adams_step_multi_noalloc(tl.array, tl.count, C.byref(cs), stream)
        else:
            rc = lib.cast_adams_step_multi(tl.array, tl.count, C.byref(cs), C.c_void_p(tl.workspace.data_ptr()),
                                           tl.workspace.numel(), stream)
        assert rc == 0, (rc, B.status_str(rc))
    torch.cuda.synchronize()
    return [{k: host(x[k]).tobytes() for k in ("w", "m", "v", "mask", "scale_grad", "refresh_stats")} for x in items]


def test_noalloc_list_call_matches_the_list_call_twice_in_a_row():
    for shapes, seed in ((BIG, 31), (SMALL, 32)):      # the second call is smaller: it must not see the first one's leftovers
        want = _run(shapes, seed, noalloc=False)
        got = _run(shapes, seed, noalloc=True)
        for i, (a, b) in enumerate(zip(want, got)):
            for k in a:
                assert a[k] == b[k], (shapes[i], k)
    # the statistics really were gathered (a refresh at t = 2 against the mask of t = 0)
    stats = np.frombuffer(got[0]["refresh_stats"], np.int64)
    assert np.frombuffer(got[0]["refresh_stats"], np.float64)[3] > 0 and stats[1] > 0
