"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every function the
header declares, sizes buffers as documented and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2509_25996_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2509_25996_amd.build import build_library
        build_library()
    return B.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "cast.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cast_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    assert B.status_str(0) == "ok"
    for s in range(-7, 0):
        assert B.status_str(s) not in ("ok", "unknown status")
    assert B.status_str(-99) == "unknown status"


def test_sizes(lib):
    # 2:4, 4096x4096: mask 1 bit/param, values half the entries, metadata 4 bits per group
    m, v, t = B.cast_sizes(4096, 4096, 2, 4, B.CAST_F32)
    assert m == 4096 * 4096 // 8 and v == 4096 * 2048 * 4 and t == 4096 * 1024 // 2
    assert m * 32 == 4096 * 4096 * 4          # 1/32 of one fp32 state (Remark, Sec. 4.1)
    m, v, t = B.cast_sizes(3, 40, 4, 8, B.CAST_BF16)
    assert m == 3 * 2 * 4 and v == 3 * 20 * 2 and t == 3 * 3 * 4   # 5 groups, 2 per word -> 3 words
    m, v, t = B.cast_sizes(5, 6, 1, 2, B.CAST_F32)
    assert m == 5 * 4 and v == 5 * 3 * 4 and t == 5 * 4
    assert B.cast_sizes(0, 128, 2, 4) == (0, 0, 0)
    for bad in [(4, 6, 2, 4), (4, 8, 4, 4), (4, 8, 0, 4), (4, 9, 1, 3), (-1, 8, 2, 4)]:
        with pytest.raises(B.CastError) as e:
            B.cast_sizes(*bad)
        assert e.value.status == -2


def _cfg(**kw):
    return B.AdamsConfig(**kw).c_struct()


def test_validation_happens_before_any_launch(lib):
    # fake, suitably aligned, non-null addresses: a call that passed validation would fault,
    # so every case below must be rejected on the host
    p = C.c_void_p(0x10000)
    odd = C.c_void_p(0x10004)
    nul = C.c_void_p(0)
    st = C.c_void_p(0)
    step = lib.cast_adams_step

    def call(cfg, w=p, g=p, m=p, v=p, k=p, a=nul, ga=nul, rows=4, cols=64, ld=None):
        return step(w, g, m, v, k, a, ga, rows, cols, cols if ld is None else ld, C.byref(cfg), st)

    assert call(_cfg(n_keep=2, m_group=3)) == -2
    assert call(_cfg(n_keep=4, m_group=4)) == -2
    assert call(_cfg(), cols=66) == -2
    assert call(_cfg(), ld=60) == -2                             # row stride shorter than a row
    assert call(_cfg(scale_segments=2)) == -1                    # segments announced, no scale buffer
    assert call(_cfg(), a=p) == -2                               # scale buffer, no segments
    assert call(_cfg(), ga=p) == -1                              # dL/dA asked without a scale
    assert call(_cfg(scale_segments=3), a=p, cols=64) == -2      # 64 % 3
    assert call(_cfg(scale_segments=32, m_group=4), a=p, cols=64) == -2   # segment of 2 entries < M
    assert call(_cfg(grad_dtype=7)) == -4
    assert call(_cfg(bias_corr1=0.0)) == -5
    assert call(_cfg(bias_corr2=-1.0)) == -5
    assert call(_cfg(bias_corr2=float("nan"))) == -5
    assert call(_cfg(flags=8)) == -5
    assert call(_cfg(rule=5)) == -5 and call(_cfg(rule=-1)) == -5
    assert call(_cfg(), w=nul) == -1
    assert call(_cfg(), k=nul) == -1
    assert call(_cfg(), w=odd) == -3
    assert call(_cfg(), m=odd) == -3
    assert step(p, p, p, p, p, nul, nul, 4, 64, 64, None, st) == -1
    # empty tensors are accepted and do nothing, even with null buffers
    assert call(_cfg(), w=nul, g=nul, m=nul, v=nul, k=nul, rows=0) == 0
    assert call(_cfg(), w=nul, g=nul, m=nul, v=nul, k=nul, cols=0) == 0

    assert lib.cast_nm_select(p, 4, 62, 62, 2, 4, p, st) == -2
    assert lib.cast_nm_select(p, 4, 64, 63, 2, 4, p, st) == -2
    assert lib.cast_nm_select(nul, 4, 64, 64, 2, 4, p, st) == -1
    assert lib.cast_nm_select(odd, 4, 64, 64, 2, 4, p, st) == -3
    assert lib.cast_nm_select(nul, 0, 64, 64, 2, 4, nul, st) == 0
    assert lib.cast_weight_scale(p, p, 4, 64, 64, 3, p, 0, st) == -2
    assert lib.cast_weight_scale(p, p, 4, 64, 32, 2, p, 0, st) == -2
    assert lib.cast_weight_scale(p, p, 4, 64, 64, 2, p, 5, st) == -4
    assert lib.cast_weight_scale(p, nul, 4, 64, 64, 2, p, 0, st) == -1
    assert lib.cast_weight_scale_grad(p, p, 0, 4, 64, 64, 0, p, st) == -2
    assert lib.cast_weight_scale_grad(p, p, 0, 4, 64, 64, 2, nul, st) == -1
    assert lib.cast_nm_project_compress(p, nul, 0, nul, 4, 64, 64, 2, 4, nul, 0, p, st) == -1
    assert lib.cast_nm_project_compress(p, p, 3, nul, 4, 64, 64, 2, 4, p, 0, p, st) == -2
    assert lib.cast_nm_project_compress(p, nul, 0, nul, 4, 64, 64, 2, 4, p, 9, p, st) == -4
    assert lib.cast_nm_project_compress(p, nul, 0, nul, 4, 60, 60, 4, 8, p, 0, p, st) == -2
    assert lib.cast_nm_project_compress(p, nul, 0, nul, 4, 64, 8, 2, 4, p, 0, p, st) == -2
    assert lib.cast_mask_stats(p, nul, nul, 4, 64, 64, p, p, st) == -1
    assert lib.cast_mask_stats(p, p, nul, 4, 64, 63, p, p, st) == -2
    emit = lib.cast_adams_step_emit
    c2 = _cfg(scale_segments=2)
    assert emit(p, p, p, p, p, nul, nul, nul, nul, 4, 64, 64, C.byref(_cfg()), st) == -1        # no compute copy
    assert emit(p, p, p, p, p, nul, nul, p, p, 4, 64, 64, C.byref(_cfg()), st) == -2            # copy_scale without segments
    assert emit(p, p, p, p, p, p, nul, nul, C.c_void_p(0x10008), 4, 64, 64, C.byref(c2), st) == -3
    assert emit(nul, nul, nul, nul, nul, nul, nul, nul, nul, 0, 64, 64, C.byref(_cfg()), st) == 0
    # a first moment kept in bf16 goes with AdamS and additive decay only
    mu16 = lambda **kw: _cfg(flags=4, **kw)
    assert step(p, p, p, p, p, nul, nul, 4, 66, 66, C.byref(mu16()), st) == -2
    assert step(p, p, p, p, p, nul, nul, 4, 64, 64, C.byref(mu16(rule=1)), st) == -5
    assert step(p, p, p, p, p, nul, nul, 4, 64, 64, C.byref(mu16(rule=4)), st) == -5
    assert emit(p, p, p, p, p, nul, nul, nul, p, 4, 64, 64, C.byref(mu16(rule=2)), st) == -5
    # the second moment in bf16 only together with the first, and under the same rules
    assert step(p, p, p, p, p, nul, nul, 4, 64, 64, C.byref(_cfg(flags=8)), st) == -5
    assert step(p, p, p, p, p, nul, nul, 4, 64, 64, C.byref(_cfg(flags=12, rule=4)), st) == -5
    assert step(p, p, p, p, p, nul, nul, 4, 64, 64, C.byref(_cfg(flags=16)), st) == -5
    # list call: rejected as a whole if any matrix is bad, before anything is enqueued
    T = B._Tensor
    good = T(0x10000, 0x10000, 0x10000, 0x10000, 0x10000, None, None, 4, 64, 64)
    bad = T(0x10000, 0x10000, 0x10000, 0x10000, 0x10000, None, None, 4, 66, 66)
    arr = (T * 2)(good, bad)
    cfg = _cfg()
    ws_bytes = lambda a, n, c: lib.cast_adams_multi_workspace_bytes(a, n, C.byref(c))
    assert ws_bytes(arr, 2, cfg) == 0 and ws_bytes(arr, 0, cfg) == 0 and ws_bytes(None, 2, cfg) == 0    # no pieces, no statistics
    # row segments of more than 16 chunks of 256 entries are stepped in pieces of 8 chunks whose dL/dA sums
    # pass through the workspace (one float per piece)
    wide = (T * 2)(T(0x10000, 0x10000, 0x10000, 0x10000, 0x10000, 0x10000, 0x10000, 3, 11008, 11008), good)
    seg = _cfg(scale_segments=2)
    assert ws_bytes(wide, 2, seg) == 4 * 20          # 3 rows x 2 segments x 3 pieces, rounded up to 4 floats
    assert ws_bytes(wide, 2, _cfg(scale_segments=8)) == 0
    assert lib.cast_adams_step_multi(wide, 1, C.byref(seg), p, 76, st) == -2      # no room for the sums
    assert lib.cast_adams_step_multi(wide, 1, C.byref(seg), nul, 80, st) == -1     # a workspace is needed and missing
    assert lib.cast_adams_step_multi(wide, 1, C.byref(_cfg(scale_segments=2, flags=2)), p, 80, st) == -5      # flag value 2 is not in use
    # refresh statistics: one 16-byte slot per workgroup of the matrix's launch (4 x 64 entries: one workgroup)
    with_stats = (T * 1)(T(0x10000, 0x10000, 0x10000, 0x10000, 0x10000, None, None, 4, 64, 64, None, None, None, 0x10000))
    assert ws_bytes(with_stats, 1, cfg) == 16
    assert lib.cast_adams_step_multi(with_stats, 1, C.byref(_cfg(flags=8, refresh_mask=1)), p, 4096, st) == -5      # bf16 v without bf16 mu
    assert lib.cast_adams_step_multi(arr, 2, C.byref(cfg), p, 176, st) == -2
    assert lib.cast_adams_step_multi(with_stats, 1, C.byref(_cfg(refresh_mask=1)), p, 8, st) == -2       # workspace too small
    assert lib.cast_adams_step_multi(with_stats, 1, C.byref(_cfg(refresh_mask=1)), nul, 112, st) == -1
    assert lib.cast_adams_step_multi(arr, 1, None, p, 112, st) == -1
    assert lib.cast_adams_step_multi(arr, 0, C.byref(cfg), nul, 0, st) == 0
    assert lib.cast_adams_step_multi(arr, -1, C.byref(cfg), p, 64, st) == -2
    assert lib.cast_hbm_copy_probe(p, p, 24, st) == -2
    assert lib.cast_hbm_copy_probe(p, odd, 32, st) == -3
    assert lib.cast_hbm_copy_probe(nul, nul, 0, st) == 0


def test_list_calls_of_the_once_per_run_entry_points_reject_bad_lists(lib):
    # all or nothing: one bad matrix and nothing is launched (fake device pointers: none is dereferenced on the host)
    M, S = B._Matrix, B._StatsMatrix
    a, st, odd = 0x100000, C.c_void_p(0), 0x100004
    good = M(a, 4, 64, 64, a, a, a, a, None)
    bad_shape = M(a, 4, 64, 60, a, a, a, a, None)      # row stride below the row length
    for arr, want in (((M * 2)(good, bad_shape), -2), ((M * 2)(good, M(None, 4, 64, 64, a, a, a, a, None)), -1),
                      ((M * 2)(good, M(odd, 4, 64, 64, a, a, a, a, None)), -3)):
        assert lib.cast_nm_select_multi(arr, 2, 2, 4, st) == want
        assert lib.cast_weight_scale_multi(arr, 2, 2, B.CAST_BF16, st) == want
        assert lib.cast_nm_project_compress_multi(arr, 2, 2, 2, 4, B.CAST_F32, st) == want
    one = (M * 1)(good)
    assert lib.cast_nm_select_multi(one, 1, 4, 4, st) == -2                      # N < M
    assert lib.cast_weight_scale_multi(one, 1, 3, B.CAST_F32, st) == -2          # 3 segments do not divide 64 columns
    assert lib.cast_weight_scale_multi(one, 1, 2, 7, st) == -4
    assert lib.cast_nm_project_compress_multi(one, 1, 2, 2, 4, 9, st) == -4
    assert lib.cast_nm_project_compress_multi((M * 1)(M(a, 4, 64, 64, a, a, a, a, 0x100002)), 1, 2, 2, 4, 0, st) == -3      # status word
    for f in (lib.cast_nm_select_multi,):
        assert f(one, 0, 2, 4, st) == 0 and f(None, 1, 2, 4, st) == -1 and f(one, -1, 2, 4, st) == -2
    empty = (M * 1)(M(None, 0, 64, 64, None, None, None, None, None))
    assert lib.cast_nm_select_multi(empty, 1, 2, 4, st) == 0
    # statistics of given masks over a list
    sgood = S(a, 4, 64, 64, a, a, a)
    ws = lib.cast_mask_stats_multi_workspace_bytes
    assert ws((S * 1)(sgood), 1) == 16 and ws((S * 1)(S(a, 5, 72, 72, a, None, a)), 1) == 16 and ws(None, 1) == 0      # one workgroup each
    assert ws((S * 1)(S(a, 11008, 4096, 12288, a, None, a)), 1) == 11008 * 2 * 16      # a workgroup per 2048 entries
    assert lib.cast_mask_stats_multi((S * 1)(sgood), 1, C.c_void_p(a), 8, st) == -2
    assert lib.cast_mask_stats_multi((S * 1)(sgood), 1, None, 16, st) == -1
    assert lib.cast_mask_stats_multi((S * 1)(S(a, 4, 64, 64, None, a, a)), 1, C.c_void_p(a), 64, st) == -1
    assert lib.cast_mask_stats_multi((S * 1)(S(a, 4, 64, 64, a, a, None)), 1, C.c_void_p(a), 64, st) == -1
    assert lib.cast_mask_stats_multi((S * 1)(S(a, 4, 64, 60, a, a, a)), 1, C.c_void_p(a), 64, st) == -2
    assert lib.cast_mask_stats_multi((S * 1)(sgood), 0, None, 0, st) == 0
    # dL/dA over a list
    G = B._ScaleGradMatrix
    ggood = G(a, a, 4, 64, 64, a)
    sg = lib.cast_weight_scale_grad_multi
    for bad, want in ((G(a, a, 4, 64, 60, a), -2), (G(None, a, 4, 64, 64, a), -1), (G(a, None, 4, 64, 64, a), -1),
                      (G(a, a, 4, 64, 64, None), -1), (G(odd, a, 4, 64, 64, a), -3), (G(a, odd, 4, 64, 64, a), -3),
                      (G(a, a, -1, 64, 64, a), -2)):
        assert sg((G * 2)(ggood, bad), 2, B.CAST_BF16, 2, st) == want
    assert sg((G * 1)(ggood), 1, B.CAST_BF16, 3, st) == -2       # 3 segments do not divide 64 columns
    assert sg((G * 1)(ggood), 1, B.CAST_BF16, 0, st) == -2
    assert sg((G * 1)(ggood), 1, 5, 2, st) == -4
    assert sg((G * 1)(ggood), 0, B.CAST_F32, 2, st) == 0 and sg(None, 1, B.CAST_F32, 2, st) == -1
    assert sg((G * 1)(ggood), -1, B.CAST_F32, 2, st) == -2
    assert sg((G * 1)(G(None, None, 0, 64, 64, None)), 1, B.CAST_F32, 2, st) == 0       # an empty matrix needs no buffers


def test_noalloc_list_call_rejects_what_does_not_fit(lib):
    # the entry point that allocates nothing has a fixed workspace (64 MiB) and a fixed list length; anything
    # beyond is refused on the host before a device is touched
    T = B._Tensor
    a = 0x100000
    st = C.c_void_p(0)
    call = lib.cast_adams_step_multi_noalloc
    ws_bytes = lambda arr, n, c: lib.cast_adams_multi_workspace_bytes(arr, n, C.byref(c))
    refresh = _cfg(refresh_mask=1)
    # refresh statistics of a 2^22 x 4096 matrix: one 16-byte slot per workgroup of 2048 entries = 128 MiB
    huge = (T * 1)(T(a, a, a, a, a, None, None, 1 << 22, 4096, 4096, None, None, None, a))
    assert ws_bytes(huge, 1, refresh) == (1 << 22) * 4096 // 2048 * 16 > (64 << 20)
    assert call(huge, 1, C.byref(refresh), st) == -7
    # 16 M row segments in pieces: five floats each
    many = (T * 1)(T(a, a, a, a, a, a, a, 1 << 23, 5120, 5120))
    seg = _cfg(scale_segments=2)
    assert ws_bytes(many, 1, seg) == (1 << 24) * 5 * 4 > (64 << 20)
    assert call(many, 1, C.byref(seg), st) == -7
    # more matrices than the fixed list length
    long_list = (T * 4097)(*[T(a, a, a, a, a, None, None, 4, 64, 64)] * 4097)
    assert call(long_list, 4097, C.byref(_cfg()), st) == -7
    # the ordinary rejections come first and are those of the list call
    bad = (T * 2)(T(a, a, a, a, a, None, None, 4, 64, 64), T(a, a, a, a, a, None, None, 4, 66, 66))
    assert call(bad, 2, C.byref(_cfg()), st) == -2
    assert call(bad, 1, None, st) == -1
    assert call(None, 1, C.byref(_cfg()), st) == -1
    assert call(bad, 0, C.byref(_cfg()), st) == 0
    assert call(bad, -1, C.byref(_cfg()), st) == -2
    assert call(bad, 1, C.byref(_cfg(flags=2)), st) == -5
    assert B.status_str(-7) not in ("ok", "unknown status")


def test_list_call_launch_tally(lib):
    # host-only: which launches the list call would make for one LLaMA2-7B-shaped layer with n = 2 scaling
    # (q, k, v, o share a launch; gate, up one each; down in pieces plus the sum of its pieces)
    T = B._Tensor
    a = 0x100000
    layer = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    arr = (T * 7)(*[T(a, a, a, a, a, a, a, r, c, 3 * c) for r, c in layer])
    cfg = B.AdamsConfig(scale_segments=2, grad_dtype=B.CAST_BF16).c_struct()
    step, other = C.c_int32(-1), C.c_int32(-1)
    assert lib.cast_adams_multi_launches(arr, 7, C.byref(cfg), C.byref(step), C.byref(other)) == 0
    assert (step.value, other.value) == (4, 1)
    # compute copies, and refresh statistics on a refresh step: q, k, v, o still share a launch
    emit = (T * 7)(*[T(a, a, a, a, a, a, a, r, c, 3 * c, a, a) for r, c in layer])
    cfg = B.AdamsConfig(scale_segments=2, grad_dtype=B.CAST_BF16).c_struct()
    assert lib.cast_adams_multi_launches(emit, 7, C.byref(cfg), C.byref(step), C.byref(other)) == 0
    assert (step.value, other.value) == (4, 1)
    stats = (T * 7)(*[T(a, a, a, a, a, a, a, r, c, 3 * c, None, None, a, a) for r, c in layer])
    cfg = B.AdamsConfig(scale_segments=2, grad_dtype=B.CAST_BF16, refresh_mask=1).c_struct()
    assert lib.cast_adams_multi_launches(stats, 7, C.byref(cfg), C.byref(step), C.byref(other)) == 0
    assert (step.value, other.value) == (4, 2)          # the sum of down's pieces, the sums of the statistics
    cfg = B.AdamsConfig(scale_segments=2, grad_dtype=B.CAST_BF16, rule=B.RULE_ADAM_L1).c_struct()
    assert lib.cast_adams_multi_launches(arr, 7, C.byref(cfg), C.byref(step), None) == 0
    assert step.value == 4                              # comparison rules share launches like the others
    bad = (T * 1)(T(a, a, a, a, a, a, a, 4, 66, 66))
    assert lib.cast_adams_multi_launches(bad, 1, C.byref(cfg), C.byref(step), C.byref(other)) == -2


def test_iteration_config_reading():
    # Algorithm 1 loops t = 0..T-1 with alpha_t = t/T; masks refresh when t mod T_1 == 0
    c0 = B.iteration_config(0, 100)
    assert c0.alpha == 0.0 and c0.refresh_mask == 1
    assert abs(c0.bias_corr1 - 0.1) < 1e-7 and abs(c0.bias_corr2 - 0.001) < 1e-7
    c = B.iteration_config(25, 100, mask_period=10, lambda_=4e-7)
    assert c.alpha == 0.25 and c.refresh_mask == 0 and c.lambda_ == 4e-7
    assert B.iteration_config(30, 100).refresh_mask == 1


def test_iteration_config_is_the_oracles_schedule_bit_for_bit():
    # the binding's helper and the oracle's pinned iteration_scalars are written independently; the GPU tests hand
    # the binding's numbers to both sides, so a wrong exponent or ramp in the helper would pass them all: here the
    # two are compared as the fp32 values the library receives, for every iteration of short and long schedules
    import numpy as np

    import oracle
    for total, b1, b2, period in ((10, 0.9, 0.999, 10), (100, 0.9, 0.999, 10), (7500, 0.9, 0.95, 7), (1, 0.5, 0.75, 1)):
        for t in range(total):
            cfg = B.iteration_config(t, total, mask_period=period, beta1=b1, beta2=b2).c_struct()
            alpha, bc1, bc2 = oracle.iteration_scalars(t, total, b1, b2)
            got = np.array([cfg.alpha, cfg.bias_corr1, cfg.bias_corr2], np.float32)
            want = np.array([alpha, bc1, bc2], np.float32)
            assert (got.view(np.uint32) == want.view(np.uint32)).all(), (total, t)
            assert cfg.refresh_mask == int(t % period == 0)


def test_division_by_a_common_divisor_is_the_ieee_quotient(lib):
    # the kernels divide by the two bias corrections with a short FMA sequence; on the host the same
    # routine must reproduce the correctly rounded quotient for every mantissa, inside and outside its fast range
    import numpy as np
    man = np.arange(2 ** 23, dtype=np.uint32)
    rng = np.random.default_rng(0)
    ys = [1 - 0.9, 1 - 0.999, 1 - 0.9 ** 7, 1 - 0.999 ** 500, 1.0, 0.99999994, 2.0 ** -12, 2.0, 3.0, 1e-5]
    ys += list(rng.uniform(2.0 ** -12, 2.0, 3))
    for k, y in enumerate(ys):
        y = np.float32(y)
        for e in ((64, 127, 192) if k < 4 else (100 + k,)) + ((0, 1, 63, 193, 254, 255) if k == 0 else ()):
            sign = (k + e) & 1
            x = ((sign << 31) | (e << 23) | man).astype(np.uint32).view(np.float32)
            got = B.cast_debug_div_by_uniform(x, float(y))
            with np.errstate(all="ignore"):
                ref = (x / y).astype(np.float32)
            same = (got.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(got) & np.isnan(ref))
            assert same.all(), (float(y), e)


def test_without_the_library_the_binding_raises_and_the_package_never_touches_the_oracle():
    """No fallback path: a missing libcast.so is an error at load(), and neither side imports the other."""
    import re
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, CAST_LIBRARY=os.path.join(root, "no_such_dir", "libcast.so"))
    run = subprocess.run([sys.executable, "-c", "from paper_2509_25996_amd import binding as B\nB.load()"], cwd=root, env=env,
                         capture_output=True, text=True, timeout=300)
    assert run.returncode != 0 and "FileNotFoundError" in run.stderr and "no fallback" in run.stderr
    imports = re.compile(r"^\s*(?:import|from)\s+([\w\.]+)", re.M)
    pkg = os.path.join(root, "paper_2509_25996_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            mods = imports.findall(open(os.path.join(pkg, name)).read())
            assert not any(m.split(".")[0] == "oracle" for m in mods), name
    for name in os.listdir(os.path.join(root, "oracle")):
        if name.endswith(".py"):
            mods = imports.findall(open(os.path.join(root, "oracle", name)).read())
            assert not any(m.split(".")[0] == "paper_2509_25996_amd" for m in mods), name
    # C sources: nothing under csrc/ or include/ includes a file of the oracle, and the reverse
    for folder, banned in ((os.path.join(pkg, "csrc"), "oracle"), (os.path.join(root, "include"), "oracle"),
                           (os.path.join(root, "oracle"), "cast.h")):
        for name in os.listdir(folder):
            if name.endswith((".h", ".hip", ".c")):
                for inc in re.findall(r'#include\s+[<"]([^>"]+)[>"]', open(os.path.join(folder, name)).read()):
                    assert banned not in inc, (name, inc)


def test_stream_skeleton_refuses_shapes_it_cannot_walk():
    # argument checks come before any HIP call: runs without a GPU
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(B.__file__)), "stream_skeleton")
    assert os.path.exists(exe), "build it with python -m paper_2509_25996_amd.build"
    for args in (["5", "100"], ["0", "1024"], ["8", "1024", "65"], ["1048576", "1024"]):
        run = subprocess.run([exe, *args], capture_output=True, text=True, timeout=60)
        assert run.returncode == 2 and "usage" in run.stdout, args
