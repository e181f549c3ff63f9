"""The storage variant that keeps the first moment in bf16 (CAST_FLAG_MU_BF16) against the oracle's
definition of it: rounded to nearest even when stored, unrounded inside the iteration.  Every bit of
w, mu, v and the mask, over the patterns, layouts, shapes and launch forms the variant has."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, GpuState, stepped_in_pieces, OracleState, assert_same_bits, dev, host, oracle_cfg, words

pytestmark = pytest.mark.gpu


def _mu(t: torch.Tensor) -> np.ndarray:
    assert t.dtype == torch.bfloat16
    return host(t.float())


@pytest.mark.parametrize("n,m", [(2, 4), (4, 8), (1, 2)])
@pytest.mark.parametrize("rows,cols,nseg", [(6, 512, 0), (6, 512, 2), (5, 1280 + 64, 2), (7, 72, 3), (3, 40, 0), (9, 24, 1),
                                            (12, 4096, 2), (5, 11008, 2), (33, 4096 + 32, 0), (6, 5120, 2), (4, 13824, 2)])
@pytest.mark.parametrize("bf16_grad", [False, True])
@pytest.mark.parametrize("interleaved", [False, True])
def test_mu_bf16_step_bit_exact(n, m, rows, cols, nseg, bf16_grad, interleaved):
    if cols % m or (nseg and (cols // nseg) % m) or (interleaved and cols % 8):
        pytest.skip("shape not valid for this M or layout")
    steps = 4
    rng = np.random.default_rng(rows * cols + n)
    w0 = synth.tie_outlier_weights(2, 7, rows, cols) if cols % 8 == 0 else synth.weights(2, 7, rows, cols)
    g = GpuState(w0, nseg, interleaved, mu_bf16=True)
    o = OracleState(w0, "f32")
    for t in range(steps):
        gr = synth.grads_f32(2, 7, t, rows, cols)
        if bf16_grad:
            gr = synth.widen_bf16(torch.from_numpy(gr).to(torch.bfloat16))
        cfg = B.iteration_config(t, steps, mask_period=2, lr=1e-3, lambda_=1e-3, n_keep=n, m_group=m, scale_segments=nseg)
        A = (1 + 0.2 * rng.standard_normal((rows, nseg))).astype(np.float32) if nseg else None
        g.step(dev(gr, torch.bfloat16 if bf16_grad else None), cfg, scale=None if A is None else dev(A))
        assert cfg.flags & B.FLAG_MU_BF16
        ref_gA = o.step(gr, oracle_cfg(cfg), A=A)
        if nseg:
            got = host(g.scale_grad)
            assert np.abs(got - ref_gA).max() <= 1e-5 * max(np.abs(ref_gA).max(), 1e-12) + 1e-9
    torch.cuda.synchronize()
    assert (words(g.mask) == oracle.pack_mask_bits(o.keep)).all()
    assert_same_bits(host(g.w), o.w, "w")
    assert_same_bits(_mu(g.m), o.m, "mu")
    assert_same_bits(host(g.v), o.v, "v")
    assert (o.m.view(np.uint32) & 0xFFFF == 0).all() and np.abs(o.m).max() > 0


def test_mu_bf16_special_values():
    # NaN, infinities, zeros of both signs, denormals and the largest finite values in w, g and mu
    rows, cols = 4, 64
    special = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-40, -1e-40, 3e38, -3e38, 1.0, -1.0, 65504.0], np.float32)
    w0 = synth.weights(3, 1, rows, cols)
    g0 = synth.grads_f32(3, 1, 0, rows, cols)
    w0[0, :12] = special
    g0[1, :12] = special
    w0[2, :12] = special
    g0[2, :12] = special[::-1]
    st = GpuState(w0, 0, False, mu_bf16=True)
    o = OracleState(w0, "f32")
    for t in range(3):
        cfg = B.iteration_config(t, 3, mask_period=1, lr=1e-3, lambda_=1e-3)
        st.step(dev(g0), cfg)
        o.step(g0, oracle_cfg(cfg))
    torch.cuda.synchronize()
    assert_same_bits(host(st.w), o.w, "w")
    assert_same_bits(_mu(st.m), o.m, "mu")
    assert_same_bits(host(st.v), o.v, "v")


@pytest.mark.parametrize("nseg", [0, 2])
def test_mu_bf16_list_call_equals_single_calls(nseg):
    # equal shapes share launches, the long rows are stepped in pieces, odd shapes one by one
    shapes = [(64, 512), (32, 1024), (64, 512), (5, 72), (64, 512), (16, 11008), (16, 11008), (7, 8768), (0, 64), (64, 512), (12, 5120),
              (6, 13824)]
    rng = np.random.default_rng(5)

    def make():
        items = []
        for i, (r, c) in enumerate(shapes):
            st = GpuState(synth.weights(9, i, r, c), nseg, interleaved=r > 0 and c % 8 == 0 and i % 2 == 0, mu_bf16=True)
            items.append(dict(w=st.w, m=st.m, v=st.v, mask=st.mask, grad=synth.grads_bf16(9, i, 0, r, c).to(DEV),
                              scale=dev((1 + 0.1 * rng.standard_normal((r, nseg))).astype(np.float32)) if nseg else None,
                              scale_grad=st.scale_grad))
        return items

    rng = np.random.default_rng(5)
    a = make()
    rng = np.random.default_rng(5)
    b = make()
    tl = B.TensorList(b, DEV)
    for t in range(3):
        cfg = B.iteration_config(t, 4, mask_period=2, lr=1e-3, lambda_=1e-3, scale_segments=nseg)
        for x in a:
            B.cast_adams_step(x["w"], x["grad"], x["m"], x["v"], x["mask"], cfg, scale=x["scale"], scale_grad=x["scale_grad"])
        B.cast_adams_step_multi(tl, cfg)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        for k in ("w", "v", "mask"):
            assert host(x[k]).tobytes() == host(y[k]).tobytes(), k
        assert host(x["m"].view(torch.int16)).tobytes() == host(y["m"].view(torch.int16)).tobytes()
        if nseg and x["w"].numel():
            ga, gb = host(x["scale_grad"]), host(y["scale_grad"])
            if stepped_in_pieces(x["w"].shape[1] // nseg):      # another, equally fixed summation order
                assert np.abs(ga.astype(np.float64) - gb).max() <= 1e-6
            else:
                assert ga.tobytes() == gb.tobytes()
    # the whole list against the oracle, one matrix of each kind
    for i in (0, 3, 5):
        r, c = shapes[i]
        o = OracleState(synth.weights(9, i, r, c), "f32")
        rng = np.random.default_rng(5)
        scales = [(1 + 0.1 * rng.standard_normal((rr, nseg))).astype(np.float32) if nseg else None for rr, _ in shapes]
        for t in range(3):
            cfg = B.iteration_config(t, 4, mask_period=2, lr=1e-3, lambda_=1e-3, scale_segments=nseg)
            cfg.flags |= B.FLAG_MU_BF16
            o.step(synth.widen_bf16(synth.grads_bf16(9, i, 0, r, c)), oracle_cfg(cfg), A=scales[i])
        assert_same_bits(host(b[i]["w"]), o.w, f"w of matrix {i}")
        assert_same_bits(_mu(b[i]["m"]), o.m, f"mu of matrix {i}")


@pytest.mark.parametrize("rows,cols", [(4096, 4096), (11008, 4096), (4096, 11008)])
def test_mu_bf16_sampled_rows_of_full_size_matrices(rows, cols):
    """LLaMA2-7B shapes, row-interleaved state with the bf16 first moment, the list call: sampled whole rows."""
    n, steps, n_sample = 2, 3, 24
    w = synth.device_gaussian((rows, cols), 0.02, torch.float32, 11, DEV)
    g = synth.device_gaussian((rows, cols), 1e-3, torch.bfloat16, 12, DEV)
    w, m, v = B.interleaved_state(w, mu_bf16=True)
    mask = B.alloc_mask(rows, cols, DEV)
    A = (1 + 0.05 * torch.randn((rows, n), device=DEV, generator=torch.Generator(DEV).manual_seed(3))).contiguous()
    gA = torch.zeros((rows, n), device=DEV)
    rng = np.random.default_rng(rows + cols)
    pick = np.unique(np.concatenate([[0, rows - 1], rng.integers(0, rows, n_sample)]))
    idx = torch.from_numpy(pick).to(DEV)
    ow, og, oA = host(w[idx]).copy(), host(g[idx].float()).copy(), host(A[idx]).copy()
    om, ov = np.zeros_like(ow), np.zeros_like(ow)
    keep = np.zeros(ow.shape, np.uint8)
    tl = B.TensorList([dict(w=w, grad=g, m=m, v=v, mask=mask, scale=A, scale_grad=gA)], DEV)
    for t in range(steps):
        cfg = B.iteration_config(t, 7500, mask_period=2, lr=2e-5, lambda_=4e-7, scale_segments=n)
        cfg.alpha = 0.25 + 0.25 * t
        B.cast_adams_step_multi(tl, cfg)
        oracle.adams_step(ow, og, om, ov, keep, oracle_cfg(cfg), A=oA, arithmetic="f32", nthreads=8)
    torch.cuda.synchronize()
    assert (words(mask[idx]) == oracle.pack_mask_bits(keep)).all()
    assert_same_bits(host(w[idx]), ow, "w")
    assert_same_bits(_mu(m[idx]), om, "mu")
    assert_same_bits(host(v[idx]), ov, "v")


@pytest.mark.parametrize("rows,cols,nseg", [(16, 1024, 2), (16, 1024, 0), (7, 72, 3), (5, 11008, 2), (6, 5120, 2), (33, 4096 + 32, 1)])
@pytest.mark.parametrize("refresh", [0, 1])
def test_mu_bf16_step_also_writes_the_compute_copy(rows, cols, nseg, refresh):
    """The bf16 first moment together with the bf16 compute copy of the next forward pass (24.125 B/param): single
    call and list call (three equal matrices, which share a launch), dense and row-interleaved state."""
    rng = np.random.default_rng(rows + cols)
    w0 = synth.weights(24, 1, rows, cols)
    w0[0, :8] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-40, 3e38, -3e38]
    gb = synth.grads_bf16(24, 1, 0, rows, cols)
    A = (1 + 0.2 * rng.standard_normal((rows, nseg))).astype(np.float32) if nseg else None
    cfg = B.iteration_config(3, 10, mask_period=1, lr=1e-3, lambda_=1e-3, scale_segments=nseg)
    cfg.refresh_mask = refresh
    cfg.flags |= B.FLAG_MU_BF16
    o = OracleState(w0, "f32")
    o.keep[:] = oracle.nm_select(w0, 2, 4)
    o.step(synth.widen_bf16(gb), oracle_cfg(cfg), A=A)
    want = oracle.bf16_rne(o.w if A is None else oracle.weight_scale(o.w, A))
    for interleaved, as_list in ((False, False), (True, False), (True, True), (False, True)):
        if interleaved and cols % 8:
            continue
        states = [GpuState(w0, nseg, interleaved=interleaved, mu_bf16=True) for _ in range(3 if as_list else 1)]
        copies = [torch.full((rows, cols), 7.0, dtype=torch.bfloat16, device=DEV) for _ in states]
        for st in states:
            B.cast_nm_select(st.w, 2, 4, st.mask)
        scale = None if A is None else dev(A)
        if as_list:
            tl = B.TensorList([dict(w=st.w, m=st.m, v=st.v, mask=st.mask, grad=gb.to(DEV), compute_copy=c, copy_scale=scale,
                                    scale=scale, scale_grad=st.scale_grad if nseg else None) for st, c in zip(states, copies)], DEV)
            B.cast_adams_step_multi(tl, cfg)
        else:
            B.cast_adams_step_emit(states[0].w, gb.to(DEV), states[0].m, states[0].v, states[0].mask, cfg, copies[0], copy_scale=scale,
                                   scale=scale, scale_grad=states[0].scale_grad if nseg else None)
        torch.cuda.synchronize()
        for st, c in zip(states, copies):
            assert_same_bits(host(st.w), o.w, "w")
            assert_same_bits(_mu(st.m), o.m, "mu")
            assert_same_bits(host(st.v), o.v, "v")
            got = host(c.view(torch.int16)).view(np.uint16)
            assert (got == want).all(), (interleaved, as_list, int((got != want).sum()))
