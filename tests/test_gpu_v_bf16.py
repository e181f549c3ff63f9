"""Both moments kept in bf16 (CAST_FLAG_MU_BF16 | CAST_FLAG_V_BF16) against the oracle's definition: the first
moment rounded to nearest even, the second one stochastically with the counter-based rounding bits of
(sr_seed, row * cols + col), both unrounded inside the iteration.  Every bit of w, mu, v and the mask, over the
patterns, layouts, shapes and launch forms the variant has: the rounding bits depend on the entry alone, so
whole-segment plans, pieces, shared launches and the one-thread-per-unit kernel must all agree."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, GpuState, OracleState, assert_same_bits, dev, host, oracle_cfg, words

pytestmark = pytest.mark.gpu


def _f(t: torch.Tensor) -> np.ndarray:
    assert t.dtype == torch.bfloat16
    return host(t.float())


@pytest.mark.parametrize("n,m", [(2, 4), (4, 8), (1, 2)])
@pytest.mark.parametrize("rows,cols,nseg", [(6, 512, 0), (6, 512, 2), (5, 1280 + 64, 2), (7, 72, 3), (3, 40, 0), (9, 24, 1),
                                            (12, 4096, 2), (5, 11008, 2), (33, 4096 + 32, 0), (6, 5120, 2), (4, 13824, 2),
                                            (2, 16384 + 256, 1)])      # the last one: 65 chunks for 16 wavefronts
@pytest.mark.parametrize("bf16_grad", [False, True])
@pytest.mark.parametrize("interleaved", [False, True])
def test_v_bf16_step_bit_exact(n, m, rows, cols, nseg, bf16_grad, interleaved):
    if cols % m or (nseg and (cols // nseg) % m) or (interleaved and cols % 8):
        pytest.skip("shape not valid for this M or layout")
    steps = 4
    rng = np.random.default_rng(rows * cols + n)
    w0 = synth.tie_outlier_weights(4, 7, rows, cols) if cols % 8 == 0 else synth.weights(4, 7, rows, cols)
    g = GpuState(w0, nseg, interleaved, mu_bf16=True, v_bf16=True)
    o = OracleState(w0, "f32")
    for t in range(steps):
        gr = synth.grads_f32(4, 7, t, rows, cols)
        if bf16_grad:
            gr = synth.widen_bf16(torch.from_numpy(gr).to(torch.bfloat16))
        cfg = B.iteration_config(t, steps, mask_period=2, lr=1e-3, lambda_=1e-3, n_keep=n, m_group=m, scale_segments=nseg)
        cfg.sr_seed = 0x9000_0000 + 77 * t
        A = (1 + 0.2 * rng.standard_normal((rows, nseg))).astype(np.float32) if nseg else None
        g.step(dev(gr, torch.bfloat16 if bf16_grad else None), cfg, scale=None if A is None else dev(A))
        assert cfg.flags & B.FLAG_MU_BF16 and cfg.flags & B.FLAG_V_BF16
        ref_gA = o.step(gr, oracle_cfg(cfg), A=A)
        if nseg:
            got = host(g.scale_grad)
            assert np.abs(got - ref_gA).max() <= 1e-5 * max(np.abs(ref_gA).max(), 1e-12) + 1e-9
    torch.cuda.synchronize()
    assert (words(g.mask) == oracle.pack_mask_bits(o.keep)).all()
    assert_same_bits(host(g.w), o.w, "w")
    assert_same_bits(_f(g.m), o.m, "mu")
    assert_same_bits(_f(g.v), o.v, "v")
    assert (o.v.view(np.uint32) & 0xFFFF == 0).all() and np.abs(o.v).max() > 0


def test_v_bf16_special_values():
    # NaN, infinities, zeros of both signs, denormals and the largest finite values in w and g (so also in v)
    rows, cols = 4, 64
    special = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-40, -1e-40, 3e38, -3e38, 1.0, -1.0, 65504.0], np.float32)
    w0 = synth.weights(5, 1, rows, cols)
    g0 = synth.grads_f32(5, 1, 0, rows, cols)
    w0[0, :12] = special
    g0[1, :12] = special
    w0[2, :12] = special
    g0[2, :12] = special[::-1]
    g0[3, :12] = np.array([1.8e19, -1.8e19, 1e19, 2e19, 1e-20, 1e-23, 3e-20, 1.0, 2.0, 3.0, 1e10, 1e-10], np.float32)   # v up to the top of the range
    st = GpuState(w0, 0, False, mu_bf16=True, v_bf16=True)
    o = OracleState(w0, "f32")
    for t in range(3):
        cfg = B.iteration_config(t, 3, mask_period=1, lr=1e-3, lambda_=1e-3)
        st.step(dev(g0), cfg)
        o.step(g0, oracle_cfg(cfg))
    torch.cuda.synchronize()
    assert_same_bits(host(st.w), o.w, "w")
    assert_same_bits(_f(st.m), o.m, "mu")
    assert_same_bits(_f(st.v), o.v, "v")


@pytest.mark.parametrize("nseg", [0, 2])
def test_v_bf16_list_call_with_and_without_compute_copy(nseg):
    # equal shapes share launches, the long rows are stepped in pieces, odd shapes one by one; every second matrix
    # also gets its bf16 compute copy written
    shapes = [(64, 512), (32, 1024), (64, 512), (5, 72), (64, 512), (16, 11008), (16, 11008), (7, 8768), (0, 64), (64, 512), (12, 5120),
              (3, 13824)]
    steps = 3
    for with_copies in (False, True):
        items, refs = [], []
        for i, (r, c) in enumerate(shapes):
            if nseg and (c // nseg) % 4:
                continue
            w0 = synth.weights(6, i, r, c)
            st = GpuState(w0, nseg, interleaved=r > 0 and c % 8 == 0 and i % 2 == 0, mu_bf16=True, v_bf16=True)
            A = (1 + 0.2 * np.random.default_rng(i).standard_normal((r, nseg))).astype(np.float32) if nseg else None
            item = dict(w=st.w, m=st.m, v=st.v, mask=st.mask, grad=None, scale=None if A is None else dev(A), scale_grad=st.scale_grad)
            if with_copies:
                item["compute_copy"] = torch.full((r, c), 3.0, dtype=torch.bfloat16, device=DEV)
                if nseg and i % 3 == 0:
                    item["copy_scale"] = item["scale"]
            items.append(item)
            refs.append((OracleState(w0, "f32"), A, i, (r, c)))
        for t in range(steps):
            cfg = B.iteration_config(t, steps, mask_period=2, lr=1e-3, lambda_=1e-3, scale_segments=nseg)
            cfg.sr_seed = 31 + t
            for item, (o, A, i, (r, c)) in zip(items, refs):
                gr = synth.grads_f32(6, i, t, r, c)
                item["grad"] = dev(gr)
                o.step(gr, oracle_cfg_with(cfg), A=A)
            B.cast_adams_step_multi(B.TensorList(items, DEV), cfg)
        torch.cuda.synchronize()
        for item, (o, A, i, (r, c)) in zip(items, refs):
            assert (words(item["mask"]) == oracle.pack_mask_bits(o.keep)).all(), (i, r, c)
            assert_same_bits(host(item["w"]), o.w, f"w of matrix {i} {r}x{c}")
            assert_same_bits(_f(item["m"]), o.m, f"mu of matrix {i} {r}x{c}")
            assert_same_bits(_f(item["v"]), o.v, f"v of matrix {i} {r}x{c}")
            if with_copies and r:
                scale = A if "copy_scale" in item else None
                want = oracle.bf16_rne(oracle.weight_scale(o.w, scale) if scale is not None else o.w)
                got = host(item["compute_copy"].view(torch.int16)).view(np.uint16)
                assert (got == want).all(), (i, r, c)


def oracle_cfg_with(cfg: B.AdamsConfig):
    """oracle_cfg for a list call: the binding sets the dtype flags inside the call, the oracle needs them before."""
    probe = B.AdamsConfig(**{k: getattr(cfg, k) for k in cfg.__dataclass_fields__})
    probe.flags |= B.FLAG_MU_BF16 | B.FLAG_V_BF16
    return oracle_cfg(probe)


@pytest.mark.parametrize("rows,cols", [(4096, 4096), (11008, 4096), (4096, 11008)])
def test_v_bf16_sampled_rows_of_full_size_matrices(rows, cols):
    """LLaMA2-7B shapes in the launch configuration bench.py times (row-interleaved state, bf16 gradients, n = 2,
    the list call): sampled whole rows.  The oracle steps the sampled rows as a small matrix with the second moment
    left in fp32, and what it would store is rounded with the exported rounding functions at the entries' true
    indices row * cols + col (the oracle's own whole-matrix step does the same; that is pinned on the CPU)."""
    n, steps, n_sample = 2, 3, 10
    w = synth.device_gaussian((rows, cols), 0.02, torch.float32, 11, DEV)
    g = synth.device_gaussian((rows, cols), 1e-3, torch.bfloat16, 12, DEV)
    w, m, v = B.interleaved_state(w, mu_bf16=True, v_bf16=True)
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
        cfg.sr_seed = 0xFFFF_FFF0 + t      # wraps around inside the key
        B.cast_adams_step_multi(tl, cfg)
        oc = oracle_cfg(cfg)
        assert oc.v_bf16 == 1 and oc.mu_bf16 == 1
        oc.v_bf16 = 0
        oracle.adams_step(ow, og, om, ov, keep, oc, A=oA, arithmetic="f32", nthreads=8)
        bits = ov.view(np.uint32)
        for k, r in enumerate(pick):
            for c in range(cols):
                bits[k, c] = oracle.bf16_stochastic(float(ov[k, c]), oracle.sr_bits(oc.sr_seed, int(r) * cols + c)) << 16
    torch.cuda.synchronize()
    assert (words(mask[idx]) == oracle.pack_mask_bits(keep)).all()
    assert_same_bits(host(w[idx]), ow, "w")
    assert_same_bits(_f(m[idx]), om, "mu")
    assert_same_bits(_f(v[idx]), ov, "v")
