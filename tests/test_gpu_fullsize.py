"""Parity at the full sizes of the benchmark workloads, in the launch configuration the
benchmark times (2:4, bf16 gradients, weight scaling with n = 2, w/mu/v row-interleaved in one
buffer, the list call, which steps long row segments in pieces) and in the plain one (three dense
arrays, one cast_adams_step call).

The AdamS step is checked on whole matrices for the LLaMA2-7B shapes and on sampled whole rows for the
others (a row is self-contained: groups and scale segments never cross rows), gathered before and after
the GPU step and recomputed by the oracle.
Selection and hard projection + pack of the tie/outlier stress input are compared in full."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, assert_same_bits, host, oracle_cfg, words

pytestmark = pytest.mark.gpu

SHAPES_7B = [(4096, 4096), (11008, 4096), (4096, 11008)]
SHAPES_13B = [(5120, 5120), (13824, 5120), (5120, 13824)]
SHAPES_LLAMA3_8B = [(1024, 4096), (4096, 14336)]      # the shapes LLaMA3-8B adds (k/v of grouped-query attention, down)


@pytest.mark.parametrize("as_benchmarked", [True, False])
@pytest.mark.parametrize("rows,cols", SHAPES_7B + SHAPES_13B + SHAPES_LLAMA3_8B)
def test_step_on_full_size_matrices(rows, cols, as_benchmarked):
    n, steps, n_sample = 2, 3, 24
    w = synth.device_gaussian((rows, cols), 0.02, torch.float32, 11, DEV)
    g = synth.device_gaussian((rows, cols), 1e-3, torch.bfloat16, 12, DEV)
    if as_benchmarked:
        w, m, v = B.interleaved_state(w)
    else:
        m, v = torch.zeros_like(w), torch.zeros_like(w)
    mask = B.alloc_mask(rows, cols, DEV)
    A = (1 + 0.05 * torch.randn((rows, n), device=DEV, generator=torch.Generator(DEV).manual_seed(3))).contiguous()
    gA = torch.zeros((rows, n), device=DEV)
    rng = np.random.default_rng(rows + cols)
    pick = np.unique(np.concatenate([[0, rows - 1], rng.integers(0, rows, n_sample)]))
    if (rows, cols) in SHAPES_7B:
        pick = np.arange(rows)      # the shapes of the headline: every entry
    idx = torch.from_numpy(pick).to(DEV)
    ow, og, oA = host(w[idx]).copy(), host(g[idx].float()).copy(), host(A[idx]).copy()
    om, ov = np.zeros_like(ow), np.zeros_like(ow)
    keep = np.zeros(ow.shape, np.uint8)
    tl = B.TensorList([dict(w=w, grad=g, m=m, v=v, mask=mask, scale=A, scale_grad=gA)], DEV) if as_benchmarked else None
    for t in range(steps):
        cfg = B.iteration_config(t, 7500, mask_period=2, lr=2e-5, lambda_=4e-7, scale_segments=n)
        cfg.alpha = 0.25 + 0.25 * t      # exercise the decay as late in training
        if as_benchmarked:
            B.cast_adams_step_multi(tl, cfg)
        else:
            B.cast_adams_step(w, g, m, v, mask, cfg, scale=A, scale_grad=gA)
        w_in = ow.copy()
        ref_gA = oracle.adams_step(ow, og, om, ov, keep, oracle_cfg(cfg), A=oA, arithmetic="f32", nthreads=16)
    torch.cuda.synchronize()
    assert (words(mask[idx]) == oracle.pack_mask_bits(keep)).all()
    assert_same_bits(host(w[idx]), ow, "w")
    assert_same_bits(host(m[idx]), om, "mu")
    assert_same_bits(host(v[idx]), ov, "v")
    terms = np.abs(og.astype(np.float64) * w_in).reshape(len(pick), n, -1).sum(-1)
    assert (np.abs(host(gA[idx]) - ref_gA) <= 1e-5 * terms + 1e-30).all()
    # properties that hold for the whole matrix: exactly 2 bits per group in every mask word, state finite
    bits = mask.view(torch.uint8)
    lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.uint8, device=DEV)
    nib_ok = torch.tensor([(bin(i & 15).count("1") == 2 and bin(i >> 4).count("1") == 2) for i in range(256)], device=DEV)
    assert bool(nib_ok[bits.long()].all())
    assert int(lut[bits.long()].sum(dtype=torch.int64)) == rows * cols // 2
    assert bool(torch.isfinite(w).all()) and bool(torch.isfinite(v).all()) and bool((v >= 0).all())


@pytest.mark.parametrize("with_copy", [False, True])
@pytest.mark.parametrize("rule", [B.RULE_ADAMW_L1, B.RULE_ADAM_L1, B.RULE_ADDITIVE, B.RULE_MASKED_FROZEN])
@pytest.mark.parametrize("rows,cols", SHAPES_7B)
def test_comparison_rules_on_sampled_rows_of_full_size_matrices(rows, cols, rule, with_copy):
    """The comparison rules (Eq. 9, Eq. 10, additive decay, frozen masked entries) on the LLaMA2-7B shapes in the
    configuration bench.py times them in (row-interleaved state, bf16 gradients, n = 2, the list call), alone and
    with the bf16 compute copy written along: sampled whole rows, every bit."""
    n, steps, n_sample = 2, 3, 16
    w = synth.device_gaussian((rows, cols), 0.02, torch.float32, 21, DEV)
    g = synth.device_gaussian((rows, cols), 1e-3, torch.bfloat16, 22, DEV)
    w, m, v = B.interleaved_state(w)
    mask = B.alloc_mask(rows, cols, DEV)
    A = (1 + 0.05 * torch.randn((rows, n), device=DEV, generator=torch.Generator(DEV).manual_seed(4))).contiguous()
    gA = torch.zeros((rows, n), device=DEV)
    copy = torch.zeros((rows, cols), dtype=torch.bfloat16, device=DEV) if with_copy else None
    rng = np.random.default_rng(rows + cols + rule)
    pick = np.unique(np.concatenate([[0, rows - 1], rng.integers(0, rows, n_sample)]))
    idx = torch.from_numpy(pick).to(DEV)
    ow, og, oA = host(w[idx]).copy(), host(g[idx].float()).copy(), host(A[idx]).copy()
    om, ov = np.zeros_like(ow), np.zeros_like(ow)
    keep = np.zeros(ow.shape, np.uint8)
    item = dict(w=w, grad=g, m=m, v=v, mask=mask, scale=A, scale_grad=gA)
    if with_copy:
        item.update(compute_copy=copy, copy_scale=A)
    tl = B.TensorList([item], DEV)
    for t in range(steps):
        cfg = B.iteration_config(t, 7500, mask_period=2, lr=2e-5, lambda_=4e-4, scale_segments=n, rule=rule)
        cfg.alpha = 0.25 + 0.25 * t
        B.cast_adams_step_multi(tl, cfg)
        oracle.adams_step(ow, og, om, ov, keep, oracle_cfg(cfg), A=oA, arithmetic="f32", nthreads=8)
    torch.cuda.synchronize()
    assert (words(mask[idx]) == oracle.pack_mask_bits(keep)).all()
    assert_same_bits(host(w[idx]), ow, "w")
    assert_same_bits(host(m[idx]), om, "mu")
    assert_same_bits(host(v[idx]), ov, "v")
    if with_copy:
        want = oracle.bf16_rne(oracle.weight_scale(ow, oA))
        assert (host(copy[idx].view(torch.int16)).view(np.uint16) == want).all()


@pytest.mark.parametrize("rows,cols", SHAPES_7B)
@pytest.mark.parametrize("n,m", [(2, 4), (4, 8), (1, 2)])
def test_tie_outlier_select_project_pack_full_size(rows, cols, n, m):
    w = synth.tie_outlier_weights(5, rows % 7, rows, cols)
    wd = torch.from_numpy(w).to(DEV)
    mask = B.alloc_mask(rows, cols, DEV)
    B.cast_nm_select(wd, n, m, mask)
    keep = oracle.nm_select(w, n, m)
    assert (words(mask) == oracle.pack_mask_bits(keep)).all()
    assert (keep.reshape(rows, -1, m).sum(-1) == n).all()
    _, vbytes, mbytes = B.cast_sizes(rows, cols, n, m, B.CAST_F32)
    values = torch.empty((rows, cols // m * n), device=DEV)
    meta = torch.empty((rows, mbytes // 4 // rows), dtype=torch.int32, device=DEV)
    B.cast_nm_project_compress(wd, n, m, values, meta)
    torch.cuda.synchronize()
    ref_v, ref_m = oracle.project_compress(w, n, m)
    assert (words(meta) == ref_m).all()
    assert_same_bits(host(values), ref_v, "values")


def test_whole_125m_set_through_the_list_call():
    """Every linear weight of the 125M-shaped set (84 matrices, 84.9 M parameters) stepped by the list call
    (which steps up to 16 small matrices of one shape per launch) over a ramp with mask refreshes, against the
    oracle tensor by tensor, bit for bit."""
    shapes = synth.weight_set("opt125m")
    n, steps = 2, 6
    items, refs = [], []
    for i, (_, r, c) in enumerate(shapes):
        w0 = synth.weights(21, i, r, c)
        w, m, v = B.interleaved_state(torch.from_numpy(w0).to(DEV))
        A = (1 + 0.05 * np.random.default_rng(i).standard_normal((r, n))).astype(np.float32)
        items.append(dict(w=w, m=m, v=v, mask=B.alloc_mask(r, c, DEV), grad=torch.zeros((r, c), dtype=torch.bfloat16, device=DEV),
                          scale=torch.from_numpy(A).to(DEV), scale_grad=torch.zeros((r, n), device=DEV)))
        refs.append(dict(w=w0.copy(), m=np.zeros_like(w0), v=np.zeros_like(w0), keep=np.zeros(w0.shape, np.uint8), A=A))
    tl = B.TensorList(items, DEV)
    step_launches, _ = B.cast_adams_multi_launches(tl, B.AdamsConfig(scale_segments=n))
    assert step_launches < len(shapes) // 2          # small matrices share launches
    for t in range(steps):
        cfg = B.iteration_config(t, steps, mask_period=2, lr=1e-3, lambda_=1e-3, scale_segments=n)
        for i, (_, r, c) in enumerate(shapes):
            g = synth.grads_bf16(21, i, t, r, c)
            items[i]["grad"].copy_(g.to(DEV))
            ref = refs[i]
            ref["gA"] = oracle.adams_step(ref["w"], synth.widen_bf16(g), ref["m"], ref["v"], ref["keep"], oracle_cfg(cfg),
                                          A=ref["A"], arithmetic="f32", nthreads=16)
        B.cast_adams_step_multi(tl, cfg)
    torch.cuda.synchronize()
    for i, (name, r, c) in enumerate(shapes):
        x, ref = items[i], refs[i]
        assert (words(x["mask"]) == oracle.pack_mask_bits(ref["keep"])).all(), name
        assert_same_bits(host(x["w"]), ref["w"], name + " w")
        assert_same_bits(host(x["m"]), ref["m"], name + " mu")
        assert_same_bits(host(x["v"]), ref["v"], name + " v")
        g = synth.widen_bf16(synth.grads_bf16(21, i, steps - 1, r, c))
        assert np.abs(host(x["scale_grad"]) - ref["gA"]).max() <= 1e-5 * np.abs(ref["gA"]).max() + 1e-7


@pytest.mark.parametrize("interleaved", [False, True])
def test_arrays_beyond_4_gib_sampled_rows(interleaved):
    """One matrix whose fp32 arrays are 4.3 GB each (65544 x 16384; with row-interleaved state the offsets inside
    the one allocation pass 2^32 entries): selection, the scaled step through both entry points and the pack,
    checked on whole rows around every place where a byte or entry offset crosses 2^31 or 2^32, on the first
    and last rows and on random ones."""
    rows, cols, n = 65536 + 8, 16384, 2
    w0 = synth.device_gaussian((rows, cols), 0.02, torch.float32, 41, DEV)
    g = synth.device_gaussian((rows, cols), 1e-3, torch.bfloat16, 42, DEV)
    if interleaved:
        w, m, v = B.interleaved_state(w0)
        del w0
    else:
        w, m, v = w0, torch.zeros_like(w0), torch.zeros_like(w0)
    ld = w.stride(0)
    crossing = []
    for limit in (1 << 31, 1 << 32):
        for unit in (4 * ld, 2 * cols, ld, cols):      # bytes of a state row, bytes of a gradient row, entries of either
            r = limit // unit
            crossing += [r - 1, r, r + 1]
    rng = np.random.default_rng(7)
    pick = np.unique(np.clip(np.concatenate([[0, 1, rows - 2, rows - 1], crossing, rng.integers(0, rows, 12)]), 0, rows - 1))
    idx = torch.from_numpy(pick).to(DEV)
    mask = B.alloc_mask(rows, cols, DEV)
    A = (1 + 0.05 * torch.randn((rows, n), device=DEV, generator=torch.Generator(DEV).manual_seed(5))).contiguous()
    gA = torch.zeros((rows, n), device=DEV)
    ow, og, oA = host(w[idx]).copy(), host(g[idx].float()).copy(), host(A[idx]).copy()
    om, ov = np.zeros_like(ow), np.zeros_like(ow)
    keep = np.zeros(ow.shape, np.uint8)
    # selection alone
    B.cast_nm_select(w, 2, 4, mask)
    torch.cuda.synchronize()
    assert (words(mask[idx]) == oracle.pack_mask_bits(oracle.nm_select(ow, 2, 4))).all()
    mask.zero_()
    # three steps: list call (split plan), single call, list call
    tl = B.TensorList([dict(w=w, grad=g, m=m, v=v, mask=mask, scale=A, scale_grad=gA)], DEV)
    for t in range(3):
        cfg = B.iteration_config(t, 7500, mask_period=2, lr=2e-5, lambda_=4e-7, scale_segments=n)
        cfg.alpha = 0.25 + 0.25 * t
        if t == 1:
            B.cast_adams_step(w, g, m, v, mask, cfg, scale=A, scale_grad=gA)
        else:
            B.cast_adams_step_multi(tl, cfg)
        ref_gA = oracle.adams_step(ow, og, om, ov, keep, oracle_cfg(cfg), A=oA, arithmetic="f32", nthreads=8)
    torch.cuda.synchronize()
    assert (words(mask[idx]) == oracle.pack_mask_bits(keep)).all()
    assert_same_bits(host(w[idx]), ow, "w")
    assert_same_bits(host(m[idx]), om, "mu")
    assert_same_bits(host(v[idx]), ov, "v")
    terms = np.abs(og.astype(np.float64) * host(w[idx])).reshape(len(pick), n, -1).sum(-1)
    assert (np.abs(host(gA[idx]) - ref_gA) <= 2e-5 * terms + 1e-12).all()
    # every mask word of the matrix has 16 of its 32 bits set (2:4)
    lut = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.uint8, device=DEV)
    assert int(lut[mask.view(torch.uint8).long()].sum(dtype=torch.int64)) == rows * cols // 2
    # hard projection + fold + pack with the stored mask
    _, vbytes, mbytes = B.cast_sizes(rows, cols, 2, 4, B.CAST_F32)
    values = torch.empty((rows, cols // 2), device=DEV)
    meta = torch.empty((rows, mbytes // 4 // rows), dtype=torch.int32, device=DEV)
    B.cast_nm_project_compress(w, 2, 4, values, meta, scale=A, mask_bits=mask)
    torch.cuda.synchronize()
    ref_v, ref_m = oracle.project_compress(ow, 2, 4, A=oA, keep=keep)
    assert (words(meta[idx]) == ref_m).all()
    assert_same_bits(host(values[idx]), ref_v, "values")


def test_whole_125m_set_100_steps_of_the_ramp_then_pack():
    """The 125M-class workload as a whole: all 84 linear weights, fp32 master weights, bf16 gradients, 100 AdamS
    2:4 steps through the list call with the decay ramped linearly from 0, masks refreshed every 10 steps, weight
    scaling n = 2, then hard projection + fold + pack; every tensor against the oracle, bit for bit.  Gradients are
    drawn on the GPU from a seeded generator, one flat buffer per step, and handed to both sides."""
    shapes = synth.weight_set("opt125m")
    n, steps, lam = 2, 100, 1e-3      # lambda of the gradients' order, so that masks flip within 100 steps
    total = synth.set_params(shapes)
    gflat = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    items, refs, at = [], [], 0
    for i, (_, r, c) in enumerate(shapes):
        w0 = synth.weights(22, i, r, c)
        w, m, v = B.interleaved_state(torch.from_numpy(w0).to(DEV))
        A = (1 + 0.05 * np.random.default_rng(100 + i).standard_normal((r, n))).astype(np.float32)
        items.append(dict(w=w, m=m, v=v, mask=B.alloc_mask(r, c, DEV), grad=gflat[at:at + r * c].view(r, c),
                          scale=torch.from_numpy(A).to(DEV), scale_grad=torch.zeros((r, n), device=DEV)))
        refs.append(dict(w=w0.copy(), m=np.zeros_like(w0), v=np.zeros_like(w0), keep=np.zeros(w0.shape, np.uint8), A=A, at=at))
        at += r * c
    tl = B.TensorList(items, DEV)
    gen = torch.Generator(device=DEV).manual_seed(2024)
    first_keep = None
    for t in range(steps):
        gflat.copy_(torch.randn(total, device=DEV, generator=gen) * 1e-3)
        ghost = gflat.float().cpu().numpy()
        cfg = B.iteration_config(t, steps, mask_period=10, lr=1e-4, lambda_=lam, scale_segments=n)
        B.cast_adams_step_multi(tl, cfg)
        for (_, r, c), ref in zip(shapes, refs):
            oracle.adams_step(ref["w"], ghost[ref["at"]:ref["at"] + r * c].reshape(r, c), ref["m"], ref["v"], ref["keep"],
                              oracle_cfg(cfg), A=ref["A"], want_gA=False, arithmetic="f32", nthreads=16)
        if t == 0:
            first_keep = [ref["keep"].copy() for ref in refs]
    torch.cuda.synchronize()
    flipped = 0
    for i, (name, r, c) in enumerate(shapes):
        x, ref = items[i], refs[i]
        assert (words(x["mask"]) == oracle.pack_mask_bits(ref["keep"])).all(), name
        assert_same_bits(host(x["w"]), ref["w"], name + " w")
        assert_same_bits(host(x["m"]), ref["m"], name + " mu")
        assert_same_bits(host(x["v"]), ref["v"], name + " v")
        flipped += int((ref["keep"] != first_keep[i]).sum())
        _, _, mbytes = B.cast_sizes(r, c, 2, 4, B.CAST_F32)
        values = torch.empty((r, c // 2), device=DEV)
        meta = torch.empty((r, mbytes // 4 // r), dtype=torch.int32, device=DEV)
        B.cast_nm_project_compress(x["w"], 2, 4, values, meta, scale=x["scale"], mask_bits=x["mask"])
        ref_v, ref_m = oracle.project_compress(ref["w"], 2, 4, A=ref["A"], keep=ref["keep"])
        assert (words(meta) == ref_m).all(), name
        assert_same_bits(host(values), ref_v, name + " values")
    assert flipped > 0
