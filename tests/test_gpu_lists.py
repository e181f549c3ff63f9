"""The list forms of the once-per-run entry points (cast_nm_select_multi, cast_weight_scale_multi,
cast_weight_scale_grad_multi, cast_nm_project_compress_multi): matrices of one shape share launches (blockIdx.y picks the matrix), other shapes
and the scalar kernels run in between; every output against the oracle, bit for bit (Eq. 6, Eq. 12, the last loop
of Algorithm 1 and the packed layout)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, assert_same_bits, dev, host, words

pytestmark = pytest.mark.gpu

# runs of equal shapes (shared launches, more than 16 of one shape: two launches), rows that end inside a workgroup's
# reach (2048 entries), rows shorter than one wavefront's, shapes for the scalar kernels (72, 40 columns), empty ones
SHAPES = [(64, 512)] * 3 + [(5, 72), (33, 4096 + 32), (64, 512), (0, 64), (7, 2048), (9, 11008), (3, 40), (7, 2048)] + [(16, 256)] * 19 + \
         [(2, 8192 + 64), (4, 64), (5, 72)]


def _state(shapes, seed, interleave_some=True):
    out = []
    for i, (r, c) in enumerate(shapes):
        w0 = synth.tie_outlier_weights(seed, i, r, c) if c % 8 == 0 and r else synth.weights(seed, i, r, c)
        if interleave_some and i % 3 == 1 and r and c % 8 == 0:
            w, _, _ = B.interleaved_state(dev(w0))
        else:
            w = dev(w0)
        out.append((w0, w))
    return out


@pytest.mark.parametrize("n,m", [(2, 4), (4, 8), (1, 2), (1, 4), (3, 4), (5, 8)])
def test_select_list_matches_the_oracle(n, m):
    state = _state(SHAPES, 61)
    masks = [B.alloc_mask(r, c, DEV) for r, c in SHAPES]
    for mk in masks:
        mk.fill_(-1)
    B.cast_nm_select_multi(B.MatrixList([dict(w=w, mask=mk) for (_, w), mk in zip(state, masks)]), n, m)
    torch.cuda.synchronize()
    for (w0, _), mk, shape in zip(state, masks, SHAPES):
        if w0.size:
            assert (words(mk) == oracle.pack_mask_bits(oracle.nm_select(w0, n, m))).all(), shape


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nseg", [1, 2, 4])
def test_weight_scale_list_matches_the_oracle(nseg, out_dtype):
    shapes = [s for s in SHAPES if s[1] % nseg == 0]
    state = _state(shapes, 62)
    rng = np.random.default_rng(5)
    A = [(1 + 0.3 * rng.standard_normal((r, nseg))).astype(np.float32) for r, _ in shapes]
    outs = [torch.full((r, c), 3.0, dtype=out_dtype, device=DEV) for r, c in shapes]
    B.cast_weight_scale_multi(B.MatrixList([dict(w=w, scale=dev(a), out=o) for (_, w), a, o in zip(state, A, outs)]))
    torch.cuda.synchronize()
    for (w0, _), a, o, shape in zip(state, A, outs, shapes):
        if not w0.size:
            continue
        ref = oracle.weight_scale(w0, a)
        if out_dtype == torch.float32:
            assert_same_bits(host(o), ref, str(shape))
        else:
            assert (host(o.view(torch.int16)).view(np.uint16) == oracle.bf16_rne(ref)).all(), shape


@pytest.mark.parametrize("grad_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nseg", [1, 2, 4])
def test_weight_scale_grad_list_matches_the_oracle_and_the_single_call(nseg, grad_dtype):
    """dL/dA (the derivative of Eq. 12 with respect to A) of a whole list: against the oracle's double sums within
    the rounding of a fp32 sum, and bit for bit what the call on one matrix gives."""
    shapes = [s for s in SHAPES if s[1] % nseg == 0 and (grad_dtype == torch.float32 or s[1] % 4 == 0)]
    state = _state(shapes, 63)
    grads = [torch.from_numpy(synth.grads_f32(9, i, 0, r, c)).to(grad_dtype) for i, (r, c) in enumerate(shapes)]
    outs = [torch.full((r, nseg), 7.0, device=DEV) for r, _ in shapes]
    dgrads = [g.to(DEV) for g in grads]
    B.cast_weight_scale_grad_multi(B.ScaleGradList([dict(w=w, grad=g, scale_grad=o) for (_, w), g, o in zip(state, dgrads, outs)]))
    torch.cuda.synchronize()
    for (w0, w), g, dg, o, (r, c) in zip(state, grads, dgrads, outs, shapes):
        if not w0.size:
            continue
        gs = g.float().numpy()
        ref = oracle.weight_scale_grad(w0, gs, nseg)
        terms = np.abs(gs.astype(np.float64) * w0).reshape(r, nseg, -1).sum(-1)
        assert (np.abs(host(o) - ref) <= 1e-5 * terms + 1e-30).all(), (r, c)
        single = torch.zeros((r, nseg), device=DEV)
        B.cast_weight_scale_grad(w, dg, nseg, single)
        assert host(single).tobytes() == host(o).tobytes(), (r, c)


@pytest.mark.parametrize("value_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,m", [(2, 4), (4, 8), (1, 2), (3, 8)])
@pytest.mark.parametrize("given_mask", [False, True])
def test_project_compress_list_matches_the_oracle(n, m, given_mask, value_dtype):
    nseg = 2
    shapes = [s for s in SHAPES if (s[1] // nseg) % m == 0]
    state = _state(shapes, 63)
    rng = np.random.default_rng(6)
    items, refs = [], []
    for i, ((w0, w), (r, c)) in enumerate(zip(state, shapes)):
        scaled = i % 4 != 2      # some matrices without a scale: they cannot share a launch with the scaled ones
        a = (1 + 0.3 * rng.standard_normal((r, nseg))).astype(np.float32) if scaled else None
        keep = None
        if given_mask and r:      # a stored mask that is NOT the projection of w: the weights of another draw decide
            keep = oracle.nm_select(synth.weights(64, i, r, c), n, m)
        _, vbytes, mbytes = B.cast_sizes(r, c, n, m, B.CAST_F32)
        values = torch.full((r, c // m * n), 5.0, dtype=value_dtype, device=DEV)
        meta = torch.full((r, (mbytes // 4 // r) if r else 0), -1, dtype=torch.int32, device=DEV)
        items.append(dict(w=w, scale=None if a is None else dev(a), out=values, meta=meta,
                          mask=None if keep is None else dev(oracle.pack_mask_bits(keep).view(np.int32))))
        refs.append((w0, a, keep))
    B.cast_nm_project_compress_multi(B.MatrixList(items), n, m)
    torch.cuda.synchronize()
    for x, (w0, a, keep), shape in zip(items, refs, shapes):
        if not w0.size:
            continue
        ref_v, ref_m = oracle.project_compress(w0, n, m, A=a, keep=keep)
        assert (words(x["meta"]) == ref_m).all(), shape
        if value_dtype == torch.float32:
            assert_same_bits(host(x["out"]), ref_v, str(shape))
        else:
            assert (host(x["out"].view(torch.int16)).view(np.uint16) == oracle.bf16_rne(ref_v)).all(), shape


def test_whole_7b_layer_through_the_list_calls():
    """One LLaMA2-7B-shaped layer (row-interleaved weights, n = 2): q, k, v, o share launches; selection, Eq. 12 into
    bf16 and the 2:4 pack with the fold, every entry against the oracle."""
    shapes = synth.weight_set("llama2_7b", 1)
    n = 2
    items, refs = [], []
    for i, (_, r, c) in enumerate(shapes):
        w, _, _ = B.interleaved_state(synth.device_gaussian((r, c), 0.02, torch.float32, 900 + i, DEV))
        A = (1 + 0.05 * torch.randn((r, n), device=DEV, generator=torch.Generator(DEV).manual_seed(i))).contiguous()
        items.append(dict(w=w, scale=A, mask=B.alloc_mask(r, c, DEV), out16=torch.empty((r, c), dtype=torch.bfloat16, device=DEV),
                          values=torch.empty((r, c // 2), device=DEV), meta=torch.empty((r, c // 32), dtype=torch.int32, device=DEV)))
        refs.append((host(w).copy(), host(A).copy()))
    B.cast_nm_select_multi(B.MatrixList([dict(w=x["w"], mask=x["mask"]) for x in items]), 2, 4)
    B.cast_weight_scale_multi(B.MatrixList([dict(w=x["w"], scale=x["scale"], out=x["out16"]) for x in items]))
    B.cast_nm_project_compress_multi(B.MatrixList([dict(w=x["w"], scale=x["scale"], out=x["values"], meta=x["meta"]) for x in items]), 2, 4)
    torch.cuda.synchronize()
    for (name, r, c), x, (w0, a) in zip(shapes, items, refs):
        assert (words(x["mask"]) == oracle.pack_mask_bits(oracle.nm_select(w0, 2, 4))).all(), name
        assert (host(x["out16"].view(torch.int16)).view(np.uint16) == oracle.bf16_rne(oracle.weight_scale(w0, a))).all(), name
        ref_v, ref_m = oracle.project_compress(w0, 2, 4, A=a)
        assert (words(x["meta"]) == ref_m).all(), name
        assert_same_bits(host(x["values"]), ref_v, name)


@pytest.mark.parametrize("n,m,rows,cols", [(2, 4, 33, 4096 + 32), (4, 8, 9, 11008), (1, 2, 7, 2048), (3, 8, 5, 72), (2, 4, 5, 72)])
def test_stored_masks_are_checked_when_a_status_word_is_given(n, m, rows, cols):
    """A stored mask must hold exactly N ones per group (Eq. 4); the oracle refuses one that does not.  The list call
    counts such groups into the caller's status word: zero for a valid mask, the exact number for a damaged one."""
    w0 = synth.weights(71, 0, rows, cols)
    keep = oracle.nm_select(w0, n, m)
    rng = np.random.default_rng(rows + cols)
    damaged = keep.copy()
    groups = damaged.reshape(rows, cols // m, m)
    hit = rng.random((rows, cols // m)) < 0.03
    hit[0, 0] = hit[-1, -1] = True
    for r, g in zip(*np.nonzero(hit)):      # one more or one fewer bit, or none at all
        kind = rng.integers(0, 3)
        if kind == 0:
            groups[r, g, np.flatnonzero(groups[r, g] == 0)[0]] = 1
        elif kind == 1:
            groups[r, g, np.flatnonzero(groups[r, g] == 1)[0]] = 0
        else:
            groups[r, g, :] = 0
    with pytest.raises(ValueError):
        oracle.project_compress(w0, n, m, keep=damaged)
    _, _, mbytes = B.cast_sizes(rows, cols, n, m, B.CAST_F32)
    for mask, want in ((keep, 0), (damaged, int(hit.sum()))):
        status = torch.zeros(1, dtype=torch.int32, device=DEV)
        item = dict(w=dev(w0), out=torch.empty((rows, cols // m * n), device=DEV), meta=torch.empty((rows, mbytes // 4 // rows), dtype=torch.int32, device=DEV),
                    mask=dev(oracle.pack_mask_bits(mask).view(np.int32)), mask_status=status)
        B.cast_nm_project_compress_multi(B.MatrixList([item]), n, m)
        torch.cuda.synchronize()
        assert int(status.item()) == want
        if want == 0:
            ref_v, ref_m = oracle.project_compress(w0, n, m, keep=keep)
            assert (words(item["meta"]) == ref_m).all()
            assert_same_bits(host(item["out"]), ref_v, "values")


@pytest.mark.parametrize("with_other", [True, False])
def test_mask_stats_list_matches_the_oracle(with_other):
    """Appendix "Mask Learning" over a list: flips against another mask (exact), ||W (.) M||_1 and ||W||_1 (1e-6
    relative: fp32 partial sums per workgroup, double across them), per matrix, and reproducible bit for bit."""
    shapes = SHAPES + [(700, 2048)]      # the last one: more workgroups than the summing kernel has threads
    state = _state(shapes, 66)
    items, refs = [], []
    for i, ((w0, w), (r, c)) in enumerate(zip(state, shapes)):
        keep = oracle.nm_select(w0, 2, 4) if r else np.zeros((0, c), np.uint8)
        other = oracle.nm_select(synth.weights(67, i, r, c), 2, 4) if (r and with_other) else None
        items.append(dict(w=w, mask=dev(oracle.pack_mask_bits(keep).view(np.int32)),
                          other=None if other is None else dev(oracle.pack_mask_bits(other).view(np.int32)),
                          stats=torch.full((4,), -1, dtype=torch.int64, device=DEV)))
        refs.append((w0, keep, other))
    sl = B.StatsList(items, DEV)
    runs = []
    for _ in range(2):
        B.cast_mask_stats_multi(sl)
        torch.cuda.synchronize()
        runs.append([host(x["stats"]).tobytes() for x in items])
    assert runs[0] == runs[1]
    for x, (w0, keep, other), shape in zip(items, refs, shapes):
        got = B.read_refresh_stats(x["stats"])
        flips, kept, total = oracle.mask_stats(w0, keep, other) if w0.size else (0, 0.0, 0.0)
        assert got["flips_prev"] == flips and got["flips_init"] == 0, shape
        assert abs(got["l1_kept"] - kept) <= 1e-6 * kept and abs(got["l1_all"] - total) <= 1e-6 * total, shape


def test_pack_1of2_with_scale_segments_of_half_a_lane():
    """1:2 with scale segments of 6 entries: groups of 2 never straddle a segment, but the 4 consecutive entries a lane
    of the fast kernel holds would; such shapes must take the scalar kernel and still match the oracle."""
    rows, cols, nseg = 8, 192, 32
    w0 = synth.weights(72, 0, rows, cols)
    A = (1 + 0.5 * np.random.default_rng(3).standard_normal((rows, nseg))).astype(np.float32)
    _, _, mbytes = B.cast_sizes(rows, cols, 1, 2, B.CAST_F32)
    values = torch.empty((rows, cols // 2), device=DEV)
    meta = torch.empty((rows, mbytes // 4 // rows), dtype=torch.int32, device=DEV)
    B.cast_nm_project_compress(dev(w0), 1, 2, values, meta, scale=dev(A))
    torch.cuda.synchronize()
    ref_v, ref_m = oracle.project_compress(w0, 1, 2, A=A)
    assert (words(meta) == ref_m).all()
    assert_same_bits(host(values), ref_v, "values")
