"""cast_hbm_stream_probe, the measurement aid that makes the list call's launches with next to no arithmetic:
its few multiply-adds have a closed form (mu' = mu/2 + g, v' = v/2 + (kept ? g : mu'), w' = w/2 + v', bf16 moments
stored by truncation), so every entry of every matrix shows whether the launch plan of the step reached it exactly
once - shared launches, split plans, interleaved rows, all four storage variants.  Not a test of the method."""
import numpy as np
import pytest
import torch

from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, GpuState, assert_same_bits, host, words

pytestmark = pytest.mark.gpu

# equal shapes (shared launches), long segments (split plans with scaling), short rows, a tail chunk
SHAPES = [(64, 512)] * 3 + [(4, 11008), (33, 4096 + 64), (64, 512), (0, 64), (7, 2048), (2, 8192 + 64)] + [(16, 256)] * 18


def _truncate_bf16(x):
    return (np.ascontiguousarray(x, np.float32).view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)


@pytest.mark.parametrize("variant", ["fp32", "fp32_grads", "mu_bf16", "both_bf16"])
@pytest.mark.parametrize("nseg", [0, 2])
@pytest.mark.parametrize("interleaved", [False, True])
def test_probe_rewrites_every_entry_exactly_once(variant, nseg, interleaved):
    mu16, v16 = variant in ("mu_bf16", "both_bf16"), variant == "both_bf16"
    gdtype = torch.float32 if variant == "fp32_grads" else torch.bfloat16
    rng = np.random.default_rng(17)
    items, before = [], []
    for i, (r, c) in enumerate(SHAPES):
        st = GpuState(synth.weights(71, i, r, c), nseg, interleaved and r > 0, mu_bf16=mu16, v_bf16=v16)
        m0 = torch.from_numpy((1e-3 * rng.standard_normal((r, c))).astype(np.float32)).to(st.m.dtype)
        v0 = torch.from_numpy((1e-3 * rng.standard_normal((r, c))).astype(np.float32)).to(st.v.dtype)
        st.m.copy_(m0.to(DEV))
        st.v.copy_(v0.to(DEV))
        st.mask.copy_(torch.from_numpy(rng.integers(-2**31, 2**31, size=tuple(st.mask.shape), dtype=np.int64).astype(np.int32)))
        g = torch.from_numpy(synth.grads_f32(72, i, 0, r, c)).to(gdtype)
        x = dict(w=st.w, m=st.m, v=st.v, mask=st.mask, grad=g.to(DEV))
        if nseg:
            x.update(scale=torch.ones((r, nseg), device=DEV), scale_grad=st.scale_grad)
        items.append(x)
        before.append((host(st.w).copy(), m0.float().numpy(), v0.float().numpy(), g.float().numpy(), words(st.mask).copy()))
    tl = B.TensorList(items, DEV)
    B.cast_hbm_stream_probe(tl, nseg)
    torch.cuda.synchronize()
    half = np.float32(0.5)
    for x, (w, m, v, g, mask), (r, c) in zip(items, before, SHAPES):
        if r == 0:
            continue
        kept = ((mask[:, np.arange(c) // 32] >> (np.arange(c) % 32).astype(np.uint32)) & 1).astype(bool)
        m1 = half * m + g
        v1 = half * v + np.where(kept, g, m1)
        w1 = half * w + v1
        assert_same_bits(host(x["w"]), w1, f"w {r}x{c}")
        assert_same_bits(host(x["m"].float()), _truncate_bf16(m1) if mu16 else m1, f"m {r}x{c}")
        assert_same_bits(host(x["v"].float()), _truncate_bf16(v1) if v16 else v1, f"v {r}x{c}")
        assert (words(x["mask"]) == mask).all()
        if nseg:
            ref = (g.astype(np.float64) * w).reshape(r, nseg, -1).sum(-1)
            terms = np.abs(g.astype(np.float64) * w).reshape(r, nseg, -1).sum(-1)
            assert (np.abs(host(x["scale_grad"]) - ref) <= 1e-5 * terms + 1e-30).all()


def test_probe_refuses_what_it_has_no_kernel_for():
    r, c = 8, 512
    st = GpuState(synth.weights(73, 0, r, c), 0, False)
    g16 = torch.zeros((r, c), dtype=torch.bfloat16, device=DEV)
    tl = B.TensorList([dict(w=st.w, m=st.m, v=st.v, mask=st.mask, grad=g16)], DEV)
    lib = B.load()
    ws, n = B._ptr(tl.workspace), tl.workspace.numel()
    call = lambda dtype, flags: lib.cast_hbm_stream_probe(tl.array, 1, 0, dtype, flags, ws, n, None)
    assert call(B.CAST_F32, B.FLAG_MU_BF16) == -5          # bf16 moments come with bf16 gradients only
    assert call(B.CAST_BF16, B.FLAG_V_BF16) == -5          # the second moment alone
    assert call(B.CAST_BF16, 1) == -5
    assert call(7, 0) == -4
    odd = GpuState(synth.weights(73, 1, 4, 72), 0, False)      # a shape the vector kernels do not take
    tl2 = B.TensorList([dict(w=odd.w, m=odd.m, v=odd.v, mask=odd.mask, grad=torch.zeros((4, 72), dtype=torch.bfloat16, device=DEV))], DEV)
    assert lib.cast_hbm_stream_probe(tl2.array, 1, 0, B.CAST_BF16, 0, B._ptr(tl2.workspace), tl2.workspace.numel(), None) == -2
    torch.cuda.synchronize()
    assert_same_bits(host(st.w), synth.weights(73, 0, r, c), "nothing ran")


def test_stand_alone_skeleton_runs_every_variant():
    """The bare kernels of paper_2509_25996_amd/stream_skeleton (built by build.py beside the library) on a small
    ragged shape: every variant launches and reports a figure."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(B.__file__)), "stream_skeleton")
    assert os.path.exists(exe), "build it with python -m paper_2509_25996_amd.build"
    run = subprocess.run([exe, "96", "2816", "3"], capture_output=True, text=True, timeout=120)      # 2816 = 11 x 256 columns
    assert run.returncode == 0, run.stdout[-1500:] + run.stderr[-500:]
    lines = [x for x in run.stdout.splitlines() if "GB/s" in x]
    assert len(lines) == 2 * 17 and "HIP error" not in run.stdout      # 18 variants; the 4 KiB tiles do not divide 2816 columns
