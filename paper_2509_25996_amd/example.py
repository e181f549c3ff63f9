"""A complete pass through the library on synthetic data: Algorithm 1's loop over a few weight matrices with
the list call (alpha_t = t/T, mask refresh every T_1 steps, weight scaling with n = 2 segments, refresh
statistics gathered by the refresh steps themselves), then the hard N:M projection with the last refreshed
mask, the fold of the scale factors and packing (Algorithm 1's last lines, Eq. 12).

    python -m paper_2509_25996_amd.example

With bf16_moments=True both moments are kept in bf16 (the second one rounded stochastically, a fresh seed per
step: iteration_config sets cfg.sr_seed = t).

Gradients are random draws, not a loss: the point is the calling sequence, and that under the ramp the
masked weights are driven to zero (Sec. 4.1, appendix "Mask Learning"), which the numbers it prints show.
The scale factors are stepped from scale_grad by a plain Adam, itself a call into the library (DenseAdam below):
the paper leaves their optimizer open.  All of them live in one flat buffer (and their gradients in another), so
that this Adam is one launch per step however many matrices there are.
"""
from __future__ import annotations

import torch

from . import binding as B
from . import synth


class DenseAdam:
    """Textbook Adam on a dense fp32 [rows, cols] tensor (cols even) as a special case of the library's step:
    alpha = 0 switches the decay off (the mask is then ignored), CAST_FLAG_V_FROM_GRAD feeds the second moment
    with g^2, and the N:M pattern is a formality (1:2).  Meant for the scale factors A of Eq. 12."""

    def __init__(self, p: torch.Tensor, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8):
        self.p, self.lr, self.beta1, self.beta2, self.eps = p, lr, beta1, beta2, eps
        self.m, self.v = torch.zeros_like(p), torch.zeros_like(p)
        self.mask = B.alloc_mask(p.shape[0], p.shape[1], p.device)      # read, never used: alpha = 0
        self.t = 0

    def step(self, grad: torch.Tensor, lr=None):
        self.t += 1
        cfg = B.AdamsConfig(n_keep=1, m_group=2, lr=self.lr if lr is None else lr, beta1=self.beta1, beta2=self.beta2,
                            eps=self.eps, lambda_=0.0, alpha=0.0, bias_corr1=1.0 - self.beta1 ** self.t,
                            bias_corr2=1.0 - self.beta2 ** self.t, refresh_mask=0, flags=B.FLAG_V_FROM_GRAD)
        B.cast_adams_step(self.p, grad, self.m, self.v, self.mask, cfg)


def run(shapes=((256, 1024), (512, 512), (256, 2048)), steps=200, mask_period=10, lr=1e-3, lam=1e-3, n_keep=2, m_group=4,
        segments=2, device="cuda:0", verbose=True, bf16_moments=False):
    """Returns a dict of what a training script would monitor; see the module docstring."""
    B.load()
    items, stats = [], []
    # every matrix's scale factors and their gradients are slices of two flat buffers, padded to whole rows of 64
    # for the dense Adam that steps them all at once
    n_scale = sum(r * segments for r, _ in shapes)
    scale_all = torch.ones(((n_scale + 63) // 64, 64), device=device)
    scale_grad_all = torch.zeros_like(scale_all)
    at = 0
    for i, (r, c) in enumerate(shapes):
        w, m, v = B.interleaved_state(synth.device_gaussian((r, c), 0.02, torch.float32, 100 + i, device),
                                      mu_bf16=bf16_moments, v_bf16=bf16_moments)
        mask, initial = B.alloc_mask(r, c, device), B.alloc_mask(r, c, device)
        stats.append(B.alloc_refresh_stats(device))
        items.append(dict(w=w, m=m, v=v, mask=mask, grad=torch.empty((r, c), dtype=torch.bfloat16, device=device),
                          scale=scale_all.view(-1)[at:at + r * segments].view(r, segments),
                          scale_grad=scale_grad_all.view(-1)[at:at + r * segments].view(r, segments),
                          initial_mask=initial, refresh_stats=stats[-1]))
        at += r * segments
    # the masks of the dense model, for the initial flip rate: Eq. 6 over the whole list in one call
    B.cast_nm_select_multi(B.MatrixList([dict(w=x["w"], mask=x["initial_mask"]) for x in items]), n_keep, m_group)
    for x in items:
        x["mask"].copy_(x["initial_mask"])
    tensors = B.TensorList(items, device)
    scale_optimizer = DenseAdam(scale_all, lr=1e-4)
    total = sum(r * c for r, c in shapes)
    history = []
    gen = torch.Generator(device=device).manual_seed(0)
    for t in range(steps):
        for x in items:                                               # stand-in for the backward pass
            x["grad"].copy_(torch.randn(x["grad"].shape, device=device, generator=gen) * 1e-3)
        cfg = B.iteration_config(t, steps, mask_period=mask_period, lr=lr, lambda_=lam, n_keep=n_keep, m_group=m_group,
                                 scale_segments=segments)
        B.cast_adams_step_multi(tensors, cfg)
        scale_optimizer.step(scale_grad_all)                          # A <- Adam(A, dL/dA); the step above used the old A
        if cfg.refresh_mask:
            s = [B.read_refresh_stats(x) for x in stats]
            flip_rate = sum(x["flips_prev"] for x in s) / total       # r_t
            initial_flip_rate = sum(x["flips_init"] for x in s) / total       # i_t
            kept_ratio = sum(x["l1_kept"] for x in s) / sum(x["l1_all"] for x in s)       # S_t
            history.append((t, flip_rate, initial_flip_rate, kept_ratio))
            if verbose and (t // mask_period) % max(1, steps // mask_period // 8) == 0:
                print(f"step {t:5d}  alpha {cfg.alpha:5.3f}  flip rate {flip_rate:.5f}  against the initial mask "
                      f"{initial_flip_rate:.5f}  ||W.M||_1 / ||W||_1 = {kept_ratio:.5f}")
    # Algorithm 1's end: prune with the last refreshed mask, fold the scale, pack values + index metadata; one list
    # call, which also checks that every stored mask holds exactly N ones per group
    packed, outputs = [], []
    bad_groups = torch.zeros(1, dtype=torch.int32, device=device)
    for x, (r, c) in zip(items, shapes):
        _, _, meta_bytes = B.cast_sizes(r, c, n_keep, m_group, B.CAST_BF16)
        values = torch.empty((r, c // m_group * n_keep), dtype=torch.bfloat16, device=device)
        meta = torch.empty((r, meta_bytes // 4 // r), dtype=torch.int32, device=device)
        outputs.append(dict(w=x["w"], scale=x["scale"], mask=x["mask"], out=values, meta=meta, mask_status=bad_groups))
        packed.append((values, meta))
    B.cast_nm_project_compress_multi(B.MatrixList(outputs), n_keep, m_group)
    torch.cuda.synchronize()
    assert int(bad_groups.item()) == 0, "a stored mask is not an N:M mask"
    # what the pruning removes: the largest masked weight and the share of the L1 norm it carried
    worst, masked_l1, all_l1 = 0.0, 0.0, 0.0
    for x, (r, c) in zip(items, shapes):
        words = x["mask"].cpu().numpy().view("uint32")
        bits = ((words[:, :, None] >> torch.arange(32).numpy()[None, None, :]) & 1).reshape(r, -1)[:, :c].astype(bool)
        w = x["w"].cpu().numpy()
        worst = max(worst, float(abs(w[~bits]).max()))
        masked_l1 += float(abs(w[~bits]).sum())
        all_l1 += float(abs(w).sum())
    if verbose:
        print(f"after {steps} steps: largest masked |w| = {worst:.3e} (lr = {lr:g}); pruning removes "
              f"{100 * masked_l1 / all_l1:.4f} % of ||W||_1; packed {len(packed)} matrices")
    return {"history": history, "largest_masked_weight": worst, "pruned_l1_share": masked_l1 / all_l1, "packed": packed,
            "items": items}


if __name__ == "__main__":
    run()
