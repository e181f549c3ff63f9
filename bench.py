#!/usr/bin/env python3
"""Benchmark of the AdamS N:M step on one MI355X.

A "step" is one AdamS iteration (Algorithm 1 with the weight scaling of Eq. 12, n = 2) over
every linear weight of a LLaMA2-7B-shaped model: 224 matrices, 6,476,005,376 parameters,
fp32 weights and moments, bf16 gradients and one mask bit per parameter, all resident in HBM.
Masks are refreshed every 10th step (T_1 = 10), so the timed region holds refresh and
non-refresh steps in the paper's 1:9 ratio.  The final hard projection + packing runs once per
training, not per step; it is timed separately and reported under "extra".

Prints ONE JSON line: the metric (Gparams/s over the whole timed region), `roofline` (algorithmic bytes of the
non-refresh step kernel per launch / its average launch duration against the 8 TB/s HBM peak, and against the
library's stream probe), `cpu_baseline` (the CPU oracle timed on a bounded sample) and `extra` (the other entry
points, step flavours, patterns, layouts and weight sets, each with ms, GB/s and fraction of peak).  Inputs are
synthetic Gaussians drawn in device memory; nothing is read from disk.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
BYTES_PER_PARAM = 26.125         # read w, mu, v (fp32) + g (bf16) + 1 mask bit; write w, mu, v
# HBM bytes per parameter of the dominant kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/; None until measured.
MEASURED_TRAFFIC_BYTES_PER_PARAM = 26.20

LR, LAMBDA, TOTAL_STEPS, MASK_PERIOD, SEGMENTS = 2e-5, 4e-7, 7500, 10, 2   # Table 11 (LLaMA), Sec. 4.1, Sec. 6.1


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Model:
    """Every linear weight of the workload with its optimizer state, in device memory."""

    def __init__(self, workload: str, layers, torch, B, synth, dev, interleaved: bool, segment_rows: bool = False):
        self.shapes = synth.weight_set(workload, layers)
        self.segments = SEGMENTS
        if segment_rows:
            # a [rows, cols] matrix with n scaling segments per row is, byte for byte, a [rows*n, cols/n]
            # matrix with one: the interleave of w, mu, v then alternates every segment instead of every row
            self.shapes = [(nm, r * SEGMENTS, c // SEGMENTS) for nm, r, c in self.shapes]
            self.segments = 1
        self.params = synth.set_params(self.shapes)
        self.t = []
        self.list = None
        self.row_splits = 1
        self.flags = 0
        self.rule = 0
        self.nm = (2, 4)
        self.launches = len(self.shapes)
        for i, (_, r, c) in enumerate(self.shapes):
            w = synth.device_gaussian((r, c), 0.02, torch.float32, 1000 + i, dev)
            g = synth.device_gaussian((r, c), 1e-3, torch.bfloat16, 500000 + i, dev)
            if interleaved:
                # w, mu, v of a matrix row-interleaved in one allocation ([rows][3][cols], row stride 3*cols):
                # the three streams stay within tens of KiB of each other in HBM
                w, m, v = B.interleaved_state(w)
            else:
                m, v = torch.zeros_like(w), torch.zeros_like(w)
            self.t.append(dict(w=w, g=g, m=m, v=v,
                               mask=B.alloc_mask(r, c, dev),
                               A=torch.ones((r, self.segments), device=dev),
                               gA=torch.zeros((r, self.segments), device=dev)))

    def tensor_list(self, B, scaled: bool, dev, copies=None, stats=None):
        """Descriptors for the one-call-per-step entry point, marshalled once."""
        self.list = B.TensorList([dict(w=x["w"], grad=x["g"], m=x["m"], v=x["v"], mask=x["mask"],
                                       scale=x["A"] if scaled else None, scale_grad=x["gA"] if scaled else None,
                                       compute_copy=None if copies is None else copies[i],
                                       copy_scale=x["A"] if scaled and copies is not None else None,
                                       initial_mask=None if stats is None else x["mask"],
                                       refresh_stats=None if stats is None else stats[i])
                                  for i, x in enumerate(self.t)], dev)
        self.flags = 0
        # launches of the step kernel per call (the list call steps several small matrices with one launch)
        probe = B.AdamsConfig(scale_segments=self.segments if scaled else 0, flags=self.flags)
        self.launches, _ = B.cast_adams_multi_launches(self.list, probe)

    def step(self, B, t: int, scaled: bool):
        cfg = B.iteration_config(t, TOTAL_STEPS, mask_period=MASK_PERIOD, lr=LR, lambda_=LAMBDA,
                                 scale_segments=self.segments if scaled else 0, flags=self.flags, rule=self.rule,
                                 n_keep=self.nm[0], m_group=self.nm[1])
        if self.list is not None:
            B.cast_adams_step_multi(self.list, cfg)
        else:
            k = self.row_splits
            for x in self.t:
                rows = x["w"].shape[0]
                for i in range(k):      # k > 1: each matrix goes out as k launches over row blocks (experiment)
                    a, b = rows * i // k, rows * (i + 1) // k
                    B.cast_adams_step(x["w"][a:b], x["g"][a:b], x["m"][a:b], x["v"][a:b], x["mask"][a:b], cfg,
                                      scale=x["A"][a:b] if scaled else None, scale_grad=x["gA"][a:b] if scaled else None)
        return cfg.refresh_mask


def time_set(torch, B, model, scaled, steps, warmup, t0=1):
    """ms per step of `steps` consecutive iterations starting at t0 (after `warmup` untimed ones), as the list call
    makes them, with the kinds of step they were."""
    t = t0
    for _ in range(warmup):
        model.step(B, t, scaled)
        t += 1
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    kinds = []
    torch.cuda.synchronize()
    marks[0].record()
    for k in range(steps):
        kinds.append(model.step(B, t, scaled))
        t += 1
        marks[k + 1].record()
    torch.cuda.synchronize()
    per = [marks[k].elapsed_time(marks[k + 1]) for k in range(steps)]
    return marks[0].elapsed_time(marks[-1]) / steps, per, kinds


def set_figures(ms, params, bpp=BYTES_PER_PARAM):
    gbs = bpp * params / (ms * 1e-3) / 1e9
    return {"ms_step": round(ms, 4), "Gparams_s": round(params / (ms * 1e-3) / 1e9, 1), "GBs": round(gbs, 1),
            "frac": round(gbs / HBM_PEAK_GBS, 4)}


def stream_probe(torch, B, model, reps=10):
    """ms per call of cast_hbm_stream_probe over the model's list (it overwrites the state): the same launches and
    the same memory accesses as a non-refresh step with next to no arithmetic."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(2):
        B.cast_hbm_stream_probe(model.list, model.segments)
    e0.record()
    for _ in range(reps):
        B.cast_hbm_stream_probe(model.list, model.segments)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def other_set(torch, B, synth, dev, workload, interleaved, steps, warmup):
    """Another resident set through the same list call: `steps` iterations with the 1-in-10 refresh mix, and the
    stream probe over the same list."""
    shapes = synth.weight_set(workload, None)
    torch.cuda.empty_cache()
    free_bytes, _ = torch.cuda.mem_get_info()
    if free_bytes < 14.5 * synth.set_params(shapes) + (1 << 30):
        return {"skipped": f"{free_bytes >> 30} GiB of device memory free"}
    model = Model(workload, None, torch, B, synth, dev, interleaved)
    model.tensor_list(B, True, dev)
    torch.cuda.synchronize()
    ms, per, kinds = time_set(torch, B, model, True, steps, warmup, t0=10)      # the first warm-up step refreshes the masks
    out = set_figures(ms, model.params)
    plain = [m for m, k in zip(per, kinds) if not k]
    out["ms_step_non_refresh"] = round(sum(plain) / len(plain), 4)
    out["matrices"], out["params"], out["steps"] = len(model.shapes), model.params, steps
    probe_ms = stream_probe(torch, B, model)
    out["stream_probe_GBs"] = round(BYTES_PER_PARAM * model.params / (probe_ms * 1e-3) / 1e9, 1)
    out["frac_of_stream_probe"] = round(probe_ms / out["ms_step_non_refresh"], 4)
    del model
    torch.cuda.empty_cache()
    return out


def cpu_baseline(synth):
    """The oracle as it stands (plain C, fp32-per-operation variant, OpenMP over rows), host cores only: the
    headline figure is non-refresh AdamS 2:4 steps with scaling n = 2 over the 7 matrices of one
    LLaMA2-7B-shaped decoder layer on all threads; one of its 4096 x 4096 matrices on one thread, the
    125M-shaped set and the single 768 x 768 matrix are given beside it.  About 15 s of timed CPU work in all."""
    import numpy as np

    import oracle
    oracle.build()
    threads = min(16, os.cpu_count() or 1)
    rng = np.random.default_rng(0)

    def run(shapes, nthreads, reps, budget_s):
        """Up to `reps` timed steps per matrix, fewer once the time budget for the whole list is used up."""
        cfg = oracle.AdamsCfg(lr=LR, lambda_=LAMBDA, alpha=0.5, bias_corr1=0.9, bias_corr2=0.1, refresh_mask=0,
                              scale_segments=SEGMENTS)
        params, elapsed = 0, 0.0
        total = sum(r * c for (_, r, c) in shapes)
        for (_, r, c) in shapes:
            w = (rng.standard_normal((r, c), np.float32) * np.float32(0.02))
            g = (rng.standard_normal((r, c), np.float32) * np.float32(1e-3))
            m, v = np.zeros_like(w), np.zeros_like(w)
            keep = np.zeros(w.shape, np.uint8)
            A = np.ones((r, SEGMENTS), np.float32)
            cfg.refresh_mask = 1
            oracle.adams_step(w, g, m, v, keep, cfg, A=A, arithmetic="f32", nthreads=nthreads)   # untimed, builds the mask
            cfg.refresh_mask = 0
            share = budget_s * (r * c) / total
            spent = 0.0
            for k in range(reps):
                t0 = time.perf_counter()
                oracle.adams_step(w, g, m, v, keep, cfg, A=A, arithmetic="f32", nthreads=nthreads)
                dt = time.perf_counter() - t0
                spent += dt
                elapsed += dt
                params += r * c
                if spent > share:
                    break
        return params, elapsed

    layer = synth.weight_set("llama2_7b", 1)
    params, elapsed = run(layer, threads, 32, 10.0)
    p1, e1 = run(layer[:1], 1, 4, 2.0)
    p2, e2 = run(synth.weight_set("opt125m", None), threads, 8, 2.0)
    p3, e3 = run([("w", 768, 768)], 1, 200, 1.0)
    return {"value": params / elapsed / 1e9, "unit": "Gparams/s", "cores": threads, "kind": "oracle",
            "sample": f"non-refresh AdamS 2:4 steps (fp32-per-operation oracle in C, OpenMP over rows, scaling n=2), "
                      f"repeated over the 7 matrices of one LLaMA2-7B-shaped layer: {params} param-updates in "
                      f"{elapsed:.2f} s wall on {threads} threads",
            "also": {"one_4096x4096_1_thread_Gparams_s": round(p1 / e1 / 1e9, 4),
                     "set_125m_all_threads_Gparams_s": round(p2 / e2 / 1e9, 4),
                     "one_768x768_1_thread_Gparams_s": round(p3 / e3 / 1e9, 4)}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama2_7b", choices=["opt125m", "llama2_7b", "llama2_13b", "llama3_8b"])
    ap.add_argument("--layers", type=int, default=None, help="use only the first LAYERS decoder blocks (debugging)")
    ap.add_argument("--no-scale", action="store_true", help="time the step without weight scaling")
    ap.add_argument("--layout", default="interleaved", choices=["interleaved", "interleaved-segments", "separate"],
                    help="w, mu, v of each matrix row-interleaved in one buffer (default) or three dense arrays")
    ap.add_argument("--launch", default="list", choices=["list", "per-matrix"],
                    help="one cast_adams_step_multi call per step (default) or one cast_adams_step call per matrix")
    ap.add_argument("--row-splits", type=int, default=1, help="per-matrix launch only: launches per matrix (experiment)")
    ap.add_argument("--nm", default="2:4", choices=["1:2", "2:4", "4:8"],
                    help="sparsity pattern of the timed steps (the metric is quoted on 2:4; the extras stay 2:4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch

    from paper_2509_25996_amd import binding as B
    from paper_2509_25996_amd import synth
    B.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    scaled = not args.no_scale

    t0 = time.time()
    model = Model(args.workload, args.layers, torch, B, synth, dev, args.layout != "separate",
                  args.layout == "interleaved-segments")
    model.row_splits = args.row_splits
    model.nm = tuple(int(x) for x in args.nm.split(":"))
    if model.nm != (2, 4) and not args.no_extra:
        sys.exit("--nm other than 2:4 needs --no-extra")
    if args.launch != "per-matrix":
        model.tensor_list(B, scaled, dev)
    torch.cuda.synchronize()
    log(f"[bench] {args.workload}: {len(model.shapes)} matrices, {model.params} params resident "
        f"({torch.cuda.memory_allocated() / 2**30:.1f} GiB) after {time.time() - t0:.1f} s")

    t = 0
    for _ in range(args.warmup):
        model.step(B, t, scaled)
        t += 1
    torch.cuda.synchronize()

    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    kinds = []
    torch.cuda.synchronize()
    marks[0].record()
    for k in range(args.steps):
        kinds.append(model.step(B, t, scaled))
        t += 1
        marks[k + 1].record()
    torch.cuda.synchronize()
    total_ms = marks[0].elapsed_time(marks[-1])
    step_ms = [marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)]
    ms_per_step = total_ms / args.steps
    value = model.params / (ms_per_step * 1e-3) / 1e9
    plain = [m for m, k in zip(step_ms, kinds) if not k]
    fresh = [m for m, k in zip(step_ms, kinds) if k]
    log(f"[bench] {ms_per_step:.3f} ms/step, {value:.1f} Gparams/s; non-refresh {sum(plain) / max(len(plain), 1):.3f} ms, "
        f"refresh {sum(fresh) / max(len(fresh), 1):.3f} ms")

    n_matrices, n_params, nm = len(model.shapes), model.params, model.nm
    # dominant kernel: the non-refresh step kernel (9 of 10 steps), all its launches of a step taken together
    launches = model.launches
    dom_ms = (sum(plain) / len(plain)) if plain else ms_per_step
    bytes_per_launch = BYTES_PER_PARAM * model.params / launches
    achieved = bytes_per_launch / (dom_ms * 1e-3 / launches) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": None if MEASURED_TRAFFIC_BYTES_PER_PARAM is None
                else MEASURED_TRAFFIC_BYTES_PER_PARAM * model.params / launches,
                "kernel": "adams_step_vec" + ("<M=4, bf16 grad, stored mask, scaled>" if scaled else "<M=4, bf16 grad, stored mask>"),
                "bytes_per_launch": bytes_per_launch, "avg_launch_us": round(dom_ms * 1e3 / launches, 2)}

    extra = {"ms_step_non_refresh": round(dom_ms, 3),
             "ms_step_refresh": round(sum(fresh) / len(fresh), 3) if fresh else None}
    if not args.no_extra:
        # achievable copy bandwidth on this machine (read + write of 2 GiB), for context beside the spec peak
        n = 1 << 30
        a = torch.empty(n // 4, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.cast_hbm_copy_probe(b, a)
        e0.record()
        for _ in range(10):
            B.cast_hbm_copy_probe(b, a)
        e1.record()
        torch.cuda.synchronize()
        extra["copy_probe_GBs"] = round(2 * n * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        del a, b
        def timed_calls(call, reps=3):
            call()
            e0.record()
            for _ in range(reps):
                call()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        def figures(ms, bpp):
            gbs = bpp * model.params / (ms * 1e-3) / 1e9
            return round(ms, 3), round(gbs, 1), round(gbs / HBM_PEAK_GBS, 4)

        # The once-per-run entry points over the whole set, each as ONE list call (matrices of one shape share
        # launches), every matrix writing into buffers of its own as a user's would:
        # the epilogue of training, hard 2:4 projection + fold + pack (6.125 B/param) ...
        free_bytes, _ = torch.cuda.mem_get_info()
        if free_bytes > 2.2 * model.params + (4 << 30):
            outs = [(torch.empty((r, c // 2), device=dev), torch.empty((r, c // 32), dtype=torch.int32, device=dev))
                    for (_, r, c) in model.shapes]
            ml = B.MatrixList([dict(w=x["w"], scale=x["A"] if scaled else None, out=o[0], meta=o[1]) for x, o in zip(model.t, outs)])
            extra["project_compress_ms"], extra["project_compress_GBs"], extra["project_compress_frac"] = \
                figures(timed_calls(lambda: B.cast_nm_project_compress_multi(ml, 2, 4)), 6.125)
            # ... with the stored masks instead of Eq. 6 on the final weights (Algorithm 1 literally: 6.25 B/param)
            ml = B.MatrixList([dict(w=x["w"], scale=x["A"] if scaled else None, out=o[0], meta=o[1], mask=x["mask"])
                               for x, o in zip(model.t, outs)])
            B.cast_nm_select_multi(B.MatrixList([dict(w=x["w"], mask=x["mask"]) for x in model.t]), 2, 4)
            extra["project_compress_stored_mask_ms"], extra["project_compress_stored_mask_GBs"], _ = \
                figures(timed_calls(lambda: B.cast_nm_project_compress_multi(ml, 2, 4)), 6.25)
            del outs, ml
        # ... mask selection alone (Eq. 6: 4.125 B/param) ...
        ml = B.MatrixList([dict(w=x["w"], mask=x["mask"]) for x in model.t])
        extra["nm_select_ms"], extra["nm_select_GBs"], extra["nm_select_frac"] = \
            figures(timed_calls(lambda: B.cast_nm_select_multi(ml, 2, 4)), 4.125)
        # ... Eq. 12 applied into a bf16 copy of every matrix (6 B/param)
        free_bytes, _ = torch.cuda.mem_get_info()
        if scaled and free_bytes > 2 * model.params + (4 << 30):
            copies16 = [torch.empty(x["w"].shape, dtype=torch.bfloat16, device=dev) for x in model.t]
            ml = B.MatrixList([dict(w=x["w"], scale=x["A"], out=o) for x, o in zip(model.t, copies16)])
            extra["weight_scale_bf16_ms"], extra["weight_scale_bf16_GBs"], extra["weight_scale_bf16_frac"] = \
                figures(timed_calls(lambda: B.cast_weight_scale_multi(ml)), 6.0)
            del copies16
        del ml
        # mask-learning statistics of given masks (flips against another mask, ||W.M||_1, ||W||_1): a pass of its own
        # over w and two masks, 4.25 B/param, as one list call (per-workgroup partial sums through a workspace)
        sl = B.StatsList([dict(w=x["w"], mask=x["mask"], other=x["mask"], stats=B.alloc_refresh_stats(dev)) for x in model.t], dev)
        extra["mask_stats_ms"], extra["mask_stats_GBs"], extra["mask_stats_frac"] = \
            figures(timed_calls(lambda: B.cast_mask_stats_multi(sl)), 4.25)
        del sl
        # dL/dA alone (6 B/param), as one list call
        if scaled:
            gl = B.ScaleGradList([dict(w=x["w"], grad=x["g"], scale_grad=x["gA"]) for x in model.t])
            extra["weight_scale_grad_ms"], extra["weight_scale_grad_GBs"], _ = \
                figures(timed_calls(lambda: B.cast_weight_scale_grad_multi(gl)), 6.0)
            del gl
        if model.list is not None:
            # the widened forms of the step, over the same set and through the same list call: a comparison
            # rule (Eq. 10), and the step that also writes the bf16 weights of the next forward pass
            # (28.125 B/param: 2 more bytes written)
            def timed(flags_rule, reps=10, t_=1):
                model.rule = flags_rule
                for _ in range(2):
                    model.step(B, t_, scaled)
                e0.record()
                for _ in range(reps):
                    model.step(B, t_, scaled)      # t_ = 1: non-refresh steps; t_ = 10: refresh steps
                e1.record()
                torch.cuda.synchronize()
                model.rule = 0
                return e0.elapsed_time(e1) / reps
            copies = [torch.empty(x["w"].shape, dtype=torch.bfloat16, device=dev) for x in model.t]
            model.tensor_list(B, scaled, dev, copies=copies)
            ms = timed(0)
            extra["emit_compute_copy_ms_step"] = round(ms, 3)
            extra["emit_compute_copy_GBs"] = round((BYTES_PER_PARAM + 2) * model.params / (ms * 1e-3) / 1e9, 1)
            del copies
            # refresh steps that also gather the mask-learning statistics (one more mask word read per 32 entries,
            # per-workgroup sums through the workspace), against plain refresh steps
            stats = [B.alloc_refresh_stats(dev) for _ in model.t]
            model.tensor_list(B, scaled, dev, stats=stats)
            extra["refresh_with_stats_ms_step"] = round(timed(0, t_=10), 3)
            model.tensor_list(B, scaled, dev)
            extra["refresh_ms_step"] = round(timed(0, t_=10), 3)
            for name, rule in (("adamw_l1", B.RULE_ADAMW_L1), ("adam_l1", B.RULE_ADAM_L1), ("additive", B.RULE_ADDITIVE),
                               ("masked_frozen", B.RULE_MASKED_FROZEN)):
                ms = timed(rule)
                extra[f"rule_{name}_ms_step"] = round(ms, 3)
                extra[f"rule_{name}_GBs"] = round(BYTES_PER_PARAM * model.params / (ms * 1e-3) / 1e9, 1)
            # the storage variant that keeps the first moment in bf16 (22.125 B/param; not the paper's configuration
            # and not the headline): a second state of the same set, rows of w (fp32), mu (bf16), v (fp32) interleaved
            free_bytes, _ = torch.cuda.mem_get_info()
            if args.layout == "interleaved" and free_bytes > 10.5 * model.params:
                kept = [(x["w"], x["m"], x["v"]) for x in model.t]
                for x in model.t:
                    x["w"], x["m"], x["v"] = B.interleaved_state(x["w"], mu_bf16=True)
                model.tensor_list(B, scaled, dev)
                ms = timed(0)
                extra["mu_bf16_ms_step"] = round(ms, 3)
                extra["mu_bf16_Gparams_s"] = round(model.params / (ms * 1e-3) / 1e9, 1)
                extra["mu_bf16_GBs"] = round((BYTES_PER_PARAM - 4) * model.params / (ms * 1e-3) / 1e9, 1)
                free_bytes, _ = torch.cuda.mem_get_info()
                if free_bytes > 2.5 * model.params:      # the same with the bf16 compute copy written along (24.125 B/param)
                    copies = [torch.empty(x["w"].shape, dtype=torch.bfloat16, device=dev) for x in model.t]
                    model.tensor_list(B, scaled, dev, copies=copies)
                    ms = timed(0)
                    extra["mu_bf16_emit_ms_step"] = round(ms, 3)
                    extra["mu_bf16_emit_GBs"] = round((BYTES_PER_PARAM - 2) * model.params / (ms * 1e-3) / 1e9, 1)
                    del copies
                    model.tensor_list(B, scaled, dev)
                # the same launches and streams with next to no arithmetic (overwrites this second state: its last use)
                extra["mu_bf16_frac_of_stream_probe"] = round(stream_probe(torch, B, model) / extra["mu_bf16_ms_step"], 4)
                # both moments in bf16, the second one rounded stochastically (18.125 B/param; 20.125 with the copy)
                for x in model.t:
                    x["m"] = x["v"] = None
                    x["w"], x["m"], x["v"] = B.interleaved_state(x["w"], mu_bf16=True, v_bf16=True)
                model.tensor_list(B, scaled, dev)
                ms = timed(0)
                extra["both_bf16_ms_step"] = round(ms, 3)
                extra["both_bf16_Gparams_s"] = round(model.params / (ms * 1e-3) / 1e9, 1)
                extra["both_bf16_GBs"] = round((BYTES_PER_PARAM - 8) * model.params / (ms * 1e-3) / 1e9, 1)
                free_bytes, _ = torch.cuda.mem_get_info()
                if free_bytes > 2.5 * model.params:
                    copies = [torch.empty(x["w"].shape, dtype=torch.bfloat16, device=dev) for x in model.t]
                    model.tensor_list(B, scaled, dev, copies=copies)
                    ms = timed(0)
                    extra["both_bf16_emit_ms_step"] = round(ms, 3)
                    extra["both_bf16_emit_GBs"] = round((BYTES_PER_PARAM - 6) * model.params / (ms * 1e-3) / 1e9, 1)
                    del copies
                    model.tensor_list(B, scaled, dev)
                extra["both_bf16_frac_of_stream_probe"] = round(stream_probe(torch, B, model) / extra["both_bf16_ms_step"], 4)
                for x, (w, m, v) in zip(model.t, kept):
                    x["w"], x["m"], x["v"] = w, m, v
                del kept

    if not args.no_extra and model.list is not None and scaled:
        # the other patterns over the same state (10 steps from a refresh step on, so that the masks fit the pattern),
        # and 2:4 with fp32 gradients (28.125 B/param: the single-matrix configuration of the workload family)
        model.tensor_list(B, scaled, dev)
        for key, pattern in (("pattern_4of8", (4, 8)), ("pattern_1of2", (1, 2))):
            model.nm = pattern
            ms, _, _ = time_set(torch, B, model, scaled, 10, 1, t0=10)
            extra[key] = set_figures(ms, model.params)
        model.nm = (2, 4)
        free_bytes, _ = torch.cuda.mem_get_info()
        if free_bytes > 4 * model.params + (4 << 30):
            g16 = [x["g"] for x in model.t]
            for x in model.t:
                x["g"] = x["g"].float()
            model.tensor_list(B, scaled, dev)
            ms, per, kinds = time_set(torch, B, model, scaled, 10, 1, t0=10)
            extra["fp32_grads"] = set_figures(ms, model.params, BYTES_PER_PARAM + 2)
            plain32 = [m for m, k in zip(per, kinds) if not k]
            extra["fp32_grads"]["frac_of_stream_probe"] = round(stream_probe(torch, B, model) / (sum(plain32) / len(plain32)), 4)
            for x in model.t:      # the probe leaves meaningless values: moments a step can start from again
                x["m"].zero_()
                x["v"].zero_()
            for x, g in zip(model.t, g16):
                x["g"] = g
            del g16
            model.tensor_list(B, scaled, dev)
        # The step's timing depends on the data in one way: a wavefront whose 256 entries hold a zero, a denormal or a
        # huge mu~ or v takes the IEEE division and square root instead of the short forms.  Worst case: one entry
        # of every 256 with w = g = mu = v = 0 (it stays that way), so that every wavefront takes the long forms.
        model.tensor_list(B, scaled, dev)
        for x in model.t:
            for k in ("w", "g", "m", "v"):
                x[k][:, ::256] = 0
        ms, _, _ = time_set(torch, B, model, scaled, 9, 2, t0=1)
        extra["long_forms"] = set_figures(ms, model.params)
        extra["long_forms"]["what"] = "non-refresh steps with one all-zero entry per 256: every wavefront takes the IEEE forms"
        # what the memory system gives the step's access pattern (overwrites the state: last use of this model)
        probe_ms = stream_probe(torch, B, model)
        extra["stream_probe"] = {"ms_call": round(probe_ms, 4), "GBs": round(BYTES_PER_PARAM * model.params / (probe_ms * 1e-3) / 1e9, 1),
                                 "what": "the list call's launches, loads, prefetches and stores with three multiply-adds per entry"}
        extra["stream_probe"]["frac_of_peak"] = round(extra["stream_probe"]["GBs"] / HBM_PEAK_GBS, 4)
        roofline["frac_of_stream_probe"] = round(probe_ms / dom_ms, 4)
    if not args.no_extra and args.workload == "llama2_7b" and args.layers is None and scaled and args.launch == "list":
        del model, x
        model = None
        torch.cuda.empty_cache()
        # the same step on the other resident sets of the workload family, and on three dense state arrays
        for key, workload, interleaved, steps, warm in (("separate_layout", "llama2_7b", False, 10, 3),
                                                        ("llama2_13b", "llama2_13b", True, 10, 3),
                                                        ("opt125m", "opt125m", True, 200, 20)):
            try:
                extra[key] = other_set(torch, B, synth, dev, workload, interleaved, steps, warm)
            except Exception as e:      # an extra must not take the headline down with it
                extra[key] = {"failed": repr(e)[:200]}
                torch.cuda.empty_cache()
            log(f"[bench] {key}: {extra[key]}")

    out = {"metric": "AdamS N:M step Gparams/s at LLaMA2-7B shape; % of MI355X peak HBM BW",
           "value": round(value, 2), "unit": "Gparams/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{args.workload} linear weight set ({n_matrices} matrices, {n_params} params), "
                                  f"{args.nm}, fp32 w/mu/v ({args.layout}) + bf16 grads + mask bits resident, "
                                  f"{'weight scaling n=2, ' if scaled else ''}mask refresh every 10th step, "
                                  f"{ {'list': 'one list call', 'per-matrix': 'one call per matrix'}[args.launch]} per step",
                      "n_keep": nm[0], "m_group": nm[1], "scale_segments": SEGMENTS if scaled else 0,
                      "pct_of_peak_hbm": round(100 * BYTES_PER_PARAM * value / HBM_PEAK_GBS, 2)},
           "roofline": roofline, "extra": extra}
    if not args.no_cpu_baseline:
        model = None
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(synth)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
