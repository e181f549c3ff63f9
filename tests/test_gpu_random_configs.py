"""Random valid configurations through the list call against the oracle: pattern, shape (odd ones, vector ones,
benchmark widths), number of scaling segments, layout, gradient dtype, update rule, bf16 first moment, compute copy,
refresh statistics, runs of equal shapes (shared launches), refresh period.  State, masks and compute
copies bit for bit.  The draws are seeded: a failure names its case."""
import random

import numpy as np
import pytest
import torch

import oracle
from paper_2509_25996_amd import binding as B
from paper_2509_25996_amd import synth

from gpu_util import DEV, GpuState, OracleState, assert_same_bits, dev, host, oracle_cfg, words

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_configurations_match_the_oracle(seed):
    count = 120
    rnd = random.Random(seed)
    done = 0
    for case in range(count):
        m = rnd.choice([2, 4, 4, 4, 8, 8])
        n = rnd.randint(1, m - 1) if rnd.random() < 0.3 else m // 2
        nseg = rnd.choice([0, 0, 1, 2, 2, 2, 3, 4])
        unit = m * max(nseg, 1)
        kind = rnd.random()
        if kind < 0.35:
            cols = unit * rnd.randint(1, 40)
        elif kind < 0.8:
            cols = 32 * max(nseg, 1) * rnd.randint(1, 90)
        else:
            cols = rnd.choice([4096, 5120, 11008, 13824, 6144, 4608, 8192, 14336, 2560])
        if cols % unit or (nseg and (cols // nseg) % m):
            continue
        rows = rnd.randint(1, 24 if cols > 4000 else 70)
        mu16 = rnd.random() < 0.25
        interleaved = rnd.random() < 0.5 and cols % 8 == 0
        rule = 0 if mu16 else rnd.choice([0, 0, 0, 1, 2, 3, 4])
        if mu16 and rnd.random() < 0.3:
            rule = 3
        bf16 = rnd.random() < 0.6
        emit = rnd.random() < 0.3
        stats = rnd.random() < 0.3
        rnd.random()      # (a draw that once chose a launch form; kept so that the seeds give the same cases)
        steps = rnd.randint(2, 4)
        period = rnd.choice([1, 2, 3])
        copies = rnd.randint(1, 3)          # equal shapes in the list: shared launches
        v16 = mu16 and rnd.random() < 0.5   # both moments in bf16, the second one rounded stochastically
        note = (f"case {case}: {n}:{m} {rows}x{cols} nseg={nseg} mu16={mu16} inter={interleaved} v16={v16} rule={rule} bf16={bf16} emit={emit} stats={stats} steps={steps} x{copies}")
        items, refs = [], []
        for k in range(copies):
            w0 = synth.tie_outlier_weights(seed, case * 8 + k, rows, cols) if cols % 8 == 0 else synth.weights(seed, case * 8 + k, rows, cols)
            st = GpuState(w0, nseg, interleaved, mu_bf16=mu16, v_bf16=v16)
            A = (1 + 0.2 * np.random.default_rng(case * 8 + k).standard_normal((rows, nseg))).astype(np.float32) if nseg else None
            item = dict(w=st.w, m=st.m, v=st.v, mask=st.mask, grad=None, scale=None if A is None else dev(A), scale_grad=st.scale_grad)
            if emit:
                item["compute_copy"] = torch.full((rows, cols), 7.0, dtype=torch.bfloat16, device=DEV)
                if nseg and k % 2 == 0:
                    item["copy_scale"] = item["scale"]
            if stats:
                item["refresh_stats"] = B.alloc_refresh_stats(DEV)
            items.append(item)
            refs.append((OracleState(w0, "f32"), A))
        for t in range(steps):
            cfg = B.iteration_config(t, steps + 1, mask_period=period, lr=1e-3, lambda_=1e-3, n_keep=n, m_group=m, scale_segments=nseg, rule=rule)
            grads = []
            for k, item in enumerate(items):
                gr = synth.grads_f32(seed, case * 8 + k, t, rows, cols)
                if bf16:
                    gr = synth.widen_bf16(torch.from_numpy(gr).to(torch.bfloat16))
                item["grad"] = dev(gr, torch.bfloat16 if bf16 else None)
                grads.append(gr)
            B.cast_adams_step_multi(B.TensorList(items, DEV), cfg)
            for k, (o, A) in enumerate(refs):
                ocfg = oracle_cfg(cfg)
                o.step(grads[k], ocfg, A=A)
        torch.cuda.synchronize()
        for k, (item, (o, A)) in enumerate(zip(items, refs)):
            assert (words(item["mask"]) == oracle.pack_mask_bits(o.keep)).all(), note
            assert_same_bits(host(item["w"]), o.w, note + " w")
            assert_same_bits(host(item["m"].float()) if mu16 else host(item["m"]), o.m, note + " mu")
            assert_same_bits(host(item["v"].float()) if v16 else host(item["v"]), o.v, note + " v")
            if emit:
                want = oracle.bf16_rne(o.w if "copy_scale" not in item else oracle.weight_scale(o.w, A))
                assert (host(item["compute_copy"].view(torch.int16)).view(np.uint16) == want).all(), note + " copy"
        done += 1
    assert done > count // 2


@pytest.mark.parametrize("seed", [21, 22])
def test_random_selection_scaling_and_packing_match_the_oracle(seed):
    """The other entry points on random shapes, patterns and layouts: mask selection, A (.) W (fp32, bf16, in place),
    dL/dA alone, mask statistics, hard projection + fold + pack with the mask recomputed or given."""
    rnd = random.Random(seed)
    for case in range(150):
        m = rnd.choice([2, 4, 4, 8, 8])
        n = rnd.randint(1, m - 1) if rnd.random() < 0.35 else m // 2
        nseg = rnd.choice([1, 2, 2, 3, 4])
        kind = rnd.random()
        if kind < 0.4:
            cols = m * nseg * rnd.randint(1, 40)
        elif kind < 0.85:
            cols = 64 * nseg * rnd.randint(1, 40)
        else:
            cols = rnd.choice([4096, 5120, 11008, 13824, 8192])
        if cols % (m * nseg) or (cols // nseg) % m:
            continue
        rows = rnd.randint(1, 16 if cols > 4000 else 60)
        interleaved = rnd.random() < 0.5
        note = f"case {case}: {n}:{m} {rows}x{cols} nseg={nseg} interleaved={interleaved}"
        w = synth.tie_outlier_weights(seed, case, rows, cols) if cols % 8 == 0 else synth.weights(seed, case, rows, cols)
        A = (1 + 0.3 * np.random.default_rng(case).standard_normal((rows, nseg))).astype(np.float32)
        wd = B.interleaved_state(dev(w))[0] if interleaved else dev(w)
        # selection
        mask = B.alloc_mask(rows, cols, DEV)
        B.cast_nm_select(wd, n, m, mask)
        keep = oracle.nm_select(w, n, m)
        assert (words(mask) == oracle.pack_mask_bits(keep)).all(), note + " select"
        # forward scale, fp32 and bf16
        out32 = torch.empty((rows, cols), device=DEV)
        out16 = torch.empty((rows, cols), dtype=torch.bfloat16, device=DEV)
        B.cast_weight_scale(wd, dev(A), out32)
        B.cast_weight_scale(wd, dev(A), out16)
        ref = oracle.weight_scale(w, A)
        assert_same_bits(host(out32), ref, note + " scale")
        assert (host(out16.view(torch.int16)).view(np.uint16) == oracle.bf16_rne(ref)).all(), note + " scale bf16"
        # dL/dA alone
        g = synth.grads_bf16(seed, case, 0, rows, cols)
        gA = torch.zeros((rows, nseg), device=DEV)
        B.cast_weight_scale_grad(wd, g.to(DEV), nseg, gA)
        ref_gA = oracle.weight_scale_grad(w, synth.widen_bf16(g), nseg)
        terms = np.abs(synth.widen_bf16(g).astype(np.float64) * w).reshape(rows, nseg, -1).sum(-1)
        assert (np.abs(host(gA) - ref_gA) <= 2e-5 * terms + 1e-12).all(), note + " dL/dA"
        # statistics against another mask
        other = B.alloc_mask(rows, cols, DEV)
        B.cast_nm_select(dev(synth.weights(seed, case + 1000, rows, cols)), n, m, other)
        flips = torch.zeros(1, dtype=torch.int64, device=DEV)
        l1 = torch.zeros(2, dtype=torch.float64, device=DEV)
        B.cast_mask_stats(wd, mask, other, flips, l1)
        f_ref, kept, total = oracle.mask_stats(w, keep, oracle.nm_select(synth.weights(seed, case + 1000, rows, cols), n, m))
        assert int(flips.item()) == f_ref, note + " flips"
        assert np.allclose(host(l1), [kept, total], rtol=1e-10), note + " norms"
        # hard projection + fold + pack: mask recomputed, and the other mask given
        for given, keep_used in ((None, None), (other, oracle.unpack_mask_bits(words(other), cols))):
            for vdtype, code in ((torch.float32, B.CAST_F32), (torch.bfloat16, B.CAST_BF16)):
                _, vbytes, mbytes = B.cast_sizes(rows, cols, n, m, code)
                values = torch.full((rows, cols // m * n), 7.0, dtype=vdtype, device=DEV)
                meta = torch.full((rows, mbytes // 4 // rows), -1, dtype=torch.int32, device=DEV)
                B.cast_nm_project_compress(wd, n, m, values, meta, scale=dev(A), mask_bits=given)
                ref_v, ref_m = oracle.project_compress(w, n, m, A=A, keep=keep_used)
                assert (words(meta) == ref_m).all(), note + " meta"
                if vdtype == torch.float32:
                    assert_same_bits(host(values), ref_v, note + " values")
                else:
                    assert (host(values.view(torch.int16)).view(np.uint16) == oracle.bf16_rne(ref_v)).all(), note + " bf16 values"
    torch.cuda.synchronize()
