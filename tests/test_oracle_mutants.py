"""Are the oracle's pins sharp?  Each case plants ONE plausible mistake in a copy of oracle/cast_oracle.c
(a wrong sign, a dropped term, a wrong index, swapped operands, a wrong rounding), builds it, and runs the
pin tests against that build: at least one pin must fail.  The untouched source, built the same way, must
pass.  Nothing here touches the GPU library: the mistakes are planted in the oracle, on the CPU."""
import os
import subprocess
import sys

import pytest

import oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "cast_oracle.c")

STEP, SELECT, SCALE_PACK, RULES, MU16, V16 = ("tests/test_oracle_step.py", "tests/test_oracle_select.py",
                                              "tests/test_oracle_scale_pack.py", "tests/test_oracle_rules.py",
                                              "tests/test_oracle_mu_bf16.py", "tests/test_oracle_v_bf16.py")

# (name, pin files expected to notice, [(text in the source, what it becomes, occurrences)])
MUTANTS = [
    ("ties go to the higher index", [SELECT],
     [("(kk == kj && k < j)", "(kk == kj && k > j)", 1)]),
    ("magnitude keeps the sign bit", [SELECT],
     [("return bits & 0x7fffffffu;", "return bits;", 1)]),
    ("the N smallest are kept", [SELECT],
     [("if (kk > kj || (kk == kj", "if (kk < kj || (kk == kj", 1)]),
    ("mask bits stored from the top of the word", [SELECT],
     [("words[r * wpr + c / 32] |= (uint32_t)1 << (c % 32);", "words[r * wpr + c / 32] |= (uint32_t)1 << (31 - c % 32);", 1)]),
    ("decay pushes away from zero (double)", [STEP],
     [("mu_tilde = (1.0 - p->alpha) * mu_t + p->alpha * p->lambda * sign_f64(theta_prev);",
       "mu_tilde = (1.0 - p->alpha) * mu_t - p->alpha * p->lambda * sign_f64(theta_prev);", 1)]),
    ("momentum of masked entries not attenuated (double)", [STEP],
     [("mu_tilde = (1.0 - p->alpha) * mu_t + p->alpha * p->lambda * sign_f64(theta_prev);",
       "mu_tilde = mu_t + p->alpha * p->lambda * sign_f64(theta_prev);", 1)]),
    ("kept entries decayed too (double)", [STEP],
     [("    else if (m_bit == 0)\n        mu_tilde = (1.0 - p->alpha)", "    else if (1)\n        mu_tilde = (1.0 - p->alpha)", 1)]),
    ("second moment from the gradient (double)", [STEP],
     [("double second = p->v_from_grad ? g * g : mu_tilde * mu_tilde;", "double second = g * g;", 1)]),
    ("the decayed momentum is what gets stored (double)", [STEP],
     [("*mu = mu_t; /* the stored first moment is the undecayed one */", "*mu = mu_tilde;", 1)]),
    ("bias corrections swapped (double)", [STEP],
     [("double mu_hat = mu_tilde / p->bias_corr1;\n    double v_hat = v_t / p->bias_corr2;",
       "double mu_hat = mu_tilde / p->bias_corr2;\n    double v_hat = v_t / p->bias_corr1;", 1)]),
    ("update not bias-corrected in the decay term (double)", [STEP],
     [("double mu_hat = mu_tilde / p->bias_corr1;", "double mu_hat = mu_t / p->bias_corr1 + (mu_tilde - mu_t);", 1)]),
    ("epsilon inside the square root (double)", [STEP],
     [("    *theta = theta_prev - p->lr * (mu_hat / (sqrt(v_hat) + p->eps));\n    *mu = mu_t; /* the stored",
       "    *theta = theta_prev - p->lr * (mu_hat / sqrt(v_hat + p->eps));\n    *mu = mu_t; /* the stored", 1)]),
    ("Sign(0) = 1 (double)", [STEP],
     [("static double sign_f64(double x) { return (double)(x > 0.0) - (double)(x < 0.0); }",
       "static double sign_f64(double x) { return (double)(x >= 0.0) - (double)(x < 0.0); }", 1)]),
    ("decay pushes away from zero (fp32)", [STEP],
     [("mu_tilde = d0 + d1;", "mu_tilde = d0 - d1;", 1)]),
    ("second moment from the gradient (fp32)", [STEP],
     [("float second = p->v_from_grad ? g * g : mu_tilde * mu_tilde;", "float second = g * g;", 1)]),
    ("the decayed momentum is what gets stored (fp32)", [STEP],
     [("    float mu_hat = mu_tilde / p->bias_corr1;\n    float v_hat = v_t / p->bias_corr2;\n    float denom = sqrtf(v_hat) + p->eps;\n"
       "    float q = mu_hat / denom;\n    float step = p->lr * q;\n    *theta = theta_prev - step;\n    *mu = mu_t;",
       "    float mu_hat = mu_tilde / p->bias_corr1;\n    float v_hat = v_t / p->bias_corr2;\n    float denom = sqrtf(v_hat) + p->eps;\n"
       "    float q = mu_hat / denom;\n    float step = p->lr * q;\n    *theta = theta_prev - step;\n    *mu = mu_tilde;", 1)]),
    ("update from the undecayed momentum (fp32)", [STEP],
     [("float mu_hat = mu_tilde / p->bias_corr1;", "float mu_hat = mu_t / p->bias_corr1;", 1)]),
    ("Sign(0) = 1 (fp32)", [STEP],
     [("float sgn = (float)(theta_prev > 0.0f) - (float)(theta_prev < 0.0f);",
       "float sgn = (float)(theta_prev >= 0.0f) - (float)(theta_prev < 0.0f);", 1)]),
    ("mask refreshed from the gradient instead of the weights", [STEP],
     [("if (cfg->refresh_mask) select_group(w + base, M, N, keep + base);",
       "if (cfg->refresh_mask) select_group(grad + base, M, N, keep + base);", 2)]),
    ("chain rule of the scale forgotten (fp32)", [SCALE_PACK],
     [("g = A[r * n + s] * grad[idx];", "g = grad[idx];", 1)]),
    ("chain rule of the scale forgotten (double)", [SCALE_PACK],
     [("g = (double)A[r * n + s] * (double)grad[idx];", "g = (double)grad[idx];", 1)]),
    ("dL/dA from the already scaled weight", [SCALE_PACK],
     [("if (gA) gA[r * n + s] += (double)grad[idx] * (double)w[idx];",
       "if (gA) gA[r * n + s] += (double)grad[idx] * (double)w[idx] * (double)A[r * n + s];", 2)]),
    ("segments interleaved instead of contiguous in the step", [SCALE_PACK],
     [("int64_t s = c / (cols / n);", "int64_t s = c % n;", 2)]),
    ("segments interleaved instead of contiguous in the forward scale", [SCALE_PACK],
     [("out[r * cols + c] = A[r * n + c / (cols / n)] * w[r * cols + c];", "out[r * cols + c] = A[r * n + c % n] * w[r * cols + c];", 1)]),
    ("dL/dA summed over the whole row", [SCALE_PACK],
     [("for (int64_t c = s * (cols / n); c < (s + 1) * (cols / n); ++c)", "for (int64_t c = 0; c < cols; ++c)", 1)]),
    ("metadata positions in descending order", [SCALE_PACK],
     [("field |= (uint32_t)j << (q * b);", "field |= (uint32_t)j << ((n_keep - 1 - q) * b);", 1)]),
    ("packed values in descending column order", [SCALE_PACK],
     [("values[r * groups * n_keep + i * n_keep + q] = val;", "values[r * groups * n_keep + i * n_keep + (n_keep - 1 - q)] = val;", 1)]),
    ("fold of the scale forgotten when packing", [SCALE_PACK],
     [("if (A) val = A[r * n + (i * m_group + j) / (cols / n)] * val;", "if (0) val = A[r * n + (i * m_group + j) / (cols / n)] * val;", 1)]),
    ("bf16 by truncation", [SCALE_PACK, MU16],
     [("bits += 0x7fffu + lsb;", "bits += 0u;", 1)]),
    ("bf16 ties away from zero", [SCALE_PACK, MU16],
     [("bits += 0x7fffu + lsb;", "bits += 0x8000u;", 1)]),
    ("kept and pruned mass swapped in the statistics", [SCALE_PACK],
     [("if (keep[i]) a += mag;", "if (!keep[i]) a += mag;", 1)]),
    ("Eq. 9 decay pushes away from zero", [RULES],
     [("if (m_bit == 0) update += p->alpha * p->lambda * sign_f64(theta_prev);",
       "if (m_bit == 0) update -= p->alpha * p->lambda * sign_f64(theta_prev);", 1)]),
    ("Eq. 10 second moment from the plain gradient", [RULES],
     [("double v_t = p->beta2 * v_prev + (1.0 - p->beta2) * g_tilde * g_tilde;", "double v_t = p->beta2 * v_prev + (1.0 - p->beta2) * g * g;", 1)]),
    ("additive decay attenuates the momentum like AdamS", [RULES],
     [("mu_tilde = mu_t + p->alpha * p->lambda * sign_f64(theta_prev);", "mu_tilde = (1.0 - p->alpha) * mu_t + p->alpha * p->lambda * sign_f64(theta_prev);", 1)]),
    ("fine-tuning freezes the kept entries instead of the masked", [RULES],
     [("if (p->rule == RULE_MASKED_FROZEN && m_bit == 0) { *theta = theta_prev; *mu = mu_prev; *v = v_prev; return; }\n    double mu_t",
       "if (p->rule == RULE_MASKED_FROZEN && m_bit == 1) { *theta = theta_prev; *mu = mu_prev; *v = v_prev; return; }\n    double mu_t", 1)]),
    ("decay acts on the old momentum (fp32)", [STEP],
     [("float d0 = p->one_minus_alpha * mu_t;", "float d0 = p->one_minus_alpha * mu_prev;", 1)]),
    ("gradient enters the momentum unweighted (double)", [STEP, RULES],
     [("double mu_t = p->beta1 * mu_prev + (1.0 - p->beta1) * g;", "double mu_t = p->beta1 * mu_prev + g;", 2)]),
    ("second moment weighted with beta1 (double)", [STEP],
     [("double v_t = p->beta2 * v_prev + (1.0 - p->beta2) * second;", "double v_t = p->beta2 * v_prev + (1.0 - p->beta1) * second;", 1)]),
    ("gradient ascent (fp32)", [STEP],
     [("*theta = theta_prev - step;", "*theta = theta_prev + step;", 3)]),
    ("second moment not bias-corrected (fp32)", [STEP],
     [("float v_hat = v_t / p->bias_corr2;\n    float denom = sqrtf(v_hat) + p->eps;\n    float q = mu_hat / denom;",
       "float v_hat = v_t;\n    float denom = sqrtf(v_hat) + p->eps;\n    float q = mu_hat / denom;", 2)]),
    ("group fields placed by index width instead of field width", [SCALE_PACK],
     [("meta[r * mwpr + i / gpw] |= field << ((i % gpw) * f);", "meta[r * mwpr + i / gpw] |= field << ((i % gpw) * b * n_keep);", 1)]),
    ("changed bits counted where the masks agree", [SCALE_PACK],
     [("if (keep_other && keep[i] != keep_other[i]) ++f;", "if (keep_other && keep[i] == keep_other[i]) ++f;", 1)]),
    ("a given mask is ignored when packing", [SCALE_PACK],
     [("if (keep_in) memcpy(keep, keep_in + r * cols + i * m_group, (size_t)m_group);\n            else select_group",
       "if (0) memcpy(keep, keep_in + r * cols + i * m_group, (size_t)m_group);\n            else select_group", 1)]),
    ("bf16 moment flag ignored", [MU16],
     [("mu[idx] = cfg->mu_bf16 ? through_bf16(m1) : m1;", "mu[idx] = m1;", 1)]),
    ("bf16 moment rounded before it is used (fp32)", [MU16],
     [("    float mu_t = t0 + t1;\n    float mu_tilde;", "    float mu_t = through_bf16(t0 + t1);\n    float mu_tilde;", 1)]),
    ("stochastic rounding always towards zero", [V16],
     [("return (uint16_t)((bits + (r16 & 0xffffu)) >> 16);", "return (uint16_t)(bits >> 16);", 1)]),
    ("stochastic rounding with 15 random bits", [V16],
     [("return (uint16_t)((bits + (r16 & 0xffffu)) >> 16);", "return (uint16_t)((bits + (r16 & 0x7fffu)) >> 16);", 1)]),
    ("second moment rounded to nearest instead of stochastically (fp32)", [V16],
     [("v[idx] = cfg->v_bf16 ? through_bf16_sr(v1, cfg->sr_seed, idx) : v1;", "v[idx] = cfg->v_bf16 ? through_bf16(v1) : v1;", 1)]),
    ("rounding bits from the column alone", [V16],
     [("v[idx] = cfg->v_bf16 ? through_bf16_sr(v1, cfg->sr_seed, idx) : v1;", "v[idx] = cfg->v_bf16 ? through_bf16_sr(v1, cfg->sr_seed, c) : v1;", 1)]),
    ("rounding bits ignore the seed", [V16],
     [("uint32_t key = mix32(seed + 0x9e3779b9u);", "uint32_t key = mix32(0x9e3779b9u);", 1)]),
    ("seed used unmixed (neighbours share their bits a step apart)", [V16],
     [("uint32_t key = mix32(seed + 0x9e3779b9u);", "uint32_t key = seed;", 1)]),
    ("upper half of the entry index ignored", [V16],
     [("x += (uint32_t)(index >> 32) * 0x9e3779b9u;", "", 1)]),
    ("rounded second moment used inside the iteration (fp32)", [V16],
     [("    float v_t = s0 + s1;\n    float mu_hat = mu_tilde / p->bias_corr1;", "    float v_t = through_bf16(s0 + s1);\n    float mu_hat = mu_tilde / p->bias_corr1;", 1)]),
]


def _run_pins(lib_path: str, files) -> subprocess.CompletedProcess:
    env = dict(os.environ, CAST_ORACLE_LIB=lib_path, OMP_NUM_THREADS="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)


def _build_and_run(workdir: str, index: int):
    """Returns (problem with the edit or None, CompletedProcess or None) for mutant `index`."""
    name, files, edits = MUTANTS[index]
    text = open(SRC).read()
    for old, new, count in edits:
        if text.count(old) != count:
            return f"{name}: the source no longer holds {old!r} {count} time(s)", None
        text = text.replace(old, new)
    src = os.path.join(workdir, f"mutant{index}.c")
    with open(src, "w") as f:
        f.write(text)
    lib = os.path.join(workdir, f"libmutant{index}.so")
    O.compile_source(src, lib)
    return None, _run_pins(lib, files)


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    """All mutants built and judged once, a few at a time side by side (each run is a pytest of its own)."""
    from concurrent.futures import ThreadPoolExecutor
    workdir = str(tmp_path_factory.mktemp("mutants"))
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as pool:
        return list(pool.map(lambda i: _build_and_run(workdir, i), range(len(MUTANTS))))


def test_untouched_source_passes_its_pins_when_built_this_way(tmp_path):
    lib = str(tmp_path / "liboracle_plain.so")
    O.compile_source(SRC, lib)
    done = _run_pins(lib, [STEP, SELECT, SCALE_PACK, RULES, MU16])
    assert done.returncode == 0, done.stdout[-3000:]


@pytest.mark.parametrize("index", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(verdicts, index):
    problem, done = verdicts[index]
    assert problem is None, problem
    assert done.returncode == 1, f"no pin noticed: {MUTANTS[index][0]}\n{done.stdout[-2000:]}"      # 1 = tests ran and some failed
    assert " failed" in done.stdout
