"""The pins must notice a plausible mistake anywhere in the oracle: each mutant below plants one
(dropped term, wrong sign, swapped operand, wrong index, wrong rounding) in a copy of
gs_oracle.c, and the pin suite is run against that build in a subprocess -- it has to fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "gs_oracle.c")

MUTANTS = [
    ("no_weight_decay", "s.decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);", "s.decay = 1.0f;"),
    ("update_sign", "float pn = t5 - t6;", "float pn = t5 + t6;"),
    ("betas_swapped", "float t1 = s.beta1 * m[i];", "float t1 = s.beta2 * m[i];"),
    ("eps_inside_sqrt", "float d = sqrtf(vn) / s.rsbc2;\n        d = d + s.eps;", "float d = sqrtf(vn + s.eps) / s.rsbc2;"),
    ("no_bias_correction2", "s.rsbc2 = (float)sqrt(bc2);", "s.rsbc2 = 1.0f;"),
    ("no_bias_correction1", "s.step_size = (float)((double)hp->lr / bc1);", "s.step_size = hp->lr;"),
    ("mean_not_sum", "    return a;\n}\n\n/* a1 on its own", "    return a / (float)k;\n}\n\n/* a1 on its own"),
    ("bf16_truncates", "u += 0x7fffu + keep_lsb;", "u += 0u * keep_lsb;"),
    ("bf16_ties_away", "u += 0x7fffu + keep_lsb;", "u += 0x8000u + 0u * keep_lsb;"),
    ("v_ignores_clip", "float gg = g * g;", "float gg = a * a;"),
    ("v_uses_omb1", "float t4 = s.omb2 * gg;", "float t4 = s.omb1 * gg;"),
    ("drops_first_buffer", "for (int j = 0; j < k; ++j)\n        a += gs_oracle_bf16_to_f32(grads[j][i]);",
     "for (int j = 1; j < k; ++j)\n        a += gs_oracle_bf16_to_f32(grads[j][i]);\n    if (k == 1) a = gs_oracle_bf16_to_f32(grads[0][i]);"),
    ("norm_sums_abs", "S += (double)a * (double)a;", "S += fabs((double)a);"),
    ("clip_not_clamped", "return c < 1.0f ? c : 1.0f;", "return c;"),
    ("m_forgets_one_minus_beta", "float t2 = s.omb1 * g;", "float t2 = g;"),
    ("quotient_transposed", "float u = mn / d;", "float u = d / mn;"),
    ("range_off_by_one", "for (int64_t i = begin; i < end; ++i) {\n        float a = accumulate_f32(grads, k, i);\n        float g = c * a;",
     "for (int64_t i = begin; i + 1 < end; ++i) {\n        float a = accumulate_f32(grads, k, i);\n        float g = c * a;"),
    ("w_from_old_p", "w[i] = gs_oracle_f32_to_bf16(pn);", "w[i] = gs_oracle_f32_to_bf16(t5);"),
    ("truth_vhat_uses_bc1", "double vhat = vn / bc2;", "double vhat = vn / bc1;"),
    ("truth_no_clip", "if (c > 1.0) c = 1.0;", "c = 1.0;"),
    ("add_forgets_buffer", "float base = first ? 0.0f : acc[i];", "float base = 0.0f;"),
    ("add_first_keeps_old", "float base = first ? 0.0f : acc[i];", "float base = acc[i];"),
    ("add_norm_before_update", "double ad = (double)a;", "double ad = (double)base;"),
    ("acc_norm_sums_plain_values", "S += x * x;", "S += x;"),
    ("acc_norm_range_start_ignored", "for (int64_t i = begin; i < end; ++i) {\n        double x = (double)acc[i];",
     "for (int64_t i = 0; i < end; ++i) {\n        double x = (double)acc[i];"),
    ("bf16_decode_shift", "uint32_t u = (uint32_t)h << 16;", "uint32_t u = (uint32_t)h << 15;"),
]


def test_every_mutation_site_exists_once():
    src = open(SRC).read()
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, f"{name}: mutation site not found exactly once"


def _run_mutant(work, name, old, new):
    """Builds the mutant and runs the pin suite against it; returns (returncode, tail of stdout)."""
    src = open(SRC).read()
    assert src.count(old) == 1
    d = os.path.join(work, name)
    os.makedirs(d, exist_ok=True)
    csrc = os.path.join(d, "mutant.c")
    with open(csrc, "w") as f:
        f.write(src.replace(old, new))
    lib = os.path.join(d, "libmutant.so")
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-shared", "-fPIC",
                    csrc, "-o", lib, "-lm"], check=True)
    env = dict(os.environ, GS_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-p", "no:xdist",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode, r.stdout[-2000:]


@pytest.fixture(scope="module")
def mutant_results(tmp_path_factory):
    """All mutants are built and judged once, a few at a time (each run is a separate process that
    mostly waits for its interpreter to start)."""
    from concurrent.futures import ThreadPoolExecutor
    work = str(tmp_path_factory.mktemp("oracle_mutants"))
    table = {m[0]: m for m in MUTANTS}
    if os.environ.get("PYTEST_XDIST_WORKER"):
        # the test run is already spread over worker processes: each test judges its own mutant
        class OnDemand(dict):
            def __missing__(self, name):
                self[name] = _run_mutant(work, *table[name])
                return self[name]
        return OnDemand()
    workers = max(1, min(6, (os.cpu_count() or 2) - 1))
    with ThreadPoolExecutor(workers) as ex:
        futs = {name: ex.submit(_run_mutant, work, *m) for name, m in table.items()}
        return {name: f.result() for name, f in futs.items()}


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_pins_catch_mutant(mutant_results, name):
    rc, out = mutant_results[name]
    assert rc != 0, f"mutant {name} survived the pins:\n{out}"
    assert "failed" in out or "error" in out.lower()
