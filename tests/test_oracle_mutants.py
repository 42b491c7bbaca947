"""Do the pins bite?  Each case below plants ONE plausible mistake in a copy of the
oracle's C source (a wrong sign, a dropped term, a transposed index, the wrong matrix,
the residual taken from the wrong tensor ...), builds the copy on the CPU and runs the
pin suite against it in a child process: at least one pin has to fail.  The unmodified
copy has to pass, so a failure really is the planted mistake.

The pin that compares with stored values written by the oracle itself is left out of
the run: it says nothing about whether the formula is right.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "swiglu_oracle.c")

# (name, [(text in the source, replacement), ...]); every text must occur exactly once.
MUTANTS = [
    ("silu_sign_of_exponent", [("return g / (1.0 + exp(-g));", "return g / (1.0 + exp(g));")]),
    ("silu_without_the_factor_g", [("return g / (1.0 + exp(-g));", "return 1.0 / (1.0 + exp(-g));")]),
    ("silu_denominator_minus", [("return g / (1.0 + exp(-g));", "return g / (1.0 - exp(-g));")]),
    ("gate_and_up_swapped", [("t->A2[o] = u * oracle_silu(g);", "t->A2[o] = g * oracle_silu(u);")]),
    ("up_factor_dropped", [("t->A2[o] = u * oracle_silu(g);", "t->A2[o] = oracle_silu(g);")]),
    ("silu_dropped", [("t->A2[o] = u * oracle_silu(g);", "t->A2[o] = u * g;")]),
    ("silu_on_the_product", [("t->A2[o] = u * oracle_silu(g);", "t->A2[o] = oracle_silu(u * g);")]),
    ("up_uses_gate_matrix", [("u += x * widen(t->Wu,", "u += x * widen(t->Wg,")]),
    ("gate_weight_transposed", [("g += x * widen(t->Wg, (size_t)j * t->d_model + k,", "g += x * widen(t->Wg, (size_t)k * t->d_ff + j,")]),
    ("up_weight_transposed", [("u += x * widen(t->Wu, (size_t)j * t->d_model + k,", "u += x * widen(t->Wu, (size_t)k * t->d_ff + j,")]),
    ("x_transposed", [("double x = widen(t->X, (size_t)m * t->d_model + k,", "double x = widen(t->X, (size_t)k * t->M + m,")]),
    ("a2_stored_transposed", [("size_t o = (size_t)m * t->d_ff + j;", "size_t o = (size_t)j * t->M + m;")]),
    ("a2_read_transposed", [("double a = t->A2[(size_t)m * t->d_ff + j];", "double a = t->A2[(size_t)j * t->M + m];")]),
    ("down_weight_transposed", [("y[n] += a * widen(t->Wd, (size_t)j * t->d_model + n,", "y[n] += a * widen(t->Wd, (size_t)n * t->d_ff + j,")]),
    ("down_sum_sign", [("y[n] += a * widen(t->Wd,", "y[n] -= a * widen(t->Wd,")]),
    ("down_sum_not_accumulated", [("y[n] += a * widen(t->Wd,", "y[n] = a * widen(t->Wd,")]),
    ("down_sum_misses_last_row", [("for (int j = 0; j < t->d_ff; ++j) {\n            double a", "for (int j = 0; j + 1 < t->d_ff; ++j) {\n            double a")]),
    ("stage_one_sum_misses_first_k", [("for (int k = 0; k < t->d_model; ++k) {\n                double x", "for (int k = 1; k < t->d_model; ++k) {\n                double x")]),
    ("bf16_shift", [("<< 16;", "<< 15;")]),
    ("fp16_exponent_bias", [("ldexp((double)(1024 + frac), e - 25)", "ldexp((double)(1024 + frac), e - 24)")]),
    ("fp16_subnormal_scale", [("ldexp((double)frac, -24)", "ldexp((double)frac, -25)")]),
    ("fp16_hidden_bit_dropped", [("ldexp((double)(1024 + frac), e - 25)", "ldexp((double)(frac), e - 25)")]),
    ("fp16_sign_ignored", [("return sign ? -v : v;", "return v;")]),
    ("rms_sum_instead_of_mean", [("sqrt(ss / (double)d_model + eps)", "sqrt(ss + eps)")]),
    ("rms_eps_sign", [("sqrt(ss / (double)d_model + eps)", "sqrt(ss / (double)d_model - eps)")]),
    ("rms_eps_outside_the_root", [("sqrt(ss / (double)d_model + eps)", "sqrt(ss / (double)d_model) + eps")]),
    ("rms_no_root", [("sqrt(ss / (double)d_model + eps)", "(ss / (double)d_model + eps)")]),
    ("rms_weight_dropped", [("= h * wk / r;", "= h / r;")]),
    ("rms_multiplies_by_the_root", [("= h * wk / r;", "= h * wk * r;")]),
    ("rms_weight_added", [("= h * wk / r;", "= (h + wk) / r;")]),
    ("rms_mean_subtracted", [("ss += h * h;", "ss += h * h; if (k + 1 == d_model) { double mu = 0; for (int q = 0; q < d_model; ++q) mu += widen(H, (size_t)m * d_model + q, dtype); mu /= d_model; ss -= d_model * mu * mu; }")]),
    ("block_residual_sign", [("Y[i] += widen(H, i, dtype);", "Y[i] -= widen(H, i, dtype);")]),
    ("block_residual_dropped", [("Y[i] += widen(H, i, dtype);", "Y[i] += 0.0;")]),
    ("block_residual_is_the_normalised_input", [("Y[i] += widen(H, i, dtype);", "Y[i] += N[i];")]),
    ("block_skips_the_normalisation", [("p.X = N; p.Wg = Wg;", "p.X = H; p.Wg = Wg;"), ("p.xdtype = ORACLE_FP64;", "p.xdtype = dtype;")]),
    ("block_ignores_eps", [("oracle_rmsnorm(H, w, N, M, d_model, dtype, eps);", "oracle_rmsnorm(H, w, N, M, d_model, dtype, 0.0);")]),
    ("block_ignores_norm_weight", [("oracle_rmsnorm(H, w, N, M, d_model, dtype, eps);", "oracle_rmsnorm(H, NULL, N, M, d_model, dtype, eps);")]),
]

DRIVER = r"""
import sys
sys.path.insert(0, {root!r})
from oracle import oracle
oracle._SRC = {src!r}
oracle._LIB = {lib!r}
import pytest
sys.exit(pytest.main([{pins!r}, "-x", "-q", "-p", "no:cacheprovider",
                      "--deselect", {pins!r} + "::test_golden_tiny_config_is_reproduced"]))
"""


def _run_pins(tmpdir, name, text):
    src = os.path.join(tmpdir, name + ".c")
    with open(src, "w") as f:
        f.write(text)
    lib = os.path.join(tmpdir, name + ".so")
    # built here, with the oracle's own flags, so that a copy that does not compile cannot pass for a caught mistake
    cc = subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-o", lib, src, "-lm", "-lpthread"],
                        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if cc.returncode != 0:
        return 99, cc.stdout
    code = DRIVER.format(root=ROOT, src=src, lib=lib,
                         pins=os.path.join(ROOT, "tests", "test_oracle_pins.py"))
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=600)
    return r.returncode, r.stdout


def _mutate(text, edits, name):
    for old, new in edits:
        assert text.count(old) == 1, f"mutant {name}: the source has {text.count(old)} occurrences of {old!r}"
        text = text.replace(old, new)
    return text


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with open(SRC) as f:
        original = f.read()
    rc, out = _run_pins(str(tmp_path), "unmodified", original)
    assert rc == 0, "the pins fail on the unmodified oracle:\n" + out[-2000:]

    jobs = [(name, _mutate(original, edits, name)) for name, edits in MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda j: (j[0],) + _run_pins(str(tmp_path), j[0], j[1]), jobs))
    survivors = [name for name, rc, out in results if rc == 0]
    # 1 = some test failed; anything else (2 interrupted, 3 internal error, 4 usage, 5 nothing collected) is a broken run
    broken = [(name, rc, out[-800:]) for name, rc, out in results if rc not in (0, 1)]
    assert not broken, broken
    assert not survivors, f"no pin notices these mistakes: {survivors}"
