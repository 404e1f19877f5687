"""Do the pins bite?  Each mutant is the oracle's C source with one plausible
mistake planted (on the CPU, in a temporary copy); the pin tests are run against
it in a subprocess and must fail.  A mutant that survives means a hole in the
pins."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "cf_oracle.c")
PIN_FILES = ["tests/test_oracle_sqnorm.py", "tests/test_oracle_blend.py", "tests/test_oracle_bf16_copy.py",
             "tests/test_oracle_adam.py"]

# (name, text in oracle/cf_oracle.c, replacement)
MUTANTS = [
    ("sqnorm: square dropped", "double v = (double)g[k];\n        acc += v * v;", "double v = (double)g[k];\n        acc += v;"),
    ("sqnorm: absolute value instead of square", "double v = (double)g[k];\n        acc += v * v;",
     "double v = (double)g[k];\n        acc += fabs(v);"),
    ("sqnorm: last tensor of the stage left out", "for (uint32_t t = 0; t < num_tensors; ++t)\n        omega += cfo_sqnorm_f32",
     "for (uint32_t t = 0; t + 1 < num_tensors; ++t)\n        omega += cfo_sqnorm_f32"),
    ("sqnorm: threaded split loses the remainder", "uint64_t hi = (p == threads - 1) ? n : n / (uint64_t)threads * (uint64_t)(p + 1);\n            piece[p]",
     "uint64_t hi = n / (uint64_t)threads * (uint64_t)(p + 1);\n            piece[p]"),
    ("sqnorm bf16: square dropped", "double v = bf16_to_f64(g[k]);\n        acc += v * v;", "double v = bf16_to_f64(g[k]);\n        acc += v;"),
    ("blend: weights swapped", "double numerator = wp * a + wn * b;", "double numerator = wn * a + wp * b;"),
    ("blend: the algorithm box's misprint (omega_{i-1} on both terms)", "double numerator = wp * a + wn * b;",
     "double numerator = wp * a + wp * b;"),
    ("blend: second term dropped", "double numerator = wp * a + wn * b;", "double numerator = wp * a;"),
    ("blend: difference instead of sum", "double numerator = wp * a + wn * b;", "double numerator = wp * a - wn * b;"),
    ("blend: not normalised", "return numerator / denominator;", "return numerator;"),
    ("blend: denominator without omega_{i+1}", "double denominator = wp + wn;", "double denominator = wp;"),
    ("blend: unweighted mean whatever the omegas", "double numerator = wp * a + wn * b;\n    double denominator = wp + wn;",
     "double numerator = a + b;\n    double denominator = 2.0;"),
    ("blend f32: next read from prev", "blend_value(wp, wn, (double)prev[k], (double)next[k])", "blend_value(wp, wn, (double)prev[k], (double)prev[k])"),
    ("blend f32: arithmetic in binary32", "out[k] = (float)blend_value(wp, wn, (double)prev[k], (double)next[k]);",
     "out[k] = ((float)wp * prev[k] + (float)wn * next[k]) / ((float)wp + (float)wn);"),
    ("blend bf16: rounded through binary32 first", "out[k] = f64_to_bf16(blend_value(",
     "out[k] = f64_to_bf16((double)(float)blend_value("),
    ("bf16: truncation instead of nearest-even", "double r = nearbyint(scaled);", "double r = floor(scaled);"),
    ("bf16: ties away from zero", "double r = nearbyint(scaled);", "double r = floor(scaled + 0.5);"),
    ("bf16: subnormals flushed", "if (E < -126) E = -126;", "if (E < -126) return sign;"),
    ("bf16: widening shift off by one", "uint32_t w = (uint32_t)h << 16;", "uint32_t w = (uint32_t)h << 15;"),
    ("weights: zero omega on one side treated as unusable", "omega_next >= 0.0 && isfinite(d)", "omega_next > 0.0 && isfinite(d)"),
    ("weights: negative omega accepted", "omega_prev >= 0.0 &&", "1 &&"),
    ("weights: zero sum accepted", "d >= 2.2250738585072014e-308", "d >= 0.0"),
    ("common scale: only one weight scaled", "*wn = ldexp(*wn, 1 - e);", ""),
    ("common scale: factor inverted (sum driven out of range instead of into [1, 2))", "*wp = ldexp(*wp, 1 - e);\n    *wn = ldexp(*wn, 1 - e);",
     "*wp = ldexp(*wp, e - 1);\n    *wn = ldexp(*wn, e - 1);"),
    ("common scale: left out of the fp32 blend", "cfo_common_scale(&wp, &wn);\n    if (threads < 1) threads = 1;\n#pragma omp parallel for num_threads(threads) schedule(static)\n    for (uint64_t k = 0; k < n; ++k)\n        out[k] = (float)",
     "if (threads < 1) threads = 1;\n#pragma omp parallel for num_threads(threads) schedule(static)\n    for (uint64_t k = 0; k < n; ++k)\n        out[k] = (float)"),
    ("range copy: source read from element 0", "const char *s = (const char *)src + first * elem_bytes;", "const char *s = (const char *)src;"),
    ("range copy: count taken as bytes", "for (uint64_t k = 0; k < count * elem_bytes; ++k) d[k] = s[k];", "for (uint64_t k = 0; k < count; ++k) d[k] = s[k];"),
    ("adam: betas swapped in the moments", "m[k] = (float)(beta1 * (double)m[k] + (1.0 - beta1) * grad);",
     "m[k] = (float)(beta2 * (double)m[k] + (1.0 - beta2) * grad);"),
    ("adam: second moment of g instead of g^2", "(1.0 - beta2) * (grad * grad));", "(1.0 - beta2) * grad);"),
    ("adam: first bias correction missing", "double mhat = (double)m[k] / correction1;", "double mhat = (double)m[k];"),
    ("adam: second bias correction missing", "double vhat = (double)v[k] / correction2;", "double vhat = (double)v[k];"),
    ("adam: step count off by one in the bias correction", "double correction1 = 1.0 - pow(beta1, (double)t);",
     "double correction1 = 1.0 - pow(beta1, (double)t + 1.0);"),
    ("adam: eps inside the square root", "(double)w[k] - lr * mhat / (sqrt(vhat) + eps)", "(double)w[k] - lr * mhat / sqrt(vhat + eps)"),
    ("adam: ascent instead of descent", "(double)w[k] - lr * mhat", "(double)w[k] + lr * mhat"),
    ("adam: no square root", "(double)w[k] - lr * mhat / (sqrt(vhat) + eps)", "(double)w[k] - lr * mhat / (vhat + eps)"),
    ("adam: update from the old first moment",
     "        m[k] = (float)(beta1 * (double)m[k] + (1.0 - beta1) * grad);\n        v[k] = (float)(beta2 * (double)v[k] + (1.0 - beta2) * (grad * grad));\n        double mhat = (double)m[k] / correction1;",
     "        double mhat = (double)m[k] / correction1;\n        m[k] = (float)(beta1 * (double)m[k] + (1.0 - beta1) * grad);\n        v[k] = (float)(beta2 * (double)v[k] + (1.0 - beta2) * (grad * grad));"),
    ("adam: omega of the first moment instead of the gradient", "omega += grad * grad;", "omega += (double)m[k] * (double)m[k];"),
    ("adam: moments kept unrounded for the update", "double mhat = (double)m[k] / correction1;",
     "double mhat = (beta1 * (double)m[k] + (1.0 - beta1) * grad) / correction1;"),
    ("copy: one byte short", "memcpy(dst, src, nbytes);\n        return;", "memcpy(dst, src, nbytes ? nbytes - 1 : 0);\n        return;"),
]


def _run_mutant(args):
    idx, (name, old, new), tmp = args
    src = open(SRC).read()
    if src.count(old) < 1:
        return name, "pattern not found in the oracle source"
    mutated = src.replace(old, new, 1)
    c_path = os.path.join(tmp, f"mutant{idx}.c")
    so_path = os.path.join(tmp, f"mutant{idx}.so")
    with open(c_path, "w") as f:
        f.write(mutated)
    cc = subprocess.run(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                         c_path, "-o", so_path, "-lm"], capture_output=True, text=True)
    if cc.returncode != 0:
        return name, "mutant does not compile: " + cc.stderr[-300:]
    env = dict(os.environ, CF_ORACLE_LIB=so_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    if r.returncode == 0:
        return name, "SURVIVED: every pin passed"
    if "passed" not in r.stdout and "failed" not in r.stdout:
        return name, "pin run broke instead of failing: " + (r.stdout + r.stderr)[-300:]
    return name, None


def test_unmutated_oracle_passes_through_the_same_harness(tmp_path):
    # the harness itself: the pristine source, built the same way, passes
    so_path = str(tmp_path / "pristine.so")
    subprocess.run(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", SRC, "-o", so_path,
                    "-lm"], check=True)
    env = dict(os.environ, CF_ORACLE_LIB=so_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES], cwd=ROOT,
                       env=env, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-500:]


def test_every_planted_mistake_is_caught(tmp_path):
    jobs = [(i, m, str(tmp_path)) for i, m in enumerate(MUTANTS)]
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run_mutant, jobs))
    problems = [f"{name}: {why}" for name, why in results if why]
    assert not problems, "\n".join(problems)
