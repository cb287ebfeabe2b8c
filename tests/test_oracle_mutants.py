"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source
(a dropped term, a wrong index, a swapped operand, a wrong rounding rule), builds it, and runs the
pin tests against that build in a child process: they must fail.  Everything happens on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mics_oracle.c")

BF16, GATHER, SYNC, ADAM, DTYPES, PIPE, COAL = (
    "tests/test_oracle_bf16.py", "tests/test_oracle_gather.py", "tests/test_oracle_gradsync.py",
    "tests/test_oracle_adam.py", "tests/test_oracle_dtypes.py", "tests/test_oracle_pipeline.py",
    "tests/test_oracle_coalesced.py")

MUTANTS = [
    # name, text in the source, replacement, pin files that must notice
    ("bf16 ties round up instead of to even",
     "else if (dropped == 0x8000u && (kept & 1u)) kept += 1;", "else if (dropped == 0x8000u) kept += 1;", [BF16]),
    ("bf16 truncates", "if (dropped > 0x8000u) kept += 1;", "if (0) kept += 1;", [BF16]),
    ("bf16 NaN with low payload becomes Inf", "if ((u & 0x007FFFFFu) != 0) kept |= 0x0040u;", "", [BF16]),
    ("stage 1 gathers consecutive ranks instead of equal local ranks",
     "shards[j * k + l]", "shards[l * nodes + j]", [GATHER]),
    ("reorder takes the chunk of the neighbouring local rank",
     "size_t l = g % (size_t)k;   /* local rank of rank g                  */",
     "size_t l = (g + 1) % (size_t)k;", [GATHER]),
    ("reorder swaps node and local rank",
     "size_t at = j * S + i;", "size_t at = (g % ((size_t)p / (size_t)k)) * S + i;", [GATHER]),
    ("concatenation is off by one element", "size_t i = x % S; /* position inside its shard */",
     "size_t i = (x + 1) % S;", [GATHER]),
    ("wrong layout gathers in node order", "(unsigned char*)W + (size_t)l * per_rank",
     "(unsigned char*)W + (size_t)(k - 1 - l) * per_rank", [GATHER]),
    ("reduce-scatter drops the last rank",
     "for (int q = 1; q < p; ++q) {\n            float gq = orc_bf16_widen(grads[q][x]);",
     "for (int q = 1; q + 1 < p; ++q) {\n            float gq = orc_bf16_widen(grads[q][x]);", [SYNC]),
    ("reduce-scatter sums ranks in descending order",
     "float partial = orc_bf16_widen(grads[0][x]);\n        for (int q = 1; q < p; ++q) {",
     "float partial = orc_bf16_widen(grads[p - 1][x]);\n        for (int q = p - 2; q >= 0; --q) {", [SYNC]),
    ("first micro-step accumulates into stale contents",
     "float before = accumulate ? acc[i] : 0.0f;\n        acc[i] = before + partial;\n    }\n    return 0;\n}\n\nstatic float widen_grad",
     "float before = acc[i];\n        acc[i] = before + partial;\n    }\n    return 0;\n}\n\nstatic float widen_grad", [SYNC]),
    ("reduce-scatter ignores the element offset", "size_t x = elem_offset + i;\n        float partial = orc_bf16_widen",
     "size_t x = i;\n        float partial = orc_bf16_widen", [SYNC, PIPE]),
    ("replica average counts the first copy twice",
     "float sum = copies[0][i];\n        for (int c = 1; c < r; ++c)", "float sum = copies[0][i];\n        for (int c = 0; c < r; ++c)", [SYNC]),
    ("replica average forgets the scale", "out[i] = sum * scale;", "out[i] = sum;", [SYNC]),
    ("Adam without the second bias correction", "double v_hat = v_new / corr2;", "double v_hat = v_new;", [ADAM]),
    ("Adam with epsilon inside the square root", "(sqrt(v_hat) + e)", "sqrt(v_hat + e)", [ADAM]),
    ("Adam second moment decays with beta1 (bias correction too)",
     "const double corr2 = 1.0 - pow(b2, (double)step);\n#pragma omp parallel for schedule(static) num_threads(g_threads)\n    for (size_t i = 0; i < count; ++i) {\n        double g = grad[i], w = master[i], m = exp_avg[i], v = exp_avg_sq[i];\n        double m_new = b1 * m + (1.0 - b1) * g;\n        double v_new = b2 * v + (1.0 - b2) * g * g;",
     "const double corr2 = 1.0 - pow(b1, (double)step);\n#pragma omp parallel for schedule(static) num_threads(g_threads)\n    for (size_t i = 0; i < count; ++i) {\n        double g = grad[i], w = master[i], m = exp_avg[i], v = exp_avg_sq[i];\n        double m_new = b1 * m + (1.0 - b1) * g;\n        double v_new = b1 * v + (1.0 - b1) * g * g;", [ADAM]),
    ("Adam steps uphill", "double w_new = w - a * (", "double w_new = w + a * (", [ADAM]),
    ("Adam drops the weight decay", "+ wd * w);", ");", [ADAM]),
    ("Adam first moment uses the squared gradient", "double m_new = b1 * m + (1.0 - b1) * g;",
     "double m_new = b1 * m + (1.0 - b1) * g * g;", [ADAM]),
    ("single-precision Adam forgets to square the gradient", "float gg = g * g;", "float gg = g;", [ADAM]),
    ("single-precision Adam divides by the wrong bias correction", "float m_hat = m_new / corr1;",
     "float m_hat = m_new / corr2;", [ADAM]),
    ("binary16 subnormals are off by a factor of two", "(127 - 15 + 1 - shift)", "(127 - 15 - shift)", [DTYPES]),
    ("binary16 narrowing rounds ties up instead of to even",
     "if (rest > half || (rest == half && (kept & 1u))) kept += 1;", "if (rest >= half) kept += 1;", [DTYPES]),
    ("binary16 narrowing truncates", "if (rest > half || (rest == half && (kept & 1u))) kept += 1;", "", [DTYPES]),
    ("binary16 narrowing drops one bit too few for subnormals", "13 + (-14 - e)", "12 + (-14 - e)", [DTYPES]),
    ("binary16 narrowing overflows one binade late", "if (e > 15) return", "if (e > 16) return", [DTYPES]),
    ("binary16 narrowing flushes the smallest subnormal's upper half to zero", "e < -25", "e < -24", [DTYPES]),
    ("typed reduction reads binary16 as bf16",
     "if (dtype == ORC_DTYPE_F16) return orc_f16_widen(((const uint16_t*)buf)[x]);", "", [DTYPES]),
]


def run_pins(lib, files):
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
                           "--oracle-lib", lib, *files], cwd=ROOT, capture_output=True, text=True, timeout=300)


def build_variant(tmp_path, text):
    import oracle
    src = tmp_path / "mics_oracle_variant.c"
    src.write_text(text)
    return oracle.build(force=True, src=str(src), out=str(tmp_path / "libvariant.so"))


def test_unmodified_copy_passes_every_pin(tmp_path):
    lib = build_variant(tmp_path, open(SRC).read())
    res = run_pins(lib, [BF16, GATHER, SYNC, ADAM, DTYPES, PIPE, COAL])
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]


@pytest.mark.parametrize("name,old,new,files", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, files):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    lib = build_variant(tmp_path, text.replace(old, new))
    res = run_pins(lib, files)
    # 1 = tests ran and at least one failed; anything else would be a broken harness
    assert res.returncode == 1, f"'{name}' went unnoticed or the run broke:\n" + res.stdout[-1500:] + res.stderr[-500:]
    assert " failed" in res.stdout
