"""The pins must notice a broken oracle.  Each case plants one plausible mistake (a dropped term, a
wrong sign, index or bound, a transposed operand) in a copy of oracle/tlin_oracle.c, builds it on
the CPU and runs tests/test_oracle_pins.py against that build: the run has to fail.  The
unmodified source, built and run the same way, has to pass."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "tlin_oracle.c")

# (name, text in the source, replacement, which occurrence: 0 = first, 1 = second, ...)
MUTATIONS = [
    ("scale dropped from the logits", "s[j] = scale * acc;", "s[j] = acc;", 0),
    ("keys read transposed", "widen(K, dtype, kbase + (size_t)j * D + k)", "widen(K, dtype, kbase + (size_t)k * n + j)", 0),
    ("value columns reversed", "widen(V, dtype, vbase + (size_t)j * D + k)", "widen(V, dtype, vbase + (size_t)j * D + (D - 1 - k))", 0),
    ("sign of the exponent", "double w = exp(s[j] - m) / z;", "double w = exp(m - s[j]) / z;", 0),
    ("log-sum-exp without the maximum", "return m + log(z);", "return log(z);", 0),
    ("causal bound off by one", "(size_t)bh * W * D, i + 1, D, scale, s, O + (size_t)u * D);", "(size_t)bh * W * D, i, D, scale, s, O + (size_t)u * D);", 0),
    ("causal mask dropped", "(size_t)bh * W * D, i + 1, D, scale, s, O + (size_t)u * D);", "(size_t)bh * W * D, W, D, scale, s, O + (size_t)u * D);", 0),
    ("SUM keeps only the history term", "for (int k = 0; k < D; ++k) o[k] += t[k];", "for (int k = 0; k < D; ++k) o[k] = t[k];", 0),
    ("JOINT window logits overwrite the history logits", "logits(q, Kw, dtype, (size_t)bh * W * D, i + 1, D, scale, s + N);", "logits(q, Kw, dtype, (size_t)bh * W * D, i + 1, D, scale, s);", 0),
    ("JOINT drops the newest key from the normaliser", "int n = N + i + 1;", "int n = N + i;", 0),
    ("JOINT history values weighted with the window's logits", "if (N > 0) weighted_values(s, N, m, z, Vh, dtype, (size_t)bh * N * D, D, o);", "if (N > 0) weighted_values(s + 1, N, m, z, Vh, dtype, (size_t)bh * N * D, D, o);", 0),
    ("batch index ignored for the history", "double l = attend(q, Kh, Vh, dtype, (size_t)bh * N * D, N, D, scale, s, O + (size_t)u * D);", "double l = attend(q, Kh, Vh, dtype, (size_t)(bh % H) * N * D, N, D, scale, s, O + (size_t)u * D);", 0),
    ("bf16 widened with the wrong shift", "<< 16;", "<< 15;", 0),
    ("slide: window rows taken from the start of the sequence", "size_t wbase = base + (size_t)N * D;", "size_t wbase = base;", 0),
    ("slide: history one chunk short", "int N = (p / W) * W;            /* history rows of this position's chunk */", "int N = (p / W) * W; int N_full = N; N = N > W ? N - W : N; (void)N_full;", 0),
    ("slide SUM keeps only the window term", "for (int k = 0; k < D; ++k) o[k] += t[k];", "for (int k = 0; k < D; ++k) o[k] += 0.0 * t[k];", 1),
]


def nth_replace(text, old, new, n):
    pos = -1
    for _ in range(n + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, f"mutation target not found: {old!r}"
    return text[:pos] + new + text[pos + len(old):]


def build_and_run_pins(tmp, tag, source):
    c = os.path.join(tmp, f"{tag}.c")
    so = os.path.join(tmp, f"lib{tag}.so")
    with open(c, "w") as f:
        f.write(source)
    subprocess.run(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", so, c, "-lm"], check=True)
    env = dict(os.environ, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-m", "not gpu", "--oracle-lib", so, "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:]


def test_pins_pass_on_the_real_oracle_and_fail_on_every_planted_mistake(tmp_path):
    src = open(SRC).read()
    jobs = [("clean", src)] + [(f"mut{i}", nth_replace(src, old, new, n)) for i, (_, old, new, n) in enumerate(MUTATIONS)]
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda j: build_and_run_pins(str(tmp_path), *j), jobs))
    rc, out = results[0]
    assert rc == 0, "pins fail on the unmodified oracle built through the hook:\n" + out
    survived = [MUTATIONS[i][0] for i, (rc, _) in enumerate(results[1:]) if rc == 0]
    assert not survived, f"planted mistakes that no pin noticed: {survived}"
    # the substitute-oracle option must be refused as soon as GPU tests are selected
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-q", "-m", "gpu", "--collect-only",
                        "--oracle-lib", SRC, "-p", "no:cacheprovider"], cwd=ROOT, capture_output=True, text=True, timeout=600)
    assert r.returncode == 4 and "refused" in (r.stdout + r.stderr), (r.returncode, r.stderr[-500:])
    for (name, *_), (rc, out) in zip(MUTATIONS, results[1:]):
        assert rc == 1, f"{name}: pytest ended with {rc} (expected test failures, not a crash):\n{out}"
