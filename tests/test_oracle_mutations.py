"""Do the pins bite?  Each case below plants ONE plausible mistake in a copy of the oracle's C source (on the
CPU, in a temporary directory), builds it, and runs the oracle's pin tests against that build in a child
process: the pins must fail.  The unmodified source must pass the same command.  A replacement that no longer
matches the source fails the test too, so the list cannot silently rot."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rapid_oracle.c")

# (name, text in the source, replacement, the pin file expected to catch it)
MUTANTS = [
    ("sign of the mixing term", "zh[v] = z[v] + eta * T * (q[v] - p[v]);", "zh[v] = z[v] + eta * T * (p[v] - q[v]);",
     "test_oracle_accept.py"),
    ("temperature dropped from the mixing term", "zh[v] = z[v] + eta * T * (q[v] - p[v]);", "zh[v] = z[v] + eta * (q[v] - p[v]);",
     "test_oracle_accept.py"),
    ("min instead of max in the residual", "double m = a > c ? a : c;", "double m = a < c ? a : c;", "test_oracle_accept.py"),
    ("tail rule replaces the head", "if (ph[v] < thr) ph[v] = p[v];", "if (ph[v] > thr) ph[v] = p[v];", "test_oracle_accept.py"),
    ("inverse CDF with >= instead of >", "if (run > t) { tok = v; break; }", "if (run >= t) { tok = v; break; }",
     "test_oracle_accept.py"),
    ("accept test without the clamp to 1 in the margin", "double thr = rho < 1.0 ? rho : 1.0;\n            if (ratio) ratio[(int64_t)b * gmax + k] = rho;\n            if (accept_margin) accept_margin[(int64_t)b * gmax + k] = fabs(thr - r);\n            if (n == g && !(r <= thr)) {",
     "double thr = rho < 1.0 ? rho : 1.0;\n            if (ratio) ratio[(int64_t)b * gmax + k] = rho;\n            if (accept_margin) accept_margin[(int64_t)b * gmax + k] = fabs(rho - r);\n            if (n == g && !(r <= thr)) {",
     "test_oracle_accept.py"),
    ("draw margin not normalised", "double a = (t - lo) / W, c = (run - t) / W;", "double a = (t - lo), c = (run - t);",
     "test_oracle_accept.py"),
    ("causal mask off by one", "int64_t nvis = L - Q + i + 1;", "int64_t nvis = L - Q + i;", "test_oracle_attn.py"),
    ("grouped-query head map", "int hkv = h / G;", "int hkv = h % Hkv;", "test_oracle_attn.py"),
    ("softmax scale dropped", "s[j] = scale * acc;", "s[j] = acc;", "test_oracle_attn.py"),
    ("greedy limit compares the wrong way", "gap_t > gap_d ? INFINITY : (gap_t < gap_d ? 0.0 : 1.0)",
     "gap_t < gap_d ? INFINITY : (gap_t > gap_d ? 0.0 : 1.0)", "test_oracle_accept.py"),
    ("freed pages off by one", "const int used_after = j * page_size < l_new;", "const int used_after = j * page_size <= l_new;",
     "test_oracle_kv.py"),
    ("retrieval keeps chunks below the threshold", "if (rank < top_k && sim[i] >= threshold)", "if (rank < top_k)",
     "test_oracle_retrieve.py"),
]


def run_pins(lib_path, pin_file):
    env = dict(os.environ, RAPID_ORACLE_LIB=lib_path)
    cmd = [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pin_file), "-x", "-q", "-p", "no:cacheprovider"]
    return subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True)


def test_unmodified_source_passes_under_the_same_harness(tmp_path):
    lib = oracle.compile_source(SRC, str(tmp_path / "clean.so"))
    for pin in sorted({m[3] for m in MUTANTS}):
        r = run_pins(lib, pin)
        assert r.returncode == 0, (pin, r.stdout[-2000:])


@pytest.mark.parametrize("name,old,new,pin", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new, pin):
    text = open(SRC).read()
    assert text.count(old) == 1, f"'{old}' must occur exactly once in the oracle source"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = oracle.compile_source(str(src), str(tmp_path / "mutant.so"))
    r = run_pins(lib, pin)
    assert r.returncode != 0, f"no pin in {pin} noticed: {name}"
    assert " failed" in r.stdout, r.stdout[-2000:]             # a test failure, not a crash of the harness
