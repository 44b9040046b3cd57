"""The pins must notice a plausible mistake anywhere in the oracle.

Each case plants ONE mistake in a copy of the oracle's source (a swapped operand, a dropped term,
a wrong index, `<` for `<=`, ...), builds it beside the real one and runs the pin suite against
it in a child process: the suite has to fail.  Everything happens on the CPU, in a temporary
directory; the real oracle library is never replaced.
"""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCE = os.path.join(ROOT, "oracle", "specsteer_oracle.c")

# (what is planted, text in the oracle's source, what replaces its first occurrence)
MUTANTS = [
    ("recovery steers away from the context (S_ctx and S_noctx swapped in Eq. 8)", "? 0.0 : hp - hm", "? 0.0 : hm - hp"),
    ("lambda dropped from Eq. 7", "- log(lam))", ")"),
    ("strict acceptance test", "(double)u[t] <= alpha", "(double)u[t] < alpha"),
    ("ratio of Eq. 7 inverted", "lpG - lpS - log(lam)", "lpS - lpG - log(lam)"),
    ("token drawn with an acceptance uniform", "u[kmax]", "u[n]"),
    ("recovery taken one row late", "seq_off + (int64_t)n * st;", "seq_off + (int64_t)(n+1) * st;"),
    ("non-strict CDF comparison", "c > us", "c >= us"),
    ("no temperature in the recovery distribution", "g[v] = hrec / T;", "g[v] = hrec;"),
    ("temperature on the generalist's term only", "g[v] = hrec / T;", "g[v] = hl / T + beta * (hp - hm);"),
    ("alpha not capped at 1", "if (alpha > 1.0) alpha = 1.0;", ""),
    ("loop goes on after a rejection", "n = t;\n            break;", "if (n == K) n = t;"),
    ("ratio test reads the context distribution",
     "scaled_row(Sm, dt, seq_off + (int64_t)t * st, V, T, sm);\n        const double lpG",
     "scaled_row(Sp, dt, seq_off + (int64_t)t * st, V, T, sm);\n        const double lpG"),
    ("log-sum-exp forgets its maximum", "return m + log(s);", "return log(s);"),
    ("beta dropped from Eq. 8", "hl + beta * ((hp", "hl + ((hp"),
    ("a token masked in both specialist rows poisons the row", "(hp == hm) ? 0.0 : hp - hm", "hp - hm"),
    ("a token the generalist masks comes back on the cloud side", "(hl == -INFINITY) ? -INFINITY : hl - beta", "hl - beta"),
    ("logits multiplied by T", "widen(base, dtype, off + v) / T", "widen(base, dtype, off + v) * T"),
    ("bf16 widened with the wrong shift", "<< 16", "<< 15"),
    ("uniforms indexed with the draft's row length", "uniforms + (size_t)b * (kmax + 1)", "uniforms + (size_t)b * (kmax)"),
    ("draft indexed with the logits' row count", "draft + (size_t)b * kmax, K", "draft + (size_t)b * (kmax+1), K"),
    ("longest allowed draft flagged", "K > kmax", "K >= kmax"),
    ("fallback token may have no probability", "if (pv > 0.0) last_pos = v;", "last_pos = v;"),
    ("greedy pick keeps the last maximum", "if (hrec > hmax) {", "if (hrec >= hmax) {"),
    ("greedy pick ignores the steering term", "if (hrec > hmax) {", "if (hl > hmax) {"),
    ("bonus row confused with the last draft row", "int n = K;\n    for (int t = 0; t < K; ++t) {", "int n = K > 0 ? K - 1 : 0;\n    for (int t = 0; t < K; ++t) {"),
    ("cloud side adds the context-free logits", "hl - beta * widen(S_noctx, dt, off + v)",
     "hl + beta * widen(S_noctx, dt, off + v)"),
    ("payload ties broken by the higher id", "return (a->idx > b->idx) - (a->idx < b->idx);",
     "return (a->idx < b->idx) - (a->idx > b->idx);"),
    ("payload in increasing order", "if (a->v > b->v) return -1;\n    if (a->v < b->v) return 1;",
     "if (a->v > b->v) return 1;\n    if (a->v < b->v) return -1;"),
    ("edge side forgets beta", "(double)vl[j] + beta * widen(S_ctx, dt, off + ix[j])", "(double)vl[j] + widen(S_ctx, dt, off + ix[j])"),
    ("edge side ignores the temperature", "x[j] = h[j] / T;", "x[j] = h[j];"),
    ("edge side falls back to an entry without probability", "if (pj > 0.0) last_pos = j;", "last_pos = j;"),
    ("edge side draws with a non-strict comparison", "c > (double)uniform[b]", "c >= (double)uniform[b]"),
]


@pytest.fixture(scope="module")
def source_text():
    with open(SOURCE) as f:
        return f.read()


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_a_planted_mistake(tmp_path, source_text, what, old, new):
    assert source_text.count(old) >= 1, f"the oracle no longer contains {old!r}: update this mutant"
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(source_text.replace(old, new, 1))
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), str(src), "-lm"],
                   check=True)
    env = dict(os.environ, SPECSTEER_ORACLE_LIBRARY=str(lib), OMP_NUM_THREADS="2")
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode != 0, f"no pin noticed: {what}"
    # 1 = a pin failed; a mutant that indexes out of bounds may also take the child down with a signal.
    # Anything else (no tests collected, usage error) would be this test's own fault.
    assert run.returncode == 1 or run.returncode < 0 or run.returncode in (134, 139), (run.returncode, run.stderr[-400:])
