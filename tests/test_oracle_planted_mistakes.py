"""Plausible mistakes planted in a copy of the oracle's C source, one at a time: each must make the named pin fail.
(A pin that still passes with the mistake in place would not be pinning that part of the oracle.)"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "dol_oracle.c")

# (what is broken, text in dol_oracle.c, its replacement, pin expected to fail as file::test)
MISTAKES = [
    ("apply: wrong operand (b indexed by i)",
     "acc[col[t]] += (double)ar[ti[t]] * (double)br[tj[t]];", "acc[col[t]] += (double)ar[ti[t]] * (double)br[ti[t] % nb];",
     "test_oracle_damp.py::test_convolution_is_order_sensitive"),
    ("apply: a dropped term (first tuple skipped)",
     "for (int64_t t = 0; t < n; ++t) {\n            if (col[t] < 0) continue;\n            acc[col[t]] +=",
     "for (int64_t t = 1; t < n; ++t) {\n            if (col[t] < 0) continue;\n            acc[col[t]] +=",
     "test_oracle_damp.py::test_sum2_is_discrete_convolution"),
    ("apply: no clamp",
     "out[(int64_t)s * ldo + c] = (float)(acc[c] < 1.0 ? acc[c] : 1.0);", "out[(int64_t)s * ldo + c] = (float)acc[c];",
     "test_oracle_damp.py::test_disjunction_clamps_at_one"),
    ("apply backward: strict clamp gradient",
     "double gh = accf[col[t]] <= 1.0f ? (double)gr[col[t]] : 0.0;", "double gh = accf[col[t]] < 1.0f ? (double)gr[col[t]] : 0.0;",
     "test_oracle_damp.py::test_clamp_gradient_convention"),
    ("apply backward: operands swapped",
     "da[ti[t]] += gh * (double)br[tj[t]];", "da[ti[t]] += gh * (double)ar[ti[t]];",
     "test_oracle_damp.py::test_apply_backward_matches_finite_differences"),
    ("apply backward: gradient of b loses a factor",
     "db[tj[t]] += gh * (double)ar[ti[t]];", "db[tj[t]] += gh;",
     "test_oracle_damp.py::test_apply_backward_euler_identity"),
    ("union: product instead of sum",
     "double t = (double)a[(int64_t)s * lda + ia[c]] + (double)b[(int64_t)s * ldb + ib[c]];",
     "double t = (double)a[(int64_t)s * lda + ia[c]] * (double)b[(int64_t)s * ldb + ib[c]];",
     "test_oracle_damp.py::test_paper_union_example"),
    ("union backward: strict clamp gradient",
     "if (!(t <= 1.0f)) gv = 0.0f;", "if (!(t < 1.0f)) gv = 0.0f;",
     "test_oracle_damp.py::test_clamp_gradient_convention"),
    ("top-k: reversed tie-break (larger mask first)",
     "return (a->mask > b->mask) - (a->mask < b->mask);", "return (a->mask < b->mask) - (a->mask > b->mask);",
     "test_oracle_dtkp.py::test_union_dedupes_and_orders"),
    ("top-k: ascending probability",
     "if (a->prob > b->prob) return -1;\n    if (a->prob < b->prob) return 1;", "if (a->prob > b->prob) return 1;\n    if (a->prob < b->prob) return -1;",
     "test_oracle_dtkp.py::test_staged_topk_matches_brute_force_over_all_tuples"),
    ("top-k: repeated proofs kept",
     "if (dup) continue;", "if (dup && 0) continue;",
     "test_oracle_dtkp.py::test_union_dedupes_and_orders"),
    ("top-k: tag probability not clamped",
     "return sum < 1.0f ? sum : 1.0f;\n}\n\n/* Natural initialisation", "return sum;\n}\n\n/* Natural initialisation",
     "test_oracle_dtkp.py::test_union_dedupes_and_orders"),
    ("proof probability: a fact left out of the product",
     "if ((mask >> j) & 1u) pr = pr * fact_prob[j];", "if (((mask >> j) & 1u) && j > 0) pr = pr * fact_prob[j];",
     "test_oracle_dtkp.py::test_natural_init"),
    ("reachability backward: strict clamp gradient",
     "double gh = pre[v] <= 1.0f ? gr[v] : 0.0;", "double gh = pre[v] < 1.0f ? gr[v] : 0.0;",
     "test_oracle_reach.py::test_clamp_boundary_passes_gradient_in_the_rounds"),
]


def _run_pin(pin, src):
    env = dict(os.environ, DOL_ORACLE_SRC=src)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", pin)]
    return subprocess.run(cmd, capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)


def test_pins_pass_on_an_unpatched_copy(tmp_path):
    """The machinery itself: a verbatim copy of the source passes the pins used below."""
    src = tmp_path / "dol_oracle.c"
    src.write_text(open(SRC).read())
    for pin in sorted({m[3] for m in MISTAKES}):
        res = _run_pin(pin, str(src))
        assert res.returncode == 0, pin + "\n" + res.stdout[-2000:]


@pytest.mark.parametrize("what,old,new,pin", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_fails_its_pin(tmp_path, what, old, new, pin):
    text = open(SRC).read()
    assert text.count(old) >= 1, "the oracle no longer contains the text this mistake is planted in: " + old
    src = tmp_path / "dol_oracle.c"
    src.write_text(text.replace(old, new, 1))
    res = _run_pin(pin, str(src))
    assert res.returncode != 0, "%s: the pin %s still passes" % (what, pin)
    assert "failed" in res.stdout or "error" in res.stdout.lower(), res.stdout[-2000:]
