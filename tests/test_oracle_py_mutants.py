"""The pins of the oracle's Python parts (cost model, plan search, granularity rule) must catch planted mistakes.

Each mutant is a one-line change to a copy of oracle/__init__.py; the cost-model, plan-search and granularity
tests are run against the copy in a child process and have to fail on an assertion.
"""
import os
import shutil
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SRC = (ROOT / "oracle" / "__init__.py").read_text()

MUTANTS = {
    "zdp_and_dp_collectives_swapped": ("steps = (3.0 if zdp else 2.0) * (N - 1)", "steps = (2.0 if zdp else 3.0) * (N - 1)"),
    "dp_states_sharded_instead": ("mem = mem + ((m_model / N if zdp else m_model) + (b * m_act + m_extra))",
                                  "mem = mem + ((m_model if zdp else m_model / N) + (b * m_act + m_extra))"),
    "time_not_per_sample": ("    return mem, time / b\n", "    return mem, time\n"),
    "ring_steps_off_by_one": ("3.0 * (N - 1) * step + b * gamma, 2.0 * (N - 1) * step + b * gamma",
                              "3.0 * N * step + b * gamma, 2.0 * N * step + b * gamma"),
    "limit_excluded": ("        ok = mem <= m_limit\n", "        ok = mem < m_limit\n"),
    "later_batch_wins_ties": ('if best is None or per_sample < best["time_per_sample"]:', 'if best is None or per_sample <= best["time_per_sample"]:'),
    "search_ignores_activations": ("            rest = b * m_act + m_extra\n", "            rest = m_act + m_extra\n"),
    "budget_excludes_equal": ("        if staging_budget and peak > staging_budget:", "        if staging_budget and peak >= staging_budget:"),
    "fastest_before_smallest": ("keep.sort(key=lambda i: (table[i][0], table[i][2], i))", "keep.sort(key=lambda i: (table[i][2], table[i][0], i))"),
    "slowdown_is_a_factor": ("keep = [i for i in fits if table[i][2] <= (1.0 + max_slowdown) * fastest]",
                             "keep = [i for i in fits if table[i][2] <= max(1.0, max_slowdown) * fastest]"),
}
PINS = ["tests/test_plan_search.py", "tests/test_granularity.py"]


def _run(tmp: Path, text: str):
    pkg = tmp / "oracle"
    pkg.mkdir()
    (pkg / "__init__.py").write_text(text)
    shutil.copy(ROOT / "oracle" / "osdp_oracle.c", pkg / "osdp_oracle.c")
    env = dict(os.environ, OSDP_ORACLE_PY=str(pkg))
    return subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                          capture_output=True, text=True, timeout=600)


def test_unmutated_copy_passes(tmp_path):
    res = _run(tmp_path, SRC)
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_python_mutant(tmp_path, name):
    old, new = MUTANTS[name]
    assert SRC.count(old) == 1, f"mutation site of {name} not found exactly once"
    res = _run(tmp_path, SRC.replace(old, new))
    assert res.returncode != 0, f"the pins did not notice the planted mistake {name!r}"
    assert "failed" in res.stdout, res.stdout[-2000:]
