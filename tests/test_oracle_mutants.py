"""The pins must catch plausible mistakes: each planted error in a copy of the oracle has to fail them.

Every mutant is a one-line change to a copy of oracle/osdp_oracle.c (a wrong index, a dropped term, a
flipped sign, a rounding direction), built with gcc and handed to the pin tests in a child process.
All mutants stay within bounds of their arrays: they compute wrong numbers, they do not crash.
"""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SRC = (ROOT / "oracle" / "osdp_oracle.c").read_text()

MUTANTS = {
    "fwd_wrong_column": ("y[o] += x * osdp_oracle_bf16_to_f64(w[o]);", "y[o] += x * osdp_oracle_bf16_to_f64(w[(o + 1) % O]);"),
    "dx_reversed_index": ("osdp_oracle_bf16_to_f64(dY[t * lddy + o]) * osdp_oracle_bf16_to_f64(W[i * ldw + o]);",
                          "osdp_oracle_bf16_to_f64(dY[t * lddy + (O - 1 - o)]) * osdp_oracle_bf16_to_f64(W[i * ldw + o]);"),
    "dw_dropped_term": ("    for (int64_t t = 0; t < T; ++t) {\n      double x = osdp_oracle_bf16_to_f64(X[t * ldx + i]);\n      const uint16_t *d = dY + t * lddy;",
                        "    for (int64_t t = 0; t < T - 1; ++t) {\n      double x = osdp_oracle_bf16_to_f64(X[t * ldx + i]);\n      const uint16_t *d = dY + t * lddy;"),
    "dx_partial_sign": ("\n    for (int64_t e = 0; e < T * I; ++e) dX[e] += part[e];", "\n    for (int64_t e = 0; e < T * I; ++e) dX[e] -= part[e];"),
    "mixed_dx_partial_sign": ("\n      for (int64_t e = 0; e < T * I; ++e) dX[e] += part[e];", "\n      for (int64_t e = 0; e < T * I; ++e) dX[e] -= part[e];"),
    "slice_bound_rounds_up": ("*c1 = ((j + 1) * O) / k;", "*c1 = ((j + 1) * O + k - 1) / k;"),
    "shard_length_off_by_one": ("return (I * O + N - 1) / N;", "return (I * O + N) / N;"),
    "gather_reversed_columns": ("Ws[r * w + c] = shards[s][off];", "Ws[r * w + (w - 1 - c)] = shards[s][off];"),
    "staging_ignores_uneven_slices": ("return slots * wmax * I * elem_bytes;", "return slots * (O / k) * I * elem_bytes;"),
    "fwd_concat_offset": ("memcpy(Y + t * O + c0, Yj + t * w, (size_t)w * sizeof(double));",
                          "memcpy(Y + t * O + (O - c0 - w), Yj + t * w, (size_t)w * sizeof(double));"),
    "dw_scatter_column": ("dW_shards[s][off] = dWj[r * w + c];", "dW_shards[s][off] = dWj[r * w + (c + 1) % w];"),
    "rows_fwd_wrong_x_offset": ("osdp_oracle_matmul_fwd(T, w, O, X + r0, I, Ws, O, part); /* X[:, r0:r1] . Ws */",
                                "osdp_oracle_matmul_fwd(T, w, O, X, I, Ws, O, part); /* X[:, r0:r1] . Ws */"),
    "rows_dx_concat_offset": ("memcpy(dX + t * I + r0, dXj + t * w, (size_t)w * sizeof(double));",
                              "memcpy(dX + t * I + (I - r0 - w), dXj + t * w, (size_t)w * sizeof(double));"),
    "rows_dw_scatter_row": ("osdp_oracle_locate(I, O, N, r0 + r, c, &s, &off);\n        dW_shards[s][off] = dWj[r * O + c];",
                            "osdp_oracle_locate(I, O, N, r0 + r, c, &s, &off);\n        dW_shards[s][off] = dWj[((r + 1) % w) * O + c];"),
    "mixed_dp_gradient_goes_to_shards": ("        if (zdp) {\n          int64_t s, off;", "        if (1) {\n          int64_t s, off;"),
    "mixed_fwd_concat_offset": ("memcpy(Y + t * O + a0, Yj + t * w, (size_t)w * sizeof(double));",
                                "memcpy(Y + t * O + (O - a0 - w), Yj + t * w, (size_t)w * sizeof(double));"),
    "mixed_dp_gradient_reversed": ("dw_dp[j][r * ld_dp + c] = dWj[r * sc + c];", "dw_dp[j][r * ld_dp + c] = dWj[r * sc + (sc - 1 - c)];"),
    "widen_drops_sign": ("uint32_t u = ((uint32_t)b) << 16;", "uint32_t u = ((uint32_t)(b & 0x7fff)) << 16;"),
    "sample_dw_short_sum": ("    for (int64_t t = 0; t < T; ++t)\n      acc += osdp_oracle_bf16_to_f64(X[t * I + i]) * osdp_oracle_bf16_to_f64(dY[t * O + o]);",
                            "    for (int64_t t = 1; t < T; ++t)\n      acc += osdp_oracle_bf16_to_f64(X[t * I + i]) * osdp_oracle_bf16_to_f64(dY[t * O + o]);"),
}


def _run_pins(lib: Path):
    env = dict(os.environ, OSDP_ORACLE_LIB=str(lib))
    return subprocess.run([sys.executable, "-m", "pytest", str(ROOT / "tests" / "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)


def _build(src: str, out: Path):
    c = out.with_suffix(".c")
    c.write_text(src)
    subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-std=c11", "-o", str(out), str(c)],
                   check=True)
    return out


def test_unmutated_copy_passes(tmp_path):
    res = _run_pins(_build(SRC, tmp_path / "liboracle_copy.so"))
    assert res.returncode == 0, res.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(tmp_path, name):
    old, new = MUTANTS[name]
    assert SRC.count(old) == 1, f"mutation site of {name} not found exactly once"
    res = _run_pins(_build(SRC.replace(old, new), tmp_path / f"liboracle_{name}.so"))
    assert res.returncode != 0, f"the pins did not notice the planted mistake {name!r}"
    assert "failed" in res.stdout, res.stdout[-2000:]  # an assertion failed; the child did not crash
