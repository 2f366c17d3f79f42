"""Automatic slice granularity (Section 4.3 leaves the choice open): the oracle's selection rule against the
paper's own curves and brute force, and the library's host-side functions against the oracle."""
import ctypes
import itertools
import json
from pathlib import Path

import numpy as np
import pytest

import paper_2209_13258_amd as osdp

GOLDEN = Path(__file__).resolve().parent / "golden"
MB = 1 << 20


def _fig7_table(h):
    """(peak MB, workspace = same, seconds as the time unit) for the figure's granularities of hidden size h."""
    g = json.loads((GOLDEN / "fig7_memory.json").read_text())
    gran = g["granularity"]
    return gran, [(m, m, t) for m, t in zip(g["mem_mb"][str(h)], g["time_s"][str(h)])]


# Picks worked out by hand from the values the slice-granularity figure of Section 4.3 prints
# (tests/golden/fig7_memory.json): (hidden size, memory budget in MB or 0, tolerated slowdown) -> granularity.
#  h = 768: memory is flat (72.8-73.7) and time only rises with the granularity -> no splitting, whatever the tolerance
#  h = 1024: granularity 4 costs 14 % time (0.037297 / 0.032728), 16 costs 73 % -> 0 at 5 %, 4 needs > 14 % ...
#  h = 8192: every time is within 1.3 % of the fastest (1.846749 at 4) -> at 5 % the least memory wins: 16 (2311.09)
#  h = 12288: fastest is 8 (4.814705); 16 is 1.4 % slower and 4.9 MB smaller -> 16 at 5 %, 8 at 0 %
FIG7_PICKS = [
    (768, 0, 0.05, 0), (768, 0, 10.0, 4),   # with no limit on time the least memory (72.79 at 4) wins
    (1024, 0, 0.05, 0), (1024, 0, 0.15, 4), (1024, 0, 0.21, 6), (1024, 0, 0.45, 8), (1024, 0, 1.0, 16),
    (1024, 90, 0.0, 4),                       # a budget of 90 MB rules out granularity 0 (105.01); fastest that fits
    (8192, 0, 0.05, 16), (8192, 0, 0.0, 4), (8192, 3100, 0.0, 4), (8192, 2600, 0.0, 16), (8192, 2600, 0.001, 16),
    (12288, 0, 0.05, 16), (12288, 0, 0.0, 8), (12288, 6000, 0.0, 8), (12288, 7000, 0.0, 8),
]


@pytest.mark.parametrize("h,budget,slow,expect", FIG7_PICKS)
def test_selection_rule_on_the_papers_curves(oracle, h, budget, slow, expect):
    gran, table = _fig7_table(h)
    assert gran[oracle.granularity_select(table, budget, 0, slow)] == expect


def test_selection_reproduces_the_papers_observation(oracle):
    """Small operators are best left unsplit, large ones want the finest granularity (Section 4.3)."""
    picks = {h: _fig7_table(h)[0][oracle.granularity_select(_fig7_table(h)[1], 0, 0, 0.05)] for h in (768, 1024, 8192, 12288)}
    assert picks == {768: 0, 1024: 0, 8192: 16, 12288: 16}


def test_selection_rule_against_brute_force(oracle):
    """The definition, checked property by property on small random tables with many ties."""
    g = np.random.default_rng(7)
    for trial in range(400):
        n = int(g.integers(1, 7))
        table = [(int(g.integers(1, 5)) * 100, int(g.integers(1, 5)) * 1000, float(g.integers(0, 4)) * 0.5) for _ in range(n)]
        sb, wb = int(g.integers(0, 5)) * 100, int(g.integers(0, 5)) * 1000
        slow = float(g.choice([0.0, 0.5, 1.0, 3.0]))
        got = oracle.granularity_select(table, sb, wb, slow)
        fits = [i for i, (p, w, ms) in enumerate(table) if ms > 0 and (sb == 0 or p <= sb) and (wb == 0 or w <= wb)]
        if not fits:
            assert got is None
            continue
        assert got in fits
        tmin = min(table[i][2] for i in fits)
        assert table[got][2] <= (1 + slow) * tmin
        for i in fits:
            if table[i][2] > (1 + slow) * tmin:
                continue
            # nothing admissible is better: less memory, or equal memory and faster, or equal both and earlier
            assert (table[i][0], table[i][2], i) >= (table[got][0], table[got][2], got)


def _as_cands(table):
    arr = (osdp.binding.osdp_granularity_candidate * len(table))()
    for c, (peak, ws, ms) in zip(arr, table):
        c.k, c.staging, c.split_dim, c.peak_weight_staging, c.workspace, c.ms = 1, 1, 0, int(peak), int(ws), float(ms)
    return arr


def test_library_selection_matches_the_oracle(oracle):
    g = np.random.default_rng(8)
    for trial in range(600):
        n = int(g.integers(1, 9))
        table = [(int(g.integers(1, 6)) * 4096, int(g.integers(1, 6)) * 65536, float(g.integers(0, 6)) * 0.25) for _ in range(n)]
        sb, wb = int(g.integers(0, 6)) * 4096, int(g.integers(0, 6)) * 65536
        slow = float(g.choice([0.0, 0.1, 0.5, 1.0, 4.0]))
        want = oracle.granularity_select(table, sb, wb, slow)
        if want is None:
            with pytest.raises(osdp.OsdpError) as e:
                osdp.osdp_granularity_select(_as_cands(table), sb, wb, slow)
            assert e.value.status == osdp.binding.OSDP_ERR_UNSUPPORTED
        else:
            assert osdp.osdp_granularity_select(_as_cands(table), sb, wb, slow) == want
    for h, budget, slow, expect in FIG7_PICKS:  # and on the paper's curves (MB and seconds scaled to integers of bytes / ms)
        gran, table = _fig7_table(h)
        scaled = [(round(m * 100), round(m * 100), t * 1e3) for m, _, t in table]
        assert gran[osdp.osdp_granularity_select(_as_cands(scaled), round(budget * 100), 0, slow)] == expect
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_granularity_select(_as_cands([(1, 1, 1.0)]), 0, 0, -0.5)


@pytest.mark.parametrize("T,I,O,N", [(8192, 1024, 4096, 8), (16384, 10240, 2560, 8), (300, 264, 528, 4), (64, 48, 40, 6)])
def test_candidates_are_exactly_what_the_kernels_take(oracle, T, I, O, N):
    """Every (k, split dimension, staging mode) whose slice bounds are multiples of 8 (halves: of 16 wide),
    once each, in the documented order, with the staging law of Section 3.3 as its peak."""
    ks = [1, 2, 3, 4, 6, 8, 12, 16]
    got = [(c.k, c.split_dim, c.staging, c.peak_weight_staging, c.workspace, c.ms)
           for c in osdp.osdp_granularity_candidates(T, I, O, N)]
    want = []
    for k in ks:
        for dim in (0, 1, 3):   # columns, rows, columns forward + rows backward (both sets of bounds must be taken)
            sets = [(O, oracle.slice_range)] * (dim != 1) + [(I, oracle.row_slice_range)] * (dim != 0)
            if any(k > length for length, _ in sets):
                continue
            bounds = [rng(length, k, j) for length, rng in sets for j in range(k)]
            if any(a % 8 or b % 8 for a, b in bounds):
                continue
            for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
                if k == 1 and (mode == osdp.OSDP_STAGING_DOUBLE or (mode == osdp.OSDP_STAGING_SINGLE and dim != 0)):
                    continue
                if mode == osdp.OSDP_STAGING_HALF and any((b - a) % 16 for a, b in bounds):
                    continue
                peak = 0
                for length, rng in sets:   # the larger of the passes' peaks
                    rows = rng is oracle.row_slice_range
                    law = oracle.peak_staging_bytes_rows if rows else oracle.peak_staging_bytes
                    widest = max(b - a for a, b in (rng(length, k, j) for j in range(k)))
                    other = O if rows else I
                    if mode == osdp.OSDP_STAGING_HALF:
                        peak = max(peak, 2 * (widest // 2) * other * 2)
                    else:
                        peak = max(peak, law(I, O, k, 2 if mode == osdp.OSDP_STAGING_DOUBLE else 1, 2))
                want.append((k, dim, mode, peak))
    assert [g[:4] for g in got] == want
    for k, dim, mode, peak, ws, ms in got:
        assert ms == 0.0
        plan = osdp.Plan([k], staging=mode, split_dim_per_op=[dim])
        assert ws == max(osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, b, plan)[0] for b in (False, True))
        assert ws >= peak
    # a caller's own list, in the caller's order; capacity smaller than the count only truncates
    mine = osdp.osdp_granularity_candidates(T, I, O, N, [8, 1])
    assert [c.k for c in mine] == sorted([c.k for c in mine], reverse=True) and {c.k for c in mine} <= {8, 1}
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_granularity_candidates(T, I, O, N, [0])


def test_measure_rejects_bad_arguments_before_launching():
    import torch
    if torch.cuda.is_available():
        pytest.skip("uses made-up device addresses: only run where nothing can be launched")
    from test_host_api import _FakeTensor
    T, I, O, N = 128, 256, 1024, 2
    cands = osdp.osdp_granularity_candidates(T, I, O, N, [1, 4])
    need = max(c.workspace for c in cands)
    X, dY = _FakeTensor(0x10000, (T, I)), _FakeTensor(0x20000, (T, O))
    Y, dX = _FakeTensor(0x30000, (T, O)), _FakeTensor(0x40000, (T, I))
    sh = [_FakeTensor(0x50000, (I * O // N,)), _FakeTensor(0x60000, (I * O // N,))]
    with pytest.raises(osdp.OsdpError) as e:   # workspace too small for the largest candidate
        osdp.osdp_granularity_measure(X, dY, sh, Y, dX, sh, _FakeTensor(0x70000, (need - 1,), elem=1), cands)
    assert e.value.status == osdp.binding.OSDP_ERR_WORKSPACE
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_granularity_measure(X, dY, sh, Y, dX, sh, _FakeTensor(0x70000, (need,), elem=1), cands, reps=0)
    assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG
