"""Cost model and execution-plan search (Section 3.1, Section 3.2, Algorithm 1): the oracle against hand-worked
values, closed forms and an independent knapsack solution; the library against the oracle's enumeration."""
import itertools

import numpy as np
import pytest

import paper_2209_13258_amd as osdp


# ------------------------------------------------------------------ cost model
def test_cost_model_worked_by_hand(oracle):
    """N = 4, alpha = 1, beta = 0.5, one operator with M_model = 100, M_act = 10, M_extra = 1, S = 16, gamma = 2, b = 3.
    DP : M = 100 + 3*10 + 1 = 131, T = 2*3*(1 + 16/4*0.5) + 3*2 = 24, per sample 8.
    ZDP: M = 100/4 + 31 = 56,      T = 3*3*3 + 6 = 33, per sample 11."""
    ops = [(100, 10, 1, 16, 2)]
    for f in (lambda m: oracle.cost_model(ops, 4, 1.0, 0.5, m, 3), lambda m: osdp.osdp_cost_model(ops, 4, 1.0, 0.5, 1e9, m, 3)):
        assert f([0]) == (131.0, 8.0)
        assert f([1]) == (56.0, 11.0)
    # two operators add up; a single worker (N = 1) communicates nothing and shards nothing
    ops2 = ops + [(40, 1, 0, 8, 1)]
    assert oracle.cost_model(ops2, 4, 1.0, 0.5, [0, 1], 3) == (131.0 + 10 + 3, (24 + 9 * 2 + 3) / 3)
    assert oracle.cost_model(ops2, 1, 1.0, 0.5, [1, 1], 2) == oracle.cost_model(ops2, 1, 1.0, 0.5, [0, 0], 2) == (163.0, 3.0)
    assert osdp.osdp_cost_model(ops2, 4, 1.0, 0.5, 0, [0, 1], 3) == oracle.cost_model(ops2, 4, 1.0, 0.5, [0, 1], 3)


def test_zdp_trades_memory_for_communication(oracle):
    """Section 3.1: ZDP divides the model states by N and adds one more collective (3 instead of 2 rounds of N-1 steps)."""
    g = np.random.default_rng(1)
    for _ in range(50):
        N = int(g.integers(2, 17))
        op = tuple(float(v) for v in g.integers(1, 1000, 5))
        a, bta, b = float(g.integers(0, 5)), float(g.integers(1, 5)) / 8, int(g.integers(1, 9))
        md, td = oracle.cost_model([op], N, a, bta, [0], b)
        mz, tz = oracle.cost_model([op], N, a, bta, [1], b)
        assert md - mz == pytest.approx(op[0] * (1 - 1 / N), rel=1e-12)
        assert (tz - td) * b == pytest.approx((N - 1) * (a + op[3] / N * bta), rel=1e-12)


# ---------------------------------------------------------------- plan search
def _same_optimum(oracle, ops, N, alpha, beta, limit, lib, want):
    """Several plans may be equally fast: the batch size and the time are unique, the plan only has to be valid,
    i.e. fit the memory limit and cost, by the oracle's model, what the library says it costs."""
    assert lib["b"] == want["b"]
    assert lib["time_per_sample"] == pytest.approx(want["time_per_sample"], rel=1e-12, abs=0)
    mem, t = oracle.cost_model(ops, N, alpha, beta, lib["modes"], lib["b"])
    assert mem <= limit
    assert (mem, t) == (lib["memory"], lib["time_per_sample"])


def _knapsack_best_time(ops, N, alpha, beta, limit, b):
    """Fastest total time at batch size b by dynamic programming (integer memory savings): start from all-DP and buy
    memory back by turning operators to ZDP, each at an extra (N-1)(alpha + S/N beta) of time."""
    rest = sum(m_model + b * m_act + m_extra for m_model, m_act, m_extra, s, gamma in ops)
    base = sum(2 * (N - 1) * (alpha + s / N * beta) + b * gamma for _, _, _, s, gamma in ops)
    need = rest - limit
    if need <= 0:
        return base
    gains = [m_model - m_model / N for m_model, *_ in ops]
    assert all(float(x).is_integer() for x in gains) and float(need).is_integer()
    gains, need = [int(x) for x in gains], int(need)
    extra = [(N - 1) * (alpha + s / N * beta) for _, _, _, s, _ in ops]
    INF = float("inf")
    dp = [0.0] + [INF] * need            # dp[c]: least extra time that saves at least c
    for gain, e in zip(gains, extra):
        new = dp[:]
        for c in range(need + 1):
            if dp[c] < INF:
                t = min(need, c + gain)
                new[t] = min(new[t], dp[c] + e)
        dp = new
    return None if dp[need] == INF else base + dp[need]


@pytest.mark.parametrize("seed", range(12))
def test_search_against_knapsack(oracle, seed):
    """For every batch size the search must reach the time an independent dynamic program reaches."""
    g = np.random.default_rng(100 + seed)
    n, N = int(g.integers(3, 9)), int(g.choice([2, 4, 8]))
    ops = [(float(N * g.integers(1, 40)), float(g.integers(0, 6)), float(g.integers(0, 4)), float(N * g.integers(1, 40)),
            float(g.integers(1, 8)) / 4) for _ in range(n)]
    alpha, beta = float(g.integers(0, 3)), float(g.integers(1, 4)) / 4
    all_dp = sum(o[0] + o[2] for o in ops)
    limit = float(int(all_dp * g.uniform(0.35, 0.9)))
    best = None
    for b in range(1, 200):
        t = _knapsack_best_time(ops, N, alpha, beta, limit, b)
        if t is None:
            break
        if best is None or t / b < best[0] - 1e-12:
            best = (t / b, b)
    got = oracle.plan_search(ops, N, alpha, beta, limit, b_max=200)
    lib = osdp.osdp_plan_search(ops, N, alpha, beta, limit, b_max=200)
    if best is None:
        assert got is None and lib is None
        return
    assert got["time_per_sample"] == pytest.approx(best[0], rel=1e-12) and got["b"] == best[1]
    mem, t = oracle.cost_model(ops, N, alpha, beta, got["modes"], got["b"])
    assert mem <= limit and t == got["time_per_sample"] and mem == got["memory"]
    _same_optimum(oracle, ops, N, alpha, beta, limit, lib, got)


def test_search_closed_forms(oracle):
    ops = [(100.0, 1.0, 0.0, 100.0, 0.5), (60.0, 2.0, 1.0, 60.0, 0.25), (10.0, 0.0, 0.0, 10.0, 0.125)]
    for f in (oracle.plan_search, osdp.osdp_plan_search):
        # no memory pressure: everything stays DP, and since the communication is paid once per step the
        # largest batch allowed wins
        r = f(ops, 8, 1.0, 0.5, 1e12, b_max=7)
        assert r["modes"] == [0, 0, 0] and r["b"] == 7
        # less memory than the sharded states alone: nothing fits, not even b = 1
        assert f(ops, 8, 1.0, 0.5, 20.0) is None
        # exactly enough for everything sharded at b = 1: all ZDP
        lim = sum(o[0] / 8 + o[1] + o[2] for o in ops)
        r = f(ops, 8, 1.0, 0.5, lim)
        assert r["modes"] == [1, 1, 1] and r["b"] == 1 and r["memory"] == lim
        # one worker: DP and ZDP cost the same, the tie goes to DP, the first in the search order
        r = f(ops, 1, 1.0, 0.5, 1e12, b_max=3)
        assert r["modes"] == [0, 0, 0]


def test_slices_get_their_own_modes(oracle):
    """Section 3.3, last paragraph: one big operator cut into 4 slices; the memory limit leaves room for three
    replicated slices, so the search keeps 3 in DP mode and shards 1 (a whole-operator choice would shard all)."""
    N, k = 8, 4
    big = (800.0, 0.0, 0.0, 800.0, 1.0)
    slices = [tuple(v / k for v in big)] * k
    limit = 3 * 200.0 + 200.0 / N          # three full slices and one shard of the fourth
    for f in (oracle.plan_search, osdp.osdp_plan_search):
        whole = f([big], N, 1.0, 0.01, limit, b_max=1)
        split = f(slices, N, 1.0, 0.01, limit, b_max=1)
        assert whole["modes"] == [1]
        assert sorted(split["modes"]) == [0, 0, 0, 1]   # which of the four equal slices is sharded is not unique
        # the extra latency terms of the four slices (8 or 9 more steps of alpha) are smaller than the saved
        # all-gather traffic only when alpha is small: here the finer plan is simply what fits
        assert split["memory"] == limit


@pytest.mark.parametrize("seed", range(40))
def test_library_search_matches_enumeration(oracle, seed):
    """Random small instances with integer-valued costs (many exact ties): same batch size, same time, a valid plan."""
    g = np.random.default_rng(seed)
    n, N = int(g.integers(1, 11)), int(g.choice([1, 2, 4, 8, 16]))
    ops = [tuple(float(v) for v in (g.integers(0, 30), g.integers(0, 4), g.integers(0, 3), g.integers(0, 30), g.integers(0, 5)))
           for _ in range(n)]
    alpha, beta = float(g.integers(0, 3)), float(g.integers(0, 3))
    total = sum(o[0] + o[1] + o[2] for o in ops)
    limit = float(g.integers(0, int(total) + 5))
    want = oracle.plan_search(ops, N, alpha, beta, limit, b_max=12)
    got = osdp.osdp_plan_search(ops, N, alpha, beta, limit, b_max=12)
    if want is None:
        assert got is None
        return
    _same_optimum(oracle, ops, N, alpha, beta, limit, got, want)
    assert osdp.osdp_cost_model(ops, N, alpha, beta, limit, got["modes"], got["b"]) == (got["memory"], got["time_per_sample"])


def test_library_search_on_a_model_sized_instance(oracle):
    """An embedding, 48 identical layers of 4 linears and a head: 2^194 plans; the result must fit, be proven optimal
    within the node budget, and no single change of mode may improve it (a necessary condition for the optimum)."""
    N, h = 8, 1024
    lin = lambda mult: (8.0 * mult * h * h * 2, float(h * 2 * 16 * mult), 0.0, float(mult * h * h * 2), 1e-6 * mult)
    ops = [lin(50)] + [lin(m) for _ in range(48) for m in (3, 1, 4, 4)] + [lin(50)]
    limit = sum(o[0] for o in ops) * 0.4
    r = osdp.osdp_plan_search(ops, N, 1e-5, 1e-10, limit, b_max=64)
    assert r is not None and r["exact"]
    mem, t = oracle.cost_model(ops, N, 1e-5, 1e-10, r["modes"], r["b"])
    assert mem <= limit and t == pytest.approx(r["time_per_sample"], rel=1e-12)
    for i in range(len(ops)):
        m2 = list(r["modes"])
        m2[i] ^= 1
        mem2, t2 = oracle.cost_model(ops, N, 1e-5, 1e-10, m2, r["b"])
        assert mem2 > limit or t2 >= t * (1 - 1e-12)


def test_bad_arguments():
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_plan_search([(1.0, 1.0, 1.0, -1.0, 1.0)], 4, 1.0, 1.0, 10.0)
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_plan_search([(1.0, 1.0, 1.0, 1.0, 1.0)], 0, 1.0, 1.0, 10.0)
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_cost_model([(1.0, 1.0, 1.0, 1.0, 1.0)], 4, 1.0, 1.0, 10.0, [2], 1)
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_cost_model([(1.0, 1.0, 1.0, 1.0, 1.0)], 4, 1.0, 1.0, 10.0, [0], 0)
