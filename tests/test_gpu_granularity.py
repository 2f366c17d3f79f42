"""GPU side of the automatic slice granularity: every candidate is run and timed through the C ABI, the
results it leaves are checked against the oracle, and the selection on the measured table against the
oracle's rule."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import gpu_harness
    return gpu_harness


def _measure(H, d, O, k_list, warmup, reps):
    import paper_2209_13258_amd as osdp
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    cands = osdp.osdp_granularity_candidates(op.T, op.I, O, op.N, k_list)
    ws = torch.empty(max(c.workspace for c in cands), dtype=torch.uint8, device="cuda")
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        osdp.osdp_granularity_measure(op.X, op.dY, op.W, op.Y, op.dX, op.dW, ws, cands, warmup=warmup, reps=reps,
                                      stream_compute=sc, stream_copy=sp)
    sc.synchronize()
    return op, cands


def _check_selection(oracle, cands):
    import paper_2209_13258_amd as osdp
    table = [(c.peak_weight_staging, c.workspace, c.ms) for c in cands]
    assert all(ms > 0 for _, _, ms in table)
    full = max(p for p, _, _ in table)
    for sb in (0, full, full // 2, full // 4, full // 16):
        for wb in (0, max(w for _, w, _ in table), min(w for _, w, _ in table)):
            for slow in (0.0, 0.1, 1.0, 100.0):
                want = oracle.granularity_select(table, sb, wb, slow)
                if want is None:
                    with pytest.raises(osdp.OsdpError):
                        osdp.osdp_granularity_select(cands, sb, wb, slow)
                    continue
                got = osdp.osdp_granularity_select(cands, sb, wb, slow)
                assert got == want
                assert sb == 0 or cands[got].peak_weight_staging <= sb
                assert wb == 0 or cands[got].workspace <= wb
    # with no limit on time the least gathered weight wins; with no tolerance the fastest
    assert cands[osdp.osdp_granularity_select(cands, 0, 0, 1e9)].peak_weight_staging == min(p for p, _, _ in table)
    assert cands[osdp.osdp_granularity_select(cands, 0, 0, 0.0)].ms == min(ms for _, _, ms in table)
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_granularity_select(cands, 8, 0, 0.0)  # eight bytes of gathered weight: nothing fits


@pytest.mark.parametrize("T,I,O,N", [(1024, 512, 2048, 8), (300, 264, 528, 4)])
def test_measure_runs_every_candidate_and_leaves_valid_results(H, oracle, T, I, O, N):
    print("CASE granularity", T, I, O, N, flush=True)
    d = wl.small_case(51, T, I, O, N)
    op, cands = _measure(H, d, O, None, warmup=1, reps=2)
    assert len(cands) >= 9
    got = op.results()
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, got[name], ref[name])
    _check_selection(oracle, cands)


def test_config2_granularity_is_chosen_from_measurements(H, oracle):
    """Both operators of config 2 at full size: the measured table, the staging law and the selection."""
    import paper_2209_13258_amd as osdp
    w = wl.workload(2, 1)
    for n, o in enumerate(w.ops):
        print("CASE granularity config 2", o.name, flush=True)
        d = wl.operator_inputs(2, 0, n, w.T, o.I, o.O, w.N)
        op, cands = _measure(H, d, o.O, [1, 2, 4, 8], warmup=2, reps=5)
        for c in cands:
            law = oracle.peak_staging_bytes_rows if c.split_dim else oracle.peak_staging_bytes
            if c.staging != osdp.OSDP_STAGING_HALF:
                assert c.peak_weight_staging == law(o.I, o.O, c.k, 2 if c.staging == osdp.OSDP_STAGING_DOUBLE else 1, 2)
            else:
                assert c.peak_weight_staging == law(o.I, o.O, c.k, 1, 2)
        _check_selection(oracle, cands)
        g = np.random.default_rng(52 + n)
        got = op.results()
        r, c = g.integers(0, w.T, 20000), g.integers(0, o.O, 20000)
        H.assert_close("Y", got["Y"][r, c], oracle.sample_y(d["X"], d["W_shards"], o.O, r, c))
        r, c = g.integers(0, w.T, 20000), g.integers(0, o.I, 20000)
        H.assert_close("dX", got["dX"][r, c], oracle.sample_dx(d["dY"], d["W_shards"], o.I, r, c))
        r, c = g.integers(0, o.I, 20000), g.integers(0, o.O, 20000)
        H.assert_close("dW", got["dW"][r, c], oracle.sample_dw(d["X"], d["dY"], r, c))
