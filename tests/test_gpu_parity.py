"""GPU parity: libosdp (HIP, through the C ABI) against the CPU oracle, element by element."""
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


def _announce(*what):
    print("CASE", *what, flush=True)


# ------------------------------------------------------------------- gather
@pytest.mark.parametrize("I,O,N,k", [
    (256, 1024, 2, 4),      # config 1
    (64, 96, 4, 3),         # row-block shards, 32-column slices
    (40, 48, 6, 2),         # N does not divide I: general flat map (L = 320)
    (24, 64, 64, 8),        # many tiny shards, L = 24: a slice row spans several shards
    (1024, 4096, 8, 8),     # config 2 up
    (520, 264, 8, 1),       # unsplit, ragged sizes
])
def test_gather_slice_bit_exact(H, oracle, I, O, N, k):
    _announce("gather", I, O, N, k)
    import paper_2209_13258_amd as osdp
    d = wl.small_case(11, 8, I, O, N)
    shards = [H.to_dev(s) for s in d["W_shards"]]
    for j in range(max(k, 1)):
        c0, c1 = oracle.slice_range(O, k, j)
        stg = torch.full((I * (c1 - c0) + 64,), float("nan"), dtype=torch.bfloat16, device="cuda")
        osdp.osdp_split_linear_gather_slice(I, O, k, j, shards, stg)
        torch.cuda.synchronize()
        got = H.to_bits(stg)
        ref = oracle.gather_slice(d["W_shards"], I, O, k, j)
        assert np.array_equal(got[: ref.size].reshape(ref.shape), ref)
        assert (got[ref.size:] == 0x7FC0).all()  # nothing written past the slice


# -------------------------------------------------- full compare, small sizes
SMALL = [
    # T, I, O, N, k
    (128, 256, 1024, 2, 4),   # config 1
    (300, 264, 528, 4, 3),    # ragged in every dimension, several tiles
    (77, 136, 200, 1, 1),     # unsplit, smaller than one tile in T
    (513, 384, 640, 8, 5),    # 128-column slices, T one past a tile edge
    (200, 72, 1040, 5, 2),    # general flat shard map (N does not divide I)
    (64, 512, 64, 8, 8),      # 8-column slices: narrower than any MFMA block
    (1, 8, 8, 1, 1),          # smallest legal problem
]


@pytest.mark.parametrize("T,I,O,N,k", SMALL)
def test_fwd_bwd_match_oracle(H, oracle, T, I, O, N, k):
    _announce("small", T, I, O, N, k)
    d = wl.small_case(12, T, I, O, N) if (T, I, O) != (128, 256, 1024) else \
        wl.operator_inputs(1, 0, 0, T, I, O, N)
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    op.fwd(k)
    op.bwd(k)
    got = op.results()
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    for name in ("Y", "dX", "dW"):
        H.assert_close(f"{name} T{T} I{I} O{O} N{N} k{k}", got[name], ref[name])
    # split route of the oracle agrees too (it is the same numbers by another road)
    Ys, _ = oracle.split_fwd(d["X"], d["W_shards"], O, k)
    H.assert_close("Y vs split route", got["Y"], Ys)


def test_shard_padding_is_never_touched(H, oracle):
    import paper_2209_13258_amd as osdp
    with pytest.raises(osdp.OsdpError):  # L = ceil(1920 / 7) = 275 is not a multiple of 8
        osdp.osdp_split_linear_workspace_bytes(40, 40, 48, 7, 2, True)
    # 40 x 24 = 960 weights over N = 11 shards: L = 88, the last shard ends in 8 elements of padding
    T, I, O, N, k = 33, 40, 24, 11, 3
    d = wl.small_case(13, T, I, O, N)
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    op.fwd(k)
    op.bwd(k)
    got = op.results()
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, got[name], ref[name])
    pad = H.to_bits(op.dW[-1])[I * O - (N - 1) * op.L:]
    assert pad.size == 8 and (pad == 0x7FC0).all()  # gradient padding left as it was


# ------------------------------------------ bit identity across k and modes
@pytest.mark.parametrize("pair", ["0", "1"])
@pytest.mark.parametrize("T,I,O,N", [(300, 264, 640, 4), (128, 256, 1024, 2), (1024, 512, 2048, 8),
                                     (256, 256, 640, 4)])  # last: k=1 takes the unchecked kernel, k=2 (320 columns) the checked one
def test_split_is_bit_identical_to_unsplit(H, T, I, O, N, pair, monkeypatch):
    """Every k, staging mode and stream choice; forward both with one launch per slice and with
    two staged slices per launch (the library's own choice is an estimate, so both are forced here)."""
    _announce("bit-identity", T, I, O, N, "pair", pair)
    monkeypatch.setenv("OSDP_FWD_PAIR", pair)
    import paper_2209_13258_amd as osdp
    d = wl.small_case(14, T, I, O, N)
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    op.fwd(1)
    op.bwd(1)
    base = op.results()
    sc, sp = H.streams()
    for k in (0, 2, 4, 5, 8, 16):
        if O % max(k, 1) or (O // max(k, 1)) % 8:
            continue
        for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
            if mode == osdp.OSDP_STAGING_HALF and (O // max(k, 1)) % 16:
                continue
            for two_streams in (False, True):
                plan = osdp.Plan([k], staging=mode)
                op2 = H.Operator(d["X"], d["dY"], d["W_shards"], O)
                torch.cuda.synchronize()
                with torch.cuda.stream(sc):
                    st = (sc, sp) if two_streams else (sc, None)
                    op2.fwd(k, plan=plan, streams=st)
                    op2.bwd(k, plan=plan, streams=st)
                sc.synchronize()  # the contract: the compute stream alone
                got = {"Y": H.to_bits(op2.Y), "dX": H.to_bits(op2.dX),
                       "dW": np.concatenate([H.to_bits(s) for s in op2.dW])[: I * O].reshape(I, O)}
                tag = f"k={k} mode={mode} two_streams={two_streams}"
                assert np.array_equal(got["Y"], base["Y"]), f"Y differs from k=1 ({tag})"
                assert np.array_equal(got["dW"], base["dW"]), f"dW differs from k=1 ({tag})"
                width = O // max(k, 1) // (2 if mode == osdp.OSDP_STAGING_HALF else 1)
                if width % 16 == 0:  # the fp32 partial sum is carried through the MFMA accumulator
                    assert np.array_equal(got["dX"], base["dX"]), f"dX differs from k=1 ({tag})"


def test_repeated_calls_reuse_workspace_safely(H, oracle):
    """Back-to-back operators sharing one workspace and both streams (the stack of a layer)."""
    import paper_2209_13258_amd as osdp
    shapes = [(256, 128, 384, 4, 3), (256, 384, 128, 4, 2), (256, 128, 512, 4, 4)]
    ops, data = [], []
    for n, (T, I, O, N, k) in enumerate(shapes):
        d = wl.small_case(20 + n, T, I, O, N)
        data.append(d)
        ops.append(H.Operator(d["X"], d["dY"], d["W_shards"], O))
    need = 0
    for (T, I, O, N, k) in shapes:
        need = max(need, osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, True)[0])
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        for rep in range(3):
            for op, (T, I, O, N, k) in zip(ops, shapes):
                op.ws = ws
                op.fwd(k, streams=(sc, sp))
            for op, (T, I, O, N, k) in reversed(list(zip(ops, shapes))):
                op.bwd(k, streams=(sc, sp))
    sc.synchronize()
    for op, d, (T, I, O, N, k) in zip(ops, data, shapes):
        got = op.results()
        ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
        for name in ("Y", "dX", "dW"):
            H.assert_close(name, got[name], ref[name])


# ------------------------------------------------ full-size configs, sampled
def _sampled_check(H, oracle, cfg, op_index, op, T, N, k, plan=None, n_samples=100_000, layer=0):
    I, O = op.I, op.O
    _announce("config", cfg, op.name, T, I, O, N, k)
    d = wl.operator_inputs(cfg, layer, op_index, T, I, O, N)
    dev = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        dev.fwd(k, plan=plan, streams=(sc, sp))
        dev.bwd(k, plan=plan, streams=(sc, sp))
    sc.synchronize()
    got = dev.results()
    g = np.random.default_rng(cfg * 1000 + op_index)
    keff = max(k, 1)
    # random entries plus entries that straddle slice and shard boundaries
    edges_o = np.unique(np.clip(np.concatenate([[j * O // keff + e for e in (-1, 0, 1)] for j in range(keff + 1)]), 0, O - 1))
    edges_i = np.unique(np.clip(np.concatenate([[s * I // N + e for e in (-1, 0, 1)] for s in range(N + 1)]), 0, I - 1))
    edges_t = np.unique(np.clip(np.array([0, 1, 127, 128, 255, 256, T - 2, T - 1]), 0, T - 1))

    def pairs(n0, n1, e0, e1):
        r = np.concatenate([g.integers(0, n0, n_samples), np.repeat(e0, e1.size)])
        c = np.concatenate([g.integers(0, n1, n_samples), np.tile(e1, e0.size)])
        return r, c

    r, c = pairs(T, O, edges_t, edges_o)
    ref = oracle.sample_y(d["X"], d["W_shards"], O, r, c)
    _sample_close(H, f"cfg{cfg} {op.name} Y", got["Y"][r, c], ref)
    r, c = pairs(T, I, edges_t, edges_i)
    ref = oracle.sample_dx(d["dY"], d["W_shards"], I, r, c)
    _sample_close(H, f"cfg{cfg} {op.name} dX", got["dX"][r, c], ref)
    r, c = pairs(I, O, edges_i, edges_o)
    ref = oracle.sample_dw(d["X"], d["dY"], r, c)
    _sample_close(H, f"cfg{cfg} {op.name} dW", got["dW"][r, c], ref)
    # properties that hold at any size: nothing left unwritten (outputs were NaN-poisoned)
    for name in ("Y", "dX", "dW"):
        assert not np.isnan(H.widen(got[name][:: max(1, got[name].shape[0] // 512)])).any(), f"{name} has unwritten entries"
    return dev, got


def _sample_close(H, name, got_bits, ref):
    H.assert_close(name, got_bits, ref)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_config2_ffn_pair(H, oracle, k):
    w = wl.workload(2, k)
    for n, op in enumerate(w.ops):
        _sampled_check(H, oracle, 2, n, op, w.T, w.N, k)


def test_config3_layer_with_plan(H, oracle):
    import paper_2209_13258_amd as osdp
    w = wl.workload(3)
    plan = osdp.Plan([op.k for op in w.ops])
    for n, op in enumerate(w.ops):
        _sampled_check_plan(H, oracle, 3, n, op, w, plan)


def _sampled_check_plan(H, oracle, cfg, n, op, w, plan):
    """Runs operator n under the plan vector (k taken from plan.k_per_op[n])."""
    import paper_2209_13258_amd as osdp
    I, O = op.I, op.O
    _announce("config", cfg, op.name, w.T, I, O, w.N, "plan", plan.k_per_op)
    d = wl.operator_inputs(cfg, 0, n, w.T, I, O, w.N)
    dev = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        dev.fwd(0, plan=plan, op_index=n, streams=(sc, sp))
        dev.bwd(0, plan=plan, op_index=n, streams=(sc, sp))
    sc.synchronize()
    got = dev.results()
    g = np.random.default_rng(cfg * 1000 + n)
    ns = 50_000
    r, c = g.integers(0, w.T, ns), g.integers(0, O, ns)
    H.assert_close(f"cfg{cfg} {op.name} Y", got["Y"][r, c], oracle.sample_y(d["X"], d["W_shards"], O, r, c))
    r, c = g.integers(0, w.T, ns), g.integers(0, I, ns)
    H.assert_close(f"cfg{cfg} {op.name} dX", got["dX"][r, c], oracle.sample_dx(d["dY"], d["W_shards"], I, r, c))
    r, c = g.integers(0, I, ns), g.integers(0, O, ns)
    H.assert_close(f"cfg{cfg} {op.name} dW", got["dW"][r, c], oracle.sample_dw(d["X"], d["dY"], r, c))
    # the plan's k must have been used: peak staging = 2 slots of |W| / k (or one slot when k = 1)
    k = plan.k_per_op[n]
    _, peak = osdp.osdp_split_linear_workspace_bytes(w.T, I, O, w.N, 0, True, plan, n)
    assert peak == oracle.peak_staging_bytes(I, O, k, 2, 2)


@pytest.mark.parametrize("k", [4, 16])
def test_config4_wide_operator(H, oracle, k):
    import paper_2209_13258_amd as osdp
    w = wl.workload(4, k)
    for n, op in enumerate(w.ops):
        _sampled_check(H, oracle, 4, n, op, w.T, w.N, k, n_samples=20_000)
        for slots, mode in ((1, osdp.OSDP_STAGING_SINGLE), (2, osdp.OSDP_STAGING_DOUBLE), (1, osdp.OSDP_STAGING_HALF)):
            _, peak = osdp.osdp_split_linear_workspace_bytes(w.T, op.I, op.O, w.N, k, True, osdp.Plan([k], staging=mode))
            assert peak == oracle.peak_staging_bytes(op.I, op.O, k, slots, 2)  # size / granularity per live slice


def test_config5_layer_stack(H, oracle):
    """4 layers x 4 operators, forward in order then backward in reverse, one shared workspace."""
    import paper_2209_13258_amd as osdp
    w = wl.workload(5)
    plan = osdp.Plan([op.k for op in w.ops])
    need = max(osdp.osdp_split_linear_workspace_bytes(w.T, op.I, op.O, w.N, 0, True, plan, n)[0]
               for n, op in enumerate(w.ops))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    sc, sp = H.streams()
    devs, data = {}, {}
    for layer in range(w.layers):
        for n, op in enumerate(w.ops):
            _announce("config 5 inputs", layer, op.name)
            d = wl.operator_inputs(5, layer, n, w.T, op.I, op.O, w.N)
            dev = H.Operator(d["X"], d["dY"], d["W_shards"], op.O)
            dev.ws = ws
            devs[layer, n], data[layer, n] = dev, d
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        for layer in range(w.layers):
            for n in range(len(w.ops)):
                devs[layer, n].fwd(0, plan=plan, op_index=n, streams=(sc, sp))
        for layer in reversed(range(w.layers)):
            for n in reversed(range(len(w.ops))):
                devs[layer, n].bwd(0, plan=plan, op_index=n, streams=(sc, sp))
    sc.synchronize()
    g = np.random.default_rng(5)
    ns = 10_000
    for (layer, n), dev in devs.items():
        op, d = w.ops[n], data[layer, n]
        _announce("config 5 check", layer, op.name)
        got = dev.results()
        r, c = g.integers(0, w.T, ns), g.integers(0, op.O, ns)
        H.assert_close("Y", got["Y"][r, c], oracle.sample_y(d["X"], d["W_shards"], op.O, r, c))
        r, c = g.integers(0, w.T, ns), g.integers(0, op.I, ns)
        H.assert_close("dX", got["dX"][r, c], oracle.sample_dx(d["dY"], d["W_shards"], op.I, r, c))
        r, c = g.integers(0, op.I, ns), g.integers(0, op.O, ns)
        H.assert_close("dW", got["dW"][r, c], oracle.sample_dw(d["X"], d["dY"], r, c))


# ------------------------------ the split along W's rows (the reduction dimension of the forward product)
def _rows_plan(k, mode=0):
    import paper_2209_13258_amd as osdp
    return osdp.Plan([k], staging=mode, split_dim_per_op=[osdp.OSDP_SPLIT_IN_FEATURES])


@pytest.mark.parametrize("I,O,N,k", [
    (256, 1024, 2, 4),      # config 1
    (96, 64, 4, 3),         # row-block shards, a slice spans more than one shard
    (48, 40, 6, 2),         # N does not divide I: general flat map (L = 320), shard edges inside rows
    (64, 24, 64, 8),        # many tiny shards, L = 24: every row spans shards
    (4096, 1024, 8, 8),     # config 2 down
    (520, 264, 8, 1),       # unsplit, ragged sizes
])
def test_gather_row_slice_bit_exact(H, oracle, I, O, N, k):
    _announce("gather rows", I, O, N, k)
    import paper_2209_13258_amd as osdp
    d = wl.small_case(31, 8, I, O, N)
    shards = [H.to_dev(s) for s in d["W_shards"]]
    for j in range(max(k, 1)):
        r0, r1 = oracle.row_slice_range(I, k, j)
        stg = torch.full(((r1 - r0) * O + 64,), float("nan"), dtype=torch.bfloat16, device="cuda")
        osdp.osdp_split_linear_gather_row_slice(I, O, k, j, shards, stg)
        torch.cuda.synchronize()
        got = H.to_bits(stg)
        ref = oracle.gather_row_slice(d["W_shards"], I, O, k, j)
        assert ref.shape == (r1 - r0, O)
        assert np.array_equal(got[: ref.size].reshape(ref.shape), ref)
        assert (got[ref.size:] == 0x7FC0).all()  # nothing written past the slice


SMALL_ROWS = [
    # T, I, O, N, k
    (128, 256, 1024, 2, 4),   # config 1
    (300, 264, 528, 4, 3),    # ragged in every dimension, 88-row slices
    (77, 136, 200, 1, 1),     # unsplit
    (513, 640, 384, 8, 5),    # 128-row slices, T one past a tile edge
    (200, 1040, 72, 5, 2),    # general flat shard map
    (64, 64, 512, 8, 8),      # 8-row slices: half an MFMA K step
    (1, 8, 8, 1, 1),          # smallest legal problem
]


@pytest.mark.parametrize("T,I,O,N,k", SMALL_ROWS)
def test_row_split_fwd_bwd_match_oracle(H, oracle, T, I, O, N, k):
    _announce("small rows", T, I, O, N, k)
    d = wl.small_case(32, T, I, O, N) if (T, I, O) != (128, 256, 1024) else \
        wl.operator_inputs(1, 0, 0, T, I, O, N)
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    plan = _rows_plan(k)
    op.fwd(k, plan=plan)
    op.bwd(k, plan=plan)
    got = op.results()
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    for name in ("Y", "dX", "dW"):
        H.assert_close(f"{name} rows T{T} I{I} O{O} N{N} k{k}", got[name], ref[name])
    # the oracle's own row-split route (the scheme of Section 3.3 step by step)
    Ys, _ = oracle.split_fwd_rows(d["X"], d["W_shards"], O, k)
    H.assert_close("Y vs row-split route", got["Y"], Ys)
    dXs, dWs, _ = oracle.split_bwd_rows(d["X"], d["dY"], d["W_shards"], O, k)
    H.assert_close("dX vs row-split route", got["dX"], dXs)
    H.assert_close("dW vs row-split route", got["dW"], oracle.dense_from_f64_shards(dWs, I, O))


@pytest.mark.parametrize("pair", ["0", "1"])
@pytest.mark.parametrize("T,I,O,N", [(300, 640, 264, 4), (128, 1024, 256, 2), (1024, 2048, 512, 8),
                                     (256, 640, 256, 4)])  # last: k=1 takes the unchecked kernel, k=2 (320 rows) the checked one for dW
def test_row_split_is_bit_identical_to_unsplit(H, T, I, O, N, pair, monkeypatch):
    """dW and dX are concatenated, so they equal the unsplit result bit for bit for every k, staging mode,
    stream choice and launch grouping; Y is a sum carried in the fp32 accumulator and is bit-identical when
    the slice height is a multiple of the MFMA's 16-deep K step."""
    _announce("bit-identity rows", T, I, O, N, "pair", pair)
    monkeypatch.setenv("OSDP_FWD_PAIR", pair)
    import paper_2209_13258_amd as osdp
    d = wl.small_case(33, T, I, O, N)
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    op.fwd(1)
    op.bwd(1)
    base = op.results()
    sc, sp = H.streams()
    for k in (0, 2, 4, 5, 8, 16):
        if I % max(k, 1) or (I // max(k, 1)) % 8:
            continue
        for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
            if mode == osdp.OSDP_STAGING_HALF and (I // max(k, 1)) % 16:
                continue
            for two_streams in (False, True):
                plan = _rows_plan(k, mode)
                op2 = H.Operator(d["X"], d["dY"], d["W_shards"], O)
                torch.cuda.synchronize()
                with torch.cuda.stream(sc):
                    st = (sc, sp) if two_streams else (sc, None)
                    op2.fwd(k, plan=plan, streams=st)
                    op2.bwd(k, plan=plan, streams=st)
                sc.synchronize()
                got = {"Y": H.to_bits(op2.Y), "dX": H.to_bits(op2.dX),
                       "dW": np.concatenate([H.to_bits(s) for s in op2.dW])[: I * O].reshape(I, O)}
                tag = f"k={k} mode={mode} two_streams={two_streams}"
                assert np.array_equal(got["dW"], base["dW"]), f"dW differs from k=1 ({tag})"
                assert np.array_equal(got["dX"], base["dX"]), f"dX differs from k=1 ({tag})"
                height = I // max(k, 1) // (2 if mode == osdp.OSDP_STAGING_HALF else 1)
                if height % 16 == 0:
                    assert np.array_equal(got["Y"], base["Y"]), f"Y differs from k=1 ({tag})"
                else:
                    assert not np.isnan(H.widen(got["Y"])).any()


def test_mixed_split_dimensions_share_one_workspace(H, oracle):
    """A plan vector that cuts some operators by columns and some by rows, run as a stack on two streams."""
    import paper_2209_13258_amd as osdp
    shapes = [(256, 128, 384, 4), (256, 384, 128, 4), (256, 128, 512, 4), (256, 512, 128, 4)]
    plan = osdp.Plan([3, 2, 4, 4], split_dim_per_op=[0, 1, 1, 0])
    ops, data = [], []
    for n, (T, I, O, N) in enumerate(shapes):
        d = wl.small_case(40 + n, T, I, O, N)
        data.append(d)
        ops.append(H.Operator(d["X"], d["dY"], d["W_shards"], O))
    need = max(max(osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, b, plan, n)[0] for b in (False, True))
               for n, (T, I, O, N) in enumerate(shapes))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        for rep in range(2):
            for n, op in enumerate(ops):
                op.ws = ws
                op.fwd(0, plan=plan, op_index=n, streams=(sc, sp))
            for n, op in reversed(list(enumerate(ops))):
                op.bwd(0, plan=plan, op_index=n, streams=(sc, sp))
    sc.synchronize()
    for op, d, (T, I, O, N) in zip(ops, data, shapes):
        got = op.results()
        ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
        for name in ("Y", "dX", "dW"):
            H.assert_close(name, got[name], ref[name])


@pytest.mark.parametrize("k", [2, 4, 8])
def test_config2_ffn_pair_row_split(H, oracle, k):
    """Config 2 at full size with both operators cut along their input features."""
    import paper_2209_13258_amd as osdp
    w = wl.workload(2, k)
    for n, op in enumerate(w.ops):
        dev, _ = _sampled_check(H, oracle, 2, n, op, w.T, w.N, k, plan=_rows_plan(k))
        _, peak = osdp.osdp_split_linear_workspace_bytes(w.T, op.I, op.O, w.N, k, False, _rows_plan(k))
        assert peak == oracle.peak_staging_bytes_rows(op.I, op.O, k, 2, 2)


def test_config3_layer_with_row_split_plan(H, oracle):
    import paper_2209_13258_amd as osdp
    w = wl.workload(3)
    plan = osdp.Plan([op.k for op in w.ops], split_dim_per_op=[osdp.OSDP_SPLIT_IN_FEATURES] * len(w.ops))
    for n, op in enumerate(w.ops):
        _sampled_check_plan(H, oracle, 3, n, op, w, plan)
