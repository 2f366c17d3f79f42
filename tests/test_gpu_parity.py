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


DEBUG_DEFAULTS = {"persistent": -1, "split_k": -1, "four_wave": -1, "fused_gather": -1, "gemm_generic": 0, "tile": -1, "deep": -1, "split_launch": -1, "fwd_pair": -1, "poison_staging": 0}


@pytest.fixture
def debug():
    """Sets the library's process-wide debug switches for one test and puts them back afterwards."""
    import paper_2209_13258_amd as osdp
    touched = set()

    def set_option(name, value):
        touched.add(name)
        osdp.osdp_debug_option(name, int(value))

    yield set_option
    for name in touched:
        osdp.osdp_debug_option(name, DEBUG_DEFAULTS[name])


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
def test_split_is_bit_identical_to_unsplit(H, T, I, O, N, pair, debug):
    """Every k, staging mode and stream choice; forward both with one launch per slice and with
    two staged slices per launch (the library's own choice is an estimate, so both are forced here)."""
    _announce("bit-identity", T, I, O, N, "pair", pair)
    debug("fwd_pair", pair)
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
def _edge_entries(n, cuts):
    """Indices just below, at and just above every cut of [0, n), plus the corners of the first 256 x 256 tile
    and the last two entries."""
    e = [c + d for c in cuts for d in (-1, 0, 1)] + [0, 1, 127, 128, 255, 256, n - 2, n - 1]
    return np.unique(np.clip(np.array(e), 0, n - 1))


def _check_samples(H, oracle, label, d, got, T, I, O, N, k, rows, g, n_samples):
    """Random entries of Y, dX and dW plus every entry whose row / column lies at a slice, shard or tile edge
    paired with every such column / row (whole edge-by-edge blocks), each against the oracle's own dot product."""
    # rows: True = W cut along its rows, False = along its columns, None = columns forward and rows backward
    cuts_o = [] if rows is True else [j * O // k for j in range(k + 1)]
    cuts_i = [s * I // N for s in range(N + 1)] + ([j * I // k for j in range(k + 1)] if rows is not False else [])
    edges_o, edges_i, edges_t = _edge_entries(O, cuts_o), _edge_entries(I, cuts_i), _edge_entries(T, [])

    def pairs(n0, n1, e0, e1):
        r = np.concatenate([g.integers(0, n0, n_samples), np.repeat(e0, e1.size)])
        c = np.concatenate([g.integers(0, n1, n_samples), np.tile(e1, e0.size)])
        return r, c

    r, c = pairs(T, O, edges_t, edges_o)
    H.assert_close(f"{label} Y", got["Y"][r, c], oracle.sample_y(d["X"], d["W_shards"], O, r, c))
    r, c = pairs(T, I, edges_t, edges_i)
    H.assert_close(f"{label} dX", got["dX"][r, c], oracle.sample_dx(d["dY"], d["W_shards"], I, r, c))
    r, c = pairs(I, O, edges_i, edges_o)
    H.assert_close(f"{label} dW", got["dW"][r, c], oracle.sample_dw(d["X"], d["dY"], r, c))


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
    rows = plan is not None and _cuts_rows(plan, 0, I, O)
    if plan is not None and plan.split_dim_per_op is not None and plan.split_dim_per_op[0] == 3:   # OSDP_SPLIT_PER_PASS
        rows = None
    _check_samples(H, oracle, f"cfg{cfg} {op.name}", d, got, T, I, O, N, max(k, 1), rows, g, n_samples)
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


def _cuts_rows(plan, n, I, O):
    """Whether the plan cuts operator n along W's rows."""
    import paper_2209_13258_amd as osdp
    dim = plan.split_dim_per_op[n] if plan.split_dim_per_op is not None else osdp.OSDP_SPLIT_OUT_FEATURES
    return dim == osdp.OSDP_SPLIT_IN_FEATURES or (dim == osdp.OSDP_SPLIT_LONGER and I > O)


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
    rows = _cuts_rows(plan, n, I, O)
    _check_samples(H, oracle, f"cfg{cfg} {op.name}", d, got, w.T, I, O, w.N, max(plan.k_per_op[n], 1), rows, g, 50_000)
    # the plan's k must have been used: peak staging = 2 slots of |W| / k (or one slot when k = 1)
    k = plan.k_per_op[n]
    _, peak = osdp.osdp_split_linear_workspace_bytes(w.T, I, O, w.N, 0, True, plan, n)
    law = oracle.peak_staging_bytes_rows if rows else oracle.peak_staging_bytes
    assert peak == law(I, O, k, 2, 2)


def test_config3_layer_cut_along_the_longer_dimension(H, oracle):
    """The plan vector of config 3 with every operator cut along its longer weight dimension (columns for qkv and
    up, rows for down), the variant the benchmark reports beside the column slices."""
    import paper_2209_13258_amd as osdp
    w = wl.workload(3)
    plan = osdp.Plan([op.k for op in w.ops], split_dim_per_op=[osdp.OSDP_SPLIT_LONGER] * len(w.ops))
    for n, op in enumerate(w.ops):
        _sampled_check_plan(H, oracle, 3, n, op, w, plan)


@pytest.mark.parametrize("k", [4, 8, 16])
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
        _check_samples(H, oracle, f"cfg5 layer {layer} {op.name}", d, got, w.T, op.I, op.O, w.N, max(op.k, 1), False, g, ns)


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
def test_row_split_is_bit_identical_to_unsplit(H, T, I, O, N, pair, debug):
    """dW and dX are concatenated, so they equal the unsplit result bit for bit for every k, staging mode,
    stream choice and launch grouping; Y is a sum carried in the fp32 accumulator and is bit-identical when
    the slice height is a multiple of the MFMA's 16-deep K step."""
    _announce("bit-identity rows", T, I, O, N, "pair", pair)
    debug("fwd_pair", pair)
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
    plan = osdp.Plan([3, 2, 4, 4], split_dim_per_op=[0, osdp.OSDP_SPLIT_LONGER, 1, osdp.OSDP_SPLIT_LONGER])  # cols, rows (I > O), rows, rows
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


# ---------------------------------------------- every slice in its own mode (DP or ZDP)
POISON = 0x7FC0  # bf16 NaN


def _mixed_host_case(oracle, seed, T, I, O, N, k, mask, rows, full_layout, cfg=None):
    """Weights that differ between the two sources: the shards hold NaN wherever a DP slice lies, the replicas
    hold the values that count there.  Returns host arrays and `used`, the matrix the operator really applies."""
    d = wl.small_case(seed, T, I, O, N) if cfg is None else wl.operator_inputs(cfg[0], 0, cfg[1], T, I, O, N)
    W = np.concatenate(d["W_shards"])[: I * O].reshape(I, O).copy()
    other = np.random.default_rng(seed + 1000)
    keff = max(k, 1)
    rng = [(oracle.row_slice_range(I, k, j) if rows else oracle.slice_range(O, k, j)) for j in range(keff)]
    used = W.copy()
    ld = O if (rows or full_layout) else max(b - a for a, b in rng) + 8   # compact replicas padded by 8 columns
    w_dp = [None] * keff
    full = None
    for j, (a, b) in enumerate(rng):
        if (mask >> j) & 1:
            continue
        sl = (slice(a, b), slice(None)) if rows else (slice(None), slice(a, b))
        vals = wl.f32_to_bf16_bits((other.standard_normal(W[sl].shape) * 0.02).astype(np.float32))
        used[sl] = vals
        W[sl] = POISON
        if rows:
            w_dp[j] = vals.copy()
        elif full_layout:
            if full is None:
                full = np.full((I, O), POISON, dtype=np.uint16)
            full[sl] = vals
            w_dp[j] = (full, a)                  # a view into one full-layout copy, made on the device side
        else:
            buf = np.full((I, ld), POISON, dtype=np.uint16)
            buf[:, : b - a] = vals
            w_dp[j] = buf
    L = oracle.shard_len(I, O, N)
    flat = np.full(N * L, POISON, dtype=np.uint16)
    flat[: I * O] = W.reshape(-1)
    shards = [flat[s * L:(s + 1) * L].copy() for s in range(N)]
    return d, shards, w_dp, ld, rng, used, full


class _MixedDevice:
    def __init__(self, H, d, shards, w_dp, ld, rng, I, O, rows, full):
        self.op = H.Operator(d["X"], d["dY"], shards, O)
        self.ld, self.rng, self.rows = ld, rng, rows
        full_dev = H.to_dev(full.reshape(-1)) if full is not None else None
        full_grad = torch.full((I * O,), float("nan"), dtype=torch.bfloat16, device="cuda") if full is not None else None
        self.w_dp, self.dw_dp = [], []
        for j, w in enumerate(w_dp):
            if w is None:
                self.w_dp.append(None)
                self.dw_dp.append(None)
            elif isinstance(w, tuple):
                self.w_dp.append(full_dev[w[1]:])
                self.dw_dp.append(full_grad[w[1]:])
            else:
                self.w_dp.append(H.to_dev(w.reshape(-1)))
                self.dw_dp.append(torch.full((w.size,), float("nan"), dtype=torch.bfloat16, device="cuda"))
        self.full_grad = full_grad

    def run(self, k, plan, streams=(None, None)):
        import paper_2209_13258_amd as osdp
        op = self.op
        ws, _ = op.workspace(k, True, plan)
        ws2, _ = op.workspace(k, False, plan)
        osdp.osdp_split_linear_fwd_mixed(op.X, op.W, self.w_dp, self.ld, op.Y, k, op.ws, plan=plan,
                                         stream_compute=streams[0], stream_copy=streams[1])
        osdp.osdp_split_linear_bwd_mixed(op.X, op.dY, op.W, self.w_dp, self.ld, op.dX, op.dW, self.dw_dp, k, op.ws,
                                         plan=plan, stream_compute=streams[0], stream_copy=streams[1])

    def gradient(self, H, I, O, mask):
        """(dense dW assembled from both destinations, what the shards hold inside DP slices, what the replicas'
        gradient arrays hold outside their slice)."""
        got = self.op.results()
        dW = got["dW"].copy()
        in_dp, outside = [], []
        for j, (a, b) in enumerate(self.rng):
            if (mask >> j) & 1:
                continue
            sl = (slice(a, b), slice(None)) if self.rows else (slice(None), slice(a, b))
            in_dp.append(dW[sl].copy().reshape(-1))
            h, w = (b - a, O) if self.rows else (I, b - a)
            buf = H.to_bits(self.dw_dp[j])
            need = (h - 1) * self.ld + w
            arr = np.full(h * self.ld, POISON, dtype=np.uint16)
            arr[:need] = buf[:need]
            arr = arr.reshape(h, self.ld)
            dW[sl] = arr[:, :w]
            if self.full_grad is None:
                outside.append(arr[:, w:].reshape(-1))
        return got, dW, in_dp, outside


MIXED_SMALL = [
    # T, I, O, N, k, zdp_mask
    (128, 256, 1024, 2, 4, 0b0001),    # the paper's example on config 1: one slice ZDP, three DP
    (300, 264, 528, 4, 3, 0b101),      # ragged everywhere
    (513, 384, 640, 8, 5, 0b01010),
    (200, 72, 1040, 5, 2, 0b00),       # every slice DP: nothing gathered at all
    (256, 512, 512, 4, 4, 0b0110),     # unchecked kernel, fusable pairs of one DP and one ZDP slice
    (77, 136, 200, 1, 1, 0b0),         # the whole operator in DP mode
]


@pytest.mark.parametrize("rows", [False, True])
@pytest.mark.parametrize("T,I,O,N,k,mask", MIXED_SMALL)
def test_per_slice_modes_match_oracle(H, oracle, T, I, O, N, k, mask, rows):
    import paper_2209_13258_amd as osdp
    if rows:
        I, O = O, I   # cut the long dimension either way
    _announce("mixed", T, I, O, N, k, bin(mask), "rows" if rows else "cols")
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    for full_layout in (False, True):
        d, shards, w_dp, ld, rng, used, full = _mixed_host_case(oracle, 61, T, I, O, N, k, mask, rows, full_layout)
        host_dp = [None if w is None else (full.reshape(-1)[w[1]:] if isinstance(w, tuple) else w) for w in w_dp]
        Y, peak = oracle.split_fwd_mixed(d["X"], shards, O, k, mask, host_dp, ld, rows=rows)
        dX, dWs, dw_ref, _ = oracle.split_bwd_mixed(d["X"], d["dY"], shards, O, k, mask, host_dp, ld, rows=rows)
        dW_ref = oracle.dense_from_f64_shards(dWs, I, O)
        for j, (a, b) in enumerate(rng):
            if not (mask >> j) & 1:
                sl = (slice(a, b), slice(None)) if rows else (slice(None), slice(a, b))
                h, w = (b - a, O) if rows else (I, b - a)
                dW_ref[sl] = dw_ref[j][:h, :w]
        for mode, two in ((osdp.OSDP_STAGING_SINGLE, False), (osdp.OSDP_STAGING_DOUBLE, True), (osdp.OSDP_STAGING_HALF, True)):
            if mode == osdp.OSDP_STAGING_HALF and any((b - a) % 16 for a, b in rng):
                continue
            plan = osdp.Plan([k], staging=mode, zdp_mask=[mask], split_dim_per_op=[dim])
            dev = _MixedDevice(H, d, shards, w_dp, ld, rng, I, O, rows, full)
            sc, sp = H.streams()
            torch.cuda.synchronize()
            with torch.cuda.stream(sc):
                dev.run(k, plan, streams=(sc, sp if two else None))
            sc.synchronize()
            got, dW, in_dp, outside = dev.gradient(H, I, O, mask)
            tag = f"mode {mode} full_layout {full_layout}"
            H.assert_close(f"Y {tag}", got["Y"], Y)
            H.assert_close(f"dX {tag}", got["dX"], dX)
            H.assert_close(f"dW {tag}", dW, dW_ref)
            for a in in_dp:
                assert (a == POISON).all(), "the sharded gradient was written inside a DP slice"
            for a in outside:
                assert (a == POISON).all(), "a DP gradient array was written outside its slice"
            # the gathered-weight peak counts ZDP slices only, and equals what the oracle's meter saw for one slot
            _, lib_peak = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, True,
                                                                 osdp.Plan([k], staging=osdp.OSDP_STAGING_SINGLE,
                                                                           zdp_mask=[mask], split_dim_per_op=[dim]))
            assert lib_peak == peak


@pytest.mark.parametrize("rows", [False, True])
@pytest.mark.parametrize("T,I,O,N,k", [(256, 512, 1024, 4, 4),
                                       (256, 16384, 1024, 4, 4)])  # column slices: the forward sums two parts of the reduction,
                                                                   # also in launches that read a DP and a ZDP slice
def test_per_slice_modes_are_bit_identical_to_all_zdp(H, oracle, rows, T, I, O, N, k):
    """With the replicas holding the same values as the shards, every mask gives the bits of the all-ZDP plan."""
    import paper_2209_13258_amd as osdp
    if rows:
        I, O = O, I
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    d = wl.small_case(62, T, I, O, N)
    base = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    plan0 = osdp.Plan([k], split_dim_per_op=[dim])
    base.fwd(k, plan=plan0)
    base.bwd(k, plan=plan0)
    ref = base.results()
    W = np.concatenate(d["W_shards"])[: I * O].reshape(I, O)
    rng = [(oracle.row_slice_range(I, k, j) if rows else oracle.slice_range(O, k, j)) for j in range(k)]
    for mask in (0b0000, 0b0001, 0b1010, 0b0111):
        _announce("mixed bit-identity", bin(mask), "rows" if rows else "cols")
        w_dp = [None if (mask >> j) & 1 else (W, a * O if rows else a) for j, (a, b) in enumerate(rng)]
        for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
            dev = _MixedDevice(H, d, d["W_shards"], w_dp, O, rng, I, O, rows, W)
            sc, sp = H.streams()
            torch.cuda.synchronize()
            with torch.cuda.stream(sc):
                dev.run(k, osdp.Plan([k], staging=mode, zdp_mask=[mask], split_dim_per_op=[dim]), streams=(sc, sp))
            sc.synchronize()
            got, dW, _, _ = dev.gradient(H, I, O, mask)
            assert np.array_equal(got["Y"], ref["Y"]), f"Y differs (mask {mask:04b}, mode {mode})"
            assert np.array_equal(got["dX"], ref["dX"]), f"dX differs (mask {mask:04b}, mode {mode})"
            assert np.array_equal(dW, ref["dW"]), f"dW differs (mask {mask:04b}, mode {mode})"


@pytest.mark.parametrize("rows", [False, True])
def test_config2_one_of_four_slices_zdp(H, oracle, rows):
    """The paper's example at full size (config 2, k = 4): one slice ZDP, three DP; sampled entries."""
    import paper_2209_13258_amd as osdp
    w = wl.workload(2, 4)
    k, mask = 4, 0b0100
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    for n, o in enumerate(w.ops):
        _announce("mixed config 2", o.name, "rows" if rows else "cols")
        d, shards, w_dp, ld, rng, used, full = _mixed_host_case(oracle, 63 + n, w.T, o.I, o.O, w.N, k, mask, rows, True,
                                                                cfg=(2, n))
        dev = _MixedDevice(H, d, shards, w_dp, ld, rng, o.I, o.O, rows, full)
        sc, sp = H.streams()
        torch.cuda.synchronize()
        with torch.cuda.stream(sc):
            dev.run(k, osdp.Plan([k], zdp_mask=[mask], split_dim_per_op=[dim]), streams=(sc, sp))
        sc.synchronize()
        got, dW, in_dp, _ = dev.gradient(H, o.I, o.O, mask)
        for a in in_dp:
            assert (a == POISON).all()
        used_shards = oracle.shard(used, w.N)   # the matrix the operator applies, for the oracle's entry sampler
        g = np.random.default_rng(64 + n)
        ns = 50_000
        r, c = g.integers(0, w.T, ns), g.integers(0, o.O, ns)
        H.assert_close("Y", got["Y"][r, c], oracle.sample_y(d["X"], used_shards, o.O, r, c))
        r, c = g.integers(0, w.T, ns), g.integers(0, o.I, ns)
        H.assert_close("dX", got["dX"][r, c], oracle.sample_dx(d["dY"], used_shards, o.I, r, c))
        r, c = g.integers(0, o.I, ns), g.integers(0, o.O, ns)
        H.assert_close("dW", dW[r, c], oracle.sample_dw(d["X"], d["dY"], r, c))
        _, peak = osdp.osdp_split_linear_workspace_bytes(w.T, o.I, o.O, w.N, k, True,
                                                         osdp.Plan([k], zdp_mask=[mask], split_dim_per_op=[dim]))
        law = oracle.peak_staging_bytes_rows if rows else oracle.peak_staging_bytes
        assert peak == law(o.I, o.O, k, 1, 2)   # one gathered slice, however many slots the mode offers


# ------------------------------------------------ every tile shape of the unchecked kernel
@pytest.mark.parametrize("T,I,O,N", [(512, 512, 768, 4), (256, 1024, 256, 8),
                                     (256, 192, 512, 4)])   # forward K = 192: the four-wave kernels' shortest K loop (3 blocks)
def test_every_tile_shape_gives_the_bits_of_the_checked_kernel(H, oracle, T, I, O, N, debug):
    """The host picks tile shapes by cost, so a test shape may never meet some of them: each of the four
    (with its own K block, LDS stage count and launch bounds per operand layout and pipeline depth) is forced in turn, for
    the unsplit operator and for splits in both dimensions, and must reproduce the bounds-checked kernel
    bit for bit (and, through it, the oracle)."""
    import paper_2209_13258_amd as osdp
    d = wl.small_case(71, T, I, O, N)
    debug("gemm_generic", 1)
    ref_op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    ref_op.fwd(1)
    ref_op.bwd(1)
    ref = ref_op.results()
    want = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, ref[name], want[name])
    debug("gemm_generic", 0)
    sc, sp = H.streams()
    # these shapes give every launch at most one tile per CU, where the library would use its deep-pipeline
    # variants of tiles 1..3 only: both pipelines of each tile are forced in turn
    # (tile 0 three times: on the eight-wave kernel, on the four-wave kernel also where the library would not pick it,
    # and on the four-wave kernel's persistent form, here with fewer workgroups than CUs and one tile each)
    for tile, deep, four_wave, persistent in (("0", "1", 0, -1), ("0", "1", 1, -1), ("0", "1", 1, 1), ("1", "0", -1, -1),
                                              ("1", "1", -1, -1), ("2", "0", -1, -1), ("2", "1", -1, -1),
                                              ("3", "0", -1, -1), ("3", "1", -1, -1)):
        debug("tile", tile)
        debug("deep", deep)
        debug("four_wave", four_wave)
        debug("persistent", persistent)
        for k, dim in ((1, 0), (2, 0), (2, 1)):
            _announce("tile", tile, "deep", deep, T, I, O, N, "k", k, "dim", dim)
            plan = osdp.Plan([k], staging=osdp.OSDP_STAGING_DOUBLE, split_dim_per_op=[dim])
            op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
            torch.cuda.synchronize()
            with torch.cuda.stream(sc):
                op.fwd(k, plan=plan, streams=(sc, sp))
                op.bwd(k, plan=plan, streams=(sc, sp))
            sc.synchronize()
            got = op.results()
            for name in ("Y", "dX", "dW"):
                assert np.array_equal(got[name], ref[name]), f"{name} differs (tile {tile}, k {k}, dim {dim})"


# ------------------------------------------------ the persistent form of the four-wave kernel
@pytest.mark.parametrize("dim", [0, 1])
def test_persistent_kernel_keeps_the_bits_of_one_tile_per_workgroup(H, oracle, debug, dim):
    """A launch of more 256 x 256 tiles than CUs runs as one workgroup per CU that walks through the tiles, the loads
    of a tile's first K blocks under way before the previous tile is stored.  272 and 289 tiles here: some
    workgroups run two tiles and most one.  With three slices every variant runs: the plain product, the three stages
    of a sum over slices (fp32 out, fp32 in and out, fp32 in), and dW into the shard-major layout.  Every bit must
    be the one that the kernel of one tile per workgroup gives, and the values the oracle's."""
    import paper_2209_13258_amd as osdp
    T, N, k = 4352, 8, 3
    I, O = (4352, 12288) if dim == 0 else (13056, 4096)
    d = wl.small_case(191 + dim, T, I, O, N)
    sc, sp = H.streams()

    def run(mode):
        plan = osdp.Plan([k], staging=mode, split_dim_per_op=[dim])
        op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
        torch.cuda.synchronize()
        osdp.osdp_profile_begin(1000)
        with torch.cuda.stream(sc):
            op.fwd(k, plan=plan, streams=(sc, sp))
            op.bwd(k, plan=plan, streams=(sc, sp))
        sc.synchronize()
        return op.results(), osdp.osdp_profile_end()["gemm_persistent"]["launches"]

    debug("tile", 0)           # (for 272 tiles the library would pick smaller tiles, or 256 large ones plus a remainder)
    debug("four_wave", 1)      # (dW reduces over T = 4352, where the library would still pick the eight-wave kernel)
    debug("persistent", 0)
    _announce("persistent off", T, I, O, N, k, dim)
    ref, n = run(osdp.OSDP_STAGING_SINGLE)
    assert n == 0
    g = np.random.default_rng(190 + dim)
    _check_samples(H, oracle, "one tile per workgroup", d, ref, T, I, O, N, k, bool(dim), g, 20_000)
    debug("persistent", -1)
    for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE):
        _announce("persistent on", T, I, O, N, k, dim, "staging", mode)
        got, n = run(mode)
        # SINGLE: a launch per slice for Y and for dX, and one for all of dW (which needs no weights); DOUBLE may
        # pair slices into launches of two K segments, which keep the plain kernel
        assert n == 7 if mode == osdp.OSDP_STAGING_SINGLE else n >= 3, f"{n} persistent launches"
        for name in ("Y", "dX", "dW"):
            assert np.array_equal(got[name], ref[name]), f"{name} differs (staging {mode})"
    debug("tile", -1)
    debug("four_wave", -1)
    _announce("persistent on, library's own launch plan", T, I, O, N, k, dim)
    got, n = run(osdp.OSDP_STAGING_DOUBLE)
    for name in ("Y", "dX", "dW"):
        assert np.array_equal(got[name], ref[name]), f"{name} differs (library's own launch plan)"


@pytest.mark.parametrize("I", [192, 256, 320])
def test_persistent_kernel_with_tiles_of_three_to_five_k_blocks(H, oracle, debug, I):
    """The loads run two K blocks ahead of the MFMAs: with three to five blocks per tile they are in the next tile
    most of the time, and the 16 workgroups that run two tiles cross a tile boundary in the prologue's shadow.
    Forward only (272 tiles of 256 x 256 with K = I), against the oracle element by element and bit for bit against
    one tile per workgroup."""
    import paper_2209_13258_amd as osdp
    T, O, N = 4352, 4096, 8
    d = wl.small_case(195, T, I, O, N)
    want = oracle.linear(d["X"], d["W_shards"], O, want=("Y",))
    debug("tile", 0)
    got = {}
    for persistent in (0, -1):
        debug("persistent", persistent)
        _announce("short K", T, I, O, "persistent", persistent)
        op = H.Operator(d["X"], None, d["W_shards"], O)
        sc, sp = H.streams()
        torch.cuda.synchronize()
        osdp.osdp_profile_begin(100)
        with torch.cuda.stream(sc):
            op.fwd(1, streams=(sc, sp))
        sc.synchronize()
        n = osdp.osdp_profile_end()["gemm_persistent"]["launches"]
        assert n == (1 if persistent else 0)
        got[persistent] = H.to_bits(op.Y)
        H.assert_close(f"Y (persistent {persistent})", got[persistent], want["Y"])
    assert np.array_equal(got[0], got[-1])


@pytest.mark.parametrize("rows", [False, True])
def test_persistent_kernel_reads_a_dp_and_a_gathered_slice_in_one_launch(H, oracle, debug, rows):
    """Launches over a DP slice (read in its replica, row length of the whole weight) and a gathered neighbour (in a
    staging slot, row length of the slice) hand the kernel two segments of B with different leading dimensions: by
    tile column where the launch concatenates, switched in the middle of every tile's K loop where it sums.  In the
    persistent form the switch happens on the load side, two K blocks ahead of the MFMAs and across tile
    boundaries.  Same bits as the all-gathered plan on one tile per workgroup."""
    import paper_2209_13258_amd as osdp
    T, I, O, N, k = 4352, 4096, 8192, 8, 4
    if rows:
        I, O = O, I
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    d = wl.small_case(193, T, I, O, N)
    debug("tile", 0)
    debug("four_wave", 1)
    debug("persistent", 0)
    base = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    plan0 = osdp.Plan([k], split_dim_per_op=[dim])
    base.fwd(k, plan=plan0)
    base.bwd(k, plan=plan0)
    ref = base.results()
    g = np.random.default_rng(193)
    _check_samples(H, oracle, "all gathered, one tile per workgroup", d, ref, T, I, O, N, k, rows, g, 10_000)
    debug("persistent", -1)
    debug("fwd_pair", 1)
    W = np.concatenate(d["W_shards"])[: I * O].reshape(I, O)
    rng = [(oracle.row_slice_range(I, k, j) if rows else oracle.slice_range(O, k, j)) for j in range(k)]
    for mask in (0b1010, 0b0110):
        _announce("persistent, DP and gathered slices", bin(mask), "rows" if rows else "cols")
        w_dp = [None if (mask >> j) & 1 else (W, a * O if rows else a) for j, (a, b) in enumerate(rng)]
        dev = _MixedDevice(H, d, d["W_shards"], w_dp, O, rng, I, O, rows, W)
        sc, sp = H.streams()
        torch.cuda.synchronize()
        osdp.osdp_profile_begin(1000)
        with torch.cuda.stream(sc):
            dev.run(k, osdp.Plan([k], staging=osdp.OSDP_STAGING_DOUBLE, zdp_mask=[mask], split_dim_per_op=[dim]), streams=(sc, sp))
        sc.synchronize()
        st = osdp.osdp_profile_end()
        n = st["gemm_persistent"]["launches"]
        # two launches over two slices each for Y and for dX, all of them persistent (dW: as the estimate cuts it)
        assert st["gemm_fwd"]["launches"] == 2 and st["gemm_dx"]["launches"] == 2 and n >= 4, \
            f"{st['gemm_fwd']['launches']} forward, {st['gemm_dx']['launches']} dX, {n} persistent launches"
        got, dW, _, _ = dev.gradient(H, I, O, mask)
        assert np.array_equal(got["Y"], ref["Y"]), f"Y differs (mask {mask:04b})"
        assert np.array_equal(got["dX"], ref["dX"]), f"dX differs (mask {mask:04b})"
        assert np.array_equal(dW, ref["dW"]), f"dW differs (mask {mask:04b})"


# ------------------------------------------------ leading dimensions and many shards
@pytest.mark.parametrize("T,I,O,N,k,dim", [(256, 256, 512, 4, 2, 0),     # unchecked kernels
                                            (77, 136, 200, 1, 1, 0),     # checked kernel
                                            (300, 264, 528, 4, 3, 1),    # row slices, ragged
                                            (128, 64, 192, 64, 3, 0)])   # 64 shards of 192 elements: rows span shards
def test_padded_leading_dimensions_and_many_shards(H, oracle, T, I, O, N, k, dim):
    """X, dY, Y and dX live inside wider arrays (ld > row length); the columns beyond the row length hold NaN and
    must neither be read (inputs) nor written (outputs)."""
    import paper_2209_13258_amd as osdp
    _announce("leading dimensions", T, I, O, N, k, dim)
    d = wl.small_case(81, T, I, O, N)
    pad_i, pad_o = 24, 40
    nan = float("nan")

    def widened(bits, pad):
        t = torch.full((bits.shape[0], bits.shape[1] + pad), nan, dtype=torch.bfloat16, device="cuda")
        t[:, : bits.shape[1]] = H.to_dev(bits)
        return t

    Xw, dYw = widened(d["X"], pad_i), widened(d["dY"], pad_o)
    Yw = torch.full((T, O + pad_o), nan, dtype=torch.bfloat16, device="cuda")
    dXw = torch.full((T, I + pad_i), nan, dtype=torch.bfloat16, device="cuda")
    X, dY, Y, dX = Xw[:, :I], dYw[:, :O], Yw[:, :O], dXw[:, :I]
    assert X.stride(0) == I + pad_i and Y.stride(0) == O + pad_o
    W = [H.to_dev(s) for s in d["W_shards"]]
    dW = [torch.full((d["W_shards"][0].size,), nan, dtype=torch.bfloat16, device="cuda") for _ in range(N)]
    plan = osdp.Plan([k], split_dim_per_op=[dim])
    need = max(osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, b, plan)[0] for b in (False, True))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        osdp.osdp_split_linear_fwd(X, W, Y, 0, ws, plan=plan, stream_compute=sc, stream_copy=sp)
        osdp.osdp_split_linear_bwd(X, dY, W, dX, dW, 0, ws, plan=plan, stream_compute=sc, stream_copy=sp)
    sc.synchronize()
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    H.assert_close("Y", H.to_bits(Yw)[:, :O], ref["Y"])
    H.assert_close("dX", H.to_bits(dXw)[:, :I], ref["dX"])
    got_dW = np.concatenate([H.to_bits(s) for s in dW])[: I * O].reshape(I, O)
    H.assert_close("dW", got_dW, ref["dW"])
    assert (H.to_bits(Yw)[:, O:] == POISON).all() and (H.to_bits(dXw)[:, I:] == POISON).all()


# ------------------------------------------------ capture into a HIP graph
@pytest.mark.parametrize("pair,persistent", [("0", -1), ("1", -1), ("1", 1)])
def test_calls_can_be_captured_into_a_graph_and_replayed(H, pair, persistent, debug):
    """A forward + backward captured on the compute stream (one-stream and two-stream pipelines, the latter with
    its cross-stream events inside the capture) replays to the bits of the eager calls, every time, with eager work
    and new inputs between the replays."""
    import paper_2209_13258_amd as osdp
    debug("fwd_pair", pair)   # "0": the forward overlaps gathers on the copy stream; "1": one stream
    debug("persistent", persistent)   # 1: the four-wave launches of this small shape run in their persistent form too
    T, I, O, N, k = 512, 2048, 4096, 8, 2       # 8 MB slices: the backward uses the copy stream too
    d = wl.small_case(91, T, I, O, N)
    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    plan = osdp.Plan([k], staging=osdp.OSDP_STAGING_DOUBLE)
    sc, sp = H.streams()

    def eager():
        with torch.cuda.stream(sc):
            op.fwd(k, plan=plan, streams=(sc, sp))
            op.bwd(k, plan=plan, streams=(sc, sp))
        sc.synchronize()
        return [op.Y.clone(), op.dX.clone()] + [s.clone() for s in op.dW]

    def poison():
        for t in [op.Y, op.dX] + op.dW:
            t.fill_(float("nan"))
        torch.cuda.synchronize()

    ref = eager()                                # also the warm-up that sets the kernels' attributes
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=sc):
        op.fwd(k, plan=plan, streams=(sc, sp))
        op.bwd(k, plan=plan, streams=(sc, sp))
    g = torch.Generator(device="cuda")
    g.manual_seed(92)
    for rep in range(3):
        _announce("graph replay", pair, persistent, rep)
        poison()
        graph.replay()
        torch.cuda.synchronize()
        got = [op.Y, op.dX] + op.dW
        for a, b in zip(got, ref):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {rep} differs from the eager result"
        # new inputs, eager work and synchronisations before the next replay
        op.X.copy_(torch.randn(op.X.shape, generator=g, device="cuda").to(torch.bfloat16))
        op.dY.copy_(torch.randn(op.dY.shape, generator=g, device="cuda").to(torch.bfloat16))
        torch.cuda.synchronize()
        ref = eager()


# ------------------------------------------------------------- no tokens at all
@pytest.mark.parametrize("rows", [False, True])
@pytest.mark.parametrize("I,O,N,k,mask", [(256, 512, 4, 4, 0b1111),   # shapes the unchecked kernels would take
                                          (264, 528, 4, 3, 0b111),    # ragged
                                          (256, 512, 4, 4, 0b0110),   # two of the four slices in DP mode
                                          (40, 24, 11, 1, 0b1)])      # general shard map with padding
def test_zero_tokens_leave_y_alone_and_zero_the_gradient(H, oracle, I, O, N, k, mask, rows):
    """T = 0: Y, dX are empty, and dW = X^T . dY is a sum over no tokens, i.e. zero - which the backward call must
    store (a gradient buffer is not assumed to be cleared), in the shards and in the DP slices' own arrays."""
    import paper_2209_13258_amd as osdp
    if rows:
        I, O = O, I
    _announce("zero tokens", I, O, N, k, bin(mask), "rows" if rows else "cols")
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    d, shards, w_dp, ld, rng, used, full = _mixed_host_case(oracle, 71, 0, I, O, N, k, mask, rows, False)
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    assert ref["Y"].shape == (0, O) and ref["dX"].shape == (0, I) and not ref["dW"].any()
    for mode, two in ((osdp.OSDP_STAGING_SINGLE, False), (osdp.OSDP_STAGING_DOUBLE, True)):
        plan = osdp.Plan([k], staging=mode, zdp_mask=[mask], split_dim_per_op=[dim])
        dev = _MixedDevice(H, d, shards, w_dp, ld, rng, I, O, rows, full)
        sc, sp = H.streams()
        torch.cuda.synchronize()
        with torch.cuda.stream(sc):
            dev.run(k, plan, streams=(sc, sp if two else None))
        sc.synchronize()
        got, dW, in_dp, outside = dev.gradient(H, I, O, mask)
        assert got["Y"].shape == (0, O) and got["dX"].shape == (0, I)
        assert dW.shape == (I, O) and (dW == 0).all()        # +0.0 everywhere: the bits of the oracle's zeros
        for a in in_dp:
            assert (a == POISON).all()
        for a in outside:
            assert (a == POISON).all()
        L = dev.op.L
        pad = H.to_bits(dev.op.dW[-1])[I * O - (N - 1) * L:]
        assert (pad == POISON).all()                         # shard padding untouched
    if mask == (1 << max(k, 1)) - 1:                         # the plain entry points take the same shape
        op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
        op.fwd(k)
        op.bwd(k)
        assert not op.results()["dW"].any()


# --------------------------------------- a weight whose flat index needs more than 32 bits
@pytest.mark.parametrize("N,rows", [(8, False),   # shards are row blocks; column slices, the last one gathered alone too
                                    (3, True)])   # N does not divide I: general flat map; row slices
def test_weight_of_more_than_2_to_32_elements(H, oracle, N, rows):
    """I x O = 32768 x 132096 = 4.33e9 weights (8.7 GB in bf16): every flat index past 2^31 and 2^32 must be formed
    in 64 bits by the gather, by the slice GEMMs' reads of an up to 2.2 GB staging slot and by the shard-major dW
    store.  The weights repeat with a period that divides neither power, so a wrapped index reads another value."""
    import paper_2209_13258_amd as osdp
    T, I, O, k = 256, 32768, 132096, 4
    _announce("wide index", T, I, O, N, k, "rows" if rows else "cols")
    d = wl.tiled_case(5, T, I, O, N, (1 << 24) + 8)
    dev = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    plan = osdp.Plan([k], split_dim_per_op=[dim])
    sc, sp = H.streams()
    torch.cuda.synchronize()
    with torch.cuda.stream(sc):
        dev.fwd(k, plan=plan, streams=(sc, sp))
        dev.bwd(k, plan=plan, streams=(sc, sp))
    sc.synchronize()
    got = dev.results()
    g = np.random.default_rng(4242 + N)
    ns = 4000
    # weight entries around flat index 2^31 and 2^32, the four corners, and random ones
    near = np.array([f + e for f in (1 << 31, 1 << 32, I * O - 1) for e in (-8, -1, 0)] + [0, O - 1, (I - 1) * O])
    wi = np.concatenate([g.integers(0, I, ns), near // O])
    wo = np.concatenate([g.integers(0, O, ns), near % O])
    H.assert_close("dW", got["dW"][wi, wo], oracle.sample_dw(d["X"], d["dY"], wi, wo))
    r = np.concatenate([g.integers(0, T, ns), np.full(near.size, T - 1)])
    c = np.concatenate([g.integers(0, O, ns), near % O])
    H.assert_close("Y", got["Y"][r, c], oracle.sample_y(d["X"], d["W_shards"], O, r, c))
    c = np.concatenate([g.integers(0, I, ns), near // O])
    H.assert_close("dX", got["dX"][r, c], oracle.sample_dx(d["dY"], d["W_shards"], I, r, c))
    for name in ("Y", "dX", "dW"):
        assert not np.isnan(H.widen(got[name][:: max(1, got[name].shape[0] // 512)])).any(), f"{name} has unwritten entries"
    if not rows:
        j = k - 1
        c0, c1 = oracle.slice_range(O, k, j)
        stg = torch.empty((I * (c1 - c0),), dtype=torch.bfloat16, device="cuda")
        osdp.osdp_split_linear_gather_slice(I, O, k, j, dev.W, stg)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_bits(stg).reshape(I, c1 - c0), oracle.gather_slice(d["W_shards"], I, O, k, j))


# ------------------------------------------------------------- calls from several host threads
def test_two_host_threads_call_concurrently(H, oracle):
    """Each thread drives its own operator, workspace and pair of streams; the bits must be those of the same
    calls made one after the other (the library keeps its cross-stream events per calling thread)."""
    import threading
    T, I, O, N, k = 512, 512, 2048, 4, 4
    _announce("threads", T, I, O, N, k)
    cases = [wl.small_case(80 + i, T, I, O, N) for i in range(2)]
    want = []
    for d in cases:
        op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
        sc, sp = H.streams()
        torch.cuda.synchronize()
        with torch.cuda.stream(sc):
            op.fwd(k, streams=(sc, sp))
            op.bwd(k, streams=(sc, sp))
        sc.synchronize()
        want.append(op.results())
    ref0 = oracle.linear(cases[0]["X"], cases[0]["W_shards"], O, dY=cases[0]["dY"])
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, want[0][name], ref0[name])
    ops = [H.Operator(d["X"], d["dY"], d["W_shards"], O) for d in cases]
    for op in ops:                       # workspaces allocated up front: the threads only enqueue
        op.workspace(k, True)
    streams = [H.streams() for _ in ops]
    torch.cuda.synchronize()
    errors = []

    def drive(op, sc, sp):
        try:
            with torch.cuda.stream(sc):
                for _ in range(20):
                    op.fwd(k, streams=(sc, sp))
                    op.bwd(k, streams=(sc, sp))
            sc.synchronize()
        except Exception as e:           # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=drive, args=(op, sc, sp)) for op, (sc, sp) in zip(ops, streams)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for op, ref in zip(ops, want):
        got = op.results()
        for name in ("Y", "dX", "dW"):
            assert np.array_equal(got[name], ref[name]), name


# ------------------------------------------------ one problem run as two launches
@pytest.mark.parametrize("T,I,O", [(4096, 256, 4352),    # forward: 16 x 17 large tiles, cut along the columns
                                   (256, 4352, 4096)])   # dW: 17 x 16 large tiles, cut along the rows (shard-major store)
def test_whole_rounds_plus_remainder_launches_keep_the_bits(H, oracle, T, I, O, debug):
    """A GEMM whose large tiles fill the CUs once plus a little is run as two launches (whole rounds, remainder):
    same bits as the single launch, and the oracle's values."""
    N = 8
    _announce("two launches", T, I, O, N)
    d = wl.small_case(91, T, I, O, N)
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    res = {}
    for flag in ("0", "1"):
        debug("split_launch", -1 if flag == "1" else 0)
        for k in (1, 2):
            op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
            op.fwd(k)
            op.bwd(k)
            res[flag, k] = op.results()
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, res["1", 1][name], ref[name])
        for k in (1, 2):
            assert np.array_equal(res["0", k][name], res["1", k][name]), f"{name} differs with two launches (k {k})"


# ------------------------------------------------ debug mode: poisoned staging slots
@pytest.mark.parametrize("fused", [-1, 0])
@pytest.mark.parametrize("pair", [0, 1])
@pytest.mark.parametrize("rows", [False, True])
def test_poisoned_staging_slots_change_nothing(H, oracle, rows, pair, fused, debug):
    """With the staging slots filled with NaN patterns whenever no gathered slice is live in them, a GEMM that ran
    ahead of its gather or a gather that landed on a slice still in use would put NaN (or wrong values) into the
    outputs: every staging mode, one and two streams, both forward schedules, gathers carried inside the GEMM launches
    and gathers as launches of their own, repeated calls on one workspace."""
    import paper_2209_13258_amd as osdp
    T, I, O, N = 512, 1024, 2048, 8
    d = wl.small_case(131, T, I, O, N)
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    base_op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    base_op.fwd(1)
    base_op.bwd(1)
    base = base_op.results()
    debug("poison_staging", 1)
    debug("fwd_pair", pair)
    debug("fused_gather", fused)
    sc, sp = H.streams()
    for k in (2, 4, 8):
        for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
            for streams in ((sc, sp), (sc, None)):
                _announce("poison", "rows" if rows else "columns", "pair", pair, "k", k, "mode", mode, "two streams", streams[1] is not None)
                plan = osdp.Plan([k], staging=mode, split_dim_per_op=[dim])
                op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
                torch.cuda.synchronize()
                with torch.cuda.stream(sc):
                    for _ in range(3):  # back to back on one workspace: the next call's gathers meet this call's GEMMs
                        op.fwd(k, plan=plan, streams=streams)
                        op.bwd(k, plan=plan, streams=streams)
                sc.synchronize()
                got = op.results()
                for name in ("Y", "dX", "dW"):
                    assert np.array_equal(got[name], base[name]), f"{name} differs from the unsplit result"
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, base[name], ref[name])


@pytest.mark.parametrize("T,I,O,N", [(512, 1024, 2304, 9),    # 9 shards do not divide 1024 rows: the general flat map
                                     (768, 2048, 1024, 8),    # row-block shards
                                     (256, 512, 1024, 64)])   # 64 shards of 8 rows
def test_gathers_carried_by_gemm_launches_match_the_gather_kernel(H, oracle, T, I, O, N, debug):
    """A GEMM launch on the large tile takes the next slice's gather along; the staged bytes, and so every result
    bit, must be those of the gather kernel: both split dimensions, every staging mode, k up to 4, against the
    unsplit result and the oracle.  The shapes keep every launch on the kernel that can carry a gather."""
    import paper_2209_13258_amd as osdp
    d = wl.small_case(141, T, I, O, N)
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    base_op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    base_op.fwd(1)
    base_op.bwd(1)
    base = base_op.results()
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, base[name], ref[name])
    sc, sp = H.streams()
    for fused in (-1, 0):
        debug("fused_gather", fused)
        for dim in (osdp.OSDP_SPLIT_OUT_FEATURES, osdp.OSDP_SPLIT_IN_FEATURES):
            for k in (2, 4):
                for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
                    _announce("carried gathers", T, I, O, N, "fused", fused, "dim", dim, "k", k, "mode", mode)
                    plan = osdp.Plan([k], staging=mode, split_dim_per_op=[dim])
                    op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
                    torch.cuda.synchronize()
                    with torch.cuda.stream(sc):
                        op.fwd(k, plan=plan, streams=(sc, sp))
                        op.bwd(k, plan=plan, streams=(sc, sp))
                    sc.synchronize()
                    got = op.results()
                    for name in ("Y", "dX", "dW"):
                        assert np.array_equal(got[name], base[name]), f"{name} differs from the unsplit result"


# ------------------------------------------------ forward products that run as parts of the reduction
@pytest.mark.parametrize("T,I,O,N", [(512, 32768, 1024, 8),    # four parts of 8192
                                     (300, 49152, 520, 4)])    # six parts; ragged T and slices: the checked kernel
def test_forward_parts_of_a_long_reduction_keep_the_bits_for_every_k_and_kernel(H, oracle, T, I, O, N, debug):
    """Few tokens and a long reduction: the forward product is the sum of 8192-long parts, each computed into an fp32
    plane of its own and added in order.  The number of parts depends on T and I alone, so Y keeps the unsplit
    operator's bits for every k, staging mode, pairing, tile shape and kernel; against the oracle it stays within the
    tolerance, as does the one-part product (switch off), whose bits differ."""
    import paper_2209_13258_amd as osdp
    d = wl.small_case(151, T, I, O, N)
    want = oracle.linear(d["X"], d["W_shards"], O, want=("Y",))
    parts = I // 8192
    tot_on = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, False)[0]
    debug("split_k", 0)
    tot_off = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, False)[0]
    one = H.Operator(d["X"], None, d["W_shards"], O)
    one.fwd(1)
    torch.cuda.synchronize()
    one_part = H.to_bits(one.Y)
    H.assert_close("Y (one part)", one_part, want["Y"])
    debug("split_k", -1)
    assert tot_on - tot_off == parts * T * O * 4   # the planes of the unsplit operator's one launch
    base_op = H.Operator(d["X"], None, d["W_shards"], O)
    base_op.fwd(1)
    torch.cuda.synchronize()
    base = H.to_bits(base_op.Y)
    H.assert_close("Y", base, want["Y"])
    assert not np.array_equal(base, one_part)   # the parts are really summed separately
    sc, sp = H.streams()
    fast = T % 128 == 0 and O % 128 == 0
    settings = [dict()] + ([dict(tile=t, four_wave=f) for t, f in ((0, 0), (0, 1), (1, -1), (2, -1), (3, -1))] +
                           [dict(tile=0, four_wave=1, persistent=1)] if fast else []) \
        + [dict(gemm_generic=1)]
    for setting in settings:
        for name, value in setting.items():
            debug(name, value)
        for k in (1, 2, 4, 8):
            if O % k or (O // k) % 8:
                continue
            for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
                if mode == osdp.OSDP_STAGING_HALF and (O // k) % 16:
                    continue
                for pair in (0, 1):
                    if mode != osdp.OSDP_STAGING_DOUBLE and pair:
                        continue
                    debug("fwd_pair", pair)
                    _announce("forward parts", T, I, O, N, setting, "k", k, "mode", mode, "pair", pair)
                    plan = osdp.Plan([k], staging=mode)
                    op = H.Operator(d["X"], None, d["W_shards"], O)
                    torch.cuda.synchronize()
                    with torch.cuda.stream(sc):
                        op.fwd(k, plan=plan, streams=(sc, sp))
                    sc.synchronize()
                    assert np.array_equal(H.to_bits(op.Y), base), f"Y differs from k=1 ({setting}, k={k}, mode={mode}, pair={pair})"
        for name in setting:
            debug(name, DEBUG_DEFAULTS[name])


# ------------------------------------------------ columns in the forward pass, rows in the backward pass
@pytest.mark.parametrize("T,I,O,N", [(300, 264, 640, 4),      # ragged: the checked kernel
                                     (512, 1024, 2048, 8),    # the unchecked kernels
                                     (256, 16384, 512, 4)])   # long forward reduction: Y is summed in parts
def test_split_per_pass_matches_the_oracle_and_the_unsplit_bits(H, oracle, T, I, O, N):
    """OSDP_SPLIT_PER_PASS cuts W along its columns for the forward pass and along its rows for the backward pass, so
    that Y, dX and dW are all concatenations: every k, staging mode and stream choice must give the unsplit
    operator's bits (no reduction is reordered anywhere), the oracle's values, and the staging law of each pass."""
    import paper_2209_13258_amd as osdp
    d = wl.small_case(161, T, I, O, N)
    want = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    base_op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
    base_op.fwd(1)
    base_op.bwd(1)
    base = base_op.results()
    for name in ("Y", "dX", "dW"):
        H.assert_close(name, base[name], want[name])
    sc, sp = H.streams()
    for k in (2, 4, 8):
        if I % k or O % k or (I // k) % 8 or (O // k) % 8:
            continue
        for mode, slots in ((osdp.OSDP_STAGING_SINGLE, 1), (osdp.OSDP_STAGING_DOUBLE, 2), (osdp.OSDP_STAGING_HALF, 1)):
            if mode == osdp.OSDP_STAGING_HALF and ((I // k) % 16 or (O // k) % 16):
                continue
            plan = osdp.Plan([k], staging=mode, split_dim_per_op=[osdp.OSDP_SPLIT_PER_PASS])
            for two_streams in (False, True):
                _announce("per pass", T, I, O, N, "k", k, "mode", mode, "two streams", two_streams)
                op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
                torch.cuda.synchronize()
                with torch.cuda.stream(sc):
                    st = (sc, sp) if two_streams else (sc, None)
                    op.fwd(k, plan=plan, streams=st)
                    op.bwd(k, plan=plan, streams=st)
                sc.synchronize()
                got = op.results()
                for name in ("Y", "dX", "dW"):
                    assert np.array_equal(got[name], base[name]), f"{name} differs from the unsplit result (k {k}, mode {mode})"
            _, peak_f = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, plan)
            tot_b, peak_b = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, True, plan)
            assert peak_f == oracle.peak_staging_bytes(I, O, k, slots, 2)
            assert peak_b == oracle.peak_staging_bytes_rows(I, O, k, slots, 2)
            assert tot_b == peak_b   # the backward pass keeps no fp32 sum (and these shapes need no planes)


def test_split_per_pass_config4(H, oracle):
    """Config 4 at k = 8 with the per-pass cut, the variant the benchmark reports beside the column slices: sampled
    entries against the oracle (the forward of `down` and the dX of `up` run in parts of the reduction)."""
    import paper_2209_13258_amd as osdp
    w = wl.workload(4, 8)
    for n, op in enumerate(w.ops):
        plan = osdp.Plan([8], split_dim_per_op=[osdp.OSDP_SPLIT_PER_PASS])
        _sampled_check(H, oracle, 4, n, op, w.T, w.N, 8, plan=plan, n_samples=20_000)
        tot_f, _ = osdp.osdp_split_linear_workspace_bytes(w.T, op.I, op.O, w.N, 8, False, plan)
        tot_b, _ = osdp.osdp_split_linear_workspace_bytes(w.T, op.I, op.O, w.N, 8, True, plan)
        assert max(tot_f, tot_b) <= 256 << 20   # two 64 MiB slots and at most 128 MiB of planes: no T x I fp32 sum


@pytest.mark.parametrize("T,I,O,N", [(512, 1024, 32768, 8),    # four parts of 8192 output features
                                     (300, 520, 49152, 4)])    # six parts; ragged: the checked kernel
def test_dx_parts_of_a_long_reduction_keep_the_bits_for_every_k_and_kernel(H, oracle, T, I, O, N, debug):
    """The mirror image for row slices: dX[:, rows_j] = dY . W[rows_j, :]^T reduces over all O output features, in
    parts of 8192 when few tokens meet a long reduction; the number of parts depends on T and O alone, so dX keeps
    the bits of the unsplit operator under a row plan for every k, staging mode, tile shape and kernel."""
    import paper_2209_13258_amd as osdp
    d = wl.small_case(171, T, I, O, N)
    want = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"], want=("dX",))
    rows = [osdp.OSDP_SPLIT_IN_FEATURES]

    def run(k, mode):
        plan = osdp.Plan([k], staging=mode, split_dim_per_op=rows)
        op = H.Operator(d["X"], d["dY"], d["W_shards"], O)
        sc, sp = H.streams()
        torch.cuda.synchronize()
        with torch.cuda.stream(sc):
            op.bwd(k, plan=plan, streams=(sc, sp))
        sc.synchronize()
        return H.to_bits(op.dX)

    base = run(1, osdp.OSDP_STAGING_SINGLE)
    H.assert_close("dX", base, want["dX"])
    debug("split_k", 0)
    one_part = run(1, osdp.OSDP_STAGING_SINGLE)
    debug("split_k", -1)
    H.assert_close("dX (one part)", one_part, want["dX"])
    assert not np.array_equal(base, one_part)
    fast = T % 128 == 0 and I % 128 == 0
    settings = [dict()] + ([dict(tile=t, four_wave=f) for t, f in ((0, 0), (0, 1), (3, -1))] +
                           [dict(tile=0, four_wave=1, persistent=1)] if fast else []) + [dict(gemm_generic=1)]
    for setting in settings:
        for name, value in setting.items():
            debug(name, value)
        for k in (1, 2, 4):
            if I % k or (I // k) % 8:
                continue
            for mode in (osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE, osdp.OSDP_STAGING_HALF):
                if mode == osdp.OSDP_STAGING_HALF and (I // k) % 16:
                    continue
                _announce("dX parts", T, I, O, N, setting, "k", k, "mode", mode)
                assert np.array_equal(run(k, mode), base), f"dX differs from k=1 ({setting}, k={k}, mode={mode})"
        for name in setting:
            debug(name, DEBUG_DEFAULTS[name])
