"""Pins for the CPU oracle: each part is checked against something other than itself.

What fixes the expected values here is the paper and the mathematics, never the
oracle and never the GPU path: exact rational arithmetic, numpy's own float64
matmul, closed forms, a tensor library's flat-parameter chunking, and the
numbers the paper prints (tests/golden/*.json, each with its citation).
"""
import json
import struct
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

import workloads as wl

GOLDEN = Path(__file__).resolve().parent / "golden"


def widen(bits):
    """bf16 bits -> float64, written independently of the oracle (via struct)."""
    bits = np.asarray(bits, dtype=np.uint16)
    out = np.empty(bits.size, dtype=np.float64)
    for n, b in enumerate(bits.reshape(-1)):
        out[n] = struct.unpack(">f", struct.pack(">HH", int(b), 0))[0]
    return out.reshape(bits.shape)


def frac(bits):
    return [[Fraction(float(v)) for v in row] for row in widen(bits)]


# ------------------------------------------------------------------ widening
def test_bf16_widen_known_values(oracle):
    known = {0x3F80: 1.0, 0xC000: -2.0, 0x0000: 0.0, 0x3DCD: 0.10009765625,
             0x0001: 2.0 ** -133, 0x7F7F: (2 - 2 ** -7) * 2.0 ** 127, 0xBF00: -0.5, 0x4049: 3.140625}
    got = oracle.bf16_to_f64(np.array(list(known), dtype=np.uint16))
    assert got.tolist() == list(known.values())


def test_bf16_widen_matches_tensor_library(oracle):
    import torch
    bits = np.arange(0, 1 << 16, 7, dtype=np.uint16)
    bits = bits[(bits & 0x7F80) != 0x7F80]  # finite values only
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    assert np.array_equal(oracle.bf16_to_f64(bits), ref)


# ---------------------------------------------------- definition: exact pins
@pytest.mark.parametrize("T,I,O,N", [(3, 4, 5, 2), (5, 6, 2, 3), (1, 8, 7, 4), (4, 3, 6, 1), (2, 5, 3, 4)])
def test_definition_against_exact_rationals(oracle, T, I, O, N):
    """Brute force in exact arithmetic; non-square shapes expose any swapped index."""
    d = wl.small_case(1, T, I, O, N, w_std=1.0)
    X, dY, shards = d["X"], d["dY"], d["W_shards"]
    flat = np.concatenate(shards)[: I * O]
    W = flat.reshape(I, O)
    Xf, dYf, Wf = frac(X), frac(dY), frac(W)
    out = oracle.linear(X, shards, O, dY=dY)
    for t in range(T):
        for o in range(O):
            ex = sum(Xf[t][i] * Wf[i][o] for i in range(I))
            mag = sum(abs(Xf[t][i] * Wf[i][o]) for i in range(I))
            assert abs(Fraction(out["Y"][t, o]) - ex) <= mag * Fraction(I, 2 ** 52)
    for t in range(T):
        for i in range(I):
            ex = sum(dYf[t][o] * Wf[i][o] for o in range(O))
            mag = sum(abs(dYf[t][o] * Wf[i][o]) for o in range(O))
            assert abs(Fraction(out["dX"][t, i]) - ex) <= mag * Fraction(O, 2 ** 52)
    for i in range(I):
        for o in range(O):
            ex = sum(Xf[t][i] * dYf[t][o] for t in range(T))
            mag = sum(abs(Xf[t][i] * dYf[t][o]) for t in range(T))
            assert abs(Fraction(out["dW"][i, o]) - ex) <= mag * Fraction(T, 2 ** 52)


@pytest.mark.parametrize("T,I,O", [(37, 48, 29), (64, 17, 80)])
def test_definition_against_library_matmul(oracle, T, I, O):
    d = wl.small_case(2, T, I, O, 1)
    X, dY, W = d["X"], d["dY"], d["W_shards"][0].reshape(I, O)
    Xd, dYd, Wd = widen(X), widen(dY), widen(W)
    np.testing.assert_allclose(oracle.matmul_fwd(X, W), Xd @ Wd, rtol=0, atol=1e-12 * np.abs(Xd @ Wd).max())
    np.testing.assert_allclose(oracle.matmul_dx(dY, W), dYd @ Wd.T, rtol=0, atol=1e-12 * np.abs(dYd @ Wd.T).max())
    np.testing.assert_allclose(oracle.matmul_dw(X, dY), Xd.T @ dYd, rtol=0, atol=1e-12 * np.abs(Xd.T @ dYd).max())


def test_closed_forms(oracle):
    T, I, O = 6, 6, 9
    d = wl.small_case(3, T, I, O, 1, w_std=1.0)
    W, dY = d["W_shards"][0].reshape(I, O), d["dY"]
    one = wl.f32_to_bf16_bits(np.float32(1.0))
    eye = np.where(np.eye(T, I, dtype=bool), one, np.uint16(0)).astype(np.uint16)
    # X = identity: Y is W itself, dW is dY itself
    assert np.array_equal(oracle.matmul_fwd(eye, W), widen(W))
    assert np.array_equal(oracle.matmul_dw(eye, dY), widen(dY))
    # W = [identity | 0]: dX picks the first I columns of dY
    Wsel = np.zeros((I, O), dtype=np.uint16)
    Wsel[np.arange(I), np.arange(I)] = one
    assert np.array_equal(oracle.matmul_dx(dY, Wsel), widen(dY)[:, :I])
    # all-ones X against a constant W: every Y entry is I * c
    ones = np.full((T, I), one, dtype=np.uint16)
    c = wl.f32_to_bf16_bits(np.float32(0.375))
    assert np.array_equal(oracle.matmul_fwd(ones, np.full((I, O), c, dtype=np.uint16)), np.full((T, O), I * 0.375))
    # rank one: X = u 1^T, W = 1 v^T  ->  Y = I * u v^T (small integers: exact)
    u = wl.f32_to_bf16_bits(np.arange(1, T + 1, dtype=np.float32))
    v = wl.f32_to_bf16_bits(np.arange(-4, O - 4, dtype=np.float32))
    Y = oracle.matmul_fwd(np.repeat(u[:, None], I, 1), np.repeat(v[None, :], I, 0))
    assert np.array_equal(Y, I * np.outer(np.arange(1, T + 1), np.arange(-4, O - 4)).astype(np.float64))


# -------------------------------------------------------------- slice bounds
@pytest.mark.parametrize("O", [1, 7, 24, 1024, 32768, 4 * 8192])
@pytest.mark.parametrize("k", [0, 1, 2, 4, 6, 8, 16])
def test_slice_ranges_partition_the_columns(oracle, O, k):
    keff = max(k, 1)
    ranges = [oracle.slice_range(O, k, j) for j in range(keff)]
    assert ranges[0][0] == 0 and ranges[-1][1] == O
    assert all(a[1] == b[0] for a, b in zip(ranges, ranges[1:]))
    widths = [c1 - c0 for c0, c1 in ranges]
    assert max(widths) - min(widths) <= 1 and sum(widths) == O
    if k == 0:  # granularity 0 of Section 4.3 = unsplit
        assert ranges == [(0, O)]


# ---------------------------------------------------------------- shard map
@pytest.mark.parametrize("I,O,N", [(8, 12, 2), (8, 12, 4), (6, 5, 4), (7, 3, 8), (16, 16, 8), (5, 5, 1)])
def test_shard_map_is_flat_parameter_chunking(oracle, I, O, N):
    """FSDP-style sharding (Section 2.2): flatten, pad to a multiple of N, chunk."""
    import torch
    W = np.arange(1, I * O + 1, dtype=np.uint16).reshape(I, O)
    L = oracle.shard_len(I, O, N)
    flat = torch.from_numpy(W.astype(np.int32)).reshape(-1)
    flat = torch.nn.functional.pad(flat, (0, N * L - I * O))
    ref = [c.numpy().astype(np.uint16) for c in torch.chunk(flat, N)]
    got = oracle.shard(W, N)
    assert len(got) == N and all(np.array_equal(a, b) for a, b in zip(got, ref))
    assert np.array_equal(oracle.assemble(got, I, O), W)
    for r in (0, I // 2, I - 1):
        for c in (0, O - 1):
            s, off = oracle.locate(I, O, N, r, c)
            assert got[s][off] == W[r, c]
    if I % N == 0:  # row-block shards
        for s in range(N):
            assert np.array_equal(got[s].reshape(I // N, O), W[s * (I // N):(s + 1) * (I // N)])


@pytest.mark.parametrize("I,O,N,k", [(8, 12, 2, 4), (8, 12, 4, 3), (6, 5, 4, 2), (7, 10, 8, 6), (16, 16, 8, 16), (4, 9, 1, 0)])
def test_gather_is_the_column_view(oracle, I, O, N, k):
    W = np.arange(1, I * O + 1, dtype=np.uint16).reshape(I, O)
    shards = oracle.shard(W, N)
    seen = np.zeros((I, O), dtype=np.int32)
    for j in range(max(k, 1)):
        c0, c1 = oracle.slice_range(O, k, j)
        Ws = oracle.gather_slice(shards, I, O, k, j)
        assert Ws.shape == (I, c1 - c0)
        assert np.array_equal(Ws, W[:, c0:c1])
        seen[:, c0:c1] += 1
    assert (seen == 1).all()  # every weight gathered exactly once over the slices


# ------------------------------------------------- split route == definition
@pytest.mark.parametrize("T,I,O,N,k", [
    (9, 16, 24, 2, 4), (9, 16, 24, 4, 1), (9, 16, 24, 4, 0), (5, 12, 20, 3, 6), (7, 10, 13, 4, 5),
    (4, 8, 16, 8, 16), (6, 6, 7, 5, 3)])
def test_split_route_reconstructs_the_unsplit_result(oracle, T, I, O, N, k):
    d = wl.small_case(4, T, I, O, N, w_std=1.0)
    X, dY, shards = d["X"], d["dY"], d["W_shards"]
    ref = oracle.linear(X, shards, O, dY=dY)
    Y, peak_f = oracle.split_fwd(X, shards, O, k)
    dX, dWs, peak_b = oracle.split_bwd(X, dY, shards, O, k)
    # concatenation does not touch any per-element sum: exact
    assert np.array_equal(Y, ref["Y"])
    assert np.array_equal(oracle.dense_from_f64_shards(dWs, I, O), ref["dW"])
    # dX regroups the sum over o into k partial sums
    np.testing.assert_allclose(dX, ref["dX"], rtol=0, atol=1e-13 * np.abs(ref["dX"]).max() + 1e-300)
    # Section 3.3: one live slice = size / granularity (largest slice when k does not divide O)
    wmax = max(c1 - c0 for c0, c1 in (oracle.slice_range(O, k, j) for j in range(max(k, 1))))
    assert peak_f == peak_b == I * wmax * 2 == oracle.peak_staging_bytes(I, O, k, 1, 2)
    if k >= 1 and O % k == 0:
        assert peak_f * k == oracle.weight_bytes(I, O, 2)


@pytest.mark.parametrize("T,I,O,N,k", [
    (9, 16, 24, 2, 4), (9, 16, 24, 4, 1), (5, 12, 20, 3, 6), (7, 10, 13, 4, 3), (4, 16, 8, 8, 16), (6, 7, 6, 5, 0)])
def test_reduction_split_route_reconstructs_the_unsplit_result(oracle, T, I, O, N, k):
    """Section 3.3 as printed: rows of W (the reduction dimension) are sliced and the outputs summed."""
    d = wl.small_case(7, T, I, O, N, w_std=1.0)
    X, dY, shards = d["X"], d["dY"], d["W_shards"]
    ref = oracle.linear(X, shards, O, dY=dY)
    W = np.concatenate(shards)[: I * O].reshape(I, O)
    seen = np.zeros(I, dtype=np.int32)
    for j in range(max(k, 1)):  # the row slices are the strided row views and cover every row once
        r0, r1 = oracle.row_slice_range(I, k, j)
        assert np.array_equal(oracle.gather_row_slice(shards, I, O, k, j), W[r0:r1])
        seen[r0:r1] += 1
    assert (seen == 1).all()
    Y, peak_f = oracle.split_fwd_rows(X, shards, O, k)
    dX, dWs, peak_b = oracle.split_bwd_rows(X, dY, shards, O, k)
    # dX and dW are concatenations here: exact; Y regroups the sum over i into k partial sums
    assert np.array_equal(dX, ref["dX"])
    assert np.array_equal(oracle.dense_from_f64_shards(dWs, I, O), ref["dW"])
    np.testing.assert_allclose(Y, ref["Y"], rtol=0, atol=1e-13 * np.abs(ref["Y"]).max() + 1e-300)
    wmax = max(r1 - r0 for r0, r1 in (oracle.row_slice_range(I, k, j) for j in range(max(k, 1))))
    assert peak_f == peak_b == wmax * O * 2 == oracle.peak_staging_bytes_rows(I, O, k, 1, 2)
    if k >= 1 and I % k == 0:
        assert peak_f * k == oracle.weight_bytes(I, O, 2)  # size / granularity


def _mixed_case(oracle, seed, T, I, O, N, k, mask, rows, full_layout):
    """Inputs for the per-slice DP/ZDP route in which the two weight sources disagree: the shards hold W with a
    NaN pattern wherever a DP slice lies, the DP replicas hold other values.  Returns the inputs and the matrix
    the operator really uses (float64)."""
    d = wl.small_case(seed, T, I, O, N, w_std=1.0)
    other = wl.small_case(seed + 100, T, I, O, N, w_std=1.0)
    W = np.concatenate(d["W_shards"])[: I * O].reshape(I, O).copy()
    W2 = np.concatenate(other["W_shards"])[: I * O].reshape(I, O)
    keff = max(k, 1)
    rng = [(oracle.row_slice_range(I, k, j) if rows else oracle.slice_range(O, k, j)) for j in range(keff)]
    used = W.copy()
    w_dp = [None] * keff
    ld = O if (rows or full_layout) else max(b - a for a, b in rng)
    for j, (a, b) in enumerate(rng):
        if (mask >> j) & 1:
            continue
        sl = (slice(a, b), slice(None)) if rows else (slice(None), slice(a, b))
        used[sl] = W2[sl]
        W[sl] = 0x7FC0                       # what the shards hold there must never be read
        if rows:
            w_dp[j] = W2[a:b].copy()
        elif full_layout:
            w_dp[j] = np.ascontiguousarray(W2).reshape(-1)[a:]      # the slice where it lies in a full [I x O] copy
        else:
            buf = np.full((I, ld), 0x7FC0, dtype=np.uint16)   # compact replica, padded to the common ld
            buf[:, : b - a] = W2[:, a:b]
            w_dp[j] = buf
    L = oracle.shard_len(I, O, N)
    flat = np.full(N * L, 0x7FC0, dtype=np.uint16)
    flat[: I * O] = W.reshape(-1)
    shards = [flat[s * L:(s + 1) * L].copy() for s in range(N)]
    return d["X"], d["dY"], shards, w_dp, ld, rng, widen(used)


@pytest.mark.parametrize("rows", [False, True])
@pytest.mark.parametrize("full_layout", [False, True])
@pytest.mark.parametrize("T,I,O,N,k,mask", [
    (9, 16, 24, 2, 4, 0b0001),   # the paper's example: one slice of four in ZDP mode, three in DP mode
    (9, 16, 24, 4, 4, 0b1010), (5, 12, 20, 3, 6, 0b110011), (7, 10, 13, 4, 3, 0b000), (7, 10, 13, 4, 3, 0b111),
    (6, 8, 8, 8, 1, 0b0), (6, 8, 8, 8, 0, 0b1)])
def test_per_slice_modes_use_each_slice_from_its_own_place(oracle, T, I, O, N, k, mask, rows, full_layout):
    """Section 3.3, last paragraph.  Expected values: numpy's float64 products with the matrix assembled by hand
    from the two sources; gradients land in the shards (ZDP slices) or in the slice's own array (DP slices) and
    nowhere else; only ZDP slices are ever staged."""
    X, dY, shards, w_dp, ld, rng, Wf = _mixed_case(oracle, 9, T, I, O, N, k, mask, rows, full_layout)
    Xf, dYf = widen(X), widen(dY)
    Y, peak_f = oracle.split_fwd_mixed(X, shards, O, k, mask, w_dp, ld, rows=rows)
    dX, dWs, dw_dp, peak_b = oracle.split_bwd_mixed(X, dY, shards, O, k, mask, w_dp, ld, rows=rows)
    np.testing.assert_allclose(Y, Xf @ Wf, rtol=0, atol=1e-12 * np.abs(Xf @ Wf).max())
    np.testing.assert_allclose(dX, dYf @ Wf.T, rtol=0, atol=1e-12 * np.abs(dYf @ Wf.T).max())
    dW_ref = Xf.T @ dYf
    dense = oracle.dense_from_f64_shards(dWs, I, O)
    for j, (a, b) in enumerate(rng):
        sl = (slice(a, b), slice(None)) if rows else (slice(None), slice(a, b))
        if (mask >> j) & 1:
            np.testing.assert_allclose(dense[sl], dW_ref[sl], rtol=0, atol=1e-12 * np.abs(dW_ref).max())
            assert dw_dp[j] is None
        else:
            assert np.isnan(dense[sl]).all()          # a DP slice's gradient is not sharded
            h, w = (b - a, O) if rows else (I, b - a)
            np.testing.assert_allclose(dw_dp[j][:h, :w], dW_ref[sl], rtol=0, atol=1e-12 * np.abs(dW_ref).max())
            if not full_layout:
                assert np.isnan(dw_dp[j][:, w:]).all()    # nothing written outside the slice's columns
    zdp = [(b - a) for j, (a, b) in enumerate(rng) if (mask >> j) & 1]
    want_peak = (max(zdp) * (O if rows else I) * 2) if zdp else 0
    assert peak_f == peak_b == want_peak


@pytest.mark.parametrize("rows", [False, True])
def test_all_zdp_mask_is_the_plain_split_route(oracle, rows):
    T, I, O, N, k = 9, 16, 24, 4, 4
    d = wl.small_case(10, T, I, O, N, w_std=1.0)
    fwd, bwd = (oracle.split_fwd_rows, oracle.split_bwd_rows) if rows else (oracle.split_fwd, oracle.split_bwd)
    Y, _ = oracle.split_fwd_mixed(d["X"], d["W_shards"], O, k, 0b1111, [None] * k, O, rows=rows)
    dX, dWs, dw_dp, _ = oracle.split_bwd_mixed(d["X"], d["dY"], d["W_shards"], O, k, 0b1111, [None] * k, O, rows=rows)
    assert np.array_equal(Y, fwd(d["X"], d["W_shards"], O, k)[0])
    ref_dX, ref_dWs, _ = bwd(d["X"], d["dY"], d["W_shards"], O, k)
    assert np.array_equal(dX, ref_dX) and dw_dp == [None] * k
    assert np.array_equal(oracle.dense_from_f64_shards(dWs, I, O), oracle.dense_from_f64_shards(ref_dWs, I, O))


def test_per_slice_modes_exact_on_small_integers(oracle):
    """Integer-valued inputs: every product and sum is exact in float64, so the expected values are exact."""
    T, I, O, N, k, mask = 5, 8, 12, 4, 3, 0b010
    g = np.random.default_rng(11)
    to_bits = lambda a: wl.f32_to_bf16_bits(a.astype(np.float32))
    Xi, dYi = g.integers(-4, 5, (T, I)), g.integers(-4, 5, (T, O))
    Wz, Wd = g.integers(-4, 5, (I, O)), g.integers(-4, 5, (I, O))
    used = Wd.copy()
    used[:, 4:8] = Wz[:, 4:8]                 # slice 1 is the ZDP one
    shards = oracle.shard(to_bits(Wz), N)
    w_dp = [to_bits(Wd[:, 0:4]), None, to_bits(Wd[:, 8:12])]
    Y, _ = oracle.split_fwd_mixed(to_bits(Xi), shards, O, k, mask, w_dp, 4)
    dX, dWs, dw_dp, _ = oracle.split_bwd_mixed(to_bits(Xi), to_bits(dYi), shards, O, k, mask, w_dp, 4)
    assert np.array_equal(Y, (Xi @ used).astype(np.float64))
    assert np.array_equal(dX, (dYi @ used.T).astype(np.float64))
    dW = Xi.T @ dYi
    assert np.array_equal(dw_dp[0], dW[:, 0:4]) and np.array_equal(dw_dp[2], dW[:, 8:12])
    assert np.array_equal(oracle.dense_from_f64_shards(dWs, I, O)[:, 4:8], dW[:, 4:8])


def test_split_route_ignores_shard_padding(oracle):
    T, I, O, N, k = 4, 5, 7, 4, 3
    d = wl.small_case(5, T, I, O, N)
    a = oracle.split_fwd(d["X"], d["W_shards"], O, k)[0]
    shards = [s.copy() for s in d["W_shards"]]
    L = oracle.shard_len(I, O, N)
    assert N * L > I * O
    shards[-1][I * O - (N - 1) * L:] = 0x7FC0  # NaN pattern in the padding
    assert np.array_equal(oracle.split_fwd(d["X"], shards, O, k)[0], a)


def test_sampled_entries_are_entries_of_the_definition(oracle):
    T, I, O, N = 11, 12, 10, 4
    d = wl.small_case(6, T, I, O, N, w_std=1.0)
    ref = oracle.linear(d["X"], d["W_shards"], O, dY=d["dY"])
    g = np.random.default_rng(0)
    r, c = g.integers(0, T, 50), g.integers(0, O, 50)
    assert np.array_equal(oracle.sample_y(d["X"], d["W_shards"], O, r, c), ref["Y"][r, c])
    r, c = g.integers(0, T, 50), g.integers(0, I, 50)
    assert np.array_equal(oracle.sample_dx(d["dY"], d["W_shards"], I, r, c), ref["dX"][r, c])
    r, c = g.integers(0, I, 50), g.integers(0, O, 50)
    assert np.array_equal(oracle.sample_dw(d["X"], d["dY"], r, c), ref["dW"][r, c])


# ----------------------------------------------- numbers the paper prints
def test_worked_size_example(oracle):
    g = json.loads((GOLDEN / "size_example.json").read_text())
    params = oracle.weight_bytes(g["I"], g["O"], 1)
    assert params == 603979776
    assert round(params / 1e9, 1) == g["params_billion_printed"]
    # the printed gigabytes follow from the printed (rounded) parameter count at 4 bytes each
    assert round(g["params_billion_printed"] * 1e9 * 4 / 2 ** 30, 2) == pytest.approx(g["gathered_gb_printed"], abs=0.006)
    exact_gib = oracle.weight_bytes(g["I"], g["O"], 4) / 2 ** 30
    assert exact_gib == 2.25 and abs(exact_gib - g["gathered_gb_printed"]) / g["gathered_gb_printed"] < 0.01


@pytest.mark.parametrize("h", [8192, 12288])
def test_staging_law_against_the_memory_curve(oracle, h):
    """Memory saved by splitting = layer weights minus two live slices per operator (k = 4, 6, 8)."""
    g = json.loads((GOLDEN / "fig7_memory.json").read_text())
    mem = dict(zip(g["granularity"], g["mem_mb"][str(h)]))
    layer = [(h, 3 * h), (h, h), (h, 4 * h), (4 * h, h)]
    full = sum(oracle.weight_bytes(i, o, 4) for i, o in layer)
    for k in (4, 6, 8):
        live = sum(oracle.peak_staging_bytes(i, o, k, 2, 4) for i, o in layer)
        saved_mib = (full - live) / 2 ** 20
        assert saved_mib == pytest.approx(mem[0] - mem[k], rel=2e-3)
        # one live slice would save visibly more than the paper measured
        one = sum(oracle.peak_staging_bytes(i, o, k, 1, 4) for i, o in layer)
        assert (full - one) / 2 ** 20 > 1.1 * (mem[0] - mem[k])
    assert mem[0] - mem[16] == pytest.approx(mem[0] - mem[8], rel=2e-3)  # flat beyond 8: not the law


def test_peak_staging_closed_form(oracle):
    # Section 3.3: size(MatMul) / slice_granularity
    for I, O, k in [(1024, 4096, 4), (10240, 2560, 4), (8192, 32768, 16), (256, 1024, 1)]:
        assert oracle.peak_staging_bytes(I, O, k, 1, 2) * k == oracle.weight_bytes(I, O, 2)
        assert oracle.peak_staging_bytes(I, O, k, 2, 2) == min(2, k) * oracle.weight_bytes(I, O, 2) // k
    assert oracle.peak_staging_bytes(64, 100, 0, 1, 2) == oracle.weight_bytes(64, 100, 2)
