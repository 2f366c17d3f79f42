"""Host-side logic of libosdp that needs no GPU: symbols, slice planning, sizes, argument checks."""
import ctypes
import re
from pathlib import Path

import pytest

import paper_2209_13258_amd as osdp

ROOT = Path(__file__).resolve().parent.parent


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "osdp.h").read_text()
    declared = re.findall(r"OSDP_API\s+[\w\s\*]+?\b(osdp_\w+)\s*\(", header)
    assert len(declared) >= 10 and {"osdp_split_linear_fwd", "osdp_split_linear_bwd",
                                    "osdp_split_linear_gather_slice"} <= set(declared)
    for name in declared:
        assert hasattr(osdp.lib, name), f"{name} is declared in osdp.h but not exported"
    assert set(declared) == set(osdp.EXPORTS)


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(osdp.binding.osdp_shape) == 32
    assert ctypes.sizeof(osdp.binding.osdp_plan) == 48
    assert ctypes.sizeof(osdp.binding.osdp_granularity_candidate) == 40
    assert ctypes.sizeof(osdp.binding.osdp_operator_cost) == 40
    assert ctypes.sizeof(osdp.binding.osdp_device_info) == 32
    assert ctypes.sizeof(osdp.binding.osdp_search_result) == 48
    assert ctypes.sizeof(osdp.binding.osdp_kernel_stats) == 32


@pytest.mark.parametrize("O", [8, 24, 1024, 7680, 32768])
@pytest.mark.parametrize("k", [0, 1, 2, 3, 4, 6, 8, 16])
def test_slice_ranges_agree_with_oracle(oracle, O, k):
    if max(k, 1) > O:
        return
    for j in range(max(k, 1)):
        assert osdp.osdp_slice_range(O, k, j) == oracle.slice_range(O, k, j)


@pytest.mark.parametrize("I", [8, 24, 1024, 10240])
@pytest.mark.parametrize("k", [0, 1, 2, 3, 4, 8, 16])
def test_row_slice_ranges_agree_with_oracle(oracle, I, k):
    if max(k, 1) > I:
        return
    for j in range(max(k, 1)):
        assert osdp.osdp_row_slice_range(I, k, j) == oracle.row_slice_range(I, k, j)
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_row_slice_range(I, k, max(k, 1))
    assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG


@pytest.mark.parametrize("T,I,O,N,k", [(128, 256, 1024, 2, 4), (8192, 1024, 4096, 8, 8), (16384, 10240, 2560, 8, 4),
                                       (4096, 32768, 8192, 8, 16), (200, 96, 64, 3, 2), (64, 64, 64, 1, 0)])
def test_row_split_workspace_and_peak_staging_follow_the_law(oracle, T, I, O, N, k):
    """Section 3.3 as printed (weight cut along its first dimension): the same size / granularity law; the fp32
    partial sum now belongs to the forward pass (T x O) and the backward pass needs none."""
    rows = [osdp.OSDP_SPLIT_IN_FEATURES]
    single = osdp.Plan([k], staging=osdp.OSDP_STAGING_SINGLE, split_dim_per_op=rows)
    double = osdp.Plan([k], staging=osdp.OSDP_STAGING_DOUBLE, split_dim_per_op=rows)
    half = osdp.Plan([k], staging=osdp.OSDP_STAGING_HALF, split_dim_per_op=rows)
    keff = max(k, 1)
    acc = T * O * 4
    for is_bwd in (False, True):
        tot1, peak1 = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, single)
        tot2, peak2 = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, double)
        toth, peakh = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, half)
        assert peak1 == oracle.peak_staging_bytes_rows(I, O, k, 1, 2) == oracle.weight_bytes(I, O, 2) // keff
        assert peak2 == oracle.peak_staging_bytes_rows(I, O, k, 2, 2)
        assert peakh == peak1
        if is_bwd:
            assert (tot1, tot2, toth) == (peak1, peak2, peakh)
        else:
            assert tot1 == peak1 + (acc if keff > 1 else 0)  # one slot: one launch per slice
            # two slots: pairs of slices may share a launch, so k = 2 may need no partial sum at all
            assert tot2 - peak2 in ((0, acc) if keff == 2 else (acc,) if keff > 2 else (0,))
            assert toth - peakh in ((0, acc) if keff == 1 else (acc,))
    # the unsplit operator is the same whichever dimension the plan names
    assert osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, True, osdp.Plan([1], split_dim_per_op=rows)) == \
        osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, True, osdp.Plan([1]))


def test_longer_dimension_split_resolves_by_shape():
    for T, I, O, N, k in [(256, 512, 2048, 4, 4), (256, 2048, 512, 4, 4), (256, 512, 512, 4, 4)]:
        longer = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, False, osdp.Plan(
            [k], staging=osdp.OSDP_STAGING_SINGLE, split_dim_per_op=[osdp.OSDP_SPLIT_LONGER]))
        want_dim = osdp.OSDP_SPLIT_IN_FEATURES if I > O else osdp.OSDP_SPLIT_OUT_FEATURES
        same = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, False, osdp.Plan(
            [k], staging=osdp.OSDP_STAGING_SINGLE, split_dim_per_op=[want_dim]))
        assert longer == same
        # the forward keeps an fp32 partial sum only when the rows are cut
        assert (longer[0] > longer[1]) == (I > O)


def test_row_split_rejects_what_the_kernels_cannot_take():
    rows = [osdp.OSDP_SPLIT_IN_FEATURES]
    for args, status in [((128, 8, 1024, 2, 16), -1),      # k > I
                         ((128, 264, 1024, 2, 2), -2),     # row bound 132 not a multiple of 8
                         ((128, 256, 1024, 2, 3), -2)]:
        with pytest.raises(osdp.OsdpError) as e:
            osdp.osdp_split_linear_workspace_bytes(*args, False, osdp.Plan([args[4]], split_dim_per_op=rows))
        assert e.value.status == status, (args, str(e.value))
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_workspace_bytes(128, 256, 1024, 2, 2, False, osdp.Plan([2], split_dim_per_op=[7]))
    assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG


@pytest.mark.parametrize("T,I,O,N,k", [(128, 256, 1024, 2, 4), (8192, 1024, 4096, 8, 8), (16384, 10240, 2560, 8, 4),
                                       (4096, 8192, 32768, 8, 16), (4096, 32768, 8192, 8, 4), (64, 64, 64, 1, 0)])
def test_workspace_and_peak_staging_follow_the_law(oracle, T, I, O, N, k):
    """Section 3.3: one live slice is size / granularity; two slots double it; halves restore it."""
    single = osdp.Plan([k], staging=osdp.OSDP_STAGING_SINGLE)
    double = osdp.Plan([k], staging=osdp.OSDP_STAGING_DOUBLE)
    half = osdp.Plan([k], staging=osdp.OSDP_STAGING_HALF)
    keff = max(k, 1)
    w = O // keff

    def passes(n_sub, width, slots):
        """dX passes: sub-slices are staged in groups of `slots`, and a group of two gathered sub-slices is
        staged as one slice across both slots and read by one pass."""
        return len(range(0, n_sub, slots))

    def planes(widths):
        """Forward products of at most 4096 tokens whose reduction is 16384 or longer run in parts of 8192 (at most
        8), each part into an fp32 plane of the widest forward launch (one slice, or two staged ones)."""
        parts = min(I // 8192, 8) if (T <= 4096 and I >= 16384) else 1
        return {0} if parts == 1 else {parts * T * x * 4 for x in widths}

    for is_bwd in (False, True):
        tot1, peak1 = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, single)
        tot2, peak2 = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, double)
        toth, peakh = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, half)
        assert peak1 == oracle.peak_staging_bytes(I, O, k, 1, 2) == oracle.weight_bytes(I, O, 2) // keff
        assert peak2 == oracle.peak_staging_bytes(I, O, k, 2, 2)
        assert peakh == peak1
        acc = T * I * 4 if is_bwd else 0  # the fp32 dX partial sum lives in the workspace between passes
        if is_bwd:
            assert tot1 == peak1 + (acc if passes(keff, w, 1) > 1 else 0)
            assert tot2 == peak2 + (acc if passes(keff, w, 2 if keff > 1 else 1) > 1 else 0)
            assert toth == peakh + (acc if passes(2 * keff, w // 2, 2) > 1 else 0)
        else:
            assert tot1 - peak1 in planes({w})
            assert tot2 - peak2 in planes({w, 2 * w} if keff > 1 else {w})
            assert toth - peakh in planes({w // 2, w})   # half slices one by one, or both halves of a slice in one launch
    # AUTO assumes two streams will be given
    assert osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False)[1] == (peak2 if keff > 1 else peak1)


def test_plan_vector_selects_k():
    plan = osdp.Plan([2, 1, 4, 4])
    peaks = [osdp.osdp_split_linear_workspace_bytes(16384, 2560, 10240, 8, 7, False, plan, n)[1] for n in range(4)]
    full = 2560 * 10240 * 2
    assert peaks == [full, full, full // 2, full // 2]  # 2 slots of 1/k, one slot when k = 1
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_workspace_bytes(16384, 2560, 10240, 8, 1, False, plan, 4)
    assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG


def test_plan_vector_selects_staging_and_split_dimension_per_operator(oracle):
    T, I, O, N = 256, 512, 1024, 4
    plan = osdp.Plan([4, 4, 4, 4], staging=osdp.OSDP_STAGING_DOUBLE, split_dim_per_op=[0, 1, 0, 1],
                     staging_per_op=[osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_SINGLE, osdp.OSDP_STAGING_DOUBLE,
                                     osdp.OSDP_STAGING_HALF])
    peaks = [osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, True, plan, n)[1] for n in range(4)]
    one = oracle.peak_staging_bytes(I, O, 4, 1, 2)
    assert peaks == [one, oracle.peak_staging_bytes_rows(I, O, 4, 1, 2), 2 * one, one]
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 0, True, osdp.Plan([4], staging_per_op=[9]))


def test_dp_slices_are_staged_nowhere(oracle):
    """Section 3.3, last paragraph: a slice in DP mode is replicated, so only the ZDP slices count towards the
    gathered-weight peak; with every slice in DP mode nothing is staged at all."""
    T, I, O, N, k = 128, 256, 1024, 2, 4
    one = oracle.peak_staging_bytes(I, O, k, 1, 2)
    for mask, slots_used in ((0b1111, 2), (0b0111, 2), (0b0001, 1), (0b1000, 1), (0b0000, 0)):
        for is_bwd in (False, True):
            tot, peak = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, is_bwd, osdp.Plan([k], zdp_mask=[mask]))
            assert peak == slots_used * one
            assert tot >= peak
    _, peak = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False,
                                                     osdp.Plan([k], staging=osdp.OSDP_STAGING_SINGLE, zdp_mask=[0b0101]))
    assert peak == one
    _, peak = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, osdp.Plan(
        [k], zdp_mask=[0b0010], split_dim_per_op=[osdp.OSDP_SPLIT_IN_FEATURES]))
    assert peak == oracle.peak_staging_bytes_rows(I, O, k, 1, 2)
    # bits beyond the k slices are ignored
    assert osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, osdp.Plan([k], zdp_mask=[0b1111]))[1] == \
        osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, osdp.Plan([k], zdp_mask=[0xFFFF_FFFF_FFFF_FFFF]))[1]


def test_dp_slices_need_the_mixed_entry_points_and_their_replicas():
    import torch
    if torch.cuda.is_available():
        pytest.skip("uses made-up device addresses: only run where nothing can be launched")
    T, I, O, N, k = 128, 256, 1024, 2, 4
    X, dY = _FakeTensor(0x10000, (T, I)), _FakeTensor(0x20000, (T, O))
    Y, dX = _FakeTensor(0x30000, (T, O)), _FakeTensor(0x40000, (T, I))
    sh = [_FakeTensor(0x50000, (I * O // N,)), _FakeTensor(0x60000, (I * O // N,))]
    plan = osdp.Plan([k], staging=osdp.OSDP_STAGING_SINGLE, zdp_mask=[0b0110])
    need = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, True, plan)[0]
    ws = _FakeTensor(0x70000, (need,), elem=1)
    with pytest.raises(osdp.OsdpError) as e:   # the plain entry point has no replicas to read DP slices from
        osdp.osdp_split_linear_fwd(X, sh, Y, k, ws, plan=plan)
    assert e.value.status == osdp.binding.OSDP_ERR_UNSUPPORTED
    rep = _FakeTensor(0x80000, (I, O // k))
    good = [rep, None, None, rep]
    cases = [
        (dict(w_dp=None), -1),                                             # DP slices but no replicas
        (dict(w_dp=[None, None, None, rep]), -1),                          # slice 0 is DP and has none
        (dict(w_dp=[_FakeTensor(0x80008, (I, O // k)), None, None, rep]), -2),   # misaligned replica
        (dict(ld=O // k - 8), -1),                                         # leading dimension below the slice width
        (dict(ld=O // k + 4), -2),                                         # not a multiple of 8
    ]
    for over, status in cases:
        a = dict(w_dp=good, ld=O // k)
        a.update(over)
        with pytest.raises(osdp.OsdpError) as e:
            osdp.osdp_split_linear_fwd_mixed(X, sh, a["w_dp"], a["ld"], Y, k, ws, plan=plan)
        assert e.value.status == status, (over, str(e.value))
    with pytest.raises(osdp.OsdpError) as e:   # backward also needs somewhere to put the DP gradients
        osdp.osdp_split_linear_bwd_mixed(X, dY, sh, good, O // k, dX, sh, None, k, ws, plan=plan)
    assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG


@pytest.mark.parametrize("args,status", [
    ((-1, 256, 1024, 2, 4), -1), ((128, 0, 1024, 2, 4), -1), ((128, 256, 1024, 0, 4), -1), ((128, 256, 1024, 2, -1), -1),
    ((128, 256, 8, 2, 16), -1),        # k > O
    ((128, 252, 1024, 2, 4), -2),      # I not a multiple of 8
    ((128, 256, 1024, 2, 3), -2),      # slice bounds not aligned to 8 columns
    ((128, 256, 1024, 65, 1), -2),     # more shards than the kernels take
])
def test_bad_shapes(args, status):
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_workspace_bytes(*args, True)
    assert e.value.status == status
    assert str(e.value)


class _FakeTensor:
    """Stands in for a device tensor in argument-validation tests: nothing is ever launched."""

    def __init__(self, ptr, shape, stride0=None, elem=2):
        self._ptr, self.shape, self._s, self._e = ptr, shape, stride0 if stride0 is not None else shape[-1], elem

    def data_ptr(self):
        return self._ptr

    def stride(self, d):
        return self._s

    def numel(self):
        n = 1
        for s in self.shape:
            n *= s
        return n

    def element_size(self):
        return self._e


def test_argument_errors_are_raised_before_anything_is_enqueued():
    import torch
    if torch.cuda.is_available():
        pytest.skip("uses made-up device addresses: only run where nothing can be launched")
    T, I, O, N, k = 128, 256, 1024, 2, 4
    X = _FakeTensor(0x10000, (T, I))
    Y = _FakeTensor(0x20000, (T, O))
    shards = [_FakeTensor(0x30000, (I * O // N,)), _FakeTensor(0x40000, (I * O // N,))]
    plan = osdp.Plan([k], staging=osdp.OSDP_STAGING_SINGLE)
    need, _ = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, plan)
    cases = [
        (dict(X=_FakeTensor(0, (T, I))), -1),                       # NULL X
        (dict(X=_FakeTensor(0x10008, (T, I))), -2),                 # misaligned X
        (dict(X=_FakeTensor(0x10000, (T, I), stride0=I - 8)), -1),  # ld below the row length
        (dict(Y=_FakeTensor(0x20000, (T, O), stride0=O + 4)), -2),  # ld not a multiple of 8
        (dict(shards=[shards[0], _FakeTensor(0, (1,))]), -1),       # NULL shard
        (dict(ws=_FakeTensor(0x50000, (need - 1,), elem=1)), -3),   # workspace one byte short
        (dict(ws=_FakeTensor(0x50010, (need,), elem=1)), -2),       # workspace not 256-byte aligned
    ]
    for over, status in cases:
        a = dict(X=X, Y=Y, shards=shards, ws=_FakeTensor(0x50000, (need,), elem=1))
        a.update(over)
        with pytest.raises(osdp.OsdpError) as e:
            osdp.osdp_split_linear_fwd(a["X"], a["shards"], a["Y"], k, a["ws"], plan=plan)
        assert e.value.status == status, (over, str(e.value))
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_gather_slice(I, O, k, 4, shards, _FakeTensor(0x50000, (1,)))
    assert e.value.status == -1  # slice index out of range
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_gather_row_slice(I, O, k, 4, shards, _FakeTensor(0x50000, (1,)))
    assert e.value.status == -1
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_gather_row_slice(I, O, k, 0, shards, _FakeTensor(0x50008, (1,)))
    assert e.value.status == -2  # misaligned staging


def test_debug_options_take_known_names_and_values_only():
    for name, good, bad in (("gemm_generic", (0, 1, 0), (-1, 2)), ("tile", (0, 3, -1), (-2, 4)), ("deep", (0, -1), (2,)),
                            ("split_launch", (0, -1), (-2,)), ("fwd_pair", (0, 1, -1), (2,)),
                            ("poison_staging", (1, 0), (-1, 2)), ("persistent", (0, 1, -1), (-2, 2)),
                            ("four_wave", (0, 1, -1), (2,)), ("fused_gather", (0, -1), (-2,)), ("split_k", (0, -1), (-2,))):
        for v in good:   # the last good value is the default: the switches are process-wide
            osdp.osdp_debug_option(name, v)
        for v in bad:
            with pytest.raises(osdp.OsdpError) as e:
                osdp.osdp_debug_option(name, v)
            assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_debug_option("no_such_switch", 0)


def test_forward_launch_plan_follows_the_pairing_switch():
    """The pairing switch changes the forward launch plan, and with it the fp32 partial sum a row-slice forward
    needs between launches: the size query answers for the switch's current value."""
    T, I, O, N, k = 8192, 4096, 1024, 8, 2
    plan = osdp.Plan([k], staging=osdp.OSDP_STAGING_DOUBLE, split_dim_per_op=[osdp.OSDP_SPLIT_IN_FEATURES])
    try:
        osdp.osdp_debug_option("fwd_pair", 1)
        paired, _ = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, plan)
        osdp.osdp_debug_option("fwd_pair", 0)
        single, _ = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, plan)
    finally:
        osdp.osdp_debug_option("fwd_pair", -1)
    assert single == paired + T * O * 4   # two accumulating launches carry Y's partial sum through the workspace


def test_no_workspace_forward_refuses_what_its_array_cannot_hold():
    """The size check of the entry point that allocates nothing comes before any device call."""
    T, I, O, N = 128, 8192, 8192, 8
    X = _FakeTensor(0x10000, (T, I))
    Y = _FakeTensor(0x20000, (T, O))
    shards = [_FakeTensor(0x30000 + 0x1000 * s, (I * O // N,)) for s in range(N)]
    need, _ = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, False)
    assert need > osdp.OSDP_NOALLOC_SCRATCH_BYTES
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_fwd_noalloc(X, shards, Y, 1)
    assert e.value.status == osdp.binding.OSDP_ERR_WORKSPACE and "scratch" in str(e.value)


def test_profile_end_without_begin_is_an_error():
    with pytest.raises(osdp.OsdpError):
        osdp.osdp_profile_end()


def test_zero_tokens_is_a_legal_shape_and_negative_is_not():
    """No tokens: the operator still has its weight, so the staging law is unchanged and the fp32 partial sum is empty."""
    total0, peak0 = osdp.osdp_split_linear_workspace_bytes(0, 1024, 4096, 8, 4, True)
    total1, peak1 = osdp.osdp_split_linear_workspace_bytes(128, 1024, 4096, 8, 4, True)
    assert peak0 == peak1 and total0 == total1 - 128 * 1024 * 4
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_workspace_bytes(-1, 1024, 4096, 8, 4, True)
    assert e.value.status == osdp.binding.OSDP_ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's share of the step; asking for more must end with a message, not a run."""
    import subprocess
    import sys
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    r = subprocess.run([sys.executable, str(root / "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus must be 1" in (r.stderr + r.stdout)


def test_public_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: include/osdp.h must compile as C99 on its own, with no warnings."""
    import subprocess
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    src = tmp_path / "use_header.c"
    src.write_text('#include "osdp.h"\nint main(void) { return (int)sizeof(osdp_plan) + (int)sizeof(osdp_shape); }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", f"-I{root / 'include'}",
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_a_c_program_links_and_calls_the_library(tmp_path):
    """No Python in between: a C99 program links libosdp.so and uses the host-side calls (slice law, errors)."""
    import subprocess
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    pkg = root / "paper_2209_13258_amd"
    src = tmp_path / "client.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "osdp.h"
int main(void) {
  osdp_shape s = {8192, 1024, 4096, 8, 4};
  int64_t c0 = -1, c1 = -1;
  size_t total = 0, peak = 0;
  if (osdp_slice_range(&s, 3, &c0, &c1) != OSDP_OK || c0 != 3072 || c1 != 4096) return 1;
  if (osdp_split_linear_workspace_bytes(&s, NULL, 0, 1, &total, &peak) != OSDP_OK) return 2;
  if (peak != (size_t)2 * 1024 * 1024 * 2 || total < peak) return 3;        /* automatic staging: two slots of size / k = 2 MiB */
  if (osdp_slice_range(&s, 4, &c0, &c1) != OSDP_ERR_INVALID_ARG) return 4;  /* slice index out of range */
  if (strlen(osdp_last_error()) == 0 || strlen(osdp_strerror(OSDP_ERR_INVALID_ARG)) == 0) return 5;
  printf("%s\n", osdp_version());
  return 0;
}
''')
    exe = tmp_path / "client"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", f"-I{root / 'include'}", str(src), "-o", str(exe),
                        f"-L{pkg}", "-losdp", f"-Wl,-rpath,{pkg}", "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.strip()


@pytest.mark.parametrize("T,I,O,N,k", [(8192, 1024, 4096, 8, 4), (16384, 2560, 10240, 8, 4), (128, 256, 1024, 2, 2)])
def test_per_pass_split_needs_no_partial_sum(oracle, T, I, O, N, k):
    """Columns in the forward pass, rows in the backward pass: both passes only concatenate, so the workspace is the
    staging slots alone (these shapes need no planes), and each pass follows its own dimension's size / k law."""
    for mode, slots in ((osdp.OSDP_STAGING_SINGLE, 1), (osdp.OSDP_STAGING_DOUBLE, 2)):
        plan = osdp.Plan([k], staging=mode, split_dim_per_op=[osdp.OSDP_SPLIT_PER_PASS])
        tot_f, peak_f = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, False, plan)
        tot_b, peak_b = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, True, plan)
        assert tot_f == peak_f == oracle.peak_staging_bytes(I, O, k, slots, 2)
        assert tot_b == peak_b == oracle.peak_staging_bytes_rows(I, O, k, slots, 2)
    with pytest.raises(osdp.OsdpError):   # a replica is laid out slice by slice: one split dimension for both passes
        osdp.osdp_split_linear_workspace_bytes(T, I, O, N, k, True, osdp.Plan([k], zdp_mask=[1], split_dim_per_op=[osdp.OSDP_SPLIT_PER_PASS]))
