"""The forward entry point that takes no workspace: its staging slots and partial sums live in a fixed array
inside the library, so it allocates nothing.  Checked bit for bit against osdp_split_linear_fwd, on two calls in
a row that share the array, the second with a smaller input; and against the oracle."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    return gpu_harness


def _fwd_pair(H, d, O, k, plan, stream):
    """(Y of the no-workspace call, Y of the workspace call) as bit patterns."""
    import paper_2209_13258_amd as osdp
    op = H.Operator(d["X"], None, d["W_shards"], O)
    Y2 = torch.full_like(op.Y, float("nan"))
    with torch.cuda.stream(stream):
        osdp.osdp_split_linear_fwd_noalloc(op.X, op.W, Y2, k, plan=plan, stream=stream)
        op.fwd(k, plan=plan, streams=(stream, None))
    stream.synchronize()
    return H.to_bits(Y2), H.to_bits(op.Y)


@pytest.mark.parametrize("rows", [False, True])
def test_two_calls_in_a_row_match_the_workspace_entry_point(H, oracle, rows):
    import paper_2209_13258_amd as osdp
    dim = osdp.OSDP_SPLIT_IN_FEATURES if rows else osdp.OSDP_SPLIT_OUT_FEATURES
    stream = torch.cuda.Stream()
    # first a larger operator (staging 2 x 1 MiB, fp32 partial sum 1.5 MiB with row slices), then a smaller, ragged
    # one whose slots and partial sum cover only the front of what the first call left in the array
    for seed, (T, I, O, N, k, mode) in enumerate([(384, 1024, 2048, 8, 4, osdp.OSDP_STAGING_DOUBLE),
                                                  (77, 264, 528, 4, 3, osdp.OSDP_STAGING_SINGLE)]):
        print("no-alloc forward", T, I, O, N, k, "rows" if rows else "columns", flush=True)
        d = wl.small_case(120 + seed, T, I, O, N)
        plan = osdp.Plan([k], staging=mode, split_dim_per_op=[dim])
        got, want = _fwd_pair(H, d, O, k, plan, stream)
        assert np.array_equal(got, want), "the no-workspace forward differs from osdp_split_linear_fwd"
        H.assert_close("Y", got, oracle.linear(d["X"], d["W_shards"], O, want=("Y",))["Y"])


def test_sizes_beyond_the_array_are_refused_before_anything_runs(H):
    import paper_2209_13258_amd as osdp
    T, I, O, N = 128, 8192, 8192, 8            # unsplit: one slot of 128 MiB
    X = torch.zeros((T, I), dtype=torch.bfloat16, device="cuda")
    W = [torch.zeros((I * O // N,), dtype=torch.bfloat16, device="cuda") for _ in range(N)]
    Y = torch.full((T, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    need, _ = osdp.osdp_split_linear_workspace_bytes(T, I, O, N, 1, False)
    assert need > osdp.OSDP_NOALLOC_SCRATCH_BYTES
    with pytest.raises(osdp.OsdpError) as e:
        osdp.osdp_split_linear_fwd_noalloc(X, W, Y, 1)
    assert e.value.status == osdp.OSDP_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.isnan(Y).all(), "a refused call must leave Y untouched"
    osdp.osdp_split_linear_fwd_noalloc(X, W, Y, 4)   # 32 MiB slots: fits
    torch.cuda.synchronize()
    assert (Y == 0).all()
