"""Test-side glue: moves seeded bf16 bit patterns to the GPU, calls libosdp, brings results back."""
from __future__ import annotations

import numpy as np
import torch

import paper_2209_13258_amd as osdp


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> bf16 tensor on cuda:0 (same bits)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.cuda().view(torch.bfloat16)


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def widen(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


class Operator:
    """One linear operator resident on the GPU with its outputs and workspace."""

    def __init__(self, X, dY, W_shards, O, poison=True):
        self.T, self.I = X.shape
        self.O = O
        self.N = len(W_shards)
        self.X = to_dev(X)
        self.dY = to_dev(dY) if dY is not None else None
        self.W = [to_dev(s) for s in W_shards]
        self.L = W_shards[0].size
        fill = float("nan") if poison else 0.0
        self.Y = torch.full((self.T, O), fill, dtype=torch.bfloat16, device="cuda")
        self.dX = torch.full((self.T, self.I), fill, dtype=torch.bfloat16, device="cuda")
        self.dW = [torch.full((self.L,), fill, dtype=torch.bfloat16, device="cuda") for _ in range(self.N)]
        self.ws = None

    def workspace(self, k, is_bwd, plan=None, op_index=0):
        total, peak = osdp.osdp_split_linear_workspace_bytes(self.T, self.I, self.O, self.N, k, is_bwd, plan, op_index)
        if self.ws is None or self.ws.numel() < total:
            self.ws = torch.empty(max(total, 256), dtype=torch.uint8, device="cuda")
        return self.ws, peak

    def fwd(self, k, plan=None, op_index=0, streams=(None, None)):
        ws, _ = self.workspace(k, False, plan, op_index)
        sc, sp = streams
        osdp.osdp_split_linear_fwd(self.X, self.W, self.Y, k, ws, plan=plan, op_index=op_index,
                                   stream_compute=sc, stream_copy=sp)

    def bwd(self, k, plan=None, op_index=0, streams=(None, None)):
        ws, _ = self.workspace(k, True, plan, op_index)
        sc, sp = streams
        osdp.osdp_split_linear_bwd(self.X, self.dY, self.W, self.dX, self.dW, k, ws, plan=plan,
                                   op_index=op_index, stream_compute=sc, stream_copy=sp)

    def results(self):
        torch.cuda.synchronize()
        dW = np.concatenate([to_bits(s) for s in self.dW])[: self.I * self.O].reshape(self.I, self.O)
        return {"Y": to_bits(self.Y), "dX": to_bits(self.dX), "dW": dW}


def streams():
    """(compute, copy) torch streams at the default priority; the compute stream is made current by the caller."""
    return torch.cuda.Stream(), torch.cuda.Stream()


REL_TOL = 2e-2  # max relative error against the fp64 oracle (bf16 inputs, fp32 accumulation)


def assert_close(name, got_bits, ref_f64):
    """max|g - o| / max|o| <= 2e-2 and no element off by more than 2e-2*|o| + 2e-2*rms(o)."""
    g = widen(got_bits)
    assert np.isfinite(g).all(), f"{name}: non-finite values in the GPU result"
    err = np.abs(g - ref_f64)
    scale = np.abs(ref_f64).max()
    rms = np.sqrt(np.mean(ref_f64 ** 2))
    worst = err.max() / scale if scale > 0 else err.max()
    assert worst <= REL_TOL, f"{name}: max relative error {worst:.3e}"
    bad = err > REL_TOL * np.abs(ref_f64) + REL_TOL * rms
    assert not bad.any(), f"{name}: {int(bad.sum())} elements outside the element-wise bound"
    # what the arithmetic itself allows: one bf16 rounding of the result (half an ulp = 2^-9 relative,
    # taken as 2^-8 to cover values that round across a binade) plus fp32 accumulation error, which
    # stays far below 1e-3 of the output's rms for K up to 32768
    tight = err > 2.0 ** -8 * np.abs(ref_f64) + 1e-3 * rms
    assert not tight.any(), f"{name}: {int(tight.sum())} elements outside the rounding-error bound"
    return worst
