"""Seeded synthetic inputs and workload shapes for the operator-split linear layer.

This module is shared by the CPU oracle's tests and the GPU harness and holds
none of the method's arithmetic: it only names shapes and draws random bf16
bit patterns.  The same uint16 arrays are handed to both sides.

Shapes follow the GPT-like models of the paper (Table 1: hidden sizes 1024 to
12288, feed-forward width 4h, the 12288 x 49152 MatMul of Section 3.3); the
paper names no dataset and states no batch or sequence length, so token counts
are chosen here.  Weights are N(0, 0.02^2), activations and upstream gradients
N(0, 1), drawn in fp32 and rounded to bf16 (round to nearest even).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

ROOT_SEED = 220913258

KIND_X, KIND_DY, KIND_W, KIND_PLAN = 0, 1, 2, 3


@dataclass(frozen=True)
class Op:
    name: str
    I: int  # in-features
    O: int  # out-features
    k: int  # slice granularity of this operator in the workload's plan


@dataclass(frozen=True)
class Workload:
    cfg: int            # 1-based index into the benchmark's configs
    name: str
    T: int              # tokens (rows of X)
    N: int              # shard count
    ops: Tuple[Op, ...]
    layers: int = 1
    k_sweep: Tuple[int, ...] = ()


def _ffn(h, ffn, k):
    return (Op("up", h, ffn, k), Op("down", ffn, h, k))


def _layer(h, ffn, ks):
    return (Op("qkv", h, 3 * h, ks[0]), Op("proj", h, h, ks[1]),
            Op("up", h, ffn, ks[2]), Op("down", ffn, h, ks[3]))


def rng(cfg: int, layer: int, op: int, kind: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([ROOT_SEED, cfg, layer, op, kind])))


def config5_plan() -> Tuple[int, ...]:
    """Seeded random plan vector over the four operators of config 5 (one draw, all layers)."""
    return tuple(int(v) for v in rng(5, 0, 0, KIND_PLAN).choice([1, 2, 4, 8], size=4))


def workload(cfg: int, k: int | None = None) -> Workload:
    """Workload ``cfg`` (1..5). ``k`` overrides the split count where the config sweeps it."""
    if cfg == 1:
        return Workload(1, "single-split-linear-256x1024", 128, 2, (Op("lin", 256, 1024, k or 4),), 1, (4,))
    if cfg == 2:
        return Workload(2, "gpt-ffn-h1024-t8192", 8192, 8, _ffn(1024, 4096, k or 4), 1, (1, 2, 4, 8))
    if cfg == 3:
        ks = (2, 1, 4, 4) if k is None else (k,) * 4
        return Workload(3, "gpt-layer-h2560-t16384", 16384, 8, _layer(2560, 10240, ks), 1, ())
    if cfg == 4:
        return Workload(4, "wide-ffn-h8192-t4096", 4096, 8, _ffn(8192, 32768, k or 8), 1, (4, 8, 16))
    if cfg == 5:
        ks = config5_plan() if k is None else (k,) * 4
        return Workload(5, "gpt-layer-h4096-t8192-x4", 8192, 8, _layer(4096, 16384, ks), 4, ())
    raise ValueError(f"unknown config {cfg}")


def flops(w: Workload) -> int:
    """Forward + backward flops of the whole workload: 6*T*I*O per operator per layer."""
    return w.layers * sum(6 * w.T * op.I * op.O for op in w.ops)


# ----------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(gen: np.random.Generator, shape, std: float) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for a in range(0, n, step):  # chunked so that the fp32 temporary stays small
        b = min(n, a + step)
        out[a:b] = f32_to_bf16_bits(gen.standard_normal(b - a, dtype=np.float32) * np.float32(std))
    return out.reshape(shape)


# ------------------------------------------------------------ operator inputs
def shard_elems(I: int, O: int, N: int) -> int:
    """Elements per shard buffer when I*O weights are cut into N equal flat pieces."""
    return -(-(I * O) // N)


def operator_inputs(cfg: int, layer: int, op_index: int, T: int, I: int, O: int, N: int,
                    need=("X", "dY", "W")) -> Dict[str, object]:
    """Seeded inputs of one operator: X [T x I], dY [T x O] and the N weight shards.

    The weight is drawn shard by shard (each a flat buffer of ``shard_elems``
    bf16 values), so the shards themselves are the given data; whatever lies in
    the last shard beyond I*O elements is padding that no consumer may read.
    """
    out: Dict[str, object] = {}
    if "X" in need:
        out["X"] = normal_bf16(rng(cfg, layer, op_index, KIND_X), (T, I), 1.0)
    if "dY" in need:
        out["dY"] = normal_bf16(rng(cfg, layer, op_index, KIND_DY), (T, O), 1.0)
    if "W" in need:
        g = rng(cfg, layer, op_index, KIND_W)
        L = shard_elems(I, O, N)
        out["W_shards"] = [normal_bf16(g, (L,), 0.02) for _ in range(N)]
    return out


def small_case(seed: int, T: int, I: int, O: int, N: int, w_std: float = 0.02):
    """Inputs for ad-hoc test shapes (not one of the five configs)."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([ROOT_SEED, 99, seed, T, I, O, N])))
    L = shard_elems(I, O, N)
    return {
        "X": normal_bf16(g, (T, I), 1.0),
        "dY": normal_bf16(g, (T, O), 1.0),
        "W_shards": [normal_bf16(g, (L,), w_std) for _ in range(N)],
    }


def tiled_case(seed: int, T: int, I: int, O: int, N: int, period: int, w_std: float = 0.02):
    """Inputs for index-width tests on very large weights: ``period`` weights are drawn as in ``small_case``
    and repeated to fill the N shards (drawing billions of values would take minutes and adds nothing to
    such a test).  Choose a period that does not divide 2^31 or 2^32, so that an index that wraps at either
    width lands on a different value."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([ROOT_SEED, 98, seed, T, I, O, N])))
    L = shard_elems(I, O, N)
    X = normal_bf16(g, (T, I), 1.0)
    dY = normal_bf16(g, (T, O), 1.0)
    block = normal_bf16(g, (period,), w_std)
    flat = np.resize(block, N * L)
    return {"X": X, "dY": dY, "W_shards": [flat[s * L:(s + 1) * L] for s in range(N)]}
