"""Seeded synthetic inputs for the BLSTM training step.

This module only draws random numbers and reshapes them; it holds none of the
method's arithmetic.  It serves both the CPU oracle's tests and the HIP path's
harness, so that both sides see the very same arrays.

The tensors take the shapes of the paper's workload (section 4.2: 260-dim fused
features, 21-frame non-overlapping subsequences, 32 000 context-dependent
states); the speech corpora themselves are not needed for a dense model's cost
and are replaced by i.i.d. draws:

  x       [T, B, D]  i.i.d. N(0, 1)
  labels  [T, B]     uniform over the V classes, one per frame
  theta   [N]        U(-0.1, 0.1), every tensor including the biases
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np


@dataclass(frozen=True)
class Workload:
    """Shape of one training step (names follow the model description, section 4.2)."""

    name: str
    T: int          # frames per unrolled subsequence
    B: int          # subsequences per batch
    D: int          # input feature dimension
    H: int          # LSTM cells per direction
    L: int          # bidirectional layers
    P: int          # linear bottleneck width, 0 = none
    V: int          # softmax classes
    mode: int       # 0 = fp32, 1 = bf16 storage with fp32 accumulation
    lr: float
    seed: int

    def dims(self) -> dict:
        d = asdict(self)
        return {k: d[k] for k in ("T", "B", "D", "H", "L", "P", "V")}


# The five workloads named by the build's baseline description.
WORKLOADS = {
    "tiny": Workload("tiny", T=21, B=8, D=40, H=32, L=1, P=0, V=100, mode=0, lr=0.1, seed=1904),
    "paper4x512": Workload("paper4x512", T=21, B=256, D=260, H=512, L=4, P=256, V=32000,
                           mode=1, lr=0.1, seed=4956),
    "largebatch": Workload("largebatch", T=21, B=2048, D=260, H=512, L=4, P=256, V=32000,
                           mode=1, lr=0.1 * 2048 / 256, seed=4957),
    "wide6x1024": Workload("wide6x1024", T=21, B=512, D=260, H=1024, L=6, P=256, V=32000,
                           mode=1, lr=0.1 * 512 / 256, seed=4958),
    "adpsgd16": Workload("adpsgd16", T=21, B=128, D=260, H=512, L=4, P=256, V=32000,
                         mode=1, lr=0.1 * 128 / 256, seed=4956),
    # the model the paper itself timed (section 4.2), 6 layers of 512 cells per direction
    "paper6x512": Workload("paper6x512", T=21, B=256, D=260, H=512, L=6, P=256, V=32000,
                           mode=1, lr=0.1, seed=4959),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Return float32 values that are exactly representable in bfloat16.

    Round-to-nearest-even on the upper 16 bits of the IEEE-754 single.  This is
    input preparation only: in bf16 mode both sides start from these values.
    """
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(f.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits (uint16) of float32 values already representable in bf16."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    return (f.view(np.uint32) >> 16).astype(np.uint16).reshape(f.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def make_theta(n: int, seed: int, bf16: bool = False) -> np.ndarray:
    """Flat parameter vector, U(-0.1, 0.1), float32 (bf16-representable if asked)."""
    rng = np.random.default_rng(seed)
    th = rng.uniform(-0.1, 0.1, size=n).astype(np.float32)
    return round_to_bf16(th) if bf16 else th


def make_batch(T: int, B: int, D: int, V: int, seed: int, bf16: bool = False):
    """One batch: features x [T,B,D] float32 and labels [T,B] int32."""
    rng = np.random.default_rng(seed + 7919)
    x = rng.standard_normal(size=(T, B, D)).astype(np.float32)
    labels = rng.integers(0, V, size=(T, B), dtype=np.int64).astype(np.int32)
    if bf16:
        x = round_to_bf16(x)
    return x, labels
