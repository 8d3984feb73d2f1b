"""Seeded synthetic inputs for the self-attention path.

This module only draws random numbers, scales them and rounds them to the
storage type.  It contains none of the method's arithmetic and is the one
module that both the GPU path and the CPU checker are fed from.

The paper (Sec. 3.1) takes n d-dimensional input vectors x and three learned
projection matrices; it names no dataset, so every workload here is synthetic:
X ~ N(0, 1), W ~ N(0, 1/d_model) (variance), drawn from numpy's PCG64 in the
fixed order X, Wq, Wk, Wv.  Key lengths of the padded workload come from a
separate generator so that they do not depend on the tensor draws.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

SCHEME_FULL = 0       # original definition, every pair (Sec. 3)
SCHEME_SYMMETRIC = 1  # q = k = v, symmetric score matrix (Sec. 4)
SCHEME_CAUSAL = 2     # masked self-attention, j <= i (Sec. 5)

SCHEME_NAMES = {SCHEME_FULL: "full", SCHEME_SYMMETRIC: "symmetric", SCHEME_CAUSAL: "causal"}

BASE_SEED = 201201114
LENGTH_SEED = 201202119


@dataclass(frozen=True)
class Workload:
    """Shape of one self-attention call.  `p` is the number of ring partitions
    (the paper's m PEs); the paper requires n divisible by it (abstract)."""
    name: str
    batch: int
    n: int
    d_model: int
    n_heads: int
    d_k: int
    p: int
    dtype: str            # "f32" or "bf16": storage type of X, W and out
    scheme: int
    seed: int
    padded: bool = False  # draw per-batch key lengths in [len_lo, len_hi]
    len_lo: int = 0
    len_hi: int = 0

    @property
    def hd(self) -> int:
        return self.n_heads * self.d_k


# The five workloads.  P of the padded one is not given with it; 256 keeps the
# 8-row partitions of the encoder/decoder shapes.
WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 16, 64, 1, 64, 4, "f32", SCHEME_FULL, BASE_SEED + 1),
    "encoder": Workload("encoder", 8, 512, 768, 12, 64, 64, "bf16", SCHEME_FULL, BASE_SEED + 2),
    "causal": Workload("causal", 8, 1024, 768, 12, 64, 128, "bf16", SCHEME_CAUSAL, BASE_SEED + 3),
    "long": Workload("long", 1, 8192, 4096, 32, 128, 256, "bf16", SCHEME_CAUSAL, BASE_SEED + 4),
    "padded": Workload("padded", 32, 2048, 1024, 16, 64, 256, "bf16", SCHEME_CAUSAL, BASE_SEED + 5,
                       padded=True, len_lo=64, len_hi=2048),
}


def with_scheme(w: Workload, scheme: int) -> Workload:
    return replace(w, scheme=scheme)


def round_to_storage(a64: np.ndarray, dtype: str):
    """Round a float64 array once to the storage type (round-to-nearest-even).

    Returns (stored, as_f64): `stored` is a torch CPU tensor of the storage
    type; `as_f64` is the same rounded values widened back to float64, so that
    input quantisation is shared by every consumer."""
    import torch

    t32 = torch.from_numpy(np.ascontiguousarray(a64, dtype=np.float32))
    if dtype == "f32":
        stored = t32
    elif dtype == "bf16":
        stored = t32.to(torch.bfloat16)
    else:
        raise ValueError(f"unknown dtype {dtype!r}")
    as_f64 = stored.to(torch.float64).numpy()
    return stored, as_f64


def draw_lengths(w: Workload) -> Optional[np.ndarray]:
    """Per-batch number of valid keys, uniform in [len_lo, len_hi]."""
    if not w.padded:
        return None
    rng = np.random.default_rng(LENGTH_SEED)
    return rng.integers(w.len_lo, w.len_hi + 1, w.batch).astype(np.int32)


def make_inputs(w: Workload, zero_wq: bool = False) -> Tuple[dict, dict]:
    """Draw one workload.

    Returns (stored, f64): two dicts with keys X [B,N,D], Wq, Wk, Wv [D,H*d_k]
    (row-major, q = x.W) and `lens` (int32 [B] or None).  `stored` holds torch
    CPU tensors of the storage type, `f64` holds numpy float64 arrays with the
    identical (already rounded) values.  `zero_wq` replaces Wq by zeros after
    the draw, for the uniform-weights special case."""
    rng = np.random.default_rng(w.seed)
    x = rng.standard_normal((w.batch, w.n, w.d_model))
    ws = [rng.standard_normal((w.d_model, w.hd)) * (w.d_model ** -0.5) for _ in range(3)]
    if zero_wq:
        ws[0] = np.zeros_like(ws[0])
    stored, f64 = {}, {}
    for key, arr in zip(("X", "Wq", "Wk", "Wv"), [x] + ws):
        stored[key], f64[key] = round_to_storage(arr, w.dtype)
    lens = draw_lengths(w)
    stored["lens"] = lens
    f64["lens"] = lens
    return stored, f64
