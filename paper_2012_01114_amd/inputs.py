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


# Key-level profiles for make_level_inputs: nats added to every score of key j (n keys).
def _levels_ramp(n: int) -> np.ndarray:
    """Falls linearly from 60 at key 0 to 0 at key n-1: along a walk towards key 0 the largest
    score of a row keeps growing, by far more than any fixed slack."""
    return 60.0 * (1.0 - np.arange(n) / max(n - 1, 1))


def _levels_steps(n: int) -> np.ndarray:
    """Three plateaus, 18 / 9 / 0 nats for keys [0, 8) / [8, 40) / [40, n): each step up outweighs
    everything met before it by a few hundred times per key, while the many keys of the lower
    plateau keep a share of the row sum that a wrong rescaling would multiply."""
    lv = np.zeros(n)
    lv[:40] = 9.0
    lv[:8] = 18.0
    return lv


LEVEL_PROFILES = {"ramp": _levels_ramp, "steps": _levels_steps}


def make_level_inputs(w: Workload, profile: str, scale: float) -> Tuple[dict, dict]:
    """The draw of make_inputs with a designed level added to the scores of every key.

    Input channel 0 carries a constant c for every vector and feeds only one unit direction u of
    each head's q; channel 1 carries t_j and feeds only the same direction of k; neither reaches v.
    Every score of key j thus gains scale * c * t_j = LEVEL_PROFILES[profile](n)[j] nats on top of
    the random part, for every row alike, so the row maxima move along the key axis as designed.
    `scale` is the score scale the run will use (1/sqrt(d_k) by default)."""
    stored, f64 = make_inputs(w)
    rng = np.random.default_rng(w.seed + 77)
    levels = LEVEL_PROFILES[profile](w.n)
    c = 8.0
    x = f64["X"].copy()
    x[:, :, 0] = c
    x[:, :, 1] = levels[None, :] / (scale * c)
    ws = {k: f64[k].copy() for k in ("Wq", "Wk", "Wv")}
    for k in ws:
        ws[k][0:2, :] = 0.0
    for h in range(w.n_heads):
        u = rng.choice([-1.0, 1.0], size=w.d_k) / np.sqrt(w.d_k)   # |u| = 1
        ws["Wq"][0, h * w.d_k:(h + 1) * w.d_k] = u
        ws["Wk"][1, h * w.d_k:(h + 1) * w.d_k] = u
    for key, arr in (("X", x), ("Wq", ws["Wq"]), ("Wk", ws["Wk"]), ("Wv", ws["Wv"])):
        stored[key], f64[key] = round_to_storage(arr, w.dtype)
    return stored, f64
