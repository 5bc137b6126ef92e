"""Seeded synthetic inputs for the token-filtered layer backward.

This module only draws random tensors and keep masks and names the layer
shapes.  It contains none of the method's arithmetic (no forward, no
backward): both the CPU oracle's tests and the GPU harness take their raw
inputs from here so that the two sides see identical data without sharing any
computational code.

Shapes are Llama-style decoder layers (RMSNorm, GQA causal attention, SwiGLU);
value distributions: weights N(0, 0.02^2), activations and upstream gradient
N(0, 1), RMSNorm gains 1 + N(0, 0.02^2).  Keep masks follow the selective-loss
indicator of the paper (Sec. 2.1, Eq. 2): 1 = token is kept, chosen as the
top-k of a per-token score; uniform scores stand in for the loss difference
that a trained reference model would supply.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np


@dataclasses.dataclass(frozen=True)
class LayerShape:
    name: str
    B: int      # sequences in the batch
    S: int      # tokens per sequence
    H: int      # hidden size
    Hq: int     # query heads
    Hkv: int    # key/value heads
    d: int      # head dim
    F: int      # SwiGLU width
    dtype: str  # "f32" or "bf16"
    rho: float = 0.5
    mask_kind: str = "topk"   # "topk" | "spans" | "ragged"

    @property
    def T(self) -> int:
        return self.B * self.S

    @property
    def Nq(self) -> int:
        return self.Hq * self.d

    @property
    def Nkv(self) -> int:
        return self.Hkv * self.d

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def P_layer(self) -> int:
        """Number of linear-layer parameters of one decoder layer."""
        return self.H * (self.Nq + 2 * self.Nkv) + self.Nq * self.H + 3 * self.H * self.F


# The five workload shapes of the benchmark contract (index = config number).
CONFIGS = (
    LayerShape("tiny_f32", B=2, S=128, H=256, Hq=4, Hkv=4, d=64, F=688, dtype="f32"),
    LayerShape("tinyllama_1b", B=4, S=2048, H=2048, Hq=32, Hkv=4, d=64, F=5632, dtype="bf16"),
    LayerShape("llama32_3b", B=2, S=4096, H=3072, Hq=24, Hkv=8, d=128, F=8192, dtype="bf16"),
    LayerShape("llama31_8b", B=2, S=4096, H=4096, Hq=32, Hkv=8, d=128, F=14336, dtype="bf16",
               mask_kind="spans"),
    LayerShape("dense_40b", B=1, S=8192, H=8192, Hq=64, Hkv=8, d=128, F=22016, dtype="bf16",
               mask_kind="ragged"),
)


def config_seed(index: int) -> int:
    return 340 * 1000 + index


def topk_count(rho: float, S: int) -> int:
    """Kept tokens per sequence for keep ratio rho: round-half-up of rho*S."""
    return int(math.floor(rho * S + 0.5))


# --------------------------------------------------------------------------
# keep masks (uint8, 1 = kept)
# --------------------------------------------------------------------------

def mask_topk(rng: np.random.Generator, B: int, S: int, rho: float) -> np.ndarray:
    """Per sequence, keep the k highest of S i.i.d. uniform scores (ties: the
    lower position wins, via a stable sort on the negated score)."""
    k = topk_count(rho, S)
    mask = np.zeros((B, S), dtype=np.uint8)
    for b in range(B):
        u = rng.random(S)
        order = np.argsort(-u, kind="stable")
        mask[b, order[:k]] = 1
    return mask


def mask_spans(rng: np.random.Generator, B: int, S: int, rho: float,
               lo: int = 8, hi: int = 64) -> np.ndarray:
    """Kept tokens arrive in contiguous runs: alternate kept / filtered runs
    with lengths uniform in [lo, hi] from a random start state, then flip
    tokens next to run boundaries until the sequence holds exactly k kept."""
    k = topk_count(rho, S)
    mask = np.zeros((B, S), dtype=np.uint8)
    for b in range(B):
        row = np.zeros(S, dtype=np.uint8)
        state = int(rng.integers(0, 2))
        pos = 0
        while pos < S:
            run = int(rng.integers(lo, hi + 1))
            row[pos:pos + run] = state
            pos += run
            state ^= 1
        # repair the count by growing / shrinking runs at their boundaries
        guard = 0
        while int(row.sum()) != k and guard < 16 * S:
            guard += 1
            have = int(row.sum())
            want = 1 if have < k else 0           # value we need more of
            edges = np.flatnonzero(row[1:] != row[:-1]) + 1   # first index of each new run
            if edges.size == 0:
                j = int(rng.integers(0, S))
                row[j] = want
                continue
            e = int(edges[int(rng.integers(0, edges.size))])
            # at a boundary, one side has value `want`: extend it by one token
            if row[e] == want:
                row[e - 1] = want
            else:
                row[e] = want
        mask[b] = row
    return mask


def mask_ragged(rng: np.random.Generator, B: int, S: int, segments: int = 8,
                lo: float = 0.2, hi: float = 0.8) -> np.ndarray:
    """Each sequence is a pack of `segments` equal pieces whose kept fractions
    are a random permutation of linspace(lo, hi, segments) (mean 0.5); within
    a piece the kept tokens are the top-k of uniform scores."""
    assert S % segments == 0
    L = S // segments
    mask = np.zeros((B, S), dtype=np.uint8)
    for b in range(B):
        fr = rng.permutation(np.linspace(lo, hi, segments))
        for s in range(segments):
            k = topk_count(float(fr[s]), L)
            u = rng.random(L)
            order = np.argsort(-u, kind="stable")
            mask[b, s * L + order[:k]] = 1
    return mask


def make_mask(shape: LayerShape, rng: np.random.Generator, rho: float | None = None,
              kind: str | None = None) -> np.ndarray:
    rho = shape.rho if rho is None else rho
    kind = shape.mask_kind if kind is None else kind
    if kind == "topk":
        return mask_topk(rng, shape.B, shape.S, rho)
    if kind == "spans":
        return mask_spans(rng, shape.B, shape.S, rho)
    if kind == "ragged":
        return mask_ragged(rng, shape.B, shape.S)
    raise ValueError(kind)


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to the nearest bfloat16 (ties to even) and return it
    widened back to fp32.  Pure bit manipulation; NaN/Inf are not expected."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def make_weights(shape: LayerShape, rng: np.random.Generator) -> dict:
    """Layer parameters, fp32, stored [in, out] row-major (Y = X @ W)."""
    def w(i, o):
        return (rng.standard_normal((i, o), dtype=np.float32) * np.float32(0.02))
    p = {
        "wq": w(shape.H, shape.Nq), "wk": w(shape.H, shape.Nkv), "wv": w(shape.H, shape.Nkv),
        "wo": w(shape.Nq, shape.H),
        "wg": w(shape.H, shape.F), "wu": w(shape.H, shape.F), "wd": w(shape.F, shape.H),
        "g1": (1.0 + 0.02 * rng.standard_normal(shape.H, dtype=np.float32)).astype(np.float32),
        "g2": (1.0 + 0.02 * rng.standard_normal(shape.H, dtype=np.float32)).astype(np.float32),
    }
    return p


def make_normal(rng: np.random.Generator, *dims: int) -> np.ndarray:
    return rng.standard_normal(dims, dtype=np.float32)


def make_independent_activations(shape: LayerShape, rng: np.random.Generator) -> dict:
    """Saved activations drawn independently N(0,1) ("independent" input mode):
    x, r, q, k, v, gate, up.  attn_out and lse are NOT drawn here: they have to
    be consistent with (q, k, v) and are derived by a forward fixture that the
    caller owns."""
    return {
        "x": make_normal(rng, shape.T, shape.H),
        "r": make_normal(rng, shape.T, shape.H),
        "q": make_normal(rng, shape.T, shape.Nq),
        "k": make_normal(rng, shape.T, shape.Nkv),
        "v": make_normal(rng, shape.T, shape.Nkv),
        "gate": make_normal(rng, shape.T, shape.F),
        "up": make_normal(rng, shape.T, shape.F),
    }


def rope_tables(S: int, d: int, base: float = 10000.0):
    """cos / sin tables [S, d/2] fp32 of the rotary position embedding: angle of
    position s and frequency i is s * base^(-2i/d)."""
    inv = base ** (-np.arange(0, d, 2, dtype=np.float64) / d)
    ang = np.outer(np.arange(S, dtype=np.float64), inv)
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def make_lora(shape: LayerShape, rng: np.random.Generator, rank: int = 64, alpha: float = 128.0) -> dict:
    """Low-rank adapters of the q, k, v, o projections (the paper's LoRA setting:
    rank 64 on the attention projections): a_p [in, rank], b_p [rank, out],
    both N(0, 0.02^2) so that every gradient path carries signal (a trained
    adapter has a non-zero b), scale = alpha / rank."""
    dims = {"q": (shape.H, shape.Nq), "k": (shape.H, shape.Nkv), "v": (shape.H, shape.Nkv), "o": (shape.Nq, shape.H)}
    out = {"scale": float(alpha) / rank, "rank": rank}
    for p, (i, o) in dims.items():
        out["a" + p] = rng.standard_normal((i, rank), dtype=np.float32) * np.float32(0.02)
        out["b" + p] = rng.standard_normal((rank, o), dtype=np.float32) * np.float32(0.02)
    return out
