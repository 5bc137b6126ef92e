"""Shared helpers of the GPU parity tests: build one seeded problem, hand the
same arrays to the CPU oracle and to the HIP library, compare.

Inputs follow the recipe of the benchmark contract: weights N(0, 0.02^2),
activations / upstream gradient N(0, 1), gains 1 + N(0, 0.02^2); in bf16
configurations every input is rounded to bf16 on the host first and the oracle
receives the rounded values widened to fp32/fp64, so the error measures the
compute path only."""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle import layer_oracle as O
from paper_2502_00340_amd import binding as Bn
from paper_2502_00340_amd import workloads as WL

SAVED = ("x", "q", "k", "v", "attn_out", "lse", "r", "gate", "up")
WEIGHTS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")
GRADS = ("dwq", "dwk", "dwv", "dwo", "dwg", "dwu", "dwd", "dg1", "dg2")

# tolerances of the benchmark contract: relative Frobenius error per gradient tensor
TOL = {"bf16": 2e-2, "f32": 1e-4}
# per-row / per-column bound (see line_err): a single wrong row, column or tile edge of a large
# tensor hardly moves the Frobenius norm of the whole tensor, but it moves its own row's
TOL_LINE = {"bf16": 5e-2, "f32": 1e-3}


def rel_fro(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    if den == 0.0:
        return float(np.linalg.norm(got))
    return float(np.linalg.norm(got - ref) / den)


def line_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Worst row and worst column of a matrix: max over rows of
    ||got_row - ref_row|| / max(||ref_row||, median row norm), the same over columns, the larger of
    the two.  The median in the denominator keeps rows that are (nearly) zero in the reference from
    blowing the ratio up."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.ndim != 2 or ref.size == 0:
        return rel_fro(got, ref)
    worst = 0.0
    for axis in (1, 0):
        num = np.sqrt(np.sum((got - ref) ** 2, axis=axis))
        den = np.sqrt(np.sum(ref ** 2, axis=axis))
        floor = float(np.median(den))
        den = np.maximum(den, floor if floor > 0.0 else 1.0)
        worst = max(worst, float(np.max(num / den)))
    return worst


def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    return WL.round_to_bf16(a) if dtype == "bf16" else a


def to_dev(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


class Problem:
    """One layer-backward problem as numpy arrays (already quantised to the
    storage dtype) plus the oracle's keyword arguments."""

    def __init__(self, shape: WL.LayerShape, seed: int, mode: str, mask: np.ndarray | None = None,
                 rho: float | None = None, oracle_dtype=np.float64, rope: bool = False):
        self.shape = shape
        self.dtype = shape.dtype
        rng = np.random.default_rng(seed)
        q = lambda a: quantize(a, shape.dtype)
        self.W = {k: q(v) for k, v in WL.make_weights(shape, rng).items()}
        self.kw = dict(B=shape.B, S=shape.S, Hq=shape.Hq, Hkv=shape.Hkv, d=shape.d)
        scale = 1.0 / math.sqrt(shape.d)
        # rotary tables (fp32 on both sides); in "independent" mode q and k are drawn directly, which
        # stands for already rotated tensors
        self.rope = WL.rope_tables(shape.S, shape.d) if rope else None
        if mode == "consistent":
            x = q(WL.make_normal(rng, shape.T, shape.H))
            _, sv = O.layer_fwd(x.astype(oracle_dtype), {k: v.astype(oracle_dtype) for k, v in self.W.items()},
                                rope=self.rope, **self.kw)
            self.saved = {k: (np.asarray(v, dtype=np.float32) if k == "lse" else q(v)) for k, v in sv.items()}
        elif mode == "independent":
            sv = {k: q(v) for k, v in WL.make_independent_activations(shape, rng).items()}
            a, lse = O.attn_fwd(sv["q"].astype(oracle_dtype), sv["k"].astype(oracle_dtype),
                                sv["v"].astype(oracle_dtype), scale=scale, **self.kw)
            sv["attn_out"] = q(a)
            sv["lse"] = np.asarray(lse, dtype=np.float32)
            self.saved = sv
        else:
            raise ValueError(mode)
        self.dy = q(WL.make_normal(rng, shape.T, shape.H))
        self.mask = WL.make_mask(shape, rng, rho=rho) if mask is None else mask
        self.oracle_dtype = oracle_dtype

    def oracle(self, dense=False):
        dt = self.oracle_dtype
        sv = {k: v.astype(dt) for k, v in self.saved.items()}
        W = {k: v.astype(dt) for k, v in self.W.items()}
        return O.layer_bwd(sv, W, self.dy.astype(dt), None if dense else self.mask, rope=self.rope, **self.kw)

    def device_tensors(self, device="cuda:0"):
        sv = {k: (torch.from_numpy(v).to(device) if k == "lse" else to_dev(v, self.dtype, device))
              for k, v in self.saved.items()}
        if self.rope is not None:
            sv["rope_cos"] = torch.from_numpy(self.rope[0]).to(device)
            sv["rope_sin"] = torch.from_numpy(self.rope[1]).to(device)
        W = {k: to_dev(v, self.dtype, device) for k, v in self.W.items()}
        dy = to_dev(self.dy, self.dtype, device)
        mask = torch.from_numpy(self.mask).to(device)
        return sv, W, dy, mask

    def desc(self):
        s = self.shape
        return Bn.make_desc(s.B, s.S, s.H, s.Hq, s.Hkv, s.d, s.F, s.dtype)


def check_layer(problem: Problem, got: dict, ref: dict, idx: np.ndarray | None, tol: float):
    """Compare GPU gradients with the oracle's.  idx None: dense dx.  Every tensor must meet the
    relative Frobenius tolerance `tol` and, row by row and column by column, the looser line bound."""
    errs, lines = {}, {}
    for name in GRADS:
        g = to_np(got[name])
        errs[name] = rel_fro(g, ref[name])
        lines[name] = line_err(g, ref[name])
    dx = to_np(got["dx"])
    if idx is None:
        rdx = ref["dx"]
    else:
        rdx = ref["dx"][idx]
        dead = np.ones(ref["dx"].shape[0], dtype=bool)
        dead[idx] = False
        assert np.all(ref["dx"][dead] == 0.0)
    errs["dx"] = rel_fro(dx, rdx)
    lines["dx"] = line_err(dx, rdx)
    bad = {k: v for k, v in errs.items() if not (v <= tol)}
    assert not bad, "relative Frobenius error above %g: %s (all: %s)" % (tol, bad, errs)
    tol_line = TOL_LINE[problem.dtype]
    bad = {k: v for k, v in lines.items() if not (v <= tol_line)}
    assert not bad, "worst row/column error above %g: %s (all: %s)" % (tol_line, bad, lines)
    errs["worst_line"] = max(lines.values())
    return errs
