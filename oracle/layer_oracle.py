"""CPU oracle for the token-filtered backward pass of one decoder layer.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this file;
it exists so that tests, the smoke check and the benchmark's cpu_baseline leg
can compare the HIP library against a plain definition.  It shares no code
with the HIP path and imports nothing from it.

What is computed (paper Sec. 3.1, Eq. 3-4, and Sec. 3.2): the ordinary dense
backward of a Llama-style decoder layer with two row-masking points,

  (1) the upstream gradient of every filtered token is set to zero
      (Sec. 3.2: the gradient matrix G is row-wise sparse), and
  (2) the key- and value-gradient rows of filtered tokens are dropped at the
      output of the attention backward (Sec. 3.1: dK and dV are produced for
      the remaining tokens only, while dQ of a kept query still uses every
      key and value it attended to in the forward pass).

The method reaches this result by shrinking the sequence dimension; the
result itself has the plain definition above, so the oracle is that
definition written out over ALL T rows with the mask applied by
multiplication.  There is no compaction, no tiling and no fusion in here.

All arithmetic runs in the dtype of the arrays passed in (use float64 for
pins and finite differences).  numpy.matmul, exp and sum are the only library
primitives.

Layouts: tokens are flat rows t = b*S + s.  x, r: [T,H]; q, attn_out: [T,Hq*d];
k, v: [T,Hkv*d]; gate, up: [T,F]; lse: [B,Hq,S].  Weights are [in,out]
row-major, Y = X @ W.  Query head h uses key/value head h // (Hq/Hkv).

Readings of the paper taken here (each is listed in the design notes):
softmax scale 1/sqrt(d) multiplies the scores (prose of Sec. 3.1; the scale is
absent from Eq. 3-4); attention is causal on original positions; D_i is the
row sum of dO*O as in the FlashAttention backward that the paper says it
follows; LSE is the forward's, over the full key row; mask 1 = kept.

Parity status: every function below is pinned in tests/test_oracle_*.py by
finite differences, closed forms, brute force or library routines.
"""
from __future__ import annotations

import numpy as np


# ---------------------------------------------------------------------------
# index and gather (Sec. 3.2: "shrink the sequence dimension")
# ---------------------------------------------------------------------------

def keep_index(mask: np.ndarray):
    """Ascending flat positions of the kept tokens, the number of kept tokens
    in all earlier sequences for every sequence, and the total.

    mask: uint8 [B,S], 1 = kept.  Returns (idx int32 [N_k], cu_kept int32
    [B+1], N_k)."""
    B, S = mask.shape
    idx = []
    cu = [0]
    for b in range(B):
        for s in range(S):
            if mask[b, s] != 0:
                idx.append(b * S + s)
        cu.append(len(idx))
    return np.asarray(idx, dtype=np.int32), np.asarray(cu, dtype=np.int32), len(idx)


def gather_rows(src: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """dst[j,:] = src[idx[j],:]."""
    dst = np.empty((len(idx),) + src.shape[1:], dtype=src.dtype)
    for j in range(len(idx)):
        dst[j] = src[int(idx[j])]
    return dst


# ---------------------------------------------------------------------------
# forward (fixture for tests and finite differences)
# ---------------------------------------------------------------------------

def rmsnorm_fwd(x, g, eps):
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + x.dtype.type(eps))
    return x * rstd * g, rstd


def silu(z):
    return z / (1.0 + np.exp(-z))


def attn_fwd(q, k, v, B, S, Hq, Hkv, d, scale):
    """Causal softmax attention with grouped key/value heads.
    Returns (attn_out [T,Hq*d], lse [B,Hq,S])."""
    G = Hq // Hkv
    T = B * S
    out = np.zeros((T, Hq * d), dtype=q.dtype)
    lse = np.zeros((B, Hq, S), dtype=q.dtype)
    future = np.triu(np.ones((S, S), dtype=bool), k=1)      # j > i
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(Hq):
            g = h // G
            Q = q[rows, h * d:(h + 1) * d]
            K = k[rows, g * d:(g + 1) * d]
            V = v[rows, g * d:(g + 1) * d]
            Sc = (Q @ K.T) * q.dtype.type(scale)
            Sc[future] = -np.inf
            m = Sc.max(axis=1, keepdims=True)
            l = m[:, 0] + np.log(np.exp(Sc - m).sum(axis=1))
            P = np.exp(Sc - l[:, None])
            out[rows, h * d:(h + 1) * d] = P @ V
            lse[b, h] = l
    return out, lse


def rope_fwd(x, cos, sin, B, S, heads, d):
    """Rotary position embedding of every head of x [T, heads*d]: the pair
    (i, i + d/2) of a head is rotated by the angle of (position, frequency i);
    cos, sin: [S, d/2].  (Not in the paper; the model families it evaluates use
    it, in this half-split pairing.)"""
    T = B * S
    out = np.empty_like(x)
    half = d // 2
    for t in range(T):
        c = cos[t % S].astype(x.dtype)
        s = sin[t % S].astype(x.dtype)
        for h in range(heads):
            lo = x[t, h * d:h * d + half]
            hi = x[t, h * d + half:(h + 1) * d]
            out[t, h * d:h * d + half] = lo * c - hi * s
            out[t, h * d + half:(h + 1) * d] = hi * c + lo * s
    return out


def rope_bwd(dy, cos, sin, B, S, heads, d):
    """Gradient of rope_fwd with respect to its input: the transposed rotation."""
    T = B * S
    out = np.empty_like(dy)
    half = d // 2
    for t in range(T):
        c = cos[t % S].astype(dy.dtype)
        s = sin[t % S].astype(dy.dtype)
        for h in range(heads):
            lo = dy[t, h * d:h * d + half]
            hi = dy[t, h * d + half:(h + 1) * d]
            out[t, h * d:h * d + half] = lo * c + hi * s
            out[t, h * d + half:(h + 1) * d] = hi * c - lo * s
    return out


def lora_linear(x, w, lora, p):
    """Y = X W, plus the low-rank adapter s * (X a_p) b_p when `lora` is given
    (Sec. 5.3: rank-64 adapters on the q, k, v and o projections; the paper gives
    no formula, this is the standard LoRA form).  lora: dict with a<p> [in,r],
    b<p> [r,out] and "scale"."""
    y = x @ w
    if lora is not None:
        y = y + (x @ lora["a" + p]) @ lora["b" + p] * x.dtype.type(lora["scale"])
    return y


def layer_fwd(x, W, B, S, Hq, Hkv, d, eps=1e-5, scale=None, rope=None, lora=None):
    """Decoder-layer forward.  Returns (y, saved) where saved holds exactly the
    tensors the backward is given: x, q, k, v, attn_out, lse, r, gate, up.
    rope: None or (cos, sin) tables [S, d/2]; q and k in `saved` are rotated.
    lora: None or the adapters of the q, k, v, o projections (see lora_linear)."""
    scale = (1.0 / np.sqrt(d)) if scale is None else scale
    h1, _ = rmsnorm_fwd(x, W["g1"], eps)
    q = lora_linear(h1, W["wq"], lora, "q")
    k = lora_linear(h1, W["wk"], lora, "k")
    v = lora_linear(h1, W["wv"], lora, "v")
    if rope is not None:
        q = rope_fwd(q, rope[0], rope[1], B, S, Hq, d)
        k = rope_fwd(k, rope[0], rope[1], B, S, Hkv, d)
    a, lse = attn_fwd(q, k, v, B, S, Hq, Hkv, d, scale)
    r = x + lora_linear(a, W["wo"], lora, "o")
    h2, _ = rmsnorm_fwd(r, W["g2"], eps)
    gate = h2 @ W["wg"]
    up = h2 @ W["wu"]
    y = r + (silu(gate) * up) @ W["wd"]
    saved = dict(x=x, q=q, k=k, v=v, attn_out=a, lse=lse, r=r, gate=gate, up=up)
    return y, saved


# ---------------------------------------------------------------------------
# backward building blocks
# ---------------------------------------------------------------------------

def linear_bwd(x, dy, w, keep=None):
    """Backward of Y = X @ W under row-sparse dY (Sec. 3.2: the two GEMM types
    G.W and G^T.X).  keep: [T] 0/1 or None.  Returns (dX, dW); dX rows of
    filtered tokens are zero, dW sums over kept tokens only."""
    if keep is not None:
        dy = dy * keep.astype(dy.dtype)[:, None]
    return dy @ w.T, x.T @ dy


def rmsnorm_bwd(dh, x, g, eps):
    """Gradient of h = x * rstd(x) * g.  Returns (dx, dg)."""
    H = x.shape[-1]
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + x.dtype.type(eps))
    n = x * rstd
    u = dh * g
    dx = rstd * (u - n * (np.sum(u * n, axis=-1, keepdims=True) / H))
    dg = np.sum(dh * n, axis=0)
    return dx, dg


def swiglu_bwd(d_act, gate, up):
    """Gradient of act = silu(gate) * up.  Returns (d_gate, d_up)."""
    sig = 1.0 / (1.0 + np.exp(-gate))
    d_gate = d_act * up * sig * (1.0 + gate * (1.0 - sig))
    d_up = d_act * gate * sig
    return d_gate, d_up


def attn_bwd(q, k, v, attn_out, lse, da, B, S, Hq, Hkv, d, scale, keep=None):
    """Attention backward with masking point (2).

    Every query row i takes part (rows whose da is zero contribute zeros), the
    probabilities are rebuilt from the forward's LSE, keys span the full causal
    row.  When keep is given, the dk/dv rows of tokens with keep == 0 are
    dropped (set to zero) before they are returned.  Returns (dq, dk, dv)."""
    G = Hq // Hkv
    T = B * S
    dq = np.zeros((T, Hq * d), dtype=q.dtype)
    dk = np.zeros((T, Hkv * d), dtype=q.dtype)
    dv = np.zeros((T, Hkv * d), dtype=q.dtype)
    future = np.triu(np.ones((S, S), dtype=bool), k=1)
    sc = q.dtype.type(scale)
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(Hq):
            g = h // G
            Q = q[rows, h * d:(h + 1) * d]
            K = k[rows, g * d:(g + 1) * d]
            V = v[rows, g * d:(g + 1) * d]
            O = attn_out[rows, h * d:(h + 1) * d]
            dO = da[rows, h * d:(h + 1) * d]
            P = np.exp((Q @ K.T) * sc - lse[b, h][:, None])
            P[future] = 0.0
            D = np.sum(dO * O, axis=1, keepdims=True)
            dP = dO @ V.T
            dS = P * (dP - D)
            dq[rows, h * d:(h + 1) * d] = (dS @ K) * sc
            dk[rows, g * d:(g + 1) * d] += (dS.T @ Q) * sc
            dv[rows, g * d:(g + 1) * d] += P.T @ dO
    if keep is not None:
        m = keep.astype(q.dtype)[:, None]
        dk = dk * m
        dv = dv * m
    return dq, dk, dv


# ---------------------------------------------------------------------------
# whole layer
# ---------------------------------------------------------------------------

def lora_linear_bwd(x, dy, w, lora, p):
    """Backward of lora_linear: returns (dX, dW, da, db); da, db are None without
    an adapter.  dX = dY W^T + s (dY b^T) a^T, da = s X^T (dY b^T), db = s (X a)^T dY."""
    dx, dw = linear_bwd(x, dy, w)
    if lora is None:
        return dx, dw, None, None
    a, b = lora["a" + p], lora["b" + p]
    sc = x.dtype.type(lora["scale"])
    t = dy @ b.T
    dx = dx + (t @ a.T) * sc
    return dx, dw, (x.T @ t) * sc, ((x @ a).T @ dy) * sc


def layer_bwd(saved, W, dy, mask, B, S, Hq, Hkv, d, eps=1e-5, scale=None, rope=None, lora=None):
    """Token-filtered backward of one decoder layer.

    saved: dict from layer_fwd (x, q, k, v, attn_out, lse, r, gate, up), or
    tensors of the same shapes drawn independently; W: weights; dy: [T,H]
    upstream gradient on ALL rows; mask: uint8 [B,S] (1 = kept) or None for
    the dense backward.  Returns a dict: dx [T,H] (zero on filtered rows),
    dwq, dwk, dwv, dwo, dwg, dwu, dwd, dg1, dg2.  Normalised activations and
    the SwiGLU product are rebuilt from the saved tensors, as the HIP path has
    to do as well.  rope: None or (cos, sin) [S, d/2] when saved q, k are rotated.
    lora: None or the adapters of the q, k, v, o projections; then the result also
    holds daq, dbq, ..., dao, dbo and dx includes the adapter paths (the base
    weight gradients are still returned; a LoRA trainer ignores them)."""
    scale = (1.0 / np.sqrt(d)) if scale is None else scale
    x, r, gate, up = saved["x"], saved["r"], saved["gate"], saved["up"]
    a = saved["attn_out"]
    T, H = x.shape
    dt = x.dtype
    keep = None if mask is None else mask.reshape(T)
    M = np.ones((T, 1), dtype=dt) if keep is None else keep.astype(dt)[:, None]

    # masking point (1)
    dy = dy * M

    # SwiGLU FFN:  y = r + act @ Wd
    act = silu(gate) * up
    d_act, dwd = linear_bwd(act, dy, W["wd"])
    d_gate, d_up = swiglu_bwd(d_act, gate, up)
    h2, _ = rmsnorm_fwd(r, W["g2"], eps)
    dh2_g, dwg = linear_bwd(h2, d_gate, W["wg"])
    dh2_u, dwu = linear_bwd(h2, d_up, W["wu"])
    dr_n, dg2 = rmsnorm_bwd(dh2_g + dh2_u, r, W["g2"], eps)
    dr = dy + dr_n

    # attention block:  r = x + attn_out @ Wo
    da, dwo, dao, dbo = lora_linear_bwd(a, dr, W["wo"], lora, "o")
    dq, dk, dv = attn_bwd(saved["q"], saved["k"], saved["v"], a, saved["lse"], da,
                          B, S, Hq, Hkv, d, scale, keep=keep)       # masking point (2)
    if rope is not None:        # saved q, k are the rotated tensors: undo the rotation on their gradients
        dq = rope_bwd(dq, rope[0], rope[1], B, S, Hq, d)
        dk = rope_bwd(dk, rope[0], rope[1], B, S, Hkv, d)
    h1, _ = rmsnorm_fwd(x, W["g1"], eps)
    dh1_q, dwq, daq, dbq = lora_linear_bwd(h1, dq, W["wq"], lora, "q")
    dh1_k, dwk, dak, dbk = lora_linear_bwd(h1, dk, W["wk"], lora, "k")
    dh1_v, dwv, dav, dbv = lora_linear_bwd(h1, dv, W["wv"], lora, "v")
    dx_n, dg1 = rmsnorm_bwd(dh1_q + dh1_k + dh1_v, x, W["g1"], eps)
    dx = dr + dx_n
    extra = {} if lora is None else dict(daq=daq, dbq=dbq, dak=dak, dbk=dbk, dav=dav, dbv=dbv, dao=dao, dbo=dbo)
    return dict(dx=dx, dwq=dwq, dwk=dwk, dwv=dwv, dwo=dwo, dwg=dwg, dwu=dwu, dwd=dwd,
                dg1=dg1, dg2=dg2, **extra,
                # intermediates, exposed for the per-entry-point parity tests
                _dr=dr, _da=da, _dq=dq, _dk=dk, _dv=dv)


def attn_bwd_filtered(q, k, v, attn_out, lse, da, mask, B, S, Hq, Hkv, d, scale=None):
    """Stand-alone attention backward as the HIP entry point defines it: da is
    taken on kept rows only (other rows are ignored, i.e. zeroed first), and
    dk/dv rows of filtered tokens are dropped.  Full-length [T,.] results."""
    scale = (1.0 / np.sqrt(d)) if scale is None else scale
    keep = mask.reshape(B * S)
    da = da * keep.astype(da.dtype)[:, None]
    return attn_bwd(q, k, v, attn_out, lse, da, B, S, Hq, Hkv, d, scale, keep=keep)
