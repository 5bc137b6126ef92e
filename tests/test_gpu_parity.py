"""GPU parity tests: every entry point of the C-ABI library against the CPU
oracle on identical seeded inputs.  Integer/byte results must be bit-exact;
floating-point results must stay within the relative Frobenius tolerance of
the benchmark contract (2e-2 in bf16, 1e-4 in the fp32 check mode)."""
import math

import numpy as np
import pytest
import torch

from oracle import layer_oracle as O
from paper_2502_00340_amd import binding as Bn
from paper_2502_00340_amd import workloads as WL
from tests import harness as Hn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


# ---------------------------------------------------------------------------
# A1 keep index
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("B,S,p", [
    (1, 1, 1.0), (1, 7, 0.5), (3, 17, 0.5), (2, 128, 0.5), (4, 2048, 0.5), (2, 4096, 0.3),
    (5, 1000, 0.7), (2, 333, 0.0), (2, 333, 1.0), (1, 8192, 0.5),
    (3, 40961, 0.5),          # above 8 blocks: two-kernel path, ragged tail
    (1, (1 << 20) + 17, 0.5),
    (8, 1 << 21, 0.5),        # 4096 blocks: every thread of the block-count scan owns several entries
])
def test_keep_index_bit_exact(B, S, p):
    say("keep_index B=%d S=%d p=%g" % (B, S, p))
    rng = np.random.default_rng(B * 7919 + S)
    mask = (rng.random((B, S)) < p).astype(np.uint8)
    if B * S > 64:
        mask.reshape(-1)[rng.integers(0, B * S, 5)] *= 255     # any non-zero byte counts as kept
    if B * S <= 200000:
        ridx, rcu, rn = O.keep_index(mask)
    else:   # the oracle's double loop is too slow here; its pins show it equals these library routines
        ridx = np.flatnonzero(mask.reshape(-1)).astype(np.int32)
        rcu = np.concatenate([[0], np.cumsum((mask != 0).sum(axis=1))]).astype(np.int32)
        rn = len(ridx)
    idx, cu, n_dev, n = Bn.build_keep_index(torch.from_numpy(mask).to(DEV))
    assert n == rn and int(n_dev.item()) == rn
    assert np.array_equal(cu.cpu().numpy(), rcu)
    assert np.array_equal(idx[:n].cpu().numpy(), ridx)


def test_keep_index_unaligned_mask_pointer():
    say("keep_index unaligned")
    rng = np.random.default_rng(5)
    raw = (rng.random(3 + 6 * 1001) < 0.5).astype(np.uint8)
    t = torch.from_numpy(raw).to(DEV)
    view = t[3:].view(6, 1001)
    ridx, rcu, rn = O.keep_index(raw[3:].reshape(6, 1001))
    idx, cu, _, n = Bn.build_keep_index(view)
    assert n == rn and np.array_equal(cu.cpu().numpy(), rcu) and np.array_equal(idx[:n].cpu().numpy(), ridx)


# ---------------------------------------------------------------------------
# A2 gather
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols,dtype,frac", [
    (256, 256, torch.float32, 0.5), (1000, 688, torch.float32, 0.5), (513, 6, torch.bfloat16, 0.5),
    (4096, 2048, torch.bfloat16, 0.5), (2048, 5632, torch.bfloat16, 0.3), (300, 8, torch.bfloat16, 1.0),
    (64, 14336, torch.bfloat16, 0.5), (100, 4, torch.float32, 0.0),
])
def test_gather_rows_bit_exact(rows, cols, dtype, frac):
    say("gather rows=%d cols=%d %s" % (rows, cols, dtype))
    rng = np.random.default_rng(rows + cols)
    src = torch.from_numpy(rng.standard_normal((rows, cols)).astype(np.float32)).to(DEV).to(dtype)
    keep = np.flatnonzero(rng.random(rows) < frac).astype(np.int32)
    idx = torch.from_numpy(keep).to(DEV)
    if len(keep) == 0:
        idx = torch.zeros(1, dtype=torch.int32, device=DEV)
    out = Bn.gather_rows(src, idx, len(keep))
    raw = src.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy()
    ref = O.gather_rows(raw, keep)
    got = out.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy()
    assert got.shape == ref.shape and np.array_equal(got, ref)


# ---------------------------------------------------------------------------
# A3 reduced linear backward
# ---------------------------------------------------------------------------

LINEAR_CASES = [
    # n_kept, in, out
    (128, 256, 688), (1, 8, 8), (77, 264, 200), (333, 64, 1024), (1000, 2048, 512),
    (257, 688, 256), (2867, 512, 1536),
    (4000, 4096, 1024),      # enough 256x256 tiles for the large-tile kernels (dX and dW)
    (2049, 3584, 4096),
    # more output tiles than CUs with ragged edges in both directions: blocks walk through several
    # tiles, the last round is cut into sub-tiles, some of which lie outside the matrix
    (520, 4232, 4360),
    # dX outputs that fill 256 CUs better as 256x192 tiles: one round with a ragged last tile column
    # (10 x 19 tiles), and two tiles per block (23 x 22 tiles)
    (2500, 3600, 264), (5700, 4200, 136),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_kept,fin,fout", LINEAR_CASES)
def test_linear_bwd_reduced(dtype, n_kept, fin, fout):
    say("linear %s n=%d in=%d out=%d" % (dtype, n_kept, fin, fout))
    rng = np.random.default_rng(n_kept + fin + fout)
    x = Hn.quantize(rng.standard_normal((n_kept, fin)), dtype)
    dy = Hn.quantize(rng.standard_normal((n_kept, fout)), dtype)
    w = Hn.quantize(rng.standard_normal((fin, fout)) * 0.02, dtype)
    rdx, rdw = O.linear_bwd(x.astype(np.float64), dy.astype(np.float64), w.astype(np.float64))
    dx, dw = Bn.linear_bwd_reduced(Hn.to_dev(x, dtype), Hn.to_dev(dy, dtype), Hn.to_dev(w, dtype))
    torch.cuda.synchronize()
    e1, e2 = Hn.rel_fro(Hn.to_np(dx), rdx), Hn.rel_fro(Hn.to_np(dw), rdw)
    say("  rel err dx %.3e dw %.3e" % (e1, e2))
    assert e1 <= Hn.TOL[dtype] and e2 <= Hn.TOL[dtype]
    # element-wise as well: no misplaced tile can hide inside a Frobenius norm
    tol_abs = (3e-2 if dtype == "bf16" else 1e-4)
    assert np.max(np.abs(Hn.to_np(dx) - rdx)) <= tol_abs * max(1.0, np.max(np.abs(rdx)))
    assert np.max(np.abs(Hn.to_np(dw) - rdw)) <= tol_abs * max(1.0, np.max(np.abs(rdw)))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_linear_dw_accumulate_and_empty(dtype):
    say("linear accumulate/empty %s" % dtype)
    rng = np.random.default_rng(3)
    n, fin, fout = 100, 72, 136
    x = Hn.quantize(rng.standard_normal((n, fin)), dtype)
    dy = Hn.quantize(rng.standard_normal((n, fout)), dtype)
    w = Hn.quantize(rng.standard_normal((fin, fout)), dtype)
    prev = Hn.quantize(rng.standard_normal((fin, fout)), dtype)
    acc = Hn.to_dev(prev, dtype)
    Bn.linear_bwd_reduced(Hn.to_dev(x, dtype), Hn.to_dev(dy, dtype), None, need_dx=False,
                          dw_accumulate_into=acc)
    ref = prev.astype(np.float64) + x.astype(np.float64).T @ dy.astype(np.float64)
    assert Hn.rel_fro(Hn.to_np(acc), ref) <= Hn.TOL[dtype]
    # dw only / dx only
    dx, dw = Bn.linear_bwd_reduced(None, Hn.to_dev(dy, dtype), Hn.to_dev(w, dtype), need_dw=False)
    assert dw is None and Hn.rel_fro(Hn.to_np(dx), dy.astype(np.float64) @ w.astype(np.float64).T) <= Hn.TOL[dtype]
    # no kept rows: dw = 0, dx has no rows
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    e = lambda c: torch.empty((0, c), dtype=tdt, device=DEV)
    dx0, dw0 = Bn.linear_bwd_reduced(e(fin), e(fout), Hn.to_dev(w, dtype))
    assert dx0.shape == (0, fin) and torch.count_nonzero(dw0).item() == 0
    keepacc = acc.clone()
    Bn.linear_bwd_reduced(e(fin), e(fout), None, need_dx=False, dw_accumulate_into=acc)
    assert torch.equal(acc, keepacc)


# ---------------------------------------------------------------------------
# A5 filtered attention backward
# ---------------------------------------------------------------------------

def _attn_case(dtype, B, S, Hq, Hkv, d, mask, seed, f8=np.float64):
    rng = np.random.default_rng(seed)
    T = B * S
    q = Hn.quantize(rng.standard_normal((T, Hq * d)), dtype)
    k = Hn.quantize(rng.standard_normal((T, Hkv * d)), dtype)
    v = Hn.quantize(rng.standard_normal((T, Hkv * d)), dtype)
    da = Hn.quantize(rng.standard_normal((T, Hq * d)), dtype)
    kw = dict(B=B, S=S, Hq=Hq, Hkv=Hkv, d=d)
    a, lse = O.attn_fwd(q.astype(f8), k.astype(f8), v.astype(f8), scale=1 / math.sqrt(d), **kw)
    a = Hn.quantize(a, dtype)
    lse = lse.astype(np.float32)
    rdq, rdk, rdv = O.attn_bwd_filtered(q.astype(f8), k.astype(f8), v.astype(f8), a.astype(f8),
                                        lse.astype(f8), da.astype(f8), mask, **kw)
    ridx, rcu, n = O.keep_index(mask)
    desc = Bn.make_desc(B, S, 8 * Hq, Hq, Hkv, d, 8, dtype)
    tidx = torch.from_numpy(ridx if n else np.zeros(1, np.int32)).to(DEV)
    sel = lambda arr: Hn.to_dev(arr[ridx], dtype)
    dq, dk, dv = Bn.attn_bwd_filtered(desc, sel(q), Hn.to_dev(k, dtype), Hn.to_dev(v, dtype), sel(a),
                                      torch.from_numpy(lse).to(DEV), sel(da), tidx,
                                      torch.from_numpy(rcu).to(DEV), n)
    torch.cuda.synchronize()
    errs = (Hn.rel_fro(Hn.to_np(dq), rdq[ridx]), Hn.rel_fro(Hn.to_np(dk), rdk[ridx]),
            Hn.rel_fro(Hn.to_np(dv), rdv[ridx]))
    say("  rel err dq %.3e dk %.3e dv %.3e (n_kept %d)" % (errs + (n,)))
    assert max(errs) <= Hn.TOL[dtype]
    # row by row and column by column: a wrong tail row or tile edge cannot hide in the norm of the tensor
    lines = (Hn.line_err(Hn.to_np(dq), rdq[ridx]), Hn.line_err(Hn.to_np(dk), rdk[ridx]),
             Hn.line_err(Hn.to_np(dv), rdv[ridx]))
    say("  worst row/column dq %.3e dk %.3e dv %.3e" % lines)
    assert max(lines) <= Hn.TOL_LINE[dtype]
    return errs


ATTN_SHAPES = [
    # B, S, Hq, Hkv, d
    (2, 128, 4, 4, 64),        # config 0 (MHA)
    (3, 200, 8, 2, 64),        # GQA, S not a tile multiple, ragged
    (2, 300, 4, 2, 128),
    (1, 1024, 4, 1, 128),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("B,S,Hq,Hkv,d", ATTN_SHAPES)
def test_attn_bwd_filtered_random_mask(dtype, B, S, Hq, Hkv, d):
    say("attn %s B=%d S=%d Hq=%d Hkv=%d d=%d" % (dtype, B, S, Hq, Hkv, d))
    rng = np.random.default_rng(S + d)
    mask = (rng.random((B, S)) < rng.uniform(0.2, 0.8, size=(B, 1))).astype(np.uint8)
    _attn_case(dtype, B, S, Hq, Hkv, d, mask, seed=S * 3 + d)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attn_bwd_filtered_degenerate_masks(dtype):
    B, S, Hq, Hkv, d = 3, 160, 4, 2, 64
    say("attn degenerate %s" % dtype)
    m = np.zeros((B, S), np.uint8)
    m[0, -1] = 1                       # only the last token of sequence 0; sequences 1, 2 empty
    _attn_case(dtype, B, S, Hq, Hkv, d, m, seed=1)
    m = np.ones((B, S), np.uint8)      # everything kept == dense attention backward
    _attn_case(dtype, B, S, Hq, Hkv, d, m, seed=2)
    m = np.zeros((B, S), np.uint8)
    m[1, 0] = 1                        # only the first token of the middle sequence
    m[2, 5:70] = 1                     # one contiguous span
    _attn_case(dtype, B, S, Hq, Hkv, d, m, seed=3)


LONG_ATTN_CASES = [
    # S, Hq, Hkv, d, mask kind: long sequences reach the unmasked steady-state steps of both kernels,
    # the span and ragged masks their tile edges; few heads keep the oracle's S x S matrices affordable
    (4096, 4, 2, 128, "spans"), (4096, 4, 1, 64, "ragged"), (8192, 2, 1, 128, "ragged"),
    (8192, 2, 2, 64, "spans"), (16384, 2, 1, 128, "topk"),
]


@pytest.mark.parametrize("S,Hq,Hkv,d,kind", LONG_ATTN_CASES)
def test_attn_bwd_filtered_long_context(S, Hq, Hkv, d, kind):
    say("attn long bf16 S=%d Hq=%d Hkv=%d d=%d %s" % (S, Hq, Hkv, d, kind))
    rng = np.random.default_rng(S + d + Hq)
    shape = WL.LayerShape("attn_long", B=1, S=S, H=8, Hq=Hq, Hkv=Hkv, d=d, F=8, dtype="bf16", rho=0.5,
                          mask_kind=kind)
    mask = WL.make_mask(shape, rng)
    _attn_case("bf16", 1, S, Hq, Hkv, d, mask, seed=S + 7 * d, f8=np.float32 if S > 4096 else np.float64)


@pytest.mark.parametrize("B,S,Hq,Hkv,d,kind,rho", [
    # enough key tiles that a dK/dV block takes several query heads of its KV group in a row
    # (the launcher wants about two blocks per CU of a 256-CU chip):
    (4, 2048, 16, 4, 64, "topk", 1.0),      # 64 key tiles x 16 heads: two heads per block, two partials per group
    (8, 2048, 8, 4, 128, "spans", 1.0),     # 128 x 8: the whole group of two in one block, no partials
    (8, 2048, 8, 4, 64, "topk", 1.0),       # the same at d = 64
    (12, 2048, 16, 2, 64, "ragged", 0.8),   # about 154 x 16, ragged sequences: four heads of a group of eight per block
])
def test_attn_bwd_filtered_heads_sharing_a_block(B, S, Hq, Hkv, d, kind, rho):
    say("attn bf16 heads per block B=%d S=%d Hq=%d Hkv=%d d=%d %s rho=%.1f" % (B, S, Hq, Hkv, d, kind, rho))
    rng = np.random.default_rng(B * S + Hq)
    shape = WL.LayerShape("attn_hp", B=B, S=S, H=8, Hq=Hq, Hkv=Hkv, d=d, F=8, dtype="bf16", rho=rho, mask_kind=kind)
    mask = np.ones((B, S), np.uint8) if rho >= 1.0 else WL.make_mask(shape, rng)
    _attn_case("bf16", B, S, Hq, Hkv, d, mask, seed=S + Hq + d, f8=np.float32)


def test_attn_fp32_small_head_dims():
    for d in (8, 32):
        say("attn f32 d=%d" % d)
        rng = np.random.default_rng(d)
        mask = (rng.random((2, 50)) < 0.5).astype(np.uint8)
        _attn_case("f32", 2, 50, 4, 2, d, mask, seed=d)


# ---------------------------------------------------------------------------
# whole layer
# ---------------------------------------------------------------------------

SMALL_BF16 = WL.LayerShape("small_bf16", B=2, S=320, H=256, Hq=4, Hkv=2, d=64, F=704, dtype="bf16")
SMALL_BF16_D128 = WL.LayerShape("small_bf16_d128", B=3, S=200, H=384, Hq=4, Hkv=1, d=128, F=520, dtype="bf16")


def _run_layer(problem, dense=False):
    sv, W, dy, mask = problem.device_tensors(DEV)
    desc = problem.desc()
    if dense:
        got = Bn.layer_bwd_dense(desc, sv, W, dy)
        torch.cuda.synchronize()
        return got, None, None
    got, idx, cu, n = Bn.layer_bwd_filtered(desc, sv, W, dy, mask)
    torch.cuda.synchronize()
    ridx, rcu, rn = O.keep_index(problem.mask)
    assert n == rn
    assert np.array_equal(idx.cpu().numpy(), ridx) and np.array_equal(cu.cpu().numpy(), rcu)
    return got, ridx, n


@pytest.mark.parametrize("mode", ["consistent", "independent"])
def test_layer_config0_tiny_fp32(mode):
    shape = WL.CONFIGS[0]
    say("layer %s %s" % (shape.name, mode))
    p = Hn.Problem(shape, WL.config_seed(0), mode)
    got, ridx, n = _run_layer(p)
    errs = Hn.check_layer(p, got, p.oracle(), ridx, Hn.TOL["f32"])
    say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    gotd, _, _ = _run_layer(p, dense=True)
    Hn.check_layer(p, gotd, p.oracle(dense=True), None, Hn.TOL["f32"])


# Hq*d and Hkv*d multiples of 256: the three projection dW run as one grouped launch
SMALL_BF16_GROUPED = WL.LayerShape("small_bf16_grouped", B=2, S=192, H=320, Hq=8, Hkv=4, d=64, F=384, dtype="bf16")


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_BF16_D128, SMALL_BF16_GROUPED], ids=lambda s: s.name)
@pytest.mark.parametrize("rho", [0.5, 0.3])
def test_layer_small_bf16(shape, rho):
    say("layer %s rho=%g" % (shape.name, rho))
    p = Hn.Problem(shape, 77, "independent", rho=rho)
    got, ridx, n = _run_layer(p)
    errs = Hn.check_layer(p, got, p.oracle(), ridx, Hn.TOL["bf16"])
    say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    gotd, _, _ = _run_layer(p, dense=True)
    Hn.check_layer(p, gotd, p.oracle(dense=True), None, Hn.TOL["bf16"])


def _random_layer_cases(seed, n):
    """Seeded random layer shapes: every size a multiple of 8 only, all head-group ratios, both head
    dims, every mask kind and keep ratio, with and without rotary tables."""
    rng = np.random.default_rng(seed)
    out = []
    for it in range(n):
        d = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 4]))
        Hq = Hkv * int(rng.choice([1, 2, 4]))
        out.append(dict(
            shape=WL.LayerShape("rand%d" % it, B=int(rng.integers(1, 4)), S=int(rng.choice([64, 128, 200, 256, 320, 512])),
                                H=8 * int(rng.integers(8, 96)), Hq=Hq, Hkv=Hkv, d=d, F=8 * int(rng.integers(8, 160)),
                                dtype="bf16" if rng.random() < 0.7 else "f32",
                                rho=float(rng.choice([0.1, 0.3, 0.5, 0.7, 0.9, 1.0])),
                                mask_kind=str(rng.choice(["topk", "spans", "ragged"]))),
            rope=bool(rng.random() < 0.3), seed=7000 + it))
    return out


@pytest.mark.parametrize("case", _random_layer_cases(2024, 14), ids=lambda c: c["shape"].name)
def test_layer_random_shapes(case):
    shape = case["shape"]
    say("layer random %s: B=%d S=%d H=%d Hq=%d Hkv=%d d=%d F=%d %s rho=%.1f %s rope=%s" % (
        shape.name, shape.B, shape.S, shape.H, shape.Hq, shape.Hkv, shape.d, shape.F, shape.dtype, shape.rho,
        shape.mask_kind, case["rope"]))
    p = Hn.Problem(shape, case["seed"], "independent",
                   oracle_dtype=np.float64 if shape.dtype == "f32" else np.float32, rope=case["rope"])
    sv, W, dy, mask = p.device_tensors(DEV)
    got, idx, cu, n = Bn.layer_bwd_filtered(p.desc(), sv, W, dy, mask)
    torch.cuda.synchronize()
    ridx = np.flatnonzero(p.mask.reshape(-1))
    assert n == len(ridx) and np.array_equal(idx.cpu().numpy()[:n], ridx)
    if n == 0:
        return
    errs = Hn.check_layer(p, got, p.oracle(), ridx, Hn.TOL[shape.dtype])
    say("  n_kept=%d max rel err %.2e worst line %.2e" % (n, max(v for k, v in errs.items() if k != "worst_line"), errs["worst_line"]))


def test_layer_with_a_count_known_beforehand_never_synchronises():
    """Top-k filtering keeps a known number of tokens: index build without the host copy, gather and
    the compact entry point give bit for bit what cf_layer_bwd_filtered gives."""
    shape = SMALL_BF16
    say("layer known count %s" % shape.name)
    p = Hn.Problem(shape, 61, "independent", rho=0.5)
    sv, W, dy, mask = p.device_tensors(DEV)
    ref = Bn.LayerBackward(p.desc(), device=DEV)
    n = ref.filtered(sv, W, dy, mask)
    assert n == int(p.mask.sum())
    plan = Bn.LayerBackward(p.desc(), device=DEV)
    plan.filtered_known(sv, W, dy, mask, n)
    torch.cuda.synchronize()
    assert torch.equal(plan.idx[:n], ref.idx[:n]) and torch.equal(plan.cu_kept, ref.cu_kept)
    assert int(plan.n_kept_dev.item()) == n
    for name in Hn.GRADS:
        assert torch.equal(plan.grads[name], ref.grads[name]), name
    assert torch.equal(plan.grads["dx"][:n], ref.grads["dx"][:n])


def test_layer_filtered_call_replays_from_a_captured_graph_with_other_masks():
    """The filtered call allocates nothing, never synchronises and sizes nothing on the host by the kept
    count, so it can be captured once into a HIP graph and replayed for ANY mask: every replay (with
    eager work and synchronisations between them, a different mask, kept count and upstream gradient
    each time) must give bit for bit what the eager call gives for the same inputs."""
    shape = SMALL_BF16_GROUPED
    say("layer graph capture %s" % shape.name)
    p = Hn.Problem(shape, 71, "independent", rho=0.5)
    sv, W, dy, mask = p.device_tensors(DEV)
    ref = Bn.LayerBackward(p.desc(), device=DEV)
    plan = Bn.LayerBackward(p.desc(), device=DEV)
    plan.filtered_async(sv, W, dy, mask)        # outside the capture: one-time function attributes
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.filtered_async(sv, W, dy, mask)
    rng = np.random.default_rng(72)
    for rep, rho in enumerate((0.5, 0.2, 0.9, 0.0)):
        new_mask = (rng.random((shape.B, shape.S)) < rho).astype(np.uint8)
        mask.copy_(torch.from_numpy(new_mask).to(DEV))
        dy.copy_(Hn.to_dev(Hn.quantize(rng.standard_normal((shape.T, shape.H)), "bf16"), "bf16", DEV))
        n = ref.filtered(sv, W, dy, mask)       # eager, synchronises
        assert n == int(new_mask.sum())
        for t in list(plan.grads.values()) + [plan.idx, plan.cu_kept, plan.n_kept_dev]:
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        say("  replay %d: n_kept %d" % (rep, n))
        assert int(plan.n_kept_dev.item()) == n and int(plan._n_host[0]) == n
        assert torch.equal(plan.idx[:n], ref.idx[:n]) and torch.equal(plan.cu_kept, ref.cu_kept)
        for name in Hn.GRADS:
            assert torch.equal(plan.grads[name], ref.grads[name]), (rep, name)
        assert torch.equal(plan.grads["dx"][:n], ref.grads["dx"][:n]), rep


def test_layer_device_side_count_with_a_tight_bound_and_a_stack_without_any_host_read():
    """The filtered call reads N_k on the device.  (1) A workspace and launch bound of exactly N_k
    (max_kept = N_k, the smallest legal one) gives bit for bit what the default bound T gives.
    (2) A layer below takes the count from the device as well (cf_layer_bwd_compact_dev): the same
    bits as cf_layer_bwd_compact with the host count.  Nothing is synchronised until the end."""
    shape = SMALL_BF16_D128
    say("layer device-side count %s" % shape.name)
    p = Hn.Problem(shape, 62, "independent", rho=0.4)
    low = Hn.Problem(shape, 63, "independent", mask=p.mask)
    sv, W, dy, mask = p.device_tensors(DEV)
    sv1, W1, _, _ = low.device_tensors(DEV)
    n_true = int(p.mask.sum())
    full = Bn.LayerBackward(p.desc(), device=DEV)                       # max_kept = T
    tight = Bn.LayerBackward(p.desc(), device=DEV, max_kept=n_true)
    assert tight.ws_bytes < full.ws_bytes
    full.filtered_async(sv, W, dy, mask)
    tight.filtered_async(sv, W, dy, mask)
    lo_dev = Bn.LayerBackward(p.desc(), device=DEV)
    lo_dev.compact_dev(sv1, W1, full.grads["dx"], full.idx, full.cu_kept, full.n_kept_dev)
    n = full.n_kept()                                                   # the first synchronisation
    assert n == n_true == tight.n_kept()
    for name in Hn.GRADS:
        assert torch.equal(full.grads[name], tight.grads[name]), name
    assert torch.equal(full.grads["dx"][:n], tight.grads["dx"][:n])
    assert torch.equal(full.idx[:n], tight.idx[:n])
    lo_host = Bn.LayerBackward(p.desc(), device=DEV)
    lo_host.compact(sv1, W1, full.grads["dx"][:n], full.idx, full.cu_kept, n)
    torch.cuda.synchronize()
    for name in Hn.GRADS:
        assert torch.equal(lo_dev.grads[name], lo_host.grads[name]), name
    assert torch.equal(lo_dev.grads["dx"][:n], lo_host.grads["dx"][:n])
    # and the result is right
    errs = Hn.check_layer(p, dict(full.grads, dx=full.grads["dx"][:n]), p.oracle(), np.flatnonzero(p.mask.reshape(-1)),
                          Hn.TOL["bf16"])
    say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))


def test_layer_mask_that_keeps_more_than_max_kept_stays_inside_its_buffers():
    """A caller's bound that the mask exceeds: the call processes the first max_kept kept tokens, writes
    nothing outside buffers sized for max_kept, and reports the true count, which exposes the mistake."""
    shape = WL.LayerShape("overflow", B=2, S=256, H=256, Hq=4, Hkv=2, d=64, F=384, dtype="bf16")
    say("layer max_kept exceeded")
    p = Hn.Problem(shape, 64, "independent", rho=0.5)
    sv, W, dy, mask = p.device_tensors(DEV)
    n_true = int(p.mask.sum())
    bound = n_true - 37
    plan = Bn.LayerBackward(p.desc(), device=DEV, max_kept=bound)
    PAD = 4096
    nbytes = plan.ws.numel()
    buf = torch.full((nbytes + 2 * PAD,), 0xA5, dtype=torch.uint8, device=DEV)
    plan.ws = buf[PAD:PAD + nbytes]
    dxb = torch.full((bound * shape.H * 2 + 2 * PAD,), 0xA5, dtype=torch.uint8, device=DEV)
    plan.grads["dx"] = dxb[PAD:PAD + bound * shape.H * 2].view(torch.bfloat16).view(bound, shape.H)
    plan._g = Bn.Grads(*([plan.grads[n].data_ptr() for n in Bn.GRAD_NAMES] + [0]))
    n = plan.filtered(sv, W, dy, mask)
    assert n == n_true > bound
    for b in (buf, dxb):
        assert bool((b[:PAD] == 0xA5).all()) and bool((b[-PAD:] == 0xA5).all())
    # the first `bound` kept tokens of a single sequence mask would be a legal problem of its own: here we only
    # require finite outputs
    assert bool(torch.isfinite(plan.grads["dx"].float()).all())
    assert bool(torch.isfinite(plan.grads["dwd"].float()).all())


MAIN_GRAD_SHAPES = [
    SMALL_BF16, SMALL_BF16_D128, SMALL_BF16_GROUPED,
    WL.LayerShape("main_grad_f32", B=2, S=96, H=128, Hq=2, Hkv=1, d=64, F=256, dtype="f32"),
]


@pytest.mark.parametrize("shape", MAIN_GRAD_SHAPES, ids=lambda s: s.name)
def test_layer_main_grad_accumulation(shape):
    """main_grad = 1: the parameter gradients are fp32 buffers the calls add to.  Start from random
    buffers G0, run the filtered backward twice and the dense one once: the buffers must hold
    G0 + 2*filtered + dense gradients of the oracle; dx is the last call's, as without the flag."""
    say("layer main-grad %s" % shape.name)
    p = Hn.Problem(shape, 91, "independent", rho=0.5)
    ref, refd = p.oracle(), p.oracle(dense=True)
    sv, W, dy, mask = p.device_tensors(DEV)
    plan = Bn.LayerBackward(p.desc(), device=DEV, main_grad=True)
    rng = np.random.default_rng(92)
    g0 = {}
    for name in Hn.GRADS:
        assert plan.grads[name].dtype == torch.float32
        g0[name] = (rng.standard_normal(ref[name].shape) * ref[name].std()).astype(np.float32)
        plan.grads[name].copy_(torch.from_numpy(g0[name]))
    n = plan.filtered(sv, W, dy, mask)
    plan.filtered(sv, W, dy, mask)
    torch.cuda.synchronize()
    ridx = np.flatnonzero(p.mask.reshape(-1))
    assert n == len(ridx)
    assert Hn.rel_fro(Hn.to_np(plan.grads["dx"][:n]), ref["dx"][ridx]) <= Hn.TOL[shape.dtype]
    plan.dense(sv, W, dy)
    torch.cuda.synchronize()
    assert Hn.rel_fro(Hn.to_np(plan.grads["dx"]), refd["dx"]) <= Hn.TOL[shape.dtype]
    errs = {}
    for name in Hn.GRADS:
        added = Hn.to_np(plan.grads[name]).astype(np.float64) - g0[name]
        errs[name] = Hn.rel_fro(added, 2.0 * ref[name] + refd[name])
    say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    bad = {k: v for k, v in errs.items() if not (v <= Hn.TOL[shape.dtype])}
    assert not bad, bad


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_invariants_on_gpu_outputs(dtype):
    """Keep ratio 1 reproduces the dense call bit for bit (same kernels, same
    shapes); an empty mask gives zero parameter gradients; garbage in the
    filtered rows of dy does not leak."""
    shape = WL.LayerShape("inv", B=2, S=192, H=256, Hq=4, Hkv=2, d=64, F=512, dtype=dtype)
    say("layer invariants %s" % dtype)
    ones = np.ones((shape.B, shape.S), np.uint8)
    p = Hn.Problem(shape, 5, "independent", mask=ones)
    got, ridx, n = _run_layer(p)
    gotd, _, _ = _run_layer(p, dense=True)
    assert n == shape.T
    for name in Hn.GRADS + ("dx",):
        assert torch.equal(got[name], gotd[name]), name
    # empty mask
    p0 = Hn.Problem(shape, 5, "independent", mask=np.zeros_like(ones))
    got0, _, n0 = _run_layer(p0)
    assert n0 == 0 and got0["dx"].shape[0] == 0
    for name in Hn.GRADS:
        assert torch.count_nonzero(got0[name]).item() == 0, name
    # garbage in filtered rows of dy
    ph = Hn.Problem(shape, 6, "independent", rho=0.5)
    got1, ridx1, _ = _run_layer(ph)
    dead = ph.mask.reshape(-1) == 0
    ph.dy[dead] = Hn.quantize(1e4 * np.ones_like(ph.dy[dead]), dtype)
    got2, _, _ = _run_layer(ph)
    for name in Hn.GRADS + ("dx",):
        assert torch.equal(got1[name], got2[name]), name


def test_layer_ragged_batch_with_empty_sequence():
    shape = WL.LayerShape("ragged", B=4, S=96, H=128, Hq=2, Hkv=1, d=64, F=256, dtype="bf16")
    say("layer ragged")
    rng = np.random.default_rng(9)
    mask = np.zeros((4, 96), np.uint8)
    mask[0] = rng.random(96) < 0.8
    mask[1] = 0
    mask[2] = rng.random(96) < 0.2
    mask[3, -1] = 1
    p = Hn.Problem(shape, 9, "independent", mask=mask)
    got, ridx, n = _run_layer(p)
    Hn.check_layer(p, got, p.oracle(), ridx, Hn.TOL["bf16"])


def test_layer_stack_of_two_shares_one_index():
    """Two layers chained: the compact dx of the upper layer is the compact upstream
    gradient of the lower one, which reuses the index and is not synchronised.  The
    oracle runs the same chain on full-length tensors (its dx is zero on filtered rows)."""
    shape = WL.LayerShape("stack", B=2, S=288, H=256, Hq=4, Hkv=2, d=64, F=640, dtype="bf16")
    say("layer stack of two")
    top = Hn.Problem(shape, 21, "independent", rho=0.5)
    low = Hn.Problem(shape, 22, "independent", mask=top.mask)
    sv2, W2, dy, mask = top.device_tensors(DEV)
    sv1, W1, _, _ = low.device_tensors(DEV)
    plan2 = Bn.LayerBackward(top.desc(), device=DEV)
    plan1 = Bn.LayerBackward(low.desc(), device=DEV)
    n = plan2.filtered(sv2, W2, dy, mask)
    plan1.compact(sv1, W1, plan2.grads["dx"][:n], plan2.idx, plan2.cu_kept, n)
    torch.cuda.synchronize()
    ref2 = top.oracle()
    low.dy = np.asarray(ref2["dx"], dtype=np.float64)      # full length, zero on filtered rows
    ref1 = low.oracle()
    ridx = np.flatnonzero(top.mask.reshape(-1))
    got = dict(plan1.grads)
    got["dx"] = got["dx"][:n]
    errs = Hn.check_layer(low, got, ref1, ridx, Hn.TOL["bf16"])
    say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    # the compact call on the upper layer's own inputs reproduces the filtered call bit for bit
    keep = {k: v.clone() for k, v in plan2.grads.items()}
    dyk = Bn.gather_rows(dy, plan2.idx, n)
    plan2.compact(sv2, W2, dyk, plan2.idx, plan2.cu_kept, n)
    torch.cuda.synchronize()
    for k in keep:
        a, b = (plan2.grads[k][:n], keep[k][:n]) if k == "dx" else (plan2.grads[k], keep[k])
        assert torch.equal(a, b), k


def test_layer_stack_of_eight_error_growth_over_depth():
    """Eight different layers chained through the compact entry point: the top layer builds the index,
    every layer below takes the compact dx of the layer above (the library's own, with its rounding)
    as upstream gradient.  The oracle runs the same chain in float64 on full-length tensors.  The
    relative error of every layer's outputs against the chained oracle is printed and must stay
    within the single-layer tolerance: rounding errors handed down the stack do not blow up."""
    depth = 8
    shape = WL.LayerShape("stack8", B=2, S=288, H=256, Hq=4, Hkv=2, d=64, F=640, dtype="bf16")
    say("layer stack of eight")
    probs = [Hn.Problem(shape, 300 + l, "independent", rho=0.5) for l in range(depth)]
    mask_np = probs[0].mask
    ridx = np.flatnonzero(mask_np.reshape(-1))
    plans = [Bn.LayerBackward(shape_p.desc(), device=DEV) for shape_p in probs[:2]]
    dev = [p.device_tensors(DEV) for p in probs]
    worst = []
    ref_dy = probs[0].dy.astype(np.float64)
    n = None
    for l in range(depth):
        sv, W, dy, mask = dev[l]
        plan = plans[l & 1]
        if l == 0:
            n = plan.filtered(sv, W, dy, mask)
        else:
            plan.compact(sv, W, plans[(l - 1) & 1].grads["dx"][:n], plans[0].idx, plans[0].cu_kept, n)
        torch.cuda.synchronize()
        probs[l].mask = mask_np
        probs[l].dy = ref_dy
        ref = probs[l].oracle()
        got = dict(plan.grads)
        got["dx"] = got["dx"][:n]
        errs = Hn.check_layer(probs[l], got, ref, ridx, Hn.TOL["bf16"])
        worst.append(max(v for k, v in errs.items() if k != "worst_line"))
        say("  layer %d below the top: dx %.2e worst tensor %.2e" % (l, errs["dx"], worst[-1]))
        ref_dy = np.asarray(ref["dx"], dtype=np.float64)       # full length, zero on filtered rows
    assert max(worst) <= Hn.TOL["bf16"]
    # no blow-up: the deepest layer is within a small factor of the top one
    assert worst[-1] <= 4.0 * worst[0] + 1e-3


@pytest.mark.parametrize("dtype,mode", [("f32", "consistent"), ("bf16", "independent")])
def test_layer_with_rotary_embedding(dtype, mode):
    """q and k are rotated tensors: the layer applies the transposed rotation to dq and dk at
    the original positions of the kept rows (filtered and dense calls)."""
    shape = WL.LayerShape("rope", B=2, S=160, H=256, Hq=4, Hkv=2, d=64, F=384, dtype=dtype)
    say("layer rotary %s" % dtype)
    p = Hn.Problem(shape, 31, mode, rho=0.5, rope=True)
    got, ridx, n = _run_layer(p)
    ref = p.oracle()
    errs = Hn.check_layer(p, got, ref, ridx, Hn.TOL[dtype])
    say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    gotd, _, _ = _run_layer(p, dense=True)
    Hn.check_layer(p, gotd, p.oracle(dense=True), None, Hn.TOL[dtype])
    # the rotation matters: without it dWq is far from the reference
    p.rope, keep = None, p.rope
    got0, _, _ = _run_layer(p)
    p.rope = keep
    assert Hn.rel_fro(Hn.to_np(got0["dwq"]), ref["dwq"]) > 10 * Hn.TOL[dtype]


def test_no_write_outside_the_outputs_and_the_workspace():
    """Every output tensor and the workspace sit inside a larger allocation filled with a
    sentinel; after filtered, compact and dense calls on a ragged shape (no dimension a tile
    multiple) the guard bands are untouched."""
    shape = WL.LayerShape("guard", B=3, S=200, H=264, Hq=6, Hkv=2, d=64, F=520, dtype="bf16")
    say("guard bands")
    p = Hn.Problem(shape, 41, "independent", rho=0.37)
    sv, W, dy, mask = p.device_tensors(DEV)
    desc = p.desc()
    plan = Bn.LayerBackward(desc, device=DEV)
    PAD = 4096                                      # bytes on each side
    raw = {}

    def guarded(t):
        nbytes = t.numel() * t.element_size()
        buf = torch.full((nbytes + 2 * PAD,), 0xA5, dtype=torch.uint8, device=DEV)
        view = buf[PAD:PAD + nbytes].view(t.dtype).view(t.shape)
        return buf, view

    for name in list(plan.grads):
        raw[name], plan.grads[name] = guarded(plan.grads[name])
    raw["idx"], plan.idx = guarded(plan.idx)
    raw["cu"], plan.cu_kept = guarded(plan.cu_kept)
    raw["ws"], plan.ws = guarded(plan.ws)
    plan._g = Bn.Grads(*[plan.grads[n].data_ptr() for n in Bn.GRAD_NAMES])
    n = plan.filtered(sv, W, dy, mask)
    dyk = Bn.gather_rows(dy, plan.idx, n)
    plan.compact(sv, W, dyk, plan.idx, plan.cu_kept, n)
    plan.dense(sv, W, dy)
    torch.cuda.synchronize()
    for name, buf in raw.items():
        assert bool((buf[:PAD] == 0xA5).all()) and bool((buf[-PAD:] == 0xA5).all()), name


LORA_NAMES = ("daq", "dbq", "dak", "dbk", "dav", "dbv", "dao", "dbo")


def _run_lora(p, lora_np, rank, mask_on=True):
    sv, W, dy, mask = p.device_tensors(DEV)
    lo = {k: (Hn.to_dev(v, p.dtype, DEV) if isinstance(v, np.ndarray) else v) for k, v in lora_np.items()}
    plan = Bn.LoraBackward(p.desc(), rank, device=DEV)
    n = plan.run(sv, W, lo, dy, mask if mask_on else None)
    torch.cuda.synchronize()
    return plan, n


LORA_SHAPES = {
    "small": dict(B=2, S=224, H=256, Hq=4, Hkv=2, d=64, F=384),
    # long enough contractions (H, Hq*d and the kept-token count above 1024) for the adapter products
    # to take the split-K path, with ragged K ranges
    "splitk": dict(B=2, S=640, H=1024, Hq=16, Hkv=4, d=64, F=512),
}


@pytest.mark.parametrize("dtype,mode,rank,which", [("f32", "consistent", 8, "small"),
                                                   ("bf16", "independent", 16, "small"),
                                                   ("bf16", "independent", 64, "small"),
                                                   ("bf16", "independent", 64, "splitk"),
                                                   ("bf16", "independent", 24, "splitk")])
def test_layer_lora(dtype, mode, rank, which):
    """Adapters on q, k, v, o with frozen base weights: adapter gradients and compact dx against
    the oracle, filtered and with every token kept."""
    shape = WL.LayerShape("lora", dtype=dtype, **LORA_SHAPES[which])
    say("layer lora %s rank %d %s" % (dtype, rank, which))
    rng = np.random.default_rng(51)
    lora_np = {k: (Hn.quantize(v, dtype) if isinstance(v, np.ndarray) else v)
               for k, v in WL.make_lora(shape, rng, rank=rank, alpha=2.0 * rank).items()}
    p = Hn.Problem(shape, 52, mode, rho=0.9 if which == "splitk" else 0.5)
    if mode == "consistent":    # saved tensors of the adapted forward
        lo64 = {k: (v.astype(np.float64) if isinstance(v, np.ndarray) else v) for k, v in lora_np.items()}
        _, sv = O.layer_fwd(p.saved["x"].astype(np.float64), {k: v.astype(np.float64) for k, v in p.W.items()},
                            lora=lo64, **p.kw)
        p.saved = {k: (np.asarray(v, dtype=np.float32) if k == "lse" else Hn.quantize(v, dtype)) for k, v in sv.items()}
    lo = {k: (v.astype(p.oracle_dtype) if isinstance(v, np.ndarray) else v) for k, v in lora_np.items()}
    svo = {k: v.astype(p.oracle_dtype) for k, v in p.saved.items()}
    Wo = {k: v.astype(p.oracle_dtype) for k, v in p.W.items()}
    for mask_on in (True, False):
        plan, n = _run_lora(p, lora_np, rank, mask_on)
        ref = O.layer_bwd(svo, Wo, p.dy.astype(p.oracle_dtype), p.mask if mask_on else None, lora=lo, **p.kw)
        ridx = np.flatnonzero(p.mask.reshape(-1)) if mask_on else np.arange(shape.T)
        assert n == len(ridx)
        errs = {k: Hn.rel_fro(Hn.to_np(plan.grads[k]), ref[k]) for k in LORA_NAMES}
        errs["dx"] = Hn.rel_fro(Hn.to_np(plan.grads["dx"][:n]), ref["dx"][ridx])
        say("  " + " ".join("%s=%.1e" % kv for kv in errs.items()))
        bad = {k: v for k, v in errs.items() if not (v <= Hn.TOL[dtype])}
        assert not bad, bad
        if mask_on:
            # the same call with the tightest bound (max_kept = N_k): launches and split-K plans are sized
            # for it instead of for T, the result must meet the same tolerance
            sv_d, W_d, dy_d, mask_d = p.device_tensors(DEV)
            lo_d = {k: (Hn.to_dev(v, p.dtype, DEV) if isinstance(v, np.ndarray) else v) for k, v in lora_np.items()}
            plan.max_kept = n
            assert plan.run(sv_d, W_d, lo_d, dy_d, mask_d) == n
            errs = {k: Hn.rel_fro(Hn.to_np(plan.grads[k]), ref[k]) for k in LORA_NAMES}
            errs["dx"] = Hn.rel_fro(Hn.to_np(plan.grads["dx"][:n]), ref["dx"][ridx])
            bad = {k: v for k, v in errs.items() if not (v <= Hn.TOL[dtype])}
            assert not bad, ("tight bound", bad)


def test_layer_lora_nothing_kept():
    """A mask that keeps no token: the count is only known on the device, every adapter gradient must
    come out zero (the kernels run on empty row and contraction ranges)."""
    shape = WL.LayerShape("lora0", dtype="bf16", **LORA_SHAPES["splitk"])
    say("layer lora, empty mask")
    rng = np.random.default_rng(53)
    lora_np = {k: (Hn.quantize(v, "bf16") if isinstance(v, np.ndarray) else v)
               for k, v in WL.make_lora(shape, rng, rank=64, alpha=128.0).items()}
    p = Hn.Problem(shape, 54, "independent", mask=np.zeros((shape.B, shape.S), np.uint8))
    plan, n = _run_lora(p, lora_np, 64, True)
    assert n == 0
    for k in LORA_NAMES:
        assert not bool(plan.grads[k].float().abs().max() > 0), k
