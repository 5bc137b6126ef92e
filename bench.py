#!/usr/bin/env python3
"""Benchmark of the token-filtered decoder-layer backward on one MI355X.

A "step" is one pass of the whole hot path over one synthetic batch:
keep mask -> keep index -> gathers -> reduced GEMMs, row-local ops, filtered
attention backward -> compact dx + all parameter gradients
(cf_layer_bwd_filtered).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` = kept tokens per second of the filtered layer
backward at keep ratio 0.5 on the Llama-3.1-8B-shaped layer (config 3); the
same line carries the speedup over the library's own dense backward, a keep
ratio sweep, the roofline of the dominant kernel (live HIP-event timing) and
the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_2502_00340_amd import binding as Bn
from paper_2502_00340_amd import workloads as WL

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
DEV = "cuda:0"


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def forward_fixture(q, k, v, shape: WL.LayerShape):
    """attn_out and lse consistent with the drawn (q, k, v): plain torch on the
    GPU, input preparation only (outside every timed region)."""
    B, S, Hq, Hkv, d = shape.B, shape.S, shape.Hq, shape.Hkv, shape.d
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(d)
    out = torch.empty((B * S, Hq * d), dtype=torch.float32, device=DEV)
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device=DEV)
    future = torch.triu(torch.ones(S, S, dtype=torch.bool, device=DEV), 1)
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(Hq):
            g = h // G
            sc = (q[rows, h * d:(h + 1) * d].float() @ k[rows, g * d:(g + 1) * d].float().T) * scale
            sc.masked_fill_(future, float("-inf"))
            l = torch.logsumexp(sc, dim=1)
            out[rows, h * d:(h + 1) * d] = torch.exp(sc - l[:, None]) @ v[rows, g * d:(g + 1) * d].float()
            lse[b, h] = l
    return out.to(q.dtype), lse


def make_inputs(shape: WL.LayerShape, seed: int):
    rng = np.random.default_rng(seed)
    W = {k: to_dev(v, shape.dtype) for k, v in WL.make_weights(shape, rng).items()}
    sv = {k: to_dev(v, shape.dtype) for k, v in WL.make_independent_activations(shape, rng).items()}
    sv["attn_out"], sv["lse"] = forward_fixture(sv["q"], sv["k"], sv["v"], shape)
    dy = to_dev(WL.make_normal(rng, shape.T, shape.H), shape.dtype)
    mask = WL.make_mask(shape, rng)
    return W, sv, dy, mask, rng


def attn_alg_flops(shape: WL.LayerShape, mask: np.ndarray) -> float:
    """2*d*Hq * sum over kept tokens of [3*(p+1) + 2*(c+1)]: three products over all
    p+1 visible keys (S, dP, dS*K) and two over the c+1 kept keys (dV, dK)."""
    tot = 0.0
    for b in range(shape.B):
        pos = np.flatnonzero(mask[b]).astype(np.float64)
        rank = np.arange(len(pos), dtype=np.float64)
        tot += float(np.sum(3.0 * (pos + 1.0) + 2.0 * (rank + 1.0)))
    return 2.0 * shape.d * shape.Hq * tot


def layer_alg_flops(shape: WL.LayerShape, mask: np.ndarray) -> float:
    n_k = int(mask.sum())
    return 4.0 * shape.P_layer * n_k + attn_alg_flops(shape, mask)


def time_steps(fn, steps: int, warmup: int) -> float:
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def event_times(fn, reps: int, warmup: int = 2):
    """Per-call durations (ms) from HIP events recorded on torch's current
    stream, which is the stream the binding launches on."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    out = []
    for _ in range(reps):
        s = torch.cuda.Event(enable_timing=True)
        e = torch.cuda.Event(enable_timing=True)
        s.record()
        fn()
        e.record()
        e.synchronize()
        out.append(s.elapsed_time(e))
    return out


def _vp(t):
    import ctypes as C
    return C.c_void_p(t.data_ptr())


def _st():
    import ctypes as C
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def back_to_back_ms(call, reps: int, warm: int = 3) -> float:
    """Mean duration of `reps` launches issued back to back on torch's current stream (the stream the
    library launches on), one HIP-event pair around all of them."""
    for _ in range(warm):
        call()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        call()
    ev1.record()
    ev1.synchronize()
    return ev0.elapsed_time(ev1) / reps


def mfma_ceiling_leg(reps: int = 20):
    """Measured matrix-core ceiling: the GEMM's wave tile (8 x 8 accumulators of 16x16x32 bf16 MFMAs,
    four waves per CU, all CUs) with every operand in registers and non-zero pseudo-random values;
    launches as long as the roofline GEMM's, timed the same way (sustained, power-limited rate)."""
    import ctypes as C
    lib = Bn.lib()
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(n_cu * 256, dtype=torch.float32, device=DEV)
    fl = C.c_double(0.0)
    iters = 640

    def call():
        rc = lib.cf_probe_mfma_bf16(n_cu, iters, _vp(sink), C.byref(fl), _st())
        assert rc == 0, rc

    ms = back_to_back_ms(call, reps)
    out = {"TFLOPs": round(fl.value / ms / 1e9, 1), "avg_launch_ms": round(ms, 4), "blocks": n_cu, "iters": iters,
           "kernel": "cf::mfma_probe_kernel (register-resident 16x16x32 bf16 MFMA loop, no LDS, no global traffic)"}
    # the same loop with the GEMM kernels' LDS fragment reads mixed in (nothing else of the GEMM)
    with_reads = {}
    for reads, name in ((0, "none"), (1, "nt_16_b128_per_64_mfma"), (2, "tn_32_tr_b64_per_64_mfma")):
        def call_r(reads=reads):
            rc = lib.cf_probe_mfma_lds_bf16(n_cu, iters, reads, _vp(sink), C.byref(fl), _st())
            assert rc == 0, rc
        ms_r = back_to_back_ms(call_r, reps)
        with_reads[name] = round(fl.value / ms_r / 1e9, 1)
    out["TFLOPs_with_lds_fragment_reads"] = with_reads
    return out


def copy_ceiling_leg(reps: int = 10):
    """Measured HBM ceiling: a plain 1 GiB -> 1 GiB device copy (bytes read + bytes written per second)."""
    lib = Bn.lib()
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=DEV)
    dst = torch.empty(n, dtype=torch.uint8, device=DEV)
    src.fill_(3)

    def call():
        rc = lib.cf_probe_copy(_vp(src), _vp(dst), n, _st())
        assert rc == 0, rc

    ms = back_to_back_ms(call, reps)
    del src, dst
    return {"GBps": round(2.0 * n / ms / 1e6, 1), "avg_launch_ms": round(ms, 4), "bytes_copied": n,
            "frac_of_8TBps": round(2.0 * n / ms / 1e6 / 8000, 4), "kernel": "cf::copy_probe_kernel"}


def roofline_leg(shape: WL.LayerShape, n_k: int, reps: int = 20):
    """Dominant kernel: the parameter-gradient GEMM dW = X_kept^T * dY_kept (the
    contraction runs over the kept tokens) at the layer's largest shape, the FFN
    projections [F x H x N_k]."""
    dt = torch.bfloat16
    x = torch.randn((n_k, shape.F), device=DEV).to(dt)
    dy = torch.randn((n_k, shape.H), device=DEV).to(dt)
    dw = torch.empty((shape.F, shape.H), dtype=dt, device=DEV)

    # raw call with a pre-allocated output keeps allocator work out of the event window
    lib = Bn.lib()
    import ctypes as C

    def call_raw():
        rc = lib.cf_linear_bwd_reduced(C.c_void_p(x.data_ptr()), C.c_void_p(dy.data_ptr()), None, n_k,
                                       shape.F, shape.H, Bn.CF_BF16, None, C.c_void_p(dw.data_ptr()),
                                       0.0, C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, rc

    # one event pair around `reps` back-to-back launches: the mean then holds the kernel and the
    # few microseconds between two kernels of a stream, not a host round trip per launch
    avg = back_to_back_ms(call_raw, reps)
    flops = 2.0 * n_k * shape.F * shape.H
    ach = flops / (avg * 1e-3) / 1e12
    # HBM bytes per launch of this kernel, from the two counter runs summarised under profiles/
    traffic = None
    traffic_source = None
    tpath = os.path.join(ROOT, "profiles", "gemm_tn_dw_8b_hbm_traffic.txt")
    if os.path.exists(tpath) and (n_k, shape.F, shape.H) == (4096, 14336, 4096):
        for line in open(tpath):
            if line.strip().startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
                # a stored figure of an earlier profiler run of this same command, not of this run
                traffic_source = "profiles/gemm_tn_dw_8b_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)"
    ceil = mfma_ceiling_leg(reps)
    return {"bound": "mfma", "achieved": round(ach, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_source": traffic_source,
            "ceiling_measured": ceil["TFLOPs"], "frac_of_ceiling": round(ach / ceil["TFLOPs"], 4),
            "ceiling": ceil,
            "kernel": "cf::gemm_bf16_kernel<1> (TN): dW[F,H] = X_kept^T dY_kept",
            "flops_per_launch": flops, "avg_launch_ms": round(avg, 4), "launches": reps}


def parts_leg(shape: WL.LayerShape, sv, W, dy, mask: np.ndarray, mask_dev, reps: int = 10):
    """Per-part timings through the single-purpose entry points (HIP events, mean of `reps`
    calls), plus scaled-up runs of the index build and the row gather: at T = 8192 those two
    are launch-latency bound and say nothing about bandwidth."""
    out = {}
    n_k = int(mask.sum())
    T, H, F, Nq, Nkv = shape.T, shape.H, shape.F, shape.Nq, shape.Nkv
    import ctypes as C
    lib = Bn.lib()
    copyc = copy_ceiling_leg()
    out["hbm_copy_ceiling"] = copyc
    hbm = lambda nbytes, ms: {"ms": round(ms, 4), "GBps": round(nbytes / ms / 1e6, 1), "bound": "hbm",
                              "frac_of_8TBps": round(nbytes / ms / 1e6 / 8000, 4),
                              "frac_of_copy_ceiling": round(nbytes / ms / 1e6 / copyc["GBps"], 4)}

    # A1 keep index: raw C calls on pre-allocated buffers (no allocation, no host copy in the timed window)
    def index_call(mask_t):
        Bq, Sq = mask_t.shape
        idx_t = torch.empty(Bq * Sq, dtype=torch.int32, device=DEV)
        cu_t = torch.empty(Bq + 1, dtype=torch.int32, device=DEV)
        n_t = torch.empty(1, dtype=torch.int32, device=DEV)
        wsb = lib.cf_index_workspace_bytes(Bq * Sq)
        ws_t = torch.empty(wsb, dtype=torch.uint8, device=DEV)

        def call():
            rc = lib.cf_build_keep_index(_vp(mask_t), Bq, Sq, _vp(idx_t), _vp(cu_t), _vp(n_t), None, _vp(ws_t), wsb, _st())
            assert rc == 0, rc
        return call, (idx_t, cu_t, n_t, ws_t)

    call, keep1 = index_call(mask_dev)
    ms = back_to_back_ms(call, reps)
    out["A1_keep_index"] = {"ms": round(ms, 4), "tokens": T}
    big = torch.from_numpy((np.random.default_rng(1).random((4096, 4096)) < 0.5).astype(np.uint8)).to(DEV)
    nb = int(big.sum().item())
    call, keep2 = index_call(big)
    ms = back_to_back_ms(call, reps)
    out["A1_keep_index_16M_tokens"] = hbm(big.numel() + 4 * nb + 4 * (big.shape[0] + 1), ms)
    del big, keep2
    # A2 gather
    idx, cu, _, _ = Bn.build_keep_index(mask_dev)
    dst = torch.empty((n_k, H), dtype=dy.dtype, device=DEV)

    def gather_call(src_t, idx_t, n_rows, dst_t):
        def call():
            rc = lib.cf_gather_rows(_vp(src_t), src_t.shape[0], src_t.shape[1], Bn.CF_BF16, _vp(idx_t), None, n_rows,
                                    _vp(dst_t), _st())
            assert rc == 0, rc
        return call

    ms = back_to_back_ms(gather_call(dy, idx, n_k, dst), reps)
    out["A2_gather_dy"] = {"ms": round(ms, 4), "GBps": round(2.0 * n_k * H * 2 / ms / 1e6, 1)}
    src = torch.empty((131072, 4096), dtype=torch.bfloat16, device=DEV)      # 1 GiB
    src.normal_()
    bm = torch.from_numpy((np.random.default_rng(2).random((1, 131072)) < 0.5).astype(np.uint8)).to(DEV)
    bidx, _, _, bn = Bn.build_keep_index(bm)
    bdst = torch.empty((bn, 4096), dtype=torch.bfloat16, device=DEV)
    ms = back_to_back_ms(gather_call(src, bidx, bn, bdst), reps)
    out["A2_gather_1GiB_source"] = hbm(2.0 * bn * 4096 * 2 + 4.0 * bn, ms)
    del src, bdst
    # A3 reduced linear backward at the FFN shape
    xk = torch.randn((n_k, F), device=DEV).to(dy.dtype)
    dyk = torch.randn((n_k, H), device=DEV).to(dy.dtype)
    dxo = torch.empty((n_k, F), dtype=dy.dtype, device=DEV)
    dwo = torch.empty((F, H), dtype=dy.dtype, device=DEV)
    fl = 2.0 * n_k * F * H

    def lin(xp, wp, dxp, dwp):
        def call():
            rc = lib.cf_linear_bwd_reduced(xp, _vp(dyk), wp, n_k, F, H, Bn.CF_BF16, dxp, dwp, 0.0, _st())
            assert rc == 0, rc
        return call

    mm = lambda ms: {"ms": round(ms, 4), "TFLOPs": round(fl / ms / 1e9, 1),
                     "frac_of_peak": round(fl / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}
    out["A3_dx_ffn"] = mm(back_to_back_ms(lin(None, _vp(W["wd"]), _vp(dxo), None), 2 * reps))
    out["A3_dw_ffn"] = mm(back_to_back_ms(lin(_vp(xk), None, None, _vp(dwo)), 2 * reps))
    del xk, dxo, dwo
    # A5 filtered attention backward (raw call, pre-allocated outputs and workspace)
    desc = Bn.make_desc(shape.B, shape.S, H, shape.Hq, shape.Hkv, shape.d, F, shape.dtype)
    qk = Bn.gather_rows(sv["q"], idx, n_k)
    ok = Bn.gather_rows(sv["attn_out"], idx, n_k)
    dok = torch.randn((n_k, Nq), device=DEV).to(dy.dtype)
    dq = torch.empty((n_k, Nq), dtype=dy.dtype, device=DEV)
    dk = torch.empty((n_k, Nkv), dtype=dy.dtype, device=DEV)
    dv = torch.empty((n_k, Nkv), dtype=dy.dtype, device=DEV)
    awsb = lib.cf_attn_workspace_bytes(C.byref(desc), n_k)
    aws = torch.empty(max(awsb, 256), dtype=torch.uint8, device=DEV)

    def attn_call():
        rc = lib.cf_attn_bwd_filtered(C.byref(desc), _vp(qk), _vp(sv["k"]), _vp(sv["v"]), _vp(ok), _vp(sv["lse"]),
                                      _vp(dok), _vp(idx), _vp(cu), n_k, _vp(dq), _vp(dk), _vp(dv), _vp(aws),
                                      aws.numel(), _st())
        assert rc == 0, rc

    ms = back_to_back_ms(attn_call, 2 * reps)
    fa = attn_alg_flops(shape, mask)
    out["A5_attn_bwd_filtered"] = {"ms": round(ms, 4), "algorithmic_TFLOPs": round(fa / ms / 1e9, 1),
                                   "frac_of_peak": round(fa / ms / 1e9 / PEAK_BF16_TFLOPS, 4)}
    return out


def make_inputs_device(shape: WL.LayerShape, seed: int):
    """The same distributions as make_inputs, drawn on the GPU (timing-only legs at long contexts, where the
    host generator would take minutes): weights N(0, 0.02^2), gains 1 + N(0, 0.02^2), activations and
    upstream gradient N(0, 1); attn_out and lse from the forward fixture."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    rn = lambda *s: torch.randn(*s, device=DEV, generator=g, dtype=torch.float32)
    H, F, Nq, Nkv, T = shape.H, shape.F, shape.Nq, shape.Nkv, shape.T
    W = {"wq": rn(H, Nq) * 0.02, "wk": rn(H, Nkv) * 0.02, "wv": rn(H, Nkv) * 0.02, "wo": rn(Nq, H) * 0.02,
         "wg": rn(H, F) * 0.02, "wu": rn(H, F) * 0.02, "wd": rn(F, H) * 0.02,
         "g1": 1.0 + 0.02 * rn(H), "g2": 1.0 + 0.02 * rn(H)}
    W = {k: v.to(dt) for k, v in W.items()}
    sv = {"x": rn(T, H).to(dt), "r": rn(T, H).to(dt), "q": rn(T, Nq).to(dt), "k": rn(T, Nkv).to(dt),
          "v": rn(T, Nkv).to(dt), "gate": rn(T, F).to(dt), "up": rn(T, F).to(dt)}
    sv["attn_out"], sv["lse"] = forward_fixture(sv["q"], sv["k"], sv["v"], shape)
    dy = rn(T, H).to(dt)
    return W, sv, dy


def context_sweep_leg(base: WL.LayerShape, steps: int, warmup: int):
    """The layer-level form of the paper's context-length and filtering-ratio experiments (Sec. 5.3):
    filtered vs dense layer backward at keep ratio 0.5 for context lengths 1K .. 32K (T = 8192 tokens up to
    S = 8K, then one sequence of S tokens), and keep ratios 0.1 .. 1.0 at the shape's own context length."""
    import dataclasses
    out = {"by_context": {}, "by_ratio": {}}
    for S in (1024, 2048, 4096, 8192, 16384, 32768):
        T = max(8192, S)
        shape = dataclasses.replace(base, B=T // S, S=S, mask_kind="topk")
        W, sv, dy = make_inputs_device(shape, 7 + S)
        rng = np.random.default_rng(S)
        md = torch.from_numpy(WL.mask_topk(rng, shape.B, shape.S, 0.5)).to(DEV)
        desc = Bn.make_desc(shape.B, shape.S, shape.H, shape.Hq, shape.Hkv, shape.d, shape.F, shape.dtype)
        plan = Bn.LayerBackward(desc, device=DEV)
        st = max(3, steps // 2) if S > 8192 else steps
        t_f = time_steps(lambda: plan.filtered_async(sv, W, dy, md), st, warmup)
        t_d = time_steps(lambda: plan.dense(sv, W, dy), st, warmup)
        out["by_context"][str(S)] = {"B": shape.B, "tokens": T, "filtered_ms": round(t_f * 1e3, 4),
                                     "dense_ms": round(t_d * 1e3, 4), "speedup": round(t_d / t_f, 4)}
        log("%s context %d (T=%d): filtered %.3f ms dense %.3f ms speedup %.3f" % (base.name, S, T, t_f * 1e3, t_d * 1e3, t_d / t_f))
        if S == base.S and T == base.T:
            for rho in (0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0):
                mdd = torch.from_numpy(WL.mask_topk(rng, shape.B, shape.S, rho)).to(DEV)
                t = time_steps(lambda: plan.filtered_async(sv, W, dy, mdd), steps, warmup)
                out["by_ratio"]["%.1f" % rho] = {"ms": round(t * 1e3, 4), "speedup": round(t_d / t, 4)}
                log("%s keep ratio %.1f: %.3f ms speedup %.3f" % (base.name, rho, t * 1e3, t_d / t))
        del plan, W, sv, dy
        torch.cuda.empty_cache()
    return out


def lora_leg(shape: WL.LayerShape, sv, W, dy, mask_dev, rng, steps: int, warmup: int, rank: int = 64):
    """The LoRA regime of the paper (rank-64 adapters on q, k, v, o; base weights frozen): filtered
    vs dense cf_layer_bwd_lora on the same layer."""
    lo = {k: (to_dev(v, shape.dtype) if isinstance(v, np.ndarray) else v)
          for k, v in WL.make_lora(shape, rng, rank=rank, alpha=2.0 * rank).items()}
    desc = Bn.make_desc(shape.B, shape.S, shape.H, shape.Hq, shape.Hkv, shape.d, shape.F, shape.dtype)
    plan = Bn.LoraBackward(desc, rank, device=DEV)
    t_f = time_steps(lambda: plan.run_async(sv, W, lo, dy, mask_dev), steps, warmup)
    t_d = time_steps(lambda: plan.run_async(sv, W, lo, dy, None), steps, warmup)
    return {"rank": rank, "filtered_ms": round(t_f * 1e3, 4), "dense_ms": round(t_d * 1e3, 4),
            "speedup": round(t_d / t_f, 4)}


def main_grad_leg(desc, sv, W, dy, mask_dev, steps: int, warmup: int):
    """The same layer with fp32 main-gradient buffers that every call adds to (gradient
    accumulation over micro-batches): each dW element is read and written as fp32."""
    plan = Bn.LayerBackward(desc, device=DEV, main_grad=True)
    t_f = time_steps(lambda: plan.filtered_async(sv, W, dy, mask_dev), steps, warmup)
    t_d = time_steps(lambda: plan.dense(sv, W, dy), steps, warmup)
    return {"filtered_ms": round(t_f * 1e3, 4), "dense_ms": round(t_d * 1e3, 4), "speedup": round(t_d / t_f, 4)}


def stack_leg(desc, sv, W, dy, mask_dev, layers: int, steps: int, warmup: int):
    """A stack of `layers` identical layers (Sec. 3.2: once the first gradient is reduced all
    later ones are): the top layer builds the index, every layer below takes the compact dx of the
    layer above, the shared index and the device-side count through cf_layer_bwd_compact_dev; the
    host never reads N_k and nothing synchronises.  The layers reuse one set of saved tensors and weights: the timing is that of
    the kernels, not of a model's memory footprint."""
    plans = [Bn.LayerBackward(desc, device=DEV) for _ in range(2)]      # ping-pong: dx of one is dy of the next

    def run_filtered():
        plans[0].filtered_async(sv, W, dy, mask_dev)
        for l in range(1, layers):
            src, dst = plans[(l - 1) & 1], plans[l & 1]
            dst.compact_dev(sv, W, src.grads["dx"], plans[0].idx, plans[0].cu_kept, plans[0].n_kept_dev)

    def run_dense():
        plans[0].dense(sv, W, dy)
        for l in range(1, layers):
            src, dst = plans[(l - 1) & 1], plans[l & 1]
            dst.dense(sv, W, src.grads["dx"])

    t_f = time_steps(run_filtered, steps, warmup)
    t_d = time_steps(run_dense, steps, warmup)
    return {"layers": layers, "filtered_ms_per_layer": round(t_f * 1e3 / layers, 4),
            "dense_ms_per_layer": round(t_d * 1e3 / layers, 4), "speedup": round(t_d / t_f, 4)}


def cpu_baseline_leg(shape: WL.LayerShape, W, sv, dy, mask):
    """The CPU oracle (fp32 arrays, numpy) on the same workload (the whole batch
    is a bounded sample already: about ten seconds of host time)."""
    from oracle import layer_oracle as O      # cpu_baseline leg only
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    f = lambda t: t.float().cpu().numpy()
    saved = {k: f(v) for k, v in sv.items()}
    Wn = {k: f(v) for k, v in W.items()}
    t0 = time.perf_counter()
    O.layer_bwd(saved, Wn, f(dy), mask, B=shape.B, S=shape.S, Hq=shape.Hq, Hkv=shape.Hkv, d=shape.d)
    dt = time.perf_counter() - t0
    n_k = int(mask.sum())
    return {"value": round(n_k / dt, 1), "unit": "kept-tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "numpy fp32 oracle, one filtered layer backward of the whole batch (B=%d,S=%d, %d kept tokens), %.1f s"
                      % (shape.B, shape.S, n_k, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="index into the workload table (default: 8B shape)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the keep-ratio sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-parts", action="store_true", help="skip the per-part timings")
    ap.add_argument("--only-roofline", action="store_true",
                    help="run the roofline leg alone (the dominant GEMM and the measured MFMA ceiling) and print it; "
                         "the short command that the profiler counter runs use")
    ap.add_argument("--lora", action="store_true", help="also time the LoRA-adapted layer backward (rank 64)")
    ap.add_argument("--main-grad", action="store_true",
                    help="also time the layer with fp32 main-gradient accumulation of the parameter gradients")
    ap.add_argument("--stack", type=int, default=0, metavar="L",
                    help="also time a stack of L layers chained through the compact entry point")
    ap.add_argument("--context-sweep", action="store_true",
                    help="also time context lengths 1K..32K and keep ratios 0.1..1.0 on the bench config (slow)")
    ap.add_argument("--sweep-configs", default="", metavar="I,J,..",
                    help="run ONLY the context-length and keep-ratio sweeps, on these configs (e.g. 1,2,3,4), and print them")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (collectives and sharding are out of scope); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    Bn.lib()        # fail loudly if the HIP library is missing

    shape = WL.CONFIGS[a.config]
    if a.sweep_configs:
        res = {}
        for ci in [int(x) for x in a.sweep_configs.split(",")]:
            res["config %d %s" % (ci, WL.CONFIGS[ci].name)] = context_sweep_leg(WL.CONFIGS[ci], a.steps, a.warmup)
        print(json.dumps({"context_and_ratio_sweeps": res}), flush=True)
        return
    if a.only_roofline:
        n_k = shape.B * WL.topk_count(shape.rho, shape.S)
        print(json.dumps({"roofline": roofline_leg(shape, n_k), "hbm_copy_ceiling": copy_ceiling_leg()}), flush=True)
        return
    log("config %d %s: generating inputs" % (a.config, shape.name))
    W, sv, dy, mask, rng = make_inputs(shape, WL.config_seed(a.config))
    mask_dev = torch.from_numpy(mask).to(DEV)
    desc = Bn.make_desc(shape.B, shape.S, shape.H, shape.Hq, shape.Hkv, shape.d, shape.F, shape.dtype)
    plan = Bn.LayerBackward(desc, device=DEV)
    n_k = int(mask.sum())

    log("timing filtered backward (n_kept=%d of %d)" % (n_k, shape.T))
    # cf_layer_bwd_filtered never synchronises (every kernel reads N_k on the device): K calls are
    # enqueued back to back, bracketed by the two synchronisations of time_steps
    t_f = time_steps(lambda: plan.filtered_async(sv, W, dy, mask_dev), a.steps, a.warmup)
    assert plan.n_kept() == n_k
    ev_f = event_times(lambda: plan.filtered_async(sv, W, dy, mask_dev), a.steps, 0)
    # the same composed from the single-purpose calls by a caller that knows N_k beforehand (top-k keeps
    # a fixed count): index build, gather of the upstream gradient, compact call with the host count
    t_k = time_steps(lambda: plan.filtered_known(sv, W, dy, mask_dev, n_k), a.steps, a.warmup)
    # and with the host waiting for N_k after every call
    t_w = time_steps(lambda: plan.filtered(sv, W, dy, mask_dev), a.steps, a.warmup)
    log("timing dense backward")
    t_d = time_steps(lambda: plan.dense(sv, W, dy), a.steps, a.warmup)
    flops_f = layer_alg_flops(shape, mask)
    flops_d = layer_alg_flops(shape, np.ones_like(mask))

    sweep = {}
    if not a.no_sweep:
        for rho in (1.0, 0.7, 0.5, 0.3):
            m = WL.mask_topk(rng, shape.B, shape.S, rho)
            md = torch.from_numpy(m).to(DEV)
            t = time_steps(lambda: plan.filtered_async(sv, W, dy, md), a.steps, a.warmup)
            sweep["%.1f" % rho] = {"ms": round(t * 1e3, 4), "speedup_vs_dense": round(t_d / t, 4),
                                   "kept_tokens_per_s": round(int(m.sum()) / t, 1),
                                   "tflops": round(layer_alg_flops(shape, m) / t / 1e12, 1)}
            log("rho %.1f: %.3f ms, speedup %.3f" % (rho, t * 1e3, t_d / t))

    # one plain device copy of known size (1 GiB read + 1 GiB written): the reference that
    # the HBM byte counters of a profiler run are scaled by
    calib = torch.empty(1 << 28, dtype=torch.float32, device=DEV)
    calib2 = torch.empty_like(calib)
    calib.fill_(1.0)
    calib2.copy_(calib)
    torch.cuda.synchronize()
    del calib, calib2

    parts = None
    if not a.no_parts:
        log("per-part timings")
        parts = parts_leg(shape, sv, W, dy, mask, mask_dev)
    ctx = None
    if a.context_sweep:
        log("context-length and keep-ratio sweeps")
        ctx = context_sweep_leg(shape, a.steps, a.warmup)
    lora = None
    if a.lora:
        log("LoRA leg")
        lora = lora_leg(shape, sv, W, dy, mask_dev, rng, a.steps, a.warmup)
        log("LoRA: filtered %.3f ms dense %.3f ms speedup %.3f" % (lora["filtered_ms"], lora["dense_ms"], lora["speedup"]))
    mgrad = None
    if a.main_grad:
        log("main-grad leg")
        mgrad = main_grad_leg(desc, sv, W, dy, mask_dev, a.steps, a.warmup)
        log("main-grad: filtered %.3f ms dense %.3f ms speedup %.3f" % (mgrad["filtered_ms"], mgrad["dense_ms"], mgrad["speedup"]))
    stack = None
    if a.stack > 0:
        log("stack leg")
        stack = stack_leg(desc, sv, W, dy, mask_dev, a.stack, max(1, a.steps // 2), 1)
        log("stack of %d: filtered %.3f ms/layer dense %.3f ms/layer speedup %.3f"
            % (a.stack, stack["filtered_ms_per_layer"], stack["dense_ms_per_layer"], stack["speedup"]))
    log("roofline leg")
    roof = roofline_leg(shape, n_k)
    cpu = None
    if not a.no_cpu:
        log("cpu oracle leg")
        cpu = cpu_baseline_leg(shape, W, sv, dy, mask)

    tfl = flops_f / t_f / 1e12
    out = {
        "metric": "filtered layer-bwd kept-tokens/s + speedup vs dense bwd at 50% keep; MFMA % peak",
        "value": round(n_k / t_f, 1), "unit": "kept-tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(t_f * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype,
        "data": "synthetic",
        "config": {"workload": "config %d: %s layer, B=%d S=%d H=%d Hq=%d Hkv=%d d=%d F=%d, keep ratio %.2f, mask %s"
                               % (a.config, shape.name, shape.B, shape.S, shape.H, shape.Hq, shape.Hkv, shape.d,
                                  shape.F, n_k / shape.T, shape.mask_kind),
                   "n_kept": n_k, "tokens": shape.T},
        "speedup_vs_dense": round(t_d / t_f, 4),
        "ms_per_step_count_known": round(t_k * 1e3, 4),
        "ms_per_step_host_reads_count_every_step": round(t_w * 1e3, 4),
        "dense_ms_per_step": round(t_d * 1e3, 4),
        "median_ms_per_step_events": round(float(np.median(ev_f)), 4),
        "algorithmic_tflops": round(tfl, 1), "mfma_frac_of_peak_layer": round(tfl / PEAK_BF16_TFLOPS, 4),
        "dense_algorithmic_tflops": round(flops_d / t_d / 1e12, 1),
        "keep_ratio_sweep": sweep,
        "parts": parts,
        "context_sweep": ctx,
        "lora": lora,
        "main_grad": mgrad,
        "stack": stack,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
