"""ctypes binding of the C-ABI library (include/centrifuge.h).

Argument marshalling only: every step of the path runs inside the HIP
library.  torch supplies device memory and the current stream.  There is no
CPU fallback: if the library has not been built, `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcentrifuge.so")

CF_BF16, CF_F32 = 0, 1
_STATUS = {0: "CF_OK", 1: "CF_ERR_NULL", 2: "CF_ERR_SHAPE", 3: "CF_ERR_DTYPE", 4: "CF_ERR_WORKSPACE",
           5: "CF_ERR_UNSUPPORTED", 6: "CF_ERR_HIP"}

EXPORTS = (
    "cf_status_str", "cf_version", "cf_index_workspace_bytes", "cf_build_keep_index",
    "cf_build_keep_index_static", "cf_gather_rows",
    "cf_linear_bwd_reduced", "cf_attn_workspace_bytes", "cf_attn_bwd_filtered",
    "cf_layer_workspace_bytes", "cf_layer_bwd_filtered", "cf_layer_bwd_compact", "cf_layer_bwd_compact_dev",
    "cf_layer_bwd_dense",
    "cf_lora_workspace_bytes", "cf_layer_bwd_lora", "cf_probe_mfma_bf16", "cf_probe_mfma_lds_bf16",
    "cf_probe_copy",
)


class CfError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, _STATUS.get(code, "?"), code))


class LayerDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("S", C.c_int32), ("H", C.c_int32), ("Hq", C.c_int32),
                ("Hkv", C.c_int32), ("d", C.c_int32), ("F", C.c_int32), ("dtype", C.c_int32),
                ("rms_eps", C.c_float), ("softmax_scale", C.c_float)]


class Saved(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("x", "q", "k", "v", "attn_out", "lse", "r", "gate", "up",
                                           "rope_cos", "rope_sin")]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")]


GRAD_NAMES = ("dwq", "dwk", "dwv", "dwo", "dwg", "dwu", "dwd", "dg1", "dg2", "dx")


class Grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in GRAD_NAMES] + [("main_grad", C.c_int32)]


_LORA_T = ("aq", "bq", "ak", "bk", "av", "bv", "ao", "bo")


class Lora(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LORA_T] + [("rank", C.c_int32), ("scale", C.c_float)]


class LoraGrads(C.Structure):
    _fields_ = [("d" + n, C.c_void_p) for n in _LORA_T] + [("dx", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Load libcentrifuge.so (built by paper_2502_00340_amd.build).  Raises if missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library not built: %s is missing (run __graft_entry__.build())" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    L.cf_status_str.restype = C.c_char_p
    L.cf_status_str.argtypes = [C.c_int]
    L.cf_version.restype = C.c_char_p
    L.cf_version.argtypes = []
    L.cf_index_workspace_bytes.restype = sz
    L.cf_index_workspace_bytes.argtypes = [i64]
    L.cf_build_keep_index.restype = C.c_int
    L.cf_build_keep_index.argtypes = [vp, i32, i32, vp, vp, vp, C.POINTER(i32), vp, sz, vp]
    L.cf_build_keep_index_static.restype = C.c_int
    L.cf_build_keep_index_static.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    L.cf_gather_rows.restype = C.c_int
    L.cf_gather_rows.argtypes = [vp, i64, i64, i32, vp, vp, i32, vp, vp]
    L.cf_linear_bwd_reduced.restype = C.c_int
    L.cf_linear_bwd_reduced.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, f32, vp]
    L.cf_attn_workspace_bytes.restype = sz
    L.cf_attn_workspace_bytes.argtypes = [C.POINTER(LayerDesc), i32]
    L.cf_attn_bwd_filtered.restype = C.c_int
    L.cf_attn_bwd_filtered.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                       vp, vp, vp, vp, sz, vp]
    L.cf_layer_workspace_bytes.restype = sz
    L.cf_layer_workspace_bytes.argtypes = [C.POINTER(LayerDesc), i32]
    L.cf_layer_bwd_filtered.restype = C.c_int
    L.cf_layer_bwd_filtered.argtypes = [C.POINTER(LayerDesc), C.POINTER(Saved), C.POINTER(Weights), vp, vp, i32,
                                        C.POINTER(Grads), vp, vp, vp, C.POINTER(i32), vp, sz, vp]
    L.cf_layer_bwd_compact_dev.restype = C.c_int
    L.cf_layer_bwd_compact_dev.argtypes = [C.POINTER(LayerDesc), C.POINTER(Saved), C.POINTER(Weights), vp, vp, vp,
                                           vp, i32, C.POINTER(Grads), vp, sz, vp]
    L.cf_layer_bwd_compact.restype = C.c_int
    L.cf_layer_bwd_compact.argtypes = [C.POINTER(LayerDesc), C.POINTER(Saved), C.POINTER(Weights), vp, vp, vp,
                                       i32, C.POINTER(Grads), vp, sz, vp]
    L.cf_layer_bwd_dense.restype = C.c_int
    L.cf_layer_bwd_dense.argtypes = [C.POINTER(LayerDesc), C.POINTER(Saved), C.POINTER(Weights), vp,
                                     C.POINTER(Grads), vp, sz, vp]
    L.cf_lora_workspace_bytes.restype = sz
    L.cf_lora_workspace_bytes.argtypes = [C.POINTER(LayerDesc), i32, i32]
    L.cf_layer_bwd_lora.restype = C.c_int
    L.cf_layer_bwd_lora.argtypes = [C.POINTER(LayerDesc), C.POINTER(Saved), C.POINTER(Weights), C.POINTER(Lora), vp,
                                    vp, i32, C.POINTER(LoraGrads), vp, vp, vp, C.POINTER(i32), vp, sz, vp]
    L.cf_probe_mfma_bf16.restype = C.c_int
    L.cf_probe_mfma_bf16.argtypes = [i32, i32, vp, C.POINTER(C.c_double), vp]
    L.cf_probe_mfma_lds_bf16.restype = C.c_int
    L.cf_probe_mfma_lds_bf16.argtypes = [i32, i32, i32, vp, C.POINTER(C.c_double), vp]
    L.cf_probe_copy.restype = C.c_int
    L.cf_probe_copy.argtypes = [vp, vp, sz, vp]
    _lib = L
    return L


def _check(code: int, where: str):
    if code != 0:
        raise CfError(code, where)


_dummy = {}


def _ptr(t):
    """Device pointer of a tensor; an empty tensor (no storage) maps to a small
    dummy allocation so that "zero rows" is not mistaken for a NULL argument."""
    if t is None:
        return None
    if t.numel() == 0:
        key = str(t.device)
        if key not in _dummy:
            _dummy[key] = torch.zeros(256, dtype=torch.uint8, device=t.device)
        return C.c_void_p(_dummy[key].data_ptr())
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return CF_BF16
    if t.dtype == torch.float32:
        return CF_F32
    raise TypeError("unsupported dtype %s" % t.dtype)


def make_desc(B, S, H, Hq, Hkv, d, F, dtype, rms_eps=1e-5, softmax_scale=0.0) -> LayerDesc:
    code = {"bf16": CF_BF16, "f32": CF_F32, torch.bfloat16: CF_BF16, torch.float32: CF_F32}[dtype]
    return LayerDesc(B, S, H, Hq, Hkv, d, F, code, rms_eps, softmax_scale)


def torch_dtype(desc: LayerDesc):
    return torch.bfloat16 if desc.dtype == CF_BF16 else torch.float32


# --------------------------------------------------------------------------
# entry points (same names as the C ABI, without the prefix)
# --------------------------------------------------------------------------

def build_keep_index(mask: torch.Tensor, sync: bool = True):
    """mask: uint8 [B,S] on the GPU.  Returns (idx [T] int32 - first N_k valid,
    cu_kept [B+1] int32, n_kept_dev [1] int32, N_k or None)."""
    assert mask.dtype == torch.uint8 and mask.is_cuda and mask.dim() == 2 and mask.is_contiguous()
    B, S = mask.shape
    dev = mask.device
    idx = torch.empty(B * S, dtype=torch.int32, device=dev)
    cu = torch.empty(B + 1, dtype=torch.int32, device=dev)
    n_dev = torch.empty(1, dtype=torch.int32, device=dev)
    wsb = lib().cf_index_workspace_bytes(B * S)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    n_host = C.c_int32(-1)
    _check(lib().cf_build_keep_index(_ptr(mask), B, S, _ptr(idx), _ptr(cu), _ptr(n_dev),
                                     C.byref(n_host) if sync else None, _ptr(ws), wsb, _stream()),
           "cf_build_keep_index")
    return idx, cu, n_dev, (int(n_host.value) if sync else None)


def build_keep_index_static(mask: torch.Tensor, idx: torch.Tensor, cu_kept: torch.Tensor, n_kept_dev: torch.Tensor):
    """cf_build_keep_index_static: every buffer is the caller's, nothing is allocated or read back."""
    assert mask.dtype == torch.uint8 and mask.is_cuda and mask.dim() == 2 and mask.is_contiguous()
    B, S = mask.shape
    assert idx.dtype == torch.int32 and idx.numel() >= B * S and cu_kept.numel() >= B + 1
    _check(lib().cf_build_keep_index_static(_ptr(mask), B, S, _ptr(idx), _ptr(cu_kept), _ptr(n_kept_dev),
                                            _stream()), "cf_build_keep_index_static")


def gather_rows(src: torch.Tensor, idx: torch.Tensor, n_rows: int, out: torch.Tensor | None = None,
                n_kept_dev: torch.Tensor | None = None):
    """n_kept_dev None: exactly n_rows rows.  Otherwise min(*n_kept_dev, n_rows) rows are copied (the
    count is read on the device) and `out` has room for n_rows."""
    assert src.is_cuda and src.dim() == 2 and src.is_contiguous() and idx.dtype == torch.int32
    rows, cols = src.shape
    if out is None:
        out = torch.empty((n_rows, cols), dtype=src.dtype, device=src.device)
    _check(lib().cf_gather_rows(_ptr(src), rows, cols, _dtype_code(src), _ptr(idx), _ptr(n_kept_dev), n_rows,
                                _ptr(out), _stream()), "cf_gather_rows")
    return out


def linear_bwd_reduced(x_kept, dy_kept, w, need_dx=True, need_dw=True, dw_accumulate_into=None):
    """Returns (dx_kept or None, dw or None)."""
    n_kept, out_f = dy_kept.shape
    in_f = w.shape[0] if w is not None else x_kept.shape[1]
    dev = dy_kept.device
    dx = torch.empty((n_kept, in_f), dtype=dy_kept.dtype, device=dev) if need_dx else None
    beta = 0.0
    dw = None
    if need_dw:
        if dw_accumulate_into is not None:
            dw, beta = dw_accumulate_into, 1.0
        else:
            dw = torch.empty((in_f, out_f), dtype=dy_kept.dtype, device=dev)
    _check(lib().cf_linear_bwd_reduced(_ptr(x_kept), _ptr(dy_kept), _ptr(w), n_kept, in_f, out_f,
                                       _dtype_code(dy_kept), _ptr(dx), _ptr(dw), beta, _stream()),
           "cf_linear_bwd_reduced")
    return dx, dw


def attn_bwd_filtered(desc: LayerDesc, q_kept, k_full, v_full, o_kept, lse_full, do_kept, idx, cu_kept,
                      n_kept: int):
    dev = q_kept.device
    Nq, Nkv = desc.Hq * desc.d, desc.Hkv * desc.d
    dt = torch_dtype(desc)
    dq = torch.empty((n_kept, Nq), dtype=dt, device=dev)
    dk = torch.empty((n_kept, Nkv), dtype=dt, device=dev)
    dv = torch.empty((n_kept, Nkv), dtype=dt, device=dev)
    wsb = lib().cf_attn_workspace_bytes(C.byref(desc), n_kept)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device=dev)
    _check(lib().cf_attn_bwd_filtered(C.byref(desc), _ptr(q_kept), _ptr(k_full), _ptr(v_full), _ptr(o_kept),
                                      _ptr(lse_full), _ptr(do_kept), _ptr(idx), _ptr(cu_kept), n_kept,
                                      _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), ws.numel(), _stream()),
           "cf_attn_bwd_filtered")
    return dq, dk, dv


_SAVED = ("x", "q", "k", "v", "attn_out", "lse", "r", "gate", "up")
_WEIGHTS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")


class LayerBackward:
    """Pre-allocated outputs + workspace for repeated calls on one layer shape."""

    def __init__(self, desc: LayerDesc, device="cuda:0", max_kept: int | None = None, main_grad: bool = False):
        """main_grad: the parameter gradients are fp32 buffers, zeroed here, that every call adds to."""
        self.desc = desc
        self.device = torch.device(device)
        dt = torch_dtype(desc)
        T = desc.B * desc.S
        H, F, Nq, Nkv = desc.H, desc.F, desc.Hq * desc.d, desc.Hkv * desc.d
        self.max_kept = T if max_kept is None else max_kept
        e = lambda *s: torch.empty(s, dtype=dt, device=self.device)
        p = (lambda *s: torch.zeros(s, dtype=torch.float32, device=self.device)) if main_grad else e
        self.grads = dict(dwq=p(H, Nq), dwk=p(H, Nkv), dwv=p(H, Nkv), dwo=p(Nq, H), dwg=p(H, F), dwu=p(H, F),
                          dwd=p(F, H), dg1=p(H), dg2=p(H), dx=e(T, H))
        # zeros, not empty: entries past N_k are never written, and must stay valid row numbers for a
        # caller that passes a wrong count to filtered_known
        self.idx = torch.zeros(T, dtype=torch.int32, device=self.device)
        self.cu_kept = torch.empty(desc.B + 1, dtype=torch.int32, device=self.device)
        self.ws_bytes = lib().cf_layer_workspace_bytes(C.byref(desc), self.max_kept)
        if self.ws_bytes == 0:
            raise CfError(2, "cf_layer_workspace_bytes")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        self._g = Grads(*([self.grads[n].data_ptr() for n in GRAD_NAMES] + [1 if main_grad else 0]))
        self.n_kept_dev = torch.zeros(1, dtype=torch.int32, device=self.device)
        # N_k comes back through page-locked host memory: the copy is asynchronous
        self._n_host = torch.empty(1, dtype=torch.int32).pin_memory()

    def _pack(self, saved: dict, weights: dict):
        rope = [saved[n].data_ptr() if saved.get(n) is not None else None for n in ("rope_cos", "rope_sin")]
        sv = Saved(*([saved[n].data_ptr() for n in _SAVED] + rope))
        w = Weights(*[weights[n].data_ptr() for n in _WEIGHTS])
        return sv, w

    def filtered_async(self, saved: dict, weights: dict, dy: torch.Tensor, mask: torch.Tensor) -> None:
        """Enqueues cf_layer_bwd_filtered and returns at once: nothing is read back and the stream is
        not synchronised.  Results land in self.grads (dx: first N_k rows), self.idx, self.cu_kept,
        self.n_kept_dev; the page-locked word behind n_kept() holds N_k once the stream has run."""
        sv, w = self._pack(saved, weights)
        self._n_host[0] = -1
        _check(lib().cf_layer_bwd_filtered(C.byref(self.desc), C.byref(sv), C.byref(w), _ptr(dy), _ptr(mask),
                                           self.max_kept, C.byref(self._g), _ptr(self.idx), _ptr(self.cu_kept),
                                           _ptr(self.n_kept_dev),
                                           C.cast(self._n_host.data_ptr(), C.POINTER(C.c_int32)), _ptr(self.ws),
                                           self.ws_bytes, _stream()),
               "cf_layer_bwd_filtered")

    def n_kept(self) -> int:
        """N_k of the last filtered call (synchronises the current stream)."""
        torch.cuda.current_stream().synchronize()
        return int(self._n_host[0])

    def filtered(self, saved: dict, weights: dict, dy: torch.Tensor, mask: torch.Tensor) -> int:
        """filtered_async, then waits for the stream and returns N_k."""
        self.filtered_async(saved, weights, dy, mask)
        return self.n_kept()

    def filtered_known(self, saved: dict, weights: dict, dy: torch.Tensor, mask: torch.Tensor, n_kept: int) -> None:
        """The filtered backward composed from the single-purpose calls by a caller that knows N_k
        beforehand (a fixed keep ratio: top-k per sequence gives N_k = B*k): cf_build_keep_index
        without the host copy, cf_gather_rows of the upstream gradient, cf_layer_bwd_compact with the
        host count.  n_kept must be the number of non-zero mask bytes."""
        if not hasattr(self, "_index_ws"):
            wsb = lib().cf_index_workspace_bytes(self.desc.B * self.desc.S)
            self._index_ws = torch.empty(wsb, dtype=torch.uint8, device=self.device)
            self._dy_kept = torch.empty((self.desc.B * self.desc.S, self.desc.H), dtype=dy.dtype, device=self.device)
        _check(lib().cf_build_keep_index(_ptr(mask), self.desc.B, self.desc.S, _ptr(self.idx), _ptr(self.cu_kept),
                                         _ptr(self.n_kept_dev), None, _ptr(self._index_ws), self._index_ws.numel(),
                                         _stream()), "cf_build_keep_index")
        _check(lib().cf_gather_rows(_ptr(dy), dy.shape[0], dy.shape[1], _dtype_code(dy), _ptr(self.idx), None, n_kept,
                                    _ptr(self._dy_kept), _stream()), "cf_gather_rows")
        self.compact(saved, weights, self._dy_kept, self.idx, self.cu_kept, n_kept)

    def compact_dev(self, saved: dict, weights: dict, dy_kept: torch.Tensor, idx: torch.Tensor,
                    cu_kept: torch.Tensor, n_kept_dev: torch.Tensor) -> None:
        """cf_layer_bwd_compact_dev: a layer below the index-building one, with the count still on the
        device (no host read anywhere in the stack)."""
        sv, w = self._pack(saved, weights)
        _check(lib().cf_layer_bwd_compact_dev(C.byref(self.desc), C.byref(sv), C.byref(w), _ptr(dy_kept), _ptr(idx),
                                              _ptr(cu_kept), _ptr(n_kept_dev), self.max_kept, C.byref(self._g),
                                              _ptr(self.ws), self.ws_bytes, _stream()),
               "cf_layer_bwd_compact_dev")

    def compact(self, saved: dict, weights: dict, dy_kept: torch.Tensor, idx: torch.Tensor,
                cu_kept: torch.Tensor, n_kept: int) -> None:
        """Runs cf_layer_bwd_compact for a layer below the one that built (idx, cu_kept); results
        land in self.grads (dx: first n_kept rows).  No host synchronisation."""
        sv, w = self._pack(saved, weights)
        _check(lib().cf_layer_bwd_compact(C.byref(self.desc), C.byref(sv), C.byref(w), _ptr(dy_kept), _ptr(idx),
                                          _ptr(cu_kept), n_kept, C.byref(self._g), _ptr(self.ws),
                                          self.ws_bytes, _stream()),
               "cf_layer_bwd_compact")

    def dense(self, saved: dict, weights: dict, dy: torch.Tensor) -> None:
        sv, w = self._pack(saved, weights)
        _check(lib().cf_layer_bwd_dense(C.byref(self.desc), C.byref(sv), C.byref(w), _ptr(dy),
                                        C.byref(self._g), _ptr(self.ws), self.ws_bytes, _stream()),
               "cf_layer_bwd_dense")


def layer_bwd_filtered(desc, saved, weights, dy, mask):
    plan = LayerBackward(desc, device=dy.device)
    n = plan.filtered(saved, weights, dy, mask)
    out = dict(plan.grads)
    out["dx"] = out["dx"][:n]
    return out, plan.idx[:n], plan.cu_kept, n


def layer_bwd_dense(desc, saved, weights, dy):
    plan = LayerBackward(desc, device=dy.device)
    plan.dense(saved, weights, dy)
    return dict(plan.grads)


class LoraBackward(LayerBackward):
    """Pre-allocated adapter gradients + workspace for cf_layer_bwd_lora (base weights frozen)."""

    def __init__(self, desc: LayerDesc, rank: int, device="cuda:0"):
        self.desc = desc
        self.device = torch.device(device)
        self.rank = rank
        dt = torch_dtype(desc)
        T = desc.B * desc.S
        H, Nq, Nkv = desc.H, desc.Hq * desc.d, desc.Hkv * desc.d
        e = lambda *s: torch.empty(s, dtype=dt, device=self.device)
        self.grads = dict(daq=e(H, rank), dbq=e(rank, Nq), dak=e(H, rank), dbk=e(rank, Nkv), dav=e(H, rank),
                          dbv=e(rank, Nkv), dao=e(Nq, rank), dbo=e(rank, H), dx=e(T, H))
        # zeros, not empty: entries past N_k are never written, and must stay valid row numbers for a
        # caller that passes a wrong count to filtered_known
        self.idx = torch.zeros(T, dtype=torch.int32, device=self.device)
        self.cu_kept = torch.empty(desc.B + 1, dtype=torch.int32, device=self.device)
        self.ws_bytes = lib().cf_lora_workspace_bytes(C.byref(desc), rank, T)
        if self.ws_bytes == 0:
            raise CfError(2, "cf_lora_workspace_bytes")
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        self._g = LoraGrads(*[self.grads[n].data_ptr() for n, _ in LoraGrads._fields_])
        self.max_kept = T
        self.n_kept_dev = torch.zeros(1, dtype=torch.int32, device=self.device)
        self._n_host = torch.empty(1, dtype=torch.int32).pin_memory()

    def run_async(self, saved: dict, weights: dict, lora: dict, dy: torch.Tensor, mask: torch.Tensor | None) -> None:
        """mask None: every token kept (the dense LoRA backward).  Nothing synchronises: the kept count is
        in self.n_kept_dev, and n_kept() reads the page-locked copy after waiting for the stream."""
        sv, w = self._pack(saved, weights)
        lo = Lora(*([lora[n].data_ptr() for n in _LORA_T] + [self.rank, float(lora["scale"])]))
        self._n_host[0] = -1
        _check(lib().cf_layer_bwd_lora(C.byref(self.desc), C.byref(sv), C.byref(w), C.byref(lo), _ptr(dy),
                                       _ptr(mask), self.max_kept, C.byref(self._g), _ptr(self.idx),
                                       _ptr(self.cu_kept), _ptr(self.n_kept_dev),
                                       C.cast(self._n_host.data_ptr(), C.POINTER(C.c_int32)), _ptr(self.ws),
                                       self.ws_bytes, _stream()),
               "cf_layer_bwd_lora")

    def run(self, saved: dict, weights: dict, lora: dict, dy: torch.Tensor, mask: torch.Tensor | None) -> int:
        """run_async, then waits for the stream and returns N_k."""
        self.run_async(saved, weights, lora, dy, mask)
        torch.cuda.current_stream().synchronize()
        return int(self._n_host[0])
