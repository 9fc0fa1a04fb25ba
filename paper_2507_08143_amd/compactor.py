"""Thin ctypes binding of libcompactor.so (argument marshalling only).

Every function here has the name of the C entry point it calls
(include/compactor.h) and does nothing but turn torch tensors into raw device
pointers, allocate the outputs with torch, and check the return code.  All of
the method's arithmetic runs in the HIP kernels; there is no CPU fallback: if
the shared library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("COMPACTOR_LIB", os.path.join(_HERE, "libcompactor.so"))

if not os.path.exists(_LIB_PATH):
    raise ImportError(
        "libcompactor.so is not built: run `python -m paper_2507_08143_amd.build` "
        "(needs hipcc; cross-compiles for gfx950 without a GPU)")

_lib = C.CDLL(_LIB_PATH)

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EALIGN, EHIP = 0, -1, -2, -3, -4, -5
STATUS_OK, STATUS_PIVOT, STATUS_NONFINITE = 0, 1, 2


class _Request(C.Structure):
    _fields_ = [("k_score", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("attn", C.c_void_p), ("stride_l", C.c_int64), ("stride_h", C.c_int64),
                ("stride_t", C.c_int64), ("n", C.c_int32), ("ratio", C.c_float)]


class _Params(C.Structure):
    _fields_ = [("layers", C.c_int32), ("kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("sketch_dim", C.c_int32), ("phi", C.c_void_p), ("ridge_rel", C.c_float),
                ("lambda_blend", C.c_float), ("group_bytes", C.c_int64),
                ("gram_wgs", C.c_int32), ("score_tokens", C.c_int32),
                ("select_scope", C.c_int32), ("stage_events", C.c_void_p)]


class _AttnRequest(C.Structure):
    _fields_ = [("q", C.c_void_p), ("k", C.c_void_p),
                ("q_stride_l", C.c_int64), ("q_stride_h", C.c_int64), ("q_stride_t", C.c_int64),
                ("k_stride_l", C.c_int64), ("k_stride_h", C.c_int64), ("k_stride_t", C.c_int64),
                ("n", C.c_int32)]


class _AttnParams(C.Structure):
    _fields_ = [("layers", C.c_int32), ("kv_heads", C.c_int32), ("q_heads", C.c_int32),
                ("head_dim", C.c_int32), ("chunk", C.c_int32), ("pool", C.c_int32),
                ("scale", C.c_float)]


class _PagePool(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p),
                ("page_stride", C.c_int64), ("layer_stride", C.c_int64),
                ("head_stride", C.c_int64), ("slot_stride", C.c_int64),
                ("page_size", C.c_int32), ("num_pages", C.c_int32)]


class _PageTable(C.Structure):
    _fields_ = [("pages", C.c_void_p), ("len", C.c_int32)]


_PP, _RP = C.POINTER(_Params), C.POINTER(_Request)
_APP, _ARP = C.POINTER(_AttnParams), C.POINTER(_AttnRequest)
_lib.compactor_attention_workspace_size.argtypes = [_APP, _ARP, C.c_int32, C.POINTER(C.c_size_t)]
_lib.compactor_attention_scores.argtypes = [_APP, _ARP, C.c_int32, C.c_void_p, C.c_void_p,
                                            C.c_size_t, C.c_void_p]
_lib.compactor_default_params.argtypes = [_PP, C.c_int32, C.c_int32]
_lib.compactor_default_params.restype = None
_lib.compactor_keep_count.argtypes = [C.c_int32, C.c_float]
_lib.compactor_keep_count.restype = C.c_int32
_lib.compactor_layout.argtypes = [_PP, _RP, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                  C.POINTER(C.c_int32)]
_lib.compactor_srht_phi.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.compactor_workspace_size.argtypes = [_PP, _RP, C.c_int32, C.POINTER(C.c_size_t)]
_lib.compactor_score.argtypes = [_PP, _RP, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
_lib.compactor_select.argtypes = [_PP, _RP, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                  C.c_void_p, C.c_size_t, C.c_void_p]
_lib.compactor_compact.argtypes = [_PP, _RP, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p]
_lib.compactor_compact_paged.argtypes = [_PP, _RP, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.POINTER(_PagePool), C.POINTER(_PageTable), C.c_int32,
                                         C.c_void_p]
_lib.compactor_compress.argtypes = [_PP, _RP, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                    C.c_void_p]
_lib.compactor_compress_static.argtypes = [_PP, _RP, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.compactor_calibrated_ratio.argtypes = [C.c_double] * 4
_lib.compactor_calibrated_ratio.restype = C.c_double
_lib.compactor_error_string.argtypes = [C.c_int]
_lib.compactor_error_string.restype = C.c_char_p
_lib.compactor_version.restype = C.c_char_p

EXPORTS = ["compactor_default_params", "compactor_keep_count", "compactor_layout",
           "compactor_workspace_size", "compactor_srht_phi", "compactor_score", "compactor_select",
           "compactor_compact", "compactor_compact_paged", "compactor_compress", "compactor_compress_static",
           "compactor_calibrated_ratio",
           "compactor_error_string", "compactor_version",
           "compactor_attention_workspace_size", "compactor_attention_scores"]


STAGES = ["gram", "reduce", "solve", "score", "blend", "select", "gather"]


class StageEvents:
    """COMPACTOR_NUM_STAGES+1 raw hipEvent_t for compactor_params_t.stage_events, created
    through the HIP runtime that torch has already loaded."""

    def __init__(self):
        self._hip = C.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self._hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.array = (C.c_void_p * (len(STAGES) + 1))()
        for i in range(len(STAGES) + 1):
            ev = C.c_void_p()
            if self._hip.hipEventCreate(C.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.array[i] = ev

    def elapsed_ms(self):
        """-> {stage: ms} for the stages whose two events were recorded (after a stream sync)."""
        out = {}
        for i, name in enumerate(STAGES):
            ms = C.c_float(0)
            if self._hip.hipEventElapsedTime(C.byref(ms), self.array[i], self.array[i + 1]) == 0:
                out[name] = float(ms.value)
        self._hip.hipGetLastError()     # asking about a stage that did not run leaves an error pending
        return out

    def __del__(self):
        try:
            for ev in self.array:
                if ev:
                    self._hip.hipEventDestroy(ev)
        except Exception:
            pass


class CompactorError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__("libcompactor: %s (%d)" % (compactor_error_string(code), code))


def _check(rc: int):
    if rc != OK:
        raise CompactorError(rc)


def _require(cond: bool, what: str):
    """The C boundary takes plain pointers and cannot see a tensor's size, type or device: what it
    cannot check is checked here, before anything reaches the GPU."""
    if not cond:
        raise ValueError("compactor: " + what)


def _out(t: Optional[torch.Tensor], numel: int, dtype, name: str):
    """A caller-supplied output (or flat input) buffer: right type, dense, large enough, on the GPU."""
    if t is None:
        return
    _require(t.dtype == dtype, "%s must be %s, got %s" % (name, dtype, t.dtype))
    _require(t.is_contiguous(), "%s must be contiguous" % name)
    _require(t.numel() >= numel, "%s holds %d elements, %d needed" % (name, t.numel(), numel))
    _require(t.is_cuda, "%s must live on the GPU" % name)


SCOPE_HEAD, SCOPE_LAYER = 0, 1


@dataclass
class Params:
    layers: int
    kv_heads: int
    sketch_dim: int = 48
    phi: Optional[torch.Tensor] = None        # fp32 [128, sketch_dim] on the device
    ridge_rel: float = 0.0
    lambda_blend: float = 0.3
    group_bytes: int = 0
    head_dim: int = 128
    stage_events: Optional["StageEvents"] = None   # profiling aid (see the header)
    gram_wgs: int = 0                              # tuning knobs, 0 = library's choice
    score_tokens: int = 0
    select_scope: int = 0                           # SCOPE_HEAD, or SCOPE_LAYER (head-adaptive)

    def c(self, on_gpu: bool = True) -> _Params:
        phi = 0
        if self.phi is not None and self.sketch_dim > 0:
            _require(self.phi.dtype == torch.float32 and self.phi.is_contiguous(),
                     "phi must be a contiguous float32 tensor")
            _require(tuple(self.phi.shape) == (self.head_dim, self.sketch_dim),
                     "phi must have shape [head_dim, sketch_dim] = [%d, %d], got %s"
                     % (self.head_dim, self.sketch_dim, tuple(self.phi.shape)))
            _require(self.phi.is_cuda or not on_gpu, "phi must live on the GPU")
            phi = self.phi.data_ptr()
        ev = C.cast(self.stage_events.array, C.c_void_p) if self.stage_events is not None else None
        return _Params(self.layers, self.kv_heads, self.head_dim, self.sketch_dim, phi,
                       self.ridge_rel, self.lambda_blend, self.group_bytes, self.gram_wgs,
                       self.score_tokens, self.select_scope, ev)


@dataclass
class Request:
    k_score: torch.Tensor                      # bf16 [L, H, n, d], d contiguous
    v_cache: torch.Tensor                      # bf16, same shape and strides
    ratio: float
    k_cache: Optional[torch.Tensor] = None     # bf16, same shape and strides; None = k_score
    attn: Optional[torch.Tensor] = None        # fp32 [L, H, n] contiguous

    def c(self, params: Optional["Params"] = None, on_gpu: bool = True) -> _Request:
        k = self.k_score
        _require(k.dtype == torch.bfloat16 and k.dim() == 4 and k.stride(3) == 1,
                 "k_score must be a bfloat16 tensor [L, H, n, d] with d contiguous")
        if params is not None:
            _require(k.shape[0] == params.layers and k.shape[1] == params.kv_heads and
                     k.shape[3] == params.head_dim,
                     "k_score has shape %s, the parameters say [%d, %d, n, %d]"
                     % (tuple(k.shape), params.layers, params.kv_heads, params.head_dim))
        for name, t in (("v_cache", self.v_cache), ("k_cache", self.k_cache)):
            if t is not None:
                _require(t.dtype == torch.bfloat16 and t.shape == k.shape and t.stride() == k.stride(),
                         "%s must be bfloat16 with the shape and strides of k_score" % name)
                _require(t.is_cuda or not on_gpu, "%s must live on the GPU" % name)
        if self.attn is not None:
            _require(self.attn.dtype == torch.float32 and self.attn.is_contiguous() and
                     self.attn.numel() >= k.shape[0] * k.shape[1] * k.shape[2],
                     "attn must be a contiguous float32 tensor of L*H*n elements")
            _require(self.attn.is_cuda or not on_gpu, "attn must live on the GPU")
        _require(k.is_cuda or not on_gpu, "k_score must live on the GPU")
        return _Request(k.data_ptr(),
                        self.k_cache.data_ptr() if self.k_cache is not None else 0,
                        self.v_cache.data_ptr() if self.v_cache is not None else 0,
                        self.attn.data_ptr() if self.attn is not None else 0,
                        k.stride(0), k.stride(1), k.stride(2), k.shape[2], self.ratio)


def _marshal(params: Params, reqs: Sequence[Request], on_gpu: bool = True):
    _require(len(reqs) >= 1, "at least one request is needed")
    arr = (_Request * len(reqs))(*[r.c(params, on_gpu) for r in reqs])
    return C.byref(params.c(on_gpu)), arr, len(reqs)


def _ptr(t: Optional[torch.Tensor]):
    return 0 if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _device(reqs):
    return reqs[0].k_score.device


def compactor_version() -> str:
    return _lib.compactor_version().decode()


def compactor_error_string(code: int) -> str:
    return _lib.compactor_error_string(code).decode()


def compactor_keep_count(n: int, ratio: float) -> int:
    return int(_lib.compactor_keep_count(n, ratio))


def compactor_calibrated_ratio(nll: float, alpha: float, beta: float, tau: float) -> float:
    return float(_lib.compactor_calibrated_ratio(nll, alpha, beta, tau))


def compactor_default_params(layers: int, kv_heads: int) -> Params:
    p = _Params()
    _lib.compactor_default_params(C.byref(p), layers, kv_heads)
    return Params(p.layers, p.kv_heads, p.sketch_dim, None, p.ridge_rel, p.lambda_blend,
                  p.group_bytes, p.head_dim, None, p.gram_wgs, p.score_tokens, p.select_scope)


def compactor_srht_phi(sketch_dim: int, signs, cols, device, stream=None) -> torch.Tensor:
    """SRHT right-sketch (App. D) -> fp32 [128, sketch_dim] on `device`.  signs: 128 values
    (nonzero = -1); cols: sketch_dim distinct rows of the Hadamard matrix."""
    sg = (C.c_uint8 * 128)(*[1 if int(x) else 0 for x in signs])
    cl = (C.c_int32 * len(cols))(*[int(x) for x in cols])
    _require(len(signs) == 128 and len(cols) == sketch_dim,
             "signs must hold 128 values and cols sketch_dim values")
    phi = torch.empty(128, sketch_dim, dtype=torch.float32, device=device)
    with torch.cuda.device(phi.device):
        _check(_lib.compactor_srht_phi(sketch_dim, sg, cl, _ptr(phi), _stream(stream)))
    return phi


def compactor_layout(params: Params, reqs: Sequence[Request]):
    """-> (score_off[nreq+1], kept_off[nreq+1], k_keep[nreq]) as Python lists."""
    pp, arr, n = _marshal(params, reqs, on_gpu=False)      # a host helper: sizes only
    so, ko, kk = (C.c_int64 * (n + 1))(), (C.c_int64 * (n + 1))(), (C.c_int32 * n)()
    _check(_lib.compactor_layout(pp, arr, n, so, ko, kk))
    return list(so), list(ko), list(kk)


def compactor_workspace_size(params: Params, reqs: Sequence[Request]) -> int:
    pp, arr, n = _marshal(params, reqs, on_gpu=False)
    out = C.c_size_t(0)
    _check(_lib.compactor_workspace_size(pp, arr, n, C.byref(out)))
    return int(out.value)


def _workspace(params, reqs, workspace, stream=None):
    if workspace is None:
        nbytes = max(256, compactor_workspace_size(params, reqs))
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=_device(reqs))
        if stream is not None:
            # the block is used on `stream`, not on the stream torch allocated it for: tell the
            # allocator, or it may hand the block out again while the kernels still run
            workspace.record_stream(stream)
    return workspace


def compactor_score(params: Params, reqs: Sequence[Request], scores=None, status=None,
                    workspace=None, stream=None):
    """-> (scores fp32 [sum L*H*n], status int32 [nreq*L*H])"""
    so, _, _ = compactor_layout(params, reqs)
    dev = _device(reqs)
    if scores is None:
        scores = torch.empty(so[-1], dtype=torch.float32, device=dev)
    if status is None:
        status = torch.empty(len(reqs) * params.layers * params.kv_heads, dtype=torch.int32, device=dev)
    workspace = _workspace(params, reqs, workspace, stream)
    pp, arr, n = _marshal(params, reqs)
    _out(scores, so[-1], torch.float32, "scores")
    _out(status, n * params.layers * params.kv_heads, torch.int32, "status")
    _out(workspace, 0, torch.uint8, "workspace")
    _check(_lib.compactor_score(pp, arr, n, _ptr(scores), _ptr(status), _ptr(workspace),
                                workspace.numel(), _stream(stream)))
    return scores, status


def compactor_select(params: Params, reqs: Sequence[Request], scores: torch.Tensor,
                     kept_idx=None, kept_cnt=None, workspace=None, stream=None):
    """-> (kept_idx int32 [sum L*H*k_keep], kept_cnt int32 [nreq*L*H])"""
    _, ko, _ = compactor_layout(params, reqs)
    dev = scores.device
    if kept_idx is None:
        kept_idx = torch.empty(ko[-1], dtype=torch.int32, device=dev)
    if kept_cnt is None:
        kept_cnt = torch.empty(len(reqs) * params.layers * params.kv_heads, dtype=torch.int32, device=dev)
    pp, arr, n = _marshal(params, reqs)
    workspace = _workspace(params, reqs, workspace, stream)
    so, _, _ = compactor_layout(params, reqs)
    _out(scores, so[-1], torch.float32, "scores")
    _out(kept_idx, ko[-1], torch.int32, "kept_idx")
    _out(kept_cnt, n * params.layers * params.kv_heads, torch.int32, "kept_cnt")
    _out(workspace, 0, torch.uint8, "workspace")
    _check(_lib.compactor_select(pp, arr, n, _ptr(scores), _ptr(kept_idx), _ptr(kept_cnt),
                                 _ptr(workspace), workspace.numel(), _stream(stream)))
    return kept_idx, kept_cnt


def compactor_compact(params: Params, reqs: Sequence[Request], kept_idx: torch.Tensor,
                      kept_cnt: torch.Tensor, k_packed=None, v_packed=None, stream=None):
    """-> (k_packed, v_packed) bf16 [sum L*H*k_keep, d]"""
    _, ko, _ = compactor_layout(params, reqs)
    dev = _device(reqs)
    if k_packed is None:
        k_packed = torch.empty(ko[-1], params.head_dim, dtype=torch.bfloat16, device=dev)
    if v_packed is None:
        v_packed = torch.empty(ko[-1], params.head_dim, dtype=torch.bfloat16, device=dev)
    pp, arr, n = _marshal(params, reqs)
    _out(kept_idx, ko[-1], torch.int32, "kept_idx")
    _out(kept_cnt, n * params.layers * params.kv_heads, torch.int32, "kept_cnt")
    _out(k_packed, ko[-1] * params.head_dim, torch.bfloat16, "k_packed")
    _out(v_packed, ko[-1] * params.head_dim, torch.bfloat16, "v_packed")
    _check(_lib.compactor_compact(pp, arr, n, _ptr(kept_idx), _ptr(kept_cnt), _ptr(k_packed),
                                  _ptr(v_packed), _stream(stream)))
    return k_packed, v_packed


def compactor_compact_paged(params: Params, reqs: Sequence[Request], kept_idx: torch.Tensor,
                            kept_cnt: torch.Tensor, k_pages: torch.Tensor, v_pages: torch.Tensor,
                            tables: Sequence[torch.Tensor], in_place: bool = False, stream=None):
    """Retained rows into a paged cache.  k_pages / v_pages: bf16 views indexed
    [page, layer, slot, head, channel] (any strides, channel contiguous, the same for both);
    tables[b]: int32 device tensor, physical page of each logical page of request b."""
    _require(k_pages.dtype == torch.bfloat16 and v_pages.dtype == torch.bfloat16,
             "k_pages and v_pages must be bfloat16")
    _require(k_pages.dim() == 5 and k_pages.stride(4) == 1 and v_pages.shape == k_pages.shape and
             v_pages.stride() == k_pages.stride(),
             "k_pages and v_pages must be [page, layer, slot, head, channel] views of equal shape and "
             "strides, channel contiguous")
    _require(k_pages.shape[1] == params.layers and k_pages.shape[3] == params.kv_heads and
             k_pages.shape[4] == params.head_dim,
             "the page pool has shape %s, the parameters say [pages, %d, slots, %d, %d]"
             % (tuple(k_pages.shape), params.layers, params.kv_heads, params.head_dim))
    _require(k_pages.is_cuda and v_pages.is_cuda, "the page pool must live on the GPU")
    pool = _PagePool(k_pages.data_ptr(), v_pages.data_ptr(), k_pages.stride(0), k_pages.stride(1),
                     k_pages.stride(3), k_pages.stride(2), k_pages.shape[2], k_pages.shape[0])
    for t in tables:
        _out(t, 0, torch.int32, "a block table")
    tabs = (_PageTable * len(tables))(*[_PageTable(t.data_ptr(), t.numel()) for t in tables])
    pp, arr, n = _marshal(params, reqs)
    _require(len(tables) == n, "one block table per request is needed")
    _, ko, _ = compactor_layout(params, reqs)
    _out(kept_idx, ko[-1], torch.int32, "kept_idx")
    _out(kept_cnt, n * params.layers * params.kv_heads, torch.int32, "kept_cnt")
    _check(_lib.compactor_compact_paged(pp, arr, n, _ptr(kept_idx), _ptr(kept_cnt), C.byref(pool),
                                        tabs, 1 if in_place else 0, _stream(stream)))


def compactor_compress(params: Params, reqs: Sequence[Request], want_scores: bool = False,
                       scores=None, kept_idx=None, kept_cnt=None, k_packed=None, v_packed=None,
                       status=None, workspace=None, stream=None):
    """Fused score -> select -> compact.  -> dict of the output tensors."""
    so, ko, _ = compactor_layout(params, reqs)
    dev = _device(reqs)
    nh = len(reqs) * params.layers * params.kv_heads
    if scores is None and want_scores:
        scores = torch.empty(so[-1], dtype=torch.float32, device=dev)
    if kept_idx is None:
        kept_idx = torch.empty(ko[-1], dtype=torch.int32, device=dev)
    if kept_cnt is None:
        kept_cnt = torch.empty(nh, dtype=torch.int32, device=dev)
    if k_packed is None:
        k_packed = torch.empty(ko[-1], params.head_dim, dtype=torch.bfloat16, device=dev)
    if v_packed is None:
        v_packed = torch.empty(ko[-1], params.head_dim, dtype=torch.bfloat16, device=dev)
    if status is None:
        status = torch.empty(nh, dtype=torch.int32, device=dev)
    workspace = _workspace(params, reqs, workspace, stream)
    pp, arr, n = _marshal(params, reqs)
    _out(scores, so[-1], torch.float32, "scores")
    _out(kept_idx, ko[-1], torch.int32, "kept_idx")
    _out(kept_cnt, nh, torch.int32, "kept_cnt")
    _out(k_packed, ko[-1] * params.head_dim, torch.bfloat16, "k_packed")
    _out(v_packed, ko[-1] * params.head_dim, torch.bfloat16, "v_packed")
    _out(status, nh, torch.int32, "status")
    _out(workspace, 0, torch.uint8, "workspace")
    _check(_lib.compactor_compress(pp, arr, n, _ptr(scores), _ptr(kept_idx), _ptr(kept_cnt),
                                   _ptr(k_packed), _ptr(v_packed), _ptr(status), _ptr(workspace),
                                   workspace.numel(), _stream(stream)))
    return {"scores": scores, "kept_idx": kept_idx, "kept_cnt": kept_cnt, "k_packed": k_packed,
            "v_packed": v_packed, "status": status, "workspace": workspace}


STATIC_SCRATCH_BYTES = 64 << 20      # COMPACTOR_STATIC_SCRATCH_BYTES of the header


def compactor_compress_static(params: Params, reqs: Sequence[Request], scores, kept_idx, kept_cnt,
                              k_packed, v_packed, status, stream=None):
    """compactor_compress on the library's own static scratch: every buffer is the caller's (none
    is allocated here, `scores` may be None) and no workspace is passed."""
    so, ko, _ = compactor_layout(params, reqs)
    nh = len(reqs) * params.layers * params.kv_heads
    pp, arr, n = _marshal(params, reqs)
    _out(scores, so[-1], torch.float32, "scores")
    for t, name in ((kept_idx, "kept_idx"), (kept_cnt, "kept_cnt"), (k_packed, "k_packed"),
                    (v_packed, "v_packed"), (status, "status")):
        _require(t is not None, "%s must be supplied" % name)
    _out(kept_idx, ko[-1], torch.int32, "kept_idx")
    _out(kept_cnt, nh, torch.int32, "kept_cnt")
    _out(k_packed, ko[-1] * params.head_dim, torch.bfloat16, "k_packed")
    _out(v_packed, ko[-1] * params.head_dim, torch.bfloat16, "v_packed")
    _out(status, nh, torch.int32, "status")
    _check(_lib.compactor_compress_static(pp, arr, n, _ptr(scores), _ptr(kept_idx), _ptr(kept_cnt),
                                          _ptr(k_packed), _ptr(v_packed), _ptr(status),
                                          _stream(stream)))


@dataclass
class AttnParams:
    layers: int
    kv_heads: int
    q_heads: int
    head_dim: int = 128
    chunk: int = 256
    pool: int = 7
    scale: float = 0.0          # 0 = 1/sqrt(head_dim)

    def c(self) -> _AttnParams:
        return _AttnParams(self.layers, self.kv_heads, self.q_heads, self.head_dim, self.chunk,
                           self.pool, self.scale)


@dataclass
class AttnRequest:
    q: torch.Tensor             # bf16 [L, Hq, n, d]
    k: torch.Tensor             # bf16 [L, H, n, d]

    def c(self, params: Optional["AttnParams"] = None) -> _AttnRequest:
        q, k = self.q, self.k
        _require(q.dtype == torch.bfloat16 and k.dtype == torch.bfloat16, "q and k must be bfloat16")
        _require(q.dim() == 4 and k.dim() == 4 and q.stride(3) == 1 and k.stride(3) == 1,
                 "q and k must be [L, heads, n, d] with d contiguous")
        _require(q.shape[2] == k.shape[2], "q and k must cover the same tokens")
        if params is not None:
            _require(tuple(q.shape[:2]) == (params.layers, params.q_heads) and
                     tuple(k.shape[:2]) == (params.layers, params.kv_heads) and
                     q.shape[3] == params.head_dim and k.shape[3] == params.head_dim,
                     "q %s / k %s do not match the parameters [%d, %d | %d, n, %d]"
                     % (tuple(q.shape), tuple(k.shape), params.layers, params.q_heads,
                        params.kv_heads, params.head_dim))
        _require(q.is_cuda and k.is_cuda, "q and k must live on the GPU")
        return _AttnRequest(q.data_ptr(), k.data_ptr(), q.stride(0), q.stride(1), q.stride(2),
                            k.stride(0), k.stride(1), k.stride(2), k.shape[2])


def compactor_attention_workspace_size(params: AttnParams, reqs: Sequence[AttnRequest]) -> int:
    arr = (_AttnRequest * len(reqs))(*[r.c(params) for r in reqs])
    out = C.c_size_t(0)
    _check(_lib.compactor_attention_workspace_size(C.byref(params.c()), arr, len(reqs), C.byref(out)))
    return int(out.value)


def compactor_attention_scores(params: AttnParams, reqs: Sequence[AttnRequest], attn=None,
                               workspace=None, stream=None):
    """-> attn fp32 [sum_b L*H*n_b]; request b starts at the prefix sum of L*H*n_b."""
    dev = reqs[0].k.device
    total = sum(params.layers * params.kv_heads * r.k.shape[2] for r in reqs)
    if attn is None:
        attn = torch.empty(total, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(256, compactor_attention_workspace_size(params, reqs)),
                                dtype=torch.uint8, device=dev)
        if stream is not None:
            workspace.record_stream(stream)
    arr = (_AttnRequest * len(reqs))(*[r.c(params) for r in reqs])
    _out(attn, total, torch.float32, "attn")
    _out(workspace, 0, torch.uint8, "workspace")
    _check(_lib.compactor_attention_scores(C.byref(params.c()), arr, len(reqs), _ptr(attn),
                                           _ptr(workspace), workspace.numel(), _stream(stream)))
    return attn
