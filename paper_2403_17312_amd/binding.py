"""Thin ctypes binding of libswa_hip.so (the C ABI declared in include/swa.h).

Argument marshalling only: every step of the decode path runs in the HIP kernels
behind the C entry points.  PyTorch supplies device memory (tensors) and the
stream.  There is no fallback: if the library has not been built, or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libswa_hip.so")

SWA_F32, SWA_F16, SWA_BF16 = 0, 1, 2
SWA_OK = 0
SWA_ERR_NULL, SWA_ERR_BAD_SHAPE, SWA_ERR_UNSUPPORTED_D, SWA_ERR_UNSUPPORTED_DTYPE = -1, -2, -3, -4
SWA_ERR_BAD_SPARSITY, SWA_ERR_CAPACITY, SWA_ERR_HIP, SWA_ERR_ALIGNMENT = -5, -6, -7, -8
SWA_ERR_HOST_STORE_FULL, SWA_ERR_BAD_REQUEST = -9, -10
SWA_MAX_CAP = 16384
SWA_MAX_PREFILL_ROWS = 128
SWA_W_EVEN_SPLIT = -1
SWA_FUSE_COMPACTION = 1
SWA_MAX_FUSED_SLOTS = 9216
SWA_UNORDERED = 2
SWA_HEAD_SHARED = 4
SWA_MAX_UNORDERED_SLOTS = 7168
SWA_KV_INT8 = 8
SWA_SPLIT_ROWS = 16
SWA_MAX_WINDOW_ROWS = 64
SWA_STATIC_SCRATCH_BYTES = 8 << 20

DTYPE_CODE = {torch.float32: SWA_F32, torch.float16: SWA_F16, torch.bfloat16: SWA_BF16}
EXPORTS = ["swa_strerror", "swa_workspace_bytes", "swa_workspace_init", "swa_check_status",
           "swa_budget", "swa_prefill_scores", "swa_decode_step", "swa_compact_kv", "swa_quantize_kv",
           "swa_decode_step_q8", "swa_prefill_rows", "swa_decode_step_window", "swa_prefill_attention", "swa_probe_stream_read",
           "swa_prepare", "swa_decode_step_static", "swa_decode_step_window_q8", "swa_offload_evicted", "swa_reload_tokens"]


class SwaParams(ctypes.Structure):
    _fields_ = [("b", ctypes.c_int32), ("h", ctypes.c_int32), ("d", ctypes.c_int32),
                ("cap", ctypes.c_int32), ("w", ctypes.c_int32), ("sparsity_bp", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("len_bound", ctypes.c_int32), ("flags", ctypes.c_int32)]


class SwaHostStore(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("score", ctypes.c_void_p),
                ("pos", ctypes.c_void_p), ("len", ctypes.c_void_p), ("host_cap", ctypes.c_int32)]


class SwaError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


_lib = None


def lib():
    """Loads libswa_hip.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2403_17312_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        pp = ctypes.POINTER(SwaParams)
        L.swa_strerror.restype = ctypes.c_char_p
        L.swa_strerror.argtypes = [ctypes.c_int]
        L.swa_workspace_bytes.restype = ctypes.c_size_t
        L.swa_workspace_bytes.argtypes = [pp]
        L.swa_workspace_init.restype = ctypes.c_int
        L.swa_workspace_init.argtypes = [pp, vp, vp]
        L.swa_check_status.restype = ctypes.c_int
        L.swa_check_status.argtypes = [pp, vp, vp, ctypes.POINTER(ctypes.c_int32)]
        L.swa_budget.restype = ctypes.c_int
        L.swa_budget.argtypes = [ctypes.c_int32] * 4 + [ctypes.POINTER(ctypes.c_int32)] * 3
        L.swa_prefill_scores.restype = ctypes.c_int
        L.swa_prefill_scores.argtypes = [pp, vp, ctypes.c_int32, vp, i32p, vp, vp, vp]
        L.swa_decode_step.restype = ctypes.c_int
        L.swa_decode_step.argtypes = [pp] + [vp] * 15
        L.swa_decode_step_static.restype = ctypes.c_int
        L.swa_decode_step_static.argtypes = [pp] + [vp] * 14
        L.swa_prepare.restype = ctypes.c_int
        L.swa_prepare.argtypes = []
        L.swa_compact_kv.restype = ctypes.c_int
        L.swa_compact_kv.argtypes = [pp] + [vp] * 9
        L.swa_quantize_kv.restype = ctypes.c_int
        L.swa_quantize_kv.argtypes = [pp] + [vp] * 7
        L.swa_decode_step_q8.restype = ctypes.c_int
        L.swa_decode_step_q8.argtypes = [pp] + [vp] * 16
        L.swa_prefill_rows.restype = ctypes.c_int
        L.swa_prefill_rows.argtypes = [pp, vp, ctypes.c_int32, vp, i32p, vp, vp, vp]
        L.swa_decode_step_window.restype = ctypes.c_int
        L.swa_decode_step_window.argtypes = [pp] + [vp] * 6 + [ctypes.c_int32] * 2 + [vp] * 10
        L.swa_decode_step_window_q8.restype = ctypes.c_int
        L.swa_decode_step_window_q8.argtypes = [pp] + [vp] * 7 + [ctypes.c_int32] * 2 + [vp] * 10
        L.swa_offload_evicted.restype = ctypes.c_int
        L.swa_offload_evicted.argtypes = [pp] + [vp] * 7 + [ctypes.POINTER(SwaHostStore), vp, vp]
        L.swa_reload_tokens.restype = ctypes.c_int
        L.swa_reload_tokens.argtypes = [pp, ctypes.POINTER(SwaHostStore), vp, vp, ctypes.c_int32] + [vp] * 8
        L.swa_prefill_attention.restype = ctypes.c_int
        L.swa_prefill_attention.argtypes = [pp, vp, vp, vp, i32p, vp, ctypes.c_int32, vp, vp, vp]
        L.swa_probe_stream_read.restype = ctypes.c_int
        L.swa_probe_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().swa_strerror(int(code)).decode()


def make_params(b: int, h: int, d: int, cap: int, w: int, sparsity_bp: int, dtype,
                scale: float = 0.0, len_bound: int = 0, flags: int = 0) -> SwaParams:
    code = DTYPE_CODE[dtype] if isinstance(dtype, torch.dtype) else int(dtype)
    return SwaParams(b, h, d, cap, w, sparsity_bp, code, scale, len_bound, flags)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to the SWA library must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(rc: int, what: str) -> None:
    if rc != SWA_OK:
        raise SwaError(rc, what)


def swa_workspace_bytes(params: SwaParams) -> int:
    return int(lib().swa_workspace_bytes(ctypes.byref(params)))


def swa_budget(n: int, m: int, w: int, sparsity_bp: int):
    keep, nl, ng = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().swa_budget(n, m, w, sparsity_bp, ctypes.byref(keep), ctypes.byref(nl),
                            ctypes.byref(ng)), "swa_budget")
    return keep.value, nl.value, ng.value


def swa_workspace_init(params: SwaParams, workspace: torch.Tensor, stream=None) -> None:
    _check(lib().swa_workspace_init(ctypes.byref(params), _ptr(workspace), _stream(stream)),
           "swa_workspace_init")


def swa_prepare() -> None:
    _check(lib().swa_prepare(), "swa_prepare")


def swa_decode_step_static(params: SwaParams, q, k_new, v_new, k_cache, v_cache, score, pos, cache_len,
                           seq_len, kept_idx, kept_cnt, out, probs_dbg, stream=None) -> None:
    _check(lib().swa_decode_step_static(ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new),
                                        _ptr(k_cache), _ptr(v_cache), _ptr(score), _ptr(pos),
                                        _ptr(cache_len), _ptr(seq_len), _ptr(kept_idx), _ptr(kept_cnt),
                                        _ptr(out), _ptr(probs_dbg), _stream(stream)),
           "swa_decode_step_static")


def swa_check_status(params: SwaParams, workspace: Optional[torch.Tensor], stream=None) -> int:
    st = ctypes.c_int32(0)
    _check(lib().swa_check_status(ctypes.byref(params), _ptr(workspace), _stream(stream),
                                  ctypes.byref(st)), "swa_check_status")
    return st.value


def swa_prefill_scores(params: SwaParams, q_tail, R: int, k_cache, cache_len, score, workspace,
                       stream=None) -> None:
    _check(lib().swa_prefill_scores(ctypes.byref(params), _ptr(q_tail), int(R), _ptr(k_cache),
                                    _ptr(cache_len), _ptr(score), _ptr(workspace),
                                    _stream(stream)), "swa_prefill_scores")


def swa_decode_step(params: SwaParams, q, k_new, v_new, k_cache, v_cache, score, pos, cache_len,
                    seq_len, kept_idx, kept_cnt, out, probs_dbg, workspace, stream=None) -> None:
    _check(lib().swa_decode_step(ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new),
                                 _ptr(k_cache), _ptr(v_cache), _ptr(score), _ptr(pos),
                                 _ptr(cache_len), _ptr(seq_len), _ptr(kept_idx), _ptr(kept_cnt),
                                 _ptr(out), _ptr(probs_dbg), _ptr(workspace), _stream(stream)),
           "swa_decode_step")


def swa_quantize_kv(params: SwaParams, k_cache, v_cache, cache_len, k_codes, v_codes, qparams,
                    stream=None) -> None:
    _check(lib().swa_quantize_kv(ctypes.byref(params), _ptr(k_cache), _ptr(v_cache), _ptr(cache_len),
                                 _ptr(k_codes), _ptr(v_codes), _ptr(qparams), _stream(stream)),
           "swa_quantize_kv")


def swa_decode_step_q8(params: SwaParams, q, k_new, v_new, k_codes, v_codes, qparams, score, pos,
                       cache_len, seq_len, kept_idx, kept_cnt, out, probs_dbg, workspace,
                       stream=None) -> None:
    _check(lib().swa_decode_step_q8(ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new),
                                    _ptr(k_codes), _ptr(v_codes), _ptr(qparams), _ptr(score),
                                    _ptr(pos), _ptr(cache_len), _ptr(seq_len), _ptr(kept_idx),
                                    _ptr(kept_cnt), _ptr(out), _ptr(probs_dbg), _ptr(workspace),
                                    _stream(stream)), "swa_decode_step_q8")


def swa_prefill_rows(params: SwaParams, q_tail, R: int, k_cache, cache_len, ring, workspace,
                     stream=None) -> None:
    _check(lib().swa_prefill_rows(ctypes.byref(params), _ptr(q_tail), int(R), _ptr(k_cache),
                                  _ptr(cache_len), _ptr(ring), _ptr(workspace), _stream(stream)),
           "swa_prefill_rows")


def swa_decode_step_window(params: SwaParams, q, k_new, v_new, k_cache, v_cache, ring, R: int,
                           ring_row: int, score, pos, cache_len, seq_len, kept_idx, kept_cnt, out,
                           probs_dbg, workspace, stream=None) -> None:
    _check(lib().swa_decode_step_window(ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new),
                                        _ptr(k_cache), _ptr(v_cache), _ptr(ring), int(R),
                                        int(ring_row), _ptr(score), _ptr(pos), _ptr(cache_len),
                                        _ptr(seq_len), _ptr(kept_idx), _ptr(kept_cnt), _ptr(out),
                                        _ptr(probs_dbg), _ptr(workspace), _stream(stream)),
           "swa_decode_step_window")


def swa_decode_step_window_q8(params: SwaParams, q, k_new, v_new, k_codes, v_codes, qparams, ring, R: int,
                              ring_row: int, score, pos, cache_len, seq_len, kept_idx, kept_cnt, out,
                              probs_dbg, workspace, stream=None) -> None:
    _check(lib().swa_decode_step_window_q8(ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new),
                                           _ptr(k_codes), _ptr(v_codes), _ptr(qparams), _ptr(ring), int(R),
                                           int(ring_row), _ptr(score), _ptr(pos), _ptr(cache_len),
                                           _ptr(seq_len), _ptr(kept_idx), _ptr(kept_cnt), _ptr(out),
                                           _ptr(probs_dbg), _ptr(workspace), _stream(stream)),
           "swa_decode_step_window_q8")


def swa_prefill_attention(params: SwaParams, q, k_cache, v_cache, cache_len, out, R: int, score,
                          workspace, stream=None) -> None:
    _check(lib().swa_prefill_attention(ctypes.byref(params), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(cache_len), _ptr(out), int(R), _ptr(score),
                                       _ptr(workspace), _stream(stream)), "swa_prefill_attention")


class HostStore:
    """Pinned host tensors of one layer's offload store plus the per-pair counters on the device
    (allocation plumbing only; the copies run in swa_offload_evicted / swa_reload_tokens)."""

    def __init__(self, params: SwaParams, host_cap: int, device="cuda"):
        b, h, d = params.b, params.h, params.d
        dt = torch.uint8 if params.flags & SWA_KV_INT8 else {v: k for k, v in DTYPE_CODE.items()}[params.dtype]
        self.k = torch.zeros((b, h, host_cap, d), dtype=dt, pin_memory=True)
        self.v = torch.zeros((b, h, host_cap, d), dtype=dt, pin_memory=True)
        self.score = torch.zeros((b, h, host_cap), dtype=torch.float32, pin_memory=True)
        self.pos = torch.full((b, h, host_cap), -1, dtype=torch.int32, pin_memory=True)
        self.len = torch.zeros((b, h), dtype=torch.int32, device=device)
        self.host_cap = host_cap
        self.c = SwaHostStore(self.k.data_ptr(), self.v.data_ptr(), self.score.data_ptr(), self.pos.data_ptr(),
                              self.len.data_ptr(), host_cap)


def swa_offload_evicted(params: SwaParams, k_cache, v_cache, score, pos, kept_idx, kept_cnt, cache_len,
                        store: HostStore, workspace, stream=None) -> None:
    _check(lib().swa_offload_evicted(ctypes.byref(params), _ptr(k_cache), _ptr(v_cache), _ptr(score), _ptr(pos),
                                     _ptr(kept_idx), _ptr(kept_cnt), _ptr(cache_len), ctypes.byref(store.c),
                                     _ptr(workspace), _stream(stream)), "swa_offload_evicted")


def swa_reload_tokens(params: SwaParams, store: HostStore, req_idx, req_cnt, max_req: int, k_cache, v_cache,
                      score, pos, cache_len, new_len, workspace, stream=None) -> None:
    _check(lib().swa_reload_tokens(ctypes.byref(params), ctypes.byref(store.c), _ptr(req_idx), _ptr(req_cnt),
                                   int(max_req), _ptr(k_cache), _ptr(v_cache), _ptr(score), _ptr(pos),
                                   _ptr(cache_len), _ptr(new_len), _ptr(workspace), _stream(stream)),
           "swa_reload_tokens")


def swa_probe_stream_read(src, nbytes: int, sink, stream=None) -> None:
    _check(lib().swa_probe_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)),
           "swa_probe_stream_read")


def swa_compact_kv(params: SwaParams, k_cache, v_cache, score, pos, kept_idx, kept_cnt, cache_len,
                   workspace, stream=None) -> None:
    _check(lib().swa_compact_kv(ctypes.byref(params), _ptr(k_cache), _ptr(v_cache), _ptr(score),
                                _ptr(pos), _ptr(kept_idx), _ptr(kept_cnt), _ptr(cache_len),
                                _ptr(workspace), _stream(stream)), "swa_compact_kv")


class DecodeState:
    """Device tensors of one layer's SWA cache (allocation plumbing only)."""

    def __init__(self, params: SwaParams, device="cuda", debug_probs: bool = False):
        b, h, d, cap = params.b, params.h, params.d, params.cap
        dt = {v: k for k, v in DTYPE_CODE.items()}[params.dtype]
        self.params = params
        self.K = torch.zeros((b, h, cap, d), dtype=dt, device=device)
        self.V = torch.zeros((b, h, cap, d), dtype=dt, device=device)
        self.score = torch.zeros((b, h, cap), dtype=torch.float32, device=device)
        self.pos = torch.full((b, h, cap), -1, dtype=torch.int32, device=device)
        self.cache_len = torch.zeros((b,), dtype=torch.int32, device=device)
        self.seq_len = torch.zeros((b,), dtype=torch.int32, device=device)
        self.kept_idx = torch.full((b, h, cap), -1, dtype=torch.int32, device=device)
        self.kept_cnt = torch.zeros((b,), dtype=torch.int32, device=device)
        self.out = torch.zeros((b, h, d), dtype=dt, device=device)
        self.probs = (torch.zeros((b, h, cap), dtype=torch.float32, device=device)
                      if debug_probs else None)
        self.workspace = torch.zeros((swa_workspace_bytes(params),), dtype=torch.uint8,
                                     device=device)
        swa_workspace_init(params, self.workspace)
        self.qparams = None     # [4,b,h,d] float32 once the cache is compressed

    def quantize(self, stream=None) -> None:
        """Replaces the fp16 K, V tensors by their 8-bit codes (swa_quantize_kv) and switches the
        params to SWA_KV_INT8."""
        codesK, codesV = torch.zeros_like(self.K, dtype=torch.uint8), torch.zeros_like(self.V, dtype=torch.uint8)
        p = self.params
        self.qparams = torch.zeros((4, p.b, p.h, p.d), dtype=torch.float32, device=self.K.device)
        swa_quantize_kv(p, self.K, self.V, self.cache_len, codesK, codesV, self.qparams, stream)
        self.K, self.V = codesK, codesV
        p.flags |= SWA_KV_INT8

    def _decode(self, params, q, k_new, v_new, cache_len, kept_idx, kept_cnt, stream) -> None:
        if self.qparams is not None:
            swa_decode_step_q8(params, q, k_new, v_new, self.K, self.V, self.qparams, self.score,
                               self.pos, cache_len, self.seq_len, kept_idx, kept_cnt, self.out,
                               self.probs, self.workspace, stream)
        else:
            swa_decode_step(params, q, k_new, v_new, self.K, self.V, self.score, self.pos,
                            cache_len, self.seq_len, kept_idx, kept_cnt, self.out, self.probs,
                            self.workspace, stream)

    def decode_step(self, q, k_new, v_new, stream=None) -> None:
        self._decode(self.params, q, k_new, v_new, self.cache_len, self.kept_idx, self.kept_cnt, stream)

    def decode_compact_step(self, q, k_new, v_new, stream=None, want_idx: bool = True) -> None:
        """Fused call (params.flags must carry SWA_FUSE_COMPACTION): the new lengths come back in
        kept_cnt, so the two length tensors are swapped afterwards."""
        self._decode(self.params, q, k_new, v_new, self.cache_len,
                     self.kept_idx if want_idx else None, self.kept_cnt, stream)
        self.cache_len, self.kept_cnt = self.kept_cnt, self.cache_len

    def compact(self, stream=None) -> None:
        swa_compact_kv(self.params, self.K, self.V, self.score, self.pos, self.kept_idx,
                       self.kept_cnt, self.cache_len, self.workspace, stream)

    def prefill_scores(self, q_tail, stream=None) -> None:
        swa_prefill_scores(self.params, q_tail, q_tail.shape[2], self.K, self.cache_len, self.score,
                           self.workspace, stream)

    def check_status(self, stream=None) -> int:
        return swa_check_status(self.params, self.workspace, stream)
