"""Thin ctypes binding of libkitty.so: argument marshalling only, every step runs in the HIP kernels.

Names follow include/kitty.h.  Tensors are torch tensors on the GPU (torch is used for device
memory and streams only); bf16 tensors are passed as they are.  The binding fails loudly when the
library has not been built: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# KITTY_LIB selects another build of the same library (A/B timing of kernel variants)
LIB_PATH = os.environ.get("KITTY_LIB") or os.path.join(_HERE, "libkitty.so")

KITTY_OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = -1, -2, -3, -4

EXPORTS = (
    "kitty_page_bytes", "kitty_page_payload_bytes", "kitty_decode_plan", "kitty_decode_workspace_bytes",
    "kitty_quantize_pages", "kitty_project_quantize_pages", "kitty_append_token", "kitty_decode_attention", "kitty_decode_split",
    "kitty_decode_merge", "kitty_decode_step", "kitty_decode_attention_static", "kitty_strerror",
)
STATIC_WORKSPACE_BYTES = 4 * 1024 * 1024


class KittyLayout(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("head_dim", "page_size", "v_group", "n_boost", "residual_window",
                                         "n_q_heads", "n_kv_heads", "rank_metric", "sink_tokens", "v_local", "v_bits")]


class KittyCache(C.Structure):
    _fields_ = [("page_pool", C.c_void_p), ("page_table", C.c_void_p), ("n_pages", C.c_void_p),
                ("resid_k", C.c_void_p), ("resid_v", C.c_void_p), ("n_resid", C.c_void_p),
                ("sink_k", C.c_void_p), ("sink_v", C.c_void_p), ("n_sink", C.c_void_p), ("seq_order", C.c_void_p),
                ("batch", C.c_int32), ("max_pages", C.c_int32), ("n_pool_pages", C.c_int32)]


class KittyError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().kitty_strerror(code).decode()} ({code})")


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if libkitty.so is missing (build it with paper_2511_18643_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: run `python -m paper_2511_18643_amd.build` first")
        L = C.CDLL(LIB_PATH)
        LP, CP = C.POINTER(KittyLayout), C.POINTER(KittyCache)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.kitty_page_bytes.restype = sz
        L.kitty_page_bytes.argtypes = [LP]
        L.kitty_page_payload_bytes.restype = sz
        L.kitty_page_payload_bytes.argtypes = [LP]
        L.kitty_decode_plan.restype = C.c_int
        L.kitty_decode_plan.argtypes = [LP, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.kitty_decode_workspace_bytes.restype = sz
        L.kitty_decode_workspace_bytes.argtypes = [LP, i32, i32, i32]
        L.kitty_quantize_pages.restype = C.c_int
        L.kitty_quantize_pages.argtypes = [LP, vp, vp, i64, i64, i64, vp, vp, i32, vp, i32, vp]
        L.kitty_project_quantize_pages.restype = C.c_int
        L.kitty_project_quantize_pages.argtypes = [LP, vp, i64, i32, vp, vp, vp, vp, i32, vp, i32, vp]
        L.kitty_append_token.restype = C.c_int
        L.kitty_append_token.argtypes = [LP, CP, vp, vp, vp, vp]
        L.kitty_decode_attention.restype = C.c_int
        L.kitty_decode_attention.argtypes = [LP, CP, vp, vp, C.c_float, i32, i32, vp, sz, vp]
        L.kitty_decode_split.restype = C.c_int
        L.kitty_decode_split.argtypes = [LP, CP, vp, C.c_float, i32, vp, sz, vp]
        L.kitty_decode_merge.restype = C.c_int
        L.kitty_decode_merge.argtypes = [LP, CP, vp, i32, i32, vp, sz, vp]
        L.kitty_decode_step.restype = C.c_int
        L.kitty_decode_step.argtypes = [LP, CP, vp, vp, vp, vp, vp, C.c_float, i32, i32, vp, sz, vp]
        L.kitty_decode_attention_static.restype = C.c_int
        L.kitty_decode_attention_static.argtypes = [LP, CP, vp, vp, C.c_float, i32, i32, vp]
        L.kitty_strerror.restype = C.c_char_p
        L.kitty_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def make_layout(n_q_heads: int, n_kv_heads: int, n_boost: int = 16, residual_window: int = 128,
                rank_metric: int = 0, head_dim: int = 128, page_size: int = 128, v_group: int = 128,
                sink_tokens: int = 0, v_local: int = 0, v_bits: int = 2) -> KittyLayout:
    return KittyLayout(head_dim, page_size, v_group, n_boost, residual_window, n_q_heads, n_kv_heads, rank_metric,
                       sink_tokens, v_local, v_bits)


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != KITTY_OK:
        raise KittyError(rc, where)


def _out_dtype(layout: KittyLayout, cache: "Cache", out, where: str) -> int:
    """out_dtype code of an output tensor; anything but contiguous bf16 / fp32 of the full shape is refused here,
    because the kernels write batch * n_q_heads * D elements of the announced width."""
    if out.dtype == torch.bfloat16:
        code = 0
    elif out.dtype == torch.float32:
        code = 1
    else:
        raise TypeError(f"{where}: out must be a bfloat16 or float32 tensor, not {out.dtype}")
    if out.numel() != cache.batch * layout.n_q_heads * layout.head_dim or not out.is_contiguous():
        raise ValueError(f"{where}: out must be a contiguous [batch][n_q_heads][head_dim] tensor")
    return code


def kitty_page_bytes(layout: KittyLayout) -> int:
    return int(lib().kitty_page_bytes(C.byref(layout)))


def kitty_page_payload_bytes(layout: KittyLayout) -> int:
    return int(lib().kitty_page_payload_bytes(C.byref(layout)))


def kitty_decode_plan(layout: KittyLayout, batch: int, max_pages: int, n_splits: int = 0):
    ns, pps = C.c_int32(0), C.c_int32(0)
    _check(lib().kitty_decode_plan(C.byref(layout), batch, max_pages, n_splits, C.byref(ns), C.byref(pps)),
           "kitty_decode_plan")
    return ns.value, pps.value


def kitty_decode_workspace_bytes(layout: KittyLayout, batch: int, max_pages: int, n_splits: int = 0) -> int:
    return int(lib().kitty_decode_workspace_bytes(C.byref(layout), batch, max_pages, n_splits))


class Cache:
    """Device buffers of one batch's cache plus the C struct that points at them."""

    def __init__(self, layout: KittyLayout, batch: int, max_pages: int, n_pool_pages: int, device="cuda"):
        self.layout, self.batch, self.max_pages, self.n_pool_pages = layout, batch, max_pages, n_pool_pages
        rb = kitty_page_bytes(layout)
        if rb == 0:
            raise KittyError(ERR_UNSUPPORTED, "kitty_page_bytes")
        self.record_bytes = rb
        self.seq_order = None      # optional int32 [batch] permutation: dispatch order of the decode kernels
        hkv, r = layout.n_kv_heads, layout.residual_window
        self.pool = torch.zeros((max(n_pool_pages, 1), hkv, rb), dtype=torch.uint8, device=device)
        self.page_table = torch.zeros((batch, max(max_pages, 1)), dtype=torch.int32, device=device)
        self.n_pages = torch.zeros((batch,), dtype=torch.int32, device=device)
        if r:
            self.resid_k = torch.zeros((batch, hkv, r, layout.head_dim), dtype=torch.bfloat16, device=device)
            halves = (2,) if layout.v_local else ()
            self.resid_v = torch.zeros((batch, hkv) + halves + (r, layout.head_dim), dtype=torch.bfloat16, device=device)
            self.n_resid = torch.zeros((batch,), dtype=torch.int32, device=device)
        else:
            self.resid_k = self.resid_v = self.n_resid = None
        if layout.sink_tokens:
            self.sink_k = torch.zeros((batch, hkv, layout.sink_tokens, layout.head_dim), dtype=torch.bfloat16, device=device)
            self.sink_v = torch.zeros_like(self.sink_k)
            self.n_sink = torch.zeros((batch,), dtype=torch.int32, device=device)
        else:
            self.sink_k = self.sink_v = self.n_sink = None

    def struct(self) -> KittyCache:
        return KittyCache(_ptr(self.pool), _ptr(self.page_table), _ptr(self.n_pages), _ptr(self.resid_k),
                          _ptr(self.resid_v), _ptr(self.n_resid), _ptr(self.sink_k), _ptr(self.sink_v),
                          _ptr(self.n_sink), _ptr(self.seq_order), self.batch, self.max_pages, self.n_pool_pages)


def kitty_quantize_pages(layout: KittyLayout, k_src, v_src, page_stride: int, head_stride: int, token_stride: int,
                         dst_page_ids, n_pages: int, page_pool, n_pool_pages: int, src_page_offsets=None,
                         stream=None) -> None:
    rc = lib().kitty_quantize_pages(C.byref(layout), _ptr(k_src), _ptr(v_src), page_stride, head_stride,
                                    token_stride, _ptr(src_page_offsets), _ptr(dst_page_ids), n_pages,
                                    _ptr(page_pool), n_pool_pages, _stream(stream))
    _check(rc, "kitty_quantize_pages")


def kitty_project_quantize_pages(layout: KittyLayout, x, x_token_stride: int, hidden: int, w_k, w_v,
                                 src_token_offsets, dst_page_ids, n_pages: int, page_pool, n_pool_pages: int,
                                 stream=None) -> None:
    rc = lib().kitty_project_quantize_pages(C.byref(layout), _ptr(x), x_token_stride, hidden, _ptr(w_k), _ptr(w_v),
                                            _ptr(src_token_offsets), _ptr(dst_page_ids), n_pages, _ptr(page_pool),
                                            n_pool_pages, _stream(stream))
    _check(rc, "kitty_project_quantize_pages")


def kitty_append_token(layout: KittyLayout, cache: Cache, k_new, v_new, fresh_page_ids, stream=None) -> None:
    cs = cache.struct()
    rc = lib().kitty_append_token(C.byref(layout), C.byref(cs), _ptr(k_new), _ptr(v_new), _ptr(fresh_page_ids),
                                  _stream(stream))
    _check(rc, "kitty_append_token")


def kitty_decode_attention(layout: KittyLayout, cache: Cache, q, out, sm_scale: float, workspace,
                           n_splits: int = 0, stream=None) -> None:
    """out: bf16 or fp32 tensor [batch][n_q_heads][D]; its dtype selects out_dtype."""
    cs = cache.struct()
    out_dtype = _out_dtype(layout, cache, out, "kitty_decode_attention")
    rc = lib().kitty_decode_attention(C.byref(layout), C.byref(cs), _ptr(q), _ptr(out), sm_scale, n_splits,
                                      out_dtype, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream))
    _check(rc, "kitty_decode_attention")


def kitty_decode_attention_static(layout: KittyLayout, cache: Cache, q, out, sm_scale: float, n_splits: int = 0,
                                  stream=None) -> None:
    """kitty_decode_attention with the library's own fixed workspace (no allocation, no workspace argument)."""
    cs = cache.struct()
    out_dtype = _out_dtype(layout, cache, out, "kitty_decode_attention_static")
    rc = lib().kitty_decode_attention_static(C.byref(layout), C.byref(cs), _ptr(q), _ptr(out), sm_scale, n_splits,
                                             out_dtype, _stream(stream))
    _check(rc, "kitty_decode_attention_static")


def kitty_decode_step(layout: KittyLayout, cache: Cache, k_new, v_new, fresh_page_ids, q, out, sm_scale: float,
                      workspace, n_splits: int = 0, stream=None) -> None:
    """kitty_append_token + kitty_decode_attention in one call (one launch when the plan has one range)."""
    cs = cache.struct()
    out_dtype = _out_dtype(layout, cache, out, "kitty_decode_step")
    rc = lib().kitty_decode_step(C.byref(layout), C.byref(cs), _ptr(k_new), _ptr(v_new), _ptr(fresh_page_ids),
                                 _ptr(q), _ptr(out), sm_scale, n_splits, out_dtype, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "kitty_decode_step")


def kitty_decode_split(layout: KittyLayout, cache: Cache, q, sm_scale: float, workspace, n_splits: int = 0,
                       stream=None) -> None:
    cs = cache.struct()
    rc = lib().kitty_decode_split(C.byref(layout), C.byref(cs), _ptr(q), sm_scale, n_splits, _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "kitty_decode_split")


def kitty_decode_merge(layout: KittyLayout, cache: Cache, out, workspace, n_splits: int = 0, stream=None) -> None:
    cs = cache.struct()
    out_dtype = _out_dtype(layout, cache, out, "kitty_decode_merge")
    rc = lib().kitty_decode_merge(C.byref(layout), C.byref(cs), _ptr(out), n_splits, out_dtype, _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "kitty_decode_merge")


def new_workspace(layout: KittyLayout, batch: int, max_pages: int, n_splits: int = 0, device="cuda"):
    n = kitty_decode_workspace_bytes(layout, batch, max_pages, n_splits)
    return torch.empty(((n + 3) // 4,), dtype=torch.float32, device=device)
