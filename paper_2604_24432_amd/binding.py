"""Thin ctypes binding of libksa.so (include/ksa.h).  Argument marshalling only.

Every step of the hot path runs in the library's HIP kernels; this module never computes
attention itself and has no fallback: if libksa.so is missing or a call fails, it raises.
PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("KSA_LIB", os.path.join(_HERE, "libksa.so"))

KSA_FLAG_SUMMARY_SELF_ONLY = 1
KSA_TILE_FULL, KSA_TILE_MASKED = 0, 1
KSA_SPACE_TEXT, KSA_SPACE_SUMMARY = 0, 1


class KsaError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


class ksa_params(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_text", C.c_int32), ("chunk_len", C.c_int32),
                ("n_summary", C.c_int32), ("compress_ratio", C.c_int32), ("window_chunks", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("softmax_scale", C.c_float), ("flags", C.c_uint32)]


def make_params(batch, n_text, chunk_len, n_summary, window_chunks, n_q_heads, n_kv_heads, head_dim,
                softmax_scale=0.0, flags=0, compress_ratio=None) -> ksa_params:
    if compress_ratio is None:
        compress_ratio = chunk_len // n_summary if n_summary else 0
    return ksa_params(batch, n_text, chunk_len, n_summary, compress_ratio, window_chunks, n_q_heads,
                      n_kv_heads, head_dim, softmax_scale, flags)


_lib = None


def lib():
    """Load libksa.so; raises if it has not been built (python -m paper_2604_24432_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_24432_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32p, i64p, u8p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
    pp = C.POINTER(ksa_params)
    sig = {
        "ksa_build_layout": (C.c_int, [pp, C.POINTER(vp)]),
        "ksa_layout_destroy": (None, [vp]),
        "ksa_layout_upload": (C.c_int, [vp]),
        "ksa_augmented_rows": (C.c_int, [pp, C.c_int64, i64p]),
        "ksa_layout_dims": (C.c_int, [vp, i64p, i32p, i32p, i32p, i32p]),
        "ksa_layout_index_maps": (C.c_int, [vp, vp, vp, vp, vp, vp]),
        "ksa_layout_row_ranges": (C.c_int, [vp, C.c_int64, i32p]),
        "ksa_layout_mask_row": (C.c_int, [vp, C.c_int64, vp]),
        "ksa_layout_tile_pairs": (C.c_int, [vp, i64p, vp, vp, vp, vp, vp, vp, vp]),
        "ksa_layout_launch_order": (C.c_int, [vp, i64p, vp, vp, vp, vp]),
        "ksa_prefill_workspace_bytes": (C.c_size_t, [vp]),
        "ksa_prefill_fwd": (C.c_int, [vp, vp, vp, vp, vp, vp, i64p, i64p, i64p, vp, C.c_size_t, vp]),
        "ksa_prefill_relayout_v": (C.c_int, [vp, vp, i64p, vp, C.c_size_t, vp]),
        "ksa_prefill_bwd_workspace_bytes": (C.c_size_t, [vp]),
        "ksa_prefill_bwd": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64p, i64p, i64p, i64p, i64p, vp,
                                      C.c_size_t, vp]),
        "ksa_cache_geometry": (C.c_int, [pp, i32p, i32p]),
        "ksa_cache_text_row": (C.c_int, [pp, C.c_int64, i32p]),
        "ksa_cache_summary_row": (C.c_int, [pp, C.c_int64, i32p]),
        "ksa_decode_ranges": (C.c_int, [pp, C.c_int64, i32p]),
        "ksa_decode_workspace_bytes": (C.c_size_t, [pp, C.c_int32]),
        "ksa_decode_fwd": (C.c_int, [pp, vp, vp, vp, vp, vp, vp, i64p, vp, C.c_size_t, C.c_int32, vp]),
        "ksa_decode_fwd_static": (C.c_int, [pp, vp, vp, vp, vp, vp, vp, i64p, C.c_int32, vp]),
        "ksa_decode_summary_ranges": (C.c_int, [pp, C.c_int64, i32p]),
        "ksa_decode_summary_fwd": (C.c_int, [pp, vp, vp, vp, vp, vp, vp, i64p, vp, C.c_size_t, C.c_int32, vp]),
        "ksa_cache_from_prefill": (C.c_int, [pp, C.c_int64, vp, vp, i64p, vp, vp, i64p, vp]),
        "ksa_cache_append": (C.c_int, [pp, C.c_int32, vp, vp, vp, vp, vp, i64p, vp]),
        "ksa_status_string": (C.c_char_p, [C.c_int]),
        "ksa_build_info": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)   # AttributeError if the library lacks a declared symbol
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


EXPORTED_SYMBOLS = ("ksa_augmented_rows", "ksa_build_layout", "ksa_layout_destroy", "ksa_layout_upload", "ksa_layout_dims",
                    "ksa_layout_index_maps", "ksa_layout_row_ranges", "ksa_layout_mask_row",
                    "ksa_layout_tile_pairs", "ksa_layout_launch_order", "ksa_prefill_workspace_bytes", "ksa_prefill_fwd", "ksa_prefill_relayout_v",
                    "ksa_prefill_bwd_workspace_bytes", "ksa_prefill_bwd", "ksa_cache_geometry", "ksa_cache_text_row",
                    "ksa_cache_summary_row", "ksa_decode_ranges", "ksa_decode_workspace_bytes",
                    "ksa_decode_fwd", "ksa_decode_fwd_static", "ksa_decode_summary_ranges", "ksa_decode_summary_fwd", "ksa_cache_from_prefill",
                    "ksa_cache_append", "ksa_status_string", "ksa_build_info")


def status_string(status: int) -> str:
    return lib().ksa_status_string(status).decode()


def build_info() -> str:
    return lib().ksa_build_info().decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise KsaError(rc, what)


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Layout:
    """Owner of a ksa_layout* (freed on garbage collection)."""

    def __init__(self, params: ksa_params):
        self.params = params
        h = C.c_void_p()
        _check(lib().ksa_build_layout(C.byref(params), C.byref(h)), "ksa_build_layout")
        self._h = h
        L, J, qt, kt, hs = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().ksa_layout_dims(h, C.byref(L), C.byref(J), C.byref(qt), C.byref(kt), C.byref(hs)),
               "ksa_layout_dims")
        self.aug_len, self.n_chunks, self.q_tile_rows, self.k_tile_rows = L.value, J.value, qt.value, kt.value
        self.heads_per_workgroup = hs.value

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            lib().ksa_layout_destroy(h)

    @property
    def handle(self):
        return self._h

    def upload(self):
        _check(lib().ksa_layout_upload(self._h), "ksa_layout_upload")

    def index_maps(self):
        p = self.params
        out = dict(aug_chunk=np.zeros(self.aug_len, np.int32), aug_is_summary=np.zeros(self.aug_len, np.uint8),
                   position_ids=np.zeros(self.aug_len, np.int32), text_to_aug=np.zeros(p.n_text, np.int32),
                   summary_to_aug=np.zeros(self.n_chunks * p.n_summary, np.int32))
        _check(lib().ksa_layout_index_maps(self._h, *[_np_ptr(out[k]) for k in
               ("aug_chunk", "aug_is_summary", "position_ids", "text_to_aug", "summary_to_aug")]), "ksa_layout_index_maps")
        return out

    def row_ranges(self, aq: int) -> np.ndarray:
        out = (C.c_int32 * 4)()
        _check(lib().ksa_layout_row_ranges(self._h, aq, out), "ksa_layout_row_ranges")
        return np.array(out[:], np.int32)

    def mask_row(self, aq: int) -> np.ndarray:
        out = np.zeros(self.aug_len, np.uint8)
        _check(lib().ksa_layout_mask_row(self._h, aq, _np_ptr(out)), "ksa_layout_mask_row")
        return out

    def tile_pairs(self):
        n = C.c_int64()
        _check(lib().ksa_layout_tile_pairs(self._h, C.byref(n), None, None, None, None, None, None, None),
               "ksa_layout_tile_pairs")
        N = n.value
        out = dict(q_space=np.zeros(N, np.uint8), q_begin=np.zeros(N, np.int32), q_count=np.zeros(N, np.int32),
                   k_space=np.zeros(N, np.uint8), k_begin=np.zeros(N, np.int32), k_count=np.zeros(N, np.int32),
                   kind=np.zeros(N, np.uint8))
        _check(lib().ksa_layout_tile_pairs(self._h, C.byref(n), *[_np_ptr(out[k]) for k in
               ("q_space", "q_begin", "q_count", "k_space", "k_begin", "k_count", "kind")]), "ksa_layout_tile_pairs")
        return out


    def launch_order(self):
        n = C.c_int64()
        _check(lib().ksa_layout_launch_order(self._h, C.byref(n), None, None, None, None), "ksa_layout_launch_order")
        N = n.value
        out = dict(q_space=np.zeros(N, np.uint8), q_begin=np.zeros(N, np.int32), batch=np.zeros(N, np.int32),
                   q_head=np.zeros(N, np.int32))
        _check(lib().ksa_layout_launch_order(self._h, C.byref(n), *[_np_ptr(out[k]) for k in
               ("q_space", "q_begin", "batch", "q_head")]), "ksa_layout_launch_order")
        return out


def ksa_build_layout(params: ksa_params) -> Layout:
    return Layout(params)


# ---- torch-facing wrappers ------------------------------------------------------------------------

def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _strides3(t, dims):
    return (C.c_int64 * 3)(*[t.stride(d) for d in dims])


def _require(t, name, dtype, ndim):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA (HIP) tensor")
    if t.dtype != dtype or t.dim() != ndim or t.stride(-1) != 1:
        raise ValueError(f"{name}: expected {ndim}-d {dtype} with contiguous last dim, got {t.dtype} {tuple(t.shape)}")


def _same_strides(x, y) -> bool:
    """Strides agree wherever they matter (a dimension of size 1 may carry any stride)."""
    return all(sx == sy for n, sx, sy in zip(x.shape, x.stride(), y.stride()) if n > 1)


def prefill_workspace_bytes(layout: Layout) -> int:
    return int(lib().ksa_prefill_workspace_bytes(layout.handle))


def ksa_prefill_fwd(layout: Layout, q, k, v, o=None, lse=None, return_lse=True, workspace=None, stream=None):
    """q [B, L, Hq, d], k/v [B, L, Hkv, d] bf16 on the GPU -> o [B, L, Hq, d] bf16, lse [B, Hq, L] fp32.
    workspace: uint8 GPU tensor of at least prefill_workspace_bytes(layout) bytes (allocated here if omitted)."""
    import torch
    p = layout.params
    for t, name in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, name, torch.bfloat16, 4)
    if tuple(q.shape) != (p.batch, layout.aug_len, p.n_q_heads, p.head_dim):
        raise ValueError(f"q shape {tuple(q.shape)} does not match the layout")
    if tuple(k.shape) != (p.batch, layout.aug_len, p.n_kv_heads, p.head_dim) or k.shape != v.shape or not _same_strides(k, v):
        raise ValueError("k / v shape or strides do not match the layout")
    if o is None:
        o = torch.empty_like(q)
    _require(o, "o", torch.bfloat16, 4)
    if lse is None and return_lse:
        lse = torch.empty((p.batch, p.n_q_heads, layout.aug_len), dtype=torch.float32, device=q.device)
    lse_ptr = C.c_void_p(lse.data_ptr()) if lse is not None else None
    if workspace is None:
        workspace = torch.empty(prefill_workspace_bytes(layout), dtype=torch.uint8, device=q.device)
    if not workspace.is_cuda or workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 GPU tensor")
    rc = lib().ksa_prefill_fwd(layout.handle, C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
                               C.c_void_p(v.data_ptr()), C.c_void_p(o.data_ptr()), lse_ptr,
                               _strides3(q, (0, 1, 2)), _strides3(k, (0, 1, 2)), _strides3(o, (0, 1, 2)),
                               C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream_ptr(stream))
    _check(rc, "ksa_prefill_fwd")
    return o, lse


def ksa_prefill_relayout_v(layout: Layout, v, workspace, stream=None):
    """Only the first kernel of ksa_prefill_fwd (key-major copy of V into the workspace); for timing."""
    import torch
    _require(v, "v", torch.bfloat16, 4)
    rc = lib().ksa_prefill_relayout_v(layout.handle, C.c_void_p(v.data_ptr()), _strides3(v, (0, 1, 2)),
                                      C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream_ptr(stream))
    _check(rc, "ksa_prefill_relayout_v")


def prefill_bwd_workspace_bytes(layout: Layout) -> int:
    return int(lib().ksa_prefill_bwd_workspace_bytes(layout.handle))


def ksa_prefill_bwd(layout: Layout, q, k, v, o, lse, d_o, dq=None, dk=None, dv=None, workspace=None, stream=None):
    """Gradients of ksa_prefill_fwd: q, o, d_o [B, L, Hq, d], k/v [B, L, Hkv, d] bf16, lse [B, Hq, L] fp32 on the GPU
    -> dq like q, dk and dv like k.  o and d_o must share their strides."""
    import torch
    p = layout.params
    for t, name in ((q, "q"), (k, "k"), (v, "v"), (o, "o"), (d_o, "d_o")):
        _require(t, name, torch.bfloat16, 4)
    _require(lse, "lse", torch.float32, 3)
    if tuple(q.shape) != (p.batch, layout.aug_len, p.n_q_heads, p.head_dim) or o.shape != q.shape or d_o.shape != q.shape:
        raise ValueError(f"q / o / d_o shape {tuple(q.shape)} does not match the layout")
    if tuple(k.shape) != (p.batch, layout.aug_len, p.n_kv_heads, p.head_dim) or k.shape != v.shape or not _same_strides(k, v):
        raise ValueError("k / v shape or strides do not match the layout")
    if not _same_strides(o, d_o):
        raise ValueError("o and d_o must have the same strides")
    if tuple(lse.shape) != (p.batch, p.n_q_heads, layout.aug_len) or not lse.is_contiguous():
        raise ValueError("lse must be contiguous [B, Hq, L]")
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(dk) if dv is None else dv
    for t, name in ((dq, "dq"), (dk, "dk"), (dv, "dv")):
        _require(t, name, torch.bfloat16, 4)
    if dq.shape != q.shape or dk.shape != k.shape or dv.shape != k.shape or not _same_strides(dk, dv):
        raise ValueError("dq / dk / dv shape or strides do not match q / k / v")
    if workspace is None:
        workspace = torch.empty(prefill_bwd_workspace_bytes(layout), dtype=torch.uint8, device=q.device)
    if not workspace.is_cuda or workspace.dtype != torch.uint8 or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous uint8 GPU tensor")
    rc = lib().ksa_prefill_bwd(layout.handle, C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
                               C.c_void_p(v.data_ptr()), C.c_void_p(o.data_ptr()), C.c_void_p(lse.data_ptr()),
                               C.c_void_p(d_o.data_ptr()), C.c_void_p(dq.data_ptr()), C.c_void_p(dk.data_ptr()),
                               C.c_void_p(dv.data_ptr()), _strides3(q, (0, 1, 2)), _strides3(k, (0, 1, 2)),
                               _strides3(o, (0, 1, 2)), _strides3(dq, (0, 1, 2)), _strides3(dk, (0, 1, 2)),
                               C.c_void_p(workspace.data_ptr()), C.c_size_t(workspace.numel()), _stream_ptr(stream))
    _check(rc, "ksa_prefill_bwd")
    return dq, dk, dv


def augmented_rows(params: ksa_params, n_text: int) -> int:
    """Rows of the augmented sequence of n_text text tokens (from the library)."""
    rows = C.c_int64()
    _check(lib().ksa_augmented_rows(C.byref(params), n_text, C.byref(rows)), "ksa_augmented_rows")
    return rows.value


def cache_geometry(params: ksa_params) -> Tuple[int, int]:
    s, r = C.c_int32(), C.c_int32()
    _check(lib().ksa_cache_geometry(C.byref(params), C.byref(s), C.byref(r)), "ksa_cache_geometry")
    return s.value, r.value


def cache_text_row(params: ksa_params, i: int) -> int:
    r = C.c_int32()
    _check(lib().ksa_cache_text_row(C.byref(params), i, C.byref(r)), "ksa_cache_text_row")
    return r.value


def cache_summary_row(params: ksa_params, u: int) -> int:
    r = C.c_int32()
    _check(lib().ksa_cache_summary_row(C.byref(params), u, C.byref(r)), "ksa_cache_summary_row")
    return r.value


def ksa_decode_ranges(params: ksa_params, pos: int) -> np.ndarray:
    out = (C.c_int32 * 6)()
    _check(lib().ksa_decode_ranges(C.byref(params), pos, out), "ksa_decode_ranges")
    return np.array(out[:], np.int32)


def decode_workspace_bytes(params: ksa_params, n_splits: int = 0) -> int:
    return int(lib().ksa_decode_workspace_bytes(C.byref(params), n_splits))


def _decode(entry, params: ksa_params, q, k_cache, v_cache, pos, o, lse, return_lse, workspace, n_splits, stream):
    import torch
    _require(q, "q", torch.bfloat16, 3)
    _require(k_cache, "k_cache", torch.bfloat16, 4)
    _require(v_cache, "v_cache", torch.bfloat16, 4)
    _require(pos, "pos", torch.int32, 1)
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    s_cap, rows = cache_geometry(params)
    if tuple(k_cache.shape) != (params.batch, params.n_kv_heads, rows, params.head_dim) or \
            k_cache.shape != v_cache.shape or k_cache.stride() != v_cache.stride():
        raise ValueError(f"cache shape must be {(params.batch, params.n_kv_heads, rows, params.head_dim)}")
    if tuple(q.shape) != (params.batch, params.n_q_heads, params.head_dim) or pos.shape[0] != params.batch:
        raise ValueError("q / pos shape does not match params")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and return_lse:
        lse = torch.empty((params.batch, params.n_q_heads), dtype=torch.float32, device=q.device)
    need = decode_workspace_bytes(params, n_splits)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = getattr(lib(), entry)(C.byref(params), C.c_void_p(q.data_ptr()), C.c_void_p(k_cache.data_ptr()),
                               C.c_void_p(v_cache.data_ptr()), C.c_void_p(pos.data_ptr()), C.c_void_p(o.data_ptr()),
                               C.c_void_p(lse.data_ptr()) if lse is not None else None,
                               _strides3(k_cache, (0, 1, 2)), C.c_void_p(workspace.data_ptr()),
                               workspace.numel() * workspace.element_size(), n_splits, _stream_ptr(stream))
    _check(rc, entry)
    return o, lse


def ksa_decode_fwd(params: ksa_params, q, k_cache, v_cache, pos, o=None, lse=None, return_lse=True,
                   workspace=None, n_splits: int = 0, stream=None):
    """q [B, Hq, d] bf16; caches [B, Hkv, cache_rows, d] bf16; pos int32 [B] on the GPU (text indices)."""
    return _decode("ksa_decode_fwd", params, q, k_cache, v_cache, pos, o, lse, return_lse, workspace, n_splits, stream)


KSA_DECODE_STATIC_SCRATCH_BYTES = 8 << 20


def ksa_decode_fwd_static(params: ksa_params, q, k_cache, v_cache, pos, o, lse=None, n_splits: int = 0, stream=None):
    """ksa_decode_fwd with the spans' partial records in the library's static device array: the call allocates
    nothing, so o (and lse, if wanted) must be passed in.  Raises KsaError (scratch limit) for problems whose
    records exceed KSA_DECODE_STATIC_SCRATCH_BYTES."""
    import torch
    _require(q, "q", torch.bfloat16, 3)
    _require(o, "o", torch.bfloat16, 3)
    _require(pos, "pos", torch.int32, 1)
    _check_cache(params, k_cache, v_cache)
    if not q.is_contiguous() or not o.is_contiguous() or o.shape != q.shape:
        raise ValueError("q and o must be contiguous and of one shape")
    if tuple(q.shape) != (params.batch, params.n_q_heads, params.head_dim) or pos.shape[0] != params.batch:
        raise ValueError("q / pos shape does not match params")
    if lse is not None:
        _require(lse, "lse", torch.float32, 2)
        if tuple(lse.shape) != (params.batch, params.n_q_heads) or not lse.is_contiguous():
            raise ValueError("lse must be a contiguous [B, Hq] tensor")
    rc = lib().ksa_decode_fwd_static(C.byref(params), C.c_void_p(q.data_ptr()), C.c_void_p(k_cache.data_ptr()),
                                     C.c_void_p(v_cache.data_ptr()), C.c_void_p(pos.data_ptr()),
                                     C.c_void_p(o.data_ptr()), C.c_void_p(lse.data_ptr()) if lse is not None else None,
                                     _strides3(k_cache, (0, 1, 2)), n_splits, _stream_ptr(stream))
    _check(rc, "ksa_decode_fwd_static")
    return o, lse


def ksa_decode_summary_fwd(params: ksa_params, q, k_cache, v_cache, ordinal, o=None, lse=None, return_lse=True,
                           workspace=None, n_splits: int = 0, stream=None):
    """The summary-token step: as ksa_decode_fwd with ordinal int32 [B] = summary ordinals j*m + slot."""
    return _decode("ksa_decode_summary_fwd", params, q, k_cache, v_cache, ordinal, o, lse, return_lse, workspace,
                   n_splits, stream)


def ksa_decode_summary_ranges(params: ksa_params, ordinal: int) -> np.ndarray:
    out = (C.c_int32 * 4)()
    _check(lib().ksa_decode_summary_ranges(C.byref(params), ordinal, out), "ksa_decode_summary_ranges")
    return np.array(out[:], np.int32)


KSA_ROW_TEXT, KSA_ROW_SUMMARY = 0, 1


def _check_cache(params, k_cache, v_cache):
    import torch
    _require(k_cache, "k_cache", torch.bfloat16, 4)
    _require(v_cache, "v_cache", torch.bfloat16, 4)
    s_cap, rows = cache_geometry(params)
    if tuple(k_cache.shape) != (params.batch, params.n_kv_heads, rows, params.head_dim) or \
            k_cache.shape != v_cache.shape or k_cache.stride() != v_cache.stride():
        raise ValueError(f"cache shape must be {(params.batch, params.n_kv_heads, rows, params.head_dim)}")


def ksa_cache_from_prefill(params: ksa_params, n_prefill: int, k, v, k_cache, v_cache, stream=None):
    """k, v [B, L, Hkv, d] bf16: augmented sequence of n_prefill text tokens; fills the caches in place."""
    import torch
    _require(k, "k", torch.bfloat16, 4)
    _require(v, "v", torch.bfloat16, 4)
    _check_cache(params, k_cache, v_cache)
    L = augmented_rows(params, n_prefill)
    if tuple(k.shape) != (params.batch, L, params.n_kv_heads, params.head_dim) or k.shape != v.shape or \
            k.stride() != v.stride() or k.stride(3) != 1:
        raise ValueError(f"k / v shape must be {(params.batch, L, params.n_kv_heads, params.head_dim)}")
    rc = lib().ksa_cache_from_prefill(C.byref(params), n_prefill, C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr()),
                                      _strides3(k, (0, 1, 2)), C.c_void_p(k_cache.data_ptr()),
                                      C.c_void_p(v_cache.data_ptr()), _strides3(k_cache, (0, 1, 2)), _stream_ptr(stream))
    _check(rc, "ksa_cache_from_prefill")


def ksa_cache_append(params: ksa_params, kind: int, k_new, v_new, pos, k_cache, v_cache, stream=None):
    """k_new, v_new [B, Hkv, d] bf16 contiguous; pos int32 [B] on the GPU (text indices or summary ordinals)."""
    import torch
    _require(k_new, "k_new", torch.bfloat16, 3)
    _require(v_new, "v_new", torch.bfloat16, 3)
    _require(pos, "pos", torch.int32, 1)
    _check_cache(params, k_cache, v_cache)
    if tuple(k_new.shape) != (params.batch, params.n_kv_heads, params.head_dim) or k_new.shape != v_new.shape or \
            not k_new.is_contiguous() or not v_new.is_contiguous() or pos.shape[0] != params.batch:
        raise ValueError("k_new / v_new / pos shape does not match params")
    rc = lib().ksa_cache_append(C.byref(params), kind, C.c_void_p(k_new.data_ptr()), C.c_void_p(v_new.data_ptr()),
                                C.c_void_p(pos.data_ptr()), C.c_void_p(k_cache.data_ptr()),
                                C.c_void_p(v_cache.data_ptr()), _strides3(k_cache, (0, 1, 2)), _stream_ptr(stream))
    _check(rc, "ksa_cache_append")


def pack_cache(params: ksa_params, k_sum, v_sum, k_txt, v_txt, txt_base: int):
    """Place logical rows into a physical cache pair following ksa_cache_geometry (data movement only).

    k_sum/v_sum [B, Hkv, S, d]: summary ordinal u at index u.  k_txt/v_txt [B, Hkv, W, d]: slot t holds text
    index txt_base + t (slots whose text index is >= n_text are ignored).  Unwritten rows stay zero.
    """
    import torch
    s_cap, rows = cache_geometry(params)
    B, Hkv, S, d = k_sum.shape
    k_cache = torch.zeros((B, Hkv, rows, d), dtype=k_sum.dtype, device=k_sum.device)
    v_cache = torch.zeros_like(k_cache)
    n = min(S, s_cap)
    k_cache[:, :, :n] = k_sum[:, :, :n]
    v_cache[:, :, :n] = v_sum[:, :, :n]
    W = k_txt.shape[2]
    slots = [t for t in range(W) if txt_base + t < params.n_text]
    dst = torch.tensor([cache_text_row(params, txt_base + t) for t in slots], dtype=torch.long, device=k_sum.device)
    src = torch.tensor(slots, dtype=torch.long, device=k_sum.device)
    k_cache[:, :, dst] = k_txt[:, :, src]
    v_cache[:, :, dst] = v_txt[:, :, src]
    return k_cache, v_cache
