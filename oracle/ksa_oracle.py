"""numpy front end of the C oracle (oracle/ksa_oracle.c).

Test infrastructure only.  Argument marshalling and nothing else: all of the
method's arithmetic is in the C file, which cites the paper passages it follows.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

FLAG_SUMMARY_SELF_ONLY = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        i32, i64, u32, f64 = C.c_int32, C.c_int64, C.c_uint32, C.c_double
        p = C.c_void_p
        L.ksa_oracle_aug_len.restype = i64
        L.ksa_oracle_aug_len.argtypes = [i64, i32, i32]
        L.ksa_oracle_visible.restype = C.c_int
        L.ksa_oracle_visible.argtypes = [i64, i64, i32, i32, i32, u32]
        L.ksa_oracle_mask_row.restype = None
        L.ksa_oracle_mask_row.argtypes = [i64, i64, i32, i32, i32, u32, p]
        L.ksa_oracle_index_maps.restype = C.c_int
        L.ksa_oracle_index_maps.argtypes = [i64, i32, i32, p, p, p, p, p]
        L.ksa_oracle_prefill.restype = C.c_int
        L.ksa_oracle_prefill.argtypes = [p, p, p, i32, i64, i32, i32, i32, i32, i32, i32, f64, u32,
                                         p, i64, p, p]
        L.ksa_oracle_prefill_bwd.restype = C.c_int
        L.ksa_oracle_prefill_bwd.argtypes = [p, p, p, p, i32, i64, i32, i32, i32, i32, i32, i32, f64, u32,
                                             p, i64, p, i64, p, p, p]
        L.ksa_oracle_row_weights.restype = C.c_int
        L.ksa_oracle_row_weights.argtypes = [p, p, i32, i64, i32, i32, i32, i32, i32, i32, f64, u32,
                                             i32, i32, i64, p, p]
        L.ksa_oracle_decode.restype = C.c_int
        L.ksa_oracle_decode.argtypes = [p, p, p, i64, p, p, i64, p, p, i32, i32, i32, i32, i32, i32,
                                        i32, f64, p, p]
        _lib = L
    return _lib


def _f32(x, shape=None):
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def num_threads():
    lib().ksa_oracle_num_threads.restype = C.c_int
    return int(lib().ksa_oracle_num_threads())


def aug_len(n, c, m):
    return int(lib().ksa_oracle_aug_len(n, c, m))


def visible(aq, ak, c, m, Cw, flags=0):
    return bool(lib().ksa_oracle_visible(aq, ak, c, m, Cw, flags))


def mask_row(aq, n, c, m, Cw, flags=0):
    L = aug_len(n, c, m)
    out = np.zeros(L, dtype=np.uint8)
    lib().ksa_oracle_mask_row(aq, L, c, m, Cw, flags, _ptr(out))
    return out


def mask(n, c, m, Cw, flags=0):
    L = aug_len(n, c, m)
    return np.stack([mask_row(a, n, c, m, Cw, flags) for a in range(L)]) if L else np.zeros((0, 0), np.uint8)


def index_maps(n, c, m):
    L = aug_len(n, c, m)
    assert L >= 0
    J = n // c
    aug_chunk = np.zeros(L, np.int32)
    is_sum = np.zeros(L, np.uint8)
    pos_ids = np.zeros(L, np.int32)
    t2a = np.zeros(n, np.int32)
    s2a = np.zeros(J * m, np.int32)
    rc = lib().ksa_oracle_index_maps(n, c, m, _ptr(aug_chunk), _ptr(is_sum), _ptr(pos_ids), _ptr(t2a), _ptr(s2a))
    assert rc == 0
    return dict(aug_chunk=aug_chunk, aug_is_summary=is_sum, position_ids=pos_ids,
                text_to_aug=t2a, summary_to_aug=s2a)


def prefill(q, k, v, n, c, m, Cw, scale=0.0, flags=0, rows=None):
    """q [B, L, Hq, d], k/v [B, L, Hkv, d] (any float dtype holding the exact input values).
    Returns o [B, R, Hq, d] and lse [B, Hq, R] in float64; R = L or len(rows)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, L, Hq, d = q.shape
    Hkv = k.shape[2]
    assert L == aug_len(n, c, m), (L, n, c, m)
    assert k.shape == (B, L, Hkv, d) and v.shape == k.shape
    if rows is None:
        R, rows_arr, rows_p = L, None, None
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        R, rows_p = rows_arr.shape[0], _ptr(rows_arr)
    o = np.zeros((B, R, Hq, d), np.float64)
    lse = np.zeros((B, Hq, R), np.float64)
    rc = lib().ksa_oracle_prefill(_ptr(q), _ptr(k), _ptr(v), B, n, c, m, Cw, Hq, Hkv, d, float(scale),
                                  flags, rows_p, R, _ptr(o), _ptr(lse))
    if rc != 0:
        raise ValueError(f"ksa_oracle_prefill rejected its arguments (rc={rc})")
    return o, lse


def prefill_bwd(q, k, v, g, n, c, m, Cw, scale=0.0, flags=0, q_rows=None, k_rows=None):
    """Gradients of sum(g * O) with respect to q, k, v.  q, g [B, L, Hq, d]; k, v [B, L, Hkv, d].
    Returns dq [B, RQ, Hq, d], dk, dv [B, RK, Hkv, d] in float64; RQ / RK = L, or the number of listed
    augmented rows (an empty list skips that output)."""
    q, k, v, g = _f32(q), _f32(k), _f32(v), _f32(g)
    B, L, Hq, d = q.shape
    Hkv = k.shape[2]
    assert L == aug_len(n, c, m), (L, n, c, m)
    assert k.shape == (B, L, Hkv, d) and v.shape == k.shape and g.shape == q.shape

    def rows_of(rows):
        if rows is None:
            return L, None, None
        arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1))
        keep = arr if arr.size else np.zeros(1, np.int64)   # a valid pointer also for an empty list
        return arr.shape[0], keep, _ptr(keep)

    RQ, q_arr, q_p = rows_of(q_rows)
    RK, k_arr, k_p = rows_of(k_rows)
    dq = np.zeros((B, RQ, Hq, d), np.float64)
    dk = np.zeros((B, RK, Hkv, d), np.float64)
    dv = np.zeros((B, RK, Hkv, d), np.float64)
    rc = lib().ksa_oracle_prefill_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(g), B, n, c, m, Cw, Hq, Hkv, d,
                                      float(scale), flags, q_p, RQ, k_p, RK, _ptr(dq), _ptr(dk), _ptr(dv))
    if rc != 0:
        raise ValueError(f"ksa_oracle_prefill_bwd rejected its arguments (rc={rc})")
    return dq, dk, dv


def row_weights(q, k, n, c, m, Cw, b, h, aq, scale=0.0, flags=0):
    q, k = _f32(q), _f32(k)
    B, L, Hq, d = q.shape
    Hkv = k.shape[2]
    w = np.zeros(L, np.float64)
    lse = C.c_double(0.0)
    rc = lib().ksa_oracle_row_weights(_ptr(q), _ptr(k), B, n, c, m, Cw, Hq, Hkv, d, float(scale), flags,
                                      b, h, aq, _ptr(w), C.byref(lse))
    if rc != 0:
        raise ValueError(f"ksa_oracle_row_weights rejected its arguments (rc={rc})")
    return w, lse.value


def decode(q, k_sum, v_sum, k_txt, v_txt, txt_base, pos, c, m, Cw, scale=0.0):
    """q [B, Hq, d]; k_sum/v_sum [B, Hkv, S, d] by summary ordinal; k_txt/v_txt [B, Hkv, W, d] where
    slot t holds text index txt_base[b] + t; pos[b] = text index of the new token.
    Returns o [B, Hq, d], lse [B, Hq] in float64."""
    q, k_sum, v_sum, k_txt, v_txt = _f32(q), _f32(k_sum), _f32(v_sum), _f32(k_txt), _f32(v_txt)
    B, Hq, d = q.shape
    Hkv, S = k_sum.shape[1], k_sum.shape[2]
    W = k_txt.shape[2]
    assert k_sum.shape == (B, Hkv, S, d) and v_sum.shape == k_sum.shape
    assert k_txt.shape == (B, Hkv, W, d) and v_txt.shape == k_txt.shape
    tb = np.ascontiguousarray(np.asarray(txt_base, dtype=np.int64))
    ps = np.ascontiguousarray(np.asarray(pos, dtype=np.int64))
    assert tb.shape == (B,) and ps.shape == (B,)
    o = np.zeros((B, Hq, d), np.float64)
    lse = np.zeros((B, Hq), np.float64)
    rc = lib().ksa_oracle_decode(_ptr(q), _ptr(k_sum), _ptr(v_sum), S, _ptr(k_txt), _ptr(v_txt), W,
                                 _ptr(tb), _ptr(ps), B, c, m, Cw, Hq, Hkv, d, float(scale), _ptr(o), _ptr(lse))
    if rc != 0:
        raise ValueError(f"ksa_oracle_decode rejected its arguments (rc={rc})")
    return o, lse
