"""Host logic of the cache lifecycle entry points (no GPU): the rows a summary query reads must be exactly the keys
the oracle's predicate makes visible to that summary position, and bad arguments must be reported before any
HIP call."""
import ctypes as C

import numpy as np
import pytest

import paper_2604_24432_amd as K
from paper_2604_24432_amd import binding
from oracle import ksa_oracle as O

SHAPES = [(512, 64, 8, 1), (8, 2, 1, 1), (8, 4, 2, 1), (384, 64, 8, 0), (384, 64, 8, 2), (300, 20, 5, 1),
          (252, 12, 3, 2), (200, 8, 1, 3)]


def params_for(n, c, m, Cw, flags=0, B=1, Hq=1, Hkv=1, d=64):
    return K.make_params(B, n, c, m, Cw, Hq, Hkv, d, flags=flags)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("flags", [0, K.KSA_FLAG_SUMMARY_SELF_ONLY])
def test_summary_query_rows_equal_oracle_predicate(shape, flags):
    """Cache rows -> logical keys -> augmented positions must reproduce the oracle's mask row of the summary."""
    n, c, m, Cw = shape
    p = params_for(n, c, m, Cw, flags)
    s_cap, rows = K.cache_geometry(p)
    maps = O.index_maps(n, c, m)
    t2a, s2a = maps["text_to_aug"], maps["summary_to_aug"]
    L = O.aug_len(n, c, m)
    for u in range(s_cap):
        j = u // m
        off0, len0, off1, len1 = (int(x) for x in K.ksa_decode_summary_ranges(p, u))
        got = np.zeros(L, np.uint8)
        for r in range(off0, off0 + len0):          # summary buffer rows are summary ordinals
            assert 0 <= r < s_cap
            got[s2a[r]] = 1
        # when the summary step of chunk j runs, ring slot j mod (C+1) holds chunk j: find the text index of each row
        row_of_text = {K.cache_text_row(p, i): i for i in range(j * c, j * c + c)}
        for r in range(off1, off1 + len1):
            assert r in row_of_text, (shape, u, r)
            got[t2a[row_of_text[r]]] = 1
        want = O.mask_row(int(s2a[u]), n, c, m, Cw, flags)
        assert np.array_equal(got, want), (shape, u)


def test_summary_ranges_reject_bad_arguments():
    p = params_for(512, 64, 8, 1)
    out = (C.c_int32 * 4)()
    lib = binding.lib()
    assert lib.ksa_decode_summary_ranges(C.byref(p), -1, out) == -5
    assert lib.ksa_decode_summary_ranges(C.byref(p), 64, out) == -5          # s_cap = 8 chunks * 8
    assert lib.ksa_decode_summary_ranges(C.byref(p), 0, None) == -1
    p0 = params_for(256, 16, 0, 2)
    assert lib.ksa_decode_summary_ranges(C.byref(p0), 0, out) == -1           # no summaries at all


def test_cache_entry_points_validate_before_touching_the_gpu():
    lib = binding.lib()
    p = params_for(512, 64, 8, 1, B=2, Hq=4, Hkv=2, d=64)
    buf = C.create_string_buffer(4096 + 16)
    a = (C.addressof(buf) + 15) & ~15            # a 16-byte aligned host address: never dereferenced by these checks
    vp = C.c_void_p
    # ksa_cache_from_prefill
    assert lib.ksa_cache_from_prefill(C.byref(p), 64, None, vp(a), None, vp(a), vp(a), None, None) == -1
    assert lib.ksa_cache_from_prefill(C.byref(p), -64, vp(a), vp(a), None, vp(a), vp(a), None, None) == -1
    assert lib.ksa_cache_from_prefill(C.byref(p), 576, vp(a), vp(a), None, vp(a), vp(a), None, None) == -5
    assert lib.ksa_cache_from_prefill(C.byref(p), 64, vp(a + 2), vp(a), None, vp(a), vp(a), None, None) == -1
    bad = (C.c_int64 * 3)(100, 12, 64)           # row stride not a multiple of 8 elements
    assert lib.ksa_cache_from_prefill(C.byref(p), 64, vp(a), vp(a), bad, vp(a), vp(a), None, None) == -1
    # ksa_cache_append
    assert lib.ksa_cache_append(C.byref(p), 2, vp(a), vp(a), vp(a), vp(a), vp(a), None, None) == -1
    assert lib.ksa_cache_append(C.byref(p), 0, vp(a), None, vp(a), vp(a), vp(a), None, None) == -1
    assert lib.ksa_cache_append(C.byref(p), 0, vp(a), vp(a), None, vp(a), vp(a), None, None) == -1
    p0 = params_for(256, 16, 0, 2, B=2, Hq=4, Hkv=2, d=64)
    assert lib.ksa_cache_append(C.byref(p0), 1, vp(a), vp(a), vp(a), vp(a), vp(a), None, None) == -1
    # ksa_decode_summary_fwd
    assert lib.ksa_decode_summary_fwd(C.byref(p), None, vp(a), vp(a), vp(a), vp(a), None, None, vp(a), 1 << 20, 0,
                                      None) == -1
    assert lib.ksa_decode_summary_fwd(C.byref(p), vp(a), vp(a), vp(a), vp(a), vp(a), None, None, vp(a), 16, 1,
                                      None) == -3
    assert lib.ksa_decode_summary_fwd(C.byref(p0), vp(a), vp(a), vp(a), vp(a), vp(a), None, None, vp(a), 1 << 20, 1,
                                      None) == -1


def test_prefill_bwd_validates_before_touching_the_gpu():
    """ksa_prefill_bwd: null / misaligned pointers, bad strides and a short workspace are reported by the argument checks,
    which run before the first HIP call; the workspace is two fp32 per (batch, query head, padded row)."""
    lib = binding.lib()
    p = params_for(600, 64, 8, 1, B=2, Hq=4, Hkv=2, d=64)
    lay = K.ksa_build_layout(p)
    n_sum = (600 // 64) * 8
    pad = lambda x: (x + 63) // 64 * 64
    assert binding.prefill_bwd_workspace_bytes(lay) == 2 * 4 * 2 * 4 * (pad(600) + pad(n_sum))
    assert lib.ksa_prefill_bwd_workspace_bytes(None) == 0
    buf = C.create_string_buffer(4096 + 16)
    a = (C.addressof(buf) + 15) & ~15            # a 16-byte aligned host address: never dereferenced by these checks
    vp = C.c_void_p
    big = 1 << 30

    def call(q=a, k=a, v=a, o=a, lse=a, g=a, dq=a, dk=a, dv=a, qs=None, ws=a, ws_bytes=big, layout=lay.handle):
        return lib.ksa_prefill_bwd(layout, vp(q), vp(k), vp(v), vp(o), vp(lse), vp(g), vp(dq), vp(dk), vp(dv), qs, None,
                                   None, None, None, vp(ws), ws_bytes, None)

    assert call(layout=None) == -1
    for name in ("q", "k", "v", "o", "lse", "g", "dq", "dk", "dv", "ws"):
        assert call(**{name: None}) == -1, name
    for name in ("q", "k", "v", "o", "g", "dq", "dk", "dv", "ws"):
        assert call(**{name: a + 2}) == -1, name
    assert call(lse=a + 2) == -1
    assert call(qs=(C.c_int64 * 3)(100, 12, 64)) == -1        # row stride not a multiple of 8 elements
    assert call(ws_bytes=64) == -3
