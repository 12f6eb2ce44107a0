"""Host logic of libksa (no GPU): the layout, row ranges, tile schedule and cache geometry must agree
bit for bit with the oracle's per-element predicate; the library must load and export every declared
symbol; bad arguments must be reported before any HIP call."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2604_24432_amd as K
from paper_2604_24432_amd import binding
from oracle import ksa_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SHAPES = [  # (n, c, m, C)
    (512, 64, 8, 1),       # the tiny benchmark shape
    (8, 2, 1, 1), (8, 4, 2, 1), (6, 2, 1, 0),
    (384, 64, 8, 0), (384, 64, 8, 2), (640, 128, 16, 1), (320, 64, 8, 9),
    (200, 8, 1, 3), (200, 8, 1, 128), (300, 20, 5, 1), (252, 12, 3, 2), (96, 96, 0, 0), (256, 16, 0, 2),
    (1024, 8, 1, 16),
    # an incomplete last chunk (text positions only)
    (100, 64, 8, 1), (7, 2, 1, 1), (300, 64, 8, 2), (1000, 128, 16, 1), (45, 8, 1, 3), (5, 8, 1, 1),
]


def params_for(n, c, m, C, flags=0, B=1, Hq=1, Hkv=1, d=64):
    return K.make_params(B, n, c, m, C, Hq, Hkv, d, flags=flags)


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.LIB_PATH)
    header = open(os.path.join(ROOT, "include", "ksa.h")).read()
    declared = set(re.findall(r"\b(ksa_[a-z0-9_]+)\s*\(", header))
    declared -= {"ksa_status", "ksa_params", "ksa_layout"}
    assert declared == set(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    assert "gfx950" in K.build_info()


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("flags", [0, K.KSA_FLAG_SUMMARY_SELF_ONLY])
def test_mask_rows_and_ranges_equal_oracle_predicate(shape, flags):
    n, c, m, C = shape
    lay = K.ksa_build_layout(params_for(n, c, m, C, flags))
    assert lay.aug_len == O.aug_len(n, c, m)
    maps_o = O.index_maps(n, c, m)
    t2a, s2a = maps_o["text_to_aug"], maps_o["summary_to_aug"]
    rows = range(lay.aug_len) if lay.aug_len <= 700 else np.random.default_rng(1).integers(0, lay.aug_len, 300)
    for a in rows:
        a = int(a)
        want = O.mask_row(a, n, c, m, C, flags)
        got = lay.mask_row(a)
        assert np.array_equal(got, want), (shape, a)
        s_lo, s_hi, t_lo, t_hi = lay.row_ranges(a)
        rebuilt = np.zeros_like(want)
        rebuilt[s2a[s_lo:s_hi]] = 1
        rebuilt[t2a[t_lo:t_hi]] = 1
        assert np.array_equal(rebuilt, want), (shape, a)


@pytest.mark.parametrize("shape", [(512, 64, 8, 1), (300, 20, 5, 1), (96, 96, 0, 0), (131072, 64, 8, 1)])
def test_index_maps_equal_oracle(shape):
    n, c, m, _ = shape
    lay = K.ksa_build_layout(params_for(n, c, m, 1))
    got, want = lay.index_maps(), O.index_maps(n, c, m)
    for key in want:
        assert np.array_equal(got[key], want[key]), key


def tile_cover(lay, n, c, m):
    """Visible-pair count matrix over (augmented q, augmented k) implied by the schedule's tiles
    (FULL tiles count every pair; MASKED tiles count the pairs inside the row ranges)."""
    L = lay.aug_len
    maps = O.index_maps(n, c, m)
    to_aug = {K.KSA_SPACE_TEXT: maps["text_to_aug"], K.KSA_SPACE_SUMMARY: maps["summary_to_aug"]}
    ranges = {a: lay.row_ranges(a) for a in range(L)}
    cover = np.zeros((L, L), np.int32)
    tp = lay.tile_pairs()
    for x in range(len(tp["kind"])):
        qs = to_aug[int(tp["q_space"][x])][tp["q_begin"][x]:tp["q_begin"][x] + tp["q_count"][x]]
        ksp = int(tp["k_space"][x])
        kb, kc = int(tp["k_begin"][x]), int(tp["k_count"][x])
        ks = to_aug[ksp][kb:kb + kc]
        assert len(qs) == tp["q_count"][x] and len(ks) == kc and kc > 0
        if tp["kind"][x] == K.KSA_TILE_FULL:
            assert kc == lay.k_tile_rows
            cover[np.ix_(qs, ks)] += 1
        else:
            for aq in qs:
                s_lo, s_hi, t_lo, t_hi = ranges[int(aq)]
                lo, hi = (t_lo, t_hi) if ksp == K.KSA_SPACE_TEXT else (s_lo, s_hi)
                lo, hi = max(lo, kb), min(hi, kb + kc)
                if hi > lo:
                    cover[aq, to_aug[ksp][lo:hi]] += 1
    return cover, tp


@pytest.mark.parametrize("shape", [(512, 64, 8, 1), (384, 64, 8, 0), (384, 64, 8, 2), (640, 128, 16, 1),
                                   (320, 64, 8, 9), (200, 8, 1, 3), (300, 20, 5, 1), (252, 12, 3, 2),
                                   (96, 96, 0, 0), (256, 16, 0, 2), (1024, 8, 1, 16), (1024, 8, 1, 128),
                                   (300, 1, 0, 40), (200, 1, 0, 130)])
def test_tile_schedule_covers_every_visible_pair_exactly_once(shape):
    n, c, m, C = shape
    lay = K.ksa_build_layout(params_for(n, c, m, C))
    cover, tp = tile_cover(lay, n, c, m)
    want = O.mask(n, c, m, C).astype(np.int32)
    # every visible pair lies in exactly one visited tile; FULL tiles contain no masked pair;
    # nothing invisible is ever counted
    assert np.array_equal(cover, want), shape


def test_every_visited_tile_is_live_and_full_tiles_dominate_at_scale():
    n, c, m, C = 131072, 64, 8, 1
    lay = K.ksa_build_layout(params_for(n, c, m, C, Hq=32, Hkv=8, d=128))
    tp = lay.tile_pairs()
    N = len(tp["kind"])
    full = int((tp["kind"] == K.KSA_TILE_FULL).sum())
    assert full / N > 0.9
    # issued pair slots vs live elements (closed form 1 085 936 128): padding overhead of the schedule
    issued = int((tp["q_count"].astype(np.int64) * tp["k_count"]).sum())
    assert 1085936128 <= issued < 1.15 * 1085936128
    # sampled masked tiles hold at least one visible pair for the tile's rows taken together
    maps = O.index_maps(n, c, m)
    rng = np.random.default_rng(3)
    masked_idx = np.nonzero(tp["kind"] == K.KSA_TILE_MASKED)[0]
    for x in rng.choice(masked_idx, 200, replace=False):
        sp_q, sp_k = int(tp["q_space"][x]), int(tp["k_space"][x])
        qmap = maps["text_to_aug"] if sp_q == K.KSA_SPACE_TEXT else maps["summary_to_aug"]
        kmap = maps["text_to_aug"] if sp_k == K.KSA_SPACE_TEXT else maps["summary_to_aug"]
        ks = kmap[tp["k_begin"][x]:tp["k_begin"][x] + tp["k_count"][x]]
        live = False
        for aq in qmap[tp["q_begin"][x]:tp["q_begin"][x] + tp["q_count"][x]]:
            if O.mask_row(int(aq), n, c, m, C)[ks].any():
                live = True
                break
        assert live, x


@pytest.mark.parametrize("shape", [(512, 64, 8, 1), (512, 64, 8, 0), (512, 64, 8, 3), (240, 8, 1, 5), (256, 16, 0, 2)])
def test_decode_ranges_hold_exactly_the_visible_set(shape):
    """Rows named by ksa_decode_ranges, translated back through the cache geometry, must be exactly the
    oracle's visible set of the text row at that position."""
    n, c, m, C = shape
    p = params_for(n, c, m, C)
    s_cap, rows = K.cache_geometry(p)
    assert s_cap == n // c * m and rows == s_cap + (C + 1) * c
    maps = O.index_maps(n, c, m)
    for pos in list(range(0, min(n, 3 * c + 2))) + [n // 2, n - c - 1, n - c, n - 1]:
        # what each cache row holds at this moment: summaries of completed chunks, text up to pos
        holds = {}
        for u in range((pos // c) * m):
            holds[K.cache_summary_row(p, u)] = ("s", u)
        for i in range(max(0, (pos // c - C)) * c, pos + 1):
            holds[K.cache_text_row(p, i)] = ("t", i)
        rg = K.ksa_decode_ranges(p, pos)
        read = []
        for off, ln in rg.reshape(3, 2):
            read += list(range(off, off + ln))
        assert len(set(read)) == len(read)
        got = set()
        for row in read:
            kind, idx = holds[row]          # KeyError = reads a row that holds nothing valid
            got.add(int(maps["text_to_aug"][idx] if kind == "t" else maps["summary_to_aug"][idx]))
        want = set(np.nonzero(O.mask_row(int(maps["text_to_aug"][pos]), n, c, m, C))[0].tolist())
        assert got == want, (shape, pos)


def test_bad_arguments_are_reported_without_a_gpu():
    bad = [
        dict(n_summary=8, compress_ratio=4),            # k * m != c
        dict(n_q_heads=3, n_kv_heads=2),                # Hq % Hkv != 0
        dict(batch=0), dict(window_chunks=-1), dict(n_summary=-1), dict(flags=2),
    ]
    base = dict(batch=1, n_text=128, chunk_len=64, n_summary=8, compress_ratio=8, window_chunks=1,
                n_q_heads=4, n_kv_heads=2, head_dim=64, softmax_scale=0.0, flags=0)
    for delta in bad:
        kw = dict(base, **delta)
        with pytest.raises(K.KsaError) as e:
            K.ksa_build_layout(K.ksa_params(**kw))
        assert e.value.status == -1, delta
    with pytest.raises(K.KsaError) as e:
        K.ksa_build_layout(K.ksa_params(**dict(base, head_dim=96)))
    assert e.value.status == -2
    lay = K.ksa_build_layout(K.ksa_params(**base))
    with pytest.raises(K.KsaError) as e:
        lay.row_ranges(lay.aug_len)
    assert e.value.status == -5
    p = K.ksa_params(**base)
    with pytest.raises(K.KsaError):
        K.ksa_decode_ranges(p, 128)
    # null tensors are rejected before any HIP call
    rc = binding.lib().ksa_prefill_fwd(lay.handle, None, None, None, None, None, None, None, None, None, 0, None)
    assert rc == -1
    # a workspace that is too small is reported as such (fake, never dereferenced, 16-byte aligned addresses)
    fake = ctypes.c_void_p(4096)
    need = K.prefill_workspace_bytes(lay)
    # batch * Hkv * d * (n_text + 16 summaries rounded up to 64) bf16, then one fp32 per (batch, KV head, 64-key tile:
    # 2 text tiles + 1 summary tile) and one per (batch, KV head)
    assert need == 1 * 2 * 64 * (128 + 64) * 2 + (1 * 2 * 3 + 1 * 2) * 4
    rc = binding.lib().ksa_prefill_fwd(lay.handle, fake, fake, fake, fake, None, None, None, None, fake, need - 1, None)
    assert rc == -3
    rc = binding.lib().ksa_decode_fwd(ctypes.byref(p), None, None, None, None, None, None, None, None, 0, 0, None)
    assert rc == -1
    assert binding.status_string(-3) == "workspace too small"
    assert K.decode_workspace_bytes(p, 4) == 1 * 4 * 4 * (64 + 2) * 4


@pytest.mark.parametrize("B,Hq,Hkv", [(2, 32, 8), (1, 32, 8), (1, 1, 1), (1, 6, 3), (3, 4, 4), (5, 2, 1)])
def test_launch_order_lists_every_unit_once_and_groups_kv_heads_per_xcd(B, Hq, Hkv):
    n, c, m = 2048, 64, 8
    lay = K.ksa_build_layout(K.make_params(B, n, c, m, 1, Hq, Hkv, 128))
    lo = lay.launch_order()
    live = lo["q_begin"] >= 0
    units = list(zip(lo["q_space"][live].tolist(), lo["q_begin"][live].tolist(), lo["batch"][live].tolist(),
                     lo["q_head"][live].tolist()))
    n_items = n // lay.q_tile_rows + (n // c * m + lay.q_tile_rows - 1) // lay.q_tile_rows
    # a workgroup stacks as many query heads of a KV group as divide it (at most 4) on a shorter query tile
    g = Hq // Hkv
    assert lay.heads_per_workgroup == (4 if g % 4 == 0 else 2 if g % 2 == 0 else 1)
    assert lay.q_tile_rows * lay.heads_per_workgroup == 256
    assert all(h % lay.heads_per_workgroup == 0 for h in lo["q_head"][live].tolist())
    assert len(units) == len(set(units)) == n_items * B * Hq // lay.heads_per_workgroup
    assert len(lo["q_begin"]) % 8 == 0
    # workgroups congruent mod 8 land on one XCD: with at least 8 (batch, KV head) groups an XCD never
    # shares a group with another XCD
    if B * Hkv >= 8:
        owner = {}
        for x in np.nonzero(live)[0]:
            grp = (int(lo["batch"][x]), int(lo["q_head"][x]) // (Hq // Hkv))
            assert owner.setdefault(grp, x % 8) == x % 8
