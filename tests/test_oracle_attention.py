"""Pins for the oracle's attention arithmetic (CPU only).

Dense-causal and sliding-window special cases against independent numpy / torch routines,
a pure-Python brute force on tiny inputs, softmax invariants, and decode == prefill row.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ksa_oracle as O
from tests.test_oracle_mask import literal_sequence, literal_visible_sets, closed_form_row_count


def rand_qkv(B, L, Hq, Hkv, d, seed):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, L, Hq, d)).astype(np.float32)
    k = rng.standard_normal((B, L, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((B, L, Hkv, d)).astype(np.float32)
    return q, k, v


def masked_attention_numpy(q, k, v, mask, scale):
    """Independent dense reference: explicit mask matrix, numpy einsum, fp64.  mask [L, L] bool."""
    B, L, Hq, d = q.shape
    Hkv = k.shape[2]
    g = Hq // Hkv
    q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))
    kk = np.repeat(k64, g, axis=2)
    vv = np.repeat(v64, g, axis=2)
    s = np.einsum("blhd,bmhd->bhlm", q64, kk) * scale
    s = np.where(mask[None, None], s, -np.inf)
    mx = s.max(axis=-1, keepdims=True)
    p = np.exp(s - mx)
    den = p.sum(axis=-1, keepdims=True)
    o = np.einsum("bhlm,bmhd->blhd", p / den, vv)
    lse = (mx + np.log(den))[..., 0]
    return o, lse


def test_single_chunk_no_summaries_is_dense_causal_torch_sdpa():
    B, n, Hq, Hkv, d = 2, 48, 4, 2, 16
    q, k, v = rand_qkv(B, n, Hq, Hkv, d, 1)
    o, lse = O.prefill(q, k, v, n=n, c=n, m=0, Cw=0)
    tq = torch.from_numpy(q).double().permute(0, 2, 1, 3)
    tk = torch.from_numpy(k).double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(v).double().permute(0, 2, 1, 3).repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    ref = ref.permute(0, 2, 1, 3).numpy()
    assert np.abs(o - ref).max() < 1e-12


@pytest.mark.parametrize("c,Cw", [(4, 11), (4, 200), (8, 5), (48, 0)])
def test_window_covering_everything_without_summaries_is_dense_causal(c, Cw):
    B, n, Hq, Hkv, d = 1, 48, 2, 1, 8
    q, k, v = rand_qkv(B, n, Hq, Hkv, d, 2)
    o, lse = O.prefill(q, k, v, n=n, c=c, m=0, Cw=Cw)
    ref_o, ref_lse = masked_attention_numpy(q, k, v, np.tril(np.ones((n, n), bool)), 1 / math.sqrt(d))
    assert np.abs(o - ref_o).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-12


@pytest.mark.parametrize("c,Cw", [(4, 0), (4, 1), (8, 2), (2, 3)])
def test_no_summaries_is_chunk_aligned_sliding_window(c, Cw):
    """Eq. 2: key i' visible iff (floor(i/c) - C)*c <= i' <= i."""
    B, n, Hq, Hkv, d = 1, 40, 2, 2, 8
    q, k, v = rand_qkv(B, n, Hq, Hkv, d, 3)
    mask = np.array([[max(0, i // c - Cw) * c <= ik <= i for ik in range(n)] for i in range(n)])
    o, lse = O.prefill(q, k, v, n=n, c=c, m=0, Cw=Cw, scale=0.37)
    ref_o, ref_lse = masked_attention_numpy(q, k, v, mask, 0.37)
    assert np.abs(o - ref_o).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-12


@pytest.mark.parametrize("w", [1, 5, 16, 100])
def test_token_window_attention_is_band_masked_softmax(w):
    """Token-level sliding window attention of width w (chunk size 1, no summaries, C = w - 1) against numpy's
    softmax under the band mask i - w < k <= i."""
    n = 48
    q, k, v = rand_qkv(2, n, 4, 2, 16, seed=30 + w)
    o, lse = O.prefill(q, k, v, n=n, c=1, m=0, Cw=w - 1)
    i = np.arange(n)
    band = (i[None, :] <= i[:, None]) & (i[:, None] - i[None, :] < w)
    ref_o, ref_lse = masked_attention_numpy(q, k, v, band, 1 / math.sqrt(16))
    assert np.abs(o - ref_o).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-12


def test_window_covering_everything_with_summaries():
    """With C >= J-1 Eq. 3's summary range is empty: text rows are dense causal attention over the
    text-only subsequence; summary rows are a softmax over their own chunk."""
    B, n, c, m, Hq, Hkv, d = 1, 32, 8, 2, 2, 1, 8
    L = O.aug_len(n, c, m)
    q, k, v = rand_qkv(B, L, Hq, Hkv, d, 4)
    o, _ = O.prefill(q, k, v, n=n, c=c, m=m, Cw=5)
    maps = O.index_maps(n, c, m)
    t2a = maps["text_to_aug"]
    ref_o, _ = masked_attention_numpy(q[:, t2a], k[:, t2a], v[:, t2a], np.tril(np.ones((n, n), bool)),
                                      1 / math.sqrt(d))
    assert np.abs(o[:, t2a] - ref_o).max() < 1e-12
    for j in range(n // c):
        for u in range(m):
            a = maps["summary_to_aug"][j * m + u]
            cols = list(t2a[j * c:(j + 1) * c]) + list(maps["summary_to_aug"][j * m:j * m + u + 1])
            for h in range(Hq):
                s = (k[0, cols, 0].astype(np.float64) @ q[0, a, h].astype(np.float64)) / math.sqrt(d)
                p = np.exp(s - s.max())
                want = (p / p.sum()) @ v[0, cols, 0].astype(np.float64)
                assert np.abs(o[0, a, h] - want).max() < 1e-12


def brute_force(q, k, v, n, c, m, Cw, scale, self_only=False):
    """Pure-Python loops over the literal visible sets, math.fsum accumulation."""
    B, L, Hq, d = q.shape
    g = Hq // k.shape[2]
    sets = literal_visible_sets(n, c, m, Cw, self_only)
    o = np.zeros((B, L, Hq, d))
    lse = np.zeros((B, Hq, L))
    for b in range(B):
        for h in range(Hq):
            for a in range(L):
                keys = sorted(sets[a])
                s = [scale * math.fsum(float(q[b, a, h, t]) * float(k[b, ak, h // g, t]) for t in range(d))
                     for ak in keys]
                mx = max(s)
                e = [math.exp(x - mx) for x in s]
                den = math.fsum(e)
                for t in range(d):
                    o[b, a, h, t] = math.fsum(e[x] / den * float(v[b, keys[x], h // g, t]) for x in range(len(keys)))
                lse[b, h, a] = mx + math.log(den)
    return o, lse


@pytest.mark.parametrize("shape", [(8, 2, 1, 1), (8, 4, 2, 1), (24, 4, 2, 0), (32, 4, 1, 2), (24, 6, 3, 1)])
@pytest.mark.parametrize("flags", [0, O.FLAG_SUMMARY_SELF_ONLY])
def test_brute_force_tiny(shape, flags):
    n, c, m, Cw = shape
    L = O.aug_len(n, c, m)
    q, k, v = rand_qkv(2, L, 4, 2, 4, seed=10 + n + c)
    scale = 0.5
    o, lse = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw, scale=scale, flags=flags)
    ref_o, ref_lse = brute_force(q, k, v, n, c, m, Cw, scale, self_only=bool(flags))
    assert np.abs(o - ref_o).max() < 1e-13
    assert np.abs(lse - ref_lse).max() < 1e-13


def test_dense_masked_reference_on_a_mid_size_ksa_shape():
    """KSA proper (summaries visible, GQA, default scale) against numpy with the literal-set mask."""
    n, c, m, Cw = 96, 8, 2, 1
    L = O.aug_len(n, c, m)
    q, k, v = rand_qkv(2, L, 8, 2, 32, seed=5)
    sets = literal_visible_sets(n, c, m, Cw)
    mask = np.zeros((L, L), bool)
    for a, s in enumerate(sets):
        mask[a, sorted(s)] = True
    o, lse = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw)
    ref_o, ref_lse = masked_attention_numpy(q, k, v, mask, 1 / math.sqrt(32))
    assert np.abs(o - ref_o).max() < 1e-12
    assert np.abs(lse - ref_lse).max() < 1e-12


def test_rows_subset_equals_full():
    n, c, m, Cw = 64, 8, 2, 1
    L = O.aug_len(n, c, m)
    q, k, v = rand_qkv(2, L, 4, 2, 16, seed=6)
    o, lse = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw)
    rows = [0, 7, 8, 9, 10, 33, L - 1]
    o2, lse2 = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw, rows=rows)
    assert np.array_equal(o[:, rows], o2)
    assert np.array_equal(lse[:, :, rows], lse2)


def test_softmax_invariants():
    n, c, m, Cw = 64, 8, 2, 1
    L = O.aug_len(n, c, m)
    q, k, v = rand_qkv(1, L, 4, 2, 16, seed=7)
    M = O.mask(n, c, m, Cw)
    for a in [0, 5, 8, 9, 27, 41, L - 2, L - 1]:
        for h in range(4):
            w, lse = O.row_weights(q, k, n, c, m, Cw, 0, h, a)
            assert abs(w.sum() - 1.0) < 1e-12
            assert np.all(w[M[a] == 0] == 0.0)      # exactly zero, not exp(-big)
            assert np.all(w[M[a] == 1] > 0.0)
    # V == 1 -> O == 1
    o, _ = O.prefill(q, k, np.ones_like(v), n=n, c=c, m=m, Cw=Cw)
    assert np.abs(o - 1.0).max() < 1e-12
    # Q == 0 -> uniform weights: O = mean of the visible V rows, exp(LSE) = number of visible keys
    o, lse = O.prefill(np.zeros_like(q), k, v, n=n, c=c, m=m, Cw=Cw)
    for a in range(L):
        cols = np.nonzero(M[a])[0]
        assert len(cols) == closed_form_row_count(a, c, m, Cw)
        for h in range(4):
            want = v[0, cols, h // 2].astype(np.float64).mean(axis=0)
            assert np.abs(o[0, a, h] - want).max() < 1e-12
            assert abs(math.exp(lse[0, h, a]) - len(cols)) < 1e-9


def test_row_weights_values_with_grouped_heads():
    """Value pin of row_weights: for several (b, h, aq) with Hq != Hkv and B > 1 the weights, applied to the V rows
    of the query head's KV head, must reproduce the prefill row, the log-sum-exp must agree, and each weight must
    equal exp(scale * q.k - lse) written out here.  A wrong batch / KV-head / row offset in the wrapper fails all
    three (every batch and every KV head holds different random data)."""
    n, c, m, Cw = 48, 8, 2, 1
    L = O.aug_len(n, c, m)
    B, Hq, Hkv, d = 2, 6, 2, 16
    q, k, v = rand_qkv(B, L, Hq, Hkv, d, seed=21)
    scale = 0.3
    o, lse = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw, scale=scale)
    M = O.mask(n, c, m, Cw)
    for b in range(B):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            for a in [0, 9, 10, 27, 31, L - 11, L - 1]:
                w, l = O.row_weights(q, k, n, c, m, Cw, b, h, a, scale=scale)
                assert abs(l - lse[b, h, a]) < 1e-13
                got = w @ v[b, :, hk, :].astype(np.float64)
                assert np.abs(got - o[b, a, h]).max() < 1e-13
                s = scale * (k[b, :, hk, :].astype(np.float64) @ q[b, a, h].astype(np.float64))
                want = np.where(M[a] == 1, np.exp(s - l), 0.0)
                assert np.abs(w - want).max() < 1e-13


def test_scale_default_and_shift_invariance():
    n, c, m, Cw = 32, 8, 1, 1
    L = O.aug_len(n, c, m)
    q, k, v = rand_qkv(1, L, 2, 1, 16, seed=8)
    o1, l1 = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw)                 # default 1/sqrt(d)
    o2, l2 = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw, scale=0.25)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    # doubling q and halving the scale leaves the result unchanged
    o3, l3 = O.prefill(2 * q, k, v, n=n, c=c, m=m, Cw=Cw, scale=0.125)
    assert np.abs(o1 - o3).max() < 1e-13 and np.abs(l1 - l3).max() < 1e-13


def logical_decode_operands(k, v, n_ctx_text, c, m, maps, W, txt_base):
    """Gather the logical decode arrays from an augmented prefill K/V [B, L, Hkv, d]."""
    s2a, t2a = maps["summary_to_aug"], maps["text_to_aug"]
    S = len(s2a)
    k_sum = np.transpose(k[:, s2a], (0, 2, 1, 3)) if S else np.zeros((k.shape[0], k.shape[2], 0, k.shape[3]), np.float32)
    v_sum = np.transpose(v[:, s2a], (0, 2, 1, 3)) if S else np.zeros_like(k_sum)
    idx = [t2a[min(txt_base + t, n_ctx_text - 1)] for t in range(W)]   # slots past the end repeat the last row
    k_txt = np.transpose(k[:, idx], (0, 2, 1, 3))
    v_txt = np.transpose(v[:, idx], (0, 2, 1, 3))
    return k_sum, v_sum, k_txt, v_txt


@pytest.mark.parametrize("shape", [(64, 8, 2, 1), (64, 8, 1, 0), (48, 4, 4, 3), (32, 8, 0, 1)])
def test_decode_equals_prefill_row(shape):
    """Section 2.3.1: the cache slice read for a new text token holds exactly that token's visible set,
    so decoding text index p equals row text_to_aug[p] of prefill."""
    n, c, m, Cw = shape
    L = O.aug_len(n, c, m)
    B, Hq, Hkv, d = 2, 4, 2, 16
    q, k, v = rand_qkv(B, L, Hq, Hkv, d, seed=20 + c)
    maps = O.index_maps(n, c, m)
    o_full, lse_full = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw)
    W = (Cw + 1) * c
    for p in [0, 1, c - 1, c, c + 1, 2 * c + 3, n - c, n - 1]:
        txt_base = max(0, p // c - Cw) * c
        k_sum, v_sum, k_txt, v_txt = logical_decode_operands(k, v, n, c, m, maps, W, txt_base)
        aq = maps["text_to_aug"][p]
        o, lse = O.decode(q[:, aq], k_sum, v_sum, k_txt, v_txt, [txt_base] * B, [p] * B, c, m, Cw)
        assert np.abs(o - o_full[:, aq]).max() < 1e-13
        assert np.abs(lse - lse_full[:, :, aq]).max() < 1e-13


def test_decode_is_order_free_and_ignores_invisible_rows():
    n, c, m, Cw = 64, 8, 2, 1
    L = O.aug_len(n, c, m)
    B, Hq, Hkv, d = 1, 2, 1, 8
    q, k, v = rand_qkv(B, L, Hq, Hkv, d, seed=30)
    maps = O.index_maps(n, c, m)
    p = 43                                       # chunk 5: sees summaries of chunks 0..3, text 32..43
    W, txt_base = 2 * c, 32
    k_sum, v_sum, k_txt, v_txt = logical_decode_operands(k, v, n, c, m, maps, W, txt_base)
    aq = maps["text_to_aug"][p]
    o, lse = O.decode(q[:, aq], k_sum, v_sum, k_txt, v_txt, [txt_base], [p], c, m, Cw)
    # garbage in rows that are resident but not visible (in-window summaries, future text) changes nothing
    k2, v2, kt2, vt2 = k_sum.copy(), v_sum.copy(), k_txt.copy(), v_txt.copy()
    k2[:, :, 4 * m:] = 1e6
    v2[:, :, 4 * m:] = -1e6
    kt2[:, :, p - txt_base + 1:] = 1e6
    vt2[:, :, p - txt_base + 1:] = -1e6
    o2, lse2 = O.decode(q[:, aq], k2, v2, kt2, vt2, [txt_base], [p], c, m, Cw)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    # the supplied rows must cover the visible set
    with pytest.raises(ValueError):
        O.decode(q[:, aq], k_sum[:, :, :3], v_sum[:, :, :3], k_txt, v_txt, [txt_base], [p], c, m, Cw)
    with pytest.raises(ValueError):
        O.decode(q[:, aq], k_sum, v_sum, k_txt, v_txt, [txt_base + 1], [p], c, m, Cw)


def test_bad_arguments_are_rejected():
    q, k, v = rand_qkv(1, 9, 3, 2, 4, seed=1)
    with pytest.raises(ValueError):
        O.prefill(q, k, v, n=8, c=8, m=1, Cw=0)          # Hq not a multiple of Hkv
    q, k, v = rand_qkv(1, 9, 2, 2, 4, seed=1)
    with pytest.raises(ValueError):
        O.prefill(q, k, v, n=8, c=8, m=1, Cw=0, rows=[9])  # row out of range


def test_ragged_prefill_is_the_leading_part_of_the_whole_chunk_prefill():
    """Rows of an incomplete-last-chunk sequence see exactly what the same rows of the sequence extended to whole
    chunks see, so outputs and log-sum-exps must agree to the last bit."""
    rng = np.random.default_rng(5)
    for (n, c, m, Cw) in [(7, 2, 1, 1), (21, 8, 2, 1), (37, 16, 4, 0), (50, 8, 1, 3)]:
        n_up = (n + c - 1) // c * c
        L, L_up = O.aug_len(n, c, m), O.aug_len(n_up, c, m)
        q = rng.standard_normal((2, L_up, 4, 16)).astype(np.float32)
        k = rng.standard_normal((2, L_up, 2, 16)).astype(np.float32)
        v = rng.standard_normal((2, L_up, 2, 16)).astype(np.float32)
        o_up, lse_up = O.prefill(q, k, v, n_up, c, m, Cw)
        o, lse = O.prefill(q[:, :L].copy(), k[:, :L].copy(), v[:, :L].copy(), n, c, m, Cw)
        assert np.array_equal(o, o_up[:, :L]) and np.array_equal(lse, lse_up[:, :, :L]), (n, c, m, Cw)
