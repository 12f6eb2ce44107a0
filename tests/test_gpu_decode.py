"""GPU parity of ksa_decode_fwd against the CPU oracle (run with -m gpu on an MI355X).

The oracle receives the logical rows (summary ordinal / text index); the library receives the same rows
placed in its physical cache (summary buffer + text ring).  Rows the token must not see are filled with
large values so that any read outside the visible set shows up in the output.
"""
import sys

import numpy as np
import pytest
import torch

import paper_2604_24432_amd as K
from paper_2604_24432_amd import synth
from oracle import ksa_oracle as O

pytestmark = pytest.mark.gpu

# decode keeps its weights and sums in fp32, so the log-sum-exp is held to fp32 accuracy
MAX_ABS, MEAN_ABS, LSE_ABS = 2e-2, 2e-3, 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_case(name, B, Hq, Hkv, d, n_cap, c, m, C, positions, n_splits=0, seed=1, poison=True):
    """positions: one text index per sequence.  All sequences share the logical K/V rows; each reads its own
    visible set.  The text window passed to the oracle is [txt_base, txt_base + (C+1)c) per sequence."""
    say(f"decode parity {name}: B{B} Hq{Hq} Hkv{Hkv} d{d} cap{n_cap} c{c} m{m} C{C} splits{n_splits}")
    cfg = synth.KsaConfig(name, B, Hq, Hkv, d, n_cap, c, m, C, seed=seed)
    p = K.make_params(B, n_cap, c, m, C, Hq, Hkv, d)
    s_cap, rows = K.cache_geometry(p)
    W = (C + 1) * c
    q, k_sum, v_sum, k_txt, v_txt = synth.make_decode_inputs(cfg, max(s_cap, 1), W)
    if m == 0:
        k_sum, v_sum = k_sum[:, :, :0], v_sum[:, :, :0]
    k_cache = torch.zeros((B, Hkv, rows, d), dtype=torch.bfloat16)
    v_cache = torch.zeros_like(k_cache)
    txt_base = []
    k_txt_l, v_txt_l = k_txt.clone(), v_txt.clone()
    for b, pos in enumerate(positions):
        j = pos // c
        base = max(0, j - C) * c
        txt_base.append(base)
        # per-sequence cache: summaries of finished chunks, text of the window up to pos; the rest is poison
        kc, vc = K.pack_cache(K.make_params(1, n_cap, c, m, C, Hq, Hkv, d), k_sum[b:b + 1], v_sum[b:b + 1],
                              k_txt[b:b + 1], v_txt[b:b + 1], base)
        if poison:
            n_vis_sum = max(0, j - C) * m
            kc[:, :, n_vis_sum:s_cap] = 40.0      # in-window / future summaries: resident, must not be read
            vc[:, :, n_vis_sum:s_cap] = -1000.0
            for t in range(pos - base + 1, W):    # text slots after pos: stale
                if base + t < n_cap:
                    r = K.cache_text_row(p, base + t)
                    kc[:, :, r] = 40.0
                    vc[:, :, r] = -1000.0
        k_cache[b], v_cache[b] = kc[0], vc[0]
    pos_t = torch.tensor(positions, dtype=torch.int32)
    o, lse = K.ksa_decode_fwd(p, q.cuda(), k_cache.cuda(), v_cache.cuda(), pos_t.cuda(), n_splits=n_splits)
    torch.cuda.synchronize()
    o_ref, lse_ref = O.decode(q.float().numpy(), k_sum.float().numpy(), v_sum.float().numpy(),
                              k_txt_l.float().numpy(), v_txt_l.float().numpy(), txt_base, positions, c, m, C)
    err = np.abs(o.float().cpu().numpy().astype(np.float64) - o_ref)
    lerr = np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref)
    say(f"  max-abs {err.max():.3e} mean-abs {err.mean():.3e} lse max-abs {lerr.max():.3e}")
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS and lerr.max() <= LSE_ABS, name


def test_decode_small_mixed_positions():
    c, m, C = 64, 8, 1
    n_cap = 64 * 40
    positions = [0, 1, 63, 64, 65, 127, 128, 200, 64 * 39, 64 * 40 - 1, 1000, 1999]
    run_case("mixed", len(positions), 8, 2, 128, n_cap, c, m, C, positions)


@pytest.mark.parametrize("n_splits", [1, 2, 3, 7, 16])
def test_decode_split_counts(n_splits):
    c, m, C = 64, 8, 1
    run_case(f"splits{n_splits}", 3, 4, 1, 128, 64 * 300, c, m, C, [64 * 299 + 5, 64 * 150 + 63, 77], n_splits=n_splits)


@pytest.mark.parametrize("case", [
    ("window0", 2, 4, 2, 128, 64 * 20, 64, 8, 0, [64 * 19 + 3, 64 * 7]),
    ("window3", 3, 4, 4, 128, 32 * 50, 32, 4, 3, [32 * 49 + 31, 32 * 2 + 1, 32 * 5]),
    ("paper_m1_c8_C128", 2, 4, 2, 128, 8 * 600, 8, 1, 128, [8 * 599 + 7, 8 * 100]),
    ("d64_gqa8", 2, 8, 1, 64, 128 * 12, 128, 16, 1, [128 * 11 + 100, 5]),
    ("gqa1_odd_chunk", 2, 2, 2, 128, 20 * 30, 20, 5, 2, [20 * 29 + 19, 20 * 3 + 7]),
    ("no_summaries", 2, 2, 1, 128, 32 * 10, 32, 0, 2, [32 * 9 + 4, 32 * 1 + 9]),
    # token-level sliding window of 256 tokens: chunks of one token, a ring of 256 rows
    ("token_window_w256", 3, 4, 2, 128, 2000, 1, 0, 255, [1999, 100, 255]),
], ids=lambda c: c[0])
def test_decode_shapes(case):
    name, B, Hq, Hkv, d, n_cap, c, m, C, positions = case
    run_case(name, B, Hq, Hkv, d, n_cap, c, m, C, positions, seed=len(name))


def test_decode_out_of_range_position_gives_nan_and_reads_nothing():
    p = K.make_params(2, 640, 64, 8, 1, 4, 2, 128)
    s_cap, rows = K.cache_geometry(p)
    q = torch.randn((2, 4, 128), device="cuda").to(torch.bfloat16)
    kc = torch.randn((2, 2, rows, 128), device="cuda").to(torch.bfloat16)
    vc = torch.randn((2, 2, rows, 128), device="cuda").to(torch.bfloat16)
    pos = torch.tensor([100, 640], dtype=torch.int32, device="cuda")
    o, lse = K.ksa_decode_fwd(p, q, kc, vc, pos)
    torch.cuda.synchronize()
    assert torch.isfinite(o[0]).all() and torch.isnan(o[1]).all() and torch.isnan(lse[1]).all()


def long_context_compare(cfg, pos, slabs):
    """One decode step of every sequence of cfg at text position pos, in the default launch configuration; the
    sequences of `slabs` (ranges of eight) are compared with the oracle."""
    c, m, C = cfg.chunk_len, cfg.n_summary, cfg.window_chunks
    n_cap = (pos // c + 1) * c
    say(f"decode parity {cfg.name}: pos {pos} capacity {n_cap}")
    p = K.make_params(cfg.batch, n_cap, c, m, C, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    s_cap, rows = K.cache_geometry(p)
    W = (C + 1) * c
    base = (pos // c - C) * c
    q, k_sum, v_sum, k_txt, v_txt = synth.make_decode_inputs(cfg, s_cap, W, device="cuda")
    k_cache, v_cache = K.pack_cache(p, k_sum, v_sum, k_txt, v_txt, base)
    pos_t = torch.full((cfg.batch,), pos, dtype=torch.int32, device="cuda")
    o, lse = K.ksa_decode_fwd(p, q, k_cache, v_cache, pos_t)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o.float()).all()) and bool(torch.isfinite(lse).all())
    o_gpu, lse_gpu = o.float().cpu().numpy(), lse.cpu().numpy()
    errs, lerrs = [], []
    for b0 in slabs:      # the oracle takes fp32 copies: go eight sequences at a time
        sl = slice(b0, b0 + 8)
        o_ref, lse_ref = O.decode(q[sl].float().cpu().numpy(), k_sum[sl].float().cpu().numpy(),
                                  v_sum[sl].float().cpu().numpy(), k_txt[sl].float().cpu().numpy(),
                                  v_txt[sl].float().cpu().numpy(), [base] * 8, [pos] * 8, c, m, C)
        errs.append(np.abs(o_gpu[sl] - o_ref))
        lerrs.append(np.abs(lse_gpu[sl] - lse_ref))
        say(f"  sequences {b0}..{b0 + 7}: max-abs {errs[-1].max():.3e}")
    err, lerr = np.concatenate(errs), np.concatenate(lerrs)
    say(f"  max-abs {err.max():.3e} mean-abs {err.mean():.3e} lse max-abs {lerr.max():.3e}")
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS and lerr.max() <= LSE_ABS
    return k_cache


def test_decode_128k_context_full_compare():
    """The benchmark workload: batch 64, 32/8 heads, d 128, position 131072+63 (16376 visible summaries +
    128 text rows per KV head), in the launch configuration bench.py times (default split count)."""
    cfg = synth.CONFIGS["decode_128k"]
    long_context_compare(cfg, cfg.decode_pos, range(0, cfg.batch, 8))


def test_decode_1m_context_cache_beyond_4_gib():
    """Position 2^20 + 63: 131 064 visible summaries + 128 text rows per KV head; 72 sequences of 8/2 heads make each
    cache 4.8 GB, so the last sequences lie more than 4 GiB behind the cache's base.  First and last eight sequences
    against the oracle."""
    cfg = synth.KsaConfig("decode_1m", 72, 8, 2, 128, (1 << 20) + 64, 64, 8, 1, seed=4242)
    k_cache = long_context_compare(cfg, (1 << 20) + 63, [0, cfg.batch - 8])
    assert k_cache.stride(0) * 2 * (cfg.batch - 8) > 1 << 32
