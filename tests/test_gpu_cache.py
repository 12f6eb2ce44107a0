"""GPU tests of the cache lifecycle (run with -m gpu on an MI355X), through the C ABI.

Placement is data movement and must be bit-exact against the cache geometry written out here from its
definition.  The generate loop (prefill hand-off, then one text step per token and one summary step per summary
of every completed chunk) is checked against the oracle of the prefill path: the attention row of an augmented
position depends only on the keys visible to it, so a decode step must reproduce the oracle's row of that
position over the whole sequence."""
import sys

import numpy as np
import pytest
import torch

import paper_2604_24432_amd as K
from paper_2604_24432_amd import synth
from oracle import ksa_oracle as O

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS, LSE_ABS = 2e-2, 2e-3, 1e-4
POISON = 0x7F5A   # bit pattern of untouched cache rows


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def bits(t):
    return t.view(torch.int16).cpu().numpy()


def aug_text(i, c, m):
    return (i // c) * (c + m) + i % c


def aug_summary(u, c, m):
    return (u // m) * (c + m) + c + u % m


def poisoned_caches(p):
    s_cap, rows = K.cache_geometry(p)
    shape = (p.batch, p.n_kv_heads, rows, p.head_dim)
    kc = torch.full(shape, POISON, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    vc = torch.full(shape, POISON, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    return kc, vc


def expected_fill(p, n_prefill, k):
    """Cache content after the hand-off, from the geometry: summary ordinal u at row u; text index i of chunk j at
    row s_cap + (j mod (C+1)) c + i mod c, for the last min(J, C+1) chunks; everything else untouched."""
    c, m, Cw = p.chunk_len, p.n_summary, p.window_chunks
    s_cap, rows = K.cache_geometry(p)
    kb = bits(k)                                     # [B, L, Hkv, d]
    out = np.full((p.batch, p.n_kv_heads, rows, p.head_dim), POISON, dtype=np.int16)
    J, tail = n_prefill // c, n_prefill % c
    for u in range(J * m):
        out[:, :, u] = kb[:, aug_summary(u, c, m)]
    # the ring has C + 1 slots; an incomplete last chunk occupies one of them
    first = max(0, J - Cw) if tail else max(0, J - (Cw + 1))
    for i in range(first * c, n_prefill):
        out[:, :, s_cap + ((i // c) % (Cw + 1)) * c + i % c] = kb[:, aug_text(i, c, m)]
    return out


FILL_CASES = [  # (B, Hkv, d, n_cap, c, m, C, n_prefill)
    (2, 2, 64, 16 * 16, 16, 2, 1, 5 * 16),
    (1, 2, 128, 12 * 64, 64, 8, 1, 7 * 64),
    (2, 1, 128, 10 * 32, 32, 4, 3, 2 * 32),      # fewer chunks than ring slots
    (1, 2, 64, 10 * 8, 8, 1, 2, 10 * 8),         # the paper's m = 1 form, cache filled to capacity
    (1, 1, 64, 6 * 16, 16, 0, 1, 4 * 16),        # no summaries
    (1, 1, 64, 6 * 16, 16, 2, 1, 0),             # nothing prefilled
    (2, 2, 64, 16 * 16, 16, 2, 1, 5 * 16 + 7),   # an incomplete last chunk
    (1, 2, 128, 12 * 64, 64, 8, 2, 64 + 1),      # ... right after a chunk boundary
    (1, 1, 64, 6 * 16, 16, 2, 1, 9),             # ... and nothing else
]


@pytest.mark.parametrize("case", FILL_CASES)
def test_cache_from_prefill_is_the_documented_placement(case):
    B, Hkv, d, n_cap, c, m, Cw, n_prefill = case
    say(f"cache_from_prefill {case}")
    p = K.make_params(B, n_cap, c, m, Cw, Hkv, Hkv, d)
    L = n_prefill // c * (c + m) + n_prefill % c
    g = torch.Generator().manual_seed(11)
    k = torch.randn((B, L, Hkv, d), generator=g).to(torch.bfloat16).cuda()
    v = torch.randn((B, L, Hkv, d), generator=g).to(torch.bfloat16).cuda()
    kc, vc = poisoned_caches(p)
    K.ksa_cache_from_prefill(p, n_prefill, k, v, kc, vc)
    torch.cuda.synchronize()
    assert np.array_equal(bits(kc), expected_fill(p, n_prefill, k))
    assert np.array_equal(bits(vc), expected_fill(p, n_prefill, v))


def test_cache_from_prefill_strided_source():
    B, Hkv, d, n_cap, c, m, Cw, n_prefill = 2, 2, 64, 8 * 16, 16, 2, 1, 4 * 16
    p = K.make_params(B, n_cap, c, m, Cw, Hkv, Hkv, d)
    L = n_prefill // c * (c + m)
    g = torch.Generator().manual_seed(12)
    big = torch.randn((B, L, 2 * Hkv, d), generator=g).to(torch.bfloat16).cuda()
    k, v = big[:, :, ::2], big[:, :, 1::2]           # head stride 2 d
    kc, vc = poisoned_caches(p)
    K.ksa_cache_from_prefill(p, n_prefill, k, v, kc, vc)
    torch.cuda.synchronize()
    assert np.array_equal(bits(kc), expected_fill(p, n_prefill, k.contiguous()))
    assert np.array_equal(bits(vc), expected_fill(p, n_prefill, v.contiguous()))


def test_cache_append_writes_one_row_per_sequence():
    B, Hkv, d, n_cap, c, m, Cw = 6, 2, 128, 10 * 16, 16, 2, 2
    p = K.make_params(B, n_cap, c, m, Cw, Hkv, Hkv, d)
    s_cap, rows = K.cache_geometry(p)
    g = torch.Generator().manual_seed(13)
    k_new = torch.randn((B, Hkv, d), generator=g).to(torch.bfloat16).cuda()
    v_new = torch.randn((B, Hkv, d), generator=g).to(torch.bfloat16).cuda()
    # text rows: two sequences outside the cache are skipped
    pos = [0, 17, 16 * 3 + 15, n_cap - 1, -1, n_cap]
    kc, vc = poisoned_caches(p)
    K.ksa_cache_append(p, K.KSA_ROW_TEXT, k_new, v_new, torch.tensor(pos, dtype=torch.int32).cuda(), kc, vc)
    torch.cuda.synchronize()
    want_k = np.full((B, Hkv, rows, d), POISON, np.int16)
    want_v = want_k.copy()
    for b, i in enumerate(pos):
        if 0 <= i < n_cap:
            r = s_cap + ((i // c) % (Cw + 1)) * c + i % c
            want_k[b, :, r], want_v[b, :, r] = bits(k_new)[b], bits(v_new)[b]
    assert np.array_equal(bits(kc), want_k) and np.array_equal(bits(vc), want_v)
    # summary rows
    ordn = [0, 1, 5, s_cap - 1, -3, s_cap]
    kc, vc = poisoned_caches(p)
    K.ksa_cache_append(p, K.KSA_ROW_SUMMARY, k_new, v_new, torch.tensor(ordn, dtype=torch.int32).cuda(), kc, vc)
    torch.cuda.synchronize()
    want_k = np.full((B, Hkv, rows, d), POISON, np.int16)
    want_v = want_k.copy()
    for b, u in enumerate(ordn):
        if 0 <= u < s_cap:
            want_k[b, :, u], want_v[b, :, u] = bits(k_new)[b], bits(v_new)[b]
    assert np.array_equal(bits(kc), want_k) and np.array_equal(bits(vc), want_v)


LOOP_CASES = [  # (B, Hq, Hkv, d, c, m, C, tokens prefilled, tokens in total, flags)
    (2, 4, 2, 64, 16, 2, 1, 3 * 16, 8 * 16, 0),
    (2, 4, 2, 64, 16, 2, 1, 3 * 16, 8 * 16, K.KSA_FLAG_SUMMARY_SELF_ONLY),
    (1, 8, 2, 128, 32, 4, 2, 32, 6 * 32, 0),
    (1, 2, 2, 128, 8, 1, 3, 0, 12 * 8, 0),        # the paper's m = 1 form, nothing prefilled
    (2, 4, 2, 64, 16, 2, 1, 3 * 16 + 5, 7 * 16 + 9, 0),   # hand-off inside a chunk, sequence ends inside a chunk
]


@pytest.mark.parametrize("case", LOOP_CASES)
def test_generate_loop_matches_the_prefill_oracle(case):
    B, Hq, Hkv, d, c, m, Cw, n0, n, flags = case
    say(f"generate loop {case}")
    cfg = synth.KsaConfig("loop", B, Hq, Hkv, d, n, c, m, Cw, seed=77)
    q, k, v = (x.cuda() for x in synth.make_prefill_inputs(cfg))       # [B, L, H, d] over the whole sequence
    p = K.make_params(B, n, c, m, Cw, Hq, Hkv, d, flags=flags)
    kc, vc = poisoned_caches(p)
    L0 = n0 // c * (c + m) + n0 % c
    K.ksa_cache_from_prefill(p, n0, k[:, :L0].contiguous(), v[:, :L0].contiguous(), kc, vc)
    rows, outs, lses = [], [], []

    def step(fn, kind, a_row, pos_value):
        pos = torch.full((B,), pos_value, dtype=torch.int32, device="cuda")
        K.ksa_cache_append(p, kind, k[:, a_row].contiguous(), v[:, a_row].contiguous(), pos, kc, vc)
        o, lse = fn(p, q[:, a_row].contiguous(), kc, vc, pos)
        rows.append(a_row), outs.append(o.float().cpu().numpy()), lses.append(lse.cpu().numpy())

    for i in range(n0, n):
        step(K.ksa_decode_fwd, K.KSA_ROW_TEXT, aug_text(i, c, m), i)
        if i % c == c - 1:                                            # chunk complete: its m summary steps
            for slot in range(m):
                u = (i // c) * m + slot
                step(K.ksa_decode_summary_fwd, K.KSA_ROW_SUMMARY, aug_summary(u, c, m), u)
    torch.cuda.synchronize()
    o_ref, lse_ref = O.prefill(q.float().cpu().numpy(), k.float().cpu().numpy(), v.float().cpu().numpy(), n, c, m, Cw,
                               flags=flags, rows=rows)                # [B, R, Hq, d], [B, Hq, R]
    o_gpu = np.stack(outs, axis=1).astype(np.float64)                 # [B, R, Hq, d]
    lse_gpu = np.stack(lses, axis=2).astype(np.float64)               # [B, Hq, R]
    err, lerr = np.abs(o_gpu - o_ref), np.abs(lse_gpu - lse_ref)
    say(f"  {len(rows)} steps: max-abs {err.max():.3e} mean-abs {err.mean():.3e} lse max-abs {lerr.max():.3e}")
    assert np.isfinite(o_gpu).all() and np.isfinite(lse_gpu).all()
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS and lerr.max() <= LSE_ABS
    # the cache now holds every summary and the text of the window: same as a hand-off of the whole sequence, except
    # that behind an incomplete last chunk its slot still holds the rest of the chunk it is overwriting
    s_cap, _ = K.cache_geometry(p)
    keep = np.ones(bits(kc).shape[2], dtype=bool)
    if n % c:
        slot0 = s_cap + ((n // c) % (Cw + 1)) * c
        keep[slot0 + n % c: slot0 + c] = False
    assert np.array_equal(bits(kc)[:, :, keep], expected_fill(p, n, k)[:, :, keep])
    assert np.array_equal(bits(vc)[:, :, keep], expected_fill(p, n, v)[:, :, keep])
