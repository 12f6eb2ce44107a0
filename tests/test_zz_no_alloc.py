"""ksa_decode_fwd_static (the entry point that allocates nothing) against ksa_decode_fwd, through the C ABI.

Both run the same kernels; the only difference is where the spans' partial records live (the library's static device
array instead of a caller workspace), so for one n_splits the outputs must agree bit for bit.  Two calls in a row, the
second on a smaller problem, show that records left behind by the first call do not leak into the second.
"""
import sys

import pytest
import torch

import paper_2604_24432_amd as K

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def one_call(B, Hq, Hkv, d, n_cap, c, m, C, positions, n_splits, seed):
    say(f"static-scratch decode: B{B} Hq{Hq} Hkv{Hkv} d{d} cap{n_cap} c{c} m{m} C{C} splits{n_splits}")
    p = K.make_params(B, n_cap, c, m, C, Hq, Hkv, d)
    _, rows = K.cache_geometry(p)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    q = torch.randn((B, Hq, d), device="cuda", generator=gen).to(torch.bfloat16)
    k_cache = torch.randn((B, Hkv, rows, d), device="cuda", generator=gen).to(torch.bfloat16)
    v_cache = torch.randn((B, Hkv, rows, d), device="cuda", generator=gen).to(torch.bfloat16)
    pos = torch.tensor(positions, dtype=torch.int32, device="cuda")
    o_ref, lse_ref = K.ksa_decode_fwd(p, q, k_cache, v_cache, pos, n_splits=n_splits)
    # outputs of the static call are allocated up front and pre-filled, so an unwritten entry would show
    o = torch.full_like(q, 7.0)
    lse = torch.full((B, Hq), 7.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    K.ksa_decode_fwd_static(p, q, k_cache, v_cache, pos, o, lse, n_splits=n_splits)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(o, o_ref)
    assert torch.equal(lse, lse_ref)


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    c, m, C = 64, 8, 1
    # first call: many sequences, several spans each; second call: a smaller problem with fewer, shorter spans
    one_call(8, 32, 8, 128, 64 * 512, c, m, C, [64 * 512 - 1 - 37 * b for b in range(8)], n_splits=5, seed=11)
    one_call(2, 8, 2, 128, 64 * 40, c, m, C, [64 * 40 - 1, 700], n_splits=2, seed=12)
    # the default span count goes through the same path
    one_call(3, 4, 4, 64, 64 * 100, c, m, C, [6399, 64, 0], n_splits=0, seed=13)


def test_static_scratch_limit_is_reported():
    # batch 512 x 32 heads x 16 spans x 130 floats = 136 MB of records: beyond the static array
    p = K.make_params(512, 64 * 64, 64, 8, 1, 32, 8, 128)
    assert K.decode_workspace_bytes(p, 16) > K.KSA_DECODE_STATIC_SCRATCH_BYTES
    q = torch.zeros((512, 32, 128), dtype=torch.bfloat16, device="cuda")
    _, rows = K.cache_geometry(p)
    cache = torch.zeros((512, 8, rows, 128), dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros(512, dtype=torch.int32, device="cuda")
    with pytest.raises(K.KsaError) as e:
        K.ksa_decode_fwd_static(p, q, cache, cache, pos, torch.empty_like(q), n_splits=16)
    assert e.value.status == -6
