"""Pins for the oracle's gradients (CPU only).

The gradients are checked against things other than the oracle's own backward formula: central differences of the
oracle's forward pass (itself pinned in test_oracle_attention.py), torch's automatic differentiation of a masked
softmax written with library calls, closed forms for degenerate rows, and consistency of the row-list mode.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ksa_oracle as O


def grid_values(shape, rng, step=2.0 ** -6, span=96):
    """Random values on a coarse binary grid, so that x +- h is exact in float32 for the steps used below."""
    return (rng.integers(-span, span + 1, size=shape) * step).astype(np.float32)


def loss_of(q, k, v, g, n, c, m, Cw, flags):
    o, _ = O.prefill(q, k, v, n=n, c=c, m=m, Cw=Cw, flags=flags)
    return float((o * g.astype(np.float64)).sum())


def fourth_order_difference(f, x, idx, h):
    """d f / d x[idx] from f(x +- h) and f(x +- h/2): error O(h^4)."""
    def at(delta):
        y = x.copy()
        y[idx] += np.float32(delta)
        assert float(y[idx]) == float(x[idx]) + delta     # exact in float32
        return f(y)
    return (8.0 * (at(h / 2) - at(-h / 2)) - (at(h) - at(-h))) / (6.0 * h)


@pytest.mark.parametrize("n,c,m,Cw,flags,Hq,Hkv", [
    (10, 4, 1, 0, 0, 2, 1),      # ragged tail, window of the own chunk only, grouped heads
    (12, 4, 2, 1, 0, 2, 2),      # two summary tokens per chunk: a summary sees its earlier sibling
    (12, 4, 2, 1, 1, 1, 1),      # ... and with the self-only flag
    (9, 3, 1, 1, 0, 2, 1),
    (8, 8, 0, 0, 0, 1, 1),       # no summaries: dense causal
])
def test_gradients_match_central_differences_of_the_forward_oracle(n, c, m, Cw, flags, Hq, Hkv):
    d, B = 4, 1
    rng = np.random.default_rng(100 + n + 7 * m + Cw)
    L = O.aug_len(n, c, m)
    q = grid_values((B, L, Hq, d), rng)
    k = grid_values((B, L, Hkv, d), rng)
    v = grid_values((B, L, Hkv, d), rng)
    g = grid_values((B, L, Hq, d), rng)
    dq, dk, dv = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw, flags=flags)
    h = 2.0 ** -5
    worst = 0.0
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        f = {"q": lambda y: loss_of(y, k, v, g, n, c, m, Cw, flags),
             "k": lambda y: loss_of(q, y, v, g, n, c, m, Cw, flags),
             "v": lambda y: loss_of(q, k, y, g, n, c, m, Cw, flags)}[name]
        for idx in np.ndindex(x.shape):
            num = fourth_order_difference(f, x, idx, h)
            worst = max(worst, abs(num - grad[idx]))
            assert abs(num - grad[idx]) < 2e-6 * max(1.0, abs(grad[idx])), (name, idx, num, grad[idx])
    assert worst < 1e-5


def torch_masked_attention_grads(q, k, v, g, mask, scale):
    """Autograd through softmax(QK^T scale + mask) V written with library calls, fp64."""
    Hq, Hkv = q.shape[2], k.shape[2]
    tq = torch.from_numpy(q).double().requires_grad_(True)
    tk = torch.from_numpy(k).double().requires_grad_(True)
    tv = torch.from_numpy(v).double().requires_grad_(True)
    kk = tk.repeat_interleave(Hq // Hkv, dim=2)
    vv = tv.repeat_interleave(Hq // Hkv, dim=2)
    s = torch.einsum("blhd,bmhd->bhlm", tq, kk) * scale
    s = s.masked_fill(~torch.from_numpy(mask.astype(bool))[None, None], float("-inf"))
    o = torch.einsum("bhlm,bmhd->blhd", torch.softmax(s, dim=-1), vv)
    (o * torch.from_numpy(g).double()).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("n,c,m,Cw,flags,Hq,Hkv,d", [
    (96, 8, 2, 1, 0, 4, 2, 16),
    (100, 8, 1, 3, 0, 4, 1, 8),     # ragged tail, paper-like m = 1
    (64, 16, 4, 0, 1, 2, 2, 8),
    (70, 70, 0, 0, 0, 2, 1, 16),    # dense causal
    (64, 4, 0, 2, 0, 2, 2, 8),      # chunk-aligned sliding window, no summaries
])
def test_gradients_match_autograd_of_a_masked_softmax(n, c, m, Cw, flags, Hq, Hkv, d):
    B = 2
    rng = np.random.default_rng(n * 31 + c)
    L = O.aug_len(n, c, m)
    q = rng.standard_normal((B, L, Hq, d)).astype(np.float32)
    k = rng.standard_normal((B, L, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((B, L, Hkv, d)).astype(np.float32)
    g = rng.standard_normal((B, L, Hq, d)).astype(np.float32)
    mask = O.mask(n, c, m, Cw, flags)
    dq, dk, dv = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw, flags=flags)
    rq, rk, rv = torch_masked_attention_grads(q, k, v, g, mask, 1 / math.sqrt(d))
    assert np.abs(dq - rq).max() < 1e-11
    assert np.abs(dk - rk).max() < 1e-11
    assert np.abs(dv - rv).max() < 1e-11


def test_explicit_scale_is_used():
    n, c, m, Cw, B, Hq, Hkv, d = 24, 4, 1, 1, 1, 2, 1, 8
    rng = np.random.default_rng(5)
    L = O.aug_len(n, c, m)
    q, g = (rng.standard_normal((B, L, Hq, d)).astype(np.float32) for _ in range(2))
    k, v = (rng.standard_normal((B, L, Hkv, d)).astype(np.float32) for _ in range(2))
    dq, dk, dv = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw, scale=0.37)
    rq, rk, rv = torch_masked_attention_grads(q, k, v, g, O.mask(n, c, m, Cw), 0.37)
    assert np.abs(dq - rq).max() < 1e-11 and np.abs(dk - rk).max() < 1e-11 and np.abs(dv - rv).max() < 1e-11


def test_single_token_closed_form():
    # one text token: its only key is itself, p = 1, so dQ = dK = 0 and dV is the upstream gradient summed over
    # the query heads of the group
    B, Hq, Hkv, d = 1, 4, 2, 8
    rng = np.random.default_rng(3)
    q, g = (rng.standard_normal((B, 1, Hq, d)).astype(np.float32) for _ in range(2))
    k, v = (rng.standard_normal((B, 1, Hkv, d)).astype(np.float32) for _ in range(2))
    dq, dk, dv = O.prefill_bwd(q, k, v, g, n=1, c=4, m=1, Cw=1)
    assert np.abs(dq).max() == 0.0 and np.abs(dk).max() == 0.0
    want = g.astype(np.float64).reshape(B, 1, Hkv, Hq // Hkv, d).sum(axis=3)
    assert np.abs(dv - want).max() < 1e-15


def test_equal_keys_give_uniform_weights_closed_form():
    # all keys equal: scores are equal, p_ij = 1 / (visible keys of row i), dS = p (g.v - g.v) = 0, hence
    # dQ = dK = 0 and dV_j = sum over the rows that see j of G_i / count_i
    n, c, m, Cw, d = 12, 4, 1, 1, 4
    L = O.aug_len(n, c, m)
    rng = np.random.default_rng(4)
    q, g = (rng.standard_normal((1, L, 1, d)).astype(np.float32) for _ in range(2))
    k = np.tile(rng.standard_normal((1, 1, 1, d)).astype(np.float32), (1, L, 1, 1))
    v = np.tile(rng.standard_normal((1, 1, 1, d)).astype(np.float32), (1, L, 1, 1))
    dq, dk, dv = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw)
    assert np.abs(dq).max() < 1e-13 and np.abs(dk).max() < 1e-13
    mask = O.mask(n, c, m, Cw).astype(np.float64)
    p = mask / mask.sum(axis=1, keepdims=True)
    want = p.T @ g[0, :, 0, :].astype(np.float64)
    assert np.abs(dv[0, :, 0, :] - want).max() < 1e-13


def test_row_lists_select_rows_of_the_full_result():
    n, c, m, Cw, B, Hq, Hkv, d = 40, 8, 2, 1, 2, 4, 2, 8
    rng = np.random.default_rng(6)
    L = O.aug_len(n, c, m)
    q, g = (rng.standard_normal((B, L, Hq, d)).astype(np.float32) for _ in range(2))
    k, v = (rng.standard_normal((B, L, Hkv, d)).astype(np.float32) for _ in range(2))
    dq, dk, dv = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw)
    q_rows, k_rows = [0, 9, 17, L - 1], [3, 8, 9, 30, L - 2]
    sq, sk, sv = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw, q_rows=q_rows, k_rows=k_rows)
    assert np.abs(sq - dq[:, q_rows]).max() < 1e-13
    assert np.abs(sk - dk[:, k_rows]).max() < 1e-13 and np.abs(sv - dv[:, k_rows]).max() < 1e-13
    only_q, ek, ev = O.prefill_bwd(q, k, v, g, n=n, c=c, m=m, Cw=Cw, q_rows=q_rows, k_rows=[])
    assert ek.shape[1] == 0 and ev.shape[1] == 0 and np.array_equal(only_q, sq)


def test_bad_arguments_are_rejected():
    x = np.zeros((1, 5, 2, 4), np.float32)
    with pytest.raises(ValueError):
        O.prefill_bwd(x, x[:, :, :1], x[:, :, :1], x, n=4, c=4, m=1, Cw=0, q_rows=[5])
    with pytest.raises(ValueError):
        O.prefill_bwd(x, x[:, :, :1], x[:, :, :1], x, n=4, c=4, m=1, Cw=0, k_rows=[-1])
