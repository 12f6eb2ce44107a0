"""Seeded synthetic inputs for the KSA hot path.

This module only draws random tensors of the right shapes.  It contains none of
the method's arithmetic (no mask, no softmax, no cache addressing), so that the
CPU oracle and the HIP path can both be fed from it without sharing any logic.

The shapes follow the paper's continual-pre-training model (32 query heads,
8 KV heads, head_dim 128; Table "model_config") at context lengths up to 128K
text tokens with compression ratio k = 8.  The tensors are i.i.d. N(0,1)
stand-ins for projected, position-encoded Q/K/V activations: the paper's
training data and weights are not available, and the attention cost depends on
shapes only.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import torch


@dataclass(frozen=True)
class KsaConfig:
    """One workload.  Symbols follow the paper's Eq. 1-3 generalised to m >= 1."""

    name: str
    batch: int            # B
    n_q_heads: int        # Hq  (paper: h)
    n_kv_heads: int       # Hkv (paper: g)
    head_dim: int         # d
    n_text: int           # n, text tokens per sequence
    chunk_len: int        # c, text tokens per chunk
    n_summary: int        # m, summary tokens appended after each chunk
    window_chunks: int    # C, previous chunks whose text stays visible
    seed: int
    key_outlier_frac: float = 0.0   # fraction of augmented K rows scaled by 8
    decode_pos: int = -1            # text index of the new token (decode only)

    @property
    def n_chunks(self) -> int:
        return self.n_text // self.chunk_len

    @property
    def aug_len(self) -> int:
        # rows of the generated tensors: every text token plus the summary tokens of the whole chunks
        return self.n_text + self.n_chunks * self.n_summary

    @property
    def compress_ratio(self) -> int:
        return self.chunk_len // self.n_summary if self.n_summary else 0

    def scaled(self, **kw) -> "KsaConfig":
        return replace(self, **kw)


CONFIGS: Dict[str, KsaConfig] = {
    # Tiny: 512 text tokens, chunks of 64, 8 summaries per chunk -> L = 576.
    "tiny": KsaConfig("tiny", 1, 1, 1, 64, 512, 64, 8, 1, seed=0),
    "prefill_4k": KsaConfig("prefill_4k", 2, 32, 8, 128, 4096, 64, 8, 1, seed=2000),
    "prefill_32k": KsaConfig("prefill_32k", 1, 32, 8, 128, 32768, 128, 16, 1, seed=3000,
                             key_outlier_frac=0.01),
    "prefill_128k": KsaConfig("prefill_128k", 1, 32, 8, 128, 131072, 64, 8, 1, seed=4000),
    # Decode: one new text token at text index 131072 + 63 (the last slot of chunk 2048),
    # 16384 resident summaries (chunks 0..2047).
    "decode_128k": KsaConfig("decode_128k", 64, 32, 8, 128, 131072, 64, 8, 1, seed=5000,
                             decode_pos=131072 + 63),
}


def _normal_bf16(shape, seed: int, device: str, block_rows: int = 1 << 14) -> torch.Tensor:
    """N(0,1) drawn in fp32 and rounded to bf16 (round-to-nearest-even).

    Drawn in slabs along dim 0 so that the fp32 staging buffer stays small.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    out = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    flat = out.view(shape[0], -1) if len(shape) > 1 else out.view(-1, 1)
    rows = flat.shape[0]
    step = max(1, min(rows, block_rows * 4096 // max(1, flat.shape[1])))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        slab = torch.randn((r1 - r0, flat.shape[1]), generator=gen, device=dev, dtype=torch.float32)
        flat[r0:r1] = slab.to(torch.bfloat16)
    return out


def make_prefill_inputs(cfg: KsaConfig, device: str = "cpu") -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Q [B, L, Hq, d], K and V [B, L, Hkv, d], bf16, over the augmented sequence.

    Row a of the augmented sequence is a text or a summary position; both kinds
    are drawn from the same distribution.  With key_outlier_frac > 0 a seeded
    random subset of round(frac * L) augmented rows has its K row (all KV heads)
    multiplied by 8, which makes some softmax rows nearly one-hot.
    """
    B, L = cfg.batch, cfg.aug_len
    # dim 0 is the slab dimension of _normal_bf16, so put L first and transpose after
    q = _normal_bf16((L, B, cfg.n_q_heads, cfg.head_dim), cfg.seed + 0, device).transpose(0, 1).contiguous()
    k = _normal_bf16((L, B, cfg.n_kv_heads, cfg.head_dim), cfg.seed + 1, device).transpose(0, 1).contiguous()
    v = _normal_bf16((L, B, cfg.n_kv_heads, cfg.head_dim), cfg.seed + 2, device).transpose(0, 1).contiguous()
    if cfg.key_outlier_frac > 0.0:
        gen = torch.Generator(device="cpu")
        gen.manual_seed(cfg.seed + 3)
        n_out = int(round(cfg.key_outlier_frac * L))
        rows = torch.randperm(L, generator=gen)[:n_out].to(k.device)
        k[:, rows] = k[:, rows] * 8  # exact in bf16
    return q, k, v


def make_upstream_gradient(cfg: KsaConfig, device: str = "cpu") -> torch.Tensor:
    """dLoss/dO [B, L, Hq, d], bf16, N(0, 1): what a following layer would hand to the backward pass."""
    B, L = cfg.batch, cfg.aug_len
    return _normal_bf16((L, B, cfg.n_q_heads, cfg.head_dim), cfg.seed + 7, device).transpose(0, 1).contiguous()


def make_decode_inputs(cfg: KsaConfig, n_summary_rows: int, n_text_rows: int, device: str = "cpu"):
    """Logical (order-free) decode operands, bf16.

    q      [B, Hq, d]                  the new token's query
    k_sum  [B, Hkv, n_summary_rows, d] key of summary ordinal u (chunk u // m, slot u % m)
    v_sum  same
    k_txt  [B, Hkv, n_text_rows, d]    key of text index text_base + t (text_base is the caller's)
    v_txt  same
    How these rows are placed in a physical cache is not decided here.
    """
    B, Hkv, d = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    q = _normal_bf16((B, cfg.n_q_heads, d), cfg.seed + 0, device)
    k_sum = _normal_bf16((B, Hkv, n_summary_rows, d), cfg.seed + 1, device)
    v_sum = _normal_bf16((B, Hkv, n_summary_rows, d), cfg.seed + 2, device)
    k_txt = _normal_bf16((B, Hkv, n_text_rows, d), cfg.seed + 4, device)
    v_txt = _normal_bf16((B, Hkv, n_text_rows, d), cfg.seed + 5, device)
    return q, k_sum, v_sum, k_txt, v_txt


def sample_rows(cfg: KsaConfig, n_random: int, seed_offset: int = 7) -> torch.Tensor:
    """Augmented row indices for sampled parity checks at large sizes: every row of the
    first three and last three chunks plus n_random seeded random rows, sorted, unique."""
    w = cfg.chunk_len + cfg.n_summary
    L = cfg.aug_len
    head = torch.arange(0, min(L, 3 * w))
    tail = torch.arange(max(0, L - 3 * w), L)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(cfg.seed + seed_offset)
    rnd = torch.randint(0, L, (n_random,), generator=gen)
    return torch.unique(torch.cat([head, tail, rnd]))
