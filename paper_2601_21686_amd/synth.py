"""Seeded synthetic inputs shaped like the paper's motivating workload.

Shared by the GPU tests, the oracle tests and the benchmark.  This module only
draws random numbers and formats them as bf16; none of the method's arithmetic
(projection, attention, rank selection) lives here.

Recipe
  * bases: Q factor (R_ii > 0) of a float64 QR of a seeded N(0,1) d_h x r
    matrix, one per KV head -- the paper obtains its bases the same way, as the
    Q factor of a dense matrix (Sec. 3.3, Eqs. 13-14) -- then rounded to bf16.
    The rounded bits ARE the basis both sides use.
  * raw keys / values: N(0,1) times a per-channel scale s_i = i^-0.7
    (i = 1..d_h), with 4 seeded outlier channels per KV head multiplied by 8;
    rounded to bf16.  Spectral decay is what makes a low-rank cache plausible
    (Sec. 1); outlier channels are the known KV-cache pathology (Sec. 4.3).
  * queries: N(0,1), bf16.
  * per-layer ranks (32-layer stack): r_K and r_V drawn independently by seed
    from {32, 48, 64, 96, 128}, as the paper's selector produces ranks that
    vary across layers with r_K != r_V (App. D).

The five workloads below stand in for Llama3-8B / Llama2-7B activations and
learned bases, which need the paper's models and calibration data.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

HEAD_DIM = 128
RANK_CHOICES = (32, 48, 64, 96, 128)


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    n_ctx: int          # tokens in the cache when decode attends (after appends)
    r_k: int            # 0 = drawn per layer
    r_v: int
    n_layers: int
    decode_steps: int
    append_chunk: int   # tokens appended in one call before the timed decode
    head_dim: int = HEAD_DIM


WORKLOADS = {
    # single layer, batch 1, context 1024, 16-token append then one decode step
    "b1_ctx1k_r64": Workload("b1_ctx1k_r64", 1, 32, 8, 1024, 64, 64, 1, 1, 16),
    # single layer, batch 4, context 32768, 64 decode steps each appending a token
    "b4_ctx32k_r64": Workload("b4_ctx32k_r64", 4, 32, 8, 32768, 64, 64, 1, 64, 1),
    # 32-layer stack, batch 4, context 32768, seeded heterogeneous ranks
    "b4_ctx32k_L32_mixed": Workload("b4_ctx32k_L32_mixed", 4, 32, 8, 32768, 0, 0, 32, 1, 1),
    # 4096-token chunk appended onto 28672 cached tokens, then one decode step
    "b8_chunk4k_r48_80": Workload("b8_chunk4k_r48_80", 8, 32, 8, 32768, 48, 80, 1, 1, 4096),
    # multi-head (no grouping), batch 8, context 131072, 32 decode steps
    "b8_ctx128k_mha_r64_96": Workload("b8_ctx128k_mha_r64_96", 8, 32, 32, 131072, 64, 96, 1, 32, 1),
}


def stable_seed(*parts) -> int:
    """Deterministic 63-bit seed from a tuple of ints/strings."""
    h = 1469598103934665603
    for p in parts:
        for byte in str(p).encode() + b"/":
            h = ((h ^ byte) * 1099511628211) & ((1 << 64) - 1)
    return h & ((1 << 63) - 1)


# ---- bf16 plumbing -------------------------------------------------------


def torch_bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns (host)."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_torch_bf16(bits: np.ndarray, device="cpu") -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 tensor on `device`."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(torch.bfloat16).to(device)


def f64_to_torch_bf16(x: np.ndarray, device="cpu") -> torch.Tensor:
    """float64 values that are float32-representable or not: go through
    float32 then bf16 (used only to format generated inputs)."""
    return torch.from_numpy(np.asarray(x, np.float64)).to(torch.float32).to(torch.bfloat16).to(device)


# ---- generators ----------------------------------------------------------


def orthonormal_bases(seed: int, n_bases: int, head_dim: int, rank: int):
    """n_bases column-orthonormal [head_dim, rank] matrices.

    Returns (float64 array [n_bases, head_dim, rank] with exactly orthonormal
    columns up to float64 rounding, bf16 tensor of the same shape)."""
    rng = np.random.default_rng(seed)
    out = np.empty((n_bases, head_dim, rank), np.float64)
    for i in range(n_bases):
        a = rng.standard_normal((head_dim, rank))
        qf, rf = np.linalg.qr(a)
        out[i] = qf * np.sign(np.diag(rf))[None, :]
    return out, f64_to_torch_bf16(out)


def channel_scales(seed: int, n_kv_heads: int, head_dim: int) -> torch.Tensor:
    """float32 [n_kv_heads, head_dim]: i^-0.7 decay, 4 outlier channels x8 per head."""
    rng = np.random.default_rng(seed)
    s = np.arange(1, head_dim + 1, dtype=np.float64) ** -0.7
    out = np.tile(s, (n_kv_heads, 1))
    for h in range(n_kv_heads):
        out[h, rng.choice(head_dim, size=4, replace=False)] *= 8.0
    return torch.from_numpy(out).to(torch.float32)


def kv_activations(seed: int, batch: int, n_tokens: int, n_kv_heads: int,
                   head_dim: int, scales: torch.Tensor, device="cpu") -> torch.Tensor:
    """bf16 [batch, n_tokens, n_kv_heads, head_dim] raw keys (or values)."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    z = torch.randn((batch, n_tokens, n_kv_heads, head_dim), generator=g,
                    device=device, dtype=torch.float32)
    return (z * scales.to(device)[None, None]).to(torch.bfloat16)


def queries(seed: int, batch: int, n_q_heads: int, head_dim: int, device="cpu") -> torch.Tensor:
    """bf16 [batch, n_q_heads, head_dim]."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn((batch, n_q_heads, head_dim), generator=g, device=device,
                       dtype=torch.float32).to(torch.bfloat16)


def chunk_queries(seed: int, batch: int, n_tokens: int, n_q_heads: int, width: int, device="cpu") -> torch.Tensor:
    """bf16 [batch, n_tokens, n_q_heads, width]: the queries of a chunk of new tokens."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn((batch, n_tokens, n_q_heads, width), generator=g, device=device,
                       dtype=torch.float32).to(torch.bfloat16)


def layer_rank_draw(seed: int, n_layers: int):
    """Per-layer (r_K, r_V) drawn independently from RANK_CHOICES."""
    rng = np.random.default_rng(seed)
    rk = rng.choice(RANK_CHOICES, size=n_layers)
    rv = rng.choice(RANK_CHOICES, size=n_layers)
    return [int(x) for x in rk], [int(x) for x in rv]


def selection_bases(seed: int, n_bases: int, head_dim: int, rank: int):
    """Signed selection matrices (columns of +-identity): projection then copies
    `rank` channels exactly, which makes the cache bit-checkable.  Returns
    (float64 [n_bases, head_dim, rank], bf16 tensor, chosen channel indices
    [n_bases, rank], signs [n_bases, rank])."""
    rng = np.random.default_rng(seed)
    out = np.zeros((n_bases, head_dim, rank), np.float64)
    idx = np.empty((n_bases, rank), np.int64)
    sgn = np.empty((n_bases, rank), np.float64)
    for i in range(n_bases):
        idx[i] = rng.permutation(head_dim)[:rank]
        sgn[i] = rng.choice([-1.0, 1.0], size=rank)
        out[i, idx[i], np.arange(rank)] = sgn[i]
    return out, f64_to_torch_bf16(out), idx, sgn
