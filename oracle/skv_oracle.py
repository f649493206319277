"""CPU float64 oracle for attention over a low-rank projected KV cache.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what
the GPU library must compute.  It may be imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg, and by nothing else: the
product path never calls it and shares no code, table or constant with it.

Everything below is the paper's definition written out with numpy float64:

  * compression            K_down = K P_K, V_down = V P_V      (Sec. 2.1, Eq. 1)
  * reconstruction         K_tilde = K_down P_K^T, same for V  (Sec. 2.1 Eq. 2; Sec. 3.2 Eq. 7)
  * per-head attention     softmax(Q K^T / sqrt(d_h)) V        (App. A.1, Eq. 18)
  * grouped-query heads    Eq. 18 per query head, several query heads
                           reading one KV head                 (App. A.1)
  * cache-size ratio       CR = (r_K + r_V) / (2 d_h)          (Sec. 2.1, Eq. 3)
  * sequential budgeted rank selection                         (Sec. 3.5, Eqs. 15-17; App. B, Alg. 2)
  * asymmetric integer quantisation of the compressed cache    (Sec. 4.3; 8 bits, group 64)
  * the folded-weights variant: attention in the compressed space (Sec. 3.4 "Overheads")
  * a chunk of queries over the compressed cache (Eq. 18 with T > 1, causal mask)
  * per-sequence context lengths (Eq. 18 per sequence of a mixed batch)
  * a paged cache: the same rows found through a block table (addressing only)
  * bases from predicted matrices: orthonormal factor of a QR, leading r columns
                                                               (Sec. 3.3 Eqs. 13-14; Sec. 3.2 Eq. 6)

Readings taken where the paper is silent (all listed in the design notes):
the softmax scale uses the ORIGINAL head dimension d_h, never the rank; no
mean is subtracted before projecting; query head h reads KV head h // G with
G = H_Q / H_KV; the cache stores bf16 (round to nearest, ties to even, one
rounding straight from the float64 sum); the decode query attends rows
[0, n_ctx) of the cache, its own freshly appended row included.

bf16 tensors cross this module's boundary as numpy uint16 bit patterns so
that oracle and GPU consume identical bytes.

Pins (tests/test_oracle_*.py): full rank with a square orthogonal basis equals
uncompressed attention computed by an independent brute force; P^T P = I and
P P^T P = P; invariance under a rotation of the basis inside its span;
in-span inputs are reproduced exactly; n = 1 and uniform-score closed forms;
the definition form equals the factored form; a pure-Python brute force on a
tiny case; the library scaled-dot-product routine when P = I; the paper's
printed 16 GB cache-size example; budget invariants and an exhaustive check
of the greedy selector; for the quantiser: on-grid inputs are recovered exactly,
the round-trip error bound, flat groups, library rounding, and the invariance
of the output to the key zero point; for the chunk form: the library's causal
attention (with and without a cached prefix, off-by-one masks rejected), a
pure-Python brute force and the first-token closed form; for per-sequence
lengths: the library's attention under a key-padding mask; for the paged
cache: a hand-labelled pool and table, the identity table, and invariance of
every result under a relabelling of the pool's pages; for the basis
construction: the three properties that make the factor unique (orthonormal
columns, Q R = A, R upper triangular with positive diagonal), a hand-computed
2 x 2 case and the projector onto the span of A's leading columns.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

# --------------------------------------------------------------------------
# bf16 <-> float64 (own helpers; storage precision per the reading above)
# --------------------------------------------------------------------------


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Exact value of each bf16 bit pattern (uint16) as float64."""
    b = np.asarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("bf16 bit patterns must be uint16")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x) -> np.ndarray:
    """Round float64 to bf16 (8 significant bits, float32 exponent range),
    nearest-even, in ONE rounding; returns uint16 bit patterns.  Finite inputs."""
    x = np.asarray(x, dtype=np.float64)
    if not np.all(np.isfinite(x)):
        raise ValueError("oracle rounding is defined for finite values only")
    mant, expo = np.frexp(x)                    # x = mant * 2**expo, 0.5 <= |mant| < 1
    e = expo - 1                                # x = (1.f) * 2**e
    e = np.maximum(e, -126)                     # below 2**-126: subnormal spacing
    quantum = np.ldexp(1.0, e - 7)              # spacing of bf16 numbers in that binade
    r = np.rint(x / quantum) * quantum          # rint = round half to even; exact in f64
    r = np.where(np.abs(r) >= 2.0 ** 128, np.copysign(np.inf, r), r)
    f32 = r.astype(np.float32)                  # exact: r has <= 8 significant bits
    out = (f32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    # keep the sign of a negative zero produced by rounding a tiny negative value
    neg_zero = (r == 0.0) & np.signbit(x)
    return np.where(neg_zero, np.uint16(0x8000), out).astype(np.uint16)


def round_to_bf16(x) -> np.ndarray:
    """float64 -> nearest bf16 value, returned as float64."""
    return bf16_bits_to_f64(f64_to_bf16_bits(x))


# --------------------------------------------------------------------------
# Sec. 2.1: compression, reconstruction, cache ratio
# --------------------------------------------------------------------------


def compress(X: np.ndarray, P: np.ndarray) -> np.ndarray:
    """X_down = X P (Eq. 1).  X: [n, d_h], P: [d_h, r] -> [n, r]."""
    return np.asarray(X, np.float64) @ np.asarray(P, np.float64)


def reconstruct(X_down: np.ndarray, P: np.ndarray) -> np.ndarray:
    """X_tilde = X_down P^T (Eq. 2 / Eq. 7).  [n, r], [d_h, r] -> [n, d_h]."""
    return np.asarray(X_down, np.float64) @ np.asarray(P, np.float64).T


def compression_ratio(r_k: int, r_v: int, d_h: int) -> float:
    """CR = (r_K + r_V) / (2 d_h) (Eq. 3); also the cost c(r_K, r_V) of App. B."""
    return (r_k + r_v) / (2.0 * d_h)


def kv_cache_bytes(n_layers: int, n_kv_heads: int, n_ctx: int, batch: int,
                   r_k: int, r_v: int, bytes_per_elem: int = 2) -> int:
    """Bytes held by a cache that stores r_K + r_V numbers per token, KV head,
    layer and sequence.  With r_K = r_V = d_h this is the uncompressed cache of
    the introduction's example."""
    return n_layers * n_kv_heads * n_ctx * batch * (r_k + r_v) * bytes_per_elem


# --------------------------------------------------------------------------
# App. A.1: attention of one query against one head's keys and values
# --------------------------------------------------------------------------


def attention_single_query(q: np.ndarray, K: np.ndarray, V: np.ndarray,
                           scale: float) -> np.ndarray:
    """softmax(q K^T * scale) V for a single query row (Eq. 18, decode case).
    Two-pass textbook softmax: subtract the maximum, exponentiate, normalise."""
    s = (K @ q) * scale                         # [n]
    s = s - np.max(s)
    w = np.exp(s)
    p = w / np.sum(w)
    return p @ V                                # [d_h]


# --------------------------------------------------------------------------
# One decoder layer's compressed cache
# --------------------------------------------------------------------------


@dataclass
class OracleLayer:
    """Plain container: shapes, bases and the compressed cache of one layer.

    p_k, p_v:  float64 [n_bases, d_h, r]; n_bases is n_kv_heads (one basis per
               KV head) or 1 (a single basis shared by all heads, the paper's
               choice for keys in Sec. 3.3 "Head sharing").
    k_cache, v_cache: float64 [batch, n_kv_heads, capacity, r]; in "bf16"
               storage every entry is a bf16-representable value.
    """
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    r_k: int
    r_v: int
    capacity: int
    p_k: np.ndarray
    p_v: np.ndarray
    k_cache: np.ndarray
    v_cache: np.ndarray
    store: str = "bf16"

    def basis_k(self, h: int) -> np.ndarray:
        return self.p_k[h if self.p_k.shape[0] > 1 else 0]

    def basis_v(self, h: int) -> np.ndarray:
        return self.p_v[h if self.p_v.shape[0] > 1 else 0]


def new_layer(batch, n_q_heads, n_kv_heads, head_dim, p_k, p_v, capacity,
              store="bf16", fill=0.0) -> OracleLayer:
    p_k = np.asarray(p_k, np.float64)
    p_v = np.asarray(p_v, np.float64)
    if n_q_heads % n_kv_heads:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    if p_k.shape[1] != head_dim or p_v.shape[1] != head_dim:
        raise ValueError("bases must be [n_bases, head_dim, r]")
    if p_k.shape[0] not in (1, n_kv_heads) or p_v.shape[0] not in (1, n_kv_heads):
        raise ValueError("one basis per KV head, or one shared basis")
    if store not in ("bf16", "f64"):
        raise ValueError("store must be 'bf16' or 'f64'")
    r_k, r_v = p_k.shape[2], p_v.shape[2]
    return OracleLayer(
        batch, n_q_heads, n_kv_heads, head_dim, r_k, r_v, capacity, p_k, p_v,
        np.full((batch, n_kv_heads, capacity, r_k), fill, np.float64),
        np.full((batch, n_kv_heads, capacity, r_v), fill, np.float64), store)


def project_append(layer: OracleLayer, k_new: np.ndarray, v_new: np.ndarray,
                   cur_len: int) -> None:
    """Project T new tokens and store them at rows [cur_len, cur_len + T).

    k_new, v_new: float64 [batch, T, n_kv_heads, head_dim] (exact values of
    the caller's bf16 inputs).  Each stored number is the float64 sum of
    Eq. 1, rounded once to bf16 when the layer stores bf16.  Rows outside the
    written range are left untouched."""
    k_new = np.asarray(k_new, np.float64)
    v_new = np.asarray(v_new, np.float64)
    B, T, H, d = k_new.shape
    if (B, H, d) != (layer.batch, layer.n_kv_heads, layer.head_dim) or v_new.shape != k_new.shape:
        raise ValueError("new keys/values must be [batch, T, n_kv_heads, head_dim]")
    if cur_len < 0 or cur_len + T > layer.capacity:
        raise ValueError("append exceeds capacity")
    for b in range(B):
        for h in range(H):
            kd = compress(k_new[b, :, h, :], layer.basis_k(h))
            vd = compress(v_new[b, :, h, :], layer.basis_v(h))
            if layer.store == "bf16":
                kd, vd = round_to_bf16(kd), round_to_bf16(vd)
            layer.k_cache[b, h, cur_len:cur_len + T, :] = kd
            layer.v_cache[b, h, cur_len:cur_len + T, :] = vd


def decode_attention(layer: OracleLayer, q: np.ndarray, n_ctx: int,
                     scale: float | None = None, heads=None) -> np.ndarray:
    """Definition form of one decode step (Sec. 3.2 Eq. 7 inside App. A.1 Eq. 18).

    q: float64 [batch, n_q_heads, head_dim].  For every sequence b and query
    head h: rebuild the full-width keys and values of KV head h // G from rows
    [0, n_ctx) of the cache, then apply single-query softmax attention with
    scale 1/sqrt(head_dim) unless another scale is given.  Returns float64
    [batch, n_q_heads, head_dim]; `heads`, if given, is an iterable of
    (b, h) pairs to compute (all other rows are NaN)."""
    q = np.asarray(q, np.float64)
    if q.shape != (layer.batch, layer.n_q_heads, layer.head_dim):
        raise ValueError("q must be [batch, n_q_heads, head_dim]")
    if not 1 <= n_ctx <= layer.capacity:
        raise ValueError("n_ctx out of range")
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(layer.head_dim)
    G = layer.n_q_heads // layer.n_kv_heads
    out = np.full(q.shape, np.nan, np.float64)
    wanted = None if heads is None else set((int(b), int(h)) for b, h in heads)
    for b in range(layer.batch):
        for kv in range(layer.n_kv_heads):
            hs = [h for h in range(kv * G, (kv + 1) * G)
                  if wanted is None or (b, h) in wanted]
            if not hs:
                continue
            K_tilde = reconstruct(layer.k_cache[b, kv, :n_ctx, :], layer.basis_k(kv))
            V_tilde = reconstruct(layer.v_cache[b, kv, :n_ctx, :], layer.basis_v(kv))
            for h in hs:
                out[b, h] = attention_single_query(q[b, h], K_tilde, V_tilde, scale)
    return out


def decode_attention_factored(layer: OracleLayer, q: np.ndarray, n_ctx: int,
                              scale: float | None = None) -> np.ndarray:
    """The algebraically equal factored form, kept only to be tested against
    decode_attention: (q P_K) K_down^T for the scores, mix the rank-r_V rows,
    lift with P_V^T.  Not used as a parity reference."""
    q = np.asarray(q, np.float64)
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(layer.head_dim)
    G = layer.n_q_heads // layer.n_kv_heads
    out = np.empty(q.shape, np.float64)
    for b in range(layer.batch):
        for h in range(layer.n_q_heads):
            kv = h // G
            q_low = q[b, h] @ layer.basis_k(kv)                   # [r_K]
            s = (layer.k_cache[b, kv, :n_ctx, :] @ q_low) * scale
            w = np.exp(s - np.max(s))
            p = w / np.sum(w)
            a_low = p @ layer.v_cache[b, kv, :n_ctx, :]           # [r_V]
            out[b, h] = layer.basis_v(kv) @ a_low                 # [d_h]
    return out


# --------------------------------------------------------------------------
# Per-sequence lengths: Eq. 18 applies to every sequence with its own context
# --------------------------------------------------------------------------


def _one_sequence(layer: OracleLayer, b: int) -> OracleLayer:
    """A batch-1 layer holding sequence b's cache (views, not copies)."""
    return OracleLayer(1, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.r_k, layer.r_v,
                       layer.capacity, layer.p_k, layer.p_v, layer.k_cache[b:b + 1], layer.v_cache[b:b + 1],
                       layer.store)


def project_append_varlen(layer: OracleLayer, k_new: np.ndarray, v_new: np.ndarray, cur_lens) -> None:
    """project_append with a first row per sequence: the T new rows of sequence b go to
    [cur_lens[b], cur_lens[b] + T)."""
    for b in range(layer.batch):
        project_append(_one_sequence(layer, b), np.asarray(k_new)[b:b + 1], np.asarray(v_new)[b:b + 1],
                       int(cur_lens[b]))


def decode_attention_varlen(layer: OracleLayer, q: np.ndarray, seq_lens, scale: float | None = None) -> np.ndarray:
    """decode_attention with a context length per sequence: sequence b attends rows [0, seq_lens[b]).
    A sequence of length 0 has nothing to attend; its outputs are zeros (a convention: the softmax over
    an empty set is undefined)."""
    q = np.asarray(q, np.float64)
    out = np.zeros(q.shape, np.float64)
    for b in range(layer.batch):
        n_b = int(seq_lens[b])
        if n_b > 0:
            out[b] = decode_attention(_one_sequence(layer, b), q[b:b + 1], n_b, scale)[0]
    return out


# --------------------------------------------------------------------------
# Paged cache: where a row lives, nothing else
# --------------------------------------------------------------------------
#
# A serving system keeps the compressed rows of Eq. 1 in a pool of pages of
# page_tokens rows and a table per sequence: row t of sequence b is row
# t % page_tokens of pool page table[b][t // page_tokens].  The attention of
# Eq. 18 is unchanged; the functions below move rows between a pool and the
# contiguous layout the functions above work on, one row at a time.


@dataclass
class OraclePagedCache:
    """k_pool, v_pool: float64 [n_pages, n_kv_heads, page_tokens, r]; block_table: int [batch, max_pages]."""
    k_pool: np.ndarray
    v_pool: np.ndarray
    block_table: np.ndarray
    page_tokens: int


def paged_rows(pool: np.ndarray, table_row, page_tokens: int, n_rows: int) -> np.ndarray:
    """Rows [0, n_rows) of one sequence, gathered from the pool: [n_kv_heads, n_rows, r]."""
    out = np.empty((pool.shape[1], n_rows, pool.shape[3]), pool.dtype)
    for t in range(n_rows):
        out[:, t, :] = pool[int(table_row[t // page_tokens]), :, t % page_tokens, :]
    return out


def paged_store_rows(pool: np.ndarray, table_row, page_tokens: int, first_row: int, rows: np.ndarray) -> None:
    """Writes rows [first_row, first_row + T) of one sequence ([n_kv_heads, T, r]) into the pool."""
    for i in range(rows.shape[1]):
        t = first_row + i
        pool[int(table_row[t // page_tokens]), :, t % page_tokens, :] = rows[:, i, :]


def paged_as_contiguous(layer: OracleLayer, cache: OraclePagedCache, n_rows) -> OracleLayer:
    """A contiguous layer holding rows [0, n_rows[b]) of every sequence of the paged cache (a copy)."""
    out = new_layer(layer.batch, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.p_k, layer.p_v,
                    max(1, int(max(n_rows))), layer.store)
    for b in range(layer.batch):
        n_b = int(n_rows[b])
        out.k_cache[b, :, :n_b] = paged_rows(cache.k_pool, cache.block_table[b], cache.page_tokens, n_b)
        out.v_cache[b, :, :n_b] = paged_rows(cache.v_pool, cache.block_table[b], cache.page_tokens, n_b)
    return out


def paged_project_append(layer: OracleLayer, cache: OraclePagedCache, k_new: np.ndarray, v_new: np.ndarray,
                         cur_lens) -> None:
    """project_append into the paged cache: the T new rows of sequence b become its rows
    [cur_lens[b], cur_lens[b] + T).  `layer` supplies shapes, bases and the storage precision."""
    T = np.asarray(k_new).shape[1]
    tmp = new_layer(layer.batch, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.p_k, layer.p_v,
                    max(1, T), layer.store)
    project_append(tmp, k_new, v_new, 0)
    for b in range(layer.batch):
        paged_store_rows(cache.k_pool, cache.block_table[b], cache.page_tokens, int(cur_lens[b]), tmp.k_cache[b, :, :T])
        paged_store_rows(cache.v_pool, cache.block_table[b], cache.page_tokens, int(cur_lens[b]), tmp.v_cache[b, :, :T])


def paged_decode_attention(layer: OracleLayer, cache: OraclePagedCache, q: np.ndarray, seq_lens,
                           scale: float | None = None) -> np.ndarray:
    """decode_attention_varlen over the rows the block table names."""
    return decode_attention_varlen(paged_as_contiguous(layer, cache, seq_lens), q, seq_lens, scale)


def paged_prefill_attention(layer: OracleLayer, cache: OraclePagedCache, q: np.ndarray, n_prev: int,
                            scale: float | None = None, rows=None) -> np.ndarray:
    """prefill_attention over the rows the block table names (the chunk's rows already stored)."""
    T = np.asarray(q).shape[1]
    return prefill_attention(paged_as_contiguous(layer, cache, [n_prev + T] * layer.batch), q, n_prev, scale, rows)


@dataclass
class OraclePagedQuantCache:
    """The four arrays of a quantised cache as page pools [n_pages, n_kv_heads, page_tokens, ...]
    (codes one per byte, value ranges as bf16 bit patterns) plus the block table."""
    k_codes: np.ndarray
    v_codes: np.ndarray
    v_scale_bits: np.ndarray
    v_zero_bits: np.ndarray
    block_table: np.ndarray
    page_tokens: int


def _paged_quant_pools(cache: "OraclePagedQuantCache"):
    return ("k_codes", cache.k_codes), ("v_codes", cache.v_codes), ("v_scale_bits", cache.v_scale_bits), \
           ("v_zero_bits", cache.v_zero_bits)


def paged_quant_project_append(layer: "OracleQuantLayer", cache: OraclePagedQuantCache, k_new: np.ndarray,
                               v_new: np.ndarray, cur_lens) -> None:
    """quant_project_append into quantised pages: sequence b's T new rows become its rows
    [cur_lens[b], cur_lens[b] + T).  `layer` supplies shapes, bases, the static key ranges and the width."""
    T = np.asarray(k_new).shape[1]
    tmp = new_quant_layer(layer.batch, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.p_k, layer.p_v,
                          layer.k_scale, layer.k_zero, max(1, T), layer.bits)
    quant_project_append(tmp, k_new, v_new, 0)
    for b in range(layer.batch):
        for name, pool in _paged_quant_pools(cache):
            paged_store_rows(pool, cache.block_table[b], cache.page_tokens, int(cur_lens[b]), getattr(tmp, name)[b, :, :T])


def paged_quant_decode_attention(layer: "OracleQuantLayer", cache: OraclePagedQuantCache, q: np.ndarray, seq_lens,
                                 scale: float | None = None) -> np.ndarray:
    """quant_decode_attention per sequence over the rows its block table names; zeros for an empty sequence."""
    q = np.asarray(q, np.float64)
    out = np.zeros(q.shape, np.float64)
    for b in range(layer.batch):
        n_b = int(seq_lens[b])
        if n_b == 0:
            continue
        one = new_quant_layer(1, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.p_k, layer.p_v,
                              layer.k_scale, layer.k_zero, n_b, layer.bits)
        for name, pool in _paged_quant_pools(cache):
            getattr(one, name)[0] = paged_rows(pool, cache.block_table[b], cache.page_tokens, n_b)
        out[b] = quant_decode_attention(one, q[b:b + 1], n_b, scale)[0]
    return out


# --------------------------------------------------------------------------
# Sec. 3.4 "Overheads": projections folded into the attention linear weights
# --------------------------------------------------------------------------
#
# The paper notes that P_K and P_V can be folded into the attention linear
# layers (W_K P_K, W_V P_V, W_Q P_K on the way in, P_V^T W_O on the way out).
# The model then hands over rows that are already projected and takes the
# attention output in rank-r_V coordinates; what is left of the path is
# attention in the compressed space, with the scale of the ORIGINAL head dim:
#     a_low = softmax(q_low K_down^T / sqrt(d_h)) V_down.


def append_projected(layer: OracleLayer, k_low: np.ndarray, v_low: np.ndarray, cur_len: int) -> None:
    """Store T already-projected tokens at rows [cur_len, cur_len + T).
    k_low: [batch, T, n_kv_heads, r_k], v_low: [batch, T, n_kv_heads, r_v]; rounded
    once to bf16 when the layer stores bf16."""
    k_low, v_low = np.asarray(k_low, np.float64), np.asarray(v_low, np.float64)
    B, T, H, _ = k_low.shape
    if cur_len < 0 or cur_len + T > layer.capacity:
        raise ValueError("append exceeds capacity")
    kd = np.transpose(k_low, (0, 2, 1, 3))
    vd = np.transpose(v_low, (0, 2, 1, 3))
    if layer.store == "bf16":
        kd, vd = round_to_bf16(kd), round_to_bf16(vd)
    layer.k_cache[:, :, cur_len:cur_len + T, :] = kd
    layer.v_cache[:, :, cur_len:cur_len + T, :] = vd


def decode_attention_folded(layer: OracleLayer, q_low: np.ndarray, n_ctx: int,
                            scale: float | None = None) -> np.ndarray:
    """Attention in the compressed space.  q_low: [batch, n_q_heads, r_k] (the
    query already multiplied by P_K); returns [batch, n_q_heads, r_v], to be
    lifted by the caller's folded output projection.  Bases are not used."""
    q_low = np.asarray(q_low, np.float64)
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(layer.head_dim)
    G = layer.n_q_heads // layer.n_kv_heads
    out = np.empty((layer.batch, layer.n_q_heads, layer.r_v), np.float64)
    for b in range(layer.batch):
        for h in range(layer.n_q_heads):
            kv = h // G
            out[b, h] = attention_single_query(q_low[b, h], layer.k_cache[b, kv, :n_ctx, :],
                                               layer.v_cache[b, kv, :n_ctx, :], scale)
    return out


def paged_append_projected(layer: OracleLayer, cache: OraclePagedCache, k_low: np.ndarray, v_low: np.ndarray,
                           cur_lens) -> None:
    """append_projected into the paged cache: the T already-projected rows of sequence b become its rows
    [cur_lens[b], cur_lens[b] + T)."""
    T = np.asarray(k_low).shape[1]
    tmp = new_layer(layer.batch, layer.n_q_heads, layer.n_kv_heads, layer.head_dim, layer.p_k, layer.p_v,
                    max(1, T), layer.store)
    append_projected(tmp, k_low, v_low, 0)
    for b in range(layer.batch):
        paged_store_rows(cache.k_pool, cache.block_table[b], cache.page_tokens, int(cur_lens[b]), tmp.k_cache[b, :, :T])
        paged_store_rows(cache.v_pool, cache.block_table[b], cache.page_tokens, int(cur_lens[b]), tmp.v_cache[b, :, :T])


def paged_decode_attention_folded(layer: OracleLayer, cache: OraclePagedCache, q_low: np.ndarray, seq_lens,
                                  scale: float | None = None) -> np.ndarray:
    """decode_attention_folded over the rows the block table names, sequence b over its first seq_lens[b]
    rows (zeros for a sequence without rows)."""
    q_low = np.asarray(q_low, np.float64)
    flat = paged_as_contiguous(layer, cache, seq_lens)
    out = np.zeros((layer.batch, layer.n_q_heads, layer.r_v), np.float64)
    for b in range(layer.batch):
        if int(seq_lens[b]) > 0:
            out[b] = decode_attention_folded(_one_sequence(flat, b), q_low[b:b + 1], int(seq_lens[b]), scale)[0]
    return out


# --------------------------------------------------------------------------
# App. A.1 Eq. 18 with a whole chunk of queries (prefill over the compressed cache)
# --------------------------------------------------------------------------
#
# Eq. 18 is written for Q in R^{T x d_h}.  With T > 1 new tokens whose
# compressed keys and values are already in the cache, token t of the chunk
# sits at position n_prev + t and, in the decoder-only models the paper
# evaluates, attends positions 0 .. n_prev + t (causal mask; the paper's
# formula leaves the mask implicit -- this is the reading taken here).


def prefill_attention(layer: OracleLayer, q: np.ndarray, n_prev: int,
                      scale: float | None = None, rows=None) -> np.ndarray:
    """Definition form for a chunk.  q: float64 [batch, T, n_q_heads, head_dim];
    rows [0, n_prev + T) of the cache are filled.  For every sequence b, chunk
    token t and query head h: rebuild K~, V~ of KV head h // G (Sec. 3.2 Eq. 7)
    for cache rows [0, n_prev + t] and apply softmax attention of that one query
    (scale 1/sqrt(head_dim) unless given).  Returns [batch, T, n_q_heads,
    head_dim]; `rows`, if given, is an iterable of (b, t, h) to compute (all
    other rows are NaN)."""
    q = np.asarray(q, np.float64)
    B, T, HQ, d = q.shape
    if (B, HQ, d) != (layer.batch, layer.n_q_heads, layer.head_dim):
        raise ValueError("q must be [batch, T, n_q_heads, head_dim]")
    if n_prev < 0 or T < 1 or n_prev + T > layer.capacity:
        raise ValueError("chunk out of range")
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(layer.head_dim)
    G = layer.n_q_heads // layer.n_kv_heads
    out = np.full(q.shape, np.nan, np.float64)
    wanted = None if rows is None else set((int(b), int(t), int(h)) for b, t, h in rows)
    for b in range(B):
        for kv in range(layer.n_kv_heads):
            todo = [(t, h) for t in range(T) for h in range(kv * G, (kv + 1) * G)
                    if wanted is None or (b, t, h) in wanted]
            if not todo:
                continue
            n_max = n_prev + 1 + max(t for t, _ in todo)
            K_tilde = reconstruct(layer.k_cache[b, kv, :n_max, :], layer.basis_k(kv))
            V_tilde = reconstruct(layer.v_cache[b, kv, :n_max, :], layer.basis_v(kv))
            for t, h in todo:
                n_vis = n_prev + t + 1                      # positions this token may see
                out[b, t, h] = attention_single_query(q[b, t, h], K_tilde[:n_vis], V_tilde[:n_vis], scale)
    return out


def prefill_attention_folded(layer: OracleLayer, q_low: np.ndarray, n_prev: int,
                             scale: float | None = None, rows=None) -> np.ndarray:
    """The same in the compressed space (Sec. 3.4 folded weights): q_low is
    [batch, T, n_q_heads, r_k], the result [batch, T, n_q_heads, r_v]."""
    q_low = np.asarray(q_low, np.float64)
    B, T, HQ, _ = q_low.shape
    if n_prev < 0 or T < 1 or n_prev + T > layer.capacity:
        raise ValueError("chunk out of range")
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(layer.head_dim)
    G = layer.n_q_heads // layer.n_kv_heads
    out = np.full((B, T, HQ, layer.r_v), np.nan, np.float64)
    wanted = None if rows is None else set((int(b), int(t), int(h)) for b, t, h in rows)
    for b in range(B):
        for t in range(T):
            for h in range(HQ):
                if wanted is not None and (b, t, h) not in wanted:
                    continue
                kv, n_vis = h // G, n_prev + t + 1
                out[b, t, h] = attention_single_query(q_low[b, t, h], layer.k_cache[b, kv, :n_vis, :],
                                                      layer.v_cache[b, kv, :n_vis, :], scale)
    return out


# --------------------------------------------------------------------------
# Sec. 3.3 "Orthonormalization via QR" and Sec. 3.2 Eq. 6: bases from predicted matrices
# --------------------------------------------------------------------------


def orthonormal_basis(A: np.ndarray, r: int) -> np.ndarray:
    """The rank-r projection matrix built from a predicted square matrix A: factor A = Q R
    (Sec. 3.3 Eqs. 13-14), keep the orthonormal factor, P-bar = Q, and take its leading r
    columns (Sec. 3.2 Eq. 6).  QR is unique only up to the signs of the columns of Q; the
    convention here is a positive diagonal of R, which makes Q unique when the leading r
    columns of A are independent.  float64 throughout; A is [..., d, d], the result [..., d, r]."""
    A = np.asarray(A, np.float64)
    if A.shape[-1] != A.shape[-2] or not 1 <= r <= A.shape[-1]:
        raise ValueError("A must be square and 1 <= r <= d")
    Q, R = np.linalg.qr(A)
    sign = np.sign(np.diagonal(R, axis1=-2, axis2=-1))
    sign = np.where(sign == 0, 1.0, sign)
    return (Q * sign[..., None, :])[..., :, :r]


# --------------------------------------------------------------------------
# Sec. 3.5 / App. B Alg. 2: sequential budgeted rank selection
# --------------------------------------------------------------------------


def layer_ranks(n_layers: int, head_dim: int, rho: float, cand_k, cand_v, delta):
    """Greedy per-layer choice of (r_K, r_V) under a cache budget.

    delta[l][i][j] is the layer-output error of layer l at ranks
    (cand_k[i], cand_v[j]); the surfaces are inputs (evaluating them needs the
    model).  Follows Alg. 2: B_1 = L*rho; for l = 1..L the per-layer allowance
    is tau_l = B_l / (L - l + 1); among pairs with cost (r_K+r_V)/(2 d_h) <=
    tau_l take the smallest error; then B_{l+1} = B_l - cost.

    Readings: the allowance uses Alg. 2's denominator (the main text's Eq. 15
    prints L-(l+1), which would not give tau_1 = rho).  Feasibility is tested
    in integer rank units, (r_K+r_V)*(L-l+1) <= 2*d_h*B_l*(1+1e-12).  Equal
    errors: lower cost, then larger r_V, then first in candidate order.  If no
    pair fits, the cheapest pair is taken (ties: lower error) and the run
    continues with a negative balance; `feasible` is then False.

    Returns (r_k list, r_v list, achieved mean ratio, feasible)."""
    delta = np.asarray(delta, np.float64)
    cand_k = [int(r) for r in cand_k]
    cand_v = [int(r) for r in cand_v]
    if delta.shape != (n_layers, len(cand_k), len(cand_v)):
        raise ValueError("delta must be [n_layers, n_k, n_v]")
    units = 2.0 * head_dim * n_layers * rho      # budget in rank units: 2 d_h B_l
    feasible = True
    rk_out, rv_out = [], []
    for l in range(n_layers):
        remaining_layers = n_layers - l          # L - l + 1 with l counted from 1
        best = None
        for i, rk in enumerate(cand_k):
            for j, rv in enumerate(cand_v):
                cost = rk + rv
                if cost * remaining_layers <= units * (1.0 + 1e-12):
                    key = (delta[l, i, j], cost, -rv, i * len(cand_v) + j)
                    if best is None or key < best[0]:
                        best = (key, rk, rv)
        if best is None:
            feasible = False
            for i, rk in enumerate(cand_k):
                for j, rv in enumerate(cand_v):
                    key = (rk + rv, delta[l, i, j], -rv, i * len(cand_v) + j)
                    if best is None or key < best[0]:
                        best = (key, rk, rv)
        _, rk, rv = best
        rk_out.append(rk)
        rv_out.append(rv)
        units -= rk + rv
    achieved = sum(a + b for a, b in zip(rk_out, rv_out)) / (2.0 * head_dim * n_layers)
    return rk_out, rv_out, achieved, feasible


# --------------------------------------------------------------------------
# Sec. 4.3: asymmetric integer quantisation of the compressed cache
# --------------------------------------------------------------------------
#
# The paper applies asymmetric integer quantisation with group size 64 to the
# compressed tensors: keys with group-wise scales shared across batch and
# sequence positions within each KV head, values with token-wise group scales,
# and reports 8 bits as essentially lossless.  Reading taken here:
#   * a group is 64 consecutive channels of a rank-r row (the last group of a
#     row may be shorter);
#   * keys: one (scale, zero) pair per KV head and channel group, float32,
#     fixed before any token is cached (a calibration result the caller brings);
#   * values: one (scale, zero) pair per token and channel group, computed when
#     the token is appended from that group's minimum and maximum, and stored
#     next to the codes as two bf16 numbers;
#   * code = clamp(round_half_even((x - zero) / scale), 0, 2^bits - 1),
#     x_hat = code * scale + zero.
# Sec. 4.3 fixes no precision for the quantiser, so it is evaluated as the
# plain definition in float64 on the float64 projection: minimum, maximum,
# subtraction, division and round-half-even all in float64.  Only what the
# cache FORMAT stores is narrower: static key ranges are float32 numbers,
# per-row value ranges are bf16 numbers (rounded once, from float64).
# Attention then runs, in float64, on the dequantised rows exactly as on a
# bf16 cache.

GROUP = 64


def group_slices(r: int):
    """Channel ranges of the quantisation groups of a rank-r row."""
    return [slice(s, min(s + GROUP, r)) for s in range(0, r, GROUP)]


def calibrate_static_range(y: np.ndarray, bits: int = 8):
    """(scale, zero) per channel group from sample rows y [n, r]:
    zero = min, scale = (max - min) / (2^bits - 1), computed in float64 and
    stored as float32 (the format of static key ranges); a flat group gets scale 1."""
    y = np.asarray(y, np.float64)
    levels = float(2 ** bits - 1)
    sc, zr = [], []
    for g in group_slices(y.shape[1]):
        lo, hi = y[:, g].min(), y[:, g].max()
        s = np.float32((hi - lo) / levels)
        sc.append(s if s > 0 else np.float32(1.0))
        zr.append(np.float32(lo))
    return np.array(sc, np.float32), np.array(zr, np.float32)


def quantize_static(y: np.ndarray, scale: np.ndarray, zero: np.ndarray, bits: int = 8) -> np.ndarray:
    """Codes (uint8) of rows y [n, r] under fixed per-group (scale, zero):
    clamp(round_half_even((y - zero) / scale), 0, 2^bits - 1) in float64."""
    y = np.asarray(y, np.float64)
    out = np.empty(y.shape, np.uint8)
    top = float(2 ** bits - 1)
    for gi, g in enumerate(group_slices(y.shape[1])):
        t = (y[:, g] - float(zero[gi])) / float(scale[gi])
        out[:, g] = np.clip(np.rint(t), 0.0, top).astype(np.uint8)
    return out


def quantize_dynamic(y: np.ndarray, bits: int = 8):
    """Per-row, per-group quantisation.  Returns (codes uint8 [n, r],
    scale bits uint16 [n, n_groups], zero bits uint16 [n, n_groups]); scale and
    zero are stored as bf16: zero = bf16(min), scale = bf16((max - min) / (2^bits - 1))
    (replaced by 1 when that is 0), each rounded once from its float64 value; the
    codes are then clamp(round_half_even((y - zero) / scale)) in float64 with the
    STORED zero and scale, so that code * scale + zero is the nearest level."""
    y = np.asarray(y, np.float64)
    n, r = y.shape
    groups = group_slices(r)
    codes = np.empty((n, r), np.uint8)
    sb = np.empty((n, len(groups)), np.uint16)
    zb = np.empty((n, len(groups)), np.uint16)
    levels = float(2 ** bits - 1)
    for gi, g in enumerate(groups):
        lo = y[:, g].min(axis=1)
        hi = y[:, g].max(axis=1)
        s_bits = f64_to_bf16_bits((hi - lo) / levels)
        s = bf16_bits_to_f64(s_bits)
        flat = s == 0
        s_bits = np.where(flat, np.uint16(0x3F80), s_bits)
        s = np.where(flat, 1.0, s)
        z_bits = f64_to_bf16_bits(lo)
        z = bf16_bits_to_f64(z_bits)
        t = (y[:, g] - z[:, None]) / s[:, None]
        codes[:, g] = np.clip(np.rint(t), 0.0, levels).astype(np.uint8)
        sb[:, gi], zb[:, gi] = s_bits, z_bits
    return codes, sb, zb


def dequantize(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """x_hat = code * scale + zero in float64.  scale, zero: per group, either
    [n_groups] (static) or [n, n_groups] (per row), any float dtype."""
    codes = np.asarray(codes)
    out = np.empty(codes.shape, np.float64)
    scale = np.asarray(scale, np.float64)
    zero = np.asarray(zero, np.float64)
    for gi, g in enumerate(group_slices(codes.shape[1])):
        s = scale[..., gi]
        z = zero[..., gi]
        if s.ndim:
            s, z = s[:, None], z[:, None]
        out[:, g] = codes[:, g].astype(np.float64) * s + z
    return out


@dataclass
class OracleQuantLayer:
    """One layer's quantised compressed cache.
    k_codes [batch, n_kv_heads, capacity, r_k] uint8 with static k_scale / k_zero
    float32 [n_kv_heads, n_groups_k]; v_codes likewise with per-row bf16
    v_scale_bits / v_zero_bits uint16 [batch, n_kv_heads, capacity, n_groups_v]."""
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    r_k: int
    r_v: int
    capacity: int
    bits: int
    p_k: np.ndarray
    p_v: np.ndarray
    k_scale: np.ndarray
    k_zero: np.ndarray
    k_codes: np.ndarray
    v_codes: np.ndarray
    v_scale_bits: np.ndarray
    v_zero_bits: np.ndarray

    def basis_k(self, h: int) -> np.ndarray:
        return self.p_k[h if self.p_k.shape[0] > 1 else 0]

    def basis_v(self, h: int) -> np.ndarray:
        return self.p_v[h if self.p_v.shape[0] > 1 else 0]


def new_quant_layer(batch, n_q_heads, n_kv_heads, head_dim, p_k, p_v, k_scale, k_zero, capacity,
                    bits=8) -> OracleQuantLayer:
    p_k, p_v = np.asarray(p_k, np.float64), np.asarray(p_v, np.float64)
    r_k, r_v = p_k.shape[2], p_v.shape[2]
    ngk, ngv = len(group_slices(r_k)), len(group_slices(r_v))
    k_scale = np.asarray(k_scale, np.float32).reshape(n_kv_heads, ngk)
    k_zero = np.asarray(k_zero, np.float32).reshape(n_kv_heads, ngk)
    return OracleQuantLayer(
        batch, n_q_heads, n_kv_heads, head_dim, r_k, r_v, capacity, bits, p_k, p_v, k_scale, k_zero,
        np.zeros((batch, n_kv_heads, capacity, r_k), np.uint8),
        np.zeros((batch, n_kv_heads, capacity, r_v), np.uint8),
        np.full((batch, n_kv_heads, capacity, ngv), 0x3F80, np.uint16),
        np.zeros((batch, n_kv_heads, capacity, ngv), np.uint16))


def quant_project_append(layer: OracleQuantLayer, k_new: np.ndarray, v_new: np.ndarray, cur_len: int) -> None:
    """Project T new tokens (Eq. 1, float64 sums), quantise, store at rows
    [cur_len, cur_len + T)."""
    k_new, v_new = np.asarray(k_new, np.float64), np.asarray(v_new, np.float64)
    B, T, H, d = k_new.shape
    if cur_len < 0 or cur_len + T > layer.capacity:
        raise ValueError("append exceeds capacity")
    for b in range(B):
        for h in range(H):
            kd = compress(k_new[b, :, h, :], layer.basis_k(h))
            vd = compress(v_new[b, :, h, :], layer.basis_v(h))
            layer.k_codes[b, h, cur_len:cur_len + T] = quantize_static(kd, layer.k_scale[h], layer.k_zero[h], layer.bits)
            c, sb, zb = quantize_dynamic(vd, layer.bits)
            layer.v_codes[b, h, cur_len:cur_len + T] = c
            layer.v_scale_bits[b, h, cur_len:cur_len + T] = sb
            layer.v_zero_bits[b, h, cur_len:cur_len + T] = zb


def quant_decode_attention(layer: OracleQuantLayer, q: np.ndarray, n_ctx: int,
                           scale: float | None = None, heads=None) -> np.ndarray:
    """Eq. 18 per query head on K~ = dequant(K codes) P_K^T, V~ = dequant(V codes) P_V^T."""
    q = np.asarray(q, np.float64)
    if scale is None or scale <= 0:
        scale = 1.0 / math.sqrt(layer.head_dim)
    G = layer.n_q_heads // layer.n_kv_heads
    out = np.full(q.shape, np.nan, np.float64)
    wanted = None if heads is None else set((int(b), int(h)) for b, h in heads)
    for b in range(layer.batch):
        for kv in range(layer.n_kv_heads):
            hs = [h for h in range(kv * G, (kv + 1) * G) if wanted is None or (b, h) in wanted]
            if not hs:
                continue
            k_low = dequantize(layer.k_codes[b, kv, :n_ctx], layer.k_scale[kv], layer.k_zero[kv])
            v_low = dequantize(layer.v_codes[b, kv, :n_ctx],
                               bf16_bits_to_f64(layer.v_scale_bits[b, kv, :n_ctx]),
                               bf16_bits_to_f64(layer.v_zero_bits[b, kv, :n_ctx]))
            K_tilde = reconstruct(k_low, layer.basis_k(kv))
            V_tilde = reconstruct(v_low, layer.basis_v(kv))
            for h in hs:
                out[b, h] = attention_single_query(q[b, h], K_tilde, V_tilde, scale)
    return out
