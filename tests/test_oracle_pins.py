"""Pins for the float64 oracle: every check here compares it with something
that is NOT the oracle -- closed forms, invariants the paper states, an
independent brute force, a library routine, or a number the paper prints."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import synth


def _rand_orthogonal(rng, d):
    q, r = np.linalg.qr(rng.standard_normal((d, d)))
    return q * np.sign(np.diag(r))


def _brute_attention(q, K, V, scale):
    """Independent pure-Python softmax attention for one query."""
    n, d = len(K), len(V[0])
    s = [sum(q[i] * K[j][i] for i in range(len(q))) * scale for j in range(n)]
    m = max(s)
    w = [math.exp(x - m) for x in s]
    z = sum(w)
    return [sum(w[j] / z * V[j][c] for j in range(n)) for c in range(d)]


def _layer_f64(rng, B, HQ, HKV, d, rk, rv, n, P_k=None, P_v=None, K=None, V=None):
    if P_k is None:
        P_k = np.stack([_rand_orthogonal(rng, d)[:, :rk] for _ in range(HKV)])
    if P_v is None:
        P_v = np.stack([_rand_orthogonal(rng, d)[:, :rv] for _ in range(HKV)])
    if K is None:
        K = rng.standard_normal((B, n, HKV, d))
    if V is None:
        V = rng.standard_normal((B, n, HKV, d))
    L = O.new_layer(B, HQ, HKV, d, P_k, P_v, capacity=n, store="f64")
    O.project_append(L, K, V, 0)
    return L, K, V


# ---------------------------------------------------------------- bf16 ----

def test_bf16_rounding_matches_library_on_float32_inputs():
    rng = np.random.default_rng(1)
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(2000) * 1e-38).astype(np.float32),   # subnormal bf16 range
        (rng.standard_normal(2000) * 1e30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 3.3895314e38], np.float32)])
    want = synth.torch_bf16_to_bits(torch.from_numpy(x).to(torch.bfloat16))
    got = O.f64_to_bf16_bits(x.astype(np.float64))
    assert np.array_equal(got, want)


def test_bf16_rounding_ties_and_single_rounding():
    # ties go to the even neighbour
    assert O.round_to_bf16(1.0 + 2.0 ** -8) == 1.0
    assert O.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert O.round_to_bf16(-(1.0 + 2.0 ** -8)) == -1.0
    # a float64 just above a tie must round up (rounding via float32 first would lose it)
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert O.round_to_bf16(x) == 1.0 + 2.0 ** -7
    # nearest-ness as a property
    rng = np.random.default_rng(2)
    v = rng.standard_normal(5000) * np.exp(rng.uniform(-20, 20, 5000))
    r = O.round_to_bf16(v)
    ulp = np.ldexp(1.0, np.floor(np.log2(np.abs(v))).astype(int) - 7)
    assert np.all(np.abs(r - v) <= ulp / 2)
    assert np.array_equal(O.round_to_bf16(r), r)          # representable values are fixed points
    bits = O.f64_to_bf16_bits(v)
    assert np.array_equal(O.bf16_bits_to_f64(bits), r)


def test_bf16_decode_of_known_patterns():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0000, 0x4049], np.uint16)
    want = np.array([1.0, -1.0, 2.0, 0.5, 0.0, 3.140625])
    assert np.array_equal(O.bf16_bits_to_f64(bits), want)


# ------------------------------------------------- Sec. 2.1 identities ----

def test_basis_orthonormal_and_projector_idempotent():
    P64, _ = synth.orthonormal_bases(7, 3, 128, 64)
    rng = np.random.default_rng(3)
    for P in P64:
        assert np.allclose(P.T @ P, np.eye(64), atol=1e-13)
        assert np.allclose(P @ P.T @ P, P, atol=1e-13)
        K = rng.standard_normal((17, 128))
        once = O.compress(K, P)
        again = O.compress(O.reconstruct(once, P), P)
        assert np.allclose(once, again, rtol=0, atol=1e-13)


def test_full_rank_equals_uncompressed_brute_force():
    rng = np.random.default_rng(4)
    B, HQ, HKV, d, n = 2, 4, 2, 8, 5
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, d, d, n)
    q = rng.standard_normal((B, HQ, d))
    got = O.decode_attention(L, q, n)
    for b in range(B):
        for h in range(HQ):
            kv = h // (HQ // HKV)
            want = _brute_attention(q[b, h].tolist(), K[b, :, kv].tolist(),
                                    V[b, :, kv].tolist(), 1 / math.sqrt(d))
            assert np.allclose(got[b, h], want, rtol=1e-12, atol=1e-13)


def test_tiny_rank_deficient_case_against_pure_python():
    # d=4, r=2, n=3: rebuild K~, V~ by hand with explicit loops, then brute-force attention
    rng = np.random.default_rng(5)
    d, r, n = 4, 2, 3
    Pk = _rand_orthogonal(rng, d)[:, :r]
    Pv = _rand_orthogonal(rng, d)[:, :r]
    K = rng.standard_normal((1, n, 1, d))
    V = rng.standard_normal((1, n, 1, d))
    q = rng.standard_normal((1, 1, d))
    L, _, _ = _layer_f64(rng, 1, 1, 1, d, r, r, n, Pk[None], Pv[None], K, V)

    def proj_rebuild(X, P):
        rows = []
        for j in range(n):
            low = [sum(X[j][i] * P[i][c] for i in range(d)) for c in range(r)]
            rows.append([sum(low[c] * P[i][c] for c in range(r)) for i in range(d)])
        return rows
    Kt = proj_rebuild(K[0, :, 0].tolist(), Pk.tolist())
    Vt = proj_rebuild(V[0, :, 0].tolist(), Pv.tolist())
    want = _brute_attention(q[0, 0].tolist(), Kt, Vt, 1 / math.sqrt(d))
    got = O.decode_attention(L, q, n)[0, 0]
    assert np.allclose(got, want, rtol=1e-13, atol=1e-14)
    # and it must differ from uncompressed attention (the compression is really applied)
    raw = _brute_attention(q[0, 0].tolist(), K[0, :, 0].tolist(), V[0, :, 0].tolist(), 0.5)
    assert not np.allclose(got, raw, rtol=1e-3)


def test_rotation_inside_the_span_changes_cache_not_output():
    rng = np.random.default_rng(6)
    B, HQ, HKV, d, rk, rv, n = 1, 4, 2, 16, 6, 10, 9
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n)
    Rk, Rv = _rand_orthogonal(rng, rk), _rand_orthogonal(rng, rv)
    L2, _, _ = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n, L.p_k @ Rk, L.p_v @ Rv, K, V)
    q = rng.standard_normal((B, HQ, d))
    assert not np.allclose(L.k_cache, L2.k_cache)
    assert np.allclose(O.decode_attention(L, q, n), O.decode_attention(L2, q, n),
                       rtol=1e-12, atol=1e-13)


def test_inputs_inside_the_span_are_exact_with_sqrt_head_dim_scale():
    rng = np.random.default_rng(7)
    B, HQ, HKV, d, rk, rv, n = 2, 6, 3, 16, 5, 7, 11
    Pk = np.stack([_rand_orthogonal(rng, d)[:, :rk] for _ in range(HKV)])
    Pv = np.stack([_rand_orthogonal(rng, d)[:, :rv] for _ in range(HKV)])
    K = np.einsum("bnhc,hdc->bnhd", rng.standard_normal((B, n, HKV, rk)), Pk)
    V = np.einsum("bnhc,hdc->bnhd", rng.standard_normal((B, n, HKV, rv)), Pv)
    L, _, _ = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n, Pk, Pv, K, V)
    q = rng.standard_normal((B, HQ, d))
    got = O.decode_attention(L, q, n)
    G = HQ // HKV
    for b in range(B):
        for h in range(HQ):
            want = _brute_attention(q[b, h].tolist(), K[b, :, h // G].tolist(),
                                    V[b, :, h // G].tolist(), 1 / math.sqrt(d))
            assert np.allclose(got[b, h], want, rtol=1e-11, atol=1e-12)


def test_definition_form_equals_factored_form():
    rng = np.random.default_rng(8)
    L, _, _ = _layer_f64(rng, 2, 8, 2, 32, 12, 20, 300)
    q = rng.standard_normal((2, 8, 32))
    a = O.decode_attention(L, q, 257)
    b = O.decode_attention_factored(L, q, 257)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-13)


def test_single_token_returns_projected_value_for_any_query():
    rng = np.random.default_rng(9)
    L, K, V = _layer_f64(rng, 1, 2, 1, 16, 4, 6, 1)
    for _ in range(3):
        q = rng.standard_normal((1, 2, 16)) * 10
        want = V[0, 0, 0] @ L.p_v[0] @ L.p_v[0].T
        got = O.decode_attention(L, q, 1)
        assert np.allclose(got[0, 0], want, rtol=1e-14, atol=1e-14)
        assert np.allclose(got[0, 1], want, rtol=1e-14, atol=1e-14)


def test_uniform_scores_give_mean_of_reconstructed_values():
    rng = np.random.default_rng(10)
    d, rk, rv, n = 16, 4, 8, 13
    Pk = _rand_orthogonal(rng, d)
    K = np.tile(rng.standard_normal((1, 1, 1, d)), (1, n, 1, 1))        # identical keys
    V = rng.standard_normal((1, n, 1, d))
    L, _, _ = _layer_f64(rng, 1, 1, 1, d, rk, rv, n, Pk[None, :, :rk], None, K, V)
    q = rng.standard_normal((1, 1, d))
    want = (V[0, :, 0] @ L.p_v[0] @ L.p_v[0].T).mean(axis=0)
    assert np.allclose(O.decode_attention(L, q, n)[0, 0], want, rtol=1e-13, atol=1e-14)
    # a query orthogonal to span(P_K) also scores every key equally
    K2 = rng.standard_normal((1, n, 1, d))
    L2, _, _ = _layer_f64(rng, 1, 1, 1, d, rk, rv, n, Pk[None, :, :rk], L.p_v, K2, V)
    q_perp = (Pk[:, rk:] @ rng.standard_normal(d - rk))[None, None]
    assert np.allclose(O.decode_attention(L2, q_perp, n)[0, 0], want, rtol=1e-12, atol=1e-13)


def test_identity_basis_matches_library_attention_with_grouped_heads():
    rng = np.random.default_rng(11)
    B, HQ, HKV, d, n = 2, 8, 2, 16, 37
    eye = np.tile(np.eye(d)[None], (HKV, 1, 1))
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, d, d, n, eye, eye)
    q = rng.standard_normal((B, HQ, d))
    G = HQ // HKV
    tq = torch.from_numpy(q)[:, :, None, :]                                  # [B,HQ,1,d]
    tk = torch.from_numpy(K).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)  # [B,HQ,n,d]
    tv = torch.from_numpy(V).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0].numpy()
    assert np.allclose(O.decode_attention(L, q, n), want, rtol=1e-12, atol=1e-13)
    # partial context: only rows [0, n_ctx) take part
    want2 = torch.nn.functional.scaled_dot_product_attention(
        tq, tk[:, :, :20], tv[:, :, :20])[:, :, 0].numpy()
    assert np.allclose(O.decode_attention(L, q, 20), want2, rtol=1e-12, atol=1e-13)


def test_shared_basis_equals_per_head_copies():
    rng = np.random.default_rng(12)
    B, HQ, HKV, d, rk, rv, n = 1, 4, 4, 16, 6, 6, 10
    Pk1 = _rand_orthogonal(rng, d)[None, :, :rk]
    K = rng.standard_normal((B, n, HKV, d))
    V = rng.standard_normal((B, n, HKV, d))
    La, _, _ = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n, Pk1, None, K, V)
    Lb, _, _ = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n, np.tile(Pk1, (HKV, 1, 1)), La.p_v, K, V)
    q = rng.standard_normal((B, HQ, d))
    assert np.array_equal(La.k_cache, Lb.k_cache)
    assert np.array_equal(O.decode_attention(La, q, n), O.decode_attention(Lb, q, n))


# ------------------------------------------------- append: layout pins ----

def test_append_places_rows_and_leaves_the_rest_untouched():
    B, HKV, d, r, cap, T, cur = 2, 3, 16, 5, 12, 4, 6
    Pk64, _, idx_k, sgn_k = synth.selection_bases(1, HKV, d, r)
    Pv64, _, idx_v, sgn_v = synth.selection_bases(2, HKV, d, r)
    L = O.new_layer(B, HKV, HKV, d, Pk64, Pv64, cap, store="bf16", fill=-77.0)
    # small integers, exactly representable in bf16, encoding (b, t, h, channel)
    b_, t_, h_, c_ = np.meshgrid(np.arange(B), np.arange(T), np.arange(HKV), np.arange(d), indexing="ij")
    K = (b_ * 64 + t_ * 16 + h_ * 4 + c_ % 4 + 1).astype(np.float64)
    V = -K + 0.5
    O.project_append(L, K, V, cur)
    for b in range(B):
        for h in range(HKV):
            assert np.array_equal(L.k_cache[b, h, cur:cur + T], K[b, :, h][:, idx_k[h]] * sgn_k[h])
            assert np.array_equal(L.v_cache[b, h, cur:cur + T], V[b, :, h][:, idx_v[h]] * sgn_v[h])
    mask = np.ones(cap, bool)
    mask[cur:cur + T] = False
    assert np.all(L.k_cache[:, :, mask] == -77.0) and np.all(L.v_cache[:, :, mask] == -77.0)


def test_bf16_store_rounds_once_and_f64_store_does_not():
    rng = np.random.default_rng(13)
    B, HKV, d, r, n = 1, 2, 32, 8, 50
    P64, Pbf = synth.orthonormal_bases(3, HKV, d, r)
    K = rng.standard_normal((B, n, HKV, d))
    Lb = O.new_layer(B, HKV, HKV, d, P64, P64, n, store="bf16")
    Lf = O.new_layer(B, HKV, HKV, d, P64, P64, n, store="f64")
    O.project_append(Lb, K, K, 0)
    O.project_append(Lf, K, K, 0)
    exact = np.einsum("bnhd,hdc->bhnc", K, P64)
    assert np.allclose(Lf.k_cache, exact, rtol=1e-14, atol=1e-15)
    assert np.array_equal(O.round_to_bf16(Lb.k_cache), Lb.k_cache)
    ulp = np.ldexp(1.0, np.floor(np.log2(np.abs(exact))).astype(int) - 7)
    assert np.all(np.abs(Lb.k_cache - exact) <= ulp / 2 * (1 + 1e-9))


# ------------------------------------------------------- sizes (Eq. 3) ----

def test_cache_size_example_printed_in_the_introduction(golden_dir):
    kv = {}
    with open(os.path.join(golden_dir, "kv_cache_size_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.strip().split("=")
                kv[k] = int(v)
    full = O.kv_cache_bytes(kv["n_layers"], kv["n_kv_heads"], kv["n_ctx"], kv["batch"],
                            kv["head_dim"], kv["head_dim"], kv["bytes_per_elem"])
    assert full == kv["printed_gigabytes"] * 2 ** 30
    assert O.compression_ratio(64, 64, 128) == 0.5
    assert O.compression_ratio(48, 80, 128) == 0.5
    assert O.compression_ratio(128, 128, 128) == 1.0
    half = O.kv_cache_bytes(kv["n_layers"], kv["n_kv_heads"], kv["n_ctx"], kv["batch"], 64, 64)
    assert half == full * O.compression_ratio(64, 64, 128)
    # one layer of the batch-4 / 32K workload at rank 64/64 is 256 MiB
    assert O.kv_cache_bytes(1, 8, 32768, 4, 64, 64) == 256 * 2 ** 20


# ------------------------------------- Sec. 3.4: folded projections ----

def test_folded_variant_equals_the_explicit_path():
    rng = np.random.default_rng(20)
    B, HQ, HKV, d, rk, rv, n = 2, 8, 2, 32, 12, 20, 150
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n)
    q = rng.standard_normal((B, HQ, d))
    G = HQ // HKV
    # what a model with folded weights would hand over
    q_low = np.stack([[q[b, h] @ L.p_k[h // G] for h in range(HQ)] for b in range(B)])
    k_low = np.einsum("bnhd,hdc->bnhc", K, L.p_k)
    v_low = np.einsum("bnhd,hdc->bnhc", V, L.p_v)
    F = O.new_layer(B, HQ, HKV, d, L.p_k, L.p_v, n, store="f64")
    O.append_projected(F, k_low, v_low, 0)
    assert np.allclose(F.k_cache, L.k_cache, rtol=1e-13, atol=1e-14)
    a_low = O.decode_attention_folded(F, q_low, 131)
    assert a_low.shape == (B, HQ, rv)
    lifted = np.stack([[L.p_v[h // G] @ a_low[b, h] for h in range(HQ)] for b in range(B)])
    assert np.allclose(lifted, O.decode_attention(L, q, 131), rtol=1e-12, atol=1e-13)


def test_folded_variant_is_library_attention_in_rank_space_with_head_dim_scale():
    rng = np.random.default_rng(21)
    B, HQ, HKV, d, rk, rv, n = 1, 6, 3, 64, 16, 24, 40
    L = O.new_layer(B, HQ, HKV, d, np.zeros((HKV, d, rk)), np.zeros((HKV, d, rv)), n, store="f64")
    k_low = rng.standard_normal((B, n, HKV, rk))
    v_low = rng.standard_normal((B, n, HKV, rv))
    O.append_projected(L, k_low, v_low, 0)
    q_low = rng.standard_normal((B, HQ, rk))
    G = HQ // HKV
    tq = torch.from_numpy(q_low)[:, :, None, :]
    tk = torch.from_numpy(k_low).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    tv = torch.from_numpy(v_low).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    # the scale is 1/sqrt(head_dim) = 1/8, not 1/sqrt(r_k) = 1/4
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=1.0 / 8.0)[:, :, 0].numpy()
    assert np.allclose(O.decode_attention_folded(L, q_low, n), want, rtol=1e-12, atol=1e-13)
    wrong = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[:, :, 0].numpy()
    assert not np.allclose(O.decode_attention_folded(L, q_low, n), wrong, rtol=1e-3)
    # bf16 storage rounds the handed-over rows once
    Lb = O.new_layer(B, HQ, HKV, d, np.zeros((HKV, d, rk)), np.zeros((HKV, d, rv)), n, store="bf16", fill=5.0)
    O.append_projected(Lb, k_low[:, :7], v_low[:, :7], 3)
    assert np.array_equal(Lb.k_cache[:, :, 3:10], O.round_to_bf16(np.transpose(k_low[:, :7], (0, 2, 1, 3))))
    assert np.all(Lb.k_cache[:, :, :3] == 5.0) and np.all(Lb.v_cache[:, :, 10:] == 5.0)


# ------------------------------------------------------ chunk prefill ----

def test_prefill_with_identity_basis_matches_library_causal_attention():
    """P = I and an empty cache before the chunk: the chunk attention is the
    library's causal scaled-dot-product attention (grouped heads)."""
    rng = np.random.default_rng(30)
    B, HQ, HKV, d, T = 2, 4, 2, 16, 23
    eye = np.tile(np.eye(d)[None], (HKV, 1, 1))
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, d, d, T, eye, eye)
    q = rng.standard_normal((B, T, HQ, d))
    G = HQ // HKV
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    tk = torch.from_numpy(K).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    tv = torch.from_numpy(V).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).permute(0, 2, 1, 3).numpy()
    assert np.allclose(O.prefill_attention(L, q, 0), want, rtol=1e-12, atol=1e-13)


def test_prefill_with_a_prefix_matches_library_attention_under_an_explicit_mask():
    """n_prev cached tokens before the chunk: token t sees positions 0..n_prev+t.
    The mask is written out here as a boolean matrix for the library routine."""
    rng = np.random.default_rng(31)
    B, HQ, HKV, d, n_prev, T = 1, 6, 3, 16, 9, 7
    n = n_prev + T
    eye = np.tile(np.eye(d)[None], (HKV, 1, 1))
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, d, d, n, eye, eye)
    q = rng.standard_normal((B, T, HQ, d))
    G = HQ // HKV
    mask = torch.tensor([[j <= n_prev + t for j in range(n)] for t in range(T)])
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    tk = torch.from_numpy(K).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    tv = torch.from_numpy(V).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).permute(0, 2, 1, 3).numpy()
    got = O.prefill_attention(L, q, n_prev)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-13)
    # an off-by-one in the visible range (token t not seeing itself, or seeing t+1) is a different result
    for bad in (-1, 1):
        mask_bad = torch.tensor([[j <= n_prev + t + bad for j in range(n)] for t in range(T)])
        other = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask_bad).permute(0, 2, 1, 3).numpy()
        assert not np.allclose(got, other, rtol=1e-3)


def test_prefill_rank_deficient_case_against_pure_python():
    rng = np.random.default_rng(32)
    B, HQ, HKV, d, rk, rv, n_prev, T = 1, 2, 1, 6, 3, 4, 2, 4
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n_prev + T)
    q = rng.standard_normal((B, T, HQ, d))
    got = O.prefill_attention(L, q, n_prev)
    Pk, Pv = L.p_k[0].tolist(), L.p_v[0].tolist()
    Kt, Vt = [], []
    for j in range(n_prev + T):          # K~ = (K P_K) P_K^T row by row, in plain loops
        kd = [sum(K[0, j, 0, i] * Pk[i][c] for i in range(d)) for c in range(rk)]
        vd = [sum(V[0, j, 0, i] * Pv[i][c] for i in range(d)) for c in range(rv)]
        Kt.append([sum(kd[c] * Pk[i][c] for c in range(rk)) for i in range(d)])
        Vt.append([sum(vd[c] * Pv[i][c] for c in range(rv)) for i in range(d)])
    for t in range(T):
        for h in range(HQ):
            want = _brute_attention(q[0, t, h].tolist(), Kt[:n_prev + t + 1], Vt[:n_prev + t + 1], 1.0 / math.sqrt(d))
            assert np.allclose(got[0, t, h], want, rtol=1e-12, atol=1e-13)


def test_prefill_first_token_of_an_empty_cache_returns_its_own_value_row():
    rng = np.random.default_rng(33)
    B, HQ, HKV, d, rk, rv, T = 2, 4, 2, 16, 5, 7, 6
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, rk, rv, T)
    q = rng.standard_normal((B, T, HQ, d))
    got = O.prefill_attention(L, q, 0)
    for b in range(B):
        for h in range(HQ):
            kv = h // (HQ // HKV)
            assert np.allclose(got[b, 0, h], L.p_v[kv] @ (L.p_v[kv].T @ V[b, 0, kv]), rtol=1e-12, atol=1e-13)


def test_prefill_rows_equal_decode_steps_and_row_selection():
    """Token t of the chunk is the decode query at n_ctx = n_prev + t + 1; the
    folded form lifted by P_V equals the explicit form."""
    rng = np.random.default_rng(34)
    B, HQ, HKV, d, rk, rv, n_prev, T = 2, 8, 2, 32, 12, 20, 40, 11
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, rk, rv, n_prev + T)
    q = rng.standard_normal((B, T, HQ, d))
    got = O.prefill_attention(L, q, n_prev)
    for t in (0, 5, T - 1):
        assert np.allclose(got[:, t], O.decode_attention(L, q[:, t], n_prev + t + 1), rtol=1e-12, atol=1e-13)
    some = [(0, 3, 1), (1, 10, 7)]
    part = O.prefill_attention(L, q, n_prev, rows=some)
    for b, t, h in some:
        assert np.array_equal(part[b, t, h], got[b, t, h])
    assert np.isnan(part[0, 0, 0]).all()
    G = HQ // HKV
    q_low = np.einsum("bthd,hdc->bthc", q, np.repeat(L.p_k, G, axis=0))
    a_low = O.prefill_attention_folded(L, q_low, n_prev)
    lifted = np.einsum("bthc,hdc->bthd", a_low, np.repeat(L.p_v, G, axis=0))
    assert np.allclose(lifted, got, rtol=1e-12, atol=1e-13)
    part_low = O.prefill_attention_folded(L, q_low, n_prev, rows=some)
    assert np.array_equal(part_low[1, 10, 7], a_low[1, 10, 7]) and np.isnan(part_low[0, 0, 0]).all()


# ------------------------------------------------- zero-padded bases ----


def test_zero_padded_basis_serves_any_rank_exactly():
    """Sec. 2.1 Eqs. 1-2: a zero column of a basis yields a zero coefficient, so a rank-77 basis padded
    with zero columns to 80 must give the rank-77 cache in its first 77 channels, zeros in the rest, and
    the very same attention output.  The reference side is a brute force on the UNPADDED rank-77
    reconstruction, so nothing here compares the oracle with itself."""
    rng = np.random.default_rng(77)
    B, HQ, HKV, d, n = 1, 4, 2, 16, 9
    rk, rv, rk_pad, rv_pad = 5, 7, 8, 16
    P_k = np.stack([_rand_orthogonal(rng, d)[:, :rk] for _ in range(HKV)])
    P_v = np.stack([_rand_orthogonal(rng, d)[:, :rv] for _ in range(HKV)])
    pad = lambda P, r: np.concatenate([P, np.zeros(P.shape[:2] + (r - P.shape[2],))], axis=2)
    L, K, V = _layer_f64(rng, B, HQ, HKV, d, rk_pad, rv_pad, n, P_k=pad(P_k, rk_pad), P_v=pad(P_v, rv_pad))
    assert np.all(L.k_cache[..., rk:] == 0.0) and np.all(L.v_cache[..., rv:] == 0.0)
    q = rng.standard_normal((B, HQ, d))
    got = O.decode_attention(L, q, n)
    for h in range(HQ):
        kv = h // 2
        Kt = (K[0, :, kv] @ P_k[kv]) @ P_k[kv].T            # rank-5 reconstruction, unpadded
        Vt = (V[0, :, kv] @ P_v[kv]) @ P_v[kv].T
        want = _brute_attention(list(q[0, h]), Kt.tolist(), Vt.tolist(), 1.0 / math.sqrt(d))
        assert np.max(np.abs(got[0, h] - np.array(want))) < 1e-12


# ------------------------------------------------- per-sequence lengths ----


def test_per_sequence_lengths_match_library_attention_under_a_padding_mask():
    """With P = I the varlen routine must equal the library's scaled-dot-product attention where each
    sequence masks the keys at and beyond its own length; rows placed by the varlen append at
    per-sequence offsets must be the ones the mask exposes."""
    rng = np.random.default_rng(123)
    B, HQ, HKV, d, cap = 3, 4, 2, 8, 12
    eye = np.stack([np.eye(d)] * HKV)
    L = O.new_layer(B, HQ, HKV, d, eye, eye, cap, store="f64", fill=7.5)      # sentinel in unwritten rows
    lens0 = [0, 4, 9]
    K = rng.standard_normal((B, cap, HKV, d))
    V = rng.standard_normal((B, cap, HKV, d))
    for b in range(B):                                                        # fill each sequence to its own length
        if lens0[b]:
            O.project_append(O._one_sequence(L, b), K[b:b + 1, :lens0[b]], V[b:b + 1, :lens0[b]], 0)
    # varlen append of 2 rows per sequence at its own offset
    k2 = np.stack([K[b, lens0[b]:lens0[b] + 2] for b in range(B)])
    v2 = np.stack([V[b, lens0[b]:lens0[b] + 2] for b in range(B)])
    O.project_append_varlen(L, k2, v2, lens0)
    lens = [n + 2 for n in lens0]
    for b in range(B):
        assert np.array_equal(L.k_cache[b, :, :lens[b]], np.transpose(K[b, :lens[b]], (1, 0, 2)))
        assert np.all(L.k_cache[b, :, lens[b]:] == 7.5)                        # nothing beyond the new rows
    q = rng.standard_normal((B, HQ, d))
    got = O.decode_attention_varlen(L, q, lens)
    G = HQ // HKV
    kt = torch.from_numpy(np.repeat(np.transpose(K, (0, 2, 1, 3)), G, axis=1))     # [B, HQ, cap, d]
    vt = torch.from_numpy(np.repeat(np.transpose(V, (0, 2, 1, 3)), G, axis=1))
    mask = torch.zeros((B, 1, 1, cap), dtype=torch.bool)
    for b in range(B):
        mask[b, ..., :lens[b]] = True
    want = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, :, None, :], kt, vt,
                                                            attn_mask=mask)[:, :, 0].numpy()
    assert np.max(np.abs(got - want)) < 1e-12
    # a sequence with no rows yields zeros
    assert np.all(O.decode_attention_varlen(L, q, [0, 3, 5])[0] == 0.0)


# ------------------------------------------------- basis construction ----


def test_orthonormal_basis_hand_computed_two_by_two():
    # A = [[3, 1], [4, 2]]: q1 = a1 / 5 = (0.6, 0.8); a2 - <q1, a2> q1 = (1, 2) - 2.2 (0.6, 0.8) = (-0.32, 0.24),
    # of norm 0.4, so q2 = (-0.8, 0.6)  (Gram-Schmidt by hand; Sec. 3.3 Eqs. 13-14)
    Q = O.orthonormal_basis(np.array([[3.0, 1.0], [4.0, 2.0]]), 2)
    assert np.allclose(Q, [[0.6, -0.8], [0.8, 0.6]], atol=1e-15)
    assert np.allclose(O.orthonormal_basis(np.array([[3.0, 1.0], [4.0, 2.0]]), 1), [[0.6], [0.8]], atol=1e-15)
    # negating a column of A must not flip the basis column's sign convention: R_11 stays positive
    Qn = O.orthonormal_basis(np.array([[-3.0, 1.0], [-4.0, 2.0]]), 2)
    assert np.allclose(Qn[:, 0], [-0.6, -0.8], atol=1e-15)


def test_orthonormal_basis_is_the_unique_positive_diagonal_factor():
    """Orthonormal columns, R = Q^T A upper triangular with positive diagonal, Q R = A: together these
    determine Q for a full-rank A, so verifying them pins the routine without calling it twice."""
    rng = np.random.default_rng(5)
    d = 128
    A = rng.standard_normal((3, d, d))
    for r in (1, 16, 77, 128):
        Q = O.orthonormal_basis(A, r)
        assert Q.shape == (3, d, r)
        for i in range(3):
            assert np.max(np.abs(Q[i].T @ Q[i] - np.eye(r))) < 1e-13
            R = Q[i].T @ A[i][:, :r]
            assert np.max(np.abs(np.tril(R, -1))) < 1e-12
            assert np.all(np.diag(R) > 0)
            assert np.max(np.abs(Q[i] @ R - A[i][:, :r])) < 1e-12
            # the projector depends on the span of A's leading columns only (Sec. 3.3)
            Ar = A[i][:, :r]
            proj = Ar @ np.linalg.solve(Ar.T @ Ar, Ar.T)
            assert np.max(np.abs(Q[i] @ Q[i].T - proj)) < 1e-10
    # a matrix that already has orthonormal columns scaled by positive numbers comes back unscaled
    Q0 = _rand_orthogonal(rng, d)
    assert np.max(np.abs(O.orthonormal_basis(Q0 * rng.uniform(0.5, 2.0, d)[None, :], 40) - Q0[:, :40])) < 1e-13
