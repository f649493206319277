"""Pins of the oracle's paged-cache functions: they only say where a row lives, so the pins are
a hand-labelled pool, the identity table and the invariance of every result under a
relabelling of the pool's pages."""
import numpy as np
import pytest

from oracle import skv_oracle as O
from paper_2601_21686_amd import synth


def _labelled_pool(n_pages, heads, page_tokens, r):
    """Entry (page, head, row, channel) holds 1000 page + 100 head + row + channel / 100."""
    pg, h, t, c = np.meshgrid(np.arange(n_pages), np.arange(heads), np.arange(page_tokens), np.arange(r), indexing="ij")
    return (1000.0 * pg + 100.0 * h + t + c / 100.0)


def test_gather_on_a_hand_labelled_pool():
    pool = _labelled_pool(5, 2, 4, 3)
    table = [3, 0, 4]                       # logical pages 0, 1, 2 of the sequence
    got = O.paged_rows(pool, table, 4, 10)
    # rows 0..3 in page 3, rows 4..7 in page 0, rows 8..9 in page 4; written out by hand for head 1, channel 2
    want_h1_c2 = [3100.02, 3101.02, 3102.02, 3103.02, 100.02, 101.02, 102.02, 103.02, 4100.02, 4101.02]
    assert got.shape == (2, 10, 3)
    assert np.allclose(got[1, :, 2], want_h1_c2, rtol=0, atol=1e-9)
    assert np.allclose(got[0, :, 0], [3000, 3001, 3002, 3003, 0, 1, 2, 3, 4000, 4001])


def test_identity_table_is_a_reshape():
    pool = _labelled_pool(6, 2, 8, 3)
    got = O.paged_rows(pool, np.arange(6), 8, 48)
    want = np.transpose(pool, (1, 0, 2, 3)).reshape(2, 48, 3)
    assert np.array_equal(got, want)


def test_store_touches_exactly_the_named_rows():
    pool = np.full((4, 2, 4, 3), -1.0)
    rows = np.arange(2 * 5 * 3, dtype=np.float64).reshape(2, 5, 3)
    O.paged_store_rows(pool, [2, 1, 3], 4, 3, rows)       # rows 3..7: last row of page 2, all of page 1
    assert np.array_equal(pool[2, :, 3], rows[:, 0])
    assert np.array_equal(pool[1].transpose(1, 0, 2), rows[:, 1:5].transpose(1, 0, 2))
    assert np.all(pool[0] == -1) and np.all(pool[3] == -1) and np.all(pool[2, :, :3] == -1)
    assert np.array_equal(O.paged_rows(pool, [2, 1, 3], 4, 8)[:, 3:8], rows)


def _setup(seed, batch, hq, hkv, r_k, r_v, page_tokens, n_pages, max_pages, store="f64"):
    _, pk = synth.orthonormal_bases(synth.stable_seed(seed, "pk"), hkv, 128, r_k)
    _, pv = synth.orthonormal_bases(synth.stable_seed(seed, "pv"), hkv, 128, r_v)
    f = lambda t: O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))
    layer = O.new_layer(batch, hq, hkv, 128, f(pk), f(pv), page_tokens * max_pages, store)
    rng = np.random.default_rng(synth.stable_seed(seed, "table"))
    table = rng.permutation(n_pages)[:batch * max_pages].reshape(batch, max_pages)
    cache = O.OraclePagedCache(np.zeros((n_pages, hkv, page_tokens, r_k)), np.zeros((n_pages, hkv, page_tokens, r_v)),
                               table, page_tokens)
    return layer, cache, rng


@pytest.mark.parametrize("store", ["f64", "bf16"])
def test_paged_append_and_attention_equal_the_contiguous_layer(store):
    # the same tokens appended to a contiguous layer and, in three chunks that straddle pages, to a paged one
    batch, hq, hkv, pt = 2, 4, 2, 8
    layer, cache, rng = _setup(("paged", store), batch, hq, hkv, 32, 48, pt, 16, 4, store)
    n = 27
    k = rng.standard_normal((batch, n, hkv, 128))
    v = rng.standard_normal((batch, n, hkv, 128))
    O.project_append(layer, k, v, 0)
    cur = np.zeros(batch, int)
    for a, b_ in ((0, 5), (5, 18), (18, 27)):
        O.paged_project_append(layer, cache, k[:, a:b_], v[:, a:b_], cur)
        cur += b_ - a
    flat = O.paged_as_contiguous(layer, cache, [n, n])
    assert np.array_equal(flat.k_cache[:, :, :n], layer.k_cache[:, :, :n])
    assert np.array_equal(flat.v_cache[:, :, :n], layer.v_cache[:, :, :n])
    q = rng.standard_normal((batch, hq, 128))
    lens = [27, 9]
    assert np.array_equal(O.paged_decode_attention(layer, cache, q, lens), O.decode_attention_varlen(layer, q, lens))
    qc = rng.standard_normal((batch, 6, hq, 128))
    assert np.array_equal(O.paged_prefill_attention(layer, cache, qc, 21), O.prefill_attention(layer, qc, 21))


def test_paged_folded_functions_equal_the_contiguous_ones_and_the_explicit_path():
    # rows handed over already projected land where the projecting append puts them, and attention in the
    # compressed space over the pages equals the contiguous one; lifted, it is the explicit attention
    batch, hq, hkv, pt, r_k, r_v = 2, 4, 2, 8, 32, 48
    layer, cache, rng = _setup(("paged-folded",), batch, hq, hkv, r_k, r_v, pt, 16, 4, "f64")
    n = 21
    k = rng.standard_normal((batch, n, hkv, 128))
    v = rng.standard_normal((batch, n, hkv, 128))
    O.project_append(layer, k, v, 0)
    k_low = np.einsum("bthd,hdc->bthc", k, layer.p_k)
    v_low = np.einsum("bthd,hdc->bthc", v, layer.p_v)
    cur = np.zeros(batch, int)
    for a, b_ in ((0, 7), (7, 8), (8, 21)):
        O.paged_append_projected(layer, cache, k_low[:, a:b_], v_low[:, a:b_], cur)
        cur += b_ - a
    flat = O.paged_as_contiguous(layer, cache, [n, n])
    assert np.allclose(flat.k_cache[:, :, :n], layer.k_cache[:, :, :n], rtol=0, atol=1e-12)
    assert np.allclose(flat.v_cache[:, :, :n], layer.v_cache[:, :, :n], rtol=0, atol=1e-12)
    q = rng.standard_normal((batch, hq, 128))
    q_low = np.einsum("bgd,gdc->bgc", q, np.repeat(layer.p_k, hq // hkv, axis=0))
    lens = [21, 6]
    got = O.paged_decode_attention_folded(layer, cache, q_low, lens)
    for b in range(batch):
        want = O.decode_attention_folded(O._one_sequence(flat, b), q_low[b:b + 1], lens[b])[0]
        assert np.array_equal(got[b], want)
    lifted = np.einsum("bgc,gdc->bgd", got, np.repeat(layer.p_v, hq // hkv, axis=0))
    assert np.allclose(lifted, O.decode_attention_varlen(layer, q, lens), rtol=1e-11, atol=1e-13)
    assert np.all(O.paged_decode_attention_folded(layer, cache, q_low, [0, 3])[0] == 0.0)


def test_results_do_not_depend_on_which_pool_page_holds_a_row():
    batch, hq, hkv, pt = 2, 4, 2, 8
    layer, cache, rng = _setup(("relabel",), batch, hq, hkv, 32, 32, pt, 12, 3)
    n = 20
    k = rng.standard_normal((batch, n, hkv, 128))
    v = rng.standard_normal((batch, n, hkv, 128))
    O.paged_project_append(layer, cache, k, v, [0, 0])
    q = rng.standard_normal((batch, hq, 128))
    base = O.paged_decode_attention(layer, cache, q, [20, 13])
    perm = rng.permutation(12)                       # page i moves to page perm[i]
    moved = O.OraclePagedCache(np.empty_like(cache.k_pool), np.empty_like(cache.v_pool), perm[cache.block_table], pt)
    moved.k_pool[perm] = cache.k_pool
    moved.v_pool[perm] = cache.v_pool
    assert np.array_equal(O.paged_decode_attention(layer, moved, q, [20, 13]), base)
    # and they do depend on the table: swapping two logical pages of a sequence changes its result
    swapped = O.OraclePagedCache(cache.k_pool, cache.v_pool, cache.block_table.copy(), pt)
    swapped.block_table[0, [0, 1]] = swapped.block_table[0, [1, 0]]
    qc = rng.standard_normal((batch, 3, hq, 128))
    other = O.paged_prefill_attention(layer, swapped, qc, 17)
    same = O.paged_prefill_attention(layer, cache, qc, 17)
    assert not np.allclose(O.paged_rows(swapped.k_pool, swapped.block_table[0], pt, 16),
                           O.paged_rows(cache.k_pool, cache.block_table[0], pt, 16))
    # attention over a set of rows does not care about their order, except through the causal mask: the
    # chunk's own rows sit in logical page 2, so sequence 0 is unchanged by a swap of pages 0 and 1 ...
    assert np.allclose(other, same, rtol=0, atol=1e-12)
    # ... but a swap that moves rows across the causal boundary changes it
    swapped.block_table[0, [0, 2]] = swapped.block_table[0, [2, 0]]
    assert not np.allclose(O.paged_prefill_attention(layer, swapped, qc, 17)[0], same[0])


@pytest.mark.parametrize("bits", [8, 4])
def test_paged_quantised_functions_equal_the_contiguous_quantised_layer(bits):
    # quantised pages: the same codes and value ranges, found through the table
    batch, hq, hkv, pt, r = 2, 4, 2, 8, 64
    _, pk = synth.orthonormal_bases(synth.stable_seed("pq", "pk"), hkv, 128, r)
    _, pv = synth.orthonormal_bases(synth.stable_seed("pq", "pv"), hkv, 128, r)
    f = lambda t: O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))
    ks, kz = np.full((hkv, 1), 0.05, np.float32), np.full((hkv, 1), -5.0, np.float32)
    flat = O.new_quant_layer(batch, hq, hkv, 128, f(pk), f(pv), ks, kz, 32, bits)
    rng = np.random.default_rng(5)
    table = rng.permutation(12)[:8].reshape(2, 4)
    shape = (12, hkv, pt)
    cache = O.OraclePagedQuantCache(np.zeros(shape + (r,), np.uint8), np.zeros(shape + (r,), np.uint8),
                                    np.zeros(shape + (1,), np.uint16), np.zeros(shape + (1,), np.uint16), table, pt)
    n = 27
    k, v = rng.standard_normal((batch, n, hkv, 128)), rng.standard_normal((batch, n, hkv, 128))
    O.quant_project_append(flat, k, v, 0)
    cur = np.zeros(batch, int)
    for a, b_ in ((0, 5), (5, 18), (18, 27)):
        O.paged_quant_project_append(flat, cache, k[:, a:b_], v[:, a:b_], cur)
        cur += b_ - a
    for b in range(batch):
        assert np.array_equal(O.paged_rows(cache.k_codes, table[b], pt, n), flat.k_codes[b, :, :n])
        assert np.array_equal(O.paged_rows(cache.v_codes, table[b], pt, n), flat.v_codes[b, :, :n])
        assert np.array_equal(O.paged_rows(cache.v_scale_bits, table[b], pt, n), flat.v_scale_bits[b, :, :n])
        assert np.array_equal(O.paged_rows(cache.v_zero_bits, table[b], pt, n), flat.v_zero_bits[b, :, :n])
    q = rng.standard_normal((batch, hq, 128))
    got = O.paged_quant_decode_attention(flat, cache, q, [27, 9])
    assert np.array_equal(got[0], O.quant_decode_attention(flat, q, 27)[0])
    assert np.array_equal(got[1], O.quant_decode_attention(flat, q, 9)[1])
