"""GPU parity of projection + append against the oracle: placement is
bit-exact, values are within one bf16 step (float32 vs float64 accumulation
can straddle a rounding boundary), for both the vector and the MFMA kernel."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, Pair, bf16_ulp_distance, vec_rel_err

pytestmark = pytest.mark.gpu

SENTINEL = 0x7FC1          # a NaN pattern no projection produces


def _check_append(P, k, v, cur, T):
    """Placement must be exact.  Values: the GPU rounds a float32 sum, the oracle a
    float64 sum.  With u = 2^-24 and 128 exact products the float32 sum is within
    128*u*sum|x_i p_i| of the exact one, then rounded once to bf16 (half a step):
    that is the bound checked per element, against the oracle's unrounded float64
    sum; and the stored bits must equal the oracle's bf16 bits except where the two
    sums straddle a rounding boundary (well under 1 % of entries)."""
    B.skv_project_append(P.gpu, k, v, cur)
    torch.cuda.synchronize()
    P.oracle_append(k.cpu(), v.cpu(), cur)
    exact = O.new_layer(P.batch, P.hq, P.hkv, 128, P.ora.p_k, P.ora.p_v, P.capacity, store="f64")
    kf = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(k))
    vf = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(v))
    O.project_append(exact, kf, vf, cur)
    mag = O.new_layer(P.batch, P.hq, P.hkv, 128, np.abs(P.ora.p_k), np.abs(P.ora.p_v), P.capacity, store="f64")
    O.project_append(mag, np.abs(kf), np.abs(vf), cur)
    for gpu_c, ora_c, ex_c, mag_c in ((P.gpu.k_cache, P.ora.k_cache, exact.k_cache, mag.k_cache),
                                      (P.gpu.v_cache, P.ora.v_cache, exact.v_cache, mag.v_cache)):
        got = synth.torch_bf16_to_bits(gpu_c)
        sl = slice(cur, cur + T)
        want = O.f64_to_bf16_bits(ora_c[:, :, sl])
        assert (got[:, :, sl] != want).mean() < 0.01
        g = O.bf16_bits_to_f64(got[:, :, sl])
        e = ex_c[:, :, sl]
        slack = 128 * 2.0 ** -24 * mag_c[:, :, sl]
        step = np.ldexp(1.0, np.floor(np.log2(np.maximum(np.abs(e) + slack, 1e-300))).astype(int) - 7)
        assert np.all(np.abs(g - e) <= slack + step / 2)
        untouched = np.ones(P.capacity, bool)
        untouched[sl] = False
        assert np.all(got[:, :, untouched] == SENTINEL)


@pytest.mark.parametrize("batch,T,cur", [(1, 1, 0), (4, 1, 37), (1, 16, 1024), (2, 32, 5),     # vector kernel
                                         (3, 100, 11), (2, 256, 0), (5, 77, 300), (1, 65, 1)])  # MFMA kernel
@pytest.mark.parametrize("r_k,r_v", [(64, 64), (48, 80), (16, 128), (112, 32)])
def test_append_values_and_placement(batch, T, cur, r_k, r_v):
    P = Pair(("app", batch, T, r_k), batch, 8, 4, r_k, r_v, cur + T + 9, fill_bits=SENTINEL)
    k, v = P.raw_kv(1, T)
    _check_append(P, k, v, cur, T)


@pytest.mark.parametrize("batch,T,cur", [(2, 20000, 3), (1, 49153, 0)])
def test_append_of_a_chunk_that_gives_waves_three_tiles(batch, T, cur):
    """The chunk kernel runs at most 64 workgroups per head, each wave taking every 16384th block of 64 tokens in
    turns of two: 40000 rows give some waves three tiles (a second turn whose second tile lies past the end) and
    the others two; 49153 rows give one wave a fourth tile of a single row."""
    P = Pair(("app-long", batch, T), batch, 8, 4, 48, 80, cur + T + 9, fill_bits=SENTINEL)
    k, v = P.raw_kv(1, T)
    _check_append(P, k, v, cur, T)


@pytest.mark.parametrize("batch,T", [(2, 3), (2, 200)])
def test_append_is_bit_exact_with_selection_bases(batch, T):
    # bases that pick +-channels: the cache must be an exact copy of those channels
    hkv, r_k, r_v, cur, cap = 4, 48, 80, 13, 260
    _, pk, idx_k, sgn_k = synth.selection_bases(11, hkv, 128, r_k)
    _, pv, idx_v, sgn_v = synth.selection_bases(12, hkv, 128, r_v)
    kc = torch.full((batch, hkv, cap, r_k), SENTINEL, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    vc = torch.full((batch, hkv, cap, r_v), SENTINEL, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    L = B.Layer(batch, hkv, hkv, pk.cuda(), pv.cuda(), cap, kc, vc)
    # small integers exactly representable in bf16 that encode (b, t, h, channel)
    b_, t_, h_, c_ = np.meshgrid(np.arange(batch), np.arange(T), np.arange(hkv), np.arange(128), indexing="ij")
    kf = ((b_ * 7 + t_ * 3 + h_ * 5 + c_) % 251 - 125).astype(np.float64)
    vf = ((b_ * 11 + t_ * 5 + h_ * 3 + c_ * 2) % 241 - 120).astype(np.float64)
    k = synth.f64_to_torch_bf16(kf, "cuda")
    v = synth.f64_to_torch_bf16(vf, "cuda")
    B.skv_project_append(L, k, v, cur)
    torch.cuda.synchronize()
    gk = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(L.k_cache[:, :, cur:cur + T]))
    gv = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(L.v_cache[:, :, cur:cur + T]))
    for h in range(hkv):
        assert np.array_equal(gk[:, h], kf[:, :, h][:, :, idx_k[h]] * sgn_k[h])
        assert np.array_equal(gv[:, h], vf[:, :, h][:, :, idx_v[h]] * sgn_v[h])
    rest = np.ones(cap, bool)
    rest[cur:cur + T] = False
    assert np.all(synth.torch_bf16_to_bits(L.k_cache)[:, :, rest] == SENTINEL)
    assert np.all(synth.torch_bf16_to_bits(L.v_cache)[:, :, rest] == SENTINEL)


def test_append_from_a_strided_view():
    # keys and values interleaved in one [b, t, 2, h, d] buffer, as a fused QKV projection leaves them
    batch, T, hkv = 2, 70, 4
    P = Pair(("strided",), batch, 8, hkv, 64, 64, 100, fill_bits=SENTINEL)
    k0, v0 = P.raw_kv(2, T)
    both = torch.stack([k0, v0], dim=2).contiguous()
    k, v = both[:, :, 0], both[:, :, 1]
    assert not k.is_contiguous()
    _check_append(P, k, v, 20, T)


def test_append_then_decode_end_to_end():
    # config-1 shape: batch 1, context 1024 reached by a 16-token append, then one decode step
    P = Pair(("e2e",), 1, 32, 8, 64, 64, 1024)
    k, v = P.raw_kv(3, 1008)
    B.skv_project_append(P.gpu, k, v, 0)
    P.oracle_append(k.cpu(), v.cpu(), 0)
    k2, v2 = P.raw_kv(4, 16)
    B.skv_project_append(P.gpu, k2, v2, 1008)
    P.oracle_append(k2.cpu(), v2.cpu(), 1008)
    q = P.queries(5)
    got = P.gpu_decode(q, 1024)
    want = P.oracle_decode(q, 1024)
    assert vec_rel_err(got, want) <= TOL


def test_zero_token_append_is_a_noop():
    P = Pair(("noop",), 1, 4, 1, 64, 64, 8, fill_bits=SENTINEL, oracle=False)
    k, v = P.raw_kv(1, 1)
    B.skv_project_append(P.gpu, k[:, :0], v[:, :0], 8)
    torch.cuda.synchronize()
    assert np.all(synth.torch_bf16_to_bits(P.gpu.k_cache) == SENTINEL)
