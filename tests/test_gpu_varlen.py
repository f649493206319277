"""Per-sequence lengths on the GPU against the oracle: a batch whose sequences have different
contexts (one of them empty), through the attention call, the append and the fused decode step."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, Pair, vec_rel_err

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("decode_engine")]
SENTINEL = 0x7FC1                     # a NaN pattern: anything that reads an unwritten row shows


def _f64(t):
    return O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))


def _lens_t(lens):
    return torch.tensor(lens, dtype=torch.int32, device="cuda")


def _ragged_pair(seed, lens, hq, hkv, r_k, r_v, cap):
    """Both sides filled per sequence to its own length through the oracle's append; NaN elsewhere on the GPU."""
    P = Pair(seed, len(lens), hq, hkv, r_k, r_v, cap, fill_bits=SENTINEL)
    k, v = P.raw_kv(seed, cap, device="cpu")
    for b, n in enumerate(lens):
        if n:
            O.project_append(O._one_sequence(P.ora, b), _f64(k[b:b + 1, :n]), _f64(v[b:b + 1, :n]), 0)
            P.gpu.k_cache[b, :, :n] = synth.bits_to_torch_bf16(O.f64_to_bf16_bits(P.ora.k_cache[b, :, :n]), "cuda")
            P.gpu.v_cache[b, :, :n] = synth.bits_to_torch_bf16(O.f64_to_bf16_bits(P.ora.v_cache[b, :, :n]), "cuda")
    return P, k, v


@pytest.mark.parametrize("lens", [[1, 77, 700, 1500], [1500, 0, 64, 63], [5, 5, 5, 5]])
@pytest.mark.parametrize("hq,hkv,r_k,r_v", [(8, 2, 64, 64), (4, 4, 48, 80)])
def test_decode_attention_with_per_sequence_lengths(lens, hq, hkv, r_k, r_v):
    P, _, _ = _ragged_pair(("vl", tuple(lens), r_k), lens, hq, hkv, r_k, r_v, 1500)
    q = P.queries(1)
    out = torch.full((len(lens), hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    B.skv_decode_attention_varlen(P.gpu, q, out, _lens_t(lens), 1500)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = O.decode_attention_varlen(P.ora, _f64(q), lens)
    assert np.all(np.isfinite(got))                       # rows beyond each length hold NaN: never read
    for b, n in enumerate(lens):
        if n == 0:
            assert np.all(got[b] == 0.0)
        else:
            assert vec_rel_err(got[b], want[b]) <= TOL


def test_lengths_are_clamped_to_the_host_bound():
    lens = [300, 200]
    P, _, _ = _ragged_pair(("vl-clamp",), lens, 8, 2, 64, 64, 400)
    q = P.queries(2)
    out = torch.empty((2, 8, 128), dtype=torch.float32, device="cuda")
    B.skv_decode_attention_varlen(P.gpu, q, out, _lens_t([100000, -7]), 300)      # device garbage: clamped to [0, 300]
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = O.decode_attention_varlen(P.ora, _f64(q), [300, 0])
    assert vec_rel_err(got[0], want[0]) <= TOL and np.all(got[1] == 0.0)


@pytest.mark.parametrize("T", [1, 3, 9, 150])                                     # fused step, few-token and chunk appends
def test_decode_step_with_per_sequence_lengths(T):
    lens = [0, 130, 1, 900]
    cap = 900 + T
    P, k, v = _ragged_pair(("vl-step", T), lens, 8, 2, 64, 96, cap)
    k1 = synth.kv_activations(11, 4, T, 2, 128, P.scales_k, "cuda")
    v1 = synth.kv_activations(12, 4, T, 2, 128, P.scales_v, "cuda")
    q = P.queries(3)
    out = torch.full((4, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    B.skv_decode_step_varlen(P.gpu, k1, v1, _lens_t(lens), 900, q, out)
    torch.cuda.synchronize()
    O.project_append_varlen(P.ora, _f64(k1), _f64(v1), lens)
    new_lens = [n + T for n in lens]
    gk = synth.torch_bf16_to_bits(P.gpu.k_cache)
    gv = synth.torch_bf16_to_bits(P.gpu.v_cache)
    for b, n in enumerate(new_lens):
        # placement: new rows where the oracle put them (bits equal up to float32-vs-float64 rounding
        # straddles), every later row still the sentinel
        assert (gk[b, :, lens[b]:n] != O.f64_to_bf16_bits(P.ora.k_cache[b, :, lens[b]:n])).mean() < 0.01
        assert (gv[b, :, lens[b]:n] != O.f64_to_bf16_bits(P.ora.v_cache[b, :, lens[b]:n])).mean() < 0.01
        assert np.all(gk[b, :, n:] == SENTINEL) and np.all(gv[b, :, n:] == SENTINEL)
    got = out.cpu().numpy()
    want = O.decode_attention_varlen(P.ora, _f64(q), new_lens)
    assert np.all(np.isfinite(got))
    assert vec_rel_err(got, want) <= TOL


def test_append_with_per_sequence_offsets_is_bit_exact_with_selection_bases():
    batch, hkv, T, r = 3, 2, 70, 32                       # 210 token rows: the matrix-core path
    lens = [0, 17, 333]
    cap = 333 + T + 5
    _, pk, idx_k, sgn_k = synth.selection_bases(1, hkv, 128, r)
    _, pv, idx_v, sgn_v = synth.selection_bases(2, hkv, 128, r)
    kc = torch.full((batch, hkv, cap, r), SENTINEL, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    vc = torch.full((batch, hkv, cap, r), SENTINEL, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    L = B.Layer(batch, 4, hkv, pk.cuda(), pv.cuda(), cap, kc, vc)
    sc = synth.channel_scales(3, hkv, 128)
    k = synth.kv_activations(4, batch, T, hkv, 128, sc, "cuda")
    v = synth.kv_activations(5, batch, T, hkv, 128, sc, "cuda")
    B.skv_project_append_varlen(L, k, v, _lens_t(lens), 333)
    torch.cuda.synchronize()
    kf, vf = _f64(k), _f64(v)
    gk, gv = _f64(L.k_cache), _f64(L.v_cache)
    bits = synth.torch_bf16_to_bits(L.k_cache)
    for b, n in enumerate(lens):
        for h in range(hkv):
            assert np.array_equal(gk[b, h, n:n + T], kf[b, :, h][:, idx_k[h]] * sgn_k[h])
            assert np.array_equal(gv[b, h, n:n + T], vf[b, :, h][:, idx_v[h]] * sgn_v[h])
        assert np.all(bits[b, :, :n] == SENTINEL) and np.all(bits[b, :, n + T:] == SENTINEL)
