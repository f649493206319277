"""Ranks that are not multiples of 16 (the paper's 50-90 % grid: 77, 90, 102, 115 for head_dim 128),
served through zero-padded bases: the GPU path with the padded basis against the oracle with the
UNPADDED basis."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, vec_rel_err

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("decode_engine")]


def _f64(t):
    return O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))


@pytest.mark.parametrize("r_k,r_v", [(77, 90), (102, 115), (5, 33), (64, 77)])
def test_padded_bases_match_the_oracle_at_the_true_rank(r_k, r_v):
    batch, hq, hkv, n, T = 2, 8, 2, 900, 3
    _, pk = synth.orthonormal_bases(synth.stable_seed("pad", r_k, "k"), hkv, 128, r_k)
    _, pv = synth.orthonormal_bases(synth.stable_seed("pad", r_v, "v"), hkv, 128, r_v)
    pk_pad, pv_pad = B.skv_pad_basis(pk.cuda()), B.skv_pad_basis(pv.cuda())
    rkp, rvp = B.skv_padded_rank(r_k), B.skv_padded_rank(r_v)
    assert pk_pad.shape == (hkv, 128, rkp) and pv_pad.shape == (hkv, 128, rvp)
    # the padding itself: a bit-exact copy followed by zero columns
    assert torch.equal(pk_pad[..., :r_k].cpu().view(torch.int16), pk.view(torch.int16))
    assert torch.all(pk_pad[..., r_k:].view(torch.int16) == 0) and torch.all(pv_pad[..., r_v:].view(torch.int16) == 0)

    L = B.Layer(batch, hq, hkv, pk_pad, pv_pad, n)
    sc = synth.channel_scales(3, hkv, 128)
    k = synth.kv_activations(4, batch, n, hkv, 128, sc, "cuda")
    v = synth.kv_activations(5, batch, n, hkv, 128, sc, "cuda")
    q = synth.queries(6, batch, hq, 128, "cuda")
    B.skv_project_append(L, k[:, :n - T], v[:, :n - T], 0)                 # chunk path
    out = torch.empty((batch, hq, 128), dtype=torch.float32, device="cuda")
    B.skv_decode_step(L, k[:, n - T:], v[:, n - T:], n - T, q, out)        # fused step
    torch.cuda.synchronize()
    # padded channels of the cache hold exact zeros
    assert torch.all(L.k_cache[..., r_k:].view(torch.int16) == 0) and torch.all(L.v_cache[..., r_v:].view(torch.int16) == 0)

    ora = O.new_layer(batch, hq, hkv, 128, _f64(pk), _f64(pv), n, store="bf16")   # true ranks, no padding
    O.project_append(ora, _f64(k), _f64(v), 0)
    want = O.decode_attention(ora, _f64(q), n)
    assert vec_rel_err(out.cpu().numpy(), want) <= TOL
    # a chunk of queries over the same cache
    cq = synth.chunk_queries(7, batch, 40, hq, 128, "cuda")
    pout = torch.empty((batch, 40, hq, 128), dtype=torch.float32, device="cuda")
    B.skv_prefill_attention(L, cq, pout, n - 40)
    torch.cuda.synchronize()
    assert vec_rel_err(pout.cpu().numpy(), O.prefill_attention(ora, _f64(cq), n - 40)) <= TOL
