"""GPU parity of the chunk (prefill) attention over the compressed cache against
the float64 oracle's definition form: every (sequence, token, head) row on
sizes the oracle finishes in seconds, spanning several key tiles, ragged
chunk ends and the causal diagonal."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, Pair, vec_rel_err

pytestmark = pytest.mark.gpu



def _filled_pair(seed, batch, hq, hkv, r_k, r_v, n, **kw):
    P = Pair(seed, batch, hq, hkv, r_k, r_v, n, **kw)
    k, v = P.raw_kv(seed, n, device="cpu")
    P.oracle_append(k, v, 0)
    P.upload_oracle_cache(n)
    return P


def _chunk_q(P, seed, T, width=128):
    return synth.chunk_queries(synth.stable_seed(seed, "cq"), P.batch, T, P.hq, width, P.device)


def _f64(t):
    return O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))


def _gpu_prefill(P, q, n_prev, mode=B.SKV_PREFILL_EXACT, scale=0.0):
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=P.device)
    B.skv_prefill_attention(P.gpu, q, out, n_prev, scale, mode)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("r_k,r_v", [(64, 64), (16, 16), (32, 48), (48, 80), (80, 32), (96, 112),
                                      (112, 96), (128, 128), (16, 128), (128, 16)])
def test_prefill_matches_oracle_across_ranks(r_k, r_v):
    n_prev, T = 150, 75                             # key tiles of 64: several, ragged, diagonal inside
    P = _filled_pair(("pf-ranks", r_k, r_v), 2, 8, 2, r_k, r_v, n_prev + T)
    q = _chunk_q(P, 1, T)
    want = O.prefill_attention(P.ora, _f64(q), n_prev)
    got = _gpu_prefill(P, q, n_prev)
    assert np.all(np.isfinite(got))
    assert vec_rel_err(got, want) <= TOL


@pytest.mark.parametrize("group", [1, 2, 4, 8])
def test_prefill_head_grouping(group):
    hkv, n_prev, T = 2, 40, 150                     # T spans more than one token tile for every grouping
    P = _filled_pair(("pf-group", group), 1, hkv * group, hkv, 48, 80, n_prev + T)
    q = _chunk_q(P, 2, T)
    assert vec_rel_err(_gpu_prefill(P, q, n_prev), O.prefill_attention(P.ora, _f64(q), n_prev)) <= TOL


@pytest.mark.parametrize("n_prev,T", [(0, 1), (0, 2), (0, 31), (0, 32), (0, 33), (0, 64), (0, 65), (0, 200),
                                      (1, 1), (63, 1), (64, 1), (65, 64), (100, 129), (257, 3), (500, 32)])
def test_prefill_chunk_shapes_and_unread_tail(n_prev, T):
    cap = n_prev + T + 70
    P = _filled_pair(("pf-shapes",), 1, 8, 2, 64, 64, cap)
    # rows beyond the chunk hold NaN: no query may see them
    nan = torch.full((1,), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.gpu.k_cache[:, :, n_prev + T:] = nan
    P.gpu.v_cache[:, :, n_prev + T:] = nan
    q = _chunk_q(P, (3, n_prev, T), T)
    got = _gpu_prefill(P, q, n_prev)
    assert np.all(np.isfinite(got))
    assert vec_rel_err(got, O.prefill_attention(P.ora, _f64(q), n_prev)) <= TOL


def test_prefill_is_causal_row_by_row():
    # Changing cache rows after position n_prev + t must not change token t's output, bit for bit.
    n_prev, T = 70, 90
    P = _filled_pair(("pf-causal",), 1, 4, 1, 64, 64, n_prev + T)
    q = _chunk_q(P, 4, T)
    base = _gpu_prefill(P, q, n_prev)
    cut = 37
    P.gpu.k_cache[:, :, n_prev + cut + 1:] *= -3.0
    P.gpu.v_cache[:, :, n_prev + cut + 1:] += 5.0
    again = _gpu_prefill(P, q, n_prev)
    assert np.array_equal(base[:, :cut + 1], again[:, :cut + 1])
    assert not np.array_equal(base[:, cut + 1:], again[:, cut + 1:])


def test_prefill_single_token_equals_decode_reference():
    # T = 1 is the decode step at n_ctx = n_prev + 1 (same oracle definition, other kernel).
    n_prev = 333
    P = _filled_pair(("pf-decode",), 2, 8, 2, 64, 96, n_prev + 1)
    q = _chunk_q(P, 5, 1)
    got = _gpu_prefill(P, q, n_prev)[:, 0]
    want = O.decode_attention(P.ora, _f64(q)[:, 0], n_prev + 1)
    assert vec_rel_err(got, want) <= TOL
    dec = P.gpu_decode(q[:, 0].contiguous(), n_prev + 1)
    assert vec_rel_err(got, dec) <= 1e-4


def test_prefill_strided_queries_scale_and_shared_key_basis():
    n_prev, T = 90, 70
    P = _filled_pair(("pf-strided",), 2, 8, 2, 64, 64, n_prev + T, shared_k=True)
    wide = synth.chunk_queries(7, 2, T, 8, 256, "cuda")
    q = wide[..., 128:]                             # last axis contiguous, other strides doubled
    want = O.prefill_attention(P.ora, _f64(q.contiguous()), n_prev, scale=0.2)
    got = _gpu_prefill(P, q, n_prev, scale=0.2)
    assert vec_rel_err(got, want) <= TOL


@pytest.mark.parametrize("r_k,r_v", [(48, 80), (64, 64), (128, 128), (96, 32)])
def test_prefill_softmax_reference_moves_tile_after_tile(r_k, r_v):
    """The kernel keeps a softmax reference that it moves only when a score exceeds it by 8 (log2 units) and
    rescales its accumulators then.  Ordinary inputs move it once; here the cached keys grow with their position
    (a ramp of 1 .. 9 over the context) and the scale is 7 and 70 times the default, so the largest score of many
    a 64-key tile exceeds the previous reference by more than the threshold (counted on the CPU: up to 10 moves
    per query row), and the early tiles end up far below the last."""
    n_prev, T = 700, 140
    n = n_prev + T
    P = _filled_pair(("pf-ramp", r_k, r_v), 1, 8, 2, r_k, r_v, n)
    ramp = 1.0 + 8.0 * np.arange(n, dtype=np.float64) / n
    kb = O.f64_to_bf16_bits(P.ora.k_cache[:, :, :n] * ramp[None, None, :, None])
    P.ora.k_cache[:, :, :n] = O.bf16_bits_to_f64(kb)            # the oracle holds what the bf16 cache holds
    P.upload_oracle_cache(n)
    q = _chunk_q(P, 12, T)
    for scale in (0.6, 6.0):                           # scores up to +-90 and +-900: 3 .. 10 moves per query row
        want = O.prefill_attention(P.ora, _f64(q), n_prev, scale=scale)
        got = _gpu_prefill(P, q, n_prev, scale=scale)
        assert np.all(np.isfinite(got))
        assert vec_rel_err(got, want) <= TOL, scale


def test_prefill_has_no_reduced_precision_mode():
    """Bit 0 of mode once selected single-term bf16 operands; it is rejected now (each operand fed as one
    bf16 term breaks the 2e-3 bound by itself, tests/test_prefill_operand_rounding.py)."""
    n_prev, T = 300, 100
    P = _filled_pair(("pf-fast",), 2, 8, 2, 64, 64, n_prev + T)
    q = _chunk_q(P, 8, T)
    with pytest.raises(B.SkvError) as e:
        _gpu_prefill(P, q, n_prev, mode=1)
    assert e.value.code == B.SKV_ERR_SHAPE


@pytest.mark.parametrize("r_k,r_v,group", [(64, 64, 4), (48, 80, 2), (128, 32, 1)])
def test_prefill_folded_matches_oracle(r_k, r_v, group):
    hkv, n_prev, T = 2, 100, 90
    P = _filled_pair(("pf-folded", r_k, r_v), 2, hkv * group, hkv, r_k, r_v, n_prev + T)
    q_low = _chunk_q(P, 9, T, width=r_k)
    want = O.prefill_attention_folded(P.ora, _f64(q_low), n_prev)
    out = torch.full((2, T, hkv * group, r_v), float("nan"), dtype=torch.float32, device="cuda")
    B.skv_prefill_attention_folded(P.gpu, q_low, out, n_prev)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    assert vec_rel_err(got, want) <= TOL


def test_prefill_step_equals_append_then_attention():
    n_prev, T = 130, 100
    P = Pair(("pf-step",), 2, 8, 2, 48, 80, n_prev + T)
    k, v = P.raw_kv(1, n_prev + T)
    q = _chunk_q(P, 10, T)
    B.skv_project_append(P.gpu, k[:, :n_prev], v[:, :n_prev], 0)
    out_step = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    B.skv_prefill_step(P.gpu, k[:, n_prev:], v[:, n_prev:], q, out_step, n_prev)
    torch.cuda.synchronize()
    kc, vc = P.gpu.k_cache.clone(), P.gpu.v_cache.clone()
    P2 = Pair(("pf-step",), 2, 8, 2, 48, 80, n_prev + T)
    B.skv_project_append(P2.gpu, k, v, 0)
    out_two = torch.empty_like(out_step)
    B.skv_prefill_attention(P2.gpu, q, out_two, n_prev)
    torch.cuda.synchronize()
    assert torch.equal(kc.view(torch.int16), P2.gpu.k_cache.view(torch.int16))
    assert torch.equal(vc.view(torch.int16), P2.gpu.v_cache.view(torch.int16))
    assert torch.equal(out_step, out_two)
    # end to end against the oracle (its own float64 append)
    P.oracle_append(k.cpu(), v.cpu(), 0)
    want = O.prefill_attention(P.ora, _f64(q), n_prev)
    assert vec_rel_err(out_step.cpu().numpy(), want) <= TOL


def test_prefill_rejects_bad_arguments_without_writing():
    P = _filled_pair(("pf-bad",), 1, 8, 2, 64, 64, 64)
    q = _chunk_q(P, 11, 16)
    out = torch.full(q.shape, 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(B.SkvError) as e:
        B.skv_prefill_attention(P.gpu, q, out, 60)              # 60 + 16 > capacity
    assert e.value.code == B.SKV_ERR_CAPACITY
    with pytest.raises(B.SkvError) as e:
        B.skv_prefill_attention(P.gpu, q, out, 0, mode=5)
    assert e.value.code == B.SKV_ERR_SHAPE
    with pytest.raises(B.SkvError) as e:
        B.skv_prefill_attention(P.gpu, q.view(-1)[4:4 + 8 * 128 * 8].view(1, 8, 8, 128), out[:, :8].contiguous(), 0)
    assert e.value.code == B.SKV_ERR_ALIGN
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)


def test_prefill_deterministic():
    n_prev, T = 200, 130
    P = _filled_pair(("pf-det",), 2, 8, 2, 64, 64, n_prev + T)
    q = _chunk_q(P, 12, T)
    a = _gpu_prefill(P, q, n_prev)
    b = _gpu_prefill(P, q, n_prev)
    assert np.array_equal(a, b)
