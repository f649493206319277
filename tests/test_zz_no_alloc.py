"""The entry point that allocates nothing (skv_decode_attention_static: the library's static device scratch
array in place of a caller's workspace) against the entry point it is a variant of, through the C ABI: two
calls in a row on one GPU, the second on a smaller input, each bit-equal to skv_decode_attention and within
the stated bound of the oracle; and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2601_21686_amd import binding as B
from _helpers import TOL, Pair, vec_rel_err

pytestmark = pytest.mark.gpu


def _filled(seed, batch, hq, hkv, r_k, r_v, n):
    P = Pair(seed, batch, hq, hkv, r_k, r_v, n)
    k, v = P.raw_kv(1, n)
    B.skv_project_append(P.gpu, k, v, 0)
    P.oracle_append(k, v, 0)
    torch.cuda.synchronize()
    return P


def _both(P, q, n_ctx):
    """(static-scratch output, workspace output) of the same attention call, through the raw C ABI."""
    lib = B.lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    a = torch.full((P.batch, P.hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    b = torch.full_like(a, float("nan"))
    st = lib.skv_decode_attention_static(C.byref(P.gpu.c), q.data_ptr(), a.data_ptr(), n_ctx, 0.0, stream)
    assert st == B.SKV_OK, B.status_string(st)
    ws = P.gpu.workspace()
    st = lib.skv_decode_attention(C.byref(P.gpu.c), q.data_ptr(), b.data_ptr(), n_ctx, 0.0, ws.data_ptr(),
                                  ws.numel(), stream)
    assert st == B.SKV_OK, B.status_string(st)
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy()


def test_static_scratch_attention_twice_in_a_row_second_call_smaller():
    big = _filled("na-big", 4, 32, 8, 64, 96, 3000)          # 16 ranges per (sequence, KV head)
    small = _filled("na-small", 1, 8, 2, 48, 32, 333)        # fewer heads, lower ranks, fewer ranges: a smaller footprint
    q_big, q_small = big.queries(2), small.queries(3)
    a, b = _both(big, q_big, 3000)
    assert np.array_equal(a, b)
    assert vec_rel_err(a, big.oracle_decode(q_big, 3000)) <= TOL
    # the second call finds the first one's partial results in the scratch array and must not see them
    a, b = _both(small, q_small, 333)
    assert np.array_equal(a, b)
    assert vec_rel_err(a, small.oracle_decode(q_small, 333)) <= TOL
    # and once more on a shorter context of the first layer
    a, b = _both(big, q_big, 65)
    assert np.array_equal(a, b)
    assert vec_rel_err(a, big.oracle_decode(q_big, 65)) <= TOL


def test_static_scratch_rejects_what_does_not_fit():
    # 64 sequences x 64 query heads at ranks 128: the projected queries alone take 2 MiB, one partial result per
    # head another 2.1 MiB -- more than the 4 MiB array.  Rejected on the host; nothing is launched.
    dev = "cuda"
    pk = torch.zeros((1, 128, 128), dtype=torch.bfloat16, device=dev)
    L = B.Layer(64, 64, 8, pk, pk, 64)
    q = torch.zeros((64, 64, 128), dtype=torch.bfloat16, device=dev)
    out = torch.full((64, 64, 128), 7.0, dtype=torch.float32, device=dev)
    st = B.lib().skv_decode_attention_static(C.byref(L.c), q.data_ptr(), out.data_ptr(), 64, 0.0, None)
    assert st == B.SKV_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
