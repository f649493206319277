"""CPU-side checks of the C-ABI library: it loads, exports every function the
header declares, rejects bad arguments before launching anything, and its
host-only rank selection agrees with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libskv.so not built")
# A build of the host layer alone (SKV_LIBRARY, see test_host_sanitizers.py) holds no .hip translation unit:
# the entry point that lives in one is absent there.
HOST_ONLY = bool(os.environ.get("SKV_LIBRARY"))


def _declared_functions(header="skv.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(skv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n) or (HOST_ONLY and n == "skv_decode_attention_static"), n


def test_every_header_is_covered_and_the_probe_library_exports_its_own():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["skv.h", "skv_probe.h"]
    names = _declared_functions("skv_probe.h")
    assert set(names) == set(B.PROBE_EXPORTS)
    probe = B.probe_lib()
    for n in names:
        assert hasattr(probe, n), n
    # the product library holds the method only: no yardstick kernels, no process-wide switches
    lib = B.lib()
    for n in list(B.PROBE_EXPORTS) + ["skv_set_decode_engine", "skv_set_cache_reads"]:
        assert not hasattr(lib, n), n


def test_status_strings():
    assert B.status_string(0) == "SKV_OK"
    assert B.status_string(B.SKV_ERR_RANK) == "SKV_ERR_RANK"
    assert B.status_string(99) == "SKV_ERR_UNKNOWN"


FAKE = 0x10000  # non-null, 16-byte aligned; never dereferenced because validation fails first


def _layer(**kw):
    d = dict(batch=4, n_q_heads=32, n_kv_heads=8, head_dim=128, r_k=64, r_v=64, capacity=1024,
             k_cache=FAKE, v_cache=FAKE, p_k=FAKE, p_v=FAKE,
             p_k_head_stride=128 * 64, p_v_head_stride=128 * 64)
    d.update(kw)
    return B.skv_layer(**d)


@pytest.mark.parametrize("kw,code", [
    (dict(k_cache=None), B.SKV_ERR_NULL),
    (dict(p_v=None), B.SKV_ERR_NULL),
    (dict(head_dim=64), B.SKV_ERR_SHAPE),
    (dict(batch=0), B.SKV_ERR_SHAPE),
    (dict(n_q_heads=30), B.SKV_ERR_SHAPE),
    (dict(n_q_heads=24), B.SKV_ERR_SHAPE),          # G = 3
    (dict(batch=10000), B.SKV_ERR_SHAPE),           # more (sequence, KV head) columns than a grid holds
    (dict(r_k=0), B.SKV_ERR_RANK),
    (dict(r_k=72), B.SKV_ERR_RANK),
    (dict(r_v=144), B.SKV_ERR_RANK),
    (dict(capacity=0), B.SKV_ERR_CAPACITY),
    (dict(p_k_head_stride=100), B.SKV_ERR_SHAPE),
    (dict(p_v_head_stride=128 * 64 + 4), B.SKV_ERR_ALIGN),
    (dict(k_cache=FAKE + 8), B.SKV_ERR_ALIGN),
])
def test_bad_layers_are_rejected_by_every_entry_point(kw, code):
    lib = B.lib()
    L = _layer(**kw)
    assert lib.skv_project_append(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, 0, None) == code
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 16, 0.0, FAKE, 1 << 30, None) == code
    assert lib.skv_decode_step(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, 0, FAKE, FAKE, 0.0, FAKE, 1 << 30, None) == code
    assert lib.skv_decode_project_query(C.byref(L), FAKE, 0.0, FAKE, 1 << 30, None) == code
    assert lib.skv_decode_partial(C.byref(L), 16, 0, FAKE, 1 << 30, None) == code
    assert lib.skv_decode_combine(C.byref(L), FAKE, 1, FAKE, 1 << 30, None) == code
    assert lib.skv_decode_workspace_bytes(C.byref(L)) == 0
    assert lib.skv_decode_default_splits(C.byref(L), 16) == 0


def test_bad_call_arguments_are_rejected():
    lib = B.lib()
    L = _layer()
    ws = lib.skv_decode_workspace_bytes(C.byref(L))
    assert ws == 4 * 32 * 64 * 4 + 4 * 32 * 256 * 66 * 4          # projected queries + partial results
    assert lib.skv_cache_bytes(C.byref(L), 1000) == 4 * 8 * 1000 * 128 * 2
    # append
    assert lib.skv_project_append(None, FAKE, FAKE, 8192, 1024, 128, 1, 0, None) == B.SKV_ERR_NULL
    assert lib.skv_project_append(C.byref(L), None, FAKE, 8192, 1024, 128, 1, 0, None) == B.SKV_ERR_NULL
    assert lib.skv_project_append(C.byref(L), FAKE, FAKE, 8192, 1024, 128, -1, 0, None) == B.SKV_ERR_SHAPE
    assert lib.skv_project_append(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 2, 1023, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_project_append(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, -1, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_project_append(C.byref(L), FAKE, FAKE, 8192, 1020, 128, 1, 0, None) == B.SKV_ERR_ALIGN
    assert lib.skv_project_append(C.byref(L), FAKE + 2, FAKE, 8192, 1024, 128, 1, 0, None) == B.SKV_ERR_ALIGN
    assert lib.skv_project_append(C.byref(L), FAKE, FAKE, -8, 1024, 128, 1, 0, None) == B.SKV_ERR_SHAPE
    # T = 0 is a no-op that needs no input pointers
    assert lib.skv_project_append(C.byref(L), None, None, 0, 0, 0, 0, 1024, None) == B.SKV_OK
    # decode
    assert lib.skv_decode_attention(C.byref(L), None, FAKE, 16, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert lib.skv_decode_attention(C.byref(L), FAKE, None, 16, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 16, 0.0, None, ws, None) == B.SKV_ERR_NULL
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 0, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 1025, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 16, 0.0, FAKE, 8, None) == B.SKV_ERR_WORKSPACE
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE + 4, 16, 0.0, FAKE, ws, None) == B.SKV_ERR_ALIGN
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 16, float("inf"), FAKE, ws, None) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_project_query(C.byref(L), None, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert lib.skv_decode_project_query(C.byref(L), FAKE, float("nan"), FAKE, ws, None) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_project_query(C.byref(L), FAKE, 0.0, FAKE, 64, None) == B.SKV_ERR_WORKSPACE
    assert lib.skv_decode_project_query(C.byref(L), FAKE + 4, 0.0, FAKE, ws, None) == B.SKV_ERR_ALIGN
    assert lib.skv_decode_partial(C.byref(L), 16, 257, FAKE, ws, None) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_partial(C.byref(L), 0, 1, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    need4 = 4 * 32 * 64 * 4 + 4 * 32 * 4 * 66 * 4
    assert lib.skv_decode_partial(C.byref(L), 16, 4, FAKE, need4 - 1, None) == B.SKV_ERR_WORKSPACE
    assert lib.skv_decode_partial(C.byref(L), 16, 4, None, need4, None) == B.SKV_ERR_NULL
    # the fused step checks the append and the decode arguments before anything runs
    step = lib.skv_decode_step
    assert step(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, 1024, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    assert step(C.byref(L), None, FAKE, 8192, 1024, 128, 1, 0, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert step(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, 0, None, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert step(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, 0, FAKE, None, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert step(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, 0, FAKE, FAKE, 0.0, FAKE, 100, None) == B.SKV_ERR_WORKSPACE
    assert step(C.byref(L), FAKE, FAKE, 8192, 1020, 128, 1, 0, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_ALIGN
    assert step(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 0, 0, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY  # nothing to attend
    assert lib.skv_decode_combine(C.byref(L), FAKE, 0, FAKE, ws, None) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_combine(C.byref(L), FAKE, 257, FAKE, ws, None) == B.SKV_ERR_SHAPE


def test_default_split_plan():
    lib = B.lib()
    L = _layer(capacity=1 << 20)
    # 32 (sequence, KV head) columns -> 16 ranges at long context (two workgroups per CU);
    # never more ranges than 64-row quanta
    assert lib.skv_decode_default_splits(C.byref(L), 32768) == 16
    assert lib.skv_decode_default_splits(C.byref(L), 1 << 20) == 16
    assert lib.skv_decode_default_splits(C.byref(L), 1) == 1
    assert lib.skv_decode_default_splits(C.byref(L), 64) == 1
    assert lib.skv_decode_default_splits(C.byref(L), 65) == 2
    assert lib.skv_decode_default_splits(C.byref(L), 1000) == 8           # one workgroup per CU below 1024 rows each
    assert lib.skv_decode_default_splits(C.byref(L), 8192) == 8           # two workgroups per CU only with 1024 rows each
    mha = _layer(n_q_heads=32, n_kv_heads=32, batch=8, capacity=1 << 20)
    assert lib.skv_decode_default_splits(C.byref(mha), 131072) == 2
    one = _layer(batch=1, capacity=1 << 20)
    assert lib.skv_decode_default_splits(C.byref(one), 1024) == 8
    assert lib.skv_decode_default_splits(C.byref(one), 4096) == 32
    assert lib.skv_decode_default_splits(C.byref(one), 32768) == 32
    assert lib.skv_decode_default_splits(C.byref(one), 1 << 20) == 64


def test_context_ranges_tile_the_context_evenly():
    rng = np.random.default_rng(3)
    cases = [(1, 1), (1, 256), (63, 4), (64, 2), (65, 2), (1000, 16), (32768, 16), (32831, 16), (131072, 2),
             (100, 256), (4097, 7)] + [(int(rng.integers(1, 200000)), int(rng.integers(1, 257))) for _ in range(200)]
    for n, s in cases:
        spans = [B.skv_decode_range(n, s, i) for i in range(s)]
        pos = 0
        sizes = []
        for a, b in spans:
            assert a <= b
            if a < b:
                assert a == pos                    # contiguous, in order, no overlap
                pos = b
                sizes.append(b - a)
        assert pos == n                            # complete
        full = [x for x in sizes[:-1]]             # all but the ragged last one are whole quanta
        assert all(x % 64 == 0 for x in full)
        if len(sizes) > 1:
            assert max(sizes) - min(sizes[:-1] or sizes) <= 64
    lib = B.lib()
    a, b = C.c_int64(), C.c_int64()
    assert lib.skv_decode_range(0, 1, 0, C.byref(a), C.byref(b)) == B.SKV_ERR_CAPACITY
    assert lib.skv_decode_range(10, 0, 0, C.byref(a), C.byref(b)) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_range(10, 4, 4, C.byref(a), C.byref(b)) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_range(10, 4, 0, None, C.byref(b)) == B.SKV_ERR_NULL


def test_layer_ranks_matches_oracle_on_random_surfaces():
    rng = np.random.default_rng(0)
    for trial in range(300):
        L = int(rng.integers(1, 12))
        d = 128
        ck = sorted(rng.choice([16, 32, 48, 64, 80, 96, 112, 128], size=int(rng.integers(1, 6)), replace=False).tolist())
        cv = sorted(rng.choice([16, 32, 48, 64, 80, 96, 112, 128], size=int(rng.integers(1, 6)), replace=False).tolist())
        rho = float(rng.choice([0.3, 0.5, 0.55, 0.6, 0.7, 0.75, 0.8, 0.9, 1.0]))
        if trial % 3 == 0:
            delta = rng.integers(0, 4, size=(L, len(ck), len(cv))).astype(float)   # ties
        else:
            delta = rng.uniform(0, 1, size=(L, len(ck), len(cv)))
        want = O.layer_ranks(L, d, rho, ck, cv, delta)
        got = B.skv_layer_ranks(L, d, rho, ck, cv, delta)
        assert got[0] == want[0] and got[1] == want[1]
        assert got[2] == want[2] and got[3] == want[3]


def test_layer_ranks_argument_errors():
    lib = B.lib()
    i32 = C.c_int32
    ck = (i32 * 2)(64, 128)
    bad = (i32 * 2)(64, 256)
    delta = (C.c_double * 8)(*([0.5] * 8))
    nan = (C.c_double * 8)(*([float("nan")] * 8))
    rk, rv = (i32 * 2)(), (i32 * 2)()
    f = lib.skv_layer_ranks
    assert f(2, 128, 0.8, ck, 2, ck, 2, delta, rk, rv, None) == B.SKV_OK
    assert f(0, 128, 0.8, ck, 2, ck, 2, delta, rk, rv, None) == B.SKV_ERR_SHAPE
    assert f(2, 128, 0.0, ck, 2, ck, 2, delta, rk, rv, None) == B.SKV_ERR_SHAPE
    assert f(2, 128, 0.8, bad, 2, ck, 2, delta, rk, rv, None) == B.SKV_ERR_SHAPE
    assert f(2, 128, 0.8, ck, 2, ck, 2, nan, rk, rv, None) == B.SKV_ERR_SHAPE
    assert f(2, 128, 0.8, None, 2, ck, 2, delta, rk, rv, None) == B.SKV_ERR_NULL
    assert f(2, 128, 0.8, ck, 2, ck, 2, delta, None, rv, None) == B.SKV_ERR_NULL
    assert f(2, 128, 0.3, ck, 2, ck, 2, delta, rk, rv, None) == B.SKV_ERR_BUDGET
    assert list(rk) == [64, 64] and list(rv) == [64, 64]


def test_quantised_layer_argument_checks():
    lib = B.lib()

    def qlayer(base_kw=None, **kw):
        d = dict(k_scale=FAKE, k_zero=FAKE, v_meta=FAKE)
        d.update(kw)
        return B.skv_q8_layer(_layer(**(base_kw or {})), d["k_scale"], d["k_zero"], d["v_meta"])

    ok = qlayer()
    ws = lib.skv_decode_workspace_bytes(C.byref(ok.base))
    assert lib.skv_q8_cache_bytes(C.byref(ok), 1000) == 4 * 8 * 1000 * (128 + 4)
    cases = [(qlayer(k_scale=None), B.SKV_ERR_NULL), (qlayer(v_meta=None), B.SKV_ERR_NULL),
             (qlayer(k_zero=FAKE + 2), B.SKV_ERR_ALIGN),
             (qlayer(dict(r_k=48, p_k_head_stride=128 * 48)), B.SKV_ERR_RANK),       # multiples of 32 only
             (qlayer(dict(r_v=80, p_v_head_stride=128 * 80)), B.SKV_ERR_RANK),
             (qlayer(dict(head_dim=64)), B.SKV_ERR_SHAPE)]
    for Q, code in cases:
        assert lib.skv_q8_project_append(C.byref(Q), FAKE, FAKE, 8192, 1024, 128, 1, 0, None) == code
        assert lib.skv_q8_decode_attention(C.byref(Q), FAKE, FAKE, 16, 0.0, FAKE, ws, None) == code
        assert lib.skv_q8_decode_step(C.byref(Q), FAKE, FAKE, 8192, 1024, 128, 1, 0, FAKE, FAKE, 0.0, FAKE, ws, None) == code
    assert lib.skv_q8_project_append(None, FAKE, FAKE, 8192, 1024, 128, 1, 0, None) == B.SKV_ERR_NULL
    assert lib.skv_q8_project_append(C.byref(ok), FAKE, FAKE, 8192, 1024, 128, 2, 1023, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_q8_decode_attention(C.byref(ok), FAKE, FAKE, 0, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_q8_decode_attention(C.byref(ok), FAKE, FAKE, 16, 0.0, FAKE, 64, None) == B.SKV_ERR_WORKSPACE
    assert lib.skv_q8_decode_step(C.byref(ok), FAKE, FAKE, 8192, 1024, 128, 1, 0, None, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL


def test_folded_variant_argument_checks():
    lib = B.lib()
    L = _layer(p_k=None, p_v=None)                       # bases are not needed here
    ws = lib.skv_decode_workspace_bytes(C.byref(_layer()))
    assert lib.skv_append_projected(C.byref(L), None, None, 0, 5, None) == B.SKV_OK          # T = 0: no-op
    assert lib.skv_append_projected(C.byref(L), None, FAKE, 1, 5, None) == B.SKV_ERR_NULL
    assert lib.skv_append_projected(C.byref(L), FAKE, FAKE, 2, 1023, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_append_projected(C.byref(L), FAKE + 4, FAKE, 1, 0, None) == B.SKV_ERR_ALIGN
    assert lib.skv_append_projected(C.byref(L), FAKE, FAKE, -1, 0, None) == B.SKV_ERR_SHAPE
    assert lib.skv_append_projected(C.byref(_layer(r_k=40)), FAKE, FAKE, 1, 0, None) == B.SKV_ERR_RANK
    f = lib.skv_decode_attention_folded
    assert f(C.byref(L), None, FAKE, 16, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert f(C.byref(L), FAKE, FAKE, 0, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    assert f(C.byref(L), FAKE, FAKE, 16, 0.0, FAKE, 100, None) == B.SKV_ERR_WORKSPACE
    assert f(C.byref(L), FAKE, FAKE, 16, float("nan"), FAKE, ws, None) == B.SKV_ERR_SHAPE
    assert f(C.byref(_layer(k_cache=None)), FAKE, FAKE, 16, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    # the explicit-projection entry points still insist on the bases
    assert lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 16, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    g = lib.skv_decode_step_folded
    assert g(C.byref(L), FAKE, FAKE, 1, 1024, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY
    assert g(C.byref(L), None, FAKE, 1, 5, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert g(C.byref(L), FAKE, FAKE, 1, 5, None, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_NULL
    assert g(C.byref(L), FAKE, FAKE, 0, 0, FAKE, FAKE, 0.0, FAKE, ws, None) == B.SKV_ERR_CAPACITY   # nothing to attend
    assert g(C.byref(L), FAKE, FAKE, 1, 5, FAKE, FAKE, 0.0, FAKE, 64, None) == B.SKV_ERR_WORKSPACE


def test_padded_rank_and_pad_basis_argument_checks():
    lib = B.lib()
    assert [lib.skv_padded_rank(r) for r in (1, 16, 17, 64, 77, 90, 102, 115, 128)] == [16, 16, 32, 64, 80, 96, 112, 128, 128]
    assert lib.skv_padded_rank(0) == 0 and lib.skv_padded_rank(129) == 0 and lib.skv_padded_rank(-3) == 0
    buf = (C.c_uint16 * 8)()
    p = C.cast(buf, C.c_void_p)
    assert lib.skv_pad_basis(None, 1, 77, p, None) == B.SKV_ERR_NULL
    assert lib.skv_pad_basis(p, 0, 77, p, None) == B.SKV_ERR_SHAPE
    assert lib.skv_pad_basis(p, 1, 0, p, None) == B.SKV_ERR_RANK
    assert lib.skv_pad_basis(p, 1, 200, p, None) == B.SKV_ERR_RANK


def test_varlen_and_prefill_argument_checks():
    lib = B.lib()
    L = _layer()
    big = 1 << 30
    # per-sequence lengths: the device array is required and 4-byte aligned; the host bound is checked like n_ctx
    assert lib.skv_decode_attention_varlen(C.byref(L), FAKE, FAKE, None, 16, 0.0, FAKE, big, None) == B.SKV_ERR_NULL
    assert lib.skv_decode_attention_varlen(C.byref(L), FAKE, FAKE, FAKE + 2, 16, 0.0, FAKE, big, None) == B.SKV_ERR_ALIGN
    assert lib.skv_decode_attention_varlen(C.byref(L), FAKE, FAKE, FAKE, 1025, 0.0, FAKE, big, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_project_append_varlen(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 4, None, 0, None) == B.SKV_ERR_NULL
    assert lib.skv_project_append_varlen(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 4, FAKE, 1021, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_decode_step_varlen(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 0, FAKE, 10, FAKE, FAKE, 0.0, FAKE, big,
                                      None) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_step_varlen(C.byref(L), FAKE, FAKE, 8192, 1024, 128, 1, FAKE, 1024, FAKE, FAKE, 0.0, FAKE,
                                      big, None) == B.SKV_ERR_CAPACITY
    # chunk attention
    assert lib.skv_prefill_attention(C.byref(L), FAKE, 8192, 4096, 128, FAKE, 16, 1010, 0.0, 0, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_prefill_attention(C.byref(L), FAKE, 8192, 4096, 128, FAKE, -1, 0, 0.0, 0, None) == B.SKV_ERR_SHAPE
    assert lib.skv_prefill_attention(C.byref(L), FAKE, 8192, 4096, 128, FAKE, 16, 0, 0.0, 0x30, None) == B.SKV_ERR_SHAPE
    assert lib.skv_prefill_attention(C.byref(L), FAKE, 8192, 4100, 128, FAKE, 16, 0, 0.0, 0, None) == B.SKV_ERR_ALIGN
    assert lib.skv_prefill_attention(C.byref(L), None, 8192, 4096, 128, FAKE, 16, 0, 0.0, 0, None) == B.SKV_ERR_NULL
    assert lib.skv_prefill_attention(C.byref(L), FAKE, 8192, 4096, 128, FAKE, 0, 0, 0.0, 0, None) == B.SKV_OK   # T = 0: no-op
    Lf = _layer(p_k=None, p_v=None)
    assert lib.skv_prefill_attention_folded(C.byref(Lf), FAKE, FAKE, 16, 2000, 0.0, 0, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_prefill_tile_tokens(C.byref(L)) == 32 and lib.skv_prefill_tile_tokens(C.byref(_layer(n_q_heads=8))) == 128


def test_orthonormalize_argument_checks():
    lib = B.lib()
    assert lib.skv_orthonormalize(None, 1, 64, 1, FAKE, None) == B.SKV_ERR_NULL
    assert lib.skv_orthonormalize(FAKE, 0, 64, 1, FAKE, None) == B.SKV_ERR_SHAPE
    assert lib.skv_orthonormalize(FAKE, 1, 0, 1, FAKE, None) == B.SKV_ERR_RANK
    assert lib.skv_orthonormalize(FAKE, 1, 129, 0, FAKE, None) == B.SKV_ERR_RANK
    assert lib.skv_orthonormalize(FAKE + 2, 1, 64, 1, FAKE, None) == B.SKV_ERR_ALIGN


def test_four_bit_layer_argument_checks():
    lib = B.lib()
    big = 1 << 30
    Q = B.skv_q8_layer(_layer(), FAKE, FAKE, FAKE)
    assert lib.skv_q4_decode_attention(C.byref(Q), FAKE, FAKE, 2000, 0.0, FAKE, big, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_q4_cache_bytes(C.byref(Q), 10) == 4 * 8 * 10 * (64 + 4)
    Q32 = B.skv_q8_layer(_layer(r_k=32, p_k_head_stride=128 * 32), FAKE, FAKE, FAKE)
    assert lib.skv_q8_decode_attention(C.byref(Q32), FAKE, FAKE, 2000, 0.0, FAKE, big, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_q4_decode_attention(C.byref(Q32), FAKE, FAKE, 16, 0.0, FAKE, big, None) == B.SKV_ERR_RANK
    assert lib.skv_q4_project_append(C.byref(Q32), FAKE, FAKE, 8192, 1024, 128, 1, 0, None) == B.SKV_ERR_RANK
    assert lib.skv_q4_decode_step(C.byref(Q), FAKE, FAKE, 8192, 1024, 128, -1, 0, FAKE, FAKE, 0.0, FAKE, big, None) == B.SKV_ERR_SHAPE


def test_paged_layer_argument_checks():
    lib = B.lib()
    big = 1 << 30

    def paged(page_tokens=64, n_pages=100, max_pages=16, table=FAKE, **kw):
        return B.skv_paged_layer(_layer(capacity=kw.pop("capacity", page_tokens * max_pages), **kw), table, page_tokens,
                                 n_pages, max_pages)

    P = paged()
    assert lib.skv_paged_pool_bytes(C.byref(P)) == 100 * 8 * 64 * (64 + 64) * 2
    att = lambda p, n: lib.skv_paged_decode_attention(C.byref(p), FAKE, FAKE, None, n, 0.0, FAKE, big, None)
    assert att(P, 1025) == B.SKV_ERR_CAPACITY                     # beyond what the table can address
    assert att(paged(page_tokens=48), 10) == B.SKV_ERR_SHAPE      # not a power of two
    assert att(paged(page_tokens=32), 10) == B.SKV_ERR_SHAPE      # smaller than a range quantum
    assert att(paged(n_pages=0), 10) == B.SKV_ERR_SHAPE
    assert att(paged(max_pages=0, capacity=64), 10) == B.SKV_ERR_SHAPE
    assert att(paged(capacity=1000), 10) == B.SKV_ERR_CAPACITY    # capacity must be page_tokens * max_pages_per_seq
    assert att(paged(table=None), 10) == B.SKV_ERR_NULL
    assert att(paged(table=FAKE + 2), 10) == B.SKV_ERR_ALIGN
    assert att(paged(r_k=72), 10) == B.SKV_ERR_RANK
    assert lib.skv_paged_pool_bytes(C.byref(paged(page_tokens=48))) == 0
    # lengths are optional here, but must be aligned when given
    assert lib.skv_paged_decode_attention(C.byref(P), FAKE, FAKE, FAKE + 2, 16, 0.0, FAKE, big, None) == B.SKV_ERR_ALIGN
    assert lib.skv_paged_project_append(C.byref(P), FAKE, FAKE, 8192, 1024, 128, 4, None, 1021, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_paged_project_append(C.byref(P), FAKE, FAKE, 8192, 1024, 128, 0, None, 10, None) == B.SKV_OK
    assert lib.skv_paged_decode_step(C.byref(P), FAKE, FAKE, 8192, 1024, 128, 0, None, 10, FAKE, FAKE, 0.0, FAKE, big,
                                     None) == B.SKV_ERR_SHAPE
    assert lib.skv_paged_decode_step(C.byref(P), FAKE, FAKE, 8192, 1024, 128, 1, None, 10, FAKE, FAKE, 0.0, FAKE, 64,
                                     None) == B.SKV_ERR_WORKSPACE
    assert lib.skv_paged_prefill_attention(C.byref(P), FAKE, 8192, 4096, 128, FAKE, 16, 1010, 0.0, 0, None) == B.SKV_ERR_CAPACITY
    assert lib.skv_paged_prefill_attention(C.byref(P), FAKE, 8192, 4096, 128, FAKE, 0, 0, 0.0, 0, None) == B.SKV_OK
    # the chunk kernel keeps one table entry per key tile in LDS: contexts up to 2^20 rows
    Pbig = paged(page_tokens=65536, max_pages=32, n_pages=64)
    assert lib.skv_paged_prefill_attention(C.byref(Pbig), FAKE, 8192, 4096, 128, FAKE, 16, (1 << 20) - 15, 0.0, 0,
                                           None) == B.SKV_ERR_CAPACITY


def test_layer_flags_are_validated_and_steer_the_choices():
    lib = B.lib()
    big = 1 << 30
    att = lambda L: lib.skv_decode_attention(C.byref(L), FAKE, FAKE, 100, 0.0, FAKE, big, None)
    # unknown bits, both bits of a field, or a non-zero reserved word: rejected before anything is launched
    assert att(_layer(flags=16)) == B.SKV_ERR_SHAPE
    assert att(_layer(flags=0x80000000)) == B.SKV_ERR_SHAPE
    assert att(_layer(flags=B.SKV_READS_STREAMING | B.SKV_READS_CACHED)) == B.SKV_ERR_SHAPE
    assert att(_layer(flags=B.SKV_ENGINE_VECTOR | B.SKV_ENGINE_MATRIX)) == B.SKV_ERR_SHAPE
    assert att(_layer(reserved=1)) == B.SKV_ERR_SHAPE
    assert lib.skv_decode_workspace_bytes(C.byref(_layer(flags=16))) == 0
    assert lib.skv_decode_engine_for(C.byref(_layer(flags=16)), 0) == -1
    # the engine by shape (32 query heads over 8 KV heads in _layer's default: groups of four) ...
    eng = lambda bits=0, **kw: lib.skv_decode_engine_for(C.byref(_layer(**kw)), bits)
    assert eng() == 1                                                        # 64/64, groups of four: matrix cores
    assert eng(r_k=48, p_k_head_stride=128 * 48) == 0                        # other ranks: vector arithmetic
    assert eng(r_v=128, p_v_head_stride=128 * 128) == 0
    assert eng(n_q_heads=8) == 0                                             # no grouping
    assert eng(n_q_heads=64) == 1                                            # groups of eight: one pass on the matrix cores
    assert eng(8, r_k=96, p_k_head_stride=128 * 96) == 1                     # quantised codes
    assert eng(4, n_q_heads=8) == 1
    assert eng(3) == -1
    # ... and forced by the layer's flag, whatever the shape
    assert eng(flags=B.SKV_ENGINE_VECTOR) == 0
    assert eng(8, flags=B.SKV_ENGINE_VECTOR) == 0
    assert eng(n_q_heads=8, flags=B.SKV_ENGINE_MATRIX) == 1
    # rows that come from HBM alone: the vector kernel also at most small ranks (the matrix kernel where it was
    # measured ahead: r_v = 128 under r_k = 32 or 64, and 32/64); groups of eight and codes stay
    assert eng(flags=B.SKV_READS_STREAMING) == 0
    assert eng(r_v=128, p_v_head_stride=128 * 128, flags=B.SKV_READS_STREAMING) == 1
    assert eng(r_k=32, p_k_head_stride=128 * 32, flags=B.SKV_READS_STREAMING) == 1
    assert eng(r_k=32, r_v=32, p_k_head_stride=128 * 32, p_v_head_stride=128 * 32, flags=B.SKV_READS_STREAMING) == 0
    assert eng(flags=B.SKV_READS_CACHED) == 1
    assert eng(n_q_heads=64, flags=B.SKV_READS_STREAMING) == 1
    assert eng(8, flags=B.SKV_READS_STREAMING) == 1
    # groups of eight: the vector kernel streams the cache twice (twice the columns, half the ranges)
    auto8, vec8 = _layer(n_q_heads=64, capacity=1 << 16), _layer(n_q_heads=64, capacity=1 << 16, flags=B.SKV_ENGINE_VECTOR)
    assert lib.skv_decode_default_splits(C.byref(auto8), 1 << 16) == 2 * lib.skv_decode_default_splits(C.byref(vec8), 1 << 16)
    # the kind of load: by size (288 MiB of rows per launch), or as the flag says
    rows = lambda n, **kw: lib.skv_decode_streams_rows(C.byref(_layer(capacity=1 << 20, **kw)), n, 0)
    assert rows(32768) == 0                                                  # 4 x 8 x 32768 x 256 B = 256 MiB
    assert rows(40000) == 1                                                  # 312 MiB
    assert rows(100, flags=B.SKV_READS_STREAMING) == 1
    assert rows(1 << 20, flags=B.SKV_READS_CACHED) == 0
    assert rows(0) == -1 and rows((1 << 20) + 1) == -1
    assert lib.skv_decode_streams_rows(C.byref(_layer(capacity=1 << 20)), 70000, 8) == 0     # half the bytes per row
    assert lib.skv_decode_streams_rows(C.byref(_layer(capacity=1 << 20)), 80000, 8) == 1


@pytest.mark.skipif(HOST_ONLY, reason="lives in a .hip translation unit, which a host-only build leaves out")
def test_static_scratch_entry_point_checks_before_it_touches_the_gpu():
    lib = B.lib()
    att = lambda L, n=100: lib.skv_decode_attention_static(C.byref(L), FAKE, FAKE, n, 0.0, None)
    assert att(_layer(r_k=72)) == B.SKV_ERR_RANK
    assert att(_layer(k_cache=None)) == B.SKV_ERR_NULL
    assert att(_layer(), 0) == B.SKV_ERR_CAPACITY
    assert att(_layer(), 1025) == B.SKV_ERR_CAPACITY
    # 64 sequences x 64 query heads at ranks 128: 2 MiB of projected queries and 2.1 MiB for one partial result
    # per head do not fit the 4 MiB array
    huge = _layer(batch=64, n_q_heads=64, r_k=128, r_v=128, p_k_head_stride=128 * 128, p_v_head_stride=128 * 128)
    assert att(huge, 64) == B.SKV_ERR_WORKSPACE
    assert lib.skv_decode_workspace_bytes(C.byref(huge)) > (4 << 20)


def test_read_probe_argument_checks():
    lib = B.probe_lib()
    n = C.c_size_t(0)
    assert lib.skv_probe_stream_read(None, 1 << 20, 4, 0, FAKE, C.byref(n), None) == B.SKV_ERR_NULL
    assert lib.skv_probe_stream_read(FAKE + 4, 1 << 20, 4, 0, FAKE, C.byref(n), None) == B.SKV_ERR_ALIGN
    assert lib.skv_probe_stream_read(FAKE, 1 << 20, 0, 1, FAKE, C.byref(n), None) == B.SKV_ERR_SHAPE
    assert lib.skv_probe_stream_read(FAKE, 1000, 4, 1, FAKE, C.byref(n), None) == B.SKV_ERR_SHAPE    # less than a slice each


def test_mix_probe_argument_checks():
    lib = B.probe_lib()
    n = C.c_size_t(0)
    assert lib.skv_probe_stream_mix(FAKE, None, FAKE, 1 << 20, 4, C.byref(n), None) == B.SKV_ERR_NULL
    assert lib.skv_probe_stream_mix(FAKE, FAKE, FAKE + 8, 1 << 20, 4, C.byref(n), None) == B.SKV_ERR_ALIGN
    assert lib.skv_probe_stream_mix(FAKE, FAKE, FAKE, 1 << 20, 70000, C.byref(n), None) == B.SKV_ERR_SHAPE
    assert lib.skv_probe_stream_mix(FAKE, FAKE, FAKE, 1000, 4, C.byref(n), None) == B.SKV_ERR_SHAPE   # less than a slice each


def test_paged_folded_argument_checks():
    lib = B.lib()
    big = 1 << 30
    P = B.skv_paged_layer(_layer(capacity=64 * 16, p_k=None, p_v=None), FAKE, 64, 100, 16)     # no bases needed
    app = lambda p, T, cur: lib.skv_paged_append_projected(C.byref(p), FAKE, FAKE, T, None, cur, None)
    assert app(P, 0, 10) == B.SKV_OK
    assert app(P, 4, 1021) == B.SKV_ERR_CAPACITY
    assert app(P, -1, 0) == B.SKV_ERR_SHAPE
    assert lib.skv_paged_append_projected(C.byref(P), None, FAKE, 4, None, 0, None) == B.SKV_ERR_NULL
    assert lib.skv_paged_append_projected(C.byref(P), FAKE, FAKE, 4, FAKE + 2, 0, None) == B.SKV_ERR_ALIGN
    att = lambda p, n, ws=big: lib.skv_paged_decode_attention_folded(C.byref(p), FAKE, FAKE, None, n, 0.0, FAKE, ws, None)
    assert att(P, 0) == B.SKV_ERR_CAPACITY
    assert att(P, 1025) == B.SKV_ERR_CAPACITY
    assert att(P, 100, 64) == B.SKV_ERR_WORKSPACE
    Q = B.skv_paged_layer(_layer(capacity=64 * 16), FAKE, 64, 100, 16, 8, FAKE, FAKE, FAKE)
    assert app(Q, 4, 0) == B.SKV_ERR_SHAPE                                                  # bf16 pages only
    assert att(Q, 100) == B.SKV_ERR_SHAPE
    assert lib.skv_paged_decode_step_folded(C.byref(Q), FAKE, FAKE, 1, None, 10, FAKE, FAKE, 0.0, FAKE, big, None) == B.SKV_ERR_SHAPE
    assert lib.skv_paged_decode_step_folded(C.byref(P), FAKE, FAKE, 1, None, 1024, FAKE, FAKE, 0.0, FAKE, big, None) == B.SKV_ERR_CAPACITY
    bad = B.skv_paged_layer(_layer(capacity=64 * 16, p_k=None, p_v=None), FAKE, 48, 100, 16)
    assert app(bad, 4, 0) == B.SKV_ERR_SHAPE                                                # page size not a power of two


def test_paged_quantised_argument_checks():
    lib = B.lib()
    big = 1 << 30

    def paged(bits, k_scale=FAKE, k_zero=FAKE, v_meta=FAKE, **kw):
        return B.skv_paged_layer(_layer(capacity=64 * 16, **kw), FAKE, 64, 100, 16, bits, k_scale, k_zero, v_meta)

    att = lambda p: lib.skv_paged_decode_attention(C.byref(p), FAKE, FAKE, None, 2000, 0.0, FAKE, big, None)
    assert att(paged(8)) == B.SKV_ERR_CAPACITY                       # a valid description: fails on the length only
    assert att(paged(3)) == B.SKV_ERR_SHAPE                          # widths: 0, 8, 4
    assert att(paged(8, k_scale=None)) == B.SKV_ERR_NULL
    assert att(paged(8, v_meta=FAKE + 2)) == B.SKV_ERR_ALIGN
    assert att(paged(8, r_k=48, p_k_head_stride=128 * 48)) == B.SKV_ERR_RANK     # 8-bit ranks: multiples of 32
    assert att(paged(4, r_v=96, p_v_head_stride=128 * 96)) == B.SKV_ERR_RANK     # 4-bit ranks: multiples of 64
    assert lib.skv_paged_pool_bytes(C.byref(paged(8))) == 100 * 8 * 64 * (64 + 64 + 4)
    assert lib.skv_paged_pool_bytes(C.byref(paged(4))) == 100 * 8 * 64 * (32 + 32 + 4)
    assert lib.skv_paged_decode_default_splits(C.byref(paged(0)), 1024) == 8       # bf16 rows: one workgroup per CU below 1024 rows each
    assert lib.skv_paged_decode_default_splits(C.byref(paged(8)), 1024) == 8       # 24 wanted; one workgroup per CU below 1024 rows each
    assert lib.skv_paged_decode_default_splits(C.byref(paged(8)), 2000) == 0
    # chunk attention and the separate first launch are offered over bf16 pages only
    assert lib.skv_paged_prefill_attention(C.byref(paged(8)), FAKE, 8192, 4096, 128, FAKE, 16, 0, 0.0, 0, None) == B.SKV_ERR_SHAPE
    assert lib.skv_paged_decode_partial_q(C.byref(paged(8)), FAKE, None, 0.0, 100, 0, FAKE, big, None) == B.SKV_ERR_SHAPE


def test_layer_stack_calls_check_every_layer_before_anything_else():
    """skv_decode_attention_layers / skv_decode_step_layers (Sec. 3.3: one descriptor per layer): the arrays
    and the count are checked, and an error in ANY layer is returned -- also in the last one, i.e. before
    the first layer would have been launched (a launch here, without a GPU, would return SKV_ERR_HIP)."""
    lib = B.lib()
    n = 3
    ptrs = (C.c_void_p * n)(FAKE, FAKE, FAKE)
    good = (B.skv_layer * n)(_layer(), _layer(r_k=32, p_k_head_stride=128 * 32), _layer(r_v=96, p_v_head_stride=128 * 96))
    att = lambda layers, cnt, q=ptrs, out=ptrs, n_ctx=16, ws=FAKE, nbytes=1 << 30: lib.skv_decode_attention_layers(
        layers, cnt, q, out, n_ctx, 0.0, ws, nbytes, None)
    step = lambda layers, cnt, k=ptrs, v=ptrs, q=ptrs, out=ptrs, T=1, cur=15, ws=FAKE, nbytes=1 << 30: \
        lib.skv_decode_step_layers(layers, cnt, k, v, 8192, 1024, 128, T, cur, q, out, 0.0, ws, nbytes, None)
    assert att(good, 0) == B.SKV_OK and step(good, 0) == B.SKV_OK
    assert att(good, -1) == B.SKV_ERR_SHAPE and step(good, -1) == B.SKV_ERR_SHAPE
    assert att(None, n) == B.SKV_ERR_NULL and att(good, n, q=None) == B.SKV_ERR_NULL and att(good, n, out=None) == B.SKV_ERR_NULL
    assert step(None, n) == B.SKV_ERR_NULL and step(good, n, k=None) == B.SKV_ERR_NULL and step(good, n, v=None) == B.SKV_ERR_NULL
    assert step(good, n, q=None) == B.SKV_ERR_NULL and step(good, n, out=None) == B.SKV_ERR_NULL
    # the last layer is the bad one
    bad_last = (B.skv_layer * n)(_layer(), _layer(), _layer(r_k=72))
    assert att(bad_last, n) == B.SKV_ERR_RANK and step(bad_last, n) == B.SKV_ERR_RANK
    # a pointer of the last layer is missing / misaligned
    holes = (C.c_void_p * n)(FAKE, FAKE, None)
    assert att(good, n, q=holes) == B.SKV_ERR_NULL and att(good, n, out=holes) == B.SKV_ERR_NULL
    assert step(good, n, k=holes) == B.SKV_ERR_NULL and step(good, n, q=holes) == B.SKV_ERR_NULL
    odd = (C.c_void_p * n)(FAKE, FAKE, FAKE + 4)
    assert att(good, n, out=odd) == B.SKV_ERR_ALIGN and step(good, n, v=odd) == B.SKV_ERR_ALIGN
    # context and capacity, shared by all layers; the workspace must serve the neediest layer
    assert att(good, n, n_ctx=0) == B.SKV_ERR_CAPACITY and att(good, n, n_ctx=1025) == B.SKV_ERR_CAPACITY
    assert step(good, n, cur=1024) == B.SKV_ERR_CAPACITY
    assert att(good, n, nbytes=4096) == B.SKV_ERR_WORKSPACE and step(good, n, nbytes=4096) == B.SKV_ERR_WORKSPACE
    assert att(good, n, ws=None) == B.SKV_ERR_NULL


def test_benchmark_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N > 1 ends with a message and a non-zero status before it touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
