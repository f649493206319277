"""ctypes binding of the C-ABI library declared in include/skv.h.

Argument marshalling only: every step of the path runs in the library's
kernels.  PyTorch tensors supply device memory and the current stream.  The
shared library must have been built (python -m paper_2601_21686_amd.build);
if it is missing, loading raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# SKV_LIBRARY names another build of the library to load instead (the host layer built with sanitizers, say).
LIB_PATH = os.environ.get("SKV_LIBRARY") or os.path.join(_PKG, "libskv.so")
PROBE_LIB_PATH = os.path.join(_PKG, "libskv_probe.so")     # the benchmark's plain streaming kernels (include/skv_probe.h)

SKV_OK = 0
SKV_ERR_NULL, SKV_ERR_SHAPE, SKV_ERR_RANK, SKV_ERR_CAPACITY = 1, 2, 3, 4
SKV_ERR_ALIGN, SKV_ERR_WORKSPACE, SKV_ERR_BUDGET, SKV_ERR_HIP = 5, 6, 7, 8
SKV_HEAD_DIM = 128
SKV_MAX_SPLITS = 256
SKV_PREFILL_EXACT = 0
SKV_PREFILL_SCHED_TOGETHER, SKV_PREFILL_SCHED_AHEAD = 0x10, 0x20
# skv_layer.flags
SKV_READS_BY_SIZE, SKV_READS_STREAMING, SKV_READS_CACHED = 0, 1, 2
SKV_ENGINE_BY_SHAPE, SKV_ENGINE_VECTOR, SKV_ENGINE_MATRIX = 0, 4, 8

# flags given to layers constructed without an explicit `flags` argument (a Python-side default of this
# binding, read when a layer object is built; the library itself keeps no state)
DEFAULT_LAYER_FLAGS = 0

EXPORTS = (
    "skv_project_append", "skv_decode_attention", "skv_decode_attention_static", "skv_decode_workspace_bytes",
    "skv_decode_default_splits", "skv_decode_range", "skv_decode_step", "skv_decode_project_query",
    "skv_decode_partial", "skv_decode_combine", "skv_decode_partial_q",
    "skv_decode_attention_layers", "skv_decode_step_layers",
    "skv_layer_ranks", "skv_cache_bytes", "skv_status_string",
    "skv_q8_project_append", "skv_q8_decode_attention", "skv_q8_decode_step", "skv_q8_cache_bytes",
    "skv_q8_decode_project_query", "skv_q8_decode_partial", "skv_q8_decode_default_splits",
    "skv_q4_project_append", "skv_q4_decode_attention", "skv_q4_decode_step", "skv_q4_cache_bytes",
    "skv_q4_decode_project_query", "skv_q4_decode_partial", "skv_q4_decode_default_splits",
    "skv_append_projected", "skv_decode_attention_folded", "skv_decode_step_folded",
    "skv_padded_rank", "skv_pad_basis", "skv_orthonormalize",
    "skv_decode_attention_varlen", "skv_project_append_varlen", "skv_decode_step_varlen",
    "skv_prefill_attention", "skv_prefill_attention_folded", "skv_prefill_step", "skv_prefill_tile_tokens",
    "skv_paged_pool_bytes", "skv_paged_project_append", "skv_paged_decode_attention", "skv_paged_decode_step",
    "skv_paged_prefill_attention", "skv_paged_decode_partial_q", "skv_decode_engine_for", "skv_decode_streams_rows", "skv_paged_decode_default_splits",
    "skv_paged_append_projected", "skv_paged_decode_attention_folded", "skv_paged_decode_step_folded",
)
PROBE_EXPORTS = ("skv_probe_stream_read", "skv_probe_stream_mix")


class SkvError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


class skv_layer(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("r_k", C.c_int32), ("r_v", C.c_int32),
        ("capacity", C.c_int64),
        ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
        ("p_k", C.c_void_p), ("p_v", C.c_void_p),
        ("p_k_head_stride", C.c_int64), ("p_v_head_stride", C.c_int64),
        ("flags", C.c_uint32), ("reserved", C.c_uint32),
    ]


class skv_q8_layer(C.Structure):
    _fields_ = [("base", skv_layer), ("k_scale", C.c_void_p), ("k_zero", C.c_void_p), ("v_meta", C.c_void_p)]


class skv_paged_layer(C.Structure):
    _fields_ = [("layer", skv_layer), ("block_table", C.c_void_p), ("page_tokens", C.c_int32),
                ("n_pages", C.c_int32), ("max_pages_per_seq", C.c_int32), ("code_bits", C.c_int32),
                ("k_scale", C.c_void_p), ("k_zero", C.c_void_p), ("v_meta", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Opens libskv.so once and declares every prototype."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2601_21686_amd.build`")
    L = C.CDLL(LIB_PATH)
    LP = C.POINTER(skv_layer)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.skv_project_append.argtypes = [LP, vp, vp, i64, i64, i64, i32, i64, vp]
    L.skv_project_append.restype = C.c_int
    L.skv_decode_attention.argtypes = [LP, vp, vp, i64, C.c_float, vp, sz, vp]
    L.skv_decode_attention.restype = C.c_int
    if hasattr(L, "skv_decode_attention_static"):              # absent from a host-only build
        L.skv_decode_attention_static.argtypes = [LP, vp, vp, i64, C.c_float, vp]
        L.skv_decode_attention_static.restype = C.c_int
    L.skv_decode_workspace_bytes.argtypes = [LP]
    L.skv_decode_workspace_bytes.restype = sz
    L.skv_decode_default_splits.argtypes = [LP, i64]
    L.skv_decode_default_splits.restype = i32
    L.skv_decode_range.argtypes = [i64, i32, i32, C.POINTER(i64), C.POINTER(i64)]
    L.skv_decode_range.restype = C.c_int
    L.skv_decode_step.argtypes = [LP, vp, vp, i64, i64, i64, i32, i64, vp, vp, C.c_float, vp, sz, vp]
    L.skv_decode_step.restype = C.c_int
    pp = C.POINTER(C.c_void_p)
    L.skv_decode_attention_layers.argtypes = [LP, i32, pp, pp, i64, C.c_float, vp, sz, vp]
    L.skv_decode_attention_layers.restype = C.c_int
    L.skv_decode_step_layers.argtypes = [LP, i32, pp, pp, i64, i64, i64, i32, i64, pp, pp, C.c_float, vp, sz, vp]
    L.skv_decode_step_layers.restype = C.c_int
    L.skv_decode_project_query.argtypes = [LP, vp, C.c_float, vp, sz, vp]
    L.skv_decode_project_query.restype = C.c_int
    L.skv_decode_partial.argtypes = [LP, i64, i32, vp, sz, vp]
    L.skv_decode_partial.restype = C.c_int
    L.skv_decode_partial_q.argtypes = [LP, vp, C.c_float, i64, i32, vp, sz, vp]
    L.skv_decode_partial_q.restype = C.c_int
    L.skv_decode_combine.argtypes = [LP, vp, i32, vp, sz, vp]
    L.skv_decode_combine.restype = C.c_int
    L.skv_layer_ranks.argtypes = [i32, i32, C.c_double, C.POINTER(i32), i32, C.POINTER(i32), i32,
                                  C.POINTER(C.c_double), C.POINTER(i32), C.POINTER(i32),
                                  C.POINTER(C.c_double)]
    L.skv_layer_ranks.restype = C.c_int
    L.skv_cache_bytes.argtypes = [LP, i64]
    L.skv_cache_bytes.restype = sz
    QP = C.POINTER(skv_q8_layer)
    L.skv_q8_project_append.argtypes = [QP, vp, vp, i64, i64, i64, i32, i64, vp]
    L.skv_q8_project_append.restype = C.c_int
    L.skv_q8_decode_attention.argtypes = [QP, vp, vp, i64, C.c_float, vp, sz, vp]
    L.skv_q8_decode_attention.restype = C.c_int
    L.skv_q8_decode_step.argtypes = [QP, vp, vp, i64, i64, i64, i32, i64, vp, vp, C.c_float, vp, sz, vp]
    L.skv_q8_decode_step.restype = C.c_int
    L.skv_q8_decode_project_query.argtypes = [QP, vp, C.c_float, vp, sz, vp]
    L.skv_q8_decode_project_query.restype = C.c_int
    L.skv_q8_decode_partial.argtypes = [QP, i64, i32, vp, sz, vp]
    L.skv_q8_decode_partial.restype = C.c_int
    L.skv_q8_cache_bytes.argtypes = [QP, i64]
    L.skv_q8_cache_bytes.restype = sz
    for w in ("q8", "q4"):
        getattr(L, f"skv_{w}_decode_default_splits").argtypes = [QP, i64]
        getattr(L, f"skv_{w}_decode_default_splits").restype = i32
    for w in ("q4",):
        getattr(L, f"skv_{w}_project_append").argtypes = [QP, vp, vp, i64, i64, i64, i32, i64, vp]
        getattr(L, f"skv_{w}_decode_attention").argtypes = [QP, vp, vp, i64, C.c_float, vp, sz, vp]
        getattr(L, f"skv_{w}_decode_step").argtypes = [QP, vp, vp, i64, i64, i64, i32, i64, vp, vp, C.c_float, vp, sz, vp]
        getattr(L, f"skv_{w}_decode_project_query").argtypes = [QP, vp, C.c_float, vp, sz, vp]
        getattr(L, f"skv_{w}_decode_partial").argtypes = [QP, i64, i32, vp, sz, vp]
        getattr(L, f"skv_{w}_cache_bytes").argtypes = [QP, i64]
        for f in ("project_append", "decode_attention", "decode_step", "decode_project_query", "decode_partial"):
            getattr(L, f"skv_{w}_{f}").restype = C.c_int
        getattr(L, f"skv_{w}_cache_bytes").restype = sz
    L.skv_append_projected.argtypes = [LP, vp, vp, i32, i64, vp]
    L.skv_append_projected.restype = C.c_int
    L.skv_decode_attention_folded.argtypes = [LP, vp, vp, i64, C.c_float, vp, sz, vp]
    L.skv_decode_attention_folded.restype = C.c_int
    L.skv_decode_step_folded.argtypes = [LP, vp, vp, i32, i64, vp, vp, C.c_float, vp, sz, vp]
    L.skv_decode_step_folded.restype = C.c_int
    L.skv_prefill_attention.argtypes = [LP, vp, i64, i64, i64, vp, i32, i64, C.c_float, i32, vp]
    L.skv_prefill_attention.restype = C.c_int
    L.skv_prefill_attention_folded.argtypes = [LP, vp, vp, i32, i64, C.c_float, i32, vp]
    L.skv_prefill_attention_folded.restype = C.c_int
    L.skv_prefill_step.argtypes = [LP, vp, vp, i64, i64, i64, vp, i64, i64, i64, vp, i32, i64, C.c_float, i32, vp]
    L.skv_prefill_step.restype = C.c_int
    L.skv_prefill_tile_tokens.argtypes = [LP]
    L.skv_prefill_tile_tokens.restype = i32
    L.skv_decode_attention_varlen.argtypes = [LP, vp, vp, vp, i64, C.c_float, vp, sz, vp]
    L.skv_decode_attention_varlen.restype = C.c_int
    L.skv_project_append_varlen.argtypes = [LP, vp, vp, i64, i64, i64, i32, vp, i64, vp]
    L.skv_project_append_varlen.restype = C.c_int
    L.skv_decode_step_varlen.argtypes = [LP, vp, vp, i64, i64, i64, i32, vp, i64, vp, vp, C.c_float, vp, sz, vp]
    L.skv_decode_step_varlen.restype = C.c_int
    PP = C.POINTER(skv_paged_layer)
    L.skv_paged_pool_bytes.argtypes = [PP]
    L.skv_paged_pool_bytes.restype = sz
    L.skv_paged_decode_default_splits.argtypes = [PP, i64]
    L.skv_paged_decode_default_splits.restype = i32
    L.skv_paged_project_append.argtypes = [PP, vp, vp, i64, i64, i64, i32, vp, i64, vp]
    L.skv_paged_project_append.restype = C.c_int
    L.skv_paged_decode_attention.argtypes = [PP, vp, vp, vp, i64, C.c_float, vp, sz, vp]
    L.skv_paged_decode_attention.restype = C.c_int
    L.skv_paged_decode_partial_q.argtypes = [PP, vp, vp, C.c_float, i64, i32, vp, sz, vp]
    L.skv_paged_decode_partial_q.restype = C.c_int
    L.skv_paged_decode_step.argtypes = [PP, vp, vp, i64, i64, i64, i32, vp, i64, vp, vp, C.c_float, vp, sz, vp]
    L.skv_paged_decode_step.restype = C.c_int
    L.skv_paged_prefill_attention.argtypes = [PP, vp, i64, i64, i64, vp, i32, i64, C.c_float, i32, vp]
    L.skv_paged_prefill_attention.restype = C.c_int
    L.skv_paged_append_projected.argtypes = [PP, vp, vp, i32, vp, i64, vp]
    L.skv_paged_append_projected.restype = C.c_int
    L.skv_paged_decode_attention_folded.argtypes = [PP, vp, vp, vp, i64, C.c_float, vp, sz, vp]
    L.skv_paged_decode_attention_folded.restype = C.c_int
    L.skv_paged_decode_step_folded.argtypes = [PP, vp, vp, i32, vp, i64, vp, vp, C.c_float, vp, sz, vp]
    L.skv_paged_decode_step_folded.restype = C.c_int
    L.skv_decode_engine_for.argtypes = [LP, i32]
    L.skv_decode_engine_for.restype = i32
    L.skv_decode_streams_rows.argtypes = [LP, i64, i32]
    L.skv_decode_streams_rows.restype = i32
    L.skv_orthonormalize.argtypes = [vp, i32, i32, i32, vp, vp]
    L.skv_orthonormalize.restype = C.c_int
    L.skv_padded_rank.argtypes = [i32]
    L.skv_padded_rank.restype = i32
    L.skv_pad_basis.argtypes = [vp, i32, i32, vp, vp]
    L.skv_pad_basis.restype = C.c_int
    L.skv_status_string.argtypes = [C.c_int]
    L.skv_status_string.restype = C.c_char_p
    _lib = L
    return L


_probe_lib = None


def probe_lib() -> C.CDLL:
    """Opens libskv_probe.so (the benchmark's plain streaming kernels) once."""
    global _probe_lib
    if _probe_lib is not None:
        return _probe_lib
    if not os.path.exists(PROBE_LIB_PATH):
        raise FileNotFoundError(
            f"{PROBE_LIB_PATH} not found: build it with `python -m paper_2601_21686_amd.build`")
    L = C.CDLL(PROBE_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    L.skv_probe_stream_read.argtypes = [vp, sz, i32, i32, vp, C.POINTER(C.c_size_t), vp]
    L.skv_probe_stream_read.restype = C.c_int
    L.skv_probe_stream_mix.argtypes = [vp, vp, vp, sz, i32, C.POINTER(C.c_size_t), vp]
    L.skv_probe_stream_mix.restype = C.c_int
    _probe_lib = L
    return L


def status_string(code: int) -> str:
    return lib().skv_status_string(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != SKV_OK:
        raise SkvError(code, where)


def _stream_ptr(stream=None) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class Layer:
    """One decoder layer's compressed cache: device tensors plus the C struct.

    p_k, p_v: bf16 CUDA tensors [n_bases, 128, r]; n_bases = n_kv_heads, or 1
    for a basis shared by all heads.  The cache tensors are allocated here
    (uninitialised) unless passed in.
    """

    def __init__(self, batch, n_q_heads, n_kv_heads, p_k, p_v, capacity,
                 k_cache=None, v_cache=None, head_dim=SKV_HEAD_DIM, flags=None):
        dev = p_k.device
        assert p_k.dtype == torch.bfloat16 and p_v.dtype == torch.bfloat16
        assert p_k.is_contiguous() and p_v.is_contiguous()
        self.batch, self.n_q_heads, self.n_kv_heads = int(batch), int(n_q_heads), int(n_kv_heads)
        self.head_dim, self.capacity = int(head_dim), int(capacity)
        self.r_k, self.r_v = int(p_k.shape[2]), int(p_v.shape[2])
        self.p_k, self.p_v = p_k, p_v
        if k_cache is None:
            k_cache = torch.empty((batch, n_kv_heads, capacity, self.r_k), dtype=torch.bfloat16, device=dev)
        if v_cache is None:
            v_cache = torch.empty((batch, n_kv_heads, capacity, self.r_v), dtype=torch.bfloat16, device=dev)
        assert k_cache.is_contiguous() and v_cache.is_contiguous()
        self.k_cache, self.v_cache = k_cache, v_cache
        self.c = skv_layer(
            self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.r_k, self.r_v,
            self.capacity, k_cache.data_ptr(), v_cache.data_ptr(), p_k.data_ptr(), p_v.data_ptr(),
            0 if p_k.shape[0] == 1 else p_k.shape[1] * p_k.shape[2],
            0 if p_v.shape[0] == 1 else p_v.shape[1] * p_v.shape[2],
            DEFAULT_LAYER_FLAGS if flags is None else int(flags), 0)
        self._ws = None

    def workspace(self) -> torch.Tensor:
        if self._ws is None:
            n = skv_decode_workspace_bytes(self)
            self._ws = torch.empty(n, dtype=torch.uint8, device=self.p_k.device)
        return self._ws


class QuantLayer:
    """One layer's quantised compressed cache: 8-bit codes (ranks multiples of 32, one byte per channel)
    or 4-bit codes (bits=4: ranks multiples of 64, two channels per byte).

    k_scale, k_zero: float32 CUDA tensors [n_kv_heads, ceil(r_k / 64)] (static key ranges).
    Codes are uint8 tensors; v_meta is int32 [batch, n_kv_heads, capacity, ceil(r_v / 64)]
    holding a bf16 scale (low half) and a bf16 zero (high half) per value row and group.
    """

    def __init__(self, batch, n_q_heads, n_kv_heads, p_k, p_v, k_scale, k_zero, capacity, bits=8, flags=None):
        dev = p_k.device
        assert bits in (8, 4)
        self.bits = int(bits)
        self.batch, self.n_q_heads, self.n_kv_heads = int(batch), int(n_q_heads), int(n_kv_heads)
        self.capacity = int(capacity)
        self.r_k, self.r_v = int(p_k.shape[2]), int(p_v.shape[2])
        self.p_k, self.p_v = p_k, p_v
        self.k_scale = k_scale.to(device=dev, dtype=torch.float32).contiguous()
        self.k_zero = k_zero.to(device=dev, dtype=torch.float32).contiguous()
        ngv = (self.r_v + 63) // 64
        self.k_cache = torch.empty((batch, n_kv_heads, capacity, self.r_k * self.bits // 8), dtype=torch.uint8, device=dev)
        self.v_cache = torch.empty((batch, n_kv_heads, capacity, self.r_v * self.bits // 8), dtype=torch.uint8, device=dev)
        self.v_meta = torch.empty((batch, n_kv_heads, capacity, ngv), dtype=torch.int32, device=dev)
        base = skv_layer(
            self.batch, self.n_q_heads, self.n_kv_heads, SKV_HEAD_DIM, self.r_k, self.r_v, self.capacity,
            self.k_cache.data_ptr(), self.v_cache.data_ptr(), p_k.data_ptr(), p_v.data_ptr(),
            0 if p_k.shape[0] == 1 else p_k.shape[1] * p_k.shape[2],
            0 if p_v.shape[0] == 1 else p_v.shape[1] * p_v.shape[2],
            DEFAULT_LAYER_FLAGS if flags is None else int(flags), 0)
        self.c = skv_q8_layer(base, self.k_scale.data_ptr(), self.k_zero.data_ptr(), self.v_meta.data_ptr())
        self._ws = None

    def workspace(self) -> torch.Tensor:
        if self._ws is None:
            n = int(lib().skv_decode_workspace_bytes(C.byref(self.c.base)))
            self._ws = torch.empty(n, dtype=torch.uint8, device=self.p_k.device)
        return self._ws


def _ref(layer):
    return C.byref(layer.c if isinstance(layer, (Layer, QuantLayer)) else layer)


def _base_ref(layer):
    """The plain skv_layer of a Layer, a QuantLayer or a PagedLayer (for calls that do not depend on the
    format or on where the rows live)."""
    if isinstance(layer, QuantLayer):
        return C.byref(layer.c.base)
    if isinstance(layer, PagedLayer):
        return C.byref(layer.c.layer)
    return _ref(layer)


# ---- the C ABI, same names -------------------------------------------------


def skv_project_append(layer, k_new: torch.Tensor, v_new: torch.Tensor, cur_len: int, stream=None) -> None:
    """k_new, v_new: bf16 [batch, T, n_kv_heads, 128], last axis contiguous."""
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    sb, st, sh, _ = k_new.stride()
    _check(lib().skv_project_append(_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                    int(k_new.shape[1]), int(cur_len), _stream_ptr(stream)),
           "skv_project_append")


def skv_decode_workspace_bytes(layer) -> int:
    return int(lib().skv_decode_workspace_bytes(_base_ref(layer)))


def skv_decode_default_splits(layer, n_ctx: int) -> int:
    return int(lib().skv_decode_default_splits(_base_ref(layer), int(n_ctx)))


def skv_decode_range(n_ctx: int, n_splits: int, rng: int):
    """(first_row, end_row) of context range `rng` out of `n_splits` over n_ctx rows."""
    a, b = C.c_int64(0), C.c_int64(0)
    _check(lib().skv_decode_range(int(n_ctx), int(n_splits), int(rng), C.byref(a), C.byref(b)), "skv_decode_range")
    return int(a.value), int(b.value)


def skv_decode_attention(layer, q: torch.Tensor, out: torch.Tensor, n_ctx: int, scale: float = 0.0,
                         workspace: torch.Tensor | None = None, stream=None) -> None:
    """q: bf16 [batch, n_q_heads, 128]; out: float32 of the same shape."""
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_attention(_ref(layer), q.data_ptr(), out.data_ptr(), int(n_ctx),
                                      float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                      _stream_ptr(stream)), "skv_decode_attention")


def skv_decode_attention_static(layer: "Layer", q: torch.Tensor, out: torch.Tensor, n_ctx: int, scale: float = 0.0,
                                stream=None) -> None:
    """skv_decode_attention without a workspace argument: the library's static device scratch array serves."""
    _check(lib().skv_decode_attention_static(_ref(layer), q.data_ptr(), out.data_ptr(), int(n_ctx), float(scale),
                                             _stream_ptr(stream)), "skv_decode_attention_static")


def skv_decode_step(layer, k_new: torch.Tensor, v_new: torch.Tensor, cur_len: int, q: torch.Tensor,
                    out: torch.Tensor, scale: float = 0.0, workspace: torch.Tensor | None = None,
                    stream=None) -> None:
    """Append k_new/v_new ([batch, T, n_kv_heads, 128]) at cur_len, then attend cur_len + T rows."""
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    sb, st, sh, _ = k_new.stride()
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_step(_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                 int(k_new.shape[1]), int(cur_len), q.data_ptr(), out.data_ptr(),
                                 float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                 _stream_ptr(stream)), "skv_decode_step")


class LayerStack:
    """The descriptors of several Layer objects as one C array, plus one workspace large enough for each of
    them (argument marshalling for the *_layers calls; built once, reused every step)."""

    def __init__(self, layers):
        self.layers = list(layers)
        self.c = (skv_layer * len(self.layers))(*[l.c for l in self.layers])
        self._ws = None

    def __len__(self):
        return len(self.layers)

    def workspace(self) -> torch.Tensor:
        if self._ws is None:
            n = max([skv_decode_workspace_bytes(l) for l in self.layers] + [16])
            self._ws = torch.empty(n, dtype=torch.uint8, device=self.layers[0].p_k.device)
        return self._ws


def _ptr_array(tensors, n):
    assert len(tensors) == n
    return (C.c_void_p * n)(*[t.data_ptr() for t in tensors])


def skv_decode_attention_layers(stack: LayerStack, q, out, n_ctx: int, scale: float = 0.0,
                                workspace: torch.Tensor | None = None, stream=None) -> None:
    """skv_decode_attention for every layer of the stack in order; q, out: one tensor per layer."""
    n = len(stack)
    ws = stack.workspace() if workspace is None else workspace
    _check(lib().skv_decode_attention_layers(stack.c, n, _ptr_array(q, n), _ptr_array(out, n), int(n_ctx),
                                             float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                             _stream_ptr(stream)), "skv_decode_attention_layers")


def skv_decode_step_layers(stack: LayerStack, k_new, v_new, cur_len: int, q, out, scale: float = 0.0,
                           workspace: torch.Tensor | None = None, stream=None) -> None:
    """skv_decode_step for every layer of the stack in order; k_new, v_new, q, out: one tensor per layer
    (all k_new / v_new with the same shape and strides)."""
    n = len(stack)
    assert all(t.dtype == torch.bfloat16 and t.stride() == k_new[0].stride() and t.shape == k_new[0].shape
               for t in list(k_new) + list(v_new)) and k_new[0].stride(3) == 1
    sb, st, sh, _ = k_new[0].stride()
    ws = stack.workspace() if workspace is None else workspace
    _check(lib().skv_decode_step_layers(stack.c, n, _ptr_array(k_new, n), _ptr_array(v_new, n), sb, st, sh,
                                        int(k_new[0].shape[1]), int(cur_len), _ptr_array(q, n), _ptr_array(out, n),
                                        float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                        _stream_ptr(stream)), "skv_decode_step_layers")


def skv_decode_project_query(layer, q: torch.Tensor, scale: float = 0.0,
                             workspace: torch.Tensor | None = None, stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_project_query(_ref(layer), q.data_ptr(), float(scale), ws.data_ptr(),
                                          ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_decode_project_query")


def skv_decode_partial(layer, n_ctx: int, n_splits: int = 0, workspace: torch.Tensor | None = None,
                       stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_partial(_ref(layer), int(n_ctx), int(n_splits), ws.data_ptr(),
                                    ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_decode_partial")


def skv_decode_partial_q(layer, q: torch.Tensor, n_ctx: int, n_splits: int = 0, scale: float = 0.0,
                         workspace: torch.Tensor | None = None, stream=None) -> None:
    """The range kernel with the query projection folded in (what skv_decode_attention launches)."""
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_partial_q(_ref(layer), q.data_ptr(), float(scale), int(n_ctx), int(n_splits),
                                      ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_decode_partial_q")


def skv_decode_combine(layer, out: torch.Tensor, n_splits: int, workspace: torch.Tensor | None = None,
                       stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_combine(_base_ref(layer), out.data_ptr(), int(n_splits), ws.data_ptr(),
                                    ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_decode_combine")


def skv_cache_bytes(layer, n_tokens: int) -> int:
    return int(lib().skv_cache_bytes(_ref(layer), int(n_tokens)))


def skv_layer_ranks(n_layers: int, head_dim: int, rho: float, cand_k, cand_v, delta):
    """Returns (r_k list, r_v list, achieved ratio, feasible flag).  Host only."""
    import numpy as np
    ck = (C.c_int32 * len(cand_k))(*[int(x) for x in cand_k])
    cv = (C.c_int32 * len(cand_v))(*[int(x) for x in cand_v])
    d = np.ascontiguousarray(np.asarray(delta, dtype=np.float64))
    if d.shape != (n_layers, len(cand_k), len(cand_v)):
        raise ValueError("delta must be [n_layers, n_k, n_v]")
    rk = (C.c_int32 * n_layers)()
    rv = (C.c_int32 * n_layers)()
    ach = C.c_double(0.0)
    code = lib().skv_layer_ranks(n_layers, head_dim, float(rho), ck, len(cand_k), cv, len(cand_v),
                                 d.ctypes.data_as(C.POINTER(C.c_double)), rk, rv, C.byref(ach))
    if code not in (SKV_OK, SKV_ERR_BUDGET):
        raise SkvError(code, "skv_layer_ranks")
    return list(rk), list(rv), float(ach.value), code == SKV_OK


# ---- folded-weights variant ------------------------------------------------------


def skv_append_projected(layer, k_low: torch.Tensor, v_low: torch.Tensor, cur_len: int, stream=None) -> None:
    """k_low: bf16 [batch, T, n_kv_heads, r_k] contiguous; v_low likewise with r_v."""
    assert k_low.dtype == torch.bfloat16 and v_low.dtype == torch.bfloat16
    assert k_low.is_contiguous() and v_low.is_contiguous()
    _check(lib().skv_append_projected(_base_ref(layer), k_low.data_ptr(), v_low.data_ptr(), int(k_low.shape[1]),
                                      int(cur_len), _stream_ptr(stream)), "skv_append_projected")


def skv_decode_attention_folded(layer, q_low: torch.Tensor, out_low: torch.Tensor, n_ctx: int,
                                scale: float = 0.0, workspace: torch.Tensor | None = None, stream=None) -> None:
    """q_low: bf16 [batch, n_q_heads, r_k]; out_low: float32 [batch, n_q_heads, r_v]."""
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_attention_folded(_base_ref(layer), q_low.data_ptr(), out_low.data_ptr(), int(n_ctx),
                                             float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                             _stream_ptr(stream)), "skv_decode_attention_folded")


def skv_decode_step_folded(layer, k_low: torch.Tensor, v_low: torch.Tensor, cur_len: int, q_low: torch.Tensor,
                           out_low: torch.Tensor, scale: float = 0.0, workspace: torch.Tensor | None = None,
                           stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    assert k_low.is_contiguous() and v_low.is_contiguous()
    _check(lib().skv_decode_step_folded(_base_ref(layer), k_low.data_ptr(), v_low.data_ptr(), int(k_low.shape[1]),
                                        int(cur_len), q_low.data_ptr(), out_low.data_ptr(), float(scale),
                                        ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_decode_step_folded")


# ---- per-sequence lengths -------------------------------------------------------------------------


def _lens_ok(t: torch.Tensor, batch: int) -> None:
    assert t.dtype == torch.int32 and t.is_cuda and t.is_contiguous() and t.numel() == batch


def skv_decode_attention_varlen(layer, q: torch.Tensor, out: torch.Tensor, seq_lens: torch.Tensor, max_len: int,
                                scale: float = 0.0, workspace: torch.Tensor | None = None, stream=None) -> None:
    """seq_lens: int32 CUDA [batch]; max_len: host upper bound of the lengths."""
    _lens_ok(seq_lens, layer.batch)
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_attention_varlen(_base_ref(layer), q.data_ptr(), out.data_ptr(), seq_lens.data_ptr(),
                                             int(max_len), float(scale), ws.data_ptr(),
                                             ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_decode_attention_varlen")


def skv_project_append_varlen(layer, k_new: torch.Tensor, v_new: torch.Tensor, cur_lens: torch.Tensor,
                              max_cur_len: int, stream=None) -> None:
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    _lens_ok(cur_lens, layer.batch)
    sb, st, sh, _ = k_new.stride()
    _check(lib().skv_project_append_varlen(_base_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                           int(k_new.shape[1]), cur_lens.data_ptr(), int(max_cur_len),
                                           _stream_ptr(stream)), "skv_project_append_varlen")


def skv_decode_step_varlen(layer, k_new: torch.Tensor, v_new: torch.Tensor, cur_lens: torch.Tensor, max_cur_len: int,
                           q: torch.Tensor, out: torch.Tensor, scale: float = 0.0,
                           workspace: torch.Tensor | None = None, stream=None) -> None:
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    _lens_ok(cur_lens, layer.batch)
    sb, st, sh, _ = k_new.stride()
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_decode_step_varlen(_base_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                        int(k_new.shape[1]), cur_lens.data_ptr(), int(max_cur_len), q.data_ptr(),
                                        out.data_ptr(), float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                        _stream_ptr(stream)), "skv_decode_step_varlen")


def skv_probe_stream_read(src: torch.Tensor, workgroups: int, sink: torch.Tensor, streaming: bool = False,
                          stream=None) -> int:
    """One read-only launch over src (a contiguous CUDA tensor), with streaming or ordinary loads; returns the
    bytes it read."""
    assert src.is_cuda and src.is_contiguous() and sink.dtype == torch.float32 and sink.numel() >= workgroups
    n = C.c_size_t(0)
    _check(probe_lib().skv_probe_stream_read(src.data_ptr(), src.numel() * src.element_size(), int(workgroups),
                                             1 if streaming else 0, sink.data_ptr(), C.byref(n), _stream_ptr(stream)),
           "skv_probe_stream_read")
    return int(n.value)


def skv_probe_stream_mix(a: torch.Tensor, b: torch.Tensor, c: torch.Tensor, workgroups: int, stream=None) -> int:
    """One launch c = a ^ b over three contiguous CUDA tensors of one size; returns the bytes taken from each."""
    nbytes = a.numel() * a.element_size()
    for t in (a, b, c):
        assert t.is_cuda and t.is_contiguous() and t.numel() * t.element_size() == nbytes
    n = C.c_size_t(0)
    _check(probe_lib().skv_probe_stream_mix(a.data_ptr(), b.data_ptr(), c.data_ptr(), nbytes, int(workgroups),
                                            C.byref(n), _stream_ptr(stream)), "skv_probe_stream_mix")
    return int(n.value)


def _layer_struct(layer) -> skv_layer:
    c = layer.c
    return c if isinstance(c, skv_layer) else (c.base if isinstance(c, skv_q8_layer) else c.layer)


def skv_decode_engine_for(layer) -> int:
    """The range kernel the decode calls run for this layer object: 0 = vector arithmetic, 1 = matrix cores."""
    bits = int(getattr(layer, "bits", 0))
    if isinstance(layer.c, skv_paged_layer) and bits:
        return 1                                   # quantised pages: the matrix kernel only
    return int(lib().skv_decode_engine_for(C.byref(_layer_struct(layer)), bits))


def skv_decode_streams_rows(layer, n_ctx: int) -> bool:
    """Whether the range kernel of a decode call over n_ctx rows of this layer reads with streaming loads."""
    r = int(lib().skv_decode_streams_rows(C.byref(_layer_struct(layer)), int(n_ctx), int(getattr(layer, "bits", 0))))
    if r < 0:
        raise SkvError(SKV_ERR_SHAPE, "skv_decode_streams_rows")
    return bool(r)


# ---- paged cache -------------------------------------------------------------------------------


class PagedLayer:
    """A layer whose compressed rows live in page pools [n_pages, n_kv_heads, page_tokens, ...] addressed
    through block_table (int32 CUDA [batch, max_pages_per_seq]).  bits = 0: bf16 rows; 8 or 4: integer codes
    (uint8 pools of r * bits / 8 bytes per row, v_meta int32 [..., groups of r_v], static key ranges k_scale /
    k_zero as for QuantLayer).  The pools are allocated here (uninitialised) unless passed in."""

    def __init__(self, batch, n_q_heads, n_kv_heads, p_k, p_v, page_tokens, n_pages, block_table,
                 k_pool=None, v_pool=None, bits=0, k_scale=None, k_zero=None, flags=None):
        dev = p_k.device
        assert p_k.dtype == torch.bfloat16 and p_v.dtype == torch.bfloat16
        assert p_k.is_contiguous() and p_v.is_contiguous()
        assert block_table.dtype == torch.int32 and block_table.is_cuda and block_table.is_contiguous()
        assert block_table.dim() == 2 and block_table.shape[0] == batch
        assert bits in (0, 8, 4)
        self.batch, self.n_q_heads, self.n_kv_heads = int(batch), int(n_q_heads), int(n_kv_heads)
        self.page_tokens, self.n_pages, self.bits = int(page_tokens), int(n_pages), int(bits)
        self.max_pages_per_seq = int(block_table.shape[1])
        self.capacity = self.page_tokens * self.max_pages_per_seq
        self.r_k, self.r_v = int(p_k.shape[2]), int(p_v.shape[2])
        self.p_k, self.p_v, self.block_table = p_k, p_v, block_table
        if bits:
            wk, wv, dt = self.r_k * bits // 8, self.r_v * bits // 8, torch.uint8
        else:
            wk, wv, dt = self.r_k, self.r_v, torch.bfloat16
        if k_pool is None:
            k_pool = torch.empty((n_pages, n_kv_heads, page_tokens, wk), dtype=dt, device=dev)
        if v_pool is None:
            v_pool = torch.empty((n_pages, n_kv_heads, page_tokens, wv), dtype=dt, device=dev)
        assert k_pool.is_contiguous() and v_pool.is_contiguous() and k_pool.dtype == dt and v_pool.dtype == dt
        self.k_pool, self.v_pool = k_pool, v_pool
        self.v_meta = self.k_scale = self.k_zero = None
        if bits:
            self.k_scale = k_scale.to(device=dev, dtype=torch.float32).contiguous()
            self.k_zero = k_zero.to(device=dev, dtype=torch.float32).contiguous()
            self.v_meta = torch.empty((n_pages, n_kv_heads, page_tokens, (self.r_v + 63) // 64), dtype=torch.int32,
                                      device=dev)
        base = skv_layer(self.batch, self.n_q_heads, self.n_kv_heads, SKV_HEAD_DIM, self.r_k, self.r_v,
                         self.capacity, k_pool.data_ptr(), v_pool.data_ptr(), p_k.data_ptr(), p_v.data_ptr(),
                         0 if p_k.shape[0] == 1 else p_k.shape[1] * p_k.shape[2],
                         0 if p_v.shape[0] == 1 else p_v.shape[1] * p_v.shape[2],
                         DEFAULT_LAYER_FLAGS if flags is None else int(flags), 0)
        self.c = skv_paged_layer(base, block_table.data_ptr(), self.page_tokens, self.n_pages,
                                 self.max_pages_per_seq, self.bits,
                                 self.k_scale.data_ptr() if bits else None, self.k_zero.data_ptr() if bits else None,
                                 self.v_meta.data_ptr() if bits else None)
        self._ws = None

    def workspace(self) -> torch.Tensor:
        if self._ws is None:
            n = int(lib().skv_decode_workspace_bytes(C.byref(self.c.layer)))
            self._ws = torch.empty(n, dtype=torch.uint8, device=self.p_k.device)
        return self._ws


def _lens_ptr(t, batch: int):
    if t is None:
        return None
    _lens_ok(t, batch)
    return t.data_ptr()


def skv_paged_decode_default_splits(layer: PagedLayer, n_ctx: int) -> int:
    return int(lib().skv_paged_decode_default_splits(C.byref(layer.c), int(n_ctx)))


def skv_paged_pool_bytes(layer: PagedLayer) -> int:
    return int(lib().skv_paged_pool_bytes(C.byref(layer.c)))


def skv_paged_project_append(layer: PagedLayer, k_new: torch.Tensor, v_new: torch.Tensor, cur_lens, max_cur_len: int,
                             stream=None) -> None:
    """cur_lens: int32 CUDA [batch], or None when every sequence stands at max_cur_len."""
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    sb, st, sh, _ = k_new.stride()
    _check(lib().skv_paged_project_append(C.byref(layer.c), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                          int(k_new.shape[1]), _lens_ptr(cur_lens, layer.batch), int(max_cur_len),
                                          _stream_ptr(stream)), "skv_paged_project_append")


def skv_paged_decode_attention(layer: PagedLayer, q: torch.Tensor, out: torch.Tensor, seq_lens, max_len: int,
                               scale: float = 0.0, workspace: torch.Tensor | None = None, stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_paged_decode_attention(C.byref(layer.c), q.data_ptr(), out.data_ptr(),
                                            _lens_ptr(seq_lens, layer.batch), int(max_len), float(scale),
                                            ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_paged_decode_attention")


def skv_paged_decode_partial_q(layer: PagedLayer, q: torch.Tensor, seq_lens, max_len: int, n_splits: int = 0,
                               scale: float = 0.0, workspace: torch.Tensor | None = None, stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_paged_decode_partial_q(C.byref(layer.c), q.data_ptr(), _lens_ptr(seq_lens, layer.batch),
                                            float(scale), int(max_len), int(n_splits), ws.data_ptr(),
                                            ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_paged_decode_partial_q")


def skv_paged_decode_step(layer: PagedLayer, k_new: torch.Tensor, v_new: torch.Tensor, cur_lens, max_cur_len: int,
                          q: torch.Tensor, out: torch.Tensor, scale: float = 0.0,
                          workspace: torch.Tensor | None = None, stream=None) -> None:
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    sb, st, sh, _ = k_new.stride()
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_paged_decode_step(C.byref(layer.c), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                       int(k_new.shape[1]), _lens_ptr(cur_lens, layer.batch), int(max_cur_len),
                                       q.data_ptr(), out.data_ptr(), float(scale), ws.data_ptr(),
                                       ws.numel() * ws.element_size(), _stream_ptr(stream)), "skv_paged_decode_step")


def skv_paged_append_projected(layer: PagedLayer, k_low: torch.Tensor, v_low: torch.Tensor, cur_lens,
                               max_cur_len: int, stream=None) -> None:
    """k_low: bf16 CUDA [batch, T, n_kv_heads, r_k] contiguous, v_low likewise with r_v; cur_lens: int32 CUDA
    [batch] or None."""
    assert k_low.dtype == torch.bfloat16 and v_low.dtype == torch.bfloat16
    assert k_low.is_contiguous() and v_low.is_contiguous()
    _check(lib().skv_paged_append_projected(C.byref(layer.c), k_low.data_ptr(), v_low.data_ptr(), int(k_low.shape[1]),
                                            _lens_ptr(cur_lens, layer.batch), int(max_cur_len), _stream_ptr(stream)),
           "skv_paged_append_projected")


def skv_paged_decode_attention_folded(layer: PagedLayer, q_low: torch.Tensor, out_low: torch.Tensor, seq_lens,
                                      max_len: int, scale: float = 0.0, workspace: torch.Tensor | None = None,
                                      stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_paged_decode_attention_folded(C.byref(layer.c), q_low.data_ptr(), out_low.data_ptr(),
                                                   _lens_ptr(seq_lens, layer.batch), int(max_len), float(scale),
                                                   ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_paged_decode_attention_folded")


def skv_paged_decode_step_folded(layer: PagedLayer, k_low: torch.Tensor, v_low: torch.Tensor, cur_lens,
                                 max_cur_len: int, q_low: torch.Tensor, out_low: torch.Tensor, scale: float = 0.0,
                                 workspace: torch.Tensor | None = None, stream=None) -> None:
    assert k_low.is_contiguous() and v_low.is_contiguous()
    ws = layer.workspace() if workspace is None else workspace
    _check(lib().skv_paged_decode_step_folded(C.byref(layer.c), k_low.data_ptr(), v_low.data_ptr(), int(k_low.shape[1]),
                                              _lens_ptr(cur_lens, layer.batch), int(max_cur_len), q_low.data_ptr(),
                                              out_low.data_ptr(), float(scale), ws.data_ptr(),
                                              ws.numel() * ws.element_size(), _stream_ptr(stream)),
           "skv_paged_decode_step_folded")


def skv_paged_prefill_attention(layer: PagedLayer, q: torch.Tensor, out: torch.Tensor, n_prev: int,
                                scale: float = 0.0, mode: int = SKV_PREFILL_EXACT, stream=None) -> None:
    assert q.dtype == torch.bfloat16 and q.stride(3) == 1
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    sb, st, sh, _ = q.stride()
    _check(lib().skv_paged_prefill_attention(C.byref(layer.c), q.data_ptr(), sb, st, sh, out.data_ptr(),
                                             int(q.shape[1]), int(n_prev), float(scale), int(mode),
                                             _stream_ptr(stream)), "skv_paged_prefill_attention")


# ---- ranks that are not multiples of 16 --------------------------------------------------------


def skv_padded_rank(r: int) -> int:
    return int(lib().skv_padded_rank(int(r)))


def skv_pad_basis(basis: torch.Tensor, stream=None) -> torch.Tensor:
    """basis: bf16 CUDA [n_bases, 128, r] contiguous -> new tensor [n_bases, 128, skv_padded_rank(r)] whose
    extra columns are zero (the allocation is the binding's; the fill is the library's)."""
    assert basis.dtype == torch.bfloat16 and basis.is_contiguous() and basis.shape[1] == SKV_HEAD_DIM
    r = int(basis.shape[2])
    r_pad = skv_padded_rank(r)
    if r_pad == 0:
        raise SkvError(SKV_ERR_RANK, "skv_pad_basis")
    out = torch.empty((basis.shape[0], SKV_HEAD_DIM, r_pad), dtype=torch.bfloat16, device=basis.device)
    _check(lib().skv_pad_basis(basis.data_ptr(), int(basis.shape[0]), r, out.data_ptr(), _stream_ptr(stream)),
           "skv_pad_basis")
    return out


def skv_orthonormalize(a: torch.Tensor, r: int, pad: bool = True, stream=None) -> torch.Tensor:
    """a: float32 CUDA [n_bases, 128, 128] -> bf16 [n_bases, 128, r_out]: the leading r columns of each
    matrix's orthonormal factor (positive diagonal of R), zero-padded to a multiple of 16 if pad."""
    assert a.dtype == torch.float32 and a.is_contiguous() and a.shape[1:] == (SKV_HEAD_DIM, SKV_HEAD_DIM)
    r_out = skv_padded_rank(r) if pad else int(r)
    if not 1 <= int(r) <= SKV_HEAD_DIM:
        raise SkvError(SKV_ERR_RANK, "skv_orthonormalize")
    out = torch.empty((a.shape[0], SKV_HEAD_DIM, r_out), dtype=torch.bfloat16, device=a.device)
    _check(lib().skv_orthonormalize(a.data_ptr(), int(a.shape[0]), int(r), 1 if pad else 0, out.data_ptr(),
                                    _stream_ptr(stream)), "skv_orthonormalize")
    return out


# ---- a chunk of queries (prefill) ---------------------------------------------------


def skv_prefill_attention(layer, q: torch.Tensor, out: torch.Tensor, n_prev: int, scale: float = 0.0,
                          mode: int = SKV_PREFILL_EXACT, stream=None) -> None:
    """q: bf16 [batch, T, n_q_heads, 128] (last axis contiguous); out: float32 of the same shape,
    contiguous.  The chunk's rows [n_prev, n_prev + T) must already be in the cache."""
    assert q.dtype == torch.bfloat16 and q.stride(3) == 1
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    sb, st, sh, _ = q.stride()
    _check(lib().skv_prefill_attention(_base_ref(layer), q.data_ptr(), sb, st, sh, out.data_ptr(),
                                       int(q.shape[1]), int(n_prev), float(scale), int(mode),
                                       _stream_ptr(stream)), "skv_prefill_attention")


def skv_prefill_attention_folded(layer, q_low: torch.Tensor, out_low: torch.Tensor, n_prev: int,
                                 scale: float = 0.0, mode: int = SKV_PREFILL_EXACT, stream=None) -> None:
    """q_low: bf16 [batch, T, n_q_heads, r_k] contiguous; out_low: float32 [batch, T, n_q_heads, r_v]."""
    assert q_low.dtype == torch.bfloat16 and q_low.is_contiguous()
    assert out_low.dtype == torch.float32 and out_low.is_contiguous()
    _check(lib().skv_prefill_attention_folded(_base_ref(layer), q_low.data_ptr(), out_low.data_ptr(),
                                              int(q_low.shape[1]), int(n_prev), float(scale), int(mode),
                                              _stream_ptr(stream)), "skv_prefill_attention_folded")


def skv_prefill_step(layer, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor, out: torch.Tensor,
                     cur_len: int, scale: float = 0.0, mode: int = SKV_PREFILL_EXACT, stream=None) -> None:
    """Append the chunk k_new/v_new ([batch, T, n_kv_heads, 128]) at cur_len, then attend it causally."""
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16 and q.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1 and q.stride(3) == 1
    assert out.dtype == torch.float32 and out.is_contiguous() and out.shape == q.shape
    sb, st, sh, _ = k_new.stride()
    qb, qt, qh, _ = q.stride()
    _check(lib().skv_prefill_step(_base_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                  q.data_ptr(), qb, qt, qh, out.data_ptr(), int(q.shape[1]), int(cur_len),
                                  float(scale), int(mode), _stream_ptr(stream)), "skv_prefill_step")


def skv_prefill_tile_tokens(layer) -> int:
    return int(lib().skv_prefill_tile_tokens(_base_ref(layer)))


# ---- quantised cache (8- or 4-bit codes; a QuantLayer knows its width) ------------------------


def _qfn(layer: "QuantLayer", name: str, bits: int):
    """The C function of that name for the given code width; it must be the layer's."""
    assert layer.bits == bits, f"a {layer.bits}-bit layer was passed to a q{bits} call"
    return getattr(lib(), f"skv_q{bits}_{name}")


def _q_project_append(bits, layer: QuantLayer, k_new: torch.Tensor, v_new: torch.Tensor, cur_len: int,
                      stream=None) -> None:
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    sb, st, sh, _ = k_new.stride()
    _check(_qfn(layer, "project_append", bits)(_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                               int(k_new.shape[1]), int(cur_len), _stream_ptr(stream)),
           f"skv_q{bits}_project_append")


def _q_decode_attention(bits, layer: QuantLayer, q: torch.Tensor, out: torch.Tensor, n_ctx: int,
                        scale: float = 0.0, workspace: torch.Tensor | None = None, stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(_qfn(layer, "decode_attention", bits)(_ref(layer), q.data_ptr(), out.data_ptr(), int(n_ctx), float(scale),
                                                 ws.data_ptr(), ws.numel() * ws.element_size(), _stream_ptr(stream)),
           f"skv_q{bits}_decode_attention")


def _q_decode_step(bits, layer: QuantLayer, k_new: torch.Tensor, v_new: torch.Tensor, cur_len: int,
                   q: torch.Tensor, out: torch.Tensor, scale: float = 0.0,
                   workspace: torch.Tensor | None = None, stream=None) -> None:
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    sb, st, sh, _ = k_new.stride()
    ws = layer.workspace() if workspace is None else workspace
    _check(_qfn(layer, "decode_step", bits)(_ref(layer), k_new.data_ptr(), v_new.data_ptr(), sb, st, sh,
                                            int(k_new.shape[1]), int(cur_len), q.data_ptr(), out.data_ptr(),
                                            float(scale), ws.data_ptr(), ws.numel() * ws.element_size(),
                                            _stream_ptr(stream)), f"skv_q{bits}_decode_step")


def _q_decode_project_query(bits, layer: QuantLayer, q: torch.Tensor, scale: float = 0.0,
                            workspace: torch.Tensor | None = None, stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(_qfn(layer, "decode_project_query", bits)(_ref(layer), q.data_ptr(), float(scale), ws.data_ptr(),
                                                     ws.numel() * ws.element_size(), _stream_ptr(stream)),
           f"skv_q{bits}_decode_project_query")


def _q_decode_partial(bits, layer: QuantLayer, n_ctx: int, n_splits: int = 0,
                      workspace: torch.Tensor | None = None, stream=None) -> None:
    ws = layer.workspace() if workspace is None else workspace
    _check(_qfn(layer, "decode_partial", bits)(_ref(layer), int(n_ctx), int(n_splits), ws.data_ptr(),
                                               ws.numel() * ws.element_size(), _stream_ptr(stream)),
           f"skv_q{bits}_decode_partial")


def _q_cache_bytes(bits, layer: QuantLayer, n_tokens: int) -> int:
    return int(_qfn(layer, "cache_bytes", bits)(_ref(layer), int(n_tokens)))


def _bind(fn, bits):
    def bound(*a, **kw):
        return fn(bits, *a, **kw)
    bound.__doc__ = fn.__doc__
    return bound


skv_q8_project_append, skv_q4_project_append = _bind(_q_project_append, 8), _bind(_q_project_append, 4)
skv_q8_decode_attention, skv_q4_decode_attention = _bind(_q_decode_attention, 8), _bind(_q_decode_attention, 4)
skv_q8_decode_step, skv_q4_decode_step = _bind(_q_decode_step, 8), _bind(_q_decode_step, 4)
skv_q8_decode_project_query, skv_q4_decode_project_query = (_bind(_q_decode_project_query, 8),
                                                            _bind(_q_decode_project_query, 4))
skv_q8_decode_partial, skv_q4_decode_partial = _bind(_q_decode_partial, 8), _bind(_q_decode_partial, 4)
skv_q8_cache_bytes, skv_q4_cache_bytes = _bind(_q_cache_bytes, 8), _bind(_q_cache_bytes, 4)


def _q_default_splits(bits, layer: QuantLayer, n_ctx: int) -> int:
    return int(_qfn(layer, "decode_default_splits", bits)(_ref(layer), int(n_ctx)))


skv_q8_decode_default_splits, skv_q4_decode_default_splits = _bind(_q_default_splits, 8), _bind(_q_default_splits, 4)
