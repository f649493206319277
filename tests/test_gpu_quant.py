"""GPU parity of the quantised cache (Sec. 4.3; 8- and 4-bit codes) against the oracle: codes
and per-row value ranges written by the append, decode attention over identical cache
bytes, and the fused decode step."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, vec_rel_err

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("decode_engine")]


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Oracle codes (one per byte) in the GPU cache's packing: 4-bit codes two per byte, even channel low."""
    if bits == 8:
        return codes
    return (codes[..., 0::2] | (codes[..., 1::2] << 4)).astype(np.uint8)


def unpack_codes(packed: np.ndarray, bits: int) -> np.ndarray:
    if bits == 8:
        return packed
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = packed & 0x0F
    out[..., 1::2] = packed >> 4
    return out


RANKS = {8: [(64, 64), (32, 96), (96, 32), (128, 128), (64, 128)], 4: [(64, 64), (128, 128), (64, 128)]}
CASES = [(bits, rk, rv) for bits in (8, 4) for rk, rv in RANKS[bits]]


def _fns(bits):
    return {8: (B.skv_q8_project_append, B.skv_q8_decode_attention, B.skv_q8_decode_step, B.skv_q8_decode_project_query,
                B.skv_q8_decode_partial, B.skv_q8_cache_bytes),
            4: (B.skv_q4_project_append, B.skv_q4_decode_attention, B.skv_q4_decode_step, B.skv_q4_decode_project_query,
                B.skv_q4_decode_partial, B.skv_q4_cache_bytes)}[bits]


class QPair:
    """The same quantised layer on the GPU and in the oracle (same bases, same static key ranges)."""

    def __init__(self, seed, batch, hq, hkv, r_k, r_v, capacity, bits=8):
        self.batch, self.hq, self.hkv, self.r_k, self.r_v, self.capacity = batch, hq, hkv, r_k, r_v, capacity
        self.bits = bits
        _, pk = synth.orthonormal_bases(synth.stable_seed(seed, "pk"), hkv, 128, r_k)
        _, pv = synth.orthonormal_bases(synth.stable_seed(seed, "pv"), hkv, 128, r_v)
        self.pk64 = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(pk))
        self.pv64 = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(pv))
        self.scales_k = synth.channel_scales(synth.stable_seed(seed, "sk"), hkv, 128)
        self.scales_v = synth.channel_scales(synth.stable_seed(seed, "sv"), hkv, 128)
        # static key ranges: calibrated by the oracle on a seeded sample of projected keys
        cal = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(
            synth.kv_activations(synth.stable_seed(seed, "cal"), 1, 512, hkv, 128, self.scales_k)))
        ngk = len(O.group_slices(r_k))
        ks, kz = np.empty((hkv, ngk), np.float32), np.empty((hkv, ngk), np.float32)
        for h in range(hkv):
            ks[h], kz[h] = O.calibrate_static_range(O.compress(cal[0, :, h], self.pk64[h]), bits)
        self.ora = O.new_quant_layer(batch, hq, hkv, 128, self.pk64, self.pv64, ks, kz, capacity, bits)
        self.gpu = B.QuantLayer(batch, hq, hkv, pk.cuda(), pv.cuda(), torch.from_numpy(ks), torch.from_numpy(kz), capacity,
                                bits)

    def raw_kv(self, seed, T):
        k = synth.kv_activations(synth.stable_seed(seed, "k"), self.batch, T, self.hkv, 128, self.scales_k, "cuda")
        v = synth.kv_activations(synth.stable_seed(seed, "v"), self.batch, T, self.hkv, 128, self.scales_v, "cuda")
        return k, v

    def oracle_append(self, k, v, cur):
        f = lambda t: O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))
        O.quant_project_append(self.ora, f(k), f(v), cur)

    def upload_oracle_cache(self, n):
        self.gpu.k_cache[:, :, :n] = torch.from_numpy(pack_codes(self.ora.k_codes[:, :, :n], self.bits)).cuda()
        self.gpu.v_cache[:, :, :n] = torch.from_numpy(pack_codes(self.ora.v_codes[:, :, :n], self.bits)).cuda()
        meta = self.ora.v_scale_bits[:, :, :n].astype(np.uint32) | (self.ora.v_zero_bits[:, :, :n].astype(np.uint32) << 16)
        self.gpu.v_meta[:, :, :n] = torch.from_numpy(meta.view(np.int32)).cuda()

    def queries(self, seed):
        return synth.queries(synth.stable_seed(seed, "q"), self.batch, self.hq, 128, "cuda")

    def oracle_decode(self, q, n, scale=None):
        return O.quant_decode_attention(self.ora, O.bf16_bits_to_f64(synth.torch_bf16_to_bits(q)), n, scale)

    def oracle_layer_over_gpu_cache(self, n):
        """An oracle layer whose rows [0, n) are the codes and value ranges the GPU stored (same bases, same
        static key ranges): what the oracle's attention gives on exactly those cache bytes."""
        lay = O.new_quant_layer(self.batch, self.hq, self.hkv, 128, self.pk64, self.pv64, self.ora.k_scale,
                                self.ora.k_zero, self.capacity, self.bits)
        lay.k_codes[:, :, :n] = unpack_codes(self.gpu.k_cache[:, :, :n].cpu().numpy(), self.bits)
        lay.v_codes[:, :, :n] = unpack_codes(self.gpu.v_cache[:, :, :n].cpu().numpy(), self.bits)
        meta = self.gpu.v_meta[:, :, :n].cpu().numpy().view(np.uint32)
        lay.v_scale_bits[:, :, :n] = (meta & 0xffff).astype(np.uint16)
        lay.v_zero_bits[:, :, :n] = (meta >> 16).astype(np.uint16)
        return lay


@pytest.mark.parametrize("bits,r_k,r_v", CASES)
@pytest.mark.parametrize("batch,T,cur", [(2, 1, 5), (1, 40, 0), (2, 100, 7), (3, 333, 0),   # the last three: matrix-core chunk path;
                                         (1, 20500, 0)])   # 20500 rows: some waves take three tiles, in two turns of the kernel's loop
def test_quantised_append_codes_and_ranges(bits, r_k, r_v, batch, T, cur):
    append_fn = _fns(bits)[0]
    P = QPair(("qapp", r_k, r_v, T), batch, 8, 4, r_k, r_v, cur + T + 3, bits)
    P.gpu.k_cache.fill_(201)
    P.gpu.v_cache.fill_(202)
    P.gpu.v_meta.fill_(-7)
    k, v = P.raw_kv(1, T)
    append_fn(P.gpu, k, v, cur)
    torch.cuda.synchronize()
    P.oracle_append(k, v, cur)
    sl = slice(cur, cur + T)
    raw_k, raw_v = P.gpu.k_cache.cpu().numpy(), P.gpu.v_cache.cpu().numpy()
    gk, gv = unpack_codes(raw_k, bits), unpack_codes(raw_v, bits)
    gm = P.gpu.v_meta.cpu().numpy().view(np.uint32)
    # keys: static ranges, so codes can differ only where float32 and float64 sums straddle a rounding boundary
    dk = np.abs(gk[:, :, sl].astype(int) - P.ora.k_codes[:, :, sl].astype(int))
    assert dk.max() <= 1 and (dk > 0).mean() < 0.01
    # values: the stored (scale, zero) pairs are bf16 roundings of float32 results; nearly all rows match bit for bit
    want_meta = P.ora.v_scale_bits[:, :, sl].astype(np.uint32) | (P.ora.v_zero_bits[:, :, sl].astype(np.uint32) << 16)
    same = gm[:, :, sl] == want_meta
    assert same.mean() > 0.98
    dv = np.abs(gv[:, :, sl].astype(int) - P.ora.v_codes[:, :, sl].astype(int))
    for gi, g in enumerate(O.group_slices(r_v)):
        rows = same[..., gi]
        assert dv[..., g][rows].max() <= 1 and (dv[..., g][rows] > 0).mean() < 0.01
    # where a range differs, the dequantised rows still agree within one step
    g_s = O.bf16_bits_to_f64((gm[:, :, sl] & 0xffff).astype(np.uint16))
    g_z = O.bf16_bits_to_f64((gm[:, :, sl] >> 16).astype(np.uint16))
    o_s = O.bf16_bits_to_f64(P.ora.v_scale_bits[:, :, sl])
    o_z = O.bf16_bits_to_f64(P.ora.v_zero_bits[:, :, sl])
    for b in range(batch):
        for h in range(4):
            a = O.dequantize(gv[b, h, sl], g_s[b, h], g_z[b, h])
            c = O.dequantize(P.ora.v_codes[b, h, sl], o_s[b, h], o_z[b, h])
            step = np.repeat(np.maximum(g_s[b, h], o_s[b, h]), [g.stop - g.start for g in O.group_slices(r_v)], axis=1)
            assert np.all(np.abs(a - c) <= 1.51 * step)
    # untouched rows keep their contents
    rest = np.ones(P.capacity, bool)
    rest[sl] = False
    assert np.all(raw_k[:, :, rest] == 201) and np.all(raw_v[:, :, rest] == 202)
    assert np.all(P.gpu.v_meta.cpu().numpy()[:, :, rest] == -7)


@pytest.mark.parametrize("bits,r_k,r_v", [(8, 64, 64), (8, 32, 32), (8, 96, 128), (8, 128, 96), (8, 32, 128),
                                           (4, 64, 64), (4, 128, 64), (4, 64, 128), (4, 128, 128)])
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 2)])
def test_quantised_decode_matches_oracle_on_identical_cache_bytes(bits, r_k, r_v, hq, hkv):
    _, attention_fn, _, project_query_fn, partial_fn, _ = _fns(bits)
    n = 1337
    P = QPair(("qdec", r_k, r_v, hq), 2, hq, hkv, r_k, r_v, n, bits)
    k, v = P.raw_kv(2, n)
    P.oracle_append(k, v, 0)
    P.upload_oracle_cache(n)
    q = P.queries(3)
    out = torch.empty((2, hq, 128), dtype=torch.float32, device="cuda")
    for n_ctx in (n, 65, 1):
        attention_fn(P.gpu, q, out, n_ctx)
        torch.cuda.synchronize()
        assert vec_rel_err(out.cpu().numpy(), P.oracle_decode(q, n_ctx)) <= TOL
    # the three stages called one by one give the same bits as the fused call
    ref = out.clone()
    s_ = B.skv_decode_default_splits(P.gpu, 1)
    project_query_fn(P.gpu, q, 0.0)
    partial_fn(P.gpu, 1, s_)
    B.skv_decode_combine(P.gpu, out, s_)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


@pytest.mark.parametrize("bits", [8, 4])
def test_value_ranges_over_many_orders_of_magnitude(bits):
    """The matrix-core range kernel takes the codes as the bf16 numbers n * 2^-133 and carries the factor on the
    weights; value ranges from 2^-20 to 2^20 times the usual ones (row by row, in both the oracle's layer and the
    bytes uploaded) must come out as the definition says."""
    _, attention_fn, _, _, _, _ = _fns(bits)
    n, hq, hkv = 700, 8, 2
    P = QPair(("qdec-ranges", bits), 2, hq, hkv, 64, 64, n, bits)
    k, v = P.raw_kv(5, n)
    P.oracle_append(k, v, 0)
    shift = (((np.arange(n) * 7) % 41) - 20).astype(np.int32)          # exponent change per row
    for arr in (P.ora.v_scale_bits, P.ora.v_zero_bits):
        a = arr[:, :, :n].astype(np.int32)
        nonzero = (a & 0x7f80) != 0                                     # a zero point of exactly 0 stays 0
        a = np.where(nonzero, a + (shift[None, None, :, None] << 7), a)
        assert ((a & 0x7f80) != 0x7f80).all() and (a >= 0).all() and (a <= 0xffff).all()
        arr[:, :, :n] = a.astype(arr.dtype)
    P.upload_oracle_cache(n)
    q = P.queries(6)
    out = torch.empty((2, hq, 128), dtype=torch.float32, device="cuda")
    for n_ctx in (n, 33):
        attention_fn(P.gpu, q, out, n_ctx)
        torch.cuda.synchronize()
        assert vec_rel_err(out.cpu().numpy(), P.oracle_decode(q, n_ctx)) <= TOL


@pytest.mark.parametrize("bits,r_k,r_v", [(8, 64, 64), (8, 96, 128), (4, 64, 64), (4, 128, 128)])
def test_large_scores_move_the_softmax_reference_often(bits, r_k, r_v):
    """The matrix-core range kernel moves its softmax reference only when a score exceeds it by a margin and
    carries a power-of-two bias on the weights; under a scale 7 and 70 times the default (scores up to several
    hundred, in log2 units) the per-tile maxima differ by far more than that margin again and again."""
    _, attention_fn, _, _, _, _ = _fns(bits)
    n, hq, hkv = 2100, 8, 2
    P = QPair(("qdec-scale", bits, r_k, r_v), 2, hq, hkv, r_k, r_v, n, bits)
    k, v = P.raw_kv(7, n)
    P.oracle_append(k, v, 0)
    P.upload_oracle_cache(n)
    q = P.queries(8)
    out = torch.empty((2, hq, 128), dtype=torch.float32, device="cuda")
    for scale in (0.6, 6.0):
        for n_ctx in (n, 500):
            attention_fn(P.gpu, q, out, n_ctx, scale)
            torch.cuda.synchronize()
            assert torch.isfinite(out).all()
            assert vec_rel_err(out.cpu().numpy(), P.oracle_decode(q, n_ctx, scale)) <= TOL, (scale, n_ctx)


@pytest.mark.parametrize("bits", [8, 4])
def test_quantised_decode_steps_end_to_end(bits):
    # Append through the library, then a few fused decode steps; both sides keep their own caches.  A code is
    # an integer decided by floating point: the library decides it in float32 on a float32 sum, the oracle in
    # float64, so a few codes sit one apart.  The end-to-end statement is therefore made of two facts, each
    # held to its own bar: (1) the cache the library built is the oracle's up to such flips (codes at most one
    # apart, on fewer than 1 % of the entries; value ranges equal on more than 98 % of the rows), and (2) on
    # the very bytes the library stored, its attention output is the oracle's within the stated 2e-3.
    append_fn, _, step_fn, _, _, bytes_fn = _fns(bits)
    n0, steps = 900, 3
    P = QPair(("qe2e",), 2, 8, 2, 64, 64, n0 + steps, bits)
    k, v = P.raw_kv(4, n0)
    append_fn(P.gpu, k, v, 0)
    P.oracle_append(k, v, 0)
    out = torch.empty((2, 8, 128), dtype=torch.float32, device="cuda")
    for s in range(steps):
        k1, v1 = P.raw_kv(("s", s), 1)
        q = P.queries(("s", s))
        step_fn(P.gpu, k1, v1, n0 + s, q, out)
        torch.cuda.synchronize()
        P.oracle_append(k1, v1, n0 + s)
        n = n0 + s + 1
        mine = P.oracle_layer_over_gpu_cache(n)
        dk = np.abs(mine.k_codes[:, :, :n].astype(int) - P.ora.k_codes[:, :, :n].astype(int))
        dv = np.abs(mine.v_codes[:, :, :n].astype(int) - P.ora.v_codes[:, :, :n].astype(int))
        same = (mine.v_scale_bits[:, :, :n] == P.ora.v_scale_bits[:, :, :n]) & (mine.v_zero_bits[:, :, :n] == P.ora.v_zero_bits[:, :, :n])
        assert dk.max() <= 1 and (dk > 0).mean() < 0.01
        assert same.mean() > 0.98
        assert dv[same[..., 0]].max() <= 1 and (dv[same[..., 0]] > 0).mean() < 0.01
        q64 = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(q))
        assert vec_rel_err(out.cpu().numpy(), O.quant_decode_attention(mine, q64, n)) <= TOL
        if bits == 8:
            # one step of an 8-bit code is well inside the tolerance: each side on its own cache as well
            assert vec_rel_err(out.cpu().numpy(), P.oracle_decode(q, n)) <= TOL
    assert bytes_fn(P.gpu, 1000) == 2 * 2 * 1000 * (128 * bits // 8 + 4)
