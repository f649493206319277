"""Quantised rows in pages on the GPU against the oracle: codes and value ranges placed through the block
table, decode attention over identical pool bytes, and decode steps, for 8- and 4-bit codes."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, vec_rel_err
from test_gpu_quant import pack_codes, unpack_codes

pytestmark = pytest.mark.gpu


def _f64(t):
    return O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))


def _lens_t(lens):
    return torch.tensor(lens, dtype=torch.int32, device="cuda")


class QPagedPair:
    """The same quantised paged layer on the GPU and in the oracle (same bases, static key ranges, block table)."""

    def __init__(self, seed, bits, batch, hq, hkv, r_k, r_v, page_tokens, max_pages, spare_pages=3):
        self.bits, self.batch, self.hq, self.hkv, self.r_k, self.r_v = bits, batch, hq, hkv, r_k, r_v
        self.pt = page_tokens
        self.n_pages = batch * max_pages + spare_pages
        _, pk = synth.orthonormal_bases(synth.stable_seed(seed, "pk"), hkv, 128, r_k)
        _, pv = synth.orthonormal_bases(synth.stable_seed(seed, "pv"), hkv, 128, r_v)
        self.scales_k = synth.channel_scales(synth.stable_seed(seed, "sk"), hkv, 128)
        self.scales_v = synth.channel_scales(synth.stable_seed(seed, "sv"), hkv, 128)
        cal = _f64(synth.kv_activations(synth.stable_seed(seed, "cal"), 1, 512, hkv, 128, self.scales_k))
        ngk, ngv = len(O.group_slices(r_k)), len(O.group_slices(r_v))
        ks, kz = np.empty((hkv, ngk), np.float32), np.empty((hkv, ngk), np.float32)
        for h in range(hkv):
            ks[h], kz[h] = O.calibrate_static_range(O.compress(cal[0, :, h], _f64(pk)[h]), bits)
        self.ora = O.new_quant_layer(batch, hq, hkv, 128, _f64(pk), _f64(pv), ks, kz, page_tokens * max_pages, bits)
        rng = np.random.default_rng(synth.stable_seed(seed, "table"))
        self.table = rng.permutation(self.n_pages)[:batch * max_pages].reshape(batch, max_pages).astype(np.int32)
        shape = (self.n_pages, hkv, page_tokens)
        # unwritten rows: code 0xEE / 0x0E and a NaN scale, so that any read of them shows in the output
        fill = 0xEE if bits == 8 else 0x0E
        self.cache = O.OraclePagedQuantCache(np.full(shape + (r_k,), fill, np.uint8), np.full(shape + (r_v,), fill, np.uint8),
                                             np.full(shape + (ngv,), 0x7FC1, np.uint16), np.full(shape + (ngv,), 0, np.uint16),
                                             self.table, page_tokens)
        self.gpu = B.PagedLayer(batch, hq, hkv, pk.cuda(), pv.cuda(), page_tokens, self.n_pages,
                                torch.from_numpy(self.table).cuda(), bits=bits, k_scale=torch.from_numpy(ks),
                                k_zero=torch.from_numpy(kz))
        self.upload()

    def raw_kv(self, seed, T):
        k = synth.kv_activations(synth.stable_seed(seed, "k"), self.batch, T, self.hkv, 128, self.scales_k, "cuda")
        v = synth.kv_activations(synth.stable_seed(seed, "v"), self.batch, T, self.hkv, 128, self.scales_v, "cuda")
        return k, v

    def upload(self):
        """The oracle's pools, in the GPU's packing, to the GPU layer."""
        self.gpu.k_pool.copy_(torch.from_numpy(pack_codes(self.cache.k_codes, self.bits)).cuda())
        self.gpu.v_pool.copy_(torch.from_numpy(pack_codes(self.cache.v_codes, self.bits)).cuda())
        meta = self.cache.v_scale_bits.astype(np.uint32) | (self.cache.v_zero_bits.astype(np.uint32) << 16)
        self.gpu.v_meta.copy_(torch.from_numpy(meta.view(np.int32)).cuda())

    def oracle_append(self, k, v, cur):
        O.paged_quant_project_append(self.ora, self.cache, _f64(k), _f64(v), cur)

    def fill(self, seed, lens):
        k, v = self.raw_kv(seed, max(max(lens), 1))
        for b, n_b in enumerate(lens):
            if n_b:
                one = O.new_quant_layer(1, self.hq, self.hkv, 128, self.ora.p_k, self.ora.p_v, self.ora.k_scale,
                                        self.ora.k_zero, n_b, self.bits)
                sub = O.OraclePagedQuantCache(self.cache.k_codes, self.cache.v_codes, self.cache.v_scale_bits,
                                              self.cache.v_zero_bits, self.table[b:b + 1], self.pt)
                O.paged_quant_project_append(one, sub, _f64(k[b:b + 1, :n_b]), _f64(v[b:b + 1, :n_b]), [0])
        self.upload()

    def queries(self, seed):
        return synth.queries(synth.stable_seed(seed, "q"), self.batch, self.hq, 128, "cuda")


@pytest.mark.parametrize("bits,r_k,r_v", [(8, 64, 64), (8, 32, 96), (8, 128, 128), (4, 64, 64), (4, 128, 64)])
@pytest.mark.parametrize("page_tokens", [64, 128])
def test_paged_quantised_decode_on_identical_pool_bytes(bits, r_k, r_v, page_tokens):
    lens = [1100, 1, 300, 0]
    P = QPagedPair(("pq-dec", bits, r_k, r_v, page_tokens), bits, 4, 8, 2, r_k, r_v, page_tokens, 1152 // page_tokens)
    P.fill(1, lens)
    q = P.queries(2)
    out = torch.full((4, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    B.skv_paged_decode_attention(P.gpu, q, out, _lens_t(lens), 1100)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = O.paged_quant_decode_attention(P.ora, P.cache, _f64(q), lens)
    assert np.all(np.isfinite(got))                       # unwritten rows carry a NaN scale
    for b, n in enumerate(lens):
        assert np.all(got[b] == 0.0) if n == 0 else vec_rel_err(got[b], want[b]) <= TOL
    # uniform length, no length array
    P2 = QPagedPair(("pq-dec-u", bits, r_k, r_v), bits, 2, 8, 2, r_k, r_v, page_tokens, 512 // page_tokens)
    P2.fill(3, [333, 333])
    out2 = torch.full((2, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    q2 = P2.queries(4)
    B.skv_paged_decode_attention(P2.gpu, q2, out2, None, 333)
    torch.cuda.synchronize()
    assert vec_rel_err(out2.cpu().numpy(), O.paged_quant_decode_attention(P2.ora, P2.cache, _f64(q2), [333, 333])) <= TOL


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("T,cur", [(1, [0, 63, 64]), (3, [62, 127, 200]), (150, [10, 64, 0])])
def test_paged_quantised_append_places_codes_and_ranges(bits, T, cur):
    P = QPagedPair(("pq-app", bits, T), bits, 3, 8, 2, 64, 128, 64, 8)
    k, v = P.raw_kv(1, T)
    B.skv_paged_project_append(P.gpu, k, v, _lens_t(cur), max(cur))
    torch.cuda.synchronize()
    before_k, before_meta = P.cache.k_codes.copy(), P.cache.v_scale_bits.copy()
    P.oracle_append(k, v, cur)
    gk = unpack_codes(P.gpu.k_pool.cpu().numpy(), bits)
    gv = unpack_codes(P.gpu.v_pool.cpu().numpy(), bits)
    gm = P.gpu.v_meta.cpu().numpy().view(np.uint32)
    written = np.any(P.cache.k_codes != before_k, axis=-1) | np.any(P.cache.v_scale_bits != before_meta, axis=-1)
    assert written.sum() >= 3 * 2 * T - 2                           # (a written row can equal the fill pattern only by accident)
    # rows the oracle did not write keep their contents
    assert np.array_equal(gk[~written], before_k[~written])
    assert np.all(gm[~written] == (0x7FC1 | (0 << 16)))
    # keys: static ranges, codes differ only where float32 and float64 sums straddle a rounding boundary
    dk = np.abs(gk[written].astype(int) - P.cache.k_codes[written].astype(int))
    assert dk.max() <= 1 and (dk > 0).mean() < 0.01
    # values: nearly all rows carry the oracle's range bit for bit, and then the same codes up to such straddles
    want_meta = P.cache.v_scale_bits.astype(np.uint32) | (P.cache.v_zero_bits.astype(np.uint32) << 16)
    same = (gm == want_meta) & written[..., None]
    assert same.sum() > 0.98 * written.sum() * gm.shape[-1]
    for gi, g in enumerate(O.group_slices(128)):
        rows = same[..., gi]
        dv = np.abs(gv[..., g][rows].astype(int) - P.cache.v_codes[..., g][rows].astype(int))
        assert dv.max() <= 1 and (dv > 0).mean() < 0.01


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("T", [1, 5])
def test_paged_quantised_decode_steps(bits, T):
    # Each side appends into its own pools.  The library decides a code in float32 on a float32 sum, the oracle
    # in float64, so a few codes sit one apart; as for the contiguous cache the end-to-end statement is two
    # facts: the pools the library built are the oracle's up to such flips, and on the very bytes the library
    # stored its attention output is the oracle's within the stated 2e-3.
    lens = [60, 126, 0, 500]
    P = QPagedPair(("pq-step", bits, T), bits, 4, 8, 2, 64, 64, 64, 9)
    # Every sequence is given the longest one's rows (one batch-wide append on either side); the lengths then
    # select how many of them count, and the steps overwrite from each sequence's own length on.
    k0, v0 = P.raw_kv(1, 500)
    n_max = max(lens)
    B.skv_paged_project_append(P.gpu, k0[:, :n_max], v0[:, :n_max], None, 0)
    torch.cuda.synchronize()
    P.oracle_append(k0[:, :n_max], v0[:, :n_max], [0, 0, 0, 0])      # every sequence holds n_max rows; lengths select
    cur = list(lens)
    out = torch.full((4, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    for s in range(3):
        k, v = P.raw_kv(("s", s), T)
        q = P.queries(("s", s))
        B.skv_paged_decode_step(P.gpu, k, v, _lens_t(cur), max(cur), q, out)
        torch.cuda.synchronize()
        P.oracle_append(k, v, cur)
        cur = [c + T for c in cur]
        got = out.cpu().numpy()
        assert np.all(np.isfinite(got))
        # (1) the library's pools against the oracle's, over the rows either side has written
        gk = unpack_codes(P.gpu.k_pool.cpu().numpy(), bits)
        gv = unpack_codes(P.gpu.v_pool.cpu().numpy(), bits)
        gm = P.gpu.v_meta.cpu().numpy().view(np.uint32)
        written = P.cache.v_scale_bits[..., 0] != 0x7FC1
        dk = np.abs(gk[written].astype(int) - P.cache.k_codes[written].astype(int))
        assert dk.max() <= 1 and (dk > 0).mean() < 0.01
        want_meta = P.cache.v_scale_bits.astype(np.uint32) | (P.cache.v_zero_bits.astype(np.uint32) << 16)
        same = (gm[..., 0] == want_meta[..., 0]) & written
        assert same.sum() > 0.98 * written.sum()
        dv = np.abs(gv[same].astype(int) - P.cache.v_codes[same].astype(int))
        assert dv.max() <= 1 and (dv > 0).mean() < 0.01
        # (2) the oracle's attention over the library's own pool bytes
        mine = O.OraclePagedQuantCache(gk, gv, (gm & 0xffff).astype(np.uint16), (gm >> 16).astype(np.uint16),
                                       P.table, P.pt)
        want = O.paged_quant_decode_attention(P.ora, mine, _f64(q), cur)
        assert vec_rel_err(got, want) <= TOL
        if bits == 8:
            # one step of an 8-bit code is well inside the tolerance: each side on its own pools as well
            assert vec_rel_err(got, O.paged_quant_decode_attention(P.ora, P.cache, _f64(q), cur)) <= TOL
