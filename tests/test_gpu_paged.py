"""The paged cache on the GPU against the oracle: rows placed through the block table bit for bit,
decode attention, decode steps and chunk attention over shuffled pages, and bit-equality with the
contiguous cache holding the same rows (only addresses differ between the two)."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, vec_rel_err

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("decode_engine")]
SENTINEL = 0x7FC1                     # a NaN pattern: anything that reads an unwritten row shows


def _f64(t):
    return O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))


def _lens_t(lens):
    return torch.tensor(lens, dtype=torch.int32, device="cuda")


class PagedPair:
    """The same paged layer on the GPU and in the oracle: same bases, same block table (a seeded
    shuffle of the pool's pages, so that neighbouring logical pages are far apart), pools filled with NaN."""

    def __init__(self, seed, batch, hq, hkv, r_k, r_v, page_tokens, max_pages, spare_pages=3, shared_k=False):
        self.batch, self.hq, self.hkv, self.r_k, self.r_v = batch, hq, hkv, r_k, r_v
        self.pt, self.max_pages = page_tokens, max_pages
        self.n_pages = batch * max_pages + spare_pages
        _, pk = synth.orthonormal_bases(synth.stable_seed(seed, "pk"), 1 if shared_k else hkv, 128, r_k)
        _, pv = synth.orthonormal_bases(synth.stable_seed(seed, "pv"), hkv, 128, r_v)
        self.pk, self.pv = pk.cuda(), pv.cuda()
        rng = np.random.default_rng(synth.stable_seed(seed, "table"))
        self.table = rng.permutation(self.n_pages)[:batch * max_pages].reshape(batch, max_pages).astype(np.int32)
        self.ora = O.new_layer(batch, hq, hkv, 128, _f64(pk), _f64(pv), page_tokens * max_pages, store="bf16")
        self.cache = O.OraclePagedCache(np.full((self.n_pages, hkv, page_tokens, r_k), np.nan),
                                        np.full((self.n_pages, hkv, page_tokens, r_v), np.nan), self.table, page_tokens)
        mk = lambda r: torch.full((self.n_pages, hkv, page_tokens, r), SENTINEL, dtype=torch.int16,
                                  device="cuda").view(torch.bfloat16)
        self.gpu = B.PagedLayer(batch, hq, hkv, self.pk, self.pv, page_tokens, self.n_pages,
                                torch.from_numpy(self.table).cuda(), mk(r_k), mk(r_v))
        self.scales_k = synth.channel_scales(synth.stable_seed(seed, "sk"), hkv, 128)
        self.scales_v = synth.channel_scales(synth.stable_seed(seed, "sv"), hkv, 128)

    def raw_kv(self, seed, T):
        k = synth.kv_activations(synth.stable_seed(seed, "k"), self.batch, T, self.hkv, 128, self.scales_k, "cuda")
        v = synth.kv_activations(synth.stable_seed(seed, "v"), self.batch, T, self.hkv, 128, self.scales_v, "cuda")
        return k, v

    def oracle_append(self, k, v, cur_lens):
        O.paged_project_append(self.ora, self.cache, _f64(k), _f64(v), cur_lens)

    def upload_oracle_pools(self):
        """The oracle's pools (its own bf16 bits; unwritten rows stay NaN) to the GPU layer."""
        for src, dst in ((self.cache.k_pool, self.gpu.k_pool), (self.cache.v_pool, self.gpu.v_pool)):
            bits = O.f64_to_bf16_bits(np.nan_to_num(src, nan=0.0))
            bits[np.isnan(src)] = SENTINEL
            dst.copy_(synth.bits_to_torch_bf16(bits, "cuda"))

    def fill(self, seed, lens):
        """Both sides hold lens[b] rows of sequence b, written by the oracle's append."""
        n = max(lens)
        k, v = self.raw_kv(seed, max(n, 1))
        for b, n_b in enumerate(lens):
            if n_b:
                one = O._one_sequence(self.ora, b)
                sub = O.OraclePagedCache(self.cache.k_pool, self.cache.v_pool, self.table[b:b + 1], self.pt)
                O.paged_project_append(one, sub, _f64(k[b:b + 1, :n_b]), _f64(v[b:b + 1, :n_b]), [0])
        self.upload_oracle_pools()

    def contiguous_gpu(self, lens):
        """A contiguous GPU layer holding the same rows (gathered by the oracle's row-by-row definition)."""
        cap = self.pt * self.max_pages
        flat = O.paged_as_contiguous(self.ora, self.cache, lens)
        L = B.Layer(self.batch, self.hq, self.hkv, self.pk, self.pv, cap)
        for src, dst in ((flat.k_cache, L.k_cache), (flat.v_cache, L.v_cache)):
            bits = np.full((self.batch, self.hkv, cap, src.shape[3]), SENTINEL, np.uint16)
            m = src.shape[2]
            part = O.f64_to_bf16_bits(np.nan_to_num(src, nan=0.0))
            part[np.isnan(src)] = SENTINEL
            bits[:, :, :m] = part
            dst.copy_(synth.bits_to_torch_bf16(bits, "cuda"))
        return L

    def queries(self, seed):
        return synth.queries(synth.stable_seed(seed, "q"), self.batch, self.hq, 128, "cuda")

    def pool_bits(self):
        return (self.gpu.k_pool.view(torch.int16).cpu().numpy().view(np.uint16),
                self.gpu.v_pool.view(torch.int16).cpu().numpy().view(np.uint16))


def _assert_pools_match(P):
    """Placement must be exact: every row the oracle wrote holds the oracle's values (the same bits, except
    where the GPU's float32 sum and the oracle's float64 sum straddle a rounding boundary: well under 1 % of
    the entries, each within a bf16 step plus the float32 summation error), and every other row of the pool
    keeps its contents."""
    gk, gv = P.pool_bits()
    for got, want in ((gk, P.cache.k_pool), (gv, P.cache.v_pool)):
        written = ~np.isnan(want)
        assert np.all(got[~written] == SENTINEL)
        w = want[written]
        assert (got[written] != O.f64_to_bf16_bits(w)).mean() < 0.01
        g = O.bf16_bits_to_f64(got[written])
        assert np.all(np.abs(g - w) <= 2.0 ** -7 * np.abs(w) + 128 * 2.0 ** -24 * np.abs(w).max())


@pytest.mark.parametrize("page_tokens", [64, 128])
@pytest.mark.parametrize("T,cur", [(1, [0, 63, 64]), (3, [62, 127, 200]), (40, [50, 0, 100]), (150, [10, 64, 0])])
def test_paged_append_places_rows_through_the_table(page_tokens, T, cur):
    # few tokens: vector projections; many: the matrix-core chunk path; rows straddle page ends
    P = PagedPair(("pg-append", page_tokens, T), 3, 8, 2, 64, 80, page_tokens, 512 // page_tokens)
    k, v = P.raw_kv(1, T)
    B.skv_paged_project_append(P.gpu, k, v, _lens_t(cur), max(cur))
    torch.cuda.synchronize()
    P.oracle_append(k, v, cur)
    _assert_pools_match(P)


def test_paged_append_with_uniform_length_and_shared_key_basis():
    P = PagedPair(("pg-append-u",), 2, 4, 4, 48, 32, 64, 4, shared_k=True)
    k, v = P.raw_kv(2, 70)
    B.skv_paged_project_append(P.gpu, k, v, None, 60)
    torch.cuda.synchronize()
    P.oracle_append(k, v, [60, 60])
    _assert_pools_match(P)


RANKS = [(16, 128), (32, 48), (48, 80), (64, 64), (80, 32), (96, 112), (112, 16), (128, 128)]


@pytest.mark.parametrize("r_k,r_v", RANKS)
@pytest.mark.parametrize("page_tokens", [64, 256])
def test_paged_decode_matches_oracle_and_contiguous_cache(r_k, r_v, page_tokens):
    lens = [1500, 1, 700, 0]
    P = PagedPair(("pg-dec", r_k, r_v, page_tokens), 4, 8, 2, r_k, r_v, page_tokens, 1536 // page_tokens)
    P.fill(1, lens)
    q = P.queries(2)
    out = torch.full((4, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    B.skv_paged_decode_attention(P.gpu, q, out, _lens_t(lens), 1500)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = O.paged_decode_attention(P.ora, P.cache, _f64(q), lens)
    assert np.all(np.isfinite(got))                              # unwritten rows and spare pages hold NaN
    for b, n in enumerate(lens):
        if n == 0:
            assert np.all(got[b] == 0.0)
        else:
            assert vec_rel_err(got[b], want[b]) <= TOL
    # the contiguous cache with the same rows runs the same arithmetic in the same order
    L = P.contiguous_gpu(lens)
    ref = torch.empty_like(out)
    B.skv_decode_attention_varlen(L, q, ref, _lens_t(lens), 1500)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    # the two launches of the call, one by one
    s_ = B.skv_decode_default_splits(P.gpu, 1500)
    out.fill_(float("nan"))
    B.skv_paged_decode_partial_q(P.gpu, q, _lens_t(lens), 1500, s_)
    B.skv_decode_combine(P.gpu, out, s_)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 4), (16, 2)])
def test_paged_decode_head_groupings_uniform_length(hq, hkv):
    n = 1337
    P = PagedPair(("pg-group", hq, hkv), 2, hq, hkv, 64, 64, 128, 11)
    P.fill(3, [n, n])
    q = P.queries(4)
    out = torch.full((2, hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    for n_ctx in (n, 129, 64, 1):
        B.skv_paged_decode_attention(P.gpu, q, out, None, n_ctx)
        torch.cuda.synchronize()
        want = O.paged_decode_attention(P.ora, P.cache, _f64(q), [n_ctx, n_ctx])
        assert vec_rel_err(out.cpu().numpy(), want) <= TOL


def test_paged_decode_ranges_longer_than_the_held_table_window():
    # one range covers more than 64 pages, so a wave refills the table entries it holds
    batch, heads, n = 8, 8, 40000
    P = PagedPair(("pg-long",), batch, heads, heads, 16, 16, 64, 626, spare_pages=5)
    rng = np.random.default_rng(7)
    # pools filled directly with bf16-exact values (the append is not under test here)
    for pool_o, pool_g in ((P.cache.k_pool, P.gpu.k_pool), (P.cache.v_pool, P.gpu.v_pool)):
        vals = torch.randn(pool_g.shape, generator=torch.Generator().manual_seed(int(rng.integers(1 << 30)))).to(torch.bfloat16)
        pool_g.copy_(vals.cuda())
        pool_o[...] = _f64(vals)
    q = P.queries(5)
    out = torch.empty((batch, heads, 128), dtype=torch.float32, device="cuda")
    B.skv_paged_decode_attention(P.gpu, q, out, None, n)
    torch.cuda.synchronize()
    # the oracle on one sequence (the others are covered by the contiguous cache below)
    one = O._one_sequence(P.ora, 3)
    sub = O.OraclePagedCache(P.cache.k_pool, P.cache.v_pool, P.table[3:4], 64)
    want = O.paged_decode_attention(one, sub, _f64(q)[3:4], [n])
    assert vec_rel_err(out[3:4].cpu().numpy(), want) <= TOL
    L = P.contiguous_gpu([n] * batch)
    lo, hi = B.skv_decode_range(n, B.skv_decode_default_splits(L, n), 0)
    assert hi - lo > 64 * 64                                     # the premise of this test
    ref = torch.empty_like(out)
    B.skv_decode_attention(L, q, ref, n)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


@pytest.mark.parametrize("T", [1, 3, 4, 6])
def test_paged_decode_steps_cross_page_ends(T):
    # fused step for T <= 4, append + attention beyond; several steps so that rows cross into fresh pages
    lens = [60, 126, 0, 300]
    P = PagedPair(("pg-step", T), 4, 8, 2, 64, 64, 64, 8)
    P.fill(6, lens)
    cur = list(lens)
    out = torch.full((4, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    for s in range(3):
        k, v = P.raw_kv(("s", s), T)
        q = P.queries(("s", s))
        B.skv_paged_decode_step(P.gpu, k, v, _lens_t(cur), max(cur), q, out)
        torch.cuda.synchronize()
        P.oracle_append(k, v, cur)
        cur = [c + T for c in cur]
        want = O.paged_decode_attention(P.ora, P.cache, _f64(q), cur)
        assert vec_rel_err(out.cpu().numpy(), want) <= TOL
    _assert_pools_match(P)


@pytest.mark.parametrize("r_k,r_v,group", [(64, 64, 4), (48, 80, 2), (128, 128, 1), (16, 96, 8)])
@pytest.mark.parametrize("page_tokens", [64, 128])
def test_paged_prefill_matches_oracle_and_contiguous_cache(r_k, r_v, group, page_tokens):
    hkv, n_prev, T = 2, 150, 139
    n = n_prev + T
    P = PagedPair(("pg-pf", r_k, r_v, page_tokens), 2, hkv * group, hkv, r_k, r_v, page_tokens, 384 // page_tokens)
    P.fill(8, [n, n])
    q = synth.chunk_queries(synth.stable_seed("pg-pf", "cq"), 2, T, hkv * group, 128, "cuda")
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    B.skv_paged_prefill_attention(P.gpu, q, out, n_prev)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    assert vec_rel_err(got, O.paged_prefill_attention(P.ora, P.cache, _f64(q), n_prev)) <= TOL
    # the contiguous cache with the same rows: the same algorithm from a build of its own (the compiler may
    # fuse multiply-adds differently), so agreement is to float32 rounding, not to the bit
    L = P.contiguous_gpu([n, n])
    ref = torch.empty_like(out)
    B.skv_prefill_attention(L, q, ref, n_prev)
    torch.cuda.synchronize()
    assert vec_rel_err(got, ref.cpu().numpy()) <= 1e-5


def test_table_entries_outside_the_pool_are_clamped():
    # garbage in the table must not fault: entries are clamped into the pool, and the result is that of the
    # clamped table (every page of the pool holds numbers here, so the oracle can follow)
    P = PagedPair(("pg-clamp",), 2, 8, 2, 64, 64, 64, 4)
    P.fill(9, [200, 200])
    for pool in (P.cache.k_pool, P.cache.v_pool):
        pool[np.isnan(pool)] = 0.5
    P.upload_oracle_pools()
    bad = P.table.copy()
    bad[0, 1], bad[1, 2] = -5, 10 ** 6
    P.gpu.block_table.copy_(torch.from_numpy(bad).cuda())
    q = P.queries(10)
    out = torch.empty((2, 8, 128), dtype=torch.float32, device="cuda")
    B.skv_paged_decode_attention(P.gpu, q, out, None, 200)
    torch.cuda.synchronize()
    cache = O.OraclePagedCache(P.cache.k_pool, P.cache.v_pool, np.clip(bad, 0, P.n_pages - 1), 64)
    want = O.paged_decode_attention(P.ora, cache, _f64(q), [200, 200])
    assert vec_rel_err(out.cpu().numpy(), want) <= TOL
    assert vec_rel_err(out.cpu().numpy(), O.paged_decode_attention(P.ora, P.cache, _f64(q), [200, 200])) > TOL


def test_paged_decode_steps_in_a_hip_graph_replay_identically():
    # a serving loop replays captured steps with the lengths and the block table on the device: capture three
    # steps over a shuffled table, replay with eager work in between, compare every replay with the eager run
    lens, steps = [900, 63, 500, 1], 3
    P = PagedPair(("pg-graph",), 4, 8, 2, 64, 64, 64, 16)
    P.fill(14, lens)
    kn, vn = P.raw_kv(15, steps)
    qs = [P.queries(20 + s) for s in range(steps)]
    ws = P.gpu.workspace()
    lens_dev = [_lens_t([n + s for n in lens]) for s in range(steps)]
    eager = torch.empty((steps, 4, 8, 128), dtype=torch.float32, device="cuda")
    for s in range(steps):
        B.skv_paged_decode_step(P.gpu, kn[:, s:s + 1], vn[:, s:s + 1], lens_dev[s], max(lens) + s, qs[s], eager[s], 0.0, ws)
    torch.cuda.synchronize()
    pool_after = P.gpu.k_pool.clone()
    outs = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for s in range(steps):
                B.skv_paged_decode_step(P.gpu, kn[:, s:s + 1], vn[:, s:s + 1], lens_dev[s], max(lens) + s, qs[s], outs[s],
                                        0.0, ws)
    torch.cuda.synchronize()
    for rep in range(3):
        outs.fill_(float("nan"))
        ws.random_(0, 255)                                # eager work between replays: scribble over the workspace
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs, eager), rep
        assert torch.equal(P.gpu.k_pool.view(torch.int16), pool_after.view(torch.int16)), rep


@pytest.mark.parametrize("r_k,r_v,hq,hkv", [(64, 64, 8, 2), (48, 80, 4, 4), (32, 128, 16, 2)])
@pytest.mark.parametrize("page_tokens", [64, 128])
def test_paged_folded_variant_places_rows_exactly_and_matches_the_oracle(r_k, r_v, hq, hkv, page_tokens):
    # rows and queries arrive projected (what a model with folded weights hands over); outputs stay in rank-r_V
    # coordinates.  Placement is a copy, so the pools must match bit for bit; rows nobody wrote keep the sentinel.
    batch, lens, T = 3, [0, 70, 300], 37
    P = PagedPair(("pg-fold", r_k, r_v, page_tokens), batch, hq, hkv, r_k, r_v, page_tokens, 8)
    P.fill(9, lens)
    g = torch.Generator(device="cuda").manual_seed(7)
    k_low = torch.randn((batch, T, hkv, r_k), generator=g, device="cuda").to(torch.bfloat16)
    v_low = torch.randn((batch, T, hkv, r_v), generator=g, device="cuda").to(torch.bfloat16)
    q_low = torch.randn((batch, hq, r_k), generator=g, device="cuda").to(torch.bfloat16)
    B.skv_paged_append_projected(P.gpu, k_low, v_low, _lens_t(lens), max(lens))
    torch.cuda.synchronize()
    O.paged_append_projected(P.ora, P.cache, _f64(k_low), _f64(v_low), lens)
    gk, gv = P.pool_bits()
    for got, want in ((gk, P.cache.k_pool), (gv, P.cache.v_pool)):
        written = ~np.isnan(want)
        assert np.all(got[~written] == SENTINEL)
        rows_new = np.zeros(want.shape[:3], bool)               # the rows this call placed: exact copies
        for b in range(batch):
            for t in range(lens[b], lens[b] + T):
                rows_new[P.table[b, t // page_tokens], :, t % page_tokens] = True
        assert np.array_equal(got[rows_new], O.f64_to_bf16_bits(want[rows_new]))
    cur = [n + T for n in lens]
    out_low = torch.full((batch, hq, r_v), float("nan"), dtype=torch.float32, device="cuda")
    for seq in (cur, [5, 0, 211]):
        B.skv_paged_decode_attention_folded(P.gpu, q_low, out_low, _lens_t(seq), max(seq))
        torch.cuda.synchronize()
        want = O.paged_decode_attention_folded(P.ora, P.cache, _f64(q_low), seq)
        got = out_low.cpu().numpy()
        live = [b for b in range(batch) if seq[b] > 0]
        assert vec_rel_err(got[live], want[live]) <= TOL
        assert all(np.all(got[b] == 0.0) for b in range(batch) if seq[b] == 0)
    # a step: one more projected row per sequence, then attention over it as well
    k1 = torch.randn((batch, 1, hkv, r_k), generator=g, device="cuda").to(torch.bfloat16)
    v1 = torch.randn((batch, 1, hkv, r_v), generator=g, device="cuda").to(torch.bfloat16)
    B.skv_paged_decode_step_folded(P.gpu, k1, v1, _lens_t(cur), max(cur), q_low, out_low)
    torch.cuda.synchronize()
    O.paged_append_projected(P.ora, P.cache, _f64(k1), _f64(v1), cur)
    want = O.paged_decode_attention_folded(P.ora, P.cache, _f64(q_low), [c + 1 for c in cur])
    assert vec_rel_err(out_low.cpu().numpy(), want) <= TOL


def test_paged_folded_uniform_length_equals_the_contiguous_folded_call():
    P = PagedPair(("pg-fold-u",), 2, 8, 2, 64, 64, 64, 8)
    n = 333
    P.fill(4, [n, n])
    L = P.contiguous_gpu([n, n])
    g = torch.Generator(device="cuda").manual_seed(3)
    q_low = torch.randn((2, 8, 64), generator=g, device="cuda").to(torch.bfloat16)
    out, ref = (torch.empty((2, 8, 64), dtype=torch.float32, device="cuda") for _ in range(2))
    B.skv_paged_decode_attention_folded(P.gpu, q_low, out, None, n)
    B.skv_decode_attention_folded(L, q_low, ref, n)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
