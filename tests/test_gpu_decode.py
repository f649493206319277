"""GPU parity of decode attention against the float64 oracle, element by
element, on sizes the oracle finishes in seconds.  Both sides read the same
cache bytes (written by the oracle's own append)."""
import numpy as np
import pytest
import torch

from paper_2601_21686_amd import binding as B
from _helpers import TOL, Pair, vec_rel_err

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("decode_engine")]


def _filled_pair(seed, batch, hq, hkv, r_k, r_v, n, capacity=None, **kw):
    P = Pair(seed, batch, hq, hkv, r_k, r_v, capacity or n, **kw)
    k, v = P.raw_kv(seed, n, device="cpu")
    P.oracle_append(k, v, 0)
    P.upload_oracle_cache(n)
    return P


@pytest.mark.parametrize("r_k,r_v", [(64, 64), (16, 16), (32, 48), (48, 80), (80, 32), (96, 112),
                                      (112, 96), (128, 128), (64, 96), (16, 128), (128, 16)])
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4)])
def test_decode_matches_oracle_across_ranks(r_k, r_v, hq, hkv):
    n = 1500                                        # several tiles and a ragged tail
    P = _filled_pair(("ranks", r_k, r_v, hq), 2, hq, hkv, r_k, r_v, n)
    q = P.queries(1)
    want = P.oracle_decode(q, n)
    got = P.gpu_decode(q, n)
    assert vec_rel_err(got, want) <= TOL


@pytest.mark.parametrize("group", [1, 2, 4, 8])
def test_decode_head_grouping(group):
    hkv = 2
    P = _filled_pair(("group", group), 2, hkv * group, hkv, 64, 64, 777)
    q = P.queries(2)
    assert vec_rel_err(P.gpu_decode(q, 777), P.oracle_decode(q, 777)) <= TOL


@pytest.mark.parametrize("n_ctx", [1, 2, 7, 8, 9, 31, 32, 33, 127, 128, 129, 255, 256, 257, 511, 513, 1024])
def test_decode_context_lengths_and_unread_tail(n_ctx):
    cap = 1100
    P = _filled_pair(("ctx",), 1, 8, 2, 64, 64, cap)
    # rows beyond n_ctx hold NaN: they must never influence the result
    nan = torch.full((1,), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.gpu.k_cache[:, :, n_ctx:] = nan
    P.gpu.v_cache[:, :, n_ctx:] = nan
    q = P.queries(3)
    got = P.gpu_decode(q, n_ctx)
    assert np.all(np.isfinite(got))
    assert vec_rel_err(got, P.oracle_decode(q, n_ctx)) <= TOL


@pytest.mark.parametrize("n_splits", [1, 2, 3, 5, 8, 64, 256])
def test_explicit_split_counts_including_empty_ranges(n_splits):
    n = 2000
    P = _filled_pair(("splits",), 2, 8, 2, 48, 80, n)
    q = P.queries(4)
    out = torch.empty((2, 8, 128), dtype=torch.float32, device="cuda")
    B.skv_decode_project_query(P.gpu, q, 0.0)
    B.skv_decode_partial(P.gpu, n, n_splits)
    B.skv_decode_combine(P.gpu, out, n_splits)
    torch.cuda.synchronize()
    assert vec_rel_err(out.cpu().numpy(), P.oracle_decode(q, n)) <= TOL


def test_shared_key_basis_and_custom_scale():
    n = 900
    P = _filled_pair(("shared",), 2, 8, 4, 64, 96, n, shared_k=True)
    assert P.gpu.c.p_k_head_stride == 0
    q = P.queries(5)
    for scale in (0.0, 0.05, 0.3):
        want = P.oracle_decode(q, n, scale if scale > 0 else None)
        assert vec_rel_err(P.gpu_decode(q, n, scale), want) <= TOL


def test_peaked_softmax_with_large_scores():
    # one key aligned with the query: the softmax is dominated by a single row
    n = 1200
    P = _filled_pair(("peaked",), 1, 4, 1, 64, 64, n)
    q = P.queries(6)
    want = P.oracle_decode(q, n, 4.0)
    got = P.gpu_decode(q, n, 4.0)
    assert vec_rel_err(got, want) <= TOL


@pytest.mark.parametrize("r_k,r_v,hq,hkv", [(64, 64, 8, 2), (48, 80, 8, 2), (128, 32, 4, 4), (32, 128, 16, 2)])
def test_softmax_reference_moves_tile_after_tile(r_k, r_v, hq, hkv):
    # Both range kernels keep a softmax reference that moves only when a score exceeds it by a margin, and
    # rescale their accumulators then.  Keys that grow with their position (a ramp of 1 .. 9 over the context)
    # under a scale 7 and 70 times the default make the largest score of many a tile exceed the previous
    # reference by more than the margin (scores up to +-90 and +-900), in every context range.
    from oracle import skv_oracle as O
    n = 2900
    P = _filled_pair(("ramp", r_k, r_v, hq), 2, hq, hkv, r_k, r_v, n)
    ramp = 1.0 + 8.0 * np.arange(n, dtype=np.float64) / n
    P.ora.k_cache[:, :, :n] = O.bf16_bits_to_f64(O.f64_to_bf16_bits(P.ora.k_cache[:, :, :n] * ramp[None, None, :, None]))
    P.upload_oracle_cache(n)
    q = P.queries(8)
    for scale in (0.6, 6.0):
        for n_ctx in (n, 777):
            got = P.gpu_decode(q, n_ctx, scale)
            assert np.all(np.isfinite(got))
            assert vec_rel_err(got, P.oracle_decode(q, n_ctx, scale)) <= TOL, (scale, n_ctx)


def test_decode_is_deterministic_and_stage_calls_equal_the_fused_call():
    n = 3000
    P = _filled_pair(("det",), 2, 8, 2, 64, 64, n)
    q = P.queries(7)
    a = P.gpu_decode(q, n)
    b = P.gpu_decode(q, n)
    assert np.array_equal(a, b)
    s = B.skv_decode_default_splits(P.gpu, n)
    out = torch.empty((2, 8, 128), dtype=torch.float32, device="cuda")
    B.skv_decode_project_query(P.gpu, q, 0.0)
    B.skv_decode_partial(P.gpu, n, s)
    B.skv_decode_combine(P.gpu, out, s)
    torch.cuda.synchronize()
    staged = out.cpu().numpy()
    assert np.array_equal(staged, a)
    # the range kernel that projects the queries itself gives the same bits as the staged projection
    B.skv_decode_partial_q(P.gpu, q, n, s)
    B.skv_decode_combine(P.gpu, out, s)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), staged)
    # a different split of the context gives the same result up to float32 rounding
    for s2 in (1, 7):
        B.skv_decode_partial(P.gpu, n, s2)
        B.skv_decode_combine(P.gpu, out, s2)
        torch.cuda.synchronize()
        assert vec_rel_err(out.cpu().numpy(), a) < 1e-5


def test_errors_leave_output_untouched():
    P = _filled_pair(("err",), 1, 4, 1, 64, 64, 64)
    q = P.queries(8)
    out = torch.full((1, 4, 128), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(B.SkvError) as e:
        B.skv_decode_attention(P.gpu, q, out, 65)
    assert e.value.code == B.SKV_ERR_CAPACITY
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.SkvError) as e:
        B.skv_decode_attention(P.gpu, q, out, 64, 0.0, small)
    assert e.value.code == B.SKV_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)


@pytest.mark.parametrize("batch,T,hq,hkv,r_k,r_v", [(4, 1, 8, 2, 64, 64), (2, 3, 4, 4, 48, 80), (1, 1, 16, 2, 32, 96),
                                                    (3, 40, 8, 2, 64, 64), (2, 4, 8, 4, 128, 16), (2, 5, 8, 4, 16, 128),
                                                    (1, 2, 8, 8, 96, 112)])
def test_decode_step_equals_append_then_decode(batch, T, hq, hkv, r_k, r_v):
    # the fused step against the two separate calls: the cache bit for bit, the outputs up to the order
    # in which context ranges are merged (the step attends its new rows as a range of their own), and
    # against the oracle
    n0 = 700
    Pa = Pair(("step", batch, T, r_k), batch, hq, hkv, r_k, r_v, n0 + T)
    Pb = Pair(("step", batch, T, r_k), batch, hq, hkv, r_k, r_v, n0 + T, oracle=False)
    k0, v0 = Pa.raw_kv(1, n0)
    for P in (Pa, Pb):
        B.skv_project_append(P.gpu, k0, v0, 0)
    Pa.oracle_append(k0.cpu(), v0.cpu(), 0)
    k1, v1 = Pa.raw_kv(2, T)
    q = Pa.queries(3)
    out_a = torch.empty((batch, hq, 128), dtype=torch.float32, device="cuda")
    B.skv_decode_step(Pa.gpu, k1, v1, n0, q, out_a)
    B.skv_project_append(Pb.gpu, k1, v1, n0)
    out_b = Pb.gpu_decode(q, n0 + T)
    torch.cuda.synchronize()
    assert torch.equal(Pa.gpu.k_cache, Pb.gpu.k_cache) and torch.equal(Pa.gpu.v_cache, Pb.gpu.v_cache)
    assert vec_rel_err(out_a.cpu().numpy(), out_b) <= 1e-5
    Pa.oracle_append(k1.cpu(), v1.cpu(), n0)
    want = Pa.oracle_decode(q, n0 + T)
    assert vec_rel_err(out_b, want) <= TOL
    assert vec_rel_err(out_a.cpu().numpy(), want) <= TOL


@pytest.mark.parametrize("r_k,r_v,hq,hkv", [(64, 64, 8, 2), (48, 80, 4, 4), (128, 32, 16, 2)])
def test_folded_variant_matches_oracle(r_k, r_v, hq, hkv):
    from oracle import skv_oracle as O
    from paper_2601_21686_amd import synth
    batch, n0, T = 2, 1000, 37
    n = n0 + T
    P = _filled_pair(("fold", r_k, r_v), batch, hq, hkv, r_k, r_v, n0, capacity=n)
    # what a model with folded weights hands over: projected rows (bf16) and projected queries (bf16)
    g = torch.Generator(device="cuda").manual_seed(5)
    k_low = torch.randn((batch, T, hkv, r_k), generator=g, device="cuda").to(torch.bfloat16)
    v_low = torch.randn((batch, T, hkv, r_v), generator=g, device="cuda").to(torch.bfloat16)
    q_low = torch.randn((batch, hq, r_k), generator=g, device="cuda").to(torch.bfloat16)
    f64 = lambda t: O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))
    B.skv_append_projected(P.gpu, k_low, v_low, n0)
    O.append_projected(P.ora, f64(k_low), f64(v_low), n0)
    torch.cuda.synchronize()
    # placement and values are bit-exact copies
    assert np.array_equal(f64(P.gpu.k_cache[:, :, :n]), P.ora.k_cache[:, :, :n])
    assert np.array_equal(f64(P.gpu.v_cache[:, :, :n]), P.ora.v_cache[:, :, :n])
    out_low = torch.empty((batch, hq, r_v), dtype=torch.float32, device="cuda")
    for n_ctx in (n, 130):
        B.skv_decode_attention_folded(P.gpu, q_low, out_low, n_ctx)
        torch.cuda.synchronize()
        want = O.decode_attention_folded(P.ora, f64(q_low), n_ctx)
        assert vec_rel_err(out_low.cpu().numpy(), want) <= TOL
    # one decode step: the same rows placed again one row earlier, then attention over n tokens
    k1, v1 = k_low[:, -1:].contiguous(), v_low[:, -1:].contiguous()
    out_step = torch.full_like(out_low, float("nan"))
    B.skv_decode_step_folded(P.gpu, k1, v1, n - 1, q_low, out_step)
    B.skv_decode_attention_folded(P.gpu, q_low, out_low, n)
    torch.cuda.synchronize()
    assert torch.equal(out_step, out_low)


def test_alternating_calls_on_one_workspace_are_bit_stable():
    # Two different query sets alternate on ONE workspace: the merge order is fixed, so every call must
    # reproduce the bits of the first call of its kind, and nothing of the other set's partial results
    # may leak into it.
    n = 6000
    P = _filled_pair(("stale",), 4, 32, 8, 64, 64, n)
    qa, qb = P.queries(21), P.queries(22)
    ref = {}
    for name, q in (("a", qa), ("b", qb)):
        s = B.skv_decode_default_splits(P.gpu, n)
        out = torch.empty((4, 32, 128), dtype=torch.float32, device="cuda")
        B.skv_decode_partial_q(P.gpu, q, n, s)
        B.skv_decode_combine(P.gpu, out, s)
        torch.cuda.synchronize()
        ref[name] = out.cpu().numpy()
    outs = torch.full((400, 4, 32, 128), float("nan"), dtype=torch.float32, device="cuda")
    for i in range(400):
        B.skv_decode_attention(P.gpu, qa if i % 2 == 0 else qb, outs[i], n)
    torch.cuda.synchronize()
    got = outs.cpu().numpy()
    assert np.all(np.isfinite(got))
    for i in range(400):
        name = "a" if i % 2 == 0 else "b"
        assert np.array_equal(got[i], got[i % 2]), i                     # same bits as the first call of its kind
        assert np.array_equal(got[i], ref[name]), i                       # which are the bits of the two-launch path


@pytest.mark.parametrize("batch,hq,hkv,r_k,r_v,n", [(4, 32, 8, 64, 64, 5000), (1, 8, 8, 48, 80, 700), (2, 8, 4, 128, 32, 1300),
                                                    (3, 16, 2, 32, 96, 2100), (2, 4, 4, 16, 16, 64), (1, 32, 8, 96, 128, 9000)])
def test_attention_ignores_what_the_workspace_held(batch, hq, hkv, r_k, r_v, n):
    """The workspace's contents on entry are irrelevant by contract: random bytes, all ones and the leftovers of
    other calls must all give the bits of the stage calls (range stage, then the merge launch)."""
    P = _filled_pair(("scribble", r_k, r_v, n), batch, hq, hkv, r_k, r_v, n)
    q = P.queries(5)
    ws = P.gpu.workspace()
    s = B.skv_decode_default_splits(P.gpu, n)
    ref = torch.empty((batch, hq, 128), dtype=torch.float32, device="cuda")
    B.skv_decode_partial_q(P.gpu, q, n, s)
    B.skv_decode_combine(P.gpu, ref, s)
    outs = torch.full((24, batch, hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    for i in range(24):
        if i % 3 == 0:
            ws.random_(0, 256)
        elif i % 3 == 1:
            ws.fill_(255)
        B.skv_decode_attention(P.gpu, q, outs[i], n)                      # i % 3 == 2: the previous call's leftovers
    torch.cuda.synchronize()
    for i in range(24):
        assert torch.equal(outs[i], ref), i
    assert vec_rel_err(ref.cpu().numpy(), P.oracle_decode(q, n)) <= TOL


def test_decode_steps_captured_in_a_hip_graph_replay_identically():
    # The benchmark replays a captured graph of decode steps.  Capture three steps, replay the graph
    # several times with eager work and synchronisations in between, and compare every replay with the
    # eager result: the launches record no memset nodes and keep no state between calls.
    n0, steps = 900, 3
    P = Pair(("graph",), 2, 8, 2, 64, 64, n0 + steps)
    k0, v0 = P.raw_kv(1, n0)
    B.skv_project_append(P.gpu, k0, v0, 0)
    kn, vn = P.raw_kv(2, steps)
    qs = [P.queries(10 + s) for s in range(steps)]
    ws = P.gpu.workspace()
    eager = torch.empty((steps, 2, 8, 128), dtype=torch.float32, device="cuda")
    for s in range(steps):
        B.skv_decode_step(P.gpu, kn[:, s:s + 1], vn[:, s:s + 1], n0 + s, qs[s], eager[s], 0.0, ws)
    torch.cuda.synchronize()
    cache_after = P.gpu.k_cache.clone()
    outs = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for s in range(steps):
                B.skv_decode_step(P.gpu, kn[:, s:s + 1], vn[:, s:s + 1], n0 + s, qs[s], outs[s], 0.0, ws)
    torch.cuda.synchronize()
    for rep in range(4):
        outs.fill_(float("nan"))
        P.gpu.k_cache[:, :, n0:] = 0                      # eager work between replays: wipe the appended rows
        ws.random_(0, 255)                                # and scribble over the workspace
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs, eager), rep
        assert torch.equal(P.gpu.k_cache.view(torch.int16), cache_after.view(torch.int16)), rep


@pytest.mark.parametrize("r_k,r_v,hq,hkv", [(64, 64, 8, 2), (48, 80, 4, 4), (32, 128, 16, 2)])
def test_kind_of_cache_load_does_not_change_a_bit(r_k, r_v, hq, hkv):
    """Streaming and ordinary loads fetch the same bytes: outputs agree bit for bit, per engine."""
    n = 2100
    P = _filled_pair(("loads", r_k, r_v), 2, hq, hkv, r_k, r_v, n)
    q = P.queries(3)
    engine = P.gpu.c.flags & (B.SKV_ENGINE_VECTOR | B.SKV_ENGINE_MATRIX)
    P.gpu.c.flags = engine | B.SKV_READS_CACHED
    plain = P.gpu_decode(q, n)
    P.gpu.c.flags = engine | B.SKV_READS_STREAMING
    streamed = P.gpu_decode(q, n)
    assert np.array_equal(plain, streamed)
    assert vec_rel_err(plain, P.oracle_decode(q, n)) <= TOL


@pytest.mark.parametrize("r,tile_rows", [(16, 256), (64, 64), (128, 32)])
@pytest.mark.parametrize("tiles", [1, 2, 3, 4, 7, 23, 24, 25, 31])
@pytest.mark.parametrize("extra", [0, 1, -1])
def test_ranges_around_the_early_request_depth(r, tile_rows, tiles, extra):
    """The range kernel that projects its queries itself requests tiles before the projection: one for a range
    of one or two whole tiles, two from three tiles on, six from twenty-four on.  Ranges of just below, at and
    above those lengths, with and without a ragged tail, in one range and in three."""
    n = tile_rows * tiles + (extra if extra >= 0 else tile_rows - 1)
    P = _filled_pair(("early", r), 1, 4, 1, r, r, 3 * n)
    q = P.queries(5)
    for n_splits, n_ctx in ((1, n), (3, 3 * n)):
        out = torch.empty((1, 4, 128), dtype=torch.float32, device="cuda")
        B.skv_decode_partial_q(P.gpu, q, n_ctx, n_splits)
        B.skv_decode_combine(P.gpu, out, n_splits)
        torch.cuda.synchronize()
        assert vec_rel_err(out.cpu().numpy(), P.oracle_decode(q, n_ctx)) <= TOL


STACK_RANKS = [(64, 64), (32, 96), (48, 80), (128, 16)]


def _stack(tag, batch, hq, hkv, n0, extra, oracle):
    pairs = [Pair((tag, l, rk, rv), batch, hq, hkv, rk, rv, n0 + extra, oracle=oracle) for l, (rk, rv) in enumerate(STACK_RANKS)]
    for l, P in enumerate(pairs):
        k0, v0 = P.raw_kv(("fill", l), n0)
        B.skv_project_append(P.gpu, k0, v0, 0)
        if oracle:
            P.oracle_append(k0.cpu(), v0.cpu(), 0)
    return pairs


@pytest.mark.gpu
def test_layer_stack_calls_equal_the_loop_of_single_layer_calls():
    # Sec. 3.3: ranks differ per layer.  skv_decode_attention_layers / skv_decode_step_layers over four layers
    # of different ranks: bit-identical to the loop of single-layer calls (outputs and caches), one shared
    # workspace, and against the oracle layer by layer.
    batch, hq, hkv, n0, T = 2, 8, 2, 700, 1
    a = _stack("stack", batch, hq, hkv, n0, T, oracle=True)
    b = _stack("stack", batch, hq, hkv, n0, T, oracle=False)
    stack = B.LayerStack([P.gpu for P in a])
    qs = [P.queries(("q", l)) for l, P in enumerate(a)]
    new = lambda: [torch.full((batch, hq, 128), float("nan"), dtype=torch.float32, device="cuda") for _ in a]
    # attention over the cached rows
    out_stack, out_loop = new(), new()
    B.skv_decode_attention_layers(stack, qs, out_stack, n0)
    for l, P in enumerate(b):
        B.skv_decode_attention(P.gpu, qs[l], out_loop[l], n0)
    torch.cuda.synchronize()
    for l, P in enumerate(a):
        assert torch.equal(out_stack[l], out_loop[l]), l
        assert vec_rel_err(out_stack[l].cpu().numpy(), P.oracle_decode(qs[l], n0)) <= TOL, l
    # one whole step: append a token per layer, attend n0 + 1 rows
    kv = [P.raw_kv(("new", l), T) for l, P in enumerate(a)]
    out_stack, out_loop = new(), new()
    B.skv_decode_step_layers(stack, [k for k, _ in kv], [v for _, v in kv], n0, qs, out_stack)
    for l, P in enumerate(b):
        B.skv_decode_step(P.gpu, kv[l][0], kv[l][1], n0, qs[l], out_loop[l])
    torch.cuda.synchronize()
    for l, P in enumerate(a):
        assert torch.equal(out_stack[l], out_loop[l]), l
        assert torch.equal(P.gpu.k_cache, b[l].gpu.k_cache) and torch.equal(P.gpu.v_cache, b[l].gpu.v_cache), l
        P.oracle_append(kv[l][0].cpu(), kv[l][1].cpu(), n0)
        assert vec_rel_err(out_stack[l].cpu().numpy(), P.oracle_decode(qs[l], n0 + T)) <= TOL, l


@pytest.mark.gpu
def test_layer_stack_step_without_new_tokens_is_the_attention_call():
    batch, hq, hkv, n0 = 2, 8, 2, 450
    a = _stack("stack-t0", batch, hq, hkv, n0, 0, oracle=False)
    stack = B.LayerStack([P.gpu for P in a])
    qs = [P.queries(("q", l)) for l, P in enumerate(a)]
    new = lambda: [torch.full((batch, hq, 128), float("nan"), dtype=torch.float32, device="cuda") for _ in a]
    none = [torch.empty((batch, 0, hkv, 128), dtype=torch.bfloat16, device="cuda") for _ in a]
    out_step, out_att = new(), new()
    B.skv_decode_step_layers(stack, none, none, n0, qs, out_step)
    B.skv_decode_attention_layers(stack, qs, out_att, n0)
    torch.cuda.synchronize()
    for l in range(len(a)):
        assert torch.equal(out_step[l], out_att[l]), l


@pytest.mark.gpu
def test_layer_stack_call_with_a_bad_last_layer_launches_nothing():
    batch, hq, hkv, n0 = 2, 8, 2, 300
    a = _stack("stack-bad", batch, hq, hkv, n0, 1, oracle=False)
    stack = B.LayerStack([P.gpu for P in a])
    stack.c[len(a) - 1].r_k = 72                       # not a rank the library is built for
    qs = [P.queries(("q", l)) for l, P in enumerate(a)]
    outs = [torch.full((batch, hq, 128), 7.0, dtype=torch.float32, device="cuda") for _ in a]
    caches = [P.gpu.k_cache.clone() for P in a]
    kv = [P.raw_kv(("new", l), 1) for l, P in enumerate(a)]
    with pytest.raises(B.SkvError) as e:
        B.skv_decode_attention_layers(stack, qs, outs, n0)
    assert e.value.code == B.SKV_ERR_RANK
    with pytest.raises(B.SkvError) as e:
        B.skv_decode_step_layers(stack, [k for k, _ in kv], [v for _, v in kv], n0, qs, outs)
    assert e.value.code == B.SKV_ERR_RANK
    torch.cuda.synchronize()
    for l, P in enumerate(a):
        assert bool((outs[l] == 7.0).all()), l
        assert torch.equal(P.gpu.k_cache, caches[l]), l
