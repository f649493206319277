"""The five benchmark workloads at full size, in the launch configuration the
benchmark uses (library-default context ranges), checked on sampled
(sequence, KV head) streams.

For a sampled stream the raw keys/values are copied to the host; the oracle
builds its own compressed cache from them and computes the outputs of that
stream's query heads.  The GPU cache (written by the GPU append) is compared
with the oracle's, and the GPU outputs with the oracle's.  Nothing the oracle
consumes comes from the library under test."""
import numpy as np
import pytest
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth
from _helpers import TOL, elem_rel_err, vec_rel_err

pytestmark = pytest.mark.gpu

CHUNK = 4096


class Stack:
    """All layers of a workload on the GPU, plus host copies of the raw inputs of sampled streams."""

    def __init__(self, wl, sample_layers, sample_streams, extra_capacity=0):
        self.wl = wl
        dev = "cuda"
        if wl.r_k:
            self.rk, self.rv = [wl.r_k] * wl.n_layers, [wl.r_v] * wl.n_layers
        else:
            self.rk, self.rv = synth.layer_rank_draw(synth.stable_seed(wl.name, "ranks"), wl.n_layers)
        self.cap = wl.n_ctx + extra_capacity
        self.layers, self.scales, self.pk_bits, self.pv_bits = [], [], [], []
        for li in range(wl.n_layers):
            _, pk = synth.orthonormal_bases(synth.stable_seed(wl.name, li, "pk"), wl.n_kv_heads, 128, self.rk[li])
            _, pv = synth.orthonormal_bases(synth.stable_seed(wl.name, li, "pv"), wl.n_kv_heads, 128, self.rv[li])
            self.pk_bits.append(synth.torch_bf16_to_bits(pk))
            self.pv_bits.append(synth.torch_bf16_to_bits(pv))
            self.layers.append(B.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, pk.to(dev), pv.to(dev), self.cap))
            self.scales.append((synth.channel_scales(synth.stable_seed(wl.name, li, "sk"), wl.n_kv_heads, 128),
                                synth.channel_scales(synth.stable_seed(wl.name, li, "sv"), wl.n_kv_heads, 128)))
        self.sample_layers = list(sample_layers)
        self.sample_streams = list(sample_streams)            # (b, kv) pairs
        self.raw = {(li, b, kv): ([], []) for li in self.sample_layers for b, kv in self.sample_streams}
        self.cur = 0
        self.ws = torch.empty(max(B.skv_decode_workspace_bytes(L) for L in self.layers),
                              dtype=torch.uint8, device=dev)

    def append(self, T, tag):
        """Appends T seeded tokens to every layer through the library; keeps the sampled raw rows."""
        wl = self.wl
        for li, L in enumerate(self.layers):
            k = synth.kv_activations(synth.stable_seed(wl.name, li, "k", tag), wl.batch, T, wl.n_kv_heads, 128,
                                     self.scales[li][0], "cuda")
            v = synth.kv_activations(synth.stable_seed(wl.name, li, "v", tag), wl.batch, T, wl.n_kv_heads, 128,
                                     self.scales[li][1], "cuda")
            B.skv_project_append(L, k, v, self.cur)
            if li in self.sample_layers:
                for b, kv in self.sample_streams:
                    self.raw[(li, b, kv)][0].append(synth.torch_bf16_to_bits(k[b, :, kv]))
                    self.raw[(li, b, kv)][1].append(synth.torch_bf16_to_bits(v[b, :, kv]))
        self.cur += T

    def fill_to(self, n):
        while self.cur < n:
            self.append(min(CHUNK, n - self.cur), ("fill", self.cur))

    def _queries(self, tag):
        wl = self.wl
        q = synth.queries(synth.stable_seed(wl.name, "q", tag), wl.batch, wl.n_q_heads * wl.n_layers, 128, "cuda")
        q = q.view(wl.batch, wl.n_layers, wl.n_q_heads, 128).transpose(0, 1).contiguous()
        out = torch.empty((wl.n_layers, wl.batch, wl.n_q_heads, 128), dtype=torch.float32, device="cuda")
        return q, out

    def step(self, tag):
        """One decode step through the fused entry point: append one seeded token per sequence, attend."""
        wl = self.wl
        q, out = self._queries(tag)
        for li, L in enumerate(self.layers):
            k = synth.kv_activations(synth.stable_seed(wl.name, li, "k", tag), wl.batch, 1, wl.n_kv_heads, 128,
                                     self.scales[li][0], "cuda")
            v = synth.kv_activations(synth.stable_seed(wl.name, li, "v", tag), wl.batch, 1, wl.n_kv_heads, 128,
                                     self.scales[li][1], "cuda")
            B.skv_decode_step(L, k, v, self.cur, q[li], out[li], 0.0, self.ws)
            if li in self.sample_layers:
                for b, kv in self.sample_streams:
                    self.raw[(li, b, kv)][0].append(synth.torch_bf16_to_bits(k[b, :, kv]))
                    self.raw[(li, b, kv)][1].append(synth.torch_bf16_to_bits(v[b, :, kv]))
        self.cur += 1
        torch.cuda.synchronize()
        return q, out

    def decode(self, tag):
        wl = self.wl
        q, out = self._queries(tag)
        for li, L in enumerate(self.layers):
            B.skv_decode_attention(L, q[li], out[li], self.cur, 0.0, self.ws)
        torch.cuda.synchronize()
        return q, out

    def check(self, q, out):
        """Oracle on every sampled stream: cache parity and output parity."""
        wl = self.wl
        G = wl.n_q_heads // wl.n_kv_heads
        n = self.cur
        worst = worst_elem = 0.0
        for li in self.sample_layers:
            for b, kv in self.sample_streams:
                kb = np.concatenate(self.raw[(li, b, kv)][0])[None, :, None, :]     # [1, n, 1, 128]
                vb = np.concatenate(self.raw[(li, b, kv)][1])[None, :, None, :]
                assert kb.shape[1] == n
                ora = O.new_layer(1, G, 1, 128, O.bf16_bits_to_f64(self.pk_bits[li][kv:kv + 1]),
                                  O.bf16_bits_to_f64(self.pv_bits[li][kv:kv + 1]), n, store="bf16")
                O.project_append(ora, O.bf16_bits_to_f64(kb), O.bf16_bits_to_f64(vb), 0)
                # cache: same bits except where float32 and float64 sums straddle a rounding boundary
                L = self.layers[li]
                gk = synth.torch_bf16_to_bits(L.k_cache[b, kv, :n])
                gv = synth.torch_bf16_to_bits(L.v_cache[b, kv, :n])
                assert (gk != O.f64_to_bf16_bits(ora.k_cache[0, 0])).mean() < 0.01
                assert (gv != O.f64_to_bf16_bits(ora.v_cache[0, 0])).mean() < 0.01
                qh = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(q[li, b, kv * G:(kv + 1) * G]))[None]
                want = O.decode_attention(ora, qh, n)[0]
                got = out[li, b, kv * G:(kv + 1) * G].cpu().numpy()
                assert np.all(np.isfinite(got))
                err = vec_rel_err(got, want)
                worst = max(worst, err)
                worst_elem = max(worst_elem, elem_rel_err(got, want))
                assert err <= TOL, (li, b, kv, err)
        return f"per vector {worst:.3e}, per element (floor 1e-3 of the vector's largest entry) {worst_elem:.3e}"


def test_b1_ctx1k_r64_append16_then_decode():
    wl = synth.WORKLOADS["b1_ctx1k_r64"]
    S = Stack(wl, [0], [(0, kv) for kv in range(wl.n_kv_heads)])
    S.fill_to(wl.n_ctx - wl.append_chunk)
    S.append(wl.append_chunk, "chunk")                       # 16 tokens: the few-token kernel
    assert S.cur == 1024
    q, out = S.decode(0)
    print("b1_ctx1k_r64 worst rel err", S.check(q, out), flush=True)


def test_b4_ctx32k_r64_consecutive_decode_steps():
    wl = synth.WORKLOADS["b4_ctx32k_r64"]
    steps = wl.decode_steps
    S = Stack(wl, [0], [(0, 0), (1, 3), (2, 5), (3, 7)])
    S.fill_to(wl.n_ctx - steps)
    for s in range(steps):                                   # each step appends one token, then attends
        q, out = S.step(("step", s))
        if s in (0, steps // 2, steps - 1):
            print(f"b4_ctx32k_r64 step {s} n_ctx {S.cur} worst rel err", S.check(q, out), flush=True)
    assert S.cur == 32768


def test_b4_ctx32k_L32_mixed_ranks_stack():
    wl = synth.WORKLOADS["b4_ctx32k_L32_mixed"]
    rk, rv = synth.layer_rank_draw(synth.stable_seed(wl.name, "ranks"), wl.n_layers)
    assert any(a != b for a, b in zip(rk, rv)) and len(set(rk)) > 2      # heterogeneous, r_K != r_V somewhere
    # sample layers that cover distinct rank pairs
    seen, pick = set(), []
    for li in range(wl.n_layers):
        if (rk[li], rv[li]) not in seen and len(pick) < 5:
            seen.add((rk[li], rv[li]))
            pick.append(li)
    S = Stack(wl, pick, [(0, 1), (3, 6)])
    S.fill_to(wl.n_ctx - 1)
    q, out = S.step("last")                                  # one decode step over all 32 layers
    assert torch.all(torch.isfinite(out))
    print("b4_ctx32k_L32_mixed layers", pick, [(rk[i], rv[i]) for i in pick], "worst rel err", S.check(q, out), flush=True)


def test_b8_chunk4k_r48_80_chunk_append_then_decode():
    wl = synth.WORKLOADS["b8_chunk4k_r48_80"]
    S = Stack(wl, [0], [(0, 0), (2, 4), (5, 1), (7, 7)])
    S.fill_to(wl.n_ctx - wl.append_chunk)
    assert S.cur == 28672
    S.append(wl.append_chunk, "chunk")                       # one 4096-token call on the matrix cores
    q, out = S.decode(0)
    print("b8_chunk4k_r48_80 worst rel err", S.check(q, out), flush=True)


def test_b8_ctx128k_mha_r64_96():
    wl = synth.WORKLOADS["b8_ctx128k_mha_r64_96"]
    S = Stack(wl, [0], [(0, 0), (3, 17), (7, 31)])
    S.fill_to(wl.n_ctx - 2)
    for s in range(2):
        q, out = S.step(("step", s))
    assert S.cur == 131072
    print("b8_ctx128k_mha_r64_96 worst rel err", S.check(q, out), flush=True)


def test_b8_chunk4k_r48_80_chunk_prefill_attention():
    """The same chunk as one step of a chunked prefill: append 4096 tokens behind 28672 cached ones and
    attend them causally (skv_prefill_step, default precision and schedule); sampled query rows of sampled
    streams against the oracle's definition form."""
    wl = synth.WORKLOADS["b8_chunk4k_r48_80"]
    T = wl.append_chunk
    S = Stack(wl, [0], [(1, 2), (6, 5)])
    S.fill_to(wl.n_ctx - T)
    L = S.layers[0]
    k = synth.kv_activations(synth.stable_seed(wl.name, 0, "k", "chunk"), wl.batch, T, wl.n_kv_heads, 128,
                             S.scales[0][0], "cuda")
    v = synth.kv_activations(synth.stable_seed(wl.name, 0, "v", "chunk"), wl.batch, T, wl.n_kv_heads, 128,
                             S.scales[0][1], "cuda")
    q = synth.chunk_queries(synth.stable_seed(wl.name, "cq"), wl.batch, T, wl.n_q_heads, 128, "cuda")
    out = torch.full((wl.batch, T, wl.n_q_heads, 128), float("nan"), dtype=torch.float32, device="cuda")
    B.skv_prefill_step(L, k, v, q, out, S.cur)
    torch.cuda.synchronize()
    assert torch.all(torch.isfinite(out))
    n_prev, G = S.cur, wl.n_q_heads // wl.n_kv_heads
    toks = [0, 1, 31, 32, 63, 64, 2047, 4064, 4095]
    worst = 0.0
    for b, kv in S.sample_streams:
        kb = np.concatenate(S.raw[(0, b, kv)][0] + [synth.torch_bf16_to_bits(k[b, :, kv])])[None, :, None, :]
        vb = np.concatenate(S.raw[(0, b, kv)][1] + [synth.torch_bf16_to_bits(v[b, :, kv])])[None, :, None, :]
        ora = O.new_layer(1, G, 1, 128, O.bf16_bits_to_f64(S.pk_bits[0][kv:kv + 1]),
                          O.bf16_bits_to_f64(S.pv_bits[0][kv:kv + 1]), n_prev + T, store="bf16")
        O.project_append(ora, O.bf16_bits_to_f64(kb), O.bf16_bits_to_f64(vb), 0)
        qh = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(q[b:b + 1, :, kv * G:(kv + 1) * G]))
        rows = [(0, t, g) for t in toks for g in range(G)]
        want = O.prefill_attention(ora, qh, n_prev, rows=rows)
        got = out[b, :, kv * G:(kv + 1) * G].cpu().numpy()
        for _, t, g in rows:
            err = float(np.max(np.abs(got[t, g] - want[0, t, g])) / np.max(np.abs(want[0, t, g])))
            worst = max(worst, err)
            assert err <= TOL, (b, kv, t, g, err)
    print("b8_chunk4k_r48_80 chunk prefill worst rel err", worst, flush=True)
