#!/usr/bin/env python3
"""Benchmark of the compressed-KV decode path on one MI355X.

One "step" is one pass of the whole hot path for one new token per sequence:
project the new key/value onto P_K / P_V and append them to the bf16 compressed
cache, then decode attention over the whole cache (query projection, scores,
online softmax, value mix, split merge, lift) -- one skv_decode_step call.  Every layer of the workload is
visited once per step.  Inputs are seeded and synthetic and already resident in
HBM when the clock starts.

Prints ONE JSON line.  `value` is algorithmic compressed-cache bytes per second
for the whole step (GB/s); tokens/s is reported beside it.  `roofline` is the
decode range kernel alone, timed with events on the launch stream; its
`hbm_only` object (and `value_hbm_only`) repeat the launch and the step rotated
over enough distinct copies of the layer's cache that no row is found in a cache
again -- the rate a model whose layers together exceed the last-level cache sees.
`cpu_baseline` is the float64 oracle timed on the host for one decode step of
the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
METRIC = "compressed-KV decode attention: achieved HBM GB/s + tokens/s at b4/32K"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="b4_ctx32k_r64")
    ap.add_argument("--splits", type=int, default=0, help="context ranges for the roofline leg (0 = library default)")
    ap.add_argument("--no-graph", action="store_true", help="launch step by step instead of replaying a captured graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hbm-only", action="store_true",
                    help="skip the leg that rotates over enough copies of a one-layer cache that no row is found in a cache again")
    ap.add_argument("--kernel-iters", type=int, default=200, help="launches of the decode range kernel for the roofline leg")
    ap.add_argument("--cache", choices=("bf16", "q8", "q4", "paged", "paged_q8", "paged_q4"), default="bf16",
                    help="bf16: the benchmarked configuration; q8 / q4: the 8- or 4-bit quantised compressed cache "
                         "(keys with static per-head group ranges, values with per-token group ranges); "
                         "paged: bf16 rows in a pool of pages behind a shuffled block table; paged_q8 / paged_q4: integer codes in such pages")
    ap.add_argument("--page-tokens", type=int, default=64, help="--cache paged: rows per page (a power of two >= 64)")
    ap.add_argument("--variant", choices=("explicit", "folded"), default="explicit",
                    help="explicit: the benchmarked configuration (the library projects keys, values and queries); "
                         "folded: the bases are folded into the model's linear layers (Sec. 3.4), so rows and queries "
                         "arrive projected and the output stays in rank-r_V coordinates")
    ap.add_argument("--prefill-sched", choices=("default", "together", "ahead"), default="default",
                    help="--mode prefill: force one of the kernel's two schedules")
    ap.add_argument("--prefill-chunk", type=int, default=0, help="--mode prefill: tokens in the chunk (0 = the workload's append chunk)")
    ap.add_argument("--prefill-prev", type=int, default=-1, help="--mode prefill: cached tokens before the chunk (-1 = n_ctx - chunk)")
    ap.add_argument("--ranks", default="", help="--mode prefill/append: override the workload's ranks, as r_k,r_v")
    ap.add_argument("--lengths", default="1.0,0.5,0.25,0.03125",
                    help="--mode varlen: per-sequence context lengths as fractions of the workload's context, cycled over the batch")
    ap.add_argument("--engine", choices=("auto", "vector", "matrix"), default="auto",
                    help="range kernel: chosen by shape (default: matrix cores for groups of 8 query heads, vector "
                         "arithmetic otherwise), or forced")
    ap.add_argument("--cache-reads", choices=("auto", "size", "stream", "plain"), default="auto",
                    help="how the range kernels load cache rows: streaming loads, ordinary loads, size = the library's "
                         "default (streaming when one launch covers clearly more than the 256 MiB last-level cache); "
                         "auto = what a caller that knows its model does: streaming when the layers of one step "
                         "together exceed that cache, else the library's default")
    ap.add_argument("--mode", choices=("bench", "kernel", "copy", "read", "append", "prefill", "varlen"), default="bench",
                    help="bench: the full run; kernel: only the decode range kernel launches (for counter runs); "
                         "copy: a plain 1 GiB device copy, to calibrate the HBM byte counters; "
                         "append: the chunk append of the workload (projection on the matrix cores) alone; "
                         "prefill: causal attention of the workload's chunk over the compressed cache (matrix cores) alone; "
                         "varlen: decode steps over a batch whose sequences have different context lengths")
    return ap.parse_args()


def read_traffic(workload: str, cache: str = "bf16"):
    """(HBM bytes per launch of the decode range kernel, the file they come from): the counter runs
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) are made apart from this program, which only reads their
    committed summary; (None, None) when there is none for the workload."""
    tag = "" if cache == "bf16" else f"_{cache}"
    rel = os.path.join("profiles", f"decode_partial{tag}_{workload}_traffic.txt")
    value = _read_traffic_file(os.path.join(ROOT, rel))
    return (value, rel) if value is not None else (None, None)


def _read_traffic_file(path: str):
    if not os.path.exists(path):
        return None
    vals = {}
    with open(path) as f:
        for line in f:
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                vals[k.strip()] = v.strip()
    try:
        return float(vals["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus {args.gpus} is not supported. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2601_21686_amd import binding as B
    from paper_2601_21686_amd import synth

    if not os.path.exists(B.LIB_PATH):
        from paper_2601_21686_amd import build
        build.build(verbose=False)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    # Engine and load kind travel in the flags word of every layer built below (binding.DEFAULT_LAYER_FLAGS is a
    # Python-side default for new layer objects; the library keeps no state).
    engine_flag = {"vector": B.SKV_ENGINE_VECTOR, "matrix": B.SKV_ENGINE_MATRIX, "auto": B.SKV_ENGINE_BY_SHAPE}[args.engine]
    reads_flag = {"stream": B.SKV_READS_STREAMING, "plain": B.SKV_READS_CACHED, "size": B.SKV_READS_BY_SIZE,
                  "auto": B.SKV_READS_BY_SIZE}[args.cache_reads]
    B.DEFAULT_LAYER_FLAGS = engine_flag | reads_flag
    STREAM_ABOVE = 288 << 20                          # the library's by-size rule, for the plain-read yardstick
    if args.mode == "read":
        # what a kernel that only reads gets from this memory system, by working-set size: the yardstick beside
        # the published peak (sizes up to the 256 MiB last-level cache are partly served from it when re-read)
        sink = torch.zeros(65536, dtype=torch.float32, device=dev)
        rows = []
        for mib in (64, 128, 256, 512, 1024, 2048, 4096, 8192):
            src = torch.empty(mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
            best = None
            streaming = args.cache_reads == "stream" or (args.cache_reads in ("auto", "size") and (mib << 20) > STREAM_ABOVE)
            for wgs in (512, 2048):
                for _ in range(3):
                    n = B.skv_probe_stream_read(src, wgs, sink, streaming)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(20):
                    B.skv_probe_stream_read(src, wgs, sink, streaming)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 20
                if best is None or us < best[0]:
                    best = (us, wgs, n)
            rows.append({"MiB": mib, "loads": "streaming" if streaming else "ordinary", "us_per_launch": round(best[0], 2), "workgroups": best[1],
                         "GBps": round(best[2] / best[0] / 1e3, 1), "frac_of_hbm_peak": round(best[2] / best[0] / 1e3 / HBM_PEAK_GBPS, 4)})
            del src
        print(json.dumps({"mode": "read", "kernel": "stream_read_kernel", "launches_per_size": 46, "sizes": rows}))
        return
    if args.mode == "copy":
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "copy", "bytes_read_per_launch": 1 << 30, "bytes_written_per_launch": 1 << 30,
                          "launches": 5}))
        return

    wl = synth.WORKLOADS[args.workload]
    if args.mode == "append":
        # the chunk append alone: T = the workload's chunk, written at the end of a cache holding n_ctx - T rows
        T = max(wl.append_chunk, 256)
        rk, rv = (wl.r_k or 64), (wl.r_v or 64)
        if args.ranks:
            rk, rv = (int(x) for x in args.ranks.split(","))
        abits = {"bf16": 0, "q8": 8, "q4": 4}[args.cache]
        _, pk = synth.orthonormal_bases(synth.stable_seed(wl.name, 0, "pk"), wl.n_kv_heads, wl.head_dim, rk)
        _, pv = synth.orthonormal_bases(synth.stable_seed(wl.name, 0, "pv"), wl.n_kv_heads, wl.head_dim, rv)
        if abits:
            ngk = (rk + 63) // 64
            ksc = torch.full((wl.n_kv_heads, ngk), 8.0 / (2 ** abits - 1))          # keys in [-4, 4): a plausible static range
            kzr = torch.full((wl.n_kv_heads, ngk), -4.0)
            L = B.QuantLayer(wl.batch, wl.n_q_heads, wl.n_kv_heads, pk.to(dev), pv.to(dev), ksc, kzr, wl.n_ctx, abits)
            append = B.skv_q8_project_append if abits == 8 else B.skv_q4_project_append
        else:
            L = B.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, pk.to(dev), pv.to(dev), wl.n_ctx)
            append = B.skv_project_append
        sc = synth.channel_scales(synth.stable_seed(wl.name, 0, "sk"), wl.n_kv_heads, wl.head_dim)
        k = synth.kv_activations(1, wl.batch, T, wl.n_kv_heads, wl.head_dim, sc, dev)
        v = synth.kv_activations(2, wl.batch, T, wl.n_kv_heads, wl.head_dim, sc, dev)
        for _ in range(5):
            append(L, k, v, wl.n_ctx - T)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = max(1, args.kernel_iters)            # enqueued back to back: the queue never runs dry
        e0.record()
        for _ in range(iters):
            append(L, k, v, wl.n_ctx - T)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        # yardstick: a plain kernel that reads two bytes per byte written, sized to this append's input
        in_bytes = wl.batch * T * wl.n_kv_heads * wl.head_dim * 2
        pa = torch.empty(in_bytes // 4, dtype=torch.int32, device=dev).fill_(1)
        pb, pc = pa.clone(), torch.empty_like(pa)
        mix_each = 0
        for _ in range(5):
            mix_each = B.skv_probe_stream_mix(pa, pb, pc, 2048)
        e0.record()
        for _ in range(iters):
            B.skv_probe_stream_mix(pa, pb, pc, 2048)
        e1.record()
        torch.cuda.synchronize()
        mix_us = e0.elapsed_time(e1) * 1e3 / iters
        mix_gbps = 3 * mix_each / mix_us / 1e3
        out_row = (rk + rv) * 2 if not abits else (rk + rv) * abits // 8 + 4 * ((rv + 63) // 64)
        nbytes = wl.batch * T * wl.n_kv_heads * (2 * wl.head_dim * 2 + out_row)
        flops = 2 * wl.batch * T * wl.n_kv_heads * wl.head_dim * (rk + rv)
        print(json.dumps({"mode": "append", "workload": wl.name, "batch": wl.batch, "T": T, "r_k": rk, "r_v": rv, "cache": args.cache,
                          "us_per_launch": round(us, 2), "bytes_per_launch": nbytes, "flops_per_launch": flops,
                          "achieved_GBps": round(nbytes / us / 1e3, 1), "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4),
                          "achieved_TFLOPs": round(flops / us / 1e6, 1), "frac_of_bf16_mfma_peak": round(flops / us / 1e6 / 2500.0, 4),
                          "plain_mix": {"kernel": "stream_mix_kernel", "bytes": 3 * mix_each, "us_per_launch": round(mix_us, 2),
                                        "GBps": round(mix_gbps, 1), "append_vs_plain_mix": round(nbytes / us / 1e3 / mix_gbps, 4)},
                          "launches": iters + 5}))
        return
    if args.mode == "varlen":
        # decode steps (append one token per sequence at its own position, attend its own context) over a batch
        # of mixed lengths; bytes counted are the rows each sequence really attends
        Bt, HQ, HKV, d = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
        rk, rv = (wl.r_k or 64), (wl.r_v or 64)
        fr = [float(x) for x in args.lengths.split(",")]
        lens0 = [max(1, int(wl.n_ctx * fr[b % len(fr)])) - 1 for b in range(Bt)]
        K = args.steps
        cap = wl.n_ctx + K + 8
        _, pk = synth.orthonormal_bases(synth.stable_seed(wl.name, 0, "pk"), HKV, d, rk)
        _, pv = synth.orthonormal_bases(synth.stable_seed(wl.name, 0, "pv"), HKV, d, rv)
        L = B.Layer(Bt, HQ, HKV, pk.to(dev), pv.to(dev), cap)
        sck = synth.channel_scales(synth.stable_seed(wl.name, 0, "sk"), HKV, d)
        for c0 in range(0, max(lens0), 4096):                       # every sequence filled up to the longest one
            t = min(4096, max(lens0) - c0)
            k = synth.kv_activations(synth.stable_seed(wl.name, 0, "k", c0), Bt, t, HKV, d, sck, dev)
            B.skv_project_append(L, k, k, c0)
        nk = synth.kv_activations(1, Bt, K + 4, HKV, d, sck, dev)
        q = synth.queries(2, Bt, HQ, d, dev)
        out = torch.empty((Bt, HQ, d), dtype=torch.float32, device=dev)
        lens = torch.tensor(lens0, dtype=torch.int32, device=dev)
        lens_steps = torch.stack([lens + s for s in range(K + 4)]).contiguous()   # the caller advances the lengths
        for s in range(4):
            B.skv_decode_step_varlen(L, nk[:, s:s + 1], nk[:, s:s + 1], lens_steps[s], max(lens0) + s, q, out)
        torch.cuda.synchronize()
        def steps():
            for s in range(4, K + 4):
                B.skv_decode_step_varlen(L, nk[:, s:s + 1], nk[:, s:s + 1], lens_steps[s], max(lens0) + s, q, out)
        use_graph = not args.no_graph
        if use_graph:                                               # as the main benchmark: the K steps as one graph
            side = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    steps()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        if use_graph:
            g.replay()
        else:
            steps()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / K
        nbytes = sum(HKV * (n + K // 2 + 5) * (rk + rv) * 2 for n in lens0)
        print(json.dumps({"mode": "varlen", "workload": wl.name, "batch": Bt, "context_lengths": [n + 1 for n in lens0],
                          "r_k": rk, "r_v": rv, "steps": K, "us_per_step": round(us, 2),
                          "cache_bytes_per_step": nbytes, "achieved_GBps": round(nbytes / us / 1e3, 1),
                          "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4),
                          "tokens_per_s": round(Bt / (us * 1e-6), 1),
                          "launch": "hip graph replay" if use_graph else "per-call launches"}))
        return
    if args.mode == "prefill":
        # attention of a chunk of T new tokens over n_prev cached ones (rows of the chunk already appended)
        T = args.prefill_chunk or max(wl.append_chunk, 256)
        n_prev = args.prefill_prev if args.prefill_prev >= 0 else wl.n_ctx - T
        rk, rv = (wl.r_k or 64), (wl.r_v or 64)
        if args.ranks:
            rk, rv = (int(x) for x in args.ranks.split(","))
        Bt, HQ, HKV, d = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
        _, pk = synth.orthonormal_bases(synth.stable_seed(wl.name, 0, "pk"), HKV, d, rk)
        _, pv = synth.orthonormal_bases(synth.stable_seed(wl.name, 0, "pv"), HKV, d, rv)
        if args.cache == "paged":
            pt = args.page_tokens
            per_seq = (n_prev + T + pt - 1) // pt
            order = np.random.default_rng(synth.stable_seed(wl.name, "pages")).permutation(Bt * per_seq + 16)
            table = torch.from_numpy(order[:Bt * per_seq].reshape(Bt, per_seq).astype(np.int32)).to(dev)
            L = B.PagedLayer(Bt, HQ, HKV, pk.to(dev), pv.to(dev), pt, Bt * per_seq + 16, table)
            append = lambda k_, v_, c_: B.skv_paged_project_append(L, k_, v_, None, c_)
            attend = lambda: B.skv_paged_prefill_attention(L, q, out, n_prev, 0.0, pmode)
        else:
            L = B.Layer(Bt, HQ, HKV, pk.to(dev), pv.to(dev), n_prev + T)
            append = lambda k_, v_, c_: B.skv_project_append(L, k_, v_, c_)
            attend = lambda: B.skv_prefill_attention(L, q, out, n_prev, 0.0, pmode)
        sck = synth.channel_scales(synth.stable_seed(wl.name, 0, "sk"), HKV, d)
        scv = synth.channel_scales(synth.stable_seed(wl.name, 0, "sv"), HKV, d)
        for c0 in range(0, n_prev + T, 4096):
            t = min(4096, n_prev + T - c0)
            k = synth.kv_activations(synth.stable_seed(wl.name, 0, "k", c0), Bt, t, HKV, d, sck, dev)
            v = synth.kv_activations(synth.stable_seed(wl.name, 0, "v", c0), Bt, t, HKV, d, scv, dev)
            append(k, v, c0)
        q = synth.chunk_queries(synth.stable_seed(wl.name, "cq"), Bt, T, HQ, d, dev)
        out = torch.empty((Bt, T, HQ, d), dtype=torch.float32, device=dev)
        pmode = B.SKV_PREFILL_EXACT | {"default": 0, "together": B.SKV_PREFILL_SCHED_TOGETHER, "ahead": B.SKV_PREFILL_SCHED_AHEAD}[args.prefill_sched]
        iters = max(1, args.kernel_iters // 20)
        for _ in range(2):
            attend()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            attend()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        # algorithmic flops: per (sequence, query head, token t): 2 (r_K + r_V) per visible row, plus the
        # query projection and the lift (2 * 128 * r each)
        visible = sum(n_prev + t + 1 for t in range(T))
        flops = Bt * HQ * (2 * (rk + rv) * visible + T * 2 * d * (rk + rv))
        nbytes = Bt * HKV * (n_prev + T) * (rk + rv) * 2 + Bt * T * HQ * d * (2 + 4)
        res = {"mode": "prefill", "workload": wl.name, "batch": Bt, "T": T, "n_prev": n_prev, "r_k": rk, "r_v": rv,
               "sched": args.prefill_sched, "cache": args.cache, "ms_per_launch": round(ms, 4),
               "chunk_tokens_per_s": round(Bt * T / (ms * 1e-3), 1),
               "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": round(flops / (ms * 1e-3) / 1e12, 1),
                            "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops / (ms * 1e-3) / 1e12 / 2500.0, 4),
                            "flops_per_launch": flops, "compulsory_hbm_bytes": nbytes},
               "launches": iters + 2}
        if not args.no_cpu_baseline:
            # sampled rows against the oracle (its own float64 append of the same seeded inputs)
            from oracle import skv_oracle as O
            f64 = lambda t_: O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t_))
            rng = np.random.default_rng(5)
            b_s, kv_s = int(rng.integers(Bt)), int(rng.integers(HKV))
            ora = O.new_layer(1, HQ // HKV, 1, d, f64(pk[kv_s:kv_s + 1]), f64(pv[kv_s:kv_s + 1]), n_prev + T, store="bf16")
            for c0 in range(0, n_prev + T, 4096):
                t = min(4096, n_prev + T - c0)
                k = synth.kv_activations(synth.stable_seed(wl.name, 0, "k", c0), Bt, t, HKV, d, sck, dev)
                v = synth.kv_activations(synth.stable_seed(wl.name, 0, "v", c0), Bt, t, HKV, d, scv, dev)
                O.project_append(ora, f64(k[b_s:b_s + 1, :, kv_s:kv_s + 1]), f64(v[b_s:b_s + 1, :, kv_s:kv_s + 1]), c0)
            G = HQ // HKV
            toks = sorted(set([0, T - 1] + [int(x) for x in rng.integers(0, T, size=6)]))
            rows = [(0, t, g) for t in toks for g in range(G)]
            qs_ = f64(q[b_s:b_s + 1, :, kv_s * G:(kv_s + 1) * G])
            tb = time.perf_counter()
            want = O.prefill_attention(ora, qs_, n_prev, rows=rows)
            spent = time.perf_counter() - tb
            got = out[b_s, :, kv_s * G:(kv_s + 1) * G].cpu().numpy().astype(np.float64)
            err = max(float(np.max(np.abs(got[t, g] - want[0, t, g])) / np.max(np.abs(want[0, t, g]))) for _, t, g in rows)
            res["parity"] = {"max_rel_err_vs_oracle": err, "rows_checked": len(rows),
                             "tolerance": 2e-3}
            row_flops = sum(2 * (rk + rv) * (n_prev + t + 1) for _, t, _ in rows)
            res["cpu_baseline"] = {"value": round(row_flops / spent / 1e12, 6), "unit": "TFLOP/s (algorithmic)",
                                   "kind": "oracle", "sample": f"{len(rows)} query rows of one (sequence, KV head), {spent:.2f} s"}
        print(json.dumps(res))
        return
    K, W = args.steps, args.warmup
    if args.mode == "kernel":
        K, W = 1, 0
    Bt, HQ, HKV, d = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    if wl.r_k:
        ranks_k, ranks_v = [wl.r_k] * wl.n_layers, [wl.r_v] * wl.n_layers
    else:
        ranks_k, ranks_v = synth.layer_rank_draw(synth.stable_seed(wl.name, "ranks"), wl.n_layers)

    # The first timed step attends exactly wl.n_ctx tokens.
    n0 = wl.n_ctx - 1 - W
    cap = wl.n_ctx + K + 8
    assert n0 >= 1

    qbits = {"bf16": 0, "q8": 8, "q4": 4, "paged": 0, "paged_q8": 8, "paged_q4": 4}[args.cache]
    paged = args.cache.startswith("paged")
    q8 = qbits != 0                                  # any quantised cache
    QF = {8: (B.skv_q8_project_append, B.skv_q8_decode_step, B.skv_q8_decode_project_query, B.skv_q8_decode_partial),
          4: (B.skv_q4_project_append, B.skv_q4_decode_step, B.skv_q4_decode_project_query, B.skv_q4_decode_partial)}
    folded = args.variant == "folded"
    if folded and (q8 or paged):
        print("bench.py: --variant folded runs over the contiguous bf16 cache only", file=sys.stderr)
        sys.exit(2)

    def low(x, basis):
        """Stand-in for a model whose linear layers carry the bases: [..., H, d] x [H, d, r] -> bf16 [..., H, r]
        (plain torch, outside every timed region)."""
        return torch.einsum("...hd,hdc->...hc", x.float(), basis.to(x.device).float()).to(torch.bfloat16).contiguous()

    append_fn = QF[qbits][0] if q8 else B.skv_project_append
    step_fn = QF[qbits][1] if q8 else B.skv_decode_step
    if paged:                                        # every sequence at the same length: no length array
        append_fn = lambda L_, k_, v_, c_: B.skv_paged_project_append(L_, k_, v_, None, c_)
        step_fn = lambda L_, k_, v_, c_, q_, o_, sc_, ws_: B.skv_paged_decode_step(L_, k_, v_, None, c_, q_, o_, sc_, ws_)

    def row_bytes(li):
        """Bytes one cached token of one KV head occupies in layer li."""
        if q8:
            return (ranks_k[li] + ranks_v[li]) * qbits // 8 + 4 * ((ranks_v[li] + 63) // 64)
        return 2 * (ranks_k[li] + ranks_v[li])

    # A caller knows its model: when the layers of one step together exceed the last-level cache, no row can
    # be found there again on the next step, whatever a single launch covers.
    step_cache_bytes = sum(Bt * HKV * wl.n_ctx * row_bytes(li) for li in range(wl.n_layers))
    cache_reads = args.cache_reads
    if cache_reads == "auto":
        cache_reads = "stream" if (wl.n_layers > 1 and step_cache_bytes > STREAM_ABOVE) else "size"
        reads_flag = {"stream": B.SKV_READS_STREAMING, "size": B.SKV_READS_BY_SIZE}[cache_reads]
        B.DEFAULT_LAYER_FLAGS = engine_flag | reads_flag

    layers, scales, k_ranges = [], [], []
    for li in range(wl.n_layers):
        _, pk = synth.orthonormal_bases(synth.stable_seed(wl.name, li, "pk"), HKV, d, ranks_k[li])
        _, pv = synth.orthonormal_bases(synth.stable_seed(wl.name, li, "pv"), HKV, d, ranks_v[li])
        scales.append((synth.channel_scales(synth.stable_seed(wl.name, li, "sk"), HKV, d),
                       synth.channel_scales(synth.stable_seed(wl.name, li, "sv"), HKV, d)))
        if q8:
            # The caller's calibration: static key ranges per KV head and 64-channel group, from the
            # minimum and maximum of a seeded sample of projected keys (plain torch, not timed).
            cal = synth.kv_activations(synth.stable_seed(wl.name, li, "cal"), 1, 2048, HKV, d, scales[li][0], dev)
            proj = torch.einsum("thd,hdc->htc", cal[0].float(), pk.to(dev).float())          # [H, t, r_k]
            groups = [(g0, min(g0 + 64, ranks_k[li])) for g0 in range(0, ranks_k[li], 64)]
            lo = torch.stack([proj[:, :, a:b].amin(dim=(1, 2)) for a, b in groups], dim=1)
            hi = torch.stack([proj[:, :, a:b].amax(dim=(1, 2)) for a, b in groups], dim=1)
            # a margin of half the observed span on either side: rows outside it would clamp
            span = hi - lo
            lo, hi = lo - 0.5 * span, hi + 0.5 * span
            ksc, kzr = ((hi - lo) / float(2 ** qbits - 1)).contiguous(), lo.contiguous()
            k_ranges.append((ksc, kzr))
        if paged:
            # a pool with a few spare pages; the table is a seeded shuffle, so consecutive logical pages of a
            # sequence are scattered over the pool
            pt = args.page_tokens
            per_seq = (cap + pt - 1) // pt
            n_pages = Bt * per_seq + 16
            order = np.random.default_rng(synth.stable_seed(wl.name, li, "pages")).permutation(n_pages)
            table = torch.from_numpy(order[:Bt * per_seq].reshape(Bt, per_seq).astype(np.int32)).to(dev)
            layers.append(B.PagedLayer(Bt, HQ, HKV, pk.to(dev), pv.to(dev), pt, n_pages, table, bits=qbits,
                                       k_scale=ksc if q8 else None, k_zero=kzr if q8 else None))
        elif q8:
            layers.append(B.QuantLayer(Bt, HQ, HKV, pk.to(dev), pv.to(dev), ksc, kzr, cap, qbits))
        else:
            layers.append(B.Layer(Bt, HQ, HKV, pk.to(dev), pv.to(dev), cap))

    # Prefill the caches through the library's own append (chunks on the matrix cores).
    CH = 4096
    for li, L in enumerate(layers):
        for c0 in range(0, n0, CH):
            t = min(CH, n0 - c0)
            k = synth.kv_activations(synth.stable_seed(wl.name, li, "k", c0), Bt, t, HKV, d, scales[li][0], dev)
            v = synth.kv_activations(synth.stable_seed(wl.name, li, "v", c0), Bt, t, HKV, d, scales[li][1], dev)
            if folded:
                B.skv_append_projected(L, low(k, L.p_k), low(v, L.p_v), c0)
            else:
                append_fn(L, k, v, c0)
    torch.cuda.synchronize()

    # Per-step inputs: one new token per sequence and layer, one query per head.
    n_steps_total = W + K
    new_k = [synth.kv_activations(synth.stable_seed(wl.name, li, "nk"), Bt, n_steps_total, HKV, d, scales[li][0], dev)
             for li in range(wl.n_layers)]
    new_v = [synth.kv_activations(synth.stable_seed(wl.name, li, "nv"), Bt, n_steps_total, HKV, d, scales[li][1], dev)
             for li in range(wl.n_layers)]
    qs = torch.stack([synth.queries(synth.stable_seed(wl.name, "q", s), Bt, HQ * wl.n_layers, d, dev)
                      .view(Bt, wl.n_layers, HQ, d).transpose(0, 1).contiguous() for s in range(n_steps_total)])
    outs = torch.empty((n_steps_total, wl.n_layers, Bt, HQ, d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(B.skv_decode_workspace_bytes(L) for L in layers), dtype=torch.uint8, device=dev)

    if folded:
        G = HQ // HKV
        # per layer: [step][batch][1][H_KV][r] rows, [step][batch][H_Q][r_k] queries, [step][batch][H_Q][r_v] outputs
        nk_low = [low(new_k[li], L.p_k).transpose(0, 1).unsqueeze(2).contiguous() for li, L in enumerate(layers)]
        nv_low = [low(new_v[li], L.p_v).transpose(0, 1).unsqueeze(2).contiguous() for li, L in enumerate(layers)]
        q_low = [low(qs[:, li], L.p_k.repeat_interleave(G, dim=0)) for li, L in enumerate(layers)]
        outs_low = [torch.empty((n_steps_total, Bt, HQ, ranks_v[li]), dtype=torch.float32, device=dev)
                    for li in range(wl.n_layers)]

    # a stack of plain bf16 layers goes through the library's own loop over layers (the same launches)
    stack = B.LayerStack(layers) if (wl.n_layers > 1 and not (folded or q8 or paged)) else None

    def step(s: int):
        cur = n0 + s
        if stack is not None:
            B.skv_decode_step_layers(stack, [x[:, s:s + 1] for x in new_k], [x[:, s:s + 1] for x in new_v], cur,
                                     [qs[s, li] for li in range(wl.n_layers)],
                                     [outs[s, li] for li in range(wl.n_layers)], 0.0, ws)
            return
        for li, L in enumerate(layers):
            if folded:
                B.skv_decode_step_folded(L, nk_low[li][s], nv_low[li][s], cur, q_low[li][s], outs_low[li][s], 0.0, ws)
            else:
                step_fn(L, new_k[li][:, s:s + 1], new_v[li][:, s:s + 1], cur, qs[s, li], outs[s, li], 0.0, ws)

    for s in range(W):
        step(s)
    torch.cuda.synchronize()

    use_graph = not args.no_graph and args.mode == "bench"
    if use_graph:
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for s in range(W, W + K):
                    step(s)
        torch.cuda.synchronize()

    # ---- timed region: exactly K steps ------------------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if use_graph:
        g.replay()
    else:
        for s in range(W, W + K):
            step(s)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    ms_per_step = elapsed * 1e3 / K

    # algorithmic compressed-cache bytes read by the K timed steps
    bytes_steps = 0
    for s in range(W, W + K):
        n_ctx = n0 + s + 1
        for li in range(wl.n_layers):
            bytes_steps += Bt * HKV * n_ctx * row_bytes(li)
    gbps = bytes_steps / elapsed / 1e9
    tokens_per_s = Bt * K / elapsed

    # ---- roofline leg: the decode range kernel alone, events on the launch stream --------
    # single layer: that layer; a stack: the layer with the median rank sum
    li_big = sorted(range(wl.n_layers), key=lambda i: ranks_k[i] + ranks_v[i])[wl.n_layers // 2]
    Lr = layers[li_big]
    n_roof = wl.n_ctx
    default_splits = {0: B.skv_decode_default_splits, 8: B.skv_q8_decode_default_splits, 4: B.skv_q4_decode_default_splits}[qbits]
    if paged and q8:
        # no separate stage calls over quantised pages: the whole attention call is timed
        splits = B.skv_paged_decode_default_splits(Lr, n_roof)
        tmp_out = torch.empty((Bt, HQ, d), dtype=torch.float32, device=dev)
        partial_fn = lambda L_, n_, s_, ws_: B.skv_paged_decode_attention(L_, qs[0, li_big], tmp_out, None, n_, 0.0, ws_)
    elif q8 or folded:
        splits = args.splits if args.splits > 0 else default_splits(Lr, n_roof)
        # these variants keep the projected queries in the workspace (prepared by a small launch)
        (QF[qbits][2] if q8 else B.skv_decode_project_query)(Lr, qs[0, li_big], 0.0, ws)
        partial_fn = QF[qbits][3] if q8 else B.skv_decode_partial
    elif paged:
        splits = args.splits if args.splits > 0 else B.skv_paged_decode_default_splits(Lr, n_roof)
        partial_fn = lambda L_, n_, s_, ws_: B.skv_paged_decode_partial_q(L_, qs[0, li_big], None, n_, s_, 0.0, ws_)
    else:
        splits = args.splits if args.splits > 0 else default_splits(Lr, n_roof)
        # the launch the decode step makes: every workgroup projects its head group's queries itself
        partial_fn = lambda L_, n_, s_, ws_: B.skv_decode_partial_q(L_, qs[0, li_big], n_, s_, 0.0, ws_)
    # Launches alternate between n_ctx and n_ctx - 1 rows, as consecutive decode steps do: the range kernels sweep
    # a sequence front to back or back to front by the parity of its length (one row in 32768 less every other
    # launch; the bytes below are those of n_ctx - 1/2 rows).
    n_alt = (n_roof, max(1, n_roof - 1))
    for i in range(10):
        partial_fn(Lr, n_alt[i & 1], splits, ws)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.kernel_iters):
        partial_fn(Lr, n_alt[i & 1], splits, ws)
    e1.record()
    torch.cuda.synchronize()
    kern_ms = e0.elapsed_time(e1) / args.kernel_iters
    # algorithmic bytes of one launch: every cache row once per KV head, the projected
    # queries in, the per-range partial results out
    rk, rv = ranks_k[li_big], ranks_v[li_big]
    q_in = Bt * HQ * rk * 4 if (q8 or folded) else Bt * HQ * d * 2 + HKV * d * rk * 2   # projected queries, or queries + key bases
    kern_bytes = Bt * HKV * (n_alt[0] + n_alt[1]) * row_bytes(li_big) // 2 + q_in + Bt * HQ * splits * (rv + 2) * 4
    achieved = kern_bytes / (kern_ms * 1e-3) / 1e9

    # the yardstick: a kernel that only reads a buffer of the same size (same launch stream, same events)
    probe_bytes = min(max(int(kern_bytes), 1 << 24), 2 << 30)
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev).random_(0, 255)
    probe_sink = torch.zeros(4096, dtype=torch.float32, device=dev)
    probe_wgs = max(1, min(2048, probe_bytes // 16384))        # a workgroup's slice is at least one 16 KiB stride
    probe_streaming = B.skv_decode_streams_rows(Lr, n_roof)        # the kind of load the range kernel itself uses here
    for _ in range(5):
        probe_n = B.skv_probe_stream_read(probe_src, probe_wgs, probe_sink, probe_streaming)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(20):
        B.skv_probe_stream_read(probe_src, probe_wgs, probe_sink, probe_streaming)
    e1.record()
    torch.cuda.synchronize()
    probe_us = e0.elapsed_time(e1) * 1e3 / 20
    probe_gbps = probe_n / probe_us / 1e3

    # ---- HBM-only leg (one-layer workloads): the same launch and the same step, rotated over enough distinct
    #      copies of the layer's cache that no row can be found in the last-level cache again, with the load
    #      kind such a caller sets on its layers (SKV_READS_STREAMING: a model's layers together exceed that cache)
    hbm_only = None
    if args.mode == "bench" and wl.n_layers == 1 and not folded and not paged and not args.no_hbm_only:
        step_rows_bytes = Bt * HKV * wl.n_ctx * row_bytes(0)
        n_rot = max(3, -(-(1280 << 20) // step_rows_bytes) + 1)         # >= 1.25 GiB pass between two reads of a row
        cold_flags = engine_flag | B.SKV_READS_STREAMING
        rot = []
        for _ in range(n_rot):
            if q8:
                Lc = B.QuantLayer(Bt, HQ, HKV, layers[0].p_k, layers[0].p_v, k_ranges[0][0], k_ranges[0][1], cap, qbits,
                                  flags=cold_flags)
                Lc.v_meta.copy_(layers[0].v_meta)
            else:
                Lc = B.Layer(Bt, HQ, HKV, layers[0].p_k, layers[0].p_v, cap, flags=cold_flags)
            Lc.k_cache.copy_(layers[0].k_cache)
            Lc.v_cache.copy_(layers[0].v_cache)
            rot.append(Lc)
        torch.cuda.synchronize()
        cold_splits = args.splits if args.splits > 0 else default_splits(rot[0], n_roof)
        if q8:
            QF[qbits][2](rot[0], qs[0, 0], 0.0, ws)                      # projected queries in the shared workspace
        for i in range(2 * n_rot):
            partial_fn(rot[i % n_rot], n_roof, cold_splits, ws)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.kernel_iters):
            partial_fn(rot[i % n_rot], n_roof, cold_splits, ws)
        e1.record()
        torch.cuda.synchronize()
        cold_kern_us = e0.elapsed_time(e1) * 1e3 / args.kernel_iters
        cold_kern_bytes = kern_bytes + Bt * HQ * (cold_splits - splits) * (rv + 2) * 4
        # the yardstick under the same conditions: a plain streaming read rotated over as many distinct buffers
        probe_rot = torch.empty(n_rot * probe_bytes, dtype=torch.uint8, device=dev).random_(0, 255)
        slices = [probe_rot[i * probe_bytes:(i + 1) * probe_bytes] for i in range(n_rot)]
        for i in range(n_rot):
            cold_probe_n = B.skv_probe_stream_read(slices[i], probe_wgs, probe_sink, True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(4 * n_rot):
            B.skv_probe_stream_read(slices[i % n_rot], probe_wgs, probe_sink, True)
        e1.record()
        torch.cuda.synchronize()
        cold_probe_us = e0.elapsed_time(e1) * 1e3 / (4 * n_rot)
        del probe_rot, slices

        cold_out = torch.empty((K, Bt, HQ, d), dtype=torch.float32, device=dev)

        def cold_step(j: int):
            cur = wl.n_ctx - 1 + j // n_rot                            # every copy advances one token per visit
            step_fn(rot[j % n_rot], new_k[0][:, W + j:W + j + 1], new_v[0][:, W + j:W + j + 1], cur, qs[W + j, 0],
                    cold_out[j], 0.0, ws)
        for j in range(n_rot):
            cold_step(j)
        torch.cuda.synchronize()
        if use_graph:
            gc = torch.cuda.CUDAGraph()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(gc, stream=side):
                    for j in range(K):
                        cold_step(j)
            torch.cuda.synchronize()
        tc0 = time.perf_counter()
        if use_graph:
            gc.replay()
        else:
            for j in range(K):
                cold_step(j)
        torch.cuda.synchronize()
        cold_elapsed = time.perf_counter() - tc0
        cold_bytes = sum(Bt * HKV * (wl.n_ctx + j // n_rot) * row_bytes(0) for j in range(K))
        cold_achieved = cold_kern_bytes / cold_kern_us / 1e3
        hbm_only = {
            "what": f"the same launch / step rotated over {n_rot} distinct copies of the layer's cache "
                    f"({n_rot * step_rows_bytes / 2**30:.2f} GiB of rows), layers flagged SKV_READS_STREAMING",
            "us_per_launch": round(cold_kern_us, 3), "achieved": round(cold_achieved, 1),
            "frac": round(cold_achieved / HBM_PEAK_GBPS, 4), "splits": cold_splits,
            "plain_read": {"us_per_launch": round(cold_probe_us, 3), "GBps": round(cold_probe_n / cold_probe_us / 1e3, 1),
                           "range_kernel_vs_plain_read": round(cold_achieved / (cold_probe_n / cold_probe_us / 1e3), 4)},
            "ms_per_step": round(cold_elapsed * 1e3 / K, 5),
            "value": round(cold_bytes / cold_elapsed / 1e9, 1),
            "step_frac": round(cold_bytes / cold_elapsed / 1e9 / HBM_PEAK_GBPS, 4),
            "tokens_per_s": round(Bt * K / cold_elapsed, 1),
        }
        del rot

    traffic, traffic_src = read_traffic(wl.name, args.cache)
    result = {
        "metric": METRIC,
        "value": round(gbps, 1),
        "unit": "GB/s",
        "tokens_per_s": round(tokens_per_s, 1),
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": Bt, "n_q_heads": HQ, "n_kv_heads": HKV, "head_dim": d,
                   "n_ctx_first_step": wl.n_ctx, "n_layers": wl.n_layers,
                   "r_k": ranks_k if wl.n_layers > 1 else ranks_k[0],
                   "r_v": ranks_v if wl.n_layers > 1 else ranks_v[0],
                   "cache": (f"{qbits}-bit codes, group 64" if q8 else "bf16") + (f", pages of {args.page_tokens} rows, shuffled block table" if paged else ""), "step": ("place 1 projected token/sequence + attention in the compressed space, every layer" if folded
                            else "append 1 token/sequence + decode attention, every layer (skv_decode_step)"),
                   "variant": args.variant, "engine": args.engine, "cache_reads": cache_reads,
                   "launch": "hip graph replay" if use_graph else "per-call launches"},
        "roofline": {"bound": "hbm", "kernel": ("projection + decode_partial_mma_kernel + merge (the whole attention call: no stage calls over quantised pages)" if (paged and q8)
                                else ("decode_partial_kernel", "decode_partial_mma_kernel")[B.skv_decode_engine_for(Lr)]),
                     "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": traffic_src, "bytes_per_launch": kern_bytes,
                     "loads": "streaming" if probe_streaming else "ordinary",
                     "us_per_launch": round(kern_ms * 1e3, 3), "n_ctx": n_roof, "r_k": rk, "r_v": rv,
                     "splits": splits,
                     "plain_read": {"kernel": "stream_read_kernel", "bytes": probe_n, "us_per_launch": round(probe_us, 3),
                                    "GBps": round(probe_gbps, 1), "range_kernel_vs_plain_read": round(achieved / probe_gbps, 4)}},
    }
    if hbm_only is not None:
        result["value_hbm_only"] = hbm_only["value"]
        result["roofline"]["hbm_only"] = hbm_only

    # ---- CPU baseline: the float64 oracle, one decode step of the same workload ----------
    if not args.no_cpu_baseline and args.mode == "bench":
        from oracle import skv_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = 1
        f64 = lambda t: O.bf16_bits_to_f64(synth.torch_bf16_to_bits(t))
        li = 0
        s_chk = W + K - 1                                  # the last timed step
        n_chk = n0 + s_chk + 1
        if q8:
            ora = O.new_quant_layer(Bt, HQ, HKV, d, f64(layers[li].p_k), f64(layers[li].p_v),
                                    k_ranges[li][0].cpu().numpy(), k_ranges[li][1].cpu().numpy(), n_chk, qbits)
            ora_append, ora_decode = O.quant_project_append, O.quant_decode_attention
        else:
            ora = O.new_layer(Bt, HQ, HKV, d, f64(layers[li].p_k), f64(layers[li].p_v), n_chk, store="bf16")
            ora_append, ora_decode = O.project_append, O.decode_attention
        if folded:
            # the oracle is handed the same projected bf16 rows and queries as the library
            ora_append = lambda lay, k_, v_, c_: O.append_projected(lay, f64(low(k_, layers[li].p_k)),
                                                                    f64(low(v_, layers[li].p_v)), c_)
            ora_decode = O.decode_attention_folded
        for c0 in range(0, n0, CH):                        # same seeded raw inputs as the GPU prefill
            t = min(CH, n0 - c0)
            k = synth.kv_activations(synth.stable_seed(wl.name, li, "k", c0), Bt, t, HKV, d, scales[li][0], dev)
            v = synth.kv_activations(synth.stable_seed(wl.name, li, "v", c0), Bt, t, HKV, d, scales[li][1], dev)
            ora_append(ora, k if folded else f64(k), v if folded else f64(v), c0)
        nk_, nv_ = new_k[li][:, :s_chk + 1], new_v[li][:, :s_chk + 1]
        ora_append(ora, nk_ if folded else f64(nk_), nv_ if folded else f64(nv_), n0)
        # Quantised caches: a code is an integer decided by floating point (the library decides it in float32 on a
        # float32 sum, the oracle in float64), so a few codes sit one apart and each side's own cache is not the
        # other's.  Parity is then stated as two facts: the library's stored codes are the oracle's up to such
        # flips, and on the very bytes the library stored its output is the oracle's within 2e-3.
        mine = None
        flips = None
        if q8:
            def unpack(t):
                a = t.cpu().numpy()
                if qbits == 8:
                    return a
                o = np.empty(a.shape[:-1] + (a.shape[-1] * 2,), np.uint8)
                o[..., 0::2], o[..., 1::2] = a & 0x0F, a >> 4
                return o
            Lg = layers[li]
            if paged:
                meta = Lg.v_meta.cpu().numpy().view(np.uint32)
                mine = O.OraclePagedQuantCache(unpack(Lg.k_pool), unpack(Lg.v_pool), (meta & 0xffff).astype(np.uint16),
                                               (meta >> 16).astype(np.uint16), Lg.block_table.cpu().numpy(), Lg.page_tokens)
                mine_decode = lambda qh_, n_: O.paged_quant_decode_attention(ora, mine, qh_, [n_] * Bt)
                got_k = np.stack([O.paged_rows(mine.k_codes, mine.block_table[b_], mine.page_tokens, n_chk) for b_ in range(Bt)])
            else:
                mine = O.new_quant_layer(Bt, HQ, HKV, d, ora.p_k, ora.p_v, ora.k_scale, ora.k_zero, n_chk, qbits)
                mine.k_codes[:] = unpack(Lg.k_cache[:, :, :n_chk])
                mine.v_codes[:] = unpack(Lg.v_cache[:, :, :n_chk])
                meta = Lg.v_meta[:, :, :n_chk].cpu().numpy().view(np.uint32)
                mine.v_scale_bits[:] = (meta & 0xffff).astype(np.uint16)
                mine.v_zero_bits[:] = (meta >> 16).astype(np.uint16)
                mine_decode = lambda qh_, n_: O.quant_decode_attention(mine, qh_, n_)
                got_k = mine.k_codes
            dk = np.abs(got_k.astype(np.int16) - ora.k_codes[:, :, :n_chk].astype(np.int16))
            flips = {"key_codes_differing": float((dk > 0).mean()), "max_key_code_distance": int(dk.max())}
        # bounded sample: the last timed steps, newest first, for about 12 s of host time
        budget_s, spent, errs, errs_stored, cpu_bytes, n_done = 12.0, 0.0, [], [], 0, 0
        rel = lambda got_, want_: float(np.max(np.max(np.abs(got_ - want_), axis=-1) / np.max(np.abs(want_), axis=-1)))
        for s_i in range(s_chk, W - 1, -1):
            n_i = n0 + s_i + 1
            qh = f64(q_low[li][s_i]) if folded else f64(qs[s_i, li])
            tb = time.perf_counter()
            want = ora_decode(ora, qh, n_i)
            spent += time.perf_counter() - tb
            got = (outs_low[li][s_i] if folded else outs[s_i, li]).cpu().numpy().astype(np.float64)
            errs.append(rel(got, want))
            if mine is not None and len(errs_stored) < 2:
                errs_stored.append(rel(got, mine_decode(qh, n_i)))
            cpu_bytes += Bt * HKV * n_i * row_bytes(li)
            n_done += 1
            if spent >= budget_s:
                break
        result["cpu_baseline"] = {
            "value": round(cpu_bytes / spent / 1e9, 4), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "tokens_per_s": round(Bt * n_done / spent / wl.n_layers, 3),
            "sample": f"decode attention of layer 0 for the last {n_done} timed steps (n_ctx {n0 + s_chk + 2 - n_done}.."
                      f"{n_chk}), all {Bt} sequences x {HQ} query heads, float64 definition form, {spent:.2f} s of host time",
        }
        if q8:
            result["parity"] = {"max_rel_err_vs_oracle": max(errs_stored), "tolerance": 2e-3,
                                "checked": f"layer 0, last {len(errs_stored)} timed steps, {Bt} sequences x {HQ} heads each: the "
                                           "oracle's attention over the codes and ranges the library stored",
                                "stored_codes_vs_oracle": flips,
                                "each_side_its_own_cache_rel_err": max(errs)}
        else:
            result["parity"] = {"max_rel_err_vs_oracle": max(errs), "tolerance": 2e-3,
                                "checked": f"layer 0, last {n_done} timed steps, {Bt} sequences x {HQ} heads each"}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
