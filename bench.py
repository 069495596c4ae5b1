#!/usr/bin/env python3
"""Benchmark of the H2O hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-graph]

A "step" is one pass of the whole hot path over one batch of synthetic input of
the OPT-6.7B-shaped layer workload: reset the cache, score the 2048-token prompt
(row statistics + column sums on the matrix cores), compress it to the 410-slot
budget, then 256 generation steps (fused attention + score accumulation +
eviction + overwrite).  All inputs are resident in HBM before the clock starts.
Prints one JSON line: tokens/s of the whole pass, the roofline record of the
dominant kernel (the generation step, HBM-bound) and the CPU oracle timed on a
bounded sample of the same workload.
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

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0       # dense bf16 / fp16 matrix peak of the part
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# Cold-cache leg: this many independent caches of the workload are visited in turn,
# so that every launch reads a cache that the 256 MB last-level cache cannot still hold.
COLD_CACHES = 8
LLC_BYTES = 256 << 20


def profiled_figures():
    """Figures that cannot be collected inside a timed run (hardware counters) come
    from the rocprofv3 summaries under profiles/: every line of the form
        bench-figure <name> <kernel> <workload> <value>
    is one figure (HBM bytes per launch from FETCH_SIZE / WRITE_SIZE scaled by what
    the same counters read for a plain 256 MiB copy; vector instructions per launch
    from SQ_INSTS_VALU).  A figure no summary holds is reported as null."""
    out = {}
    pdir = os.path.join(ROOT, "profiles")
    if os.path.isdir(pdir):
        for fn in sorted(os.listdir(pdir)):
            if not fn.endswith((".md", ".txt")):
                continue
            with open(os.path.join(pdir, fn)) as f:
                for line in f:
                    w = line.split()
                    if len(w) == 5 and w[0] == "bench-figure":
                        try:
                            out[(w[1], w[2], w[3])] = float(w[4])
                        except ValueError:
                            pass
    return out


def decode_bytes_per_head_step(k: int, d: int, esize: int, kv_bits: int = 0) -> int:
    """Algorithmic bytes one head moves per generation step: K and V rows read
    once, scores read + written and positions read (12 B per slot), q / k_new /
    v_new read and the new K row, V row and output written (6 rows), plus the
    victim's score and position written (8 B).  With 4-bit storage a cached row is
    d/2 bytes of codes + 8 bytes of (scale, min) per 64 elements."""
    if kv_bits == 4:
        row = d // 2 + 8 * (d // 64)
        return 2 * k * row + 12 * k + 4 * d * esize + 2 * row + 8
    return 2 * k * d * esize + 12 * k + 6 * d * esize + 8


def prefill_flops_per_pass(n: int, d: int, heads: int) -> int:
    """Algorithmic flops of one masked QK^T over all heads: n(n+1)/2 visible
    products per head, 2d flops each."""
    return n * (n + 1) * d * heads


def time_prefill_passes(hb, cfg, Q, K, n, ws, stream, reps=5):
    """Average duration (ms) of the two matrix-core passes (row statistics +
    column sums) launched back to back, HIP events on the launch stream."""
    import torch
    out = torch.empty((cfg.batch, cfg.heads, n), dtype=torch.float32, device=Q.device)
    sp = stream.cuda_stream
    hb.h2o_prefill_colsum(cfg, Q, K, n, ws, ws.numel(), out, sp)
    stream.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(3):
        e0.record(stream)
        for _ in range(reps):
            hb.h2o_prefill_colsum(cfg, Q, K, n, ws, ws.numel(), out, sp)
        e1.record(stream)
        stream.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps)
    return best


def time_attention(hb, cfg, Q, K, V, n, ws, out, stream, reps=5):
    """Average duration (ms) of the prompt attention (transpose of V + the
    attention kernel), HIP events on the launch stream."""
    import torch
    sp = stream.cuda_stream
    hb.h2o_prefill_attention(cfg, Q, K, V, n, ws, ws.numel(), out, None, sp)
    stream.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(3):
        e0.record(stream)
        for _ in range(reps):
            hb.h2o_prefill_attention(cfg, Q, K, V, n, ws, ws.numel(), out, None, sp)
        e1.record(stream)
        stream.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps)
    return best


def cpu_baseline(w, sample_heads: int):
    """The oracle as it stands on this host's cores: prompt phase + all generation
    steps for `sample_heads` heads of the workload, threads over heads."""
    import torch
    from oracle.h2o_oracle import OracleHead, map_heads
    from paper_2306_14048_amd import synth
    Q, K, V = synth.make_prompt(1, sample_heads, w.prompt, w.head_dim, w.dtype, w.sigma, "cpu")
    qs, ks, vs = synth.make_steps(1, sample_heads, w.head_dim, w.steps, w.dtype, w.sigma, "cpu")
    Q, K, V = Q.double().numpy(), K.double().numpy(), V.double().numpy()
    qs, ks, vs = qs.double().numpy(), ks.double().numpy(), vs.double().numpy()
    scale = 1.0 / float(w.head_dim) ** 0.5

    def one(h):
        o = OracleHead(w.head_dim, w.heavy, w.recent, scale, score_f32=True, cap=w.prompt + w.steps)
        o.prefill(Q[0, h], K[0, h], V[0, h])
        for s in range(w.steps):
            o.decode(qs[s, 0, h], ks[s, 0, h], vs[s, 0, h])
        return o.t

    t0 = time.perf_counter()
    _, threads = map_heads(one, range(sample_heads))
    dt = time.perf_counter() - t0
    heads = w.batch * w.heads
    whole = dt * heads / sample_heads                    # heads are independent and identical
    tokens = w.batch * (w.steps if w.steps else w.prompt)
    return {"value": tokens / whole, "unit": "tokens/s", "cores": threads,
            "kind": "oracle",
            "sample": "%d of %d heads, full prompt phase + %d steps each, %.1f s measured, "
                      "scaled by head count" % (sample_heads, heads, w.steps, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="opt6.7b_layer_f16")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cold-cache leg (the generation step rotating over %d independent "
                         "caches so that no launch finds its cache in the last-level cache)" % COLD_CACHES)
    ap.add_argument("--cpu-heads", type=int, default=0, help="heads the oracle is timed on (0 = all)")
    ap.add_argument("--prompt", choices=("scores", "attention", "chunked"), default="scores",
                    help="prompt phase: 'scores' = row statistics + column sums + compression (the "
                         "default step); 'attention' = causal attention output whose row statistics "
                         "feed the column sums, + compression (a layer's whole prompt phase); "
                         "'chunked' = the prompt in chunks of --chunk tokens, each scored against "
                         "cache + chunk and compressed to the budget (bounded memory)")
    ap.add_argument("--chunk", type=int, default=1024, help="chunk length for --prompt chunked")
    ap.add_argument("--chunk-output", action="store_true",
                    help="--prompt chunked: also produce every chunk's attention output")
    ap.add_argument("--kv-bits", type=int, default=0, choices=(0, 4),
                    help="cache storage: 0 = the workload's element type, 4 = 4-bit group-wise codes")
    ap.add_argument("--decode-steps", type=int, default=0,
                    help="profiling aid: run only this many generation steps per pass (0 = the "
                         "workload's own count); the JSON line reports the count it ran")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (calibrates the profiler's "
                         "FETCH_SIZE / WRITE_SIZE counters against a kernel of known traffic)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (heads are independent and would "
                 "shard with no communication, but no multi-GPU path is part of it); use --gpus 1")

    import torch
    from paper_2306_14048_amd import binding as hb, synth
    figures = profiled_figures()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    w = synth.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    B, Hh, d, n, T = w.batch, w.heads, w.head_dim, w.prompt, w.steps
    if args.decode_steps > 0:
        T = min(T, args.decode_steps)
    k = w.budget
    esize = 4 if w.dtype == torch.float32 else 2

    L = w.layers
    step_stride = B * Hh * d * esize
    caches, steps_in = [], []
    if L == 1:
        Q, K, V = synth.make_prompt(B, Hh, n, d, w.dtype, w.sigma, dev)
        cache = hb.H2OCache(B, Hh, d, w.heavy, w.recent, w.dtype, device=dev, kv_bits=args.kv_bits)
        ws = cache.workspace(n)
        attn_out = None
        if args.prompt == "attention":
            ws = torch.empty(hb.h2o_prefill_attention_workspace_bytes(cache.cfg, n),
                             dtype=torch.uint8, device=dev)
            attn_out = torch.empty_like(Q)
        chunks, chunk_out = [], None
        if args.prompt == "chunked":
            # the chunk entry point takes [B, Hh, m, d] blocks: cut the prompt up before the clock starts
            m = max(1, min(args.chunk, n))
            ws = torch.empty(hb.h2o_prefill_chunk_workspace_bytes(cache.cfg, m, args.chunk_output),
                             dtype=torch.uint8, device=dev)
            if args.chunk_output:
                chunk_out = torch.empty((B, Hh, m, d), dtype=w.dtype, device=dev).data_ptr()
            for t0 in range(0, n, m):
                chunks.append(tuple(x[:, :, t0:t0 + m].contiguous() for x in (Q, K, V)))
        Qp, Kp, Vp, wsp, wsn = Q.data_ptr(), K.data_ptr(), V.data_ptr(), ws.data_ptr(), ws.numel()
        caches.append(cache)
    else:
        # a stack of layers: every layer's cache stays resident; prompts are drawn,
        # scored and compressed one layer at a time before the clock starts (all
        # layers' prompts together would not fit), and the timed pass is the
        # generation phase: T token steps, each visiting every layer in turn
        for layer in range(L):
            Q, K, V = synth.make_prompt(B, Hh, n, d, w.dtype, w.sigma, dev, layer=layer)
            cache = hb.H2OCache(B, Hh, d, w.heavy, w.recent, w.dtype, device=dev, kv_bits=args.kv_bits)
            cache.prefill_scores(Q, K, V)
            torch.cuda.synchronize()
            cache._ws = None
            del Q, K, V
            caches.append(cache)
            # (a line per layer: this set-up takes minutes and would otherwise be silent)
            print("bench.py: layer %d of %d scored and compressed" % (layer + 1, L), file=sys.stderr, flush=True)
    for layer in range(L):
        steps_in.append(synth.make_steps(B, Hh, d, T, w.dtype, w.sigma, dev, layer=layer))
    outs = torch.empty((T, B, Hh, d), dtype=w.dtype, device=dev)
    op = outs.data_ptr()
    ptrs = [(c.handle, q.data_ptr(), k_.data_ptr(), v.data_ptr()) for c, (q, k_, v) in zip(caches, steps_in)]

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def decode_all(sp):
        for s in range(T):
            off = s * step_stride
            for (h, qp, kp, vp) in ptrs:
                hb.h2o_decode_step(h, qp + off, kp + off, vp + off, op + off, sp)

    def one_pass(stream, timed_events=False):
        sp = stream.cuda_stream
        if L == 1:
            hb.h2o_cache_reset(ptrs[0][0], sp)
        if timed_events:
            ev[0].record(stream)
        if L == 1 and args.prompt == "attention":
            hb.h2o_prefill_attention_scores(ptrs[0][0], Qp, Kp, Vp, n, wsp, wsn, attn_out.data_ptr(),
                                            None, sp)
        elif L == 1 and args.prompt == "chunked":
            for (cq, ck, cv) in chunks:
                hb.h2o_prefill_chunk(ptrs[0][0], cq.data_ptr(), ck.data_ptr(), cv.data_ptr(),
                                     cq.shape[2], wsp, wsn, chunk_out, sp)
        elif L == 1:
            hb.h2o_prefill_scores(ptrs[0][0], Qp, Kp, Vp, n, wsp, wsn, None, sp)
        if timed_events:
            ev[1].record(stream)
        decode_all(sp)
        if timed_events:
            ev[2].record(stream)

    stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    graph = None
    with torch.cuda.stream(stream):
        for _ in range(max(1, args.warmup)):
            one_pass(stream)
        stream.synchronize()
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                one_pass(stream)
            graph.replay()
            stream.synchronize()

        # kernel-level timing with events on the launch stream (eager launches:
        # events cannot be placed inside a captured graph)
        prefill_ms, decode_ms = [], []
        for _ in range(3):
            one_pass(stream, timed_events=True)
            stream.synchronize()
            prefill_ms.append(ev[0].elapsed_time(ev[1]))
            decode_ms.append(ev[1].elapsed_time(ev[2]))

        # whole-pass timing
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            if graph is not None:
                graph.replay()
            else:
                one_pass(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0

        # the two matrix-core passes of the prompt phase on their own
        pre_pass_ms = attn_ms = None
        if L == 1 and args.prompt != "chunked":
            pre_pass_ms = time_prefill_passes(hb, caches[0].cfg, Q, K, n, ws, stream)
        if L == 1 and args.prompt == "attention":
            attn_ms = time_attention(hb, caches[0].cfg, Q, K, V, n, ws, attn_out, stream)

        # generation-only timing in the same launch mode (graph of all step launches)
        dec_graph_us = None
        if graph is not None and T > 0:
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2, stream=stream):
                decode_all(stream.cuda_stream)
            g2.replay()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 5 if L == 1 else 2
            e0.record(stream)
            for _ in range(reps):
                g2.replay()
            e1.record(stream)
            stream.synchronize()
            dec_graph_us = e0.elapsed_time(e1) * 1e3 / (reps * T * L)

        # Cold-cache leg of the generation step.  One layer's cache (C2: 108 MB) fits the
        # 256 MB last-level cache, so the loop above may be served from there; here
        # COLD_CACHES independent caches of the same workload are visited in turn (one
        # graph of T x COLD_CACHES launches), so that a cache is re-read only after
        # COLD_CACHES - 1 others of its size have been swept: the HBM-proof figure.
        cold = None
        if L == 1 and T > 0 and not args.no_cold and graph is not None:
            cache_bytes = caches[0].nbytes
            extra = []
            n_ring = min(32, max(COLD_CACHES, -(-860_000_000 // cache_bytes)))   # >= ~0.86 GB swept per round
            for _ in range(n_ring - 1):
                c = hb.H2OCache(B, Hh, d, w.heavy, w.recent, w.dtype, device=dev, kv_bits=args.kv_bits)
                hb.h2o_prefill_scores(c.handle, Qp, Kp, Vp, n, wsp, wsn, None, stream.cuda_stream)
                extra.append(c)
            hb.h2o_cache_reset(ptrs[0][0], stream.cuda_stream)
            hb.h2o_prefill_scores(ptrs[0][0], Qp, Kp, Vp, n, wsp, wsn, None, stream.cuda_stream)
            stream.synchronize()
            ring = [ptrs[0][0]] + [c.handle for c in extra]
            (_, qp, kp, vp) = ptrs[0]

            def decode_ring(sp):
                for s in range(T):
                    off = s * step_stride
                    for h in ring:
                        hb.h2o_decode_step(h, qp + off, kp + off, vp + off, op + off, sp)
            decode_ring(stream.cuda_stream)          # warm-up pass (t advances; the budget is already full)
            stream.synchronize()
            g3 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g3, stream=stream):
                decode_ring(stream.cuda_stream)
            g3.replay()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            best = float("inf")
            for _ in range(3):
                e0.record(stream)
                g3.replay()
                e1.record(stream)
                stream.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1e3 / (T * len(ring)))
            cold = {"us_per_launch": best, "caches": len(ring), "working_set_bytes": cache_bytes * len(ring)}
            for c in extra:
                c.close()
            del extra

    ms_per_step = dt * 1e3 / args.steps
    # generated tokens per second; a prompt-only workload counts prompt tokens
    tokens_per_s = B * (T if T else n) / (dt / args.steps)
    mfma_roofline = None
    if pre_pass_ms is not None:
        fl = 2 * prefill_flops_per_pass(n, d, B * Hh)
        tf = fl / (pre_pass_ms * 1e-3) / 1e12
        mfma_roofline = {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / MFMA_PEAK_TFLOPS, "traffic": figures.get(("traffic_bytes_per_launch_pair", "prefill_pass_kernel", w.name)),
                         "kernel": "prefill_pass_kernel (row statistics + column sums, two launches)",
                         "flops_per_launch_pair": fl, "ms_per_launch_pair": pre_pass_ms}
    if T > 0:
        dec_us_eager = min(decode_ms) * 1e3 / (T * L)
        dec_us = dec_graph_us if dec_graph_us is not None else dec_us_eager
        bytes_per_launch = decode_bytes_per_head_step(k, d, esize, args.kv_bits) * B * Hh
        achieved = bytes_per_launch / (dec_us * 1e-6) / 1e9
    rec = {
        "metric": "H2O decode step: achieved HBM GB/s (% peak) + tokens/s, OPT-6.7B-shape layer",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": {torch.float16: "f16", torch.bfloat16: "bf16", torch.float32: "f32"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "heads": Hh, "head_dim": d, "prompt": n,
                   "decode_steps": T, "layers": L, "budget": k, "heavy": w.heavy, "recent": w.recent,
                   "step": ("cache reset + prompt scoring/compression" +
                            (" + %d generation steps" % T if T else "")) if L == 1
                   else ("%d generation steps x %d resident layer caches (prompt phase done before "
                         "the clock starts)" % (T, L)),
                   "launch": "eager" if graph is None else "hip-graph replay",
                   "kv_bits": args.kv_bits or 8 * esize},
        "prefill_ms": min(prefill_ms) if L == 1 else None,
    }
    if attn_ms is not None:
        # QK^T and PV over the visible half: twice the flops of one scoring pass
        fl = 2 * prefill_flops_per_pass(n, d, B * Hh)
        tf = fl / (attn_ms * 1e-3) / 1e12
        rec["attention_roofline"] = {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS,
                                     "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS, "traffic": None,
                                     "kernel": "transpose_v_kernel + prefill_attn_kernel",
                                     "flops_per_launch": fl, "ms_per_launch": attn_ms}
        rec["config"]["prompt_phase"] = "attention output + column sums + compression"
    if L == 1 and args.prompt == "chunked":
        # logits the two passes form over all chunks: every chunk query against the
        # cached tokens and the chunk's own visible part
        pairs, occ = 0, 0
        for (cq, _, _) in chunks:
            m = cq.shape[2]
            pairs += m * occ + m * (m + 1) // 2
            occ = min(k, occ + m)
        fl = 2 * 2 * d * pairs * B * Hh
        tf = fl / (min(prefill_ms) * 1e-3) / 1e12
        mfma_roofline = {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / MFMA_PEAK_TFLOPS, "traffic": None,
                         "kernel": "whole chunked prompt phase: per chunk concat_kernel + two "
                                   "prefill_pass_kernel launches + select_gather_kernel",
                         "flops": fl, "ms": min(prefill_ms), "chunk": chunks[0][0].shape[2],
                         "chunks": len(chunks)}
        rec["config"]["prompt_phase"] = "chunks of %d tokens, compressed to the budget after each" \
            % chunks[0][0].shape[2]
    if T > 0:
        # the dominant kernel: the generation step, HBM-bound
        kname = "decode_resident_kernel" if args.kv_bits == 0 else "decode_q4_kernel"
        ws_bytes = sum(c.nbytes for c in caches)
        rec["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": achieved / HBM_PEAK_GBS,
                           "traffic": figures.get(("traffic_bytes_per_launch", kname, w.name)),
                           "kernel": kname,
                           "bytes_per_launch": bytes_per_launch,
                           "us_per_launch": dec_us, "us_per_launch_eager": dec_us_eager,
                           "working_set_bytes": ws_bytes,
                           "working_set": "fits the 256 MB last-level cache: see roofline_cold for the HBM-proof figure"
                           if ws_bytes <= LLC_BYTES else "exceeds the 256 MB last-level cache"}
        if cold is not None:
            ach = bytes_per_launch / (cold["us_per_launch"] * 1e-6) / 1e9
            rec["roofline_cold"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": ach / HBM_PEAK_GBS, "kernel": kname,
                                    "bytes_per_launch": bytes_per_launch,
                                    "us_per_launch": cold["us_per_launch"], "caches": cold["caches"],
                                    "working_set_bytes": cold["working_set_bytes"],
                                    "launch": "one hip-graph of %d steps x %d independent caches visited in turn"
                                    % (T, cold["caches"])}
        rec["decode_tokens_per_s"] = B / (dec_us * L * 1e-6)
        q4_valu = figures.get(("vector_instructions_per_launch", "decode_q4_kernel", w.name))
        if args.kv_bits == 4 and q4_valu:
            ops = q4_valu * 64 / (dec_us * 1e-6) / 1e12
            rec["alu_roofline"] = {"bound": "alu", "achieved": ops, "peak": ALU_PEAK_TLANEOPS,
                                   "unit": "T vector-instruction lanes/s", "frac": ops / ALU_PEAK_TLANEOPS,
                                   "kernel": "decode_q4_kernel",
                                   "vector_instructions_per_launch": q4_valu}
        if mfma_roofline is not None:
            rec["prefill_roofline"] = mfma_roofline
    else:
        rec["roofline"] = mfma_roofline
    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)                       # the dispatch to read: 256 MiB in, 256 MiB out
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and L == 1:
        heads_total = B * Hh
        rec["cpu_baseline"] = cpu_baseline(w, args.cpu_heads if args.cpu_heads > 0 else heads_total)
    print(json.dumps(rec))
    for c in caches:
        c.close()


if __name__ == "__main__":
    main()
