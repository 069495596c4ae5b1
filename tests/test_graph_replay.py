"""The benchmark replays the whole pass (reset + prompt phase + generation steps)
as one captured HIP graph.  A captured pass must give the same results on every
replay as the eager run, with eager work and synchronisation between replays."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["scores", "scores-4bit", "chunked", "chunked-output"])
def test_captured_pass_replays_identically(mode):
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, T, H, R = 2, 8, 128, 384, 24, 48, 48
    dtype = torch.float16
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 77)
    qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, 1.0, dev, 77)
    cache = hb.H2OCache(B, Hh, d, H, R, dtype, device=dev, kv_bits=4 if mode == "scores-4bit" else 0)
    outs = torch.empty((T, B, Hh, d), dtype=dtype, device=dev)
    if mode.startswith("chunked"):
        m = 128
        chunks = [tuple(x[:, :, t0:t0 + m].contiguous() for x in (Q, K, V)) for t0 in range(0, n, m)]
        ws = torch.empty(hb.h2o_prefill_chunk_workspace_bytes(cache.cfg, m, mode == "chunked-output"),
                         dtype=torch.uint8, device=dev)
        chunk_out = torch.empty((len(chunks), B, Hh, m, d), dtype=dtype, device=dev)
    else:
        ws = cache.workspace(n)

    def one_pass(stream):
        sp = stream.cuda_stream
        hb.h2o_cache_reset(cache.handle, sp)
        if mode.startswith("chunked"):
            for i, (cq, ck, cv) in enumerate(chunks):
                hb.h2o_prefill_chunk(cache.handle, cq, ck, cv, m, ws, ws.numel(),
                                     chunk_out[i] if mode == "chunked-output" else None, sp)
        else:
            hb.h2o_prefill_scores(cache.handle, Q, K, V, n, ws, ws.numel(), None, sp)
        for s in range(T):
            hb.h2o_decode_step(cache.handle, qs[s], ks[s], vs[s], outs[s], sp)

    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        one_pass(stream)
        stream.synchronize()
        ref_out = outs.clone()
        ref_pos, ref_acc = (x.clone() for x in cache.snapshot(stream))
        stream.synchronize()
        ref_kv = [x.clone() for x in cache.views()[:2]]
        ref_chunk_out = chunk_out.clone() if mode == "chunked-output" else None
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            one_pass(stream)
        for rep in range(4):
            outs.zero_()                                   # eager work between replays
            if mode == "chunked-output":
                chunk_out.zero_()
            scratch = torch.randn(1 << 20, device=dev).sum()
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            pos, acc = cache.snapshot(stream)
            stream.synchronize()
            assert torch.equal(outs, ref_out), "replay %d: outputs differ from the eager pass" % rep
            assert torch.equal(pos, ref_pos) and torch.equal(acc, ref_acc), \
                "replay %d: cache state differs from the eager pass" % rep
            for x, y in zip(cache.views()[:2], ref_kv):
                assert torch.equal(x, y), "replay %d: cached rows differ from the eager pass" % rep
            if mode == "chunked-output":
                assert torch.equal(chunk_out, ref_chunk_out)
            assert torch.isfinite(scratch)
    cache.close()


def test_captured_stack_of_layer_caches_against_the_oracle():
    """What the benchmark does for the 32-layer workload, at a small size: several layer
    caches resident at once, the generation phase (every token step visits every layer's
    cache in turn) captured as ONE HIP graph and replayed; before each replay the caches
    are restored to the same starting state.  Every replay's outputs and final states must
    equal the eager run's bit for bit, and the eager run is checked head by head against
    the oracle."""
    import numpy as np
    from paper_2306_14048_amd import binding as hb, synth
    from tests import parity
    dev = torch.device("cuda:0")
    L, B, Hh, d, n, T, H, R = 6, 2, 4, 128, 300, 12, 40, 40
    dtype = torch.float16
    k = H + R
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    scale = parity.oracle_scale(d)
    caches, starts, oracles, steps_in = [], [], [], []
    for layer in range(L):
        Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 55, layer=layer)
        orc, _ = parity.oracle_prefill_heads(Q.cpu(), K.cpu(), V.cpu(), heads, H, R, scale, cap=n + T)
        state = tuple(x.to(dev) for x in parity.cache_state_from_oracles(orc, B, Hh, k, K.cpu(), V.cpu()))
        c = hb.H2OCache(B, Hh, d, H, R, dtype, device=dev)
        caches.append(c); starts.append(state); oracles.append(orc)
        steps_in.append(synth.make_steps(B, Hh, d, T, dtype, 1.0, dev, 55, layer=layer))
    outs = torch.empty((L, T, B, Hh, d), dtype=dtype, device=dev)
    snaps = torch.empty((L, T, B, Hh, k), dtype=torch.int32, device=dev)

    def restore_all(stream):
        for c, (Kc, Vc, acc, pos) in zip(caches, starts):
            c.restore(Kc, Vc, acc, pos, n, stream=stream)

    def generate(stream):
        sp = stream.cuda_stream
        for s in range(T):
            for layer, c in enumerate(caches):
                q, kk, v = steps_in[layer]
                hb.h2o_decode_step(c.handle, q[s], kk[s], v[s], outs[layer, s], sp)
                hb.h2o_cache_snapshot(c.handle, snaps[layer, s], None, sp)

    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        restore_all(stream)
        generate(stream)
        stream.synchronize()
        ref_out, ref_snaps = outs.clone(), snaps.clone()
        ref_state = [[x.clone() for x in c.views()] for c in caches]
        # the eager run against the oracle, every layer, head and step
        total = parity.DecodeStats()
        for layer in range(L):
            q, kk, v = (x.cpu() for x in steps_in[layer])
            o_l, s_l = ref_out[layer].cpu(), ref_snaps[layer].cpu()
            for (b, h) in heads:
                total.merge(parity.check_head_decode(oracles[layer][(b, h)], q[:, b, h], kk[:, b, h], v[:, b, h],
                                                     o_l[:, b, h], s_l[:, b, h], R, parity.OUT_TOL[dtype]))
        assert total.head_steps == L * B * Hh * T and total.excused == 0
        # captured once (t is a launch argument: the graph holds these T steps from this start)
        restore_all(stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            generate(stream)
        for rep in range(3):
            restore_all(stream)                            # eager work between replays
            outs.zero_(); snaps.zero_()
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            assert torch.equal(outs, ref_out), "replay %d: outputs differ from the eager run" % rep
            assert torch.equal(snaps, ref_snaps), "replay %d: kept positions differ from the eager run" % rep
            for c, ref in zip(caches, ref_state):
                for x, y in zip(c.views(), ref):
                    assert torch.equal(x, y), "replay %d: a layer's cache differs from the eager run" % rep
    for c in caches:
        c.close()
