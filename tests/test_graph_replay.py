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
