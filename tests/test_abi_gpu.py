"""Error paths and state machine of the C ABI with a device present."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu


def test_state_machine_and_errors():
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n = 1, 2, 64, 96
    Q, K, V = synth.make_prompt(B, Hh, n, d, torch.float16, 1.0, dev, 1)
    cache = hb.H2OCache(B, Hh, d, 8, 8, torch.float16, device=dev)
    assert cache.tokens_seen == 0
    cache.prefill_scores(Q, K, V)
    assert cache.tokens_seen == n
    with pytest.raises(hb.H2OError) as e:                 # second prompt without reset
        cache.prefill_scores(Q, K, V)
    assert e.value.status == hb.H2O_ESTATE
    with pytest.raises(hb.H2OError) as e:
        cache.prefill_select(K, V, torch.zeros((B, Hh, n), device=dev))
    assert e.value.status == hb.H2O_ESTATE
    cache.reset()
    assert cache.tokens_seen == 0
    pos, acc = cache.snapshot()
    torch.cuda.synchronize()
    assert torch.all(pos == -1) and torch.all(acc == 0)
    cache.prefill_scores(Q, K, V)
    # misaligned step pointer
    q = torch.zeros(B * Hh * d + 8, dtype=torch.float16, device=dev)
    out = torch.empty((B, Hh, d), dtype=torch.float16, device=dev)
    with pytest.raises(hb.H2OError) as e:
        hb.h2o_decode_step(cache.handle, q.data_ptr() + 2, q, q, out)
    assert e.value.status == hb.H2O_EINVAL
    assert cache.tokens_seen == n
    # workspace too small
    ws = torch.empty(64, dtype=torch.uint8, device=dev)
    cache.reset()
    with pytest.raises(hb.H2OError) as e:
        hb.h2o_prefill_scores(cache.handle, Q, K, V, n, ws, ws.numel())
    assert e.value.status == hb.H2O_ENOMEM
    # cache memory too small
    mem = torch.empty(1024, dtype=torch.uint8, device=dev)
    with pytest.raises(hb.H2OError) as e:
        hb.h2o_cache_init(cache.cfg, mem, mem.numel())
    assert e.value.status == hb.H2O_ENOMEM
    torch.cuda.synchronize()
    cache.close()


def test_prefill_then_decode_smoke_invariants():
    """Device-only properties that hold at any size: cache stays full, the recent
    window is resident, scores never exceed the number of queries seen and the
    kept scores sum to at most that number."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, T, H, R = 2, 4, 128, 512, 40, 32, 32
    Q, K, V = synth.make_prompt(B, Hh, n, d, torch.float16, 1.0, dev, 4)
    qs, ks, vs = synth.make_steps(B, Hh, d, T, torch.float16, 1.0, dev, 4)
    cache = hb.H2OCache(B, Hh, d, H, R, torch.float16, device=dev)
    cache.prefill_scores(Q, K, V)
    out = torch.empty((B, Hh, d), dtype=torch.float16, device=dev)
    for s in range(T):
        cache.decode_step(qs[s], ks[s], vs[s], out)
        pos, acc = cache.snapshot()
        torch.cuda.synchronize()
        t = n + s + 1
        assert torch.all(pos >= 0) and torch.all(pos < t)
        srt = pos.sort(dim=-1).values
        assert torch.all(srt[..., 1:] > srt[..., :-1])
        assert torch.all(srt[..., -R:] == torch.arange(t - R, t, device=dev))
        assert torch.all(acc >= 0) and torch.all(acc <= (t - pos).float() * (1 + 1e-5))
        assert torch.all(acc.sum(-1) <= t * (1 + 1e-5))
        assert torch.all(torch.isfinite(out.float()))
    cache.close()
