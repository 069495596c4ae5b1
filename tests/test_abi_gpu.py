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


def test_validate_flags_inconsistent_restored_states():
    """h2o_cache_validate: states the library produced pass; a restored state with a hole in
    the occupied prefix, an occupied slot beyond it, a position out of range, a duplicate
    position or a negative / non-finite score is flagged per head, and restore(validate=True)
    raises for it.  (Nothing is stepped on the bad states.)"""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, H, R = 2, 3, 64, 300, 20, 20
    k = H + R
    Q, K, V = synth.make_prompt(B, Hh, n, d, torch.float16, 1.0, dev, 8)
    qs, ks, vs = synth.make_steps(B, Hh, d, 5, torch.float16, 1.0, dev, 8)
    good = hb.H2OCache(B, Hh, d, H, R, torch.float16, device=dev)
    assert not bool(good.validate().any())                        # empty cache
    good.prefill_scores(Q, K, V)
    out = torch.empty((B, Hh, d), dtype=torch.float16, device=dev)
    for s in range(5):
        good.decode_step(qs[s], ks[s], vs[s], out)
    assert not bool(good.validate().any())                        # after prompt + steps
    Kc, Vc, acc, pos = (x.clone() for x in good.views())
    t = good.tokens_seen

    def flags_of(mut, tokens_seen=t):
        a, p = acc.clone(), pos.clone()
        mut(a, p)
        c = hb.H2OCache(B, Hh, d, H, R, torch.float16, device=dev)
        c.restore(Kc, Vc, a, p, tokens_seen)
        f = c.validate().cpu()
        with pytest.raises(ValueError):
            c.restore(Kc, Vc, a, p, tokens_seen, validate=True)
        c.close()
        return f

    def hole(a, p): p[0, 1, 7] = -1
    def dup(a, p): p[1, 2, 3] = p[1, 2, 30]
    def high(a, p): p[0, 0, 5] = t
    def neg(a, p): a[1, 0, 0] = -0.0
    def nan(a, p): a[0, 2, 39] = float("nan")

    f = flags_of(hole)
    assert int(f[0, 1]) == hb.H2O_BAD_HOLE and int(f.sum()) == hb.H2O_BAD_HOLE
    f = flags_of(dup)
    assert int(f[1, 2]) == hb.H2O_BAD_DUPLICATE and int(f.sum()) == hb.H2O_BAD_DUPLICATE
    f = flags_of(high)
    assert int(f[0, 0]) == hb.H2O_BAD_RANGE and int(f.sum()) == hb.H2O_BAD_RANGE
    f = flags_of(neg)
    assert int(f[1, 0]) == hb.H2O_BAD_SCORE and int(f.sum()) == hb.H2O_BAD_SCORE
    f = flags_of(nan)
    assert int(f[0, 2]) == hb.H2O_BAD_SCORE
    # a cache that claims fewer tokens than it holds: slots beyond min(t, k) are occupied
    f = flags_of(lambda a, p: None, tokens_seen=k - 4)
    assert bool((f & hb.H2O_BAD_BEYOND).all())
    # the good state restores cleanly and steps on
    c = hb.H2OCache(B, Hh, d, H, R, torch.float16, device=dev)
    c.restore(Kc, Vc, acc, pos, t, validate=True)
    c.decode_step(qs[0], ks[0], vs[0], out)
    torch.cuda.synchronize()
    # the class refuses tensors of the wrong shape or type on the host
    with pytest.raises(ValueError):
        c.decode_step(qs[0][:, :2], ks[0], vs[0], out)
    with pytest.raises(ValueError):
        c.decode_step(qs[0].float(), ks[0], vs[0], out)
    with pytest.raises(ValueError):
        c.restore(Kc, Vc, acc[:, :, :-1].contiguous(), pos, t)
    c.close(); good.close()
