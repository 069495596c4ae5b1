"""GPU parity of the pattern-protected variants (a strided or fixed sparse-attention
pattern in the recent window's place, combined with heavy hitters: Sec. 5.2, Table 2)
against the CPU oracle, through the C ABI: the prompt compression bit for bit on given
scores, the generation step on every kernel, the chunked prompt, and the whole path with
the device's own prompt scoring."""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead, map_heads
from tests import parity

pytestmark = pytest.mark.gpu

torch_dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
MODE = {"strided": 1, "fixed": 2}


def select_case(B, Hh, d, n, heavy, recent, pattern, score, dtype=torch.float16, rank=0, seed=5, kv_bits=0):
    """Device compression of given scores under a pattern against the oracle's: kept positions in
    slot order, stored scores, copied rows."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    _, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, seed)
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev, rank=rank, kv_bits=kv_bits,
                        protect=MODE[pattern[0]], stride=pattern[1])
    cache.prefill_select(K, V, torch.from_numpy(score.astype(np.float32)).to(dev))
    pos, acc = (x.cpu() for x in cache.snapshot())
    assert not bool(cache.validate().cpu().any())
    Kc, Vc = (x.cpu() for x in cache.kv_views())
    Kh, Vh = K.cpu(), V.cpu()
    sizes = []
    for b in range(B):
        for h in range(Hh):
            o = OracleHead(d, heavy, recent, 1.0, score_f32=True, cap=n, policy=rank,
                           protect=MODE[pattern[0]], stride=pattern[1])
            o.load_and_select(parity.host64(Kh[b, h]), parity.host64(Vh[b, h]),
                              score[b, h].astype(np.float32).astype(np.float64))
            rp, rs = o.resident()
            c = len(rp)
            sizes.append(c)
            assert pos[b, h, :c].tolist() == rp.tolist(), "kept positions differ (b=%d h=%d)" % (b, h)
            assert torch.all(pos[b, h, c:] == -1)
            assert np.array_equal(acc[b, h, :c].double().numpy(), rs)
            if kv_bits == 0:
                idx = torch.from_numpy(rp.astype(np.int64))
                assert torch.equal(Kc[b, h, :c].view(torch.uint8), Kh[b, h, idx].view(torch.uint8))
                assert torch.equal(Vc[b, h, :c].view(torch.uint8), Vh[b, h, idx].view(torch.uint8))
    cache.close()
    return sizes


@pytest.mark.parametrize("kind", ["random", "ties"])
@pytest.mark.parametrize("n,heavy,recent,pattern", [
    (300, 64, 8, ("strided", 16)),      # 8 + 18 covered, 46 of the others kept
    (300, 64, 8, ("fixed", 32)),        # the last block's start + 8 summary columns per block
    (1000, 103, 16, ("strided", 7)),    # many strided positions
    (1000, 30, 12, ("fixed", 16)),      # 12 of every 16 positions covered: more than the budget -> the best covered
    (4096, 410, 409, ("strided", 64)),
    (4096, 410, 64, ("fixed", 128)),
    (200, 0, 24, ("strided", 5)),       # no heavy part: covered entries only as far as the budget goes
    (260, 16, 0, ("strided", 4)),       # no band: the period alone
    (50, 40, 30, ("fixed", 8)),         # prompt shorter than the budget: everything kept
    (9000, 2048, 2048, ("fixed", 4096)),
])
def test_pattern_select_gather_exact(n, heavy, recent, pattern, kind):
    rng = np.random.default_rng(n + heavy + len(kind))
    B, Hh = 2, 2
    score = rng.random((B, Hh, n)) * 5 if kind == "random" else np.round(rng.random((B, Hh, n)) * 6) / 4
    sizes = select_case(B, Hh, 128, n, heavy, recent, pattern, score)
    assert all(c == min(n, heavy + recent) for c in sizes)


def test_pattern_select_other_rankings_and_storage():
    rng = np.random.default_rng(3)
    score = rng.random((2, 2, 700)) * 3
    select_case(2, 2, 128, 700, 50, 10, ("strided", 9), score, rank=1)
    select_case(2, 2, 64, 700, 50, 10, ("fixed", 25), score, dtype=torch.bfloat16, rank=1)
    select_case(2, 2, 64, 700, 50, 10, ("fixed", 25), score, dtype=torch.float32)
    select_case(2, 2, 128, 700, 50, 10, ("strided", 9), score, kv_bits=4)


def pattern_decode_case(B, Hh, d, n, T, heavy, recent, pattern, dtype, seed, rank=0, kv_bits=0, sigma=1.0):
    """Prompt compressed on the oracle's scores (bit-exact index work on both sides), then T steps
    compared step by step: kept sets (1e-6 near-tie rule), outputs, final scores."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    scale = parity.oracle_scale(d)
    mode, stride = MODE[pattern[0]], pattern[1]
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev, rank=rank, kv_bits=kv_bits,
                        protect=mode, stride=stride)
    mk = lambda: OracleHead(d, heavy, recent, scale, score_f32=True, cap=n + T, policy=rank, kv_bits=kv_bits,
                            protect=mode, stride=stride)
    oracles = {}
    if n > 0:
        Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
        Qh, Kh, Vh = Q.cpu(), K.cpu(), V.cpu()

        def pre(bh):
            o = mk()
            col, _ = o.prefill(parity.host64(Qh[bh]), parity.host64(Kh[bh]), parity.host64(Vh[bh]))
            return o, col
        res, _ = map_heads(pre, heads)
        score = torch.empty((B, Hh, n), dtype=torch.float32)
        for bh, (o, col) in zip(heads, res):
            oracles[bh] = o
            score[bh] = torch.from_numpy(col.astype(np.float32))
        cache.prefill_select(K, V, score.to(dev))
        pos0 = cache.snapshot()[0].cpu().numpy()
        for bh in heads:
            assert sorted(pos0[bh][pos0[bh] >= 0].tolist()) == oracles[bh].resident()[0].tolist()
    else:
        oracles = {bh: mk() for bh in heads}
    qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, sigma, dev, seed)
    outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs)
    pos_f, acc_f = (x.cpu() for x in cache.snapshot())
    assert not bool(cache.validate().cpu().any())
    qh, kh, vh = qs.cpu(), ks.cpu(), vs.cpu()
    # (parity.check_head_decode tests whether the device's choice was a legal candidate with the
    # window rule; under a pattern legality is the pattern's, so the per-step check is spelled out)

    def one(bh):
        b, h = bh
        o = oracles[bh]
        st = parity.DecodeStats()
        for s in range(T):
            t = o.t
            r = o.decode(parity.host64(qh[s, b, h]), parity.host64(kh[s, b, h]), parity.host64(vh[s, b, h]))
            st.head_steps += 1
            f_l2, f_el, l2, li = (float(x) for x in parity.output_error(outs[s, b, h].double().numpy(), r.out, dtype))
            st.max_out_l2, st.max_out_linf = max(st.max_out_l2, l2), max(st.max_out_linf, li)
            assert f_l2 <= 1.0 and f_el <= 1.0, "output mismatch at step %d: %.3e %.3e" % (s, l2, li)
            row = snaps[s, b, h].numpy()
            got = sorted(row[row >= 0].tolist())
            ref = o.resident()[0].tolist()
            if got != ref:
                only_ref, only_gpu = set(ref) - set(got), set(got) - set(ref)
                assert len(only_ref) == 1 and only_gpu == {r.evicted}
                g = next(iter(only_ref))
                sg = parity.rank_of(o, g, t, rank)
                assert (sg - r.lowest) <= parity.NEAR_TIE * max(abs(sg), abs(r.lowest)), \
                    "step %d: device evicted %d (%.9g), oracle %d (%.9g)" % (s, g, sg, r.evicted, r.lowest)
                o.resync(r.evicted, g)
                st.excused += 1
        parity.check_final_scores(o, pos_f[b, h], acc_f[b, h], st)
        return st
    res, _ = map_heads(one, heads)
    total = parity.DecodeStats()
    for st in res:
        total.merge(st)
    print("\n[pattern %s/%d] d=%d n=%d T=%d H=%d R=%d %s rank=%d bits=%d: head-steps %d, excused %d, out l2 %.2e "
          "linf %.2e, scores not bit-equal %d" % (pattern[0], pattern[1], d, n, T, heavy, recent,
                                                  str(dtype).split(".")[-1], rank, kv_bits or 16, total.head_steps,
                                                  total.excused, total.max_out_l2, total.max_out_linf,
                                                  total.score_mismatch), flush=True)
    assert total.excused <= max(1, total.head_steps // 1000)
    assert total.max_score_rel <= 1e-6
    cache.close()
    return total


@pytest.mark.parametrize("pattern", [("strided", 8), ("fixed", 32)])
@pytest.mark.parametrize("dt,d,n,T,heavy,recent", [
    ("f16", 128, 96, 60, 13, 10),       # four waves, a few rounds
    ("f16", 128, 400, 70, 103, 102),    # four waves, 13 rounds
    ("bf16", 128, 700, 40, 205, 205),   # eight waves
    ("f16", 128, 900, 30, 300, 333),    # chunked
    ("f32", 64, 200, 50, 24, 8),
    ("bf16", 64, 0, 120, 20, 12),       # from an empty cache
])
def test_pattern_decode_every_kernel(dt, d, n, T, heavy, recent, pattern):
    if pattern[0] == "fixed" and recent > pattern[1]:
        pattern = ("fixed", 512)             # blocks wide enough for that many summary columns
    pattern_decode_case(2, 2, d, n, T, heavy, recent, pattern, torch_dt[dt], 81)


@pytest.mark.parametrize("pattern", [("strided", 1), ("fixed", 1000)])
def test_pattern_covers_everything_so_protection_is_void(pattern):
    """A strided period of 1, and one fixed block over the whole text: no cached token is ever
    outside the pattern, so on every step the lowest score of all (the new token aside) goes."""
    pattern_decode_case(1, 3, 128, 100, 80, 10, 30, pattern, torch.float16, 82)
    pattern_decode_case(1, 2, 128, 900, 20, 300, 333, pattern, torch.float16, 83)      # chunked kernel


@pytest.mark.parametrize("pattern", [("strided", 8), ("fixed", 32)])
def test_pattern_decode_averaged_ranking_and_4bit_cache(pattern):
    pattern_decode_case(2, 2, 128, 300, 60, 50, 16, pattern, torch.float16, 84, rank=1)
    pattern_decode_case(2, 2, 128, 300, 60, 50, 16, pattern, torch.float16, 85, kv_bits=4)
    pattern_decode_case(1, 2, 128, 900, 30, 257, 256, pattern, torch.bfloat16, 86, kv_bits=4)
    pattern_decode_case(1, 2, 64, 0, 90, 24, 8, pattern, torch.float32, 87, kv_bits=4, rank=1)


@pytest.mark.parametrize("pattern", [("strided", 6), ("fixed", 20)])
def test_pattern_exact_ties(pattern):
    """The constructed tie / zero-score inputs of tests/test_decode_ties.py under a pattern: the
    device must evict the oracle's position on every step."""
    from paper_2306_14048_amd import binding as hb
    from tests.test_decode_ties import crafted_inputs
    dev = torch.device("cuda:0")
    for (heavy, recent, d, dtype, kv_bits) in [(40, 10, 128, torch.float16, 0), (300, 12, 128, torch.float16, 0),
                                               (60, 10, 128, torch.float16, 4)]:
        k = heavy + recent
        n, T = k + 5, 150
        K, V, score, qs, ks, vs = crafted_inputs(1, 3, d, n, T, dtype, 500 + k)
        mode, stride = MODE[pattern[0]], pattern[1]
        cache = hb.H2OCache(1, 3, d, heavy, recent, dtype, device=dev, kv_bits=kv_bits, protect=mode, stride=stride)
        cache.prefill_select(K.to(dev), V.to(dev), torch.from_numpy(score).to(dev))
        outs, snaps = parity.run_gpu_decode(cache, qs.to(dev), ks.to(dev), vs.to(dev))
        tied = 0
        for h in range(3):
            o = OracleHead(d, heavy, recent, parity.oracle_scale(d), score_f32=True, cap=n + T, kv_bits=kv_bits,
                           protect=mode, stride=stride)
            o.load_and_select(parity.host64(K[0, h]), parity.host64(V[0, h]), score[0, h].astype(np.float64))
            for s in range(T):
                r = o.decode(parity.host64(qs[s, 0, h]), parity.host64(ks[s, 0, h]), parity.host64(vs[s, 0, h]))
                tied += int(r.evicted >= 0 and r.second == r.lowest)
                row = snaps[s, 0, h].numpy()
                assert sorted(row[row >= 0].tolist()) == o.resident()[0].tolist(), \
                    "head %d step %d: device and oracle evicted different tokens" % (h, s)
        assert tied > 20
        cache.close()


@pytest.mark.parametrize("pattern", [("strided", 16), ("fixed", 64)])
def test_pattern_whole_path_with_device_prompt_scoring_and_chunks(pattern):
    """h2o_prefill_scores and h2o_prefill_chunk under a pattern, then steps: kept sets equal to
    the oracle's (tokens at the selection threshold excepted, as in the window mode)."""
    from paper_2306_14048_amd import binding as hb, synth
    from tests.test_prefill_parity import COLSUM_RTOL, SELECT_RTOL
    dev = torch.device("cuda:0")
    B, Hh, d, n, T, heavy, recent, dtype = 2, 3, 128, 640, 30, 64, 16, torch.float16
    mode, stride = MODE[pattern[0]], pattern[1]
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    scale = parity.oracle_scale(d)
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 91)
    qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, 1.0, dev, 91)
    for chunks in ([n], [200, 300, 140]):
        cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev, protect=mode, stride=stride)
        oracles = {bh: OracleHead(d, heavy, recent, scale, score_f32=True, cap=n + T, protect=mode, stride=stride)
                   for bh in heads}
        c0 = 0
        for m in chunks:
            q, kk, v = (x[:, :, c0:c0 + m].contiguous() for x in (Q, K, V))
            if len(chunks) == 1:
                cache.prefill_scores(q, kk, v)
            else:
                cache.prefill_chunk(q, kk, v)
            pos = cache.snapshot()[0].cpu().numpy()
            for bh in heads:
                o = oracles[bh]
                if len(chunks) == 1:
                    o.prefill(parity.host64(q[bh]), parity.host64(kk[bh]), parity.host64(v[bh]))
                else:
                    o.prefill_chunk(parity.host64(q[bh]), parity.host64(kk[bh]), parity.host64(v[bh]))
                got = sorted(pos[bh][pos[bh] >= 0].tolist())
                ref = o.resident()[0].tolist()
                if got != ref:
                    # only tokens whose rank value ties the threshold within the score tolerance
                    t_last = c0 + m - 1
                    vals = [parity.rank_of(o, j, t_last, 0) for j in set(got) ^ set(ref)]
                    assert max(vals) - min(vals) <= SELECT_RTOL * max(vals)
                    for a, b_ in zip(sorted(set(got) - set(ref)), sorted(set(ref) - set(got))):
                        o.resync(a, b_)
            c0 += m
        outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs)
        for bh in heads:
            o = oracles[bh]
            for s in range(T):
                r = o.decode(parity.host64(qs[s][bh]), parity.host64(ks[s][bh]), parity.host64(vs[s][bh]))
                f_l2, f_el, _, _ = parity.output_error(outs[s][bh].double().numpy(), r.out, dtype)
                assert f_l2 <= 1.0 and f_el <= 1.0
                row = snaps[s][bh].numpy()
                got = sorted(row[row >= 0].tolist())
                if got != o.resident()[0].tolist():
                    g = (set(o.resident()[0].tolist()) - set(got)).pop()
                    sg = parity.rank_of(o, g, o.t - 1, 0)
                    assert (sg - r.lowest) <= SELECT_RTOL * max(abs(sg), abs(r.lowest))
                    o.resync(r.evicted, g)
        cache.close()
