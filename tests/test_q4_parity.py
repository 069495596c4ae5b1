"""GPU parity of the 4-bit cache (group-wise min-max codes along the head
dimension) against the CPU oracle, through the C ABI: the codes a row gets when
it enters the cache are compared bit for bit, the generation step over stored
codes to the tolerances of the unquantised step."""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead, map_heads
from tests import parity

pytestmark = pytest.mark.gpu

torch_dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def check_stored_rows(hb, cache, oracles, d):
    """Every occupied slot holds exactly the oracle's codes and (scale, min) pairs
    of the token at that position.  Returns the number of rows compared."""
    Kq, Vq, _, pos = (x.cpu() for x in cache.views())
    kc, kp = hb.unpack_q4_rows(Kq, d)
    vc, vp = hb.unpack_q4_rows(Vq, d)
    kc, kp, vc, vp, pos = kc.numpy(), kp.numpy(), vc.numpy(), vp.numpy(), pos.numpy()
    rows = 0
    for (b, h), o in oracles.items():
        assert set(pos[b, h][pos[b, h] >= 0].tolist()) == set(o.resident()[0].tolist())
        for s in np.flatnonzero(pos[b, h] >= 0):
            rk, rkp, rv, rvp = o.token_codes(int(pos[b, h, s]))
            where = "head (%d, %d) slot %d position %d" % (b, h, s, pos[b, h, s])
            assert np.array_equal(kc[b, h, s], rk), "key codes differ: " + where
            assert np.array_equal(vc[b, h, s], rv), "value codes differ: " + where
            assert np.array_equal(kp[b, h, s].view(np.uint32), rkp.view(np.uint32)), "key (scale, min): " + where
            assert np.array_equal(vp[b, h, s].view(np.uint32), rvp.view(np.uint32)), "value (scale, min): " + where
            rows += 1
    return rows


def q4_case(B, Hh, d, n, T, heavy, recent, dtype, sigma, seed, rank=0, prompt="select", sample=None):
    """Prompt phase, then T generation steps on a 4-bit cache.  prompt = "select":
    the device compresses on the ORACLE's binary32 scores (bit-exact index work,
    both sides start from the same set); "scores": the device's own prompt scoring."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    k = heavy + recent
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    if sample is not None:                       # full-size runs: the oracle follows a sample of the heads
        assert prompt != "select"
        rng = np.random.default_rng(seed)
        heads = [heads[i] for i in sorted(rng.choice(len(heads), size=sample, replace=False))]
    scale = parity.oracle_scale(d)
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev, rank=rank, kv_bits=4)
    if n > 0:
        Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
        oracles, cols = parity.oracle_prefill_heads(Q.cpu(), K.cpu(), V.cpu(), heads, heavy, recent, scale,
                                                     n + T, policy=rank, kv_bits=4)
        if prompt == "select":
            score = torch.empty((B, Hh, n), dtype=torch.float32)
            for (b, h) in heads:
                score[b, h] = torch.from_numpy(cols[(b, h)].astype(np.float32))
            cache.prefill_select(K, V, score.to(dev))
        elif prompt == "attention":
            need = hb.h2o_prefill_attention_workspace_bytes(cache.cfg, n)
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
            hb.h2o_prefill_attention_scores(cache.handle, Q, K, V, n, ws, need, torch.empty_like(Q))
        else:
            cache.prefill_scores(Q, K, V)
        torch.cuda.synchronize()
        if prompt != "select":
            # the device's own column sums: a token at the selection threshold may change sides
            # (only there: every token that changes sides lies within the selection band of the
            # oracle's threshold, and the oracle then adopts the device's set, re-quantising the
            # rows that enter; no head is dropped)
            from tests.test_prefill_parity import SELECT_RTOL
            pos = cache.views()[3].cpu().numpy()
            swapped = sum(parity.adopt_kept_set(oracles[bh], pos[bh], n - 1, recent, rank, SELECT_RTOL)
                          for bh in heads)
            assert swapped <= max(1, len(heads) * k // 1000)
        rows = check_stored_rows(hb, cache, oracles, d)
        assert rows == len(heads) * min(n, k)
    else:
        oracles = {bh: OracleHead(d, heavy, recent, scale, score_f32=True, cap=T, policy=rank, kv_bits=4)
                   for bh in heads}
    if T == 0:
        cache.close()
        return None
    qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, sigma, dev, seed)
    outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs)
    pos_f, acc_f = (x.cpu() for x in cache.snapshot())
    qs, ks, vs = qs.cpu(), ks.cpu(), vs.cpu()

    # scores seeded by the device's own column sums carry that pass's tolerance, and so
    # does the order of two candidates whose values are closer than twice that
    from tests.test_prefill_parity import SELECT_RTOL
    band = parity.NEAR_TIE if prompt == "select" or n == 0 else SELECT_RTOL

    def one(bh):
        b, h = bh
        st = parity.check_head_decode(oracles[bh], qs[:, b, h], ks[:, b, h], vs[:, b, h], outs[:, b, h],
                                      snaps[:, b, h], recent, parity.OUT_TOL[dtype], policy=rank, band=band)
        parity.check_final_scores(oracles[bh], pos_f[b, h], acc_f[b, h], st)
        return st
    res, _ = map_heads(one, heads)
    total = parity.DecodeStats()
    for st in res:
        total.merge(st)
    rows = check_stored_rows(hb, cache, oracles, d)      # tokens written by the steps included
    print("\n[4-bit cache] B=%d Hh=%d d=%d n=%d T=%d H=%d R=%d %s rank=%d: head-steps %d, excused %d, "
          "out l2 %.2e linf %.2e, score mismatches %d (max rel %.1e), stored rows compared %d"
          % (B, Hh, d, n, T, heavy, recent, str(dtype).split(".")[-1], rank, total.head_steps,
             total.excused, total.max_out_l2, total.max_out_linf, total.score_mismatch,
             total.max_score_rel, rows), flush=True)
    assert total.excused + total.excused_band <= max(1, total.head_steps // 1000)
    # scores seeded by the device's own column sums carry that pass's tolerance
    from tests.test_prefill_parity import COLSUM_RTOL
    assert total.max_score_rel <= (1e-6 if prompt == "select" else COLSUM_RTOL)
    cache.close()
    return total


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n,heavy,recent", [(300, 40, 40), (50, 64, 64), (1000, 300, 212)])
def test_q4_rows_entering_the_cache_are_quantised_bit_exactly(dt, d, n, heavy, recent):
    q4_case(2, 3, d, n, 0, heavy, recent, torch_dt[dt], 1.0, 61)


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
def test_q4_decode_small(dt, d):
    q4_case(2, 3, d, 96, 40, 24, 24, torch_dt[dt], 1.0, 62)


@pytest.mark.parametrize("n,T,heavy,recent", [
    (0, 150, 50, 50),          # from an empty cache: fills up, then evicts
    (700, 64, 205, 205),       # the OPT-6.7B-shaped budget
    (300, 48, 128, 128),       # exactly the 256 slots of the four-wave kernel
    (300, 48, 129, 128),       # one more
    (900, 32, 256, 256),       # exactly 512
    (900, 24, 257, 256),       # 513: two slots per lane
    (400, 40, 0, 100),         # window only
    (400, 40, 100, 0),         # heavy hitters only: the new token competes
])
def test_q4_decode_budgets(n, T, heavy, recent):
    q4_case(1, 4, 128, n, T, heavy, recent, torch.float16, 1.0, 63)


@pytest.mark.parametrize("heavy,recent", [(1, 0), (0, 1), (1, 1), (3, 2)])
def test_q4_smallest_budgets(heavy, recent):
    q4_case(1, 3, 128, 9, 14, heavy, recent, torch.float16, 1.0, 72)
    q4_case(1, 3, 64, 0, 10, heavy, recent, torch.bfloat16, 1.0, 73)


def test_q4_decode_large_budgets():
    q4_case(1, 2, 128, 1500, 16, 512, 512, torch.float16, 1.0, 64)       # 1024
    q4_case(1, 2, 128, 2300, 12, 1024, 1024, torch.bfloat16, 1.0, 65)    # the largest supported
    q4_case(1, 2, 64, 2300, 12, 1024, 1024, torch.float16, 1.0, 66)


def test_q4_decode_averaged_ranking():
    q4_case(2, 2, 128, 400, 64, 60, 60, torch.float16, 1.0, 67, rank=1)


def test_q4_end_to_end_with_device_prompt_scoring():
    q4_case(2, 4, 128, 1024, 32, 103, 102, torch.float16, 1.0, 68, prompt="scores")


def test_q4_end_to_end_with_attention_based_prompt_phase():
    q4_case(2, 4, 128, 1024, 16, 103, 102, torch.bfloat16, 1.0, 70, prompt="attention")


def test_q4_full_size_layer_workload_sampled():
    """The OPT-6.7B-shaped layer (batch 16, 32 heads, prompt 2048, budget 205 + 205, f16) on a 4-bit
    cache: device prompt scoring, 64 generation steps, 12 sampled heads."""
    q4_case(16, 32, 128, 2048, 64, 205, 205, torch.float16, 1.0, 71, prompt="scores", sample=12)


def test_q4_long_run():
    """Several cache turnovers: every slot is rewritten many times by quantised new tokens."""
    q4_case(1, 4, 128, 100, 600, 20, 20, torch.float16, 1.0, 74)
    q4_case(1, 2, 64, 0, 500, 33, 31, torch.bfloat16, 1.25, 75)


def test_q4_heavy_tailed_keys():
    q4_case(1, 4, 128, 500, 48, 50, 50, torch.float16, 1.5, 69)


def test_q4_restore_round_trip_and_unsupported_calls():
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, dtype = 1, 2, 128, torch.float16
    Q, K, V = synth.make_prompt(B, Hh, 200, d, dtype, 1.0, dev, 5)
    a = hb.H2OCache(B, Hh, d, 30, 30, dtype, device=dev, kv_bits=4)
    a.prefill_scores(Q, K, V)
    Ka, Va, acc, pos = (x.clone() for x in a.views())
    b = hb.H2OCache(B, Hh, d, 30, 30, dtype, device=dev, kv_bits=4)
    b.restore(Ka, Va, acc, pos, 200)
    qs, ks, vs = synth.make_steps(B, Hh, d, 6, dtype, 1.0, dev, 5)
    oa = torch.empty((B, Hh, d), dtype=dtype, device=dev)
    ob = torch.empty_like(oa)
    for s in range(6):
        a.decode_step(qs[s], ks[s], vs[s], oa)
        b.decode_step(qs[s], ks[s], vs[s], ob)
        assert torch.equal(oa, ob)
    for x, y in zip(a.views(), b.views()):
        assert torch.equal(x, y)
    with pytest.raises(hb.H2OError) as ei:
        a.prefill_chunk(Q[:, :, :8].contiguous(), K[:, :, :8].contiguous(), V[:, :, :8].contiguous())
    assert ei.value.status == hb.H2O_EUNSUPPORTED
    a.close(); b.close()
