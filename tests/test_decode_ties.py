"""Eviction on exact ties, zero scores and subnormal scores, on the device.

Definition 4.3 / Algorithm 1 evict the arg-max of F_score(S minus v), i.e. the
token with the smallest accumulated score; the paper does not say which of
several equal scores goes, the reading taken is the smallest (score, position)
pair.  Random inputs never produce an exact tie, so these cases construct them:

  * every cached key is either 0 ("live": logit 0 against any query) or a
    constant -256 row ("dead": logit about -2900 against the all-ones query, so
    its probability is exactly 0 in fp64 and in binary32);
  * the prompt scores are drawn from a handful of binary32 values: 0.0, two
    subnormals, the smallest normal number, and a few ordinary values, so that
    many tokens share a score bit for bit;
  * every step's query is the all-ones vector: all live tokens gain the same
    probability, dead tokens gain exactly 0 and keep their zero / subnormal
    scores, so groups of equal scores stay equal step after step and almost
    every eviction is decided by the position alone.

Both sides start from the same state: the prompt compression on the given scores
(bit-exact index work on both sides, itself tie-laden), then T steps.  The
device has to evict the oracle's position on EVERY step (no excuse is accepted
here: an exact tie broken the other way would count as a near tie in the
ordinary parity rule).  Budgets are chosen to reach every step kernel: four- and
eight-wave register-resident, chunked, and the 4-bit cache's; both rankings.
"""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead, map_heads
from tests import parity

pytestmark = pytest.mark.gpu

torch_dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
SUB_A = float(np.float32(1e-42))          # binary32 subnormals
SUB_B = float(np.float32(3e-39))
MIN_NORMAL = float(np.float32(2.0 ** -126))
DEAD = -256.0


def crafted_inputs(B, Hh, d, n, T, dtype, seed, dead_frac=0.35):
    """Prompt K, V, scores and step q, k, v (host tensors) as described above."""
    rng = np.random.default_rng(seed)
    g = torch.Generator().manual_seed(seed)
    dead = torch.from_numpy(rng.random((B, Hh, n)) < dead_frac)
    K = torch.zeros((B, Hh, n, d), dtype=dtype)
    K[dead] = DEAD
    V = torch.randn((B, Hh, n, d), generator=g).to(dtype)
    dead_scores = np.array([0.0, 0.0, SUB_A, SUB_A, SUB_B, MIN_NORMAL], dtype=np.float32)
    live_scores = np.array([0.0, 0.5, 0.5, 0.5, 0.75, 1.0, 1.0, 2.5], dtype=np.float32)
    score = np.where(dead.numpy(), dead_scores[rng.integers(0, len(dead_scores), (B, Hh, n))],
                     live_scores[rng.integers(0, len(live_scores), (B, Hh, n))]).astype(np.float32)
    qs = torch.ones((T, B, Hh, d), dtype=dtype)
    ks = torch.zeros((T, B, Hh, d), dtype=dtype)
    ks[torch.from_numpy(rng.random((T, B, Hh)) < 0.25)] = DEAD      # some new tokens are dead too
    vs = torch.randn((T, B, Hh, d), generator=g).to(dtype)
    return K, V, score, qs, ks, vs


def tie_case(B, Hh, d, n, T, heavy, recent, dtype, seed, rank=0, kv_bits=0):
    from paper_2306_14048_amd import binding as hb
    dev = torch.device("cuda:0")
    k = heavy + recent
    K, V, score, qs, ks, vs = crafted_inputs(B, Hh, d, n, T, dtype, seed)
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    scale = parity.oracle_scale(d)
    assert DEAD * d * scale < -1500.0            # exp() of it is 0 in fp64

    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev, rank=rank, kv_bits=kv_bits)
    cache.prefill_select(K.to(dev), V.to(dev), torch.from_numpy(score).to(dev))
    pos0 = cache.snapshot()[0].cpu().numpy()
    oracles = {}
    for (b, h) in heads:
        o = OracleHead(d, heavy, recent, scale, score_f32=True, cap=n + T, policy=rank, kv_bits=kv_bits)
        o.load_and_select(parity.host64(K[b, h]), parity.host64(V[b, h]), score[b, h].astype(np.float64))
        assert sorted(pos0[b, h][pos0[b, h] >= 0].tolist()) == o.resident()[0].tolist(), \
            "prompt compression differs (b=%d h=%d)" % (b, h)
        oracles[(b, h)] = o

    qd, kd, vd = qs.to(dev), ks.to(dev), vs.to(dev)
    outs, snaps = parity.run_gpu_decode(cache, qd, kd, vd)
    pos_f, acc_f = (x.cpu() for x in cache.snapshot())

    def one(bh):
        b, h = bh
        st = parity.check_head_decode(oracles[bh], qs[:, b, h], ks[:, b, h], vs[:, b, h], outs[:, b, h],
                                      snaps[:, b, h], recent, parity.OUT_TOL[dtype], policy=rank)
        parity.check_final_scores(oracles[bh], pos_f[b, h], acc_f[b, h], st)
        return st
    res, _ = map_heads(one, heads)
    total = parity.DecodeStats()
    for st in res:
        total.merge(st)
    print("\n[ties] d=%d n=%d T=%d H=%d R=%d %s rank=%d bits=%d: head-steps %d, exactly tied evictions %d, "
          "zero-score evictions %d, subnormal-score evictions %d, device chose differently %d, scores not "
          "bit-equal %d" % (d, n, T, heavy, recent, str(dtype).split(".")[-1], rank, kv_bits or 16,
                            total.head_steps, total.exact_tied_steps, total.zero_low_steps,
                            total.subnormal_low_steps, total.excused, total.score_mismatch), flush=True)
    assert total.excused == 0, "the device broke %d exact ties differently from (score, position) order" \
        % total.excused
    assert total.score_mismatch == 0
    cache.close()
    return total


# (heavy, recent, d, dtype): which step kernel the budget reaches
KERNELS = [
    (20, 12, 128, "f16"),      # register-resident, four waves, 2 rounds
    (103, 102, 128, "f16"),    # register-resident, four waves, 13 rounds (the OPT-30B-shaped budget)
    (205, 205, 128, "f16"),    # register-resident, eight waves (the OPT-6.7B-shaped budget)
    (230, 230, 128, "bf16"),   # register-resident, eight waves, 15 rounds
    (300, 333, 128, "f16"),    # chunked
    (40, 24, 64, "f32"),       # binary32 elements, d = 64
    (500, 524, 64, "bf16"),    # chunked, d = 64
    (33, 0, 128, "f16"),       # no recent window: the new token competes (and ties) as well
    (0, 17, 64, "f16"),        # window only
]


@pytest.mark.parametrize("rank", [0, 1])
@pytest.mark.parametrize("heavy,recent,d,dt", KERNELS)
def test_exact_ties_and_zero_scores(heavy, recent, d, dt, rank):
    k = heavy + recent
    T = min(3 * k // 2 + 40, 400)
    # the prompt is barely longer than the budget, so tokens of every score value are cached
    st = tie_case(1, 3, d, k + 5, T, heavy, recent, torch_dt[dt], 900 + k, rank=rank)
    # the case really exercises what it is for (counts are the oracle's, fixed by the seed)
    assert st.zero_low_steps > 0 and st.subnormal_low_steps > 0
    assert st.exact_tied_steps > 0 or heavy == 0


@pytest.mark.parametrize("rank", [0, 1])
@pytest.mark.parametrize("heavy,recent,d,dt", [(20, 12, 128, "f16"), (103, 102, 128, "f16"),
                                               (205, 205, 128, "f16"), (300, 333, 128, "bf16"),
                                               (513, 512, 128, "f16"), (40, 24, 64, "f32"), (33, 0, 64, "f16")])
def test_exact_ties_and_zero_scores_q4(heavy, recent, d, dt, rank):
    k = heavy + recent
    T = min(3 * k // 2 + 40, 300)
    st = tie_case(1, 3, d, k + 5, T, heavy, recent, torch_dt[dt], 1900 + k, rank=rank, kv_bits=4)
    assert st.zero_low_steps > 0 and st.subnormal_low_steps > 0 and st.exact_tied_steps > 0


@pytest.mark.parametrize("heavy,recent,dt,d", [(16, 16, "f16", 128), (103, 102, "bf16", 128), (205, 205, "f16", 128),
                                               (300, 333, "f16", 128), (24, 40, "f32", 64)])
def test_equal_logits_closed_form_through_the_device_prompt_phase(heavy, recent, dt, d):
    """All logits equal (Q = 0): column sum of token j (1-based) is H_n - H_{j-1}, strictly
    decreasing, so the prompt phase keeps the first `heavy` and the last `recent` tokens; in
    every later step (q = 0) each cached token gains 1 / (k + 1), the oldest token of the
    window has the smallest score of all candidates when it leaves the window and is the one
    evicted: the kept set stays {first heavy} + {last recent} for ever.  Device prompt
    scoring + device steps, against the closed form and the oracle."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    dtype = torch_dt[dt]
    B, Hh, n, T = 1, 3, heavy + recent + 150, 60
    k = heavy + recent
    _, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 77)
    Q = torch.zeros_like(K)
    qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, 1.0, dev, 77)
    qs.zero_()
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    col = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    cache.prefill_scores(Q, K, V, colsum_out=col)
    pos0 = cache.snapshot()[0].cpu().numpy()
    harm = np.cumsum(1.0 / np.arange(1, n + 1))                    # H_1 .. H_n
    want = harm[-1] - np.concatenate(([0.0], harm[:-1]))           # H_n - H_{j-1}, j = 1..n
    got = col.cpu().double().numpy()
    assert np.abs(got - want).max() <= 3e-6 * want.max(), "column sums differ from the harmonic closed form"
    first = list(range(heavy))
    for b in range(B):
        for h in range(Hh):
            assert pos0[b, h].tolist() == first + list(range(n - recent, n))
    outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs)
    snaps = snaps.numpy()
    vh = torch.cat([V.cpu().double(), vs.cpu().double().permute(1, 2, 0, 3)], dim=2).numpy()   # [B, Hh, n+T, d]
    for s in range(T):
        t = n + s
        kept = first + list(range(t - recent + 1, t + 1))
        for b in range(B):
            for h in range(Hh):
                assert sorted(snaps[s, b, h].tolist()) == kept, "step %d head (%d, %d)" % (s, b, h)
                # the output is the mean of the values attended to: kept set before the step + the token
                att = first + list(range(t - recent, t + 1))
                ref = vh[b, h, att].mean(0)
                f_l2, f_el, _, _ = parity.output_error(outs[s, b, h].double().numpy(), ref, dtype)
                assert f_l2 <= 1.0 and f_el <= 1.0
    # and the oracle agrees with the closed form's kept set (the pin, restated on the same tensors)
    o = OracleHead(d, heavy, recent, parity.oracle_scale(d), score_f32=True, cap=n + T)
    o.prefill(parity.host64(Q[0, 0]), parity.host64(K[0, 0]), parity.host64(V[0, 0]))
    for s in range(T):
        o.decode(parity.host64(qs[s, 0, 0]), parity.host64(ks[s, 0, 0]), parity.host64(vs[s, 0, 0]))
    assert o.resident()[0].tolist() == first + list(range(n + T - recent, n + T))
    cache.close()
