"""Pins for the CPU oracle: what the paper and the mathematics fix.

Each test checks ``oracle/`` against something that is NOT the oracle: a brute
force written differently (tests/brute.py), a library routine the method must
reduce to (torch.softmax causal attention), a closed form (harmonic numbers), or
an invariant of the eviction policy (Definition 2.1, Definition 2.2).
"""
import os

import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead
from tests.brute import brute_h2o

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_inputs(seed, N, d, sigma=0.75):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((N, d))
    K = rng.standard_normal((N, d)) * np.exp(sigma * rng.standard_normal((N, 1)))
    V = rng.standard_normal((N, d))
    return Q, K, V


def run_oracle(Q, K, V, n, heavy, recent, scale, score_f32=False, policy=0):
    N, d = Q.shape
    o = OracleHead(d, heavy, recent, scale, score_f32=score_f32, cap=N, policy=policy)
    sets, outs, evicted, lows = [], [], [], []
    colsum = attn = None
    if n > 0:
        colsum, attn = o.prefill(Q[:n], K[:n], V[:n], want_attn=True)
        sets.append(set(o.resident()[0].tolist()))
    for t in range(n, N):
        r = o.decode(Q[t], K[t], V[t])
        outs.append(r.out); evicted.append(r.evicted); lows.append((r.lowest, r.second))
        sets.append(set(o.resident()[0].tolist()))
    return o, dict(sets=sets, outs=np.array(outs), evicted=evicted, colsum=colsum,
                   attn=attn, lows=lows)


# ---------------------------------------------------------------- N1 brute force
@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("n,T,heavy,recent", [
    (8, 12, 2, 2), (10, 10, 3, 1), (6, 14, 1, 3), (0, 16, 2, 3), (12, 8, 4, 0),
    (9, 9, 0, 3), (5, 12, 3, 3), (14, 6, 2, 4), (4, 4, 4, 4),
])
def test_matches_brute_force(seed, n, T, heavy, recent):
    d = 4
    Q, K, V = make_inputs(1000 + seed, n + T, d)
    scale = 0.5
    o, got = run_oracle(Q, K, V, n, heavy, recent, scale)
    ref = brute_h2o(Q, K, V, n, heavy, recent, scale)
    # the comparison is only meaningful away from ties
    for lo, se in got["lows"]:
        if np.isfinite(se):
            assert se - lo > 1e-9
    assert got["sets"] == ref["sets"]
    assert got["evicted"] == ref["evicted"]
    np.testing.assert_allclose(got["outs"], ref["outs"], rtol=1e-12, atol=1e-13)
    if n > 0:
        np.testing.assert_allclose(got["colsum"], ref["colsum"], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(got["attn"], ref["attn_prompt"], rtol=1e-12, atol=1e-13)
    pos, sc = o.resident()
    np.testing.assert_allclose(sc, ref["acc"][pos], rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("seed", range(6))
def test_matches_brute_force_f32_scores(seed):
    """Scores stored in binary32: each probability is rounded to binary32 and
    added in binary32 (numpy float32 arithmetic is the independent reference)."""
    n, T, heavy, recent, d = 9, 14, 2, 3, 4
    Q, K, V = make_inputs(2000 + seed, n + T, d)
    o, got = run_oracle(Q, K, V, n, heavy, recent, 0.5, score_f32=True)
    ref = brute_h2o(Q, K, V, n, heavy, recent, 0.5, score_dtype=np.float32)
    assert got["sets"] == ref["sets"]
    pos, sc = o.resident()
    assert np.array_equal(sc, ref["acc"][pos])            # bit-exact
    assert np.array_equal(sc, sc.astype(np.float32).astype(np.float64))


# -------------------------------------------- N2 budget >= length == full attention
def torch_causal_attention(Q, K, V, scale):
    Qt, Kt, Vt = (torch.from_numpy(np.ascontiguousarray(x)) for x in (Q, K, V))
    S = scale * Qt @ Kt.T
    N = S.shape[0]
    S = S.masked_fill(torch.triu(torch.ones(N, N, dtype=torch.bool), diagonal=1), float("-inf"))
    P = torch.softmax(S, dim=-1)
    return (P @ Vt).numpy(), P.sum(0).numpy()


@pytest.mark.parametrize("n,T,d", [(24, 16, 8), (1, 30, 16), (40, 0, 4), (0, 20, 8)])
def test_budget_covers_sequence_is_full_causal_attention(n, T, d):
    Q, K, V = make_inputs(7, n + T, d, sigma=1.0)
    scale = 1.0 / np.sqrt(d)
    heavy, recent = (n + T + 1) // 2, (n + T) // 2 + 1
    o, got = run_oracle(Q, K, V, n, heavy, recent, scale)
    ref_out, ref_col = torch_causal_attention(Q, K, V, scale)
    if n:
        np.testing.assert_allclose(got["attn"], ref_out[:n], rtol=1e-11, atol=1e-12)
    if T:
        np.testing.assert_allclose(got["outs"], ref_out[n:], rtol=1e-11, atol=1e-12)
    pos, sc = o.resident()
    assert pos.tolist() == list(range(n + T))
    np.testing.assert_allclose(sc, ref_col, rtol=1e-11, atol=1e-13)
    assert all(e == -1 for e in got["evicted"])


def test_prompt_column_sums_are_softmax_column_sums():
    n, d = 33, 8
    Q, K, V = make_inputs(11, n, d, sigma=1.0)
    scale = 1.0 / np.sqrt(d)
    o = OracleHead(d, 4, 4, scale, cap=n)
    col, attn = o.prefill(Q, K, V, want_attn=True)
    ref_out, ref_col = torch_causal_attention(Q, K, V, scale)
    np.testing.assert_allclose(col, ref_col, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(attn, ref_out, rtol=1e-11, atol=1e-12)


# ---------------------------------------------- N3 decode-from-empty == prefill
def test_decode_from_empty_equals_prefill():
    n, d = 20, 8
    Q, K, V = make_inputs(3, n, d)
    scale = 0.3
    a = OracleHead(d, 10, 10, scale, cap=n)
    last = None
    for t in range(n):
        last = a.decode(Q[t], K[t], V[t])
    b = OracleHead(d, 10, 10, scale, cap=n)
    col, attn = b.prefill(Q, K, V, want_attn=True)
    pa, sa = a.resident(); pb, sb = b.resident()
    assert pa.tolist() == pb.tolist() == list(range(n))
    np.testing.assert_allclose(sa, sb, rtol=1e-12)
    np.testing.assert_allclose(last.out, attn[-1], rtol=1e-12, atol=1e-14)


# ------------------------------------------------- N4 equal logits: harmonic numbers
def test_equal_logits_closed_form():
    n, T, d, heavy, recent = 40, 25, 4, 5, 7
    rng = np.random.default_rng(0)
    K = rng.standard_normal((n + T, d)); V = rng.standard_normal((n + T, d))
    Q = np.zeros((n + T, d))
    o = OracleHead(d, heavy, recent, 1.0, cap=n + T)
    col, attn = o.prefill(Q[:n], K[:n], V[:n], want_attn=True)
    # 1-based: c_j = sum_{i=j..n} 1/i = H_n - H_{j-1}
    Hn = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, n + 1))])
    np.testing.assert_allclose(col, Hn[n] - Hn[:n], rtol=1e-13)
    # row i of uniform attention is the running mean of V
    np.testing.assert_allclose(attn, np.cumsum(V[:n], 0) / np.arange(1, n + 1)[:, None], rtol=1e-12,
                               atol=1e-13)
    expect_heavy = list(range(heavy))                # strictly decreasing scores
    assert o.resident()[0].tolist() == expect_heavy + list(range(n - recent, n))
    for t in range(n, n + T):
        r = o.decode(Q[t], K[t], V[t])
        # uniform over budget + 1 entries
        assert abs(r.p_self - 1.0 / (heavy + recent + 1)) < 1e-15
        # the token leaving the window has the lowest score and goes
        assert r.evicted == t - recent
        assert o.resident()[0].tolist() == expect_heavy + list(range(t - recent + 1, t + 1))
        members = expect_heavy + list(range(t - recent, t + 1))
        np.testing.assert_allclose(r.out, V[members].mean(0), rtol=1e-12, atol=1e-13)
    # every heavy token gained 1/(k+1) per step
    pos, sc = o.resident()
    np.testing.assert_allclose(sc[:heavy], (Hn[n] - Hn[:heavy]) + T / (heavy + recent + 1.0),
                               rtol=1e-12)


# ------------------------------------------------------ N5 heavy = 0: sliding window
def test_heavy_zero_is_sliding_window_attention():
    n, T, d, recent = 10, 20, 8, 4
    Q, K, V = make_inputs(5, n + T, d)
    scale = 1.0 / np.sqrt(d)
    o, got = run_oracle(Q, K, V, n, 0, recent, scale)
    for idx, t in enumerate(range(n, n + T)):
        lo = max(0, t - recent)                       # R cached tokens + the token itself
        s = torch.from_numpy(scale * (K[lo:t + 1] @ Q[t]))
        p = torch.softmax(s, 0).numpy()
        np.testing.assert_allclose(got["outs"][idx], p @ V[lo:t + 1], rtol=1e-11, atol=1e-12)
        assert got["sets"][idx + 1] == set(range(t - recent + 1, t + 1))
        assert got["evicted"][idx] == t - recent


def test_recent_zero_new_token_can_be_dropped():
    """R = 0: the new token is itself a candidate (Algorithm 1's G_i includes i)."""
    d = 4
    o = OracleHead(d, 2, 0, 1.0, cap=8)
    e = np.eye(d)
    big = 6.0
    # two prompt tokens that every later query loves
    o.prefill(np.stack([e[0], e[0]]) * big, np.stack([e[0], e[0]]) * big, np.ones((2, d)))
    r = o.decode(e[0] * big, -e[0] * big, np.ones(d))      # its own key repels its query
    assert r.evicted == 2 and o.resident()[0].tolist() == [0, 1]
    assert r.n_candidates == 3


# ----------------------------------------------- N6-N8 invariants on random runs
@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("n,T,heavy,recent,f32", [
    (64, 64, 8, 8, False), (30, 100, 5, 11, True), (0, 80, 7, 3, False), (100, 30, 16, 16, True),
])
def test_invariants(seed, n, T, heavy, recent, f32):
    d = 8
    k = heavy + recent
    Q, K, V = make_inputs(300 + seed, n + T, d, sigma=1.0)
    o = OracleHead(d, heavy, recent, 1.0 / np.sqrt(d), score_f32=f32, cap=n + T)
    if n:
        o.prefill(Q[:n], K[:n], V[:n])
    prev = set(o.resident()[0].tolist())
    gone = set(range(n)) - prev
    tol = 1e-4 if f32 else 1e-10
    for t in range(n, n + T):
        r = o.decode(Q[t], K[t], V[t])
        pos, sc = o.resident()
        cur = set(pos.tolist())
        seen = t + 1
        assert len(cur) == min(seen, k)                              # |S_i| = k (<= k while filling)
        assert len(cur - prev) <= 1 and cur - prev <= {t}            # at most one token enters
        assert len(prev - cur) <= 1                                  # at most one leaves
        assert not (cur & gone)                                      # evicted tokens never return
        gone |= (prev | {t}) - cur
        assert set(range(max(0, seen - recent), seen)) <= cur        # recent window resident
        assert abs(sc.sum() + o.evicted_mass - o.queries) < tol * seen   # mass conservation
        assert o.queries == seen
        # a score never exceeds the number of queries issued since the token arrived
        assert np.all(sc <= (seen - pos) * (1 + 1e-6))
        assert sc.sum() <= seen * (1 + 1e-6)
        if r.evicted >= 0:
            assert r.evicted <= t - recent and r.lowest <= r.second
        prev = cur


# ------------------------------------------------------------ N9 a dominant key
def test_dominant_key_is_never_evicted():
    n, T, d, heavy, recent = 20, 40, 8, 2, 3
    rng = np.random.default_rng(9)
    Q = rng.standard_normal((n + T, d)); Q[:, 0] = 3.0      # all queries agree on axis 0
    K = rng.standard_normal((n + T, d)) * 0.1
    V = rng.standard_normal((n + T, d))
    star = 5
    K[star] = 0.0; K[star, 0] = 20.0                         # logit ~ 60 above the rest
    o = OracleHead(d, heavy, recent, 1.0, cap=n + T)
    o.prefill(Q[:n], K[:n], V[:n])
    for t in range(n, n + T):
        r = o.decode(Q[t], K[t], V[t])
        assert o.is_resident(star)
        np.testing.assert_allclose(r.out, V[star], atol=1e-12)
    # it collected (almost) one unit from every query issued after it arrived
    assert abs(o.score(star) - (n + T - star)) < 1e-9


# ----------------------------------------------------- N10 shift invariance, range
def test_large_logits_do_not_overflow_and_shift_invariance():
    n, T, d = 12, 12, 4
    Q, K, V = make_inputs(21, n + T, d)
    Q2 = Q * 40.0                                            # logits of order +-150
    _, a = run_oracle(Q2, K, V, n, 3, 3, 1.0)
    assert np.all(np.isfinite(a["outs"])) and np.all(np.isfinite(a["colsum"]))
    # adding a constant vector c to every key shifts each row's logits by q.c:
    # probabilities (hence everything) are unchanged
    c = np.array([0.7, -1.1, 0.3, 2.0])
    _, b = run_oracle(Q, K, V, n, 3, 3, 0.5)
    _, s = run_oracle(Q, K + c, V, n, 3, 3, 0.5)
    assert b["sets"] == s["sets"]
    np.testing.assert_allclose(b["outs"], s["outs"], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(b["colsum"], s["colsum"], rtol=1e-9)


# ------------------------------------------------------------------ tie-breaking
def test_exact_ties_evict_lowest_position():
    d = 2
    o = OracleHead(d, 3, 1, 1.0, cap=16)
    K = np.zeros((4, d)); Q = np.zeros((4, d)); V = np.arange(8.0).reshape(4, d)
    # decode four tokens with identical logits: scores 1+1/2+1/3+1/4, 1/2+1/3+1/4, ...
    for t in range(4):
        o.decode(Q[t], K[t], V[t])
    # craft a tie: tokens 4 and 5 arrive with equal keys and get equal probability after
    r = o.decode(np.zeros(d), np.zeros(d), np.zeros(d))     # t=4: full (k=4) -> someone leaves
    assert r.evicted == 3                                    # lowest score among positions <= 3
    # load exactly equal scores and check the position rule directly
    o2 = OracleHead(d, 2, 1, 1.0, cap=8)
    o2.load_and_select(np.zeros((5, d)), np.zeros((5, d)), np.array([0.5, 0.25, 0.25, 0.25, 9.0]))
    assert o2.resident()[0].tolist() == [0, 3, 4]            # ties: lowest positions dropped first
    r = o2.decode(np.zeros(d), np.zeros(d), np.zeros(d))     # all gain 1/4; candidates 0,3,4
    assert r.evicted == 3 and r.lowest == 0.5 and r.second == 0.75


def test_select_equals_repeated_eviction_and_respects_window():
    rng = np.random.default_rng(4)
    n, d, heavy, recent = 50, 4, 6, 9
    K = rng.standard_normal((n, d)); V = rng.standard_normal((n, d))
    score = rng.random(n); score[[3, 17, 30]] = 0.5          # a three-way tie in the middle
    o = OracleHead(d, heavy, recent, 1.0, cap=n)
    o.load_and_select(K, V, score)
    older = sorted(range(n - recent), key=lambda j: (score[j], j), reverse=True)[:heavy]
    assert o.resident()[0].tolist() == sorted(older) + list(range(n - recent, n))
    assert abs(o.evicted_mass + o.resident()[1].sum() - score.sum()) < 1e-12


# ----------------------------------------------------- resync (test bookkeeping)
def test_resync_swaps_membership_and_mass():
    Q, K, V = make_inputs(8, 30, 4)
    o = OracleHead(4, 3, 3, 0.5, cap=30)
    o.prefill(Q[:20], K[:20], V[:20])
    r = o.decode(Q[20], K[20], V[20])
    pos, sc = o.resident()
    other = int(pos[0]) if pos[0] != r.evicted else int(pos[1])
    total = sc.sum() + o.evicted_mass
    o.resync(r.evicted, other)
    pos2, sc2 = o.resident()
    assert r.evicted in pos2 and other not in pos2 and len(pos2) == len(pos)
    assert abs(sc2.sum() + o.evicted_mass - total) < 1e-12


# ------------------------------------- the paper's one worked example (outcome only)
def test_worked_example_outcome():
    """Sec. 4.2, the illustration of Algorithm 1: budget 3, after the fourth
    decoding step the third token is the one evicted.  The figure's numbers are
    not in the text, so inputs realising the stated outcome are constructed."""
    with open(os.path.join(GOLDEN, "alg1_worked_example.txt")) as f:
        fields = dict(line.split("=", 1) for line in f.read().split() if "=" in line)
    budget, step, victim = int(fields["budget"]), int(fields["step"]), int(fields["evicted_token"])
    d = 4
    e = np.eye(d)
    # tokens 1, 2 and 4 have keys aligned with every query, token 3's key is opposed
    K = np.stack([e[0], e[0], -e[0], e[0]]) * 2.0
    Q = np.stack([e[0]] * 4) * 2.0
    V = np.ones((4, d))
    o = OracleHead(d, budget, 0, 1.0, cap=4)                 # Algorithm 1 has no recent window
    ev = [o.decode(Q[t], K[t], V[t]).evicted for t in range(step)]
    assert ev[:budget] == [-1] * budget                      # cache not full: expand only
    assert ev[step - 1] == victim - 1                        # 1-based token 3
    assert o.resident()[0].tolist() == [0, 1, 3]


# ------------------------------------------------ averaged-score ranking (App. B)
@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("n,T,heavy,recent", [(8, 12, 2, 2), (10, 10, 3, 1), (0, 16, 2, 3), (12, 8, 4, 0),
                                              (14, 6, 2, 4)])
@pytest.mark.parametrize("f32", [False, True])
def test_average_policy_matches_brute_force(seed, n, T, heavy, recent, f32):
    """Ranking by score / (number of queries that scored the token): the brute
    force evaluates F(G \\ {v}) = sum of the averaged scores for every allowed v."""
    d = 4
    Q, K, V = make_inputs(5000 + seed, n + T, d)
    scale = 0.5
    o, got = run_oracle(Q, K, V, n, heavy, recent, scale, score_f32=f32, policy=1)
    ref = brute_h2o(Q, K, V, n, heavy, recent, scale, np.float32 if f32 else np.float64, policy=1)
    for lo, se in got["lows"]:
        if np.isfinite(se):
            assert se - lo > 1e-9
    assert got["sets"] == ref["sets"]
    assert got["evicted"] == ref["evicted"]
    np.testing.assert_allclose(got["outs"], ref["outs"], rtol=1e-12, atol=1e-13)
    pos, sc = o.resident()
    # what is stored stays the ACCUMULATED score
    if f32:
        assert np.array_equal(sc, ref["acc"][pos])
    else:
        np.testing.assert_allclose(sc, ref["acc"][pos], rtol=1e-12, atol=1e-14)


def test_average_policy_differs_from_accumulated_where_it_should():
    """An old token with a long record of small scores against a younger one
    with a short record of larger scores: the accumulated score keeps the old
    one, the averaged score keeps the young one.  Scores are constructed through
    load_and_select (positions 0 and 6 of an 8-token prompt, window of one)."""
    d, n = 2, 8
    K = np.zeros((n, d)); V = np.zeros((n, d))
    score = np.full(n, 5.0)                # everything else is clearly better
    score[0] = 1.6                         # 8 queries: average 0.2
    score[6] = 1.0                         # 2 queries: average 0.5
    kept = {}
    for policy in (0, 1):
        o = OracleHead(d, n - 2, 1, 1.0, cap=n, policy=policy)   # drop exactly one older token
        o.load_and_select(K, V, score)
        kept[policy] = set(o.resident()[0].tolist())
    assert 6 not in kept[0] and 0 in kept[0]
    assert 0 not in kept[1] and 6 in kept[1]


def test_average_policy_uniform_attention_closed_form():
    """Equal logits, prompt 12, budget 3 + 2.  Every query spreads 1/|G| over its
    |G| tokens, so scores are sums of unit fractions:
      * step t = 12 evicts token 10 (just out of the window): scored by the
        queries 10, 11 (prompt rows: 1/11, 1/12) and 12 (cache of 6: 1/6),
        average (1/11 + 1/12 + 1/6) / 3;
      * a token that arrives once the cache is full averages exactly 1/6, while
        an old heavy hitter's average keeps falling towards 1/6 from the prompt
        rows it collected: token 2 has (H_12 - H_2 + 3/6) / 13 < 1/6 at t = 14
        and is evicted there -- under the accumulated score it never is."""
    d, n, T, heavy, recent = 3, 12, 10, 3, 2
    Q = np.zeros((n + T, d)); K = np.ones((n + T, d)); V = np.arange((n + T) * d, dtype=float).reshape(-1, d)
    H = lambda m: sum(1.0 / i for i in range(1, m + 1))
    avg = OracleHead(d, heavy, recent, 1.0, cap=n + T, policy=1)
    acc = OracleHead(d, heavy, recent, 1.0, cap=n + T, policy=0)
    for o in (avg, acc):
        o.prefill(Q[:n], K[:n], V[:n])
        assert set(o.resident()[0].tolist()) == set(range(heavy)) | set(range(n - recent, n))
    evicted = {}
    for t in range(n, n + T):
        ra = avg.decode(Q[t], K[t], V[t])
        rs = acc.decode(Q[t], K[t], V[t])
        evicted[t] = ra.evicted
        assert rs.evicted == t - recent               # accumulated score: always the newcomer
        if t == 12:
            assert ra.evicted == 10
            assert ra.lowest == pytest.approx((1 / 11 + 1 / 12 + 1 / 6) / 3, rel=1e-13)
        if t == 14:
            assert ra.evicted == 2
            assert ra.lowest == pytest.approx((H(12) - H(2) + 3 / 6) / 13, rel=1e-13)
            assert ra.lowest < 1 / 6
    assert evicted[13] == 11
    assert set(range(heavy)) <= set(acc.resident()[0].tolist())
    assert 2 not in set(avg.resident()[0].tolist())


def test_policy_argument_is_validated():
    with pytest.raises(ValueError):
        OracleHead(4, 2, 2, 1.0, cap=8, policy=2)


# ------------------------------------------------------- chunked prompt processing
from tests.brute import brute_chunked  # noqa: E402


def run_chunked(Q, K, V, chunks, heavy, recent, scale, score_f32=False, policy=0):
    N, d = Q.shape
    o = OracleHead(d, heavy, recent, scale, score_f32=score_f32, cap=N, policy=policy)
    outs, sets = np.zeros((N, d)), []
    t0 = 0
    for m in chunks:
        _, attn = o.prefill_chunk(Q[t0:t0 + m], K[t0:t0 + m], V[t0:t0 + m], want_attn=True)
        outs[t0:t0 + m] = attn
        sets.append(set(o.resident()[0].tolist()))
        t0 += m
    return o, outs, sets


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("chunks,heavy,recent", [
    ([5, 5, 5, 5], 3, 2), ([1, 7, 2, 9, 1], 2, 3), ([12, 8], 4, 0), ([3, 3, 3, 3, 3, 3], 0, 4),
    ([20], 3, 3), ([2, 18], 5, 5), ([9, 1, 1, 1, 8], 1, 1),
])
@pytest.mark.parametrize("f32,policy", [(False, 0), (True, 0), (False, 1), (True, 1)])
def test_chunked_matches_brute_force(seed, chunks, heavy, recent, f32, policy):
    d = 4
    N = sum(chunks)
    Q, K, V = make_inputs(7000 + seed, N, d)
    scale = 0.5
    o, outs, sets = run_chunked(Q, K, V, chunks, heavy, recent, scale, f32, policy)
    ref = brute_chunked(Q, K, V, chunks, heavy, recent, scale, np.float32 if f32 else np.float64, policy)
    assert sets == ref["sets"]
    np.testing.assert_allclose(outs, ref["outs"], rtol=1e-12, atol=1e-13)
    pos, sc = o.resident()
    if f32:
        assert np.array_equal(sc, ref["acc"][pos])
    else:
        np.testing.assert_allclose(sc, ref["acc"][pos], rtol=1e-12, atol=1e-14)
    k = heavy + recent
    assert len(pos) == min(N, k)
    assert set(range(N - min(recent, N), N)) <= set(pos.tolist())
    # every softmax row sums to one: nothing is lost except what was evicted
    assert o.queries == N
    assert sc.sum() + o.evicted_mass == pytest.approx(N, rel=1e-6 if f32 else 1e-12)


@pytest.mark.parametrize("f32", [False, True])
def test_chunks_of_one_are_generation_steps(f32):
    """Algorithm 1 end of the range: chunks of a single token give, bit for bit,
    what the generation step gives (outputs, kept sets, scores)."""
    d, N, heavy, recent = 4, 40, 4, 3
    Q, K, V = make_inputs(81, N, d)
    a = OracleHead(d, heavy, recent, 0.5, score_f32=f32, cap=N)
    b = OracleHead(d, heavy, recent, 0.5, score_f32=f32, cap=N)
    for t in range(N):
        r = a.decode(Q[t], K[t], V[t])
        _, attn = b.prefill_chunk(Q[t:t + 1], K[t:t + 1], V[t:t + 1], want_attn=True)
        assert np.array_equal(attn[0], r.out)
        pa, sa = a.resident(); pb, sb = b.resident()
        assert np.array_equal(pa, pb) and np.array_equal(sa, sb)


@pytest.mark.parametrize("f32", [False, True])
def test_one_chunk_is_the_one_shot_prompt_phase(f32):
    """App. A end of the range: a single chunk holding the whole prompt gives, bit
    for bit, the one-shot prompt phase."""
    d, n, heavy, recent = 4, 30, 5, 4
    Q, K, V = make_inputs(82, n, d)
    a = OracleHead(d, heavy, recent, 0.5, score_f32=f32, cap=n)
    b = OracleHead(d, heavy, recent, 0.5, score_f32=f32, cap=n)
    ca, aa = a.prefill(Q, K, V, want_attn=True)
    cb, ab = b.prefill_chunk(Q, K, V, want_attn=True)
    assert np.array_equal(ca, cb) and np.array_equal(aa, ab)
    pa, sa = a.resident(); pb, sb = b.resident()
    assert np.array_equal(pa, pb) and np.array_equal(sa, sb)
    assert a.evicted_mass == b.evicted_mass


def test_chunking_is_invisible_while_nothing_is_evicted():
    """Budget >= sequence length: however the prompt is cut into chunks, outputs
    are full causal attention and scores the full column sums."""
    d, n = 4, 36
    Q, K, V = make_inputs(83, n, d)
    full = OracleHead(d, n, n, 0.5, cap=n)
    col, attn = full.prefill(Q, K, V, want_attn=True)
    for chunks in ([36], [1] * 36, [10, 1, 25], [17, 19]):
        o, outs, _ = run_chunked(Q, K, V, chunks, n, n, 0.5)
        np.testing.assert_allclose(outs, attn, rtol=1e-13, atol=1e-14)
        pos, sc = o.resident()
        assert pos.tolist() == list(range(n))
        np.testing.assert_allclose(sc, col, rtol=1e-12, atol=1e-14)


# ------------------------------------------------ 4-bit group-wise cache storage
from tests.brute import nearest_level_quantise  # noqa: E402


def as_stored(x, kind):
    """Random rows as a cache element type would hold them (exactly representable)."""
    t = torch.from_numpy(np.asarray(x, np.float64))
    dt = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[kind]
    return t.to(dt).double().numpy()


def dequantise(codes, par, group):
    """Stored values from codes and (scale, min) pairs, in exact arithmetic (fp64 holds
    a 4-bit integer times a binary32 plus a binary32 to well below 1e-15 relative)."""
    c = codes.astype(np.float64).reshape(-1, group)
    return (par[:, 1:2].astype(np.float64) + c * par[:, 0:1].astype(np.float64)).reshape(-1)


@pytest.mark.parametrize("kind", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("d,group", [(128, 64), (64, 64), (8, 4)])
def test_quantised_rows_are_the_nearest_of_sixteen_even_levels(kind, d, group):
    rng = np.random.default_rng(7)
    n = 24
    K = as_stored(rng.standard_normal((n, d)) * np.exp(rng.standard_normal((n, 1))), kind)
    V = as_stored(rng.standard_normal((n, d)), kind)
    o = OracleHead(d, n, n, 0.3, cap=n, kv_bits=4, group=group)
    o.prefill(as_stored(rng.standard_normal((n, d)), kind), K, V)     # budget covers it: all kept
    seen = unclear = 0
    for j in range(n):
        kc, kp, vc, vp = o.token_codes(j)
        for row, codes, par in ((K[j], kc, kp), (V[j], vc, vp)):
            ref, ref_codes, margin = nearest_level_quantise(row, group)
            # an element on a half-way point (16-bit data hit them exactly now and then) may
            # go either way in the search; everywhere else the code is the nearest level
            clear = margin > 1e-6
            seen += clear.size; unclear += int((~clear).sum())
            np.testing.assert_array_equal(codes[clear], ref_codes[clear])
            assert np.all(np.abs(codes.astype(np.int64) - ref_codes) <= 1)
            g = row.reshape(-1, group)
            np.testing.assert_array_equal(par[:, 1], g.min(axis=1).astype(np.float32))
            np.testing.assert_array_equal(
                par[:, 0], ((g.max(axis=1).astype(np.float32) - g.min(axis=1).astype(np.float32))
                            / np.float32(15)).astype(np.float32))
            stored = dequantise(codes, par, group)
            np.testing.assert_allclose(stored[clear], ref[clear], rtol=0, atol=1e-12)
            # uniform quantiser: never further than half a step from the input; ends are exact
            step = np.repeat(par[:, 0].astype(np.float64), group)
            assert np.all(np.abs(stored - row) <= 0.5 * step * (1 + 1e-6))
            cg = codes.reshape(-1, group)
            assert np.all(cg.min(axis=1) == 0) and np.all(cg.max(axis=1) == 15)
            assert np.all(cg[np.arange(len(g)), g.argmin(axis=1)] == 0)
            assert np.all(cg[np.arange(len(g)), g.argmax(axis=1)] == 15)
        ks, vs = o.token_kv(j)
        np.testing.assert_array_equal(ks, dequantise(kc, kp, group))
        np.testing.assert_array_equal(vs, dequantise(vc, vp, group))
    assert unclear < 0.03 * seen


def test_quantised_constant_group_and_group_independence():
    d, group = 8, 4
    K = np.array([[2.5] * 4 + [1.0, -3.0, 0.25, 7.0]])
    V = np.array([[0.0] * 4 + [0.5, 0.5, 0.5, 0.5]])
    o = OracleHead(d, 1, 1, 1.0, cap=4, kv_bits=4, group=group)
    o.prefill(np.ones((1, d)), K, V)
    kc, kp, vc, vp = o.token_codes(0)
    assert kp[0, 0] == 0 and kp[0, 1] == 2.5 and np.all(kc[:4] == 0)
    assert np.all(vc == 0) and np.all(vp[:, 0] == 0) and list(vp[:, 1]) == [0.0, 0.5]
    np.testing.assert_array_equal(o.token_kv(0)[1], V[0])
    # the second group's contents do not reach the first group's codes
    K2 = K.copy(); K2[0, :4] = [1.0, 2.0, 4.0, 1.5]
    K3 = K2.copy(); K3[0, 4:] = [100.0, -100.0, 3.0, 0.0]
    a = OracleHead(d, 1, 1, 1.0, cap=4, kv_bits=4, group=group); a.prefill(np.ones((1, d)), K2, V)
    b = OracleHead(d, 1, 1, 1.0, cap=4, kv_bits=4, group=group); b.prefill(np.ones((1, d)), K3, V)
    np.testing.assert_array_equal(a.token_codes(0)[0][:4], b.token_codes(0)[0][:4])
    np.testing.assert_array_equal(a.token_codes(0)[1][0], b.token_codes(0)[1][0])
    assert list(a.token_codes(0)[0][:4]) == [0, 5, 15, 2]      # (x - 1) / 0.2 = 0, 5, 15, 2.5 -> even


def grid_rows(rng, n, d, group):
    """Rows that lie exactly on their own 16 levels (spacing a power of two, both
    ends present in every group): storing them in 4 bits loses nothing."""
    rows = np.empty((n, d))
    for i in range(n):
        for g0 in range(0, d, group):
            c = rng.integers(0, 16, group)
            c[rng.permutation(group)[:2]] = [0, 15]
            rows[i, g0:g0 + group] = rng.integers(-16, 16) / 8.0 + c * 2.0 ** rng.integers(-4, 1)
    return rows


@pytest.mark.parametrize("f32", [False, True])
@pytest.mark.parametrize("n,T,heavy,recent", [(20, 30, 4, 4), (0, 40, 3, 5), (16, 24, 6, 0)])
def test_rows_on_their_levels_make_quantised_storage_invisible(n, T, heavy, recent, f32):
    rng = np.random.default_rng(n + T)
    d, group = 16, 8
    Q = rng.standard_normal((n + T, d))
    K, V = grid_rows(rng, n + T, d, group), grid_rows(rng, n + T, d, group)
    runs = []
    for bits in (0, 4):
        o = OracleHead(d, heavy, recent, 0.25, score_f32=f32, cap=n + T, kv_bits=bits, group=group)
        outs, ev = [], []
        if n:
            o.prefill(Q[:n], K[:n], V[:n])
        for t in range(n, n + T):
            r = o.decode(Q[t], K[t], V[t])
            outs.append(r.out); ev.append(r.evicted)
        runs.append((np.array(outs), ev, o.resident()))
    np.testing.assert_array_equal(runs[0][0], runs[1][0])
    assert runs[0][1] == runs[1][1]
    np.testing.assert_array_equal(runs[0][2][0], runs[1][2][0])
    np.testing.assert_array_equal(runs[0][2][1], runs[1][2][1])


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("n,T,heavy,recent", [(8, 12, 2, 2), (0, 16, 2, 3), (12, 8, 4, 0), (9, 9, 0, 3)])
def test_quantised_cache_matches_brute_force(seed, n, T, heavy, recent):
    d, group = 8, 4
    # binary32 data: 16-bit data land on half-way points between levels too often for a search
    Q, K, V = (as_stored(x, "f32") for x in make_inputs(3000 + seed, n + T, d))
    scale = 0.5
    margins = []

    def store(row):
        out, _, margin = nearest_level_quantise(row, group)
        margins.append(margin.min())
        return out
    ref = brute_h2o(Q, K, V, n, heavy, recent, scale, store=store)
    assert min(margins) > 1e-4, "test data sits on a half-way point; pick another seed"
    o = OracleHead(d, heavy, recent, scale, cap=n + T, kv_bits=4, group=group)
    sets, outs, ev = [], [], []
    if n:
        o.prefill(Q[:n], K[:n], V[:n])
        sets.append(set(o.resident()[0].tolist()))
    for t in range(n, n + T):
        r = o.decode(Q[t], K[t], V[t])
        if np.isfinite(r.second):
            assert r.second - r.lowest > 1e-9
        outs.append(r.out); ev.append(r.evicted); sets.append(set(o.resident()[0].tolist()))
    assert sets == ref["sets"] and ev == ref["evicted"]
    np.testing.assert_allclose(np.array(outs), ref["outs"], rtol=1e-12, atol=1e-13)
    pos, sc = o.resident()
    np.testing.assert_allclose(sc, ref["acc"][pos], rtol=1e-12, atol=1e-14)
    # the run differs from unquantised storage (the pin above is not vacuous)
    plain = brute_h2o(Q, K, V, n, heavy, recent, scale)
    assert np.abs(plain["outs"] - ref["outs"]).max() > 1e-4


def test_token_attends_to_itself_unquantised_and_is_stored_quantised():
    d, group = 8, 4
    rng = np.random.default_rng(5)
    q, k, v = (as_stored(rng.standard_normal((2, d)), "f16") for _ in range(3))
    o = OracleHead(d, 2, 2, 0.5, cap=4, kv_bits=4, group=group)
    r0 = o.decode(q[0], k[0], v[0])
    np.testing.assert_array_equal(r0.out, v[0])          # alone in the cache: p_self = 1, its own value as given
    kc, kp, vc, vp = o.token_codes(0)
    k0, v0 = dequantise(kc, kp, group), dequantise(vc, vp, group)
    assert np.abs(k0 - k[0]).max() > 1e-3 and np.abs(v0 - v[0]).max() > 1e-3
    r1 = o.decode(q[1], k[1], v[1])
    s = 0.5 * np.array([q[1] @ k0, q[1] @ k[1]])         # stored key for token 0, own key as given
    p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(r1.out, p[0] * v0 + p[1] * v[1], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(o.score(0), 1.0 + p[0], rtol=1e-14)


def test_resync_on_a_quantised_cache_stores_the_restored_token():
    """h2o_oracle_resync on 4-bit storage: the token that becomes resident again holds the
    nearest-of-sixteen-levels codes of its original row (search in tests/brute.py), the token
    that leaves keeps nothing that is read later, membership and mass swap as without
    quantisation."""
    rng = np.random.default_rng(21)
    d, group, n = 8, 4, 14
    Q, K, V = (as_stored(rng.standard_normal((n + 3, d)), "f16") for _ in range(3))
    o = OracleHead(d, 3, 3, 0.4, score_f32=True, cap=n + 3, kv_bits=4, group=group)
    o.prefill(Q[:n], K[:n], V[:n])
    evicted = [j for j in range(n) if not o.is_resident(j)]
    assert len(evicted) == n - 6
    back = evicted[2]
    with pytest.raises(RuntimeError):
        o.token_codes(back)                          # never entered the cache: nothing stored
    out = int(o.resident()[0][0])
    total = o.resident()[1].sum() + o.evicted_mass
    o.resync(back, out)
    assert o.is_resident(back) and not o.is_resident(out)
    assert abs(o.resident()[1].sum() + o.evicted_mass - total) < 1e-12
    kc, kp, vc, vp = o.token_codes(back)
    for row, codes, par in ((K[back], kc, kp), (V[back], vc, vp)):
        ref, ref_codes, margin = nearest_level_quantise(row, group)
        clear = margin > 1e-6
        np.testing.assert_array_equal(codes[clear], ref_codes[clear])
        np.testing.assert_allclose(dequantise(codes, par, group)[clear], ref[clear], rtol=0, atol=1e-12)
    ks, vs = o.token_kv(back)
    np.testing.assert_array_equal(ks, dequantise(kc, kp, group))
    # and the next step attends to the stored (quantised) row of the restored token
    r = o.decode(Q[n], K[n], V[n])
    # attended to: what was resident before the step (incl. the token the step evicted), as
    # stored, and the new token itself with its row as given
    res = [j for j in range(n) if o.is_resident(j) or j == r.evicted]
    assert back in res and len(res) == 6
    Kd = np.stack([o.token_kv(j)[0] for j in res] + [K[n]])
    Vd = np.stack([o.token_kv(j)[1] for j in res] + [V[n]])
    s = 0.4 * Kd @ Q[n]
    p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(r.out, p @ Vd, rtol=1e-12, atol=1e-12)


def test_quantised_storage_arguments():
    with pytest.raises(ValueError):
        OracleHead(8, 2, 2, kv_bits=8)
    with pytest.raises(ValueError):
        OracleHead(8, 2, 2, kv_bits=4, group=3)
    o = OracleHead(8, 2, 2, cap=16, kv_bits=4, group=4)
    x = np.zeros((3, 8))
    with pytest.raises(RuntimeError):
        o.prefill_chunk(x, x, x)                          # not defined with quantised storage
    with pytest.raises(RuntimeError):
        OracleHead(8, 2, 2, cap=16).token_codes(0)


# ------------------------------------------------ invariants over random schedules
from hypothesis import given, settings, strategies as st  # noqa: E402


@settings(max_examples=60, deadline=None)
@given(seed=st.integers(0, 2 ** 31 - 1), heavy=st.integers(0, 6), recent=st.integers(0, 6),
       schedule=st.lists(st.tuples(st.sampled_from(["chunk", "steps"]), st.integers(1, 9)), min_size=1, max_size=6),
       f32=st.booleans(), policy=st.integers(0, 1), bits=st.sampled_from([0, 4]))
def test_invariants_over_random_schedules(seed, heavy, recent, schedule, f32, policy, bits):
    """Whatever mix of prompt chunks and generation steps: the cache never exceeds the
    budget, holds everything while it is not full, always holds the recent window,
    evicted tokens never return, scores are bounded by the queries that could have
    scored the token, and attention mass is conserved."""
    if heavy + recent == 0:
        heavy = 1
    if bits == 4:
        schedule = [("steps", m) if kind == "chunk" else (kind, m) for kind, m in schedule]
    d, k = 8, heavy + recent
    N = sum(m for _, m in schedule)
    Q, K, V = (as_stored(x, "f16") for x in make_inputs(seed % 100000, N, d, sigma=1.0))
    o = OracleHead(d, heavy, recent, 0.4, score_f32=f32, cap=N, policy=policy, kv_bits=bits, group=4)
    t, gone, prev = 0, set(), set()
    for kind, m in schedule:
        if kind == "chunk":
            o.prefill_chunk(Q[t:t + m], K[t:t + m], V[t:t + m])
            t += m
        else:
            for _ in range(m):
                r = o.decode(Q[t], K[t], V[t])
                assert np.all(np.isfinite(r.out))
                t += 1
        pos, sc = o.resident()
        cur = set(pos.tolist())
        assert o.t == t and len(cur) == min(t, k)
        assert set(range(max(0, t - recent), t)) <= cur
        assert not (cur & gone)
        gone |= (prev | set(range(t))) - cur
        assert np.all(sc >= 0) and np.all(sc <= (t - pos) * (1 + 1e-5))
        assert abs(sc.sum() + o.evicted_mass - o.queries) <= (1e-4 if f32 else 1e-9) * max(t, 1)
        assert o.queries == t
        prev = cur


# ------------------------------- sparse-attention patterns as the protected set (+ heavy hitters)
from tests.brute import pattern_cover  # noqa: E402

PATTERN_MODE = {"strided": 1, "fixed": 2}


def run_oracle_pattern(Q, K, V, n, heavy, recent, scale, pattern, score_f32=False, policy=0):
    N, d = Q.shape
    o = OracleHead(d, heavy, recent, scale, score_f32=score_f32, cap=N, policy=policy,
                   protect=PATTERN_MODE[pattern[0]], stride=pattern[1])
    sets, outs, evicted = [], [], []
    if n > 0:
        o.prefill(Q[:n], K[:n], V[:n])
        sets.append(set(o.resident()[0].tolist()))
    for t in range(n, N):
        r = o.decode(Q[t], K[t], V[t])
        outs.append(r.out); evicted.append(r.evicted)
        sets.append(set(o.resident()[0].tolist()))
    return o, dict(sets=sets, outs=np.array(outs), evicted=evicted)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("f32,policy", [(False, 0), (True, 0), (True, 1)])
@pytest.mark.parametrize("pattern", [("strided", 2), ("strided", 3), ("strided", 5), ("fixed", 3),
                                     ("fixed", 4), ("fixed", 7)])
@pytest.mark.parametrize("n,T,heavy,recent", [(10, 12, 2, 2), (0, 18, 3, 1), (13, 9, 1, 3), (16, 8, 4, 2),
                                              (9, 10, 3, 0)])
def test_pattern_protection_matches_brute_force(seed, f32, policy, pattern, n, T, heavy, recent):
    """The brute force builds the covered set of every query by enumeration, keeps the prompt by
    sorting, and evicts by evaluating F_score of every allowed removal."""
    if pattern[0] == "fixed" and recent > pattern[1]:
        pytest.skip("a block has fewer positions than summary columns asked for")
    d = 4
    Q, K, V = make_inputs(7000 + seed, n + T, d)
    o, got = run_oracle_pattern(Q, K, V, n, heavy, recent, 0.5, pattern, score_f32=f32, policy=policy)
    ref = brute_h2o(Q, K, V, n, heavy, recent, 0.5, np.float32 if f32 else np.float64, policy=policy,
                    pattern=pattern)
    assert got["sets"] == ref["sets"]
    assert got["evicted"] == ref["evicted"]
    np.testing.assert_allclose(got["outs"], ref["outs"], rtol=1e-12, atol=1e-12)


def test_strided_pattern_worked_by_hand():
    """Budget 1 + 1, strided pattern of period 2, band of 1.  Two tokens are loaded with scores
    (1, 5); every later query gives each cached token and itself the same probability (q = 0).
      t = 2: scores (4/3, 16/3, 1/3); the pattern covers {2} and {2, 0}; only token 1 competes
             and goes although it has the highest score             -> {0, 2}
      t = 3: scores 0: 5/3, 2: 2/3; covers {3} and {3, 1}; tokens 0 and 2 compete, 2 is lower -> {0, 3}
      t = 4: covers {4} and {4, 2, 0}; only token 3 competes                                   -> {0, 4}
      t = 5: covers {5} and {5, 3, 1}; 0 (score 2 + 1/3) and 4 (2/3) compete                   -> {0, 5}
    (Under the recent-window rule token 0, the lowest score outside the window at t = 2, would
    have gone first.)"""
    d = 2
    o = OracleHead(d, 1, 1, 1.0, cap=8, protect=1, stride=2)
    o.load_and_select(np.ones((2, d)), np.ones((2, d)), np.array([1.0, 5.0]))
    z, one = np.zeros(d), np.ones(d)
    kept, ev = [], []
    for _ in range(4):
        r = o.decode(z, one, one)
        kept.append(o.resident()[0].tolist()); ev.append(r.evicted)
    assert ev == [1, 2, 3, 4]
    assert kept == [[0, 2], [0, 3], [0, 4], [0, 5]]
    assert abs(o.score(0) - (1.0 + 4 / 3.0)) < 1e-12
    w = OracleHead(d, 1, 1, 1.0, cap=8)                      # the window rule on the same input
    w.load_and_select(np.ones((2, d)), np.ones((2, d)), np.array([1.0, 5.0]))
    assert w.decode(z, one, one).evicted == 0


def test_fixed_pattern_worked_by_hand():
    """Budget 2 + 1, fixed pattern with blocks of 3 and one summary column per block (positions
    2, 5, 8, ...), from an empty cache, equal probabilities (q = 0).
      t = 0..2 fill the cache; scores after t = 2: (11/6, 5/6, 1/3)
      t = 3: scores (25/12, 13/12, 7/12, 1/4); covered: block {3}, summary {2}; 0 and 1 compete,
             1 is lower                                                               -> {0, 2, 3}
      t = 4: covered: block {3, 4}, summary {2}; only token 0 competes and goes, the highest
             score of all                                                             -> {2, 3, 4}
      t = 5: covered: block {3, 4, 5}, summary {2, 5}: everything, so protection is void and the
             lowest score among the others goes: 2: 13/12, 3: 3/4, 4: 1/2             -> {2, 3, 5}"""
    d = 2
    o = OracleHead(d, 2, 1, 1.0, cap=8, protect=2, stride=3)
    z, one = np.zeros(d), np.ones(d)
    ev = [o.decode(z, one, one).evicted for _ in range(6)]
    assert ev == [-1, -1, -1, 1, 0, 4]
    assert o.resident()[0].tolist() == [2, 3, 5]
    np.testing.assert_allclose(o.resident()[1], [13 / 12.0, 3 / 4.0, 1 / 4.0], rtol=0, atol=1e-12)


@pytest.mark.parametrize("f32", [False, True])
def test_strided_pattern_with_a_period_longer_than_the_text_is_the_recent_window(f32):
    """(t - p) mod stride == 0 then only holds for p = t, which the band covers anyway: the
    pattern is exactly "the last `recent` positions".  Bit for bit, prompt phase included."""
    Q, K, V = make_inputs(31, 40, 4)
    for (n, heavy, recent) in [(20, 3, 4), (0, 2, 2), (25, 5, 1)]:
        _, a = run_oracle_pattern(Q, K, V, n, heavy, recent, 0.5, ("strided", 1000), score_f32=f32)
        _, b = run_oracle(Q, K, V, n, heavy, recent, 0.5, score_f32=f32)
        assert a["sets"] == b["sets"] and a["evicted"] == b["evicted"]
        assert np.array_equal(a["outs"], b["outs"])


def test_fixed_pattern_with_one_block_is_plain_lowest_score_eviction():
    """One block holding the whole text covers every cached token, so protection is always void:
    the lowest score among the tokens other than the new one goes.  That is the recent-window
    rule with a window of one (the new token) and the same total budget, once generation starts
    from an empty cache."""
    Q, K, V = make_inputs(32, 30, 4)
    _, a = run_oracle_pattern(Q, K, V, 0, 3, 2, 0.5, ("fixed", 1000))
    _, b = run_oracle(Q, K, V, 0, 4, 1, 0.5)
    assert a["sets"] == b["sets"] and a["evicted"] == b["evicted"]
    assert np.array_equal(a["outs"], b["outs"])


@pytest.mark.parametrize("pattern", [("strided", 4), ("fixed", 5)])
def test_pattern_protection_invariants(pattern):
    """Cache size, one in / at most one out, an evicted token never returns, mass conservation;
    and the point of the rule: a covered token is never evicted while an uncovered one is cached."""
    Q, K, V = make_inputs(33, 90, 4, sigma=1.0)
    n, heavy, recent = 30, 6, 3
    k = heavy + recent
    o = OracleHead(4, heavy, recent, 0.5, cap=90, protect=PATTERN_MODE[pattern[0]], stride=pattern[1])
    o.prefill(Q[:n], K[:n], V[:n])
    prev = set(o.resident()[0].tolist())
    assert len(prev) == k
    gone = set(range(n)) - prev
    for t in range(n, 90):
        r = o.decode(Q[t], K[t], V[t])
        cur = set(o.resident()[0].tolist())
        assert len(cur) == k and t in cur
        assert cur - prev == {t} and len(prev - cur) == 1 and not (cur & gone)
        cover = pattern_cover(pattern, recent, t)
        before = prev | {t}
        if r.evicted in cover:
            assert before <= cover, "a covered token went while an uncovered one was cached"
        gone |= prev - cur
        prev = cur
        pos, sc = o.resident()
        assert abs(sc.sum() + o.evicted_mass - o.queries) < 1e-9


def test_pattern_arguments():
    with pytest.raises(ValueError):
        OracleHead(4, 2, 2, 0.5, cap=8, protect=3, stride=2)
    with pytest.raises(ValueError):
        OracleHead(4, 2, 2, 0.5, cap=8, protect=1, stride=0)
