"""GPU parity of the prompt-phase attention kernel (causal attention output +
row statistics) and of the one-call prompt phase built on it (attention, column
sums from the attention's row statistics, compression) against the CPU oracle,
through the C ABI."""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead, map_heads
from tests import parity
from tests.test_prefill_parity import COLSUM_ATOL, COLSUM_RTOL, ROW_MASS_RTOL, SELECT_RTOL

pytestmark = pytest.mark.gpu

torch_dt = {"f16": torch.float16, "bf16": torch.bfloat16}


def oracle_prompt(Qc, Kc, Vc, heads, heavy, recent, scale_d, n):
    """Oracle prompt phase per head: (oracle, column sums, attention rows)."""
    def one(bh):
        b, h = bh
        o = OracleHead(Qc.shape[-1], heavy, recent, scale_d, score_f32=True, cap=n)
        col, attn = o.prefill(parity.host64(Qc[b, h]), parity.host64(Kc[b, h]),
                              parity.host64(Vc[b, h]), want_attn=True)
        return o, col, attn
    res, _ = map_heads(one, heads)
    return {bh: r for bh, r in zip(heads, res)}


def check_rows(got, ref, dtype, where):
    """Output bar of the generation step applied to every prompt row (vector of
    head_dim values): L2 and element-wise bounds of parity.output_error."""
    assert np.all(np.isfinite(got)), where
    f_l2, f_el, l2, li = parity.output_error(got, ref, dtype, p_rounded=True)
    assert f_l2.max() <= 1.0, "%s: row %d L2 error %.3e = %.2f of its allowance" % (
        where, int(f_l2.argmax()), l2[f_l2.argmax()], f_l2.max())
    assert f_el.max() <= 1.0, "%s: row %d element error %.3e = %.2f of its allowance" % (
        where, int(f_el.argmax()), li[f_el.argmax()], f_el.max())
    return float(l2.max()), float(li.max())


def attention_case(B, Hh, d, n, dtype, sigma, seed, scale=0.0):
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
    cfg = hb.make_config(B, Hh, d, 1, 1, dtype, scale)
    need = hb.h2o_prefill_attention_workspace_bytes(cfg, n)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = torch.empty_like(Q)
    lse = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    hb.h2o_prefill_attention(cfg, Q, K, V, n, ws, need, out, lse)
    torch.cuda.synchronize()
    got, lse = out.cpu().double().numpy(), lse.cpu().double().numpy()
    scale_d = parity.oracle_scale(d, scale)
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    ref = oracle_prompt(Q.cpu(), K.cpu(), V.cpu(), heads, 1, 1, scale_d, n)
    worst = (0.0, 0.0)
    Qd, Kd = Q.cpu().double().numpy(), K.cpu().double().numpy()
    for (b, h) in heads:
        e = check_rows(got[b, h], ref[(b, h)][2], dtype, "head (%d, %d)" % (b, h))
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        # by-product: the row log-sum-exp (consistency with a float64 evaluation of
        # its definition; its use, the column sums, is checked against the oracle below)
        S = scale_d * (Qd[b, h] @ Kd[b, h].T)
        S[np.triu_indices(n, 1)] = -np.inf
        m = S.max(-1)
        ref_lse = m + np.log(np.exp(S - m[:, None]).sum(-1))
        assert np.abs(lse[b, h] - ref_lse).max() <= 2e-5 * max(1.0, np.abs(ref_lse).max())
    print("\n[attention] B=%d Hh=%d d=%d n=%d %s: worst row L2 %.2e, max %.2e"
          % (B, Hh, d, n, str(dtype).split(".")[-1], worst[0], worst[1]), flush=True)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n", [1, 17, 64, 129, 300])
def test_attention_small_and_ragged(dt, d, n):
    attention_case(2, 3, d, n, torch_dt[dt], 1.0, 200 + n)


@pytest.mark.parametrize("dt,n", [("bf16", 1000), ("f16", 777)])
def test_attention_several_blocks(dt, n):
    attention_case(1, 4, 128, n, torch_dt[dt], 1.0, 9)


def test_attention_explicit_scale_heavy_tail():
    attention_case(1, 2, 64, 260, torch.float16, 1.25, 4, scale=0.3)


def layer_case(B, Hh, d, n, heavy, recent, dtype, sigma, seed):
    """h2o_prefill_attention_scores against the oracle's prompt phase: attention
    rows, column sums, kept sets (threshold rule of the scoring tests)."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    k = heavy + recent
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    need = hb.h2o_prefill_attention_workspace_bytes(cache.cfg, n)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = torch.empty_like(Q)
    col = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    hb.h2o_prefill_attention_scores(cache.handle, Q, K, V, n, ws, need, out, col)
    assert cache.tokens_seen == n
    pos, acc = cache.snapshot()
    torch.cuda.synchronize()
    pos, acc, col = pos.cpu().numpy(), acc.cpu().numpy(), col.cpu().double().numpy()
    got = out.cpu().double().numpy()
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    ref = oracle_prompt(Q.cpu(), K.cpu(), V.cpu(), heads, heavy, recent, parity.oracle_scale(d), n)
    flips = 0
    for (b, h) in heads:
        o, rcol, rattn = ref[(b, h)]
        check_rows(got[b, h], rattn, dtype, "head (%d, %d)" % (b, h))
        assert np.all(np.abs(col[b, h] - rcol) <= COLSUM_RTOL * np.abs(rcol) + COLSUM_ATOL)
        rp, _ = o.resident()
        gp = pos[b, h][pos[b, h] >= 0]
        assert len(gp) == len(rp) == min(n, k)
        assert np.all(np.diff(gp) > 0)
        assert np.array_equal(acc[b, h][:len(gp)], col[b, h][gp].astype(np.float32))
        diff = set(gp.tolist()) ^ set(rp.tolist())
        if diff:
            thr = np.sort(rcol[: n - recent])[::-1][heavy - 1]
            for j in diff:
                assert j < n - recent and abs(rcol[j] - thr) <= SELECT_RTOL * thr
            flips += len(diff) // 2
    print("\n[prompt layer] B=%d Hh=%d d=%d n=%d H=%d R=%d %s: heads %d, threshold flips %d"
          % (B, Hh, d, n, heavy, recent, str(dtype).split(".")[-1], len(heads), flips), flush=True)
    # a second prompt without a reset is refused, a reset allows it again
    with pytest.raises(hb.H2OError) as ei:
        hb.h2o_prefill_attention_scores(cache.handle, Q, K, V, n, ws, need, out, None)
    assert ei.value.status == hb.H2O_ESTATE
    cache.close()
    return flips


@pytest.mark.parametrize("dt,d,n,heavy,recent", [("bf16", 128, 640, 64, 64), ("f16", 64, 300, 30, 30),
                                                 ("f16", 128, 100, 64, 64)])
def test_prompt_layer_end_to_end(dt, d, n, heavy, recent):
    layer_case(2, 2, d, n, heavy, recent, torch_dt[dt], 1.0, 21)


def test_prompt_layer_then_generation_matches_scores_path():
    """The cache that the attention-based prompt phase leaves behind continues
    exactly like the one the two-pass scoring leaves behind (same kept tokens,
    same outputs over 16 steps)."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, heavy, recent, dtype = 2, 4, 128, 520, 40, 40, torch.float16
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 31)
    qs, ks, vs = synth.make_steps(B, Hh, d, 16, dtype, 1.0, dev, 31)
    a = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    b = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    a.prefill_scores(Q, K, V)
    need = hb.h2o_prefill_attention_workspace_bytes(b.cfg, n)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = torch.empty_like(Q)
    hb.h2o_prefill_attention_scores(b.handle, Q, K, V, n, ws, need, out, None)
    pa, _ = a.snapshot()
    pb, _ = b.snapshot()
    if not torch.equal(pa, pb):
        pytest.skip("a score within rounding of the selection threshold differs between the two "
                    "row-statistics kernels for this seed; nothing to compare step by step")
    oa, ob = torch.empty((B, Hh, d), dtype=dtype, device=dev), torch.empty((B, Hh, d), dtype=dtype, device=dev)
    for s in range(16):
        a.decode_step(qs[s], ks[s], vs[s], oa)
        b.decode_step(qs[s], ks[s], vs[s], ob)
        assert torch.equal(a.snapshot()[0], b.snapshot()[0])
        assert torch.allclose(oa.float(), ob.float(), rtol=2e-3, atol=1e-4)
    a.close(); b.close()


def test_prompt_layer_bf16_config_full():
    """Workload 3 at full size through the attention-based prompt phase: batch
    4 x 32 heads, d 128, prompt 4096, bf16, budget 410 + 409; every head and
    every row checked against the oracle."""
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS["prefill_bf16"]
    flips = layer_case(w.batch, w.heads, w.head_dim, w.prompt, w.heavy, w.recent, w.dtype, w.sigma,
                       synth.BASE_SEED)
    assert flips <= 0.001 * w.batch * w.heads * w.budget


def test_attention_rejects_f32():
    from paper_2306_14048_amd import binding as hb
    cfg = hb.make_config(1, 1, 64, 4, 4, torch.float32)
    assert hb.h2o_prefill_attention_workspace_bytes(cfg, 64) == 0
    x = torch.zeros((1, 1, 64, 64), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(hb.H2OError) as ei:
        hb.h2o_prefill_attention(cfg, x, x, x, 64, ws, ws.numel(), x, None)
    assert ei.value.status == hb.H2O_EUNSUPPORTED


def test_largest_prompt_sampled():
    """The largest supported prompt (65536 tokens), one head, in the launch shape
    any caller gets: attention rows and row log-sum-exps of sampled queries, and
    the column sums of the last columns (each needs only its own rows), against a
    float64 evaluation of the definitions on the same tensors; plus what holds at
    any size: the column sums are positive and add up to n.  (The oracle's prompt
    phase is quadratic and would take hours here.)"""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, dtype = 1, 1, 64, hb.H2O_MAX_PROMPT, torch.float16
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 41)
    cache = hb.H2OCache(B, Hh, d, 2048, 2048, dtype, device=dev)
    need = hb.h2o_prefill_attention_workspace_bytes(cache.cfg, n)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = torch.empty_like(Q)
    col = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    hb.h2o_prefill_attention_scores(cache.handle, Q, K, V, n, ws, need, out, col)
    lse = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    hb.h2o_prefill_attention(cache.cfg, Q, K, V, n, ws, need, out, lse)
    col2 = hb.prefill_colsum(cache.cfg, Q, K)                 # the two-pass scoring path
    torch.cuda.synchronize()
    Qd, Kd, Vd = (x[0, 0].cpu().double().numpy() for x in (Q, K, V))
    got, lse, col, col2 = (x[0, 0].cpu().double().numpy() for x in (out, lse, col, col2))
    scale = parity.oracle_scale(d)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 255, 256, n - 1], rng.integers(0, n, 40)]))
    ref_lse_all = {}
    for i in rows:
        s = scale * (Kd[: i + 1] @ Qd[i])
        m = s.max()
        e = np.exp(s - m)
        ref_lse_all[int(i)] = m + np.log(e.sum())
        ref = (e / e.sum()) @ Vd[: i + 1]
        check_rows(got[i][None], ref[None], dtype, "row %d" % i)
        assert abs(lse[i] - ref_lse_all[int(i)]) <= 2e-5 * max(1.0, abs(ref_lse_all[int(i)]))
    # last columns: c_j = sum_{i >= j} exp(s_ij - LSE_i) with every LSE_i from float64
    tail = 48
    S = scale * (Qd[n - tail:] @ Kd.T)                        # rows n-tail .. n-1, all keys
    for r in range(tail):
        S[r, n - tail + r + 1:] = -np.inf
    m = S.max(-1, keepdims=True)
    L = m[:, 0] + np.log(np.exp(S - m).sum(-1))
    P = np.exp(S - L[:, None])
    ref_tail = np.array([P[j - (n - tail):, j].sum() for j in range(n - tail, n)])
    for c in (col, col2):
        assert np.all(np.abs(c[n - tail:] - ref_tail) <= COLSUM_RTOL * ref_tail + COLSUM_ATOL)
        assert np.all(c > 0) and np.all(np.isfinite(c))
        print("\n[longest prompt] sum of column sums off by %.2e n, last columns off by %.2e"
              % (abs(c.sum() - n) / n, float((np.abs(c[n - tail:] - ref_tail) / ref_tail).max())), flush=True)
        assert abs(c.sum() - n) <= ROW_MASS_RTOL * n
    # the two scoring paths agree column by column
    assert np.all(np.abs(col - col2) <= 2 * COLSUM_RTOL * np.abs(col2) + COLSUM_ATOL)
    # compression: budget 4096 of 65536, window resident, positions ascending
    pos, _ = cache.snapshot()
    pos = pos[0, 0].cpu().numpy()
    assert np.all(np.diff(pos) > 0) and pos[-2048:].tolist() == list(range(n - 2048, n))
    cache.close()
