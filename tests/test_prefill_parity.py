"""GPU parity of the prompt phase (column-sum scoring on the matrix cores and
the select + gather compression) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead, map_heads
from tests import parity

pytestmark = pytest.mark.gpu

torch_dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

# Column sums: the device forms the logits on the matrix cores (exact products of
# 16-bit inputs, fp32 accumulation over d <= 128 terms), scales and exponentiates in
# fp32 (v_exp_f32 / v_log_f32, about 1 ulp each) at logits of magnitude up to ~1e2,
# where one fp32 ulp of the scaled logit is already 8e-6 relative in the exponential,
# and adds up to n terms in fp32.  Measured over every case of this file and the
# full-size workloads: at most 1.0e-5 relative (binary32 inputs; 7.6e-6 for 16-bit
# inputs).  The bar is three times that, plus an absolute floor for sums that
# underflow binary32; every case prints its measured maximum.
COLSUM_RTOL = 3e-5
COLSUM_ATOL = 1e-30
# Every softmax row sums to one, so a head's column sums add up to n (measured: 4e-7 n).
ROW_MASS_RTOL = 2e-6
# A token can change sides of the selection threshold only if its score is
# within twice the column-sum tolerance of the threshold score.
SELECT_RTOL = 2 * COLSUM_RTOL


def oracle_colsums(Q, K, V, scale_d):
    B, Hh, n, d = Q.shape
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    Qh, Kh, Vh = Q.cpu(), K.cpu(), V.cpu()

    def one(bh):
        b, h = bh
        o = OracleHead(d, 1, 1, scale_d, cap=n)
        return o.prefill(parity.host64(Qh[b, h]), parity.host64(Kh[b, h]), parity.host64(Vh[b, h]))[0]

    res, _ = map_heads(one, heads)
    return np.stack(res).reshape(B, Hh, n)


def colsum_case(B, Hh, d, n, dtype, sigma, seed, scale=0.0):
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
    cfg = hb.make_config(B, Hh, d, 1, 1, dtype, scale)
    got = hb.prefill_colsum(cfg, Q, K)
    torch.cuda.synchronize()
    got = got.cpu().double().numpy()
    ref = oracle_colsums(Q, K, V, parity.oracle_scale(d, scale))
    err = np.abs(got - ref) / (COLSUM_RTOL * np.abs(ref) + COLSUM_ATOL)
    print("\n[colsum] B=%d Hh=%d d=%d n=%d %s: max rel err %.2e, row-mass error %.2e"
          % (B, Hh, d, n, str(dtype).split(".")[-1],
             float((np.abs(got - ref) / np.maximum(np.abs(ref), 1e-20)).max()),
             float(np.abs(got.sum(-1) - n).max() / n)), flush=True)
    assert np.all(np.isfinite(got))
    assert err.max() <= 1.0, "column sums off by %.2f tolerances" % err.max()
    # every softmax row sums to one, so the column sums add up to n
    assert np.abs(got.sum(-1) - n).max() <= ROW_MASS_RTOL * n
    return got, ref


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n", [1, 17, 64, 129, 300])
def test_colsum_small_and_ragged(dt, d, n):
    colsum_case(2, 3, d, n, torch_dt[dt], 1.0, 100 + n)


@pytest.mark.parametrize("dt,n", [("bf16", 1000), ("f16", 777), ("f32", 515)])
def test_colsum_several_blocks(dt, n):
    colsum_case(1, 4, 128, n, torch_dt[dt], 1.0, 7)


def test_colsum_explicit_scale_heavy_tail():
    colsum_case(1, 2, 64, 260, torch.bfloat16, 1.25, 3, scale=0.3)


def select_case(B, Hh, d, n, heavy, recent, dtype, score, seed, rank=0):
    """Device select+gather on given scores against the oracle's compression of
    the same scores: same kept positions in ascending slot order, identical
    rows, identical scores."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    k = heavy + recent
    _, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, seed)
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev, rank=rank)
    sc = torch.from_numpy(score.astype(np.float32)).to(dev)
    cache.prefill_select(K, V, sc)
    pos, acc = cache.snapshot()
    Kc, Vc = cache.kv_views()
    torch.cuda.synchronize()
    assert cache.tokens_seen == n
    pos, acc, Kc, Vc = pos.cpu(), acc.cpu(), Kc.cpu(), Vc.cpu()
    Kh, Vh = K.cpu(), V.cpu()
    for b in range(B):
        for h in range(Hh):
            o = OracleHead(d, heavy, recent, 1.0, score_f32=True, cap=n, policy=rank)
            o.load_and_select(parity.host64(Kh[b, h]), parity.host64(Vh[b, h]),
                              score[b, h].astype(np.float32).astype(np.float64))
            rp, rs = o.resident()
            c = len(rp)
            assert pos[b, h, :c].tolist() == rp.tolist(), "kept positions differ (b=%d h=%d)" % (b, h)
            assert torch.all(pos[b, h, c:] == -1)
            assert np.array_equal(acc[b, h, :c].double().numpy(), rs)
            idx = torch.from_numpy(rp.astype(np.int64))
            assert torch.equal(Kc[b, h, :c].view(torch.uint8), Kh[b, h, idx].view(torch.uint8))
            assert torch.equal(Vc[b, h, :c].view(torch.uint8), Vh[b, h, idx].view(torch.uint8))
    cache.close()


@pytest.mark.parametrize("n,heavy,recent", [(50, 6, 9), (300, 64, 64), (1000, 103, 102),
                                            (4096, 410, 409), (40, 30, 30), (64, 32, 32),
                                            (65, 32, 32), (200, 0, 16), (200, 16, 0), (9000, 2048, 2048)])
@pytest.mark.parametrize("kind", ["random", "ties", "signed"])
def test_select_gather_exact(n, heavy, recent, kind):
    rng = np.random.default_rng(n * 7 + len(kind))
    B, Hh = 2, 2
    if kind == "random":
        score = rng.random((B, Hh, n)) * 5
    elif kind == "ties":
        score = np.round(rng.random((B, Hh, n)) * 6) / 4      # a handful of distinct values
    else:
        score = rng.standard_normal((B, Hh, n))
        score[..., ::7] = 0.0
        score[..., 3::11] = -0.0
    select_case(B, Hh, 128, n, heavy, recent, torch.float16, score, 5)


@pytest.mark.parametrize("n,heavy,recent", [(50, 6, 9), (1000, 103, 102), (4096, 410, 409), (200, 16, 0)])
@pytest.mark.parametrize("kind", ["random", "ties"])
def test_select_gather_averaged_ranking(n, heavy, recent, kind):
    """Prompt compression with the older tokens ranked by score / (n - position)."""
    rng = np.random.default_rng(n * 13 + len(kind))
    B, Hh = 2, 2
    if kind == "random":
        score = rng.random((B, Hh, n)) * 5
    else:
        # equal AVERAGES on purpose: score proportional to the number of queries
        score = np.round(rng.random((B, Hh, n)) * 3 + 1) * (n - np.arange(n)) / 8.0
    select_case(B, Hh, 128, n, heavy, recent, torch.float16, score, 5, rank=1)


def test_select_gather_other_row_sizes():
    rng = np.random.default_rng(1)
    select_case(1, 2, 64, 333, 20, 13, torch.bfloat16, rng.random((1, 2, 333)), 2)
    select_case(1, 2, 128, 333, 20, 13, torch.float32, rng.random((1, 2, 333)), 2)


def scores_case(B, Hh, d, n, heavy, recent, dtype, sigma, seed):
    """Whole prompt phase on the device against the oracle's: column sums within
    tolerance; kept sets equal except for tokens whose oracle score lies within
    SELECT_RTOL of the selection threshold."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    k = heavy + recent
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    col = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    cache.prefill_scores(Q, K, V, colsum_out=col)
    pos, acc = cache.snapshot()
    torch.cuda.synchronize()
    pos, acc, col = pos.cpu().numpy(), acc.cpu().numpy(), col.cpu().double().numpy()
    scale_d = parity.oracle_scale(d)
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    oracles, cols = parity.oracle_prefill_heads(Q.cpu(), K.cpu(), V.cpu(), heads, heavy, recent,
                                                scale_d, cap=n)
    flips = 0
    worst = 0.0
    for (b, h) in heads:
        ref = cols[(b, h)]
        worst = max(worst, float((np.abs(col[b, h] - ref) / (np.abs(ref) + COLSUM_ATOL / COLSUM_RTOL)).max()))
        assert np.all(np.abs(col[b, h] - ref) <= COLSUM_RTOL * np.abs(ref) + COLSUM_ATOL), \
            "column sums off by %.2e relative" % worst
        rp, rs = oracles[(b, h)].resident()
        gp = pos[b, h][pos[b, h] >= 0]
        assert len(gp) == len(rp) == min(n, k)
        assert np.all(np.diff(gp) > 0), "slots must hold ascending positions"
        # scores stored are the device's own column sums of those tokens
        assert np.array_equal(acc[b, h][:len(gp)], col[b, h][gp].astype(np.float32))
        diff = set(gp.tolist()) ^ set(rp.tolist())
        if diff:
            older = np.sort(ref[: n - recent])[::-1]
            thr = older[heavy - 1]                     # oracle's heavy-th best older score
            for j in diff:
                assert j < n - recent
                assert abs(ref[j] - thr) <= SELECT_RTOL * thr, \
                    "token %d (score %.9g) changed sides of threshold %.9g" % (j, ref[j], thr)
            flips += len(diff) // 2
    print("\n[prefill] B=%d Hh=%d d=%d n=%d H=%d R=%d %s: heads %d, max column-sum error %.2e, threshold flips %d"
          % (B, Hh, d, n, heavy, recent, str(dtype).split(".")[-1], len(heads), worst, flips), flush=True)
    cache.close()
    return flips


@pytest.mark.parametrize("dt,d,n,heavy,recent", [("bf16", 128, 640, 64, 64), ("f16", 64, 300, 30, 30),
                                                 ("f32", 64, 256, 32, 32), ("f16", 128, 100, 64, 64)])
def test_prefill_scores_end_to_end(dt, d, n, heavy, recent):
    scores_case(2, 2, d, n, heavy, recent, torch_dt[dt], 1.0, 13)


def test_prefill_bf16_config_full():
    """Workload 3 at full size: batch 4 x 32 heads, d 128, prompt 4096, bf16,
    budget 410 + 409; every head checked against the oracle."""
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS["prefill_bf16"]
    flips = scores_case(w.batch, w.heads, w.head_dim, w.prompt, w.heavy, w.recent, w.dtype, w.sigma,
                        synth.BASE_SEED)
    assert flips <= 0.001 * w.batch * w.heads * w.budget
