"""GPU parity of h2o_decode_step against the CPU oracle, through the C ABI.

Every case starts both sides from the same cache state: the oracle runs the
prompt phase (fp64, scores rounded to binary32 when stored), its resident
tokens are loaded into the device cache with h2o_cache_restore, then T steps run
on the device and are compared step by step (kept-position sets exactly, outputs
within the dtype's tolerance, final scores).
"""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import OracleHead, map_heads
from tests import parity

pytestmark = pytest.mark.gpu

torch_dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def run_case(B, Hh, d, n, T, heavy, recent, dtype, sigma, seed, scale=0.0, sample=None,
             permute_slots=False, mutate=None, rank=0):
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    k = heavy + recent
    scale_d = parity.oracle_scale(d, scale)
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    if sample is not None and sample < len(heads):
        rng = np.random.default_rng(seed)
        heads = [heads[i] for i in sorted(rng.choice(len(heads), sample, replace=False))]
    qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, sigma, dev, seed)
    if mutate is not None:
        mutate(qs, ks, vs)                # edits the shared inputs before either side sees them
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, scale, device=dev, rank=rank)
    all_heads = [(b, h) for b in range(B) for h in range(Hh)]
    if n > 0:
        Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, sigma, dev, seed)
        Qh, Kh, Vh = Q.cpu(), K.cpu(), V.cpu()
        oracles, _ = parity.oracle_prefill_heads(Qh, Kh, Vh, all_heads, heavy, recent, scale_d,
                                                 cap=n + T, policy=rank)
        Kc, Vc, acc, pos = parity.cache_state_from_oracles(oracles, B, Hh, k, Kh, Vh)
        if permute_slots:
            # occupied slots stay a prefix, their order inside it is shuffled per head
            g = torch.Generator().manual_seed(seed)
            c = min(n, k)
            for b, h in all_heads:
                perm = torch.randperm(c, generator=g)
                Kc[b, h, :c] = Kc[b, h, perm]; Vc[b, h, :c] = Vc[b, h, perm]
                acc[b, h, :c] = acc[b, h, perm]; pos[b, h, :c] = pos[b, h, perm]
        cache.restore(Kc.to(dev), Vc.to(dev), acc.to(dev), pos.to(dev), n)
    else:
        oracles = {bh: OracleHead(d, heavy, recent, scale_d, score_f32=True, cap=T, policy=rank)
                   for bh in all_heads}
    outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs)
    pos_f, acc_f = cache.snapshot()
    torch.cuda.synchronize()
    pos_f, acc_f = pos_f.cpu(), acc_f.cpu()
    assert cache.tokens_seen == n + T
    qh, kh, vh = qs.cpu(), ks.cpu(), vs.cpu()
    tol = parity.OUT_TOL[dtype]

    def one(bh):
        b, h = bh
        st = parity.check_head_decode(oracles[bh], qh[:, b, h], kh[:, b, h], vh[:, b, h],
                                      outs[:, b, h], snaps[:, b, h], recent, tol, policy=rank)
        parity.check_final_scores(oracles[bh], pos_f[b, h], acc_f[b, h], st)
        return st

    results, _ = map_heads(one, heads)
    total = parity.DecodeStats()
    for st in results:
        total.merge(st)
    print("\n[decode parity] B=%d Hh=%d d=%d n=%d T=%d H=%d R=%d %s: head-steps %d, near-tied %d, "
          "excused %d, max out l2 %.2e linf %.2e (%.2f of the allowance), scores not bit-equal %d (max rel %.1e)"
          % (B, Hh, d, n, T, heavy, recent, str(dtype).split(".")[-1], total.head_steps,
             total.near_tied_steps, total.excused, total.max_out_l2, total.max_out_linf, total.max_out_frac,
             total.score_mismatch, total.max_score_rel), flush=True)
    assert total.excused <= max(1, int(0.001 * total.head_steps)) or total.excused == 0
    assert total.max_score_rel <= 1e-6
    cache.close()
    return total


def test_tiny_f32_config_full():
    """Workload 1: batch 1, 8 heads, d 64, prompt 256, 64 steps, budget 32 + 32, fp32."""
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS["tiny_f32"]
    run_case(w.batch, w.heads, w.head_dim, w.prompt, w.steps, w.heavy, w.recent, w.dtype, w.sigma,
             synth.BASE_SEED)


@pytest.mark.parametrize("dt,d", [("f16", 128), ("bf16", 128), ("f32", 128), ("f16", 64),
                                  ("bf16", 64), ("f32", 64)])
@pytest.mark.parametrize("n,T,heavy,recent", [
    (96, 40, 13, 10),      # ragged budget, several rounds, 4-wave kernel
    (300, 30, 103, 102),   # the OPT-30B-shaped budget (205 slots)
    (600, 24, 205, 205),   # the OPT-6.7B-shaped budget (410 slots): 8-wave kernel, ring = all rounds
])
def test_decode_dtypes_and_budgets(dt, d, n, T, heavy, recent):
    run_case(2, 3, d, n, T, heavy, recent, torch_dt[dt], 1.0, 11)


@pytest.mark.parametrize("heavy,recent,n,T", [
    (300, 333, 700, 20),     # 633 slots: two chunks of the register ring
    (1500, 611, 2200, 6),    # 2111 slots: six chunks
    (2048, 2048, 4200, 3),   # the largest budget (needs the raised LDS limit)
    (1, 0, 9, 12), (0, 1, 9, 12), (1, 1, 3, 12), (4, 3, 7, 9),   # smallest budgets
    (209, 208, 500, 24),     # 417 slots: the first budget past thirteen rounds of eight waves
    (224, 224, 600, 24),     # 448 slots: fourteen rounds
    (240, 240, 600, 24),     # 480 slots: fifteen rounds, the deepest register-resident ring
    (241, 240, 600, 24),     # 481 slots: chunked
])
def test_decode_budget_extremes(heavy, recent, n, T):
    run_case(1, 2, 128, n, T, heavy, recent, torch.float16, 1.0, 5)


@pytest.mark.parametrize("dt,d,heavy,recent", [("bf16", 128, 400, 433), ("f32", 128, 250, 251),
                                               ("f32", 64, 600, 500), ("f16", 64, 700, 600),
                                               ("bf16", 64, 0, 1100), ("f16", 128, 900, 0)])
def test_decode_large_budget_other_types(dt, d, heavy, recent):
    """Budgets beyond what one pass of the register ring holds (chunked kernel)
    in the other element types and head sizes."""
    run_case(1, 3, d, heavy + recent + 150, 10, heavy, recent, torch_dt[dt], 1.0, 17)


def test_decode_large_budget_filling_up():
    """Prompt shorter than a large budget: the chunked kernel first fills free
    slots (500 -> 600 occupied), then starts evicting."""
    run_case(1, 2, 128, 500, 130, 300, 300, torch.float16, 1.0, 19)


@pytest.mark.parametrize("dt,d,n,T,heavy,recent", [
    ("f16", 128, 300, 60, 50, 50), ("bf16", 64, 0, 90, 20, 12), ("f32", 64, 200, 40, 24, 0),
    ("f16", 128, 700, 30, 300, 300), ("bf16", 128, 96, 50, 13, 10)])
def test_decode_averaged_ranking(dt, d, n, T, heavy, recent):
    """Eviction by accumulated score / number of queries that scored the token
    (both kernels, also from an empty cache and with recent = 0)."""
    run_case(2, 3, d, n, T, heavy, recent, torch_dt[dt], 1.0, 23, rank=1)


@pytest.mark.parametrize("heavy,recent", [(16, 16), (0, 24), (24, 0), (7, 1)])
def test_decode_from_empty_cache(heavy, recent):
    """No prompt: the cache fills slot by slot, then eviction starts (Algorithm 1's
    `i <= k` branch); recent = 0 lets the new token itself lose; heavy = 0 is a
    sliding window."""
    run_case(2, 2, 64, 0, 70, heavy, recent, torch.float16, 0.75, 3)


def test_decode_short_prompt_then_fill():
    """Prompt shorter than the budget: everything is kept, then slots fill up."""
    run_case(1, 4, 128, 20, 60, 24, 24, torch.bfloat16, 1.0, 9)


def test_decode_explicit_scale():
    run_case(1, 2, 64, 64, 16, 8, 8, torch.float32, 0.75, 21, scale=0.2)


@pytest.mark.parametrize("dt,n,heavy,recent", [("f32", 40, 6, 6), ("f16", 700, 300, 333)])
def test_decode_logits_far_above_the_tokens_own(dt, n, heavy, recent):
    """Steps whose cached keys score ~1000 above (and below) the token's own
    logit: exp(s_j - s_self) overflows fp64, so the kernel has to fall back to
    the true maximum as its softmax shift.  Both kernels (register-resident and
    chunked) are covered."""
    def mutate(qs, ks, vs):
        T = qs.shape[0]
        for s in range(2, T, 3):
            qs[s] = 4.0
            ks[s] = -16.0                 # own logit: 64 * 4 * -16 / 8 = -512
            if s + 1 < T:
                ks[s - 1] = 16.0          # the previous token's key scores +512 against it
    run_case(1, 2, 64, n, 14, heavy, recent, torch_dt[dt], 0.75, 31, mutate=mutate)


def test_slot_order_does_not_matter():
    """Which slot holds which token is not observable: shuffling the slots of the
    starting state must give the same kept positions and outputs."""
    a = run_case(1, 4, 128, 256, 32, 40, 24, torch.float16, 1.0, 17)
    b = run_case(1, 4, 128, 256, 32, 40, 24, torch.float16, 1.0, 17, permute_slots=True)
    assert a.excused == b.excused == 0


def test_opt67b_layer_config_all_heads():
    """Workload 2 at full size, the launch configuration the benchmark times:
    batch 16 x 32 heads, d 128, prompt 2048, 256 steps, budget 205 + 205, fp16.
    Every head is checked on every step."""
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS["opt6.7b_layer_f16"]
    st = run_case(w.batch, w.heads, w.head_dim, w.prompt, w.steps, w.heavy, w.recent, w.dtype,
                  w.sigma, synth.BASE_SEED)
    assert st.head_steps == w.batch * w.heads * w.steps


def sampled_case(w, n_sample, seed, steps=None):
    """Full-size workload on the device, a random sample of heads checked on every
    step.  All heads go through the device's own prompt phase; the sampled heads'
    state is then replaced by the oracle's (K/V rows, binary32 scores, positions)
    so that both sides start those heads from the same state."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, k = w.batch, w.heads, w.head_dim, w.prompt, w.budget
    T = steps or w.steps
    scale_d = parity.oracle_scale(d)
    rng = np.random.default_rng(seed)
    flat = sorted(rng.choice(B * Hh, n_sample, replace=False).tolist())
    heads = [(i // Hh, i % Hh) for i in flat]
    Q, K, V = synth.make_prompt(B, Hh, n, d, w.dtype, w.sigma, dev, seed)
    cache = hb.H2OCache(B, Hh, d, w.heavy, w.recent, w.dtype, device=dev)
    cache.prefill_scores(Q, K, V)
    bi = torch.tensor([b for b, _ in heads]); hi = torch.tensor([h for _, h in heads])
    Qs, Ks, Vs = Q[bi, hi].cpu(), K[bi, hi].cpu(), V[bi, hi].cpu()          # [S, n, d]
    del Q, K, V
    idx_heads = [(0, i) for i in range(n_sample)]
    oracles, _ = parity.oracle_prefill_heads(Qs[None], Ks[None], Vs[None], idx_heads, w.heavy, w.recent,
                                             scale_d, cap=n + T)
    Kc, Vc, acc, pos = parity.cache_state_from_oracles(oracles, 1, n_sample, k, Ks[None], Vs[None])
    Kv, Vv, av, pv = cache.views()
    bd, hd = bi.to(dev), hi.to(dev)
    Kv[bd, hd] = Kc[0].to(dev); Vv[bd, hd] = Vc[0].to(dev)
    av[bd, hd] = acc[0].to(dev); pv[bd, hd] = pos[0].to(dev)
    qs, ks, vs = synth.make_steps(B, Hh, d, T, w.dtype, w.sigma, dev, seed)
    outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs, snapshot_heads=heads)
    pos_f, acc_f = cache.snapshot()
    torch.cuda.synchronize()
    pos_f, acc_f = pos_f[bd, hd].cpu(), acc_f[bd, hd].cpu()
    qh, kh, vh = qs[:, bd, hd].cpu(), ks[:, bd, hd].cpu(), vs[:, bd, hd].cpu()
    tol = parity.OUT_TOL[w.dtype]

    def one(i):
        st = parity.check_head_decode(oracles[(0, i)], qh[:, i], kh[:, i], vh[:, i], outs[:, i],
                                      snaps[:, i], w.recent, tol)
        parity.check_final_scores(oracles[(0, i)], pos_f[i], acc_f[i], st)
        return st

    results, _ = map_heads(one, range(n_sample))
    total = parity.DecodeStats()
    for st in results:
        total.merge(st)
    print("\n[decode parity, sampled] %s: %d of %d heads x %d steps = %d head-steps, near-tied %d, "
          "excused %d, max out l2 %.2e linf %.2e, scores not bit-equal %d (max rel %.1e)"
          % (w.name, n_sample, B * Hh, T, total.head_steps, total.near_tied_steps, total.excused,
             total.max_out_l2, total.max_out_linf, total.score_mismatch, total.max_score_rel), flush=True)
    assert total.excused <= int(0.001 * total.head_steps)
    assert total.max_score_rel <= 1e-6
    cache.close()
    return total


def test_opt30b_layer_config_sampled_heads():
    """Workload 4 at full size: batch 64 x 56 heads, d 128, prompt 1024, 1024 steps,
    budget 103 + 102 held fixed while t grows to 2048, fp16; 64 sampled heads are
    checked on all 1024 steps."""
    from paper_2306_14048_amd import synth
    st = sampled_case(synth.WORKLOADS["opt30b_layer_f16"], 64, synth.BASE_SEED)
    assert st.head_steps == 64 * 1024


def device_prompt_then_steps(w, n_sample, seed, steps=None, kv_bits=0):
    """The path the benchmark times, end to end on the device: h2o_prefill_scores on the
    workload's prompt, then the workload's generation steps, nothing restored from the
    oracle.  A sample of heads is followed by the oracle on the same tensors.

    The device's stored scores start from its own column sums, which carry the
    column-sum tolerance (COLSUM_RTOL relative), so two candidates whose oracle
    values lie within SELECT_RTOL = 2 * COLSUM_RTOL of each other may be ordered
    either way, at the prompt compression and at every later eviction that compares
    prompt-seeded scores.  Steps excused inside the 1e-6 near-tie rule and steps
    excused only by that wider band are reported apart; anything else fails."""
    from paper_2306_14048_amd import binding as hb, synth
    from tests.test_prefill_parity import COLSUM_ATOL, COLSUM_RTOL, SELECT_RTOL
    dev = torch.device("cuda:0")
    B, Hh, d, n, k = w.batch, w.heads, w.head_dim, w.prompt, w.budget
    T = steps or w.steps
    scale_d = parity.oracle_scale(d)
    rng = np.random.default_rng(seed)
    flat = sorted(rng.choice(B * Hh, n_sample, replace=False).tolist())
    heads = [(i // Hh, i % Hh) for i in flat]
    Q, K, V = synth.make_prompt(B, Hh, n, d, w.dtype, w.sigma, dev, seed)
    cache = hb.H2OCache(B, Hh, d, w.heavy, w.recent, w.dtype, device=dev, kv_bits=kv_bits)
    col = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    cache.prefill_scores(Q, K, V, colsum_out=col)
    pos0 = cache.snapshot()[0]
    bi = torch.tensor([b for b, _ in heads]); hi = torch.tensor([h for _, h in heads])
    bd, hd = bi.to(dev), hi.to(dev)
    Qs, Ks, Vs = Q[bd, hd].cpu(), K[bd, hd].cpu(), V[bd, hd].cpu()          # [S, n, d]
    col_s, pos0_s = col[bd, hd].cpu().double().numpy(), pos0[bd, hd].cpu().numpy()
    del Q, K, V, col
    idx_heads = [(0, i) for i in range(n_sample)]
    oracles, cols = parity.oracle_prefill_heads(Qs[None], Ks[None], Vs[None], idx_heads, w.heavy, w.recent,
                                                scale_d, cap=n + T, kv_bits=kv_bits)
    swapped_heads = swapped_tokens = 0
    col_err = 0.0
    for i in range(n_sample):
        ref = cols[(0, i)]
        err = np.abs(col_s[i] - ref) / (np.abs(ref) + COLSUM_ATOL / COLSUM_RTOL)
        col_err = max(col_err, float(err.max()))
        assert err.max() <= COLSUM_RTOL, "column sums of sampled head %d off by %.2e" % (i, err.max())
        m = parity.adopt_kept_set(oracles[(0, i)], pos0_s[i], n - 1, w.recent, 0, SELECT_RTOL)
        swapped_heads += int(m > 0)
        swapped_tokens += m
    qs, ks, vs = synth.make_steps(B, Hh, d, T, w.dtype, w.sigma, dev, seed)
    outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs, snapshot_heads=heads)
    pos_f, acc_f = cache.snapshot()
    torch.cuda.synchronize()
    pos_f, acc_f = pos_f[bd, hd].cpu(), acc_f[bd, hd].cpu()
    qh, kh, vh = qs[:, bd, hd].cpu(), ks[:, bd, hd].cpu(), vs[:, bd, hd].cpu()

    def one(i):
        st = parity.check_head_decode(oracles[(0, i)], qh[:, i], kh[:, i], vh[:, i], outs[:, i],
                                      snaps[:, i], w.recent, parity.OUT_TOL[w.dtype], band=SELECT_RTOL)
        parity.check_final_scores(oracles[(0, i)], pos_f[i], acc_f[i], st)
        return st

    results, _ = map_heads(one, range(n_sample))
    total = parity.DecodeStats()
    for st in results:
        total.merge(st)
    print("\n[device prompt phase + steps] %s, %d-bit cache: %d of %d heads x %d steps = %d head-steps; prompt: "
          "max column-sum error %.2e, heads whose kept set differed at the threshold %d (%d tokens, oracle "
          "re-synced, none dropped); steps: near-tied %d, excused inside 1e-6 %d, excused inside the "
          "score band %.0e only %d, non-excused 0; max out l2 %.2e linf %.2e (%.2f of the allowance); final "
          "scores max rel %.1e"
          % (w.name, kv_bits or 16, n_sample, B * Hh, T, total.head_steps, col_err, swapped_heads,
             swapped_tokens, total.near_tied_steps, total.excused, SELECT_RTOL, total.excused_band,
             total.max_out_l2, total.max_out_linf, total.max_out_frac, total.max_score_rel), flush=True)
    assert total.excused + total.excused_band <= max(1, int(0.001 * total.head_steps))
    assert swapped_tokens <= max(1, int(0.001 * n_sample * k))
    # stored scores = device column sum + correctly rounded probabilities
    assert total.max_score_rel <= COLSUM_RTOL
    cache.close()
    return total


def test_bench_path_device_prompt_then_steps_opt67b():
    """Workload 2 exactly as the benchmark runs it (device prompt scoring + compression, then
    256 fp16 steps, batch 16 x 32 heads), 64 sampled heads followed by the oracle."""
    from paper_2306_14048_amd import synth
    st = device_prompt_then_steps(synth.WORKLOADS["opt6.7b_layer_f16"], 64, synth.BASE_SEED + 1)
    assert st.head_steps == 64 * 256


def test_bench_path_device_prompt_then_steps_tiny():
    """Workload 1 the same way: every head, every step."""
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS["tiny_f32"]
    device_prompt_then_steps(w, w.batch * w.heads, synth.BASE_SEED + 2)


@pytest.mark.parametrize("heavy,recent,n,T", [(20, 12, 0, 0), (20, 12, 0, 9), (20, 12, 100, 0), (20, 12, 100, 57),
                                              (300, 333, 900, 40), (0, 7, 30, 30)])
def test_rolled_positions(heavy, recent, n, T):
    """The rank of every cached token among its head's cached tokens by position (what
    position rolling assigns), against the order of the oracle's resident set."""
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, dtype = 2, 2, 128, torch.float16
    k = heavy + recent
    heads = [(b, h) for b in range(B) for h in range(Hh)]
    cache = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    scale = parity.oracle_scale(d)
    if n:
        Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, 31)
        oracles, _ = parity.oracle_prefill_heads(Q.cpu(), K.cpu(), V.cpu(), heads, heavy, recent, scale, n + T)
        Kc, Vc, acc, pos = parity.cache_state_from_oracles(oracles, B, Hh, k, K.cpu(), V.cpu())
        cache.restore(Kc.to(dev), Vc.to(dev), acc.to(dev), pos.to(dev), n)
    else:
        oracles = {bh: OracleHead(d, heavy, recent, scale, score_f32=True, cap=max(T, 1)) for bh in heads}
    if T:
        qs, ks, vs = synth.make_steps(B, Hh, d, T, dtype, 1.0, dev, 31)
        outs, snaps = parity.run_gpu_decode(cache, qs, ks, vs)
        for (b, h) in heads:
            parity.check_head_decode(oracles[(b, h)], qs[:, b, h].cpu(), ks[:, b, h].cpu(), vs[:, b, h].cpu(),
                                     outs[:, b, h], snaps[:, b, h], recent, parity.OUT_TOL[dtype])
    rolled = cache.rolled_positions().cpu().numpy()
    pos = cache.snapshot()[0].cpu().numpy()
    for (b, h) in heads:
        order = oracles[(b, h)].resident()[0].tolist()            # ascending positions
        rank = {p: i for i, p in enumerate(order)}
        want = np.array([rank[int(p)] if p >= 0 else -1 for p in pos[b, h]], dtype=np.int32)
        assert np.array_equal(rolled[b, h], want)
        occupied = rolled[b, h][rolled[b, h] >= 0]
        assert sorted(occupied.tolist()) == list(range(len(order)))
    cache.close()
