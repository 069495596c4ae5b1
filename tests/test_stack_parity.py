"""Workload 5: a 32-layer stack of H2O attention, all layer caches resident in
HBM at once (27.5 GB), long prompt, small budget.  Sampled (layer, batch, head)
triples are checked on every step; generation visits the layers in turn within
each token step, as a model would."""
import numpy as np
import pytest
import torch

from oracle.h2o_oracle import map_heads
from tests import parity

pytestmark = pytest.mark.gpu


def stack_case(w, layers, n_sample, seed, steps):
    from paper_2306_14048_amd import binding as hb, synth
    dev = torch.device("cuda:0")
    B, Hh, d, n, k = w.batch, w.heads, w.head_dim, w.prompt, w.budget
    T = steps
    scale_d = parity.oracle_scale(d)
    rng = np.random.default_rng(seed)
    picks = sorted(rng.choice(layers * B * Hh, n_sample, replace=False).tolist())
    triples = [(p // (B * Hh), (p // Hh) % B, p % Hh) for p in picks]
    caches, prompts = [], {}
    for layer in range(layers):
        Q, K, V = synth.make_prompt(B, Hh, n, d, w.dtype, w.sigma, dev, seed, layer=layer)
        cache = hb.H2OCache(B, Hh, d, w.heavy, w.recent, w.dtype, device=dev)
        cache.prefill_scores(Q, K, V)
        for (l, b, h) in triples:
            if l == layer:
                prompts[(l, b, h)] = (Q[b, h].cpu(), K[b, h].cpu(), V[b, h].cpu())
        torch.cuda.synchronize()
        cache._ws = None
        del Q, K, V
        caches.append(cache)
        print("layer %d scored and compressed" % layer, flush=True)

    # oracle prompt phase for the sampled triples; their device state is replaced by the oracle's
    def pre(tr):
        Qh, Kh, Vh = prompts[tr]
        o, _ = parity.oracle_prefill_heads(Qh[None, None], Kh[None, None], Vh[None, None], [(0, 0)],
                                           w.heavy, w.recent, scale_d, cap=n + T, threads=1)
        return o[(0, 0)]

    oracles, _ = map_heads(pre, triples)
    oracles = dict(zip(triples, oracles))
    print("oracle prompt phase done for %d sampled heads" % n_sample, flush=True)
    for tr in triples:
        l, b, h = tr
        _, Kh, Vh = prompts[tr]
        Kc, Vc, acc, pos = parity.cache_state_from_oracles({(0, 0): oracles[tr]}, 1, 1, k,
                                                           Kh[None, None], Vh[None, None])
        Kv, Vv, av, pv = caches[l].views()
        Kv[b, h] = Kc[0, 0].to(dev); Vv[b, h] = Vc[0, 0].to(dev)
        av[b, h] = acc[0, 0].to(dev); pv[b, h] = pos[0, 0].to(dev)

    steps_in = [synth.make_steps(B, Hh, d, T, w.dtype, w.sigma, dev, seed, layer=l) for l in range(layers)]
    out = torch.empty((B, Hh, d), dtype=w.dtype, device=dev)
    outs = torch.empty((T, n_sample, d), dtype=w.dtype, device=dev)
    snaps = torch.empty((T, n_sample, k), dtype=torch.int32, device=dev)
    pos_views = [c.views()[3] for c in caches]
    by_layer = {}
    for i, (l, b, h) in enumerate(triples):
        by_layer.setdefault(l, []).append((i, b, h))
    for s in range(T):
        for l in range(layers):
            qs, ks, vs = steps_in[l]
            caches[l].decode_step(qs[s], ks[s], vs[s], out)
            for (i, b, h) in by_layer.get(l, ()):
                outs[s, i] = out[b, h]
                snaps[s, i] = pos_views[l][b, h]
    torch.cuda.synchronize()
    outs, snaps = outs.cpu(), snaps.cpu()
    tol = parity.OUT_TOL[w.dtype]

    def one(i):
        l, b, h = triples[i]
        qs, ks, vs = steps_in[l]
        st = parity.check_head_decode(oracles[triples[i]], qs[:, b, h].cpu(), ks[:, b, h].cpu(),
                                      vs[:, b, h].cpu(), outs[:, i], snaps[:, i], w.recent, tol)
        pos_f, acc_f = caches[l].views()[3][b, h].cpu(), caches[l].views()[2][b, h].cpu()
        parity.check_final_scores(oracles[triples[i]], pos_f, acc_f, st)
        return st

    results, _ = map_heads(one, range(n_sample))
    total = parity.DecodeStats()
    for st in results:
        total.merge(st)
    print("\n[stack parity] %s: %d layers resident, %d sampled (layer, b, h) x %d steps = %d head-steps, "
          "near-tied %d, excused %d, max out l2 %.2e linf %.2e, scores not bit-equal %d"
          % (w.name, layers, n_sample, T, total.head_steps, total.near_tied_steps, total.excused,
             total.max_out_l2, total.max_out_linf, total.score_mismatch), flush=True)
    assert total.excused <= int(0.001 * total.head_steps)
    assert total.max_score_rel <= 1e-6
    for c in caches:
        c.close()
    return total


def test_stack32_config_sampled():
    """batch 128 x 32 heads, d 128, prompt 8192, budget 205 + 205 (5 %), fp16,
    sigma 1.25, 32 layers, 128 steps per layer; 16 sampled (layer, b, h)."""
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS["stack32_f16"]
    st = stack_case(w, w.layers, 16, synth.BASE_SEED, w.steps)
    assert st.head_steps == 16 * w.steps
