"""h2o_prefill_scores_noalloc (the prompt phase on the library's built-in scratch)
against h2o_prefill_scores (caller-provided workspace), through the C ABI.

Both entry points run the same kernels, so everything is compared bit for bit:
column sums, kept positions, scores and the gathered K/V rows.  Two calls in a
row on the same GPU, the second on a smaller prompt (the scratch keeps the first
call's contents), plus the size limit and the state check.  This file is named
so that it is collected last.
"""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu


def _both(hb, synth, B, Hh, d, n, heavy, recent, dtype, seed):
    dev = torch.device("cuda:0")
    Q, K, V = synth.make_prompt(B, Hh, n, d, dtype, 1.0, dev, seed=seed)
    ref = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    col_ref = torch.empty((B, Hh, n), dtype=torch.float32, device=dev)
    ref.prefill_scores(Q, K, V, colsum_out=col_ref)
    new = hb.H2OCache(B, Hh, d, heavy, recent, dtype, device=dev)
    col_new = torch.full((B, Hh, n), -1.0, dtype=torch.float32, device=dev)
    hb.h2o_prefill_scores_noalloc(new.handle, Q, K, V, n, col_new)
    torch.cuda.synchronize()
    assert new.tokens_seen == ref.tokens_seen == n
    assert torch.equal(col_new, col_ref), "column sums differ"
    Kn, Vn, an, pn = new.views()
    Kr, Vr, ar, pr = ref.views()
    assert torch.equal(pn, pr), "positions differ"
    assert torch.equal(an.view(torch.int32), ar.view(torch.int32)), "scores differ"
    occ = pr >= 0                      # rows of free slots are not defined
    assert int(occ.sum()) == B * Hh * min(n, heavy + recent)
    esz = Kn.element_size()
    for a, b, what in ((Kn, Kr, "K rows"), (Vn, Vr, "V rows")):
        a = a.view(torch.uint8).view(B, Hh, heavy + recent, d * esz)[occ]
        b = b.view(torch.uint8).view(B, Hh, heavy + recent, d * esz)[occ]
        assert torch.equal(a, b), what + " differ"       # bit for bit
    # and without the optional output
    new.reset()
    hb.h2o_prefill_scores_noalloc(new.handle, Q, K, V, n, None)
    torch.cuda.synchronize()
    assert torch.equal(new.views()[3], ref.views()[3]) and torch.equal(new.views()[2], ref.views()[2])
    ref.close()
    new.close()


def test_noalloc_prompt_phase_twice_second_smaller():
    from paper_2306_14048_amd import binding as hb, synth
    _both(hb, synth, 2, 4, 128, 700, 40, 33, torch.float16, 41)     # several tiles + a ragged tail
    _both(hb, synth, 1, 3, 64, 130, 9, 8, torch.bfloat16, 42)       # smaller: stale scratch behind it
    _both(hb, synth, 1, 2, 64, 90, 60, 60, torch.float32, 43)       # budget >= prompt: keep all


def test_noalloc_limit_and_state():
    from paper_2306_14048_amd import binding as hb
    dev = torch.device("cuda:0")
    # 64 heads x 40 000 tokens: 2 x 10.24 MB of row statistics + column sums > 16 MiB
    c = hb.H2OCache(2, 32, 64, 8, 8, torch.float16, device=dev)
    n = 40000
    assert hb.h2o_prefill_workspace_bytes(c.cfg, n) > hb.H2O_NOALLOC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.float16, device=dev)       # never read: the size is refused first
    rc = hb._lib.h2o_prefill_scores_noalloc(c.handle, dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(),
                                            n, None, None)
    assert rc == hb.H2O_ESCRATCH
    assert "scratch" in hb.h2o_status_str(rc)
    assert c.tokens_seen == 0
    # a cache that already holds a prompt is refused like h2o_prefill_scores refuses it
    from paper_2306_14048_amd import synth
    Q, K, V = synth.make_prompt(2, 32, 64, 64, torch.float16, 1.0, dev, seed=5)
    hb.h2o_prefill_scores_noalloc(c.handle, Q, K, V, 64, None)
    rc = hb._lib.h2o_prefill_scores_noalloc(c.handle, Q.data_ptr(), K.data_ptr(), V.data_ptr(), 64, None, None)
    assert rc == hb.H2O_ESTATE
    torch.cuda.synchronize()
    c.close()
