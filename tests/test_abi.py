"""The C-ABI library: it loads, exports every function the header declares, and
its host-side argument checks answer without touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hb():
    lib = os.path.join(ROOT, "paper_2306_14048_amd", "libh2o_hip.so")
    if not os.path.exists(lib):
        from paper_2306_14048_amd import build
        build.build(verbose=False)
    from paper_2306_14048_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "h2o.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(h2o_[a-z_0-9]+)\s*\(", text)))


def test_header_and_library_agree(hb):
    names = declared_functions()
    assert len(names) >= 14
    lib = ctypes.CDLL(hb.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n
    assert sorted(hb.EXPORTS) == names, "python binding and header list different entry points"


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_h2o.c"
    src.write_text('#include "h2o.h"\n'
                   'int main(void) { h2o_config c = {0}; c.kv_bits = 4; '
                   'int (*step)(h2o_cache *, const void *, const void *, const void *, void *, void *) = h2o_decode_step; '
                   'return (int)sizeof(c) + H2O_Q4_ROW_BYTES(128) + (step == 0); }\n')
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(root, "include"), str(src)])


def test_size_queries_and_validation(hb):
    ok = hb.make_config(16, 32, 128, 205, 205, hb.H2O_F16)
    # K | V | acc | pos, each padded to 256 bytes
    kv = 16 * 32 * 410 * 128 * 2
    meta = 16 * 32 * 410 * 4
    assert hb.h2o_cache_bytes(ok) == 2 * kv + 2 * meta
    assert hb.h2o_prefill_workspace_bytes(ok, 2048) == 2 * 16 * 32 * 2048 * 4
    bad = [hb.make_config(0, 32, 128, 4, 4, hb.H2O_F16), hb.make_config(1, 1, 96, 4, 4, hb.H2O_F16),
           hb.make_config(1, 1, 128, 0, 0, hb.H2O_F16), hb.make_config(1, 1, 128, -1, 4, hb.H2O_F16),
           hb.make_config(1, 1, 128, 4000, 4000, hb.H2O_F16), hb.make_config(1, 1, 128, 4, 4, 7)]
    bad.append(hb.make_config(1, 1, 128, 4, 4, hb.H2O_F16, rank=2))
    for c in bad:
        assert hb.h2o_cache_bytes(c) == 0
    assert hb.h2o_cache_bytes(hb.make_config(16, 32, 128, 205, 205, hb.H2O_F16, rank=hb.H2O_RANK_AVERAGED)) \
        == 2 * kv + 2 * meta
    assert ctypes.sizeof(hb.h2o_config) == 44
    # the protected set: a pattern needs a period; unknown modes are refused
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 4, 4, hb.H2O_F16, protect=hb.H2O_PROTECT_STRIDED, stride=8)) > 0
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 4, 4, hb.H2O_F16, protect=hb.H2O_PROTECT_FIXED, stride=16)) > 0
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 4, 4, hb.H2O_F16, protect=hb.H2O_PROTECT_STRIDED, stride=0)) == 0
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 4, 4, hb.H2O_F16, protect=3, stride=8)) == 0
    # 4-bit storage: rows of head_dim/2 code bytes + 16 bytes of (scale, min) pairs
    q4 = hb.make_config(16, 32, 128, 205, 205, hb.H2O_F16, kv_bits=4)
    assert hb.h2o_cache_bytes(q4) == 2 * 16 * 32 * 410 * 80 + 2 * meta
    assert hb.h2o_cache_bytes(hb.make_config(2, 2, 64, 8, 8, hb.H2O_BF16, kv_bits=4)) == \
        2 * 2 * 2 * 16 * 48 + 2 * 256
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 8, 8, hb.H2O_F16, kv_bits=8)) == 0
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 1024, 1024, hb.H2O_F16, kv_bits=4)) > 0
    assert hb.h2o_cache_bytes(hb.make_config(1, 1, 128, 1025, 1024, hb.H2O_F16, kv_bits=4)) == 0
    assert hb.h2o_prefill_chunk_workspace_bytes(q4, 512) == 0      # no chunked prompt on a 4-bit cache
    assert hb.q4_row_bytes(128) == 80 and hb.q4_row_bytes(64) == 48
    assert hb.h2o_prefill_workspace_bytes(ok, 0) == 0
    assert hb.h2o_prefill_workspace_bytes(ok, hb.H2O_MAX_PROMPT + 1) == 0
    # transposed V padded to whole 64-key tiles, then the scoring scratch
    assert hb.h2o_prefill_attention_workspace_bytes(ok, 2000) == \
        16 * 32 * 128 * 2048 * 2 + hb.h2o_prefill_workspace_bytes(ok, 2000)
    assert hb.h2o_prefill_attention_workspace_bytes(ok, 0) == 0
    # cache + chunk as one candidate list: K, V rows; old scores, positions, column sums; row statistics
    ncat = 410 + 512
    assert hb.h2o_prefill_chunk_workspace_bytes(ok, 512) == \
        2 * 16 * 32 * ncat * 128 * 2 + 3 * 16 * 32 * ncat * 4 + 16 * 32 * 512 * 4 + 16 * 32 * 410 * 4
    # with the attention output: + V of cache + chunk transposed, padded to whole 64-key tiles
    assert hb.h2o_prefill_chunk_workspace_bytes(ok, 512, True) == \
        hb.h2o_prefill_chunk_workspace_bytes(ok, 512) + 16 * 32 * 128 * 960 * 2
    assert hb.h2o_prefill_chunk_workspace_bytes(hb.make_config(1, 1, 128, 4, 4, hb.H2O_F32), 8, True) == 0
    assert hb.h2o_prefill_chunk_workspace_bytes(ok, 0) == 0
    assert hb.h2o_prefill_chunk_workspace_bytes(ok, hb.H2O_MAX_PROMPT - 409) == 0
    assert hb.h2o_prefill_chunk_workspace_bytes(bad[0], 8) == 0


def test_error_codes_without_device(hb):
    lib = hb._lib
    ok = hb.make_config(1, 1, 128, 4, 4, hb.H2O_F16)
    out = ctypes.c_void_p()
    assert lib.h2o_cache_init(None, 0x1000, 1 << 20, None, ctypes.byref(out)) == hb.H2O_EINVAL
    assert lib.h2o_cache_init(ctypes.byref(ok), None, 1 << 20, None, ctypes.byref(out)) == hb.H2O_EINVAL
    assert lib.h2o_cache_init(ctypes.byref(ok), 0x1008, 1 << 20, None, ctypes.byref(out)) == hb.H2O_EINVAL
    assert lib.h2o_cache_init(ctypes.byref(ok), 0x1000, 16, None, ctypes.byref(out)) == hb.H2O_ENOMEM
    odd = hb.make_config(1, 1, 80, 4, 4, hb.H2O_F16)
    assert lib.h2o_cache_init(ctypes.byref(odd), 0x1000, 1 << 20, None, ctypes.byref(out)) == hb.H2O_EUNSUPPORTED
    assert out.value is None
    assert lib.h2o_decode_step(None, 0x1000, 0x1000, 0x1000, 0x1000, None) == hb.H2O_EINVAL
    assert lib.h2o_cache_reset(None, None) == hb.H2O_EINVAL
    assert lib.h2o_cache_tokens_seen(None) == hb.H2O_EINVAL
    assert lib.h2o_prefill_colsum(ctypes.byref(ok), None, 0x1000, 8, 0x1000, 1 << 20, 0x1000, None) == hb.H2O_EINVAL
    assert lib.h2o_prefill_colsum(ctypes.byref(ok), 0x1000, 0x1000, 8, 0x1000, 8, 0x1000, None) == hb.H2O_ENOMEM
    assert lib.h2o_prefill_colsum(ctypes.byref(ok), 0x1000, 0x1000, hb.H2O_MAX_PROMPT + 1, 0x1000,
                                  1 << 30, 0x1000, None) == hb.H2O_EUNSUPPORTED
    assert lib.h2o_prefill_attention(ctypes.byref(ok), 0x1000, 0x1000, None, 8, 0x1000, 1 << 20, 0x1000,
                                     None, None) == hb.H2O_EINVAL
    assert lib.h2o_prefill_attention(ctypes.byref(ok), 0x1000, 0x1000, 0x1000, 8, 0x1000, 8, 0x1000,
                                     None, None) == hb.H2O_ENOMEM
    f32 = hb.make_config(1, 1, 128, 4, 4, hb.H2O_F32)
    assert lib.h2o_prefill_attention(ctypes.byref(f32), 0x1000, 0x1000, 0x1000, 8, 0x1000, 1 << 20,
                                     0x1000, None, None) == hb.H2O_EUNSUPPORTED
    assert lib.h2o_prefill_attention_scores(None, 0x1000, 0x1000, 0x1000, 8, 0x1000, 1 << 20, 0x1000,
                                            None, None) == hb.H2O_EINVAL
    assert lib.h2o_prefill_chunk(None, 0x1000, 0x1000, 0x1000, 8, 0x1000, 1 << 20, None, None) == hb.H2O_EINVAL
    assert lib.h2o_cache_rolled_positions(None, 0x1000, None) == hb.H2O_EINVAL
    lib.h2o_cache_destroy(None)
    assert hb.h2o_status_str(0) == "ok"
    assert "unsupported" in hb.h2o_status_str(hb.H2O_EUNSUPPORTED)
    assert hb.h2o_status_str(-99) == "unknown status"


def test_synthetic_inputs_are_seeded_and_shaped():
    import torch
    from paper_2306_14048_amd import synth
    w = synth.WORKLOADS
    assert (w["opt6.7b_layer_f16"].heavy, w["opt6.7b_layer_f16"].recent) == (205, 205)
    assert (w["opt30b_layer_f16"].heavy, w["opt30b_layer_f16"].recent) == (103, 102)
    assert (w["stack32_f16"].heavy, w["stack32_f16"].recent) == (205, 205)
    assert (w["prefill_bf16"].heavy, w["prefill_bf16"].recent) == (410, 409)
    a = synth.make_prompt(2, 3, 16, 8, torch.float16, 1.0, "cpu", seed=5)
    b = synth.make_prompt(2, 3, 16, 8, torch.float16, 1.0, "cpu", seed=5)
    c = synth.make_prompt(2, 3, 16, 8, torch.float16, 1.0, "cpu", seed=6)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert not torch.equal(a[1], c[1])
    q, k, v = synth.make_steps(2, 3, 8, 5, torch.bfloat16, 1.0, "cpu", seed=5)
    assert q.shape == (5, 2, 3, 8) and k.dtype == torch.bfloat16
    # heavy-tailed keys: per-token norms spread over more than a decade at sigma = 1
    K = synth.make_prompt(1, 1, 4096, 64, torch.float32, 1.0, "cpu", seed=1)[1]
    norms = K[0, 0].norm(dim=-1)
    assert norms.max() / norms.median() > 8
