"""Properties of the compiled kernels that no numerical test can see, checked on the
assembly hipcc emits for gfx950 (no GPU needed).

* The prompt-scoring passes run two wave groups one phase apart: a step is
  `matrix phase, barrier, vector phase, barrier`.  Pass 1's vector phase touches no
  memory, so only a data dependence on the closing barrier keeps the compiler from
  scheduling its arithmetic behind that barrier (a build did exactly that: the
  results stay right, the two groups then take turns and the pass is ~10 % slower).
  Every steady-state loop must therefore have its exponentials between its barriers.
* The kernels the benchmark times must not spill registers to scratch memory.
"""
import os
import re
import subprocess
from collections import Counter

import pytest

from paper_2306_14048_amd import build as hb


def device_asm(src: str, tmp_path) -> str:
    out = os.path.join(str(tmp_path), src.replace(".hip", ".s"))
    cmd = ["hipcc", *hb.FLAGS, "--cuda-device-only", "-S", os.path.join(hb.CSRC, src), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return open(out).read()


def functions(asm: str):
    """name -> list of basic blocks, each a list of instruction lines"""
    lines = asm.split("\n")
    fns = {}
    for i, l in enumerate(lines):
        m = re.match(r"^(_Z\S+):", l)
        if not m:
            continue
        blocks, cur = [], []
        for x in lines[i + 1:]:
            if x.startswith(".Lfunc_end"):
                break
            if re.match(r"^\.LBB\d+_\d+:", x):
                if cur:
                    blocks.append(cur)
                cur = []
                continue
            t = x.strip()
            if t and not t.startswith(";") and not t.startswith("."):
                cur.append(t)
        if cur:
            blocks.append(cur)
        fns[m.group(1)] = blocks
    return fns


def metadata(asm: str):
    """name -> {vgpr_count, vgpr_spill_count, ...} from the code object metadata"""
    meta, name = {}, None
    for l in asm.split("\n"):
        m = re.match(r"^\s+\.name:\s+(\S+)", l)
        if m:
            name = m.group(1)
            meta[name] = {}
        m = re.match(r"^\s+\.(vgpr_count|vgpr_spill_count|sgpr_spill_count|private_segment_fixed_size):\s+(\d+)", l)
        if m and name:
            meta[name][m.group(1)] = int(m.group(2))
    return meta


@pytest.fixture(scope="module")
def scores_asm(tmp_path_factory):
    return device_asm("prefill_scores.hip", tmp_path_factory.mktemp("isa"))


def test_vector_phase_of_the_scoring_passes_sits_between_the_barriers(scores_asm):
    fns = {n: b for n, b in functions(scores_asm).items() if "prefill_pass_kernel" in n}
    assert len(fns) == 12                                   # 3 element types x 2 head dims x 2 passes
    for name, blocks in fns.items():
        loops = 0
        for ins in blocks:
            ops = [x.split()[0] for x in ins]
            if ops.count("s_barrier") != 2 or not any("mfma" in o for o in ops):
                continue
            loops += 1
            first = ops.index("s_barrier")
            second = len(ops) - 1 - ops[::-1].index("s_barrier")
            last_mfma = max(i for i, o in enumerate(ops) if "mfma" in o)
            exps = [i for i, o in enumerate(ops) if o.startswith("v_exp_f32")]
            assert last_mfma < first, name
            between = [i for i in exps if first < i < second]
            assert len(between) >= 16 and not [i for i in exps if i > second], \
                "%s: %d exponentials between the barriers, %d behind the second" % (
                    name, len(between), len([i for i in exps if i > second]))
        assert loops >= 1, name                             # the unmasked steady-state loop was found


def test_benchmarked_kernels_do_not_spill(scores_asm, tmp_path):
    meta = metadata(scores_asm)
    checked = 0
    for name, m in meta.items():
        # 16-bit element types (1 = f16, 2 = bf16): the shapes of every workload in the benchmark
        if "prefill_pass_kernel" in name and ("ILi1E" in name or "ILi2E" in name):
            assert m["vgpr_spill_count"] == 0 and m["vgpr_count"] <= 128, (name, m)
            checked += 1
    assert checked == 8
    meta = metadata(device_asm("decode_step.hip", tmp_path))
    checked = 0
    for name, m in meta.items():
        if "decode_resident_kernel" in name:
            # two workgroups of eight waves per CU need <= 128 registers per lane
            assert m["vgpr_spill_count"] == 0 and m["vgpr_count"] <= 128, (name, m)
            checked += 1
    assert checked >= 8
