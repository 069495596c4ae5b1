"""Shared machinery of the GPU parity tests: drives the CPU oracle on the same
tensors the device sees and compares per step.

Rules applied (stated in the design notes):
  * kept-token sets must be equal after every step.  If they differ, the step
    is excused only when the position the device evicted is an eviction
    candidate whose oracle score is within NEAR_TIE relative of the oracle's
    lowest candidate score; the oracle then adopts the device's choice
    (resync) and the step is counted.  Anything else fails.
  * outputs: ||o_gpu - o_ref||_2 / ||o_ref||_2 and max|diff| / max|o_ref| both
    within `out_tol` (1e-5 fp32, 2e-3 fp16/bf16) plus, for bf16 only, 2^-8: the
    device stores its fp32 result in the output dtype with one rounding, and a
    bf16 value (8 significand bits) is off by up to 2^-8 relative from that
    rounding alone, which no kernel can avoid (fp16: 2^-11, inside the tolerance).
Nothing the oracle consumes or is compared against ever comes from the device
except the device's own results under test.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

from oracle.h2o_oracle import OracleHead, map_heads

NEAR_TIE = 1e-6
OUT_TOL = {torch.float32: 1e-5, torch.float16: 2e-3, torch.bfloat16: 2e-3}
# allowance for storing the fp32 result in the output dtype: only bf16's rounding
# step is coarser than the tolerance itself
OUT_STORE_SLACK = {torch.float32: 0.0, torch.float16: 0.0, torch.bfloat16: 2.0 ** -8}


def oracle_scale(d: int, scale: float = 0.0) -> float:
    """The double the library uses: the config's float if non-zero, else 1/sqrt(d)."""
    return float(np.float32(scale)) if scale else 1.0 / float(np.sqrt(np.float64(d)))


def host64(x: torch.Tensor) -> np.ndarray:
    return x.detach().to("cpu").double().numpy()


@dataclasses.dataclass
class DecodeStats:
    head_steps: int = 0
    near_tied_steps: int = 0      # oracle's two lowest candidates within NEAR_TIE
    excused: int = 0              # device chose the other member of a near tie
    max_out_l2: float = 0.0
    max_out_linf: float = 0.0
    score_mismatch: int = 0       # final scores not bit-identical
    max_score_rel: float = 0.0

    def merge(self, o: "DecodeStats"):
        self.head_steps += o.head_steps
        self.near_tied_steps += o.near_tied_steps
        self.excused += o.excused
        self.max_out_l2 = max(self.max_out_l2, o.max_out_l2)
        self.max_out_linf = max(self.max_out_linf, o.max_out_linf)
        self.score_mismatch += o.score_mismatch
        self.max_score_rel = max(self.max_score_rel, o.max_score_rel)


def oracle_prefill_heads(Q, K, V, heads, heavy, recent, scale, cap, score_f32=True, threads=None,
                         policy=0, kv_bits=0):
    """Runs the oracle's prompt phase for the listed (b, h) pairs.
    Q, K, V: torch tensors [B, Hh, n, d] (any device).  Returns
    ({(b, h): OracleHead}, {(b, h): colsum float64[n]})."""
    d = Q.shape[-1]

    def one(bh):
        b, h = bh
        o = OracleHead(d, heavy, recent, scale, score_f32=score_f32, cap=cap, policy=policy, kv_bits=kv_bits)
        col, _ = o.prefill(host64(Q[b, h]), host64(K[b, h]), host64(V[b, h]))
        return o, col

    res, _ = map_heads(one, heads, threads)
    return ({bh: r[0] for bh, r in zip(heads, res)}, {bh: r[1] for bh, r in zip(heads, res)})


def cache_state_from_oracles(oracles, B, Hh, k, Kp, Vp, base=None):
    """Builds (K, V, acc, pos) cache tensors on the host from oracle heads: the
    resident tokens in ascending position order occupy slots 0..c-1.
    Kp, Vp: the prompt tensors the tokens came from (host).  `base` optionally
    supplies tensors to start from (heads without an oracle keep their state)."""
    d = Kp.shape[-1]
    if base is None:
        Kc = torch.zeros((B, Hh, k, d), dtype=Kp.dtype)
        Vc = torch.zeros((B, Hh, k, d), dtype=Kp.dtype)
        acc = torch.zeros((B, Hh, k), dtype=torch.float32)
        pos = torch.full((B, Hh, k), -1, dtype=torch.int32)
    else:
        Kc, Vc, acc, pos = (x.clone() for x in base)
    for (b, h), o in oracles.items():
        p, s = o.resident()
        c = len(p)
        idx = torch.from_numpy(p.astype(np.int64))
        Kc[b, h, :c] = Kp[b, h, idx]
        Vc[b, h, :c] = Vp[b, h, idx]
        s32 = s.astype(np.float32)
        assert np.array_equal(s32.astype(np.float64), s), "oracle scores must be binary32 values"
        acc[b, h, :c] = torch.from_numpy(s32)
        acc[b, h, c:] = 0
        pos[b, h, :c] = torch.from_numpy(p)
        pos[b, h, c:] = -1
    return Kc, Vc, acc, pos


def run_gpu_decode(cache, qs, ks, vs, snapshot_heads=None):
    """T decode steps through the C ABI, enqueued back to back.  Returns the
    outputs and the slot->position table after every step, both on the host:
    [T, B, Hh, d] and [T, B, Hh, k], or, with `snapshot_heads` = list of (b, h),
    [T, S, d] and [T, S, k] for those heads only."""
    from paper_2306_14048_amd import binding as hb
    T, B, Hh, d = qs.shape
    k = cache.budget
    dev = qs.device
    if snapshot_heads is None:
        outs = torch.empty((T, B, Hh, d), dtype=qs.dtype, device=dev)
        snaps = torch.empty((T, B, Hh, k), dtype=torch.int32, device=dev)
        for s in range(T):
            cache.decode_step(qs[s], ks[s], vs[s], outs[s])
            hb.h2o_cache_snapshot(cache.handle, snaps[s], None)
        torch.cuda.synchronize()
        return outs.cpu(), snaps.cpu()
    bi = torch.tensor([b for b, _ in snapshot_heads], device=dev)
    hi = torch.tensor([h for _, h in snapshot_heads], device=dev)
    pos_view = cache.views()[3]
    out = torch.empty((B, Hh, d), dtype=qs.dtype, device=dev)
    outs = torch.empty((T, len(snapshot_heads), d), dtype=qs.dtype, device=dev)
    snaps = torch.empty((T, len(snapshot_heads), k), dtype=torch.int32, device=dev)
    for s in range(T):
        cache.decode_step(qs[s], ks[s], vs[s], out)
        outs[s] = out[bi, hi]
        snaps[s] = pos_view[bi, hi]
    torch.cuda.synchronize()
    return outs.cpu(), snaps.cpu()


def rank_of(o: OracleHead, pos: int, t: int, policy: int) -> float:
    """The value that ranks `pos` after the query at position t, in the precision
    the scores are stored in (binary32): the score itself or, for the averaged
    ranking, score / (t - pos + 1)."""
    s = np.float32(o.score(pos))
    return float(s) if policy == 0 else float(s / np.float32(t - pos + 1))


def check_head_decode(o: OracleHead, qs, ks, vs, outs, snaps, recent, out_tol, policy=0) -> DecodeStats:
    """Steps one oracle head through T steps and compares with the device's
    per-step outputs [T, d] and slot tables [T, k] of the same head."""
    out_tol = out_tol + OUT_STORE_SLACK[outs.dtype]
    st = DecodeStats()
    T = qs.shape[0]
    q64, k64, v64, o_gpu = host64(qs), host64(ks), host64(vs), host64(outs)
    snaps = snaps.numpy()
    for s in range(T):
        t = o.t
        r = o.decode(q64[s], k64[s], v64[s])
        st.head_steps += 1
        # outputs
        ref = r.out
        diff = o_gpu[s] - ref
        l2 = float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
        linf = float(np.abs(diff).max() / max(np.abs(ref).max(), 1e-300))
        st.max_out_l2 = max(st.max_out_l2, l2)
        st.max_out_linf = max(st.max_out_linf, linf)
        assert l2 <= out_tol and linf <= out_tol, \
            "output mismatch at step %d (t=%d): l2 %.3e linf %.3e > %.1e" % (s, t, l2, linf, out_tol)
        # kept sets
        if np.isfinite(r.second) and (r.second - r.lowest) <= NEAR_TIE * max(abs(r.second), abs(r.lowest)):
            st.near_tied_steps += 1
        row = snaps[s]
        gpu_sorted = np.sort(row[row >= 0])
        assert np.all(np.diff(gpu_sorted) > 0), "duplicate position in device cache"
        ref_sorted = o.resident()[0]
        if len(gpu_sorted) == len(ref_sorted) and np.array_equal(gpu_sorted, ref_sorted):
            continue
        gpu_set, ref_set = set(gpu_sorted.tolist()), set(ref_sorted.tolist())
        if gpu_set != ref_set:
            only_ref = ref_set - gpu_set          # what the device evicted instead
            only_gpu = gpu_set - ref_set          # what the oracle evicted
            ok = (len(only_ref) == 1 and len(only_gpu) == 1 and r.evicted in only_gpu)
            if ok:
                g = next(iter(only_ref))
                sg = rank_of(o, g, t, policy)
                ok = (g <= t - recent and
                      (sg - r.lowest) <= NEAR_TIE * max(abs(sg), abs(r.lowest)))
            assert ok, ("kept-set mismatch at step %d (t=%d): device-only %s oracle-only %s, "
                        "oracle lowest %.9g second %.9g" % (s, t, sorted(only_gpu), sorted(only_ref),
                                                            r.lowest, r.second))
            o.resync(r.evicted, g)
            st.excused += 1
    return st


def check_final_scores(o: OracleHead, pos_row, acc_row, st: DecodeStats):
    """Device scores after the run against the oracle's (same token set)."""
    ref_pos, ref_sc = o.resident()
    lut = dict(zip(ref_pos.tolist(), ref_sc.tolist()))
    pos_row = pos_row.numpy(); acc_row = acc_row.numpy()
    for p, a in zip(pos_row, acc_row):
        if p < 0:
            continue
        ref = lut[int(p)]
        if float(a) != ref:
            st.score_mismatch += 1
            st.max_score_rel = max(st.max_score_rel, abs(float(a) - ref) / max(abs(ref), 1e-300))
