"""Shared machinery of the GPU parity tests: drives the CPU oracle on the same
tensors the device sees and compares per step.

Rules applied (stated in the design notes):
  * kept-token sets must be equal after every step.  If they differ, the step
    is excused only when the position the device evicted is an eviction
    candidate whose oracle score is within NEAR_TIE relative of the oracle's
    lowest candidate score; the oracle then adopts the device's choice
    (resync) and the step is counted.  Anything else fails.
  * outputs, per head vector: ||o_gpu - o_ref||_2 <= tol * ||o_ref||_2 and, element
    by element, |o_gpu - o_ref| <= tol * max|o_ref| (tol = 1e-5 fp32, 2e-3
    fp16/bf16).  For bf16 outputs only, each element is additionally allowed the
    half unit in the last place of the bf16 number it is stored as (and the L2
    bound the norm of those half-ulps): the device rounds its fp32 result once
    into the output dtype, and a bf16 value has 8 significand bits, so that one
    rounding alone is up to 2^-9 relative per element, which no kernel can avoid
    (fp16's 2^-12 is inside the tolerance).
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


# unit roundoff of the element types (half an ulp, relative)
UNIT_ROUNDOFF = {torch.float32: 2.0 ** -24, torch.float16: 2.0 ** -11, torch.bfloat16: 2.0 ** -8}


def output_error(got: np.ndarray, ref: np.ndarray, dtype, p_rounded: bool = False) -> tuple:
    """Error of device output vectors `got` [..., d] (float64 images of values stored
    in `dtype`) against the oracle's `ref`, as fractions of what is allowed: (L2,
    element-wise maximum), each <= 1 when the output passes.  Also returns the plain
    relative errors (L2, max) for reporting.  `p_rounded`: the kernel under test feeds
    the probabilities to a matrix product in the element type (the prompt attention
    kernel does; the generation step does not), which moves every probability by up
    to one unit roundoff of that type: the tolerance is widened by half of that (the
    roundings are independent over the keys of a row, so they largely average out;
    bf16 rows measure up to 3.2e-3 in L2 and 5.0e-3 per element against bounds of
    3.95e-3 of the norm / of the largest element plus the half-ulps of storing)."""
    tol = OUT_TOL[dtype] + (0.5 * UNIT_ROUNDOFF[dtype] if p_rounded else 0.0)
    diff = np.abs(got - ref)
    mx = np.abs(ref).max(-1, keepdims=True)
    allow = tol * mx + np.zeros_like(ref)
    if dtype == torch.bfloat16:
        # half an ulp of the bf16 number the element is stored as: 2^(e - 8) for a value
        # in [2^e, 2^(e+1)); the value rounded may sit up to tol * max above the oracle's
        mag = np.maximum(np.abs(ref) + tol * mx, 2.0 ** -126)
        half_ulp = np.exp2(np.floor(np.log2(mag)) - 8.0)
        allow = allow + half_ulp
        l2_allow = tol * np.linalg.norm(ref, axis=-1) + np.linalg.norm(half_ulp, axis=-1)
    else:
        l2_allow = tol * np.linalg.norm(ref, axis=-1)
    l2 = np.linalg.norm(got - ref, axis=-1)
    frac_l2 = l2 / np.maximum(l2_allow, 1e-300)
    frac_el = (diff / np.maximum(allow, 1e-300)).max(-1)
    rel_l2 = l2 / np.maximum(np.linalg.norm(ref, axis=-1), 1e-300)
    rel_max = diff.max(-1) / np.maximum(mx[..., 0], 1e-300)
    return frac_l2, frac_el, rel_l2, rel_max


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
    excused_band: int = 0         # ... of a pair further apart than NEAR_TIE but inside the caller's band
    max_out_l2: float = 0.0
    max_out_linf: float = 0.0
    max_out_frac: float = 0.0     # worst output error as a fraction of its allowance
    score_mismatch: int = 0       # final scores not bit-identical
    max_score_rel: float = 0.0
    exact_tied_steps: int = 0     # oracle's two lowest candidates exactly equal
    zero_low_steps: int = 0       # oracle evicted a candidate whose rank value is 0
    subnormal_low_steps: int = 0  # ... or a binary32 subnormal

    def merge(self, o: "DecodeStats"):
        self.head_steps += o.head_steps
        self.near_tied_steps += o.near_tied_steps
        self.excused += o.excused
        self.excused_band += o.excused_band
        self.max_out_l2 = max(self.max_out_l2, o.max_out_l2)
        self.max_out_linf = max(self.max_out_linf, o.max_out_linf)
        self.max_out_frac = max(self.max_out_frac, o.max_out_frac)
        self.score_mismatch += o.score_mismatch
        self.max_score_rel = max(self.max_score_rel, o.max_score_rel)
        self.exact_tied_steps += o.exact_tied_steps
        self.zero_low_steps += o.zero_low_steps
        self.subnormal_low_steps += o.subnormal_low_steps


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


def check_head_decode(o: OracleHead, qs, ks, vs, outs, snaps, recent, out_tol, policy=0,
                      band=NEAR_TIE) -> DecodeStats:
    """Steps one oracle head through T steps and compares with the device's
    per-step outputs [T, d] and slot tables [T, k] of the same head.  `band`:
    how far (relative) the oracle's value of the token the device evicted may lie
    above the oracle's lowest for the step to be excused; NEAR_TIE when both sides
    hold the same stored scores, wider only where the device's scores themselves
    carry a stated tolerance (a prompt phase scored on the device).  Steps excused
    inside NEAR_TIE and those between NEAR_TIE and `band` are counted apart."""
    assert out_tol == OUT_TOL[outs.dtype]
    st = DecodeStats()
    T = qs.shape[0]
    q64, k64, v64, o_gpu = host64(qs), host64(ks), host64(vs), host64(outs)
    snaps = snaps.numpy()
    for s in range(T):
        t = o.t
        r = o.decode(q64[s], k64[s], v64[s])
        st.head_steps += 1
        # outputs
        f_l2, f_el, l2, linf = (float(x) for x in output_error(o_gpu[s], r.out, outs.dtype))
        st.max_out_l2 = max(st.max_out_l2, l2)
        st.max_out_linf = max(st.max_out_linf, linf)
        st.max_out_frac = max(st.max_out_frac, f_l2, f_el)
        assert f_l2 <= 1.0 and f_el <= 1.0, \
            ("output mismatch at step %d (t=%d): l2 %.3e linf %.3e rel, %.2f / %.2f of the allowance (tol %.1e)"
             % (s, t, l2, linf, f_l2, f_el, out_tol))
        # kept sets
        if np.isfinite(r.second) and (r.second - r.lowest) <= NEAR_TIE * max(abs(r.second), abs(r.lowest)):
            st.near_tied_steps += 1
        if r.evicted >= 0:
            st.exact_tied_steps += int(r.second == r.lowest)
            st.zero_low_steps += int(r.lowest == 0.0)
            st.subnormal_low_steps += int(0.0 < r.lowest < 2.0 ** -126)
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
                gap = (sg - r.lowest) / max(abs(sg), abs(r.lowest), 1e-300)
                ok = g <= t - recent and gap <= band
            assert ok, ("kept-set mismatch at step %d (t=%d): device-only %s oracle-only %s, "
                        "oracle lowest %.9g second %.9g" % (s, t, sorted(only_gpu), sorted(only_ref),
                                                            r.lowest, r.second))
            o.resync(r.evicted, g)
            if gap <= NEAR_TIE:
                st.excused += 1
            else:
                st.excused_band += 1
    return st


def adopt_kept_set(o: OracleHead, device_positions, t_last: int, recent: int, policy: int, band: float):
    """After a prompt phase scored on the device: if the device kept other tokens than
    the oracle, every token that changed sides must have an oracle rank value within
    `band` (relative) of the oracle's selection threshold; the oracle then adopts the
    device's set.  Returns the number of tokens swapped (0 = sets equal)."""
    ref = set(o.resident()[0].tolist())
    got = set(int(p) for p in device_positions if p >= 0)
    if got == ref:
        return 0
    only_ref, only_gpu = sorted(ref - got), sorted(got - ref)
    assert len(only_ref) == len(only_gpu), "kept sets differ in size"
    thr = min(rank_of(o, j, t_last, policy) for j in ref if j <= t_last - recent)
    for j in only_ref + only_gpu:
        assert j <= t_last - recent, "token %d of the recent window changed sides" % j
        v = rank_of(o, j, t_last, policy)
        assert abs(v - thr) <= band * max(abs(thr), 1e-30), \
            "token %d (rank value %.9g) changed sides away from the threshold %.9g" % (j, v, thr)
    for a, b in zip(only_gpu, only_ref):
        o.resync(a, b)              # a becomes resident, b leaves
    return len(only_ref)


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
