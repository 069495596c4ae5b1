"""ctypes front end of the CPU oracle (``h2o_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg; the GPU library and its Python binding never
import it.  It does argument marshalling only; every number comes from the C
file, which states the method as the paper defines it (Definition 2.2,
Algorithm 2, App. A).

All inputs are widened to float64 *exactly* (fp16/bf16/fp32 values are exactly
representable), so the oracle sees the same numbers as the device.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "h2o_oracle.c")
_LIB = os.path.join(_HERE, "libh2o_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fno-fast-math",
             "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    P = ctypes.c_void_p
    D = ctypes.POINTER(ctypes.c_double)
    I = ctypes.POINTER(ctypes.c_int)
    lib.h2o_oracle_new.restype = P
    lib.h2o_oracle_new.argtypes = [ctypes.c_int] * 3 + [ctypes.c_double, ctypes.c_int, ctypes.c_int]
    lib.h2o_oracle_free.argtypes = [P]
    lib.h2o_oracle_free.restype = None
    lib.h2o_oracle_prefill.argtypes = [P, D, D, D, ctypes.c_int, D, D]
    lib.h2o_oracle_load_and_select.argtypes = [P, D, D, D, ctypes.c_int]
    lib.h2o_oracle_prefill_chunk.argtypes = [P, D, D, D, ctypes.c_int, D, D]
    lib.h2o_oracle_decode.argtypes = [P, D, D, D, D, I, D, D]
    lib.h2o_oracle_resync.argtypes = [P, ctypes.c_int, ctypes.c_int]
    lib.h2o_oracle_set_policy.argtypes = [P, ctypes.c_int]
    lib.h2o_oracle_set_protect.argtypes = [P, ctypes.c_int, ctypes.c_int]
    lib.h2o_oracle_tokens_seen.argtypes = [P]
    lib.h2o_oracle_num_resident.argtypes = [P]
    lib.h2o_oracle_evicted_mass.argtypes = [P]
    lib.h2o_oracle_evicted_mass.restype = ctypes.c_double
    lib.h2o_oracle_queries.argtypes = [P]
    lib.h2o_oracle_queries.restype = ctypes.c_double
    lib.h2o_oracle_is_resident.argtypes = [P, ctypes.c_int]
    lib.h2o_oracle_score.argtypes = [P, ctypes.c_int]
    lib.h2o_oracle_score.restype = ctypes.c_double
    lib.h2o_oracle_resident.argtypes = [P, I, D]
    lib.h2o_oracle_token_kv.argtypes = [P, ctypes.c_int, D, D]
    U8 = ctypes.POINTER(ctypes.c_ubyte)
    F = ctypes.POINTER(ctypes.c_float)
    lib.h2o_oracle_set_kv_bits.argtypes = [P, ctypes.c_int, ctypes.c_int]
    lib.h2o_oracle_token_codes.argtypes = [P, ctypes.c_int, U8, F, U8, F]
    _lib = lib
    return lib


def _f64(a) -> np.ndarray:
    """Exact widening of a torch tensor / array to a contiguous float64 array."""
    if hasattr(a, "detach"):                      # torch tensor (any float dtype, any device)
        a = a.detach().to("cpu").double().numpy()
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


class DecodeResult:
    __slots__ = ("out", "evicted", "n_candidates", "lowest", "second", "p_self")

    def __init__(self, out, evicted, n_candidates, lowest, second, p_self):
        self.out = out
        self.evicted = evicted
        self.n_candidates = n_candidates
        self.lowest = lowest
        self.second = second
        self.p_self = p_self


class OracleHead:
    """One (batch, head) pair of the H2O process, position-indexed."""

    def __init__(self, d: int, heavy: int, recent: int, scale: float | None = None,
                 score_f32: bool = False, cap: int = 4096, policy: int = 0, kv_bits: int = 0,
                 group: int = 64, protect: int = 0, stride: int = 0):
        self._lib = _load()
        self.d, self.heavy, self.recent = int(d), int(heavy), int(recent)
        self.budget = self.heavy + self.recent
        self.scale = float(scale) if scale is not None else 1.0 / float(np.sqrt(np.float64(d)))
        self.cap = int(cap)
        self._h = self._lib.h2o_oracle_new(self.d, self.heavy, self.recent, self.scale,
                                           1 if score_f32 else 0, self.cap)
        if not self._h:
            raise ValueError("bad oracle configuration")
        if self._lib.h2o_oracle_set_policy(self._h, int(policy)) != 0:
            raise ValueError("unknown eviction policy %r" % (policy,))
        self.protect, self.stride = int(protect), int(stride)
        if self._lib.h2o_oracle_set_protect(self._h, self.protect, self.stride) != 0:
            raise ValueError("bad protection pattern: mode %r, stride %r" % (protect, stride))
        self.kv_bits, self.group = int(kv_bits), int(group)
        if self._lib.h2o_oracle_set_kv_bits(self._h, self.kv_bits, self.group) != 0:
            raise ValueError("unsupported cache storage: %r bits in groups of %r" % (kv_bits, group))

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            self._lib.h2o_oracle_free(h)
            self._h = None

    # -- prompt phase ------------------------------------------------------
    def prefill(self, Q, K, V, want_attn: bool = False):
        """Full causal attention over the prompt, column sums, compression.

        Returns (colsum[n] fp64 before compression, attn[n, d] or None)."""
        Q, K, V = _f64(Q), _f64(K), _f64(V)
        n = Q.shape[0]
        assert Q.shape == K.shape == V.shape == (n, self.d)
        col = np.empty(n, dtype=np.float64)
        attn = np.empty((n, self.d), dtype=np.float64) if want_attn else None
        rc = self._lib.h2o_oracle_prefill(self._h, _dp(Q), _dp(K), _dp(V), n, _dp(col),
                                          _dp(attn) if want_attn else None)
        if rc != 0:
            raise RuntimeError("oracle prefill failed (state or capacity)")
        return col, attn

    def prefill_chunk(self, Q, K, V, want_attn: bool = False):
        """The next m prompt tokens as one chunk (attend to cache + causally to the
        chunk, accumulate, compress).  Returns (the chunk's column sums by position,
        float64[t + m], attention outputs [m, d] or None)."""
        Q, K, V = _f64(Q), _f64(K), _f64(V)
        m = Q.shape[0]
        assert Q.shape == K.shape == V.shape == (m, self.d)
        col = np.empty(self.t + m, dtype=np.float64)
        attn = np.empty((m, self.d), dtype=np.float64) if want_attn else None
        rc = self._lib.h2o_oracle_prefill_chunk(self._h, _dp(Q), _dp(K), _dp(V), m, _dp(col),
                                                _dp(attn) if want_attn else None)
        if rc != 0:
            raise RuntimeError("oracle prefill_chunk failed (capacity)")
        return col, attn

    def load_and_select(self, K, V, score):
        K, V, score = _f64(K), _f64(V), _f64(score)
        n = K.shape[0]
        assert K.shape == V.shape == (n, self.d) and score.shape == (n,)
        rc = self._lib.h2o_oracle_load_and_select(self._h, _dp(K), _dp(V), _dp(score), n)
        if rc != 0:
            raise RuntimeError("oracle load_and_select failed")

    # -- generation phase --------------------------------------------------
    def decode(self, q, k_new, v_new) -> DecodeResult:
        q, k_new, v_new = _f64(q), _f64(k_new), _f64(v_new)
        assert q.shape == k_new.shape == v_new.shape == (self.d,)
        out = np.empty(self.d, dtype=np.float64)
        info = (ctypes.c_int * 2)()
        low = (ctypes.c_double * 2)()
        ps = ctypes.c_double()
        rc = self._lib.h2o_oracle_decode(self._h, _dp(q), _dp(k_new), _dp(v_new), _dp(out),
                                         info, low, ctypes.byref(ps))
        if rc != 0:
            raise RuntimeError("oracle decode failed (capacity exhausted?)")
        return DecodeResult(out, int(info[0]), int(info[1]), float(low[0]), float(low[1]),
                            float(ps.value))

    def resync(self, restore_pos: int, evict_pos: int) -> None:
        if self._lib.h2o_oracle_resync(self._h, int(restore_pos), int(evict_pos)) != 0:
            raise RuntimeError("oracle resync refused")

    # -- state -------------------------------------------------------------
    @property
    def t(self) -> int:
        return self._lib.h2o_oracle_tokens_seen(self._h)

    @property
    def evicted_mass(self) -> float:
        return self._lib.h2o_oracle_evicted_mass(self._h)

    @property
    def queries(self) -> float:
        return self._lib.h2o_oracle_queries(self._h)

    def score(self, pos: int) -> float:
        return self._lib.h2o_oracle_score(self._h, int(pos))

    def is_resident(self, pos: int) -> bool:
        return bool(self._lib.h2o_oracle_is_resident(self._h, int(pos)))

    def resident(self):
        """(positions ascending int32[c], scores float64[c])."""
        c = self._lib.h2o_oracle_num_resident(self._h)
        pos = np.empty(max(c, 1), dtype=np.int32)
        sc = np.empty(max(c, 1), dtype=np.float64)
        got = self._lib.h2o_oracle_resident(
            self._h, pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), _dp(sc))
        assert got == c
        return pos[:c], sc[:c]

    def token_codes(self, pos: int):
        """What a 4-bit cache holds for resident position `pos`: key codes uint8[d],
        key (scale, min) float32[d/group, 2], value codes, value (scale, min)."""
        ng = self.d // self.group
        kc, vc = np.empty(self.d, np.uint8), np.empty(self.d, np.uint8)
        kp, vp = np.empty((ng, 2), np.float32), np.empty((ng, 2), np.float32)
        u8, f = ctypes.POINTER(ctypes.c_ubyte), ctypes.POINTER(ctypes.c_float)
        rc = self._lib.h2o_oracle_token_codes(self._h, int(pos), kc.ctypes.data_as(u8), kp.ctypes.data_as(f),
                                              vc.ctypes.data_as(u8), vp.ctypes.data_as(f))
        if rc != 0:
            raise RuntimeError("no stored codes for position %d" % pos)
        return kc, kp, vc, vp

    def token_kv(self, pos: int):
        k = np.empty(self.d, dtype=np.float64)
        v = np.empty(self.d, dtype=np.float64)
        if self._lib.h2o_oracle_token_kv(self._h, int(pos), _dp(k), _dp(v)) != 0:
            raise IndexError(pos)
        return k, v


def map_heads(fn, items, threads: int | None = None):
    """Run ``fn(item)`` for every item on a thread pool (the C calls release
    the GIL).  Returns (results in order, number of threads used)."""
    items = list(items)
    if threads is None:
        threads = min(len(items), os.cpu_count() or 1, 16)
    threads = max(1, threads)
    if threads == 1:
        return [fn(x) for x in items], 1
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(fn, items)), threads
