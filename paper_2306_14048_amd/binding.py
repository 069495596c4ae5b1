"""ctypes binding of libh2o_hip.so: same entry points as include/h2o.h.

Argument marshalling only (tensor -> device pointer, stream -> hipStream_t);
every step of the path runs in the HIP kernels.  PyTorch is used for device
memory and streams.  There is no fallback: if the library has not been built
(`python -m paper_2306_14048_amd.build`) importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libh2o_hip.so")

H2O_OK, H2O_EINVAL, H2O_EUNSUPPORTED, H2O_ENOMEM, H2O_ESTATE, H2O_EHIP = 0, -1, -2, -3, -4, -5
H2O_ESCRATCH = -6
H2O_NOALLOC_SCRATCH_BYTES = 16 << 20
H2O_F32, H2O_F16, H2O_BF16 = 0, 1, 2
H2O_RANK_ACCUMULATED, H2O_RANK_AVERAGED = 0, 1
H2O_PROTECT_RECENT, H2O_PROTECT_STRIDED, H2O_PROTECT_FIXED = 0, 1, 2
H2O_BAD_HOLE, H2O_BAD_BEYOND, H2O_BAD_RANGE, H2O_BAD_DUPLICATE, H2O_BAD_SCORE = 1, 2, 4, 8, 16
H2O_MAX_BUDGET = 4096
H2O_MAX_PROMPT = 65536

DTYPES = {torch.float32: H2O_F32, torch.float16: H2O_F16, torch.bfloat16: H2O_BF16}
TORCH_DTYPES = {v: k for k, v in DTYPES.items()}

EXPORTS = (
    "h2o_cache_bytes", "h2o_prefill_workspace_bytes", "h2o_cache_init", "h2o_cache_reset",
    "h2o_cache_destroy", "h2o_prefill_colsum", "h2o_prefill_select", "h2o_prefill_scores",
    "h2o_decode_step", "h2o_cache_snapshot", "h2o_cache_restore", "h2o_cache_tokens_seen",
    "h2o_cache_regions", "h2o_status_str", "h2o_prefill_attention_workspace_bytes",
    "h2o_prefill_attention", "h2o_prefill_attention_scores", "h2o_prefill_chunk_workspace_bytes",
    "h2o_prefill_chunk", "h2o_cache_rolled_positions", "h2o_prefill_scores_noalloc",
    "h2o_cache_validate",
)


class h2o_config(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("heavy", ctypes.c_int32), ("recent", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("scale", ctypes.c_float), ("rank", ctypes.c_int32), ("kv_bits", ctypes.c_int32),
                ("protect", ctypes.c_int32), ("stride", ctypes.c_int32)]


class H2OError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, h2o_status_str(status), status))


if not os.path.exists(LIB_PATH):
    raise ImportError("libh2o_hip.so is not built; run `python -m paper_2306_14048_amd.build` "
                      "(there is no CPU fallback)")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
_cfgp = ctypes.POINTER(h2o_config)
_lib.h2o_cache_bytes.restype = _sz
_lib.h2o_cache_bytes.argtypes = [_cfgp]
_lib.h2o_prefill_workspace_bytes.restype = _sz
_lib.h2o_prefill_workspace_bytes.argtypes = [_cfgp, _i32]
_lib.h2o_cache_init.argtypes = [_cfgp, _vp, _sz, _vp, ctypes.POINTER(_vp)]
_lib.h2o_cache_reset.argtypes = [_vp, _vp]
_lib.h2o_cache_destroy.argtypes = [_vp]
_lib.h2o_cache_destroy.restype = None
_lib.h2o_prefill_colsum.argtypes = [_cfgp, _vp, _vp, _i32, _vp, _sz, _vp, _vp]
_lib.h2o_prefill_select.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp]
_lib.h2o_prefill_scores.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp, _vp]
_lib.h2o_prefill_scores_noalloc.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _vp]
_lib.h2o_prefill_attention_workspace_bytes.restype = _sz
_lib.h2o_prefill_attention_workspace_bytes.argtypes = [_cfgp, _i32]
_lib.h2o_prefill_attention.argtypes = [_cfgp, _vp, _vp, _vp, _i32, _vp, _sz, _vp, _vp, _vp]
_lib.h2o_prefill_attention_scores.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp, _vp, _vp]
_lib.h2o_prefill_chunk_workspace_bytes.restype = _sz
_lib.h2o_prefill_chunk_workspace_bytes.argtypes = [_cfgp, _i32, _i32]
_lib.h2o_prefill_chunk.argtypes = [_vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp, _vp]
_lib.h2o_cache_rolled_positions.argtypes = [_vp, _vp, _vp]
_lib.h2o_cache_validate.argtypes = [_vp, _vp, _vp]
_lib.h2o_decode_step.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp]
_lib.h2o_cache_snapshot.argtypes = [_vp, _vp, _vp, _vp]
_lib.h2o_cache_restore.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _vp]
_lib.h2o_cache_tokens_seen.argtypes = [_vp]
_lib.h2o_cache_regions.argtypes = [_vp] + [ctypes.POINTER(_vp)] * 4
_lib.h2o_status_str.restype = ctypes.c_char_p
_lib.h2o_status_str.argtypes = [ctypes.c_int]


def _ptr(x):
    """Device (or null) pointer of a tensor / raw int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_contiguous():
        raise ValueError("the C ABI takes dense row-major arrays; got a non-contiguous tensor")
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != H2O_OK:
        raise H2OError(rc, where)


H2O_Q4_GROUP = 64
H2O_Q4_MAX_BUDGET = 2048


def q4_row_bytes(head_dim: int) -> int:
    """Bytes of one cached K (or V) row in 4-bit storage: codes, then (scale, min) pairs."""
    return head_dim // 2 + 16


def unpack_q4_rows(rows: torch.Tensor, head_dim: int):
    """Splits stored rows [..., row bytes] (uint8) into codes [..., head_dim] (uint8,
    one per element) and parameters [..., head_dim / 64, 2] (float32: scale, min)."""
    cb = head_dim // 2
    packed = rows[..., :cb]
    codes = torch.stack((packed & 15, packed >> 4), dim=-1).reshape(*rows.shape[:-1], head_dim)
    ng = head_dim // H2O_Q4_GROUP
    par = rows[..., cb:cb + 8 * ng].contiguous().view(torch.float32).reshape(*rows.shape[:-1], ng, 2)
    return codes, par


def make_config(batch, heads, head_dim, heavy, recent, dtype, scale=0.0, rank=0, kv_bits=0,
                protect=0, stride=0) -> h2o_config:
    if isinstance(dtype, torch.dtype):
        dtype = DTYPES[dtype]
    return h2o_config(int(batch), int(heads), int(head_dim), int(heavy), int(recent), int(dtype),
                      float(scale), int(rank), int(kv_bits), int(protect), int(stride))


def h2o_status_str(status: int) -> str:
    return _lib.h2o_status_str(int(status)).decode()


def h2o_cache_bytes(cfg: h2o_config) -> int:
    return int(_lib.h2o_cache_bytes(ctypes.byref(cfg)))


def h2o_prefill_workspace_bytes(cfg: h2o_config, n: int) -> int:
    return int(_lib.h2o_prefill_workspace_bytes(ctypes.byref(cfg), int(n)))


def h2o_cache_init(cfg: h2o_config, dev_mem, nbytes: int, stream=None) -> int:
    """Returns the opaque handle (an integer address)."""
    out = _vp()
    _check(_lib.h2o_cache_init(ctypes.byref(cfg), _ptr(dev_mem), int(nbytes), _stream(stream),
                               ctypes.byref(out)), "h2o_cache_init")
    return out.value


def h2o_cache_reset(cache: int, stream=None) -> None:
    _check(_lib.h2o_cache_reset(cache, _stream(stream)), "h2o_cache_reset")


def h2o_cache_destroy(cache: int) -> None:
    _lib.h2o_cache_destroy(cache)


def h2o_prefill_colsum(cfg, Q, K, n, workspace, ws_bytes, colsum_out, stream=None) -> None:
    _check(_lib.h2o_prefill_colsum(ctypes.byref(cfg), _ptr(Q), _ptr(K), int(n), _ptr(workspace),
                                   int(ws_bytes), _ptr(colsum_out), _stream(stream)),
           "h2o_prefill_colsum")


def h2o_prefill_select(cache, K, V, score, n, stream=None) -> None:
    _check(_lib.h2o_prefill_select(cache, _ptr(K), _ptr(V), _ptr(score), int(n), _stream(stream)),
           "h2o_prefill_select")


def h2o_prefill_scores(cache, Q, K, V, n, workspace, ws_bytes, colsum_out=None, stream=None) -> None:
    _check(_lib.h2o_prefill_scores(cache, _ptr(Q), _ptr(K), _ptr(V), int(n), _ptr(workspace),
                                   int(ws_bytes), _ptr(colsum_out), _stream(stream)),
           "h2o_prefill_scores")


def h2o_prefill_scores_noalloc(cache, Q, K, V, n, colsum_out=None, stream=None) -> None:
    _check(_lib.h2o_prefill_scores_noalloc(cache, _ptr(Q), _ptr(K), _ptr(V), int(n),
                                           _ptr(colsum_out), _stream(stream)),
           "h2o_prefill_scores_noalloc")


def h2o_prefill_attention_workspace_bytes(cfg: h2o_config, n: int) -> int:
    return int(_lib.h2o_prefill_attention_workspace_bytes(ctypes.byref(cfg), int(n)))


def h2o_prefill_attention(cfg, Q, K, V, n, workspace, ws_bytes, out, lse_out=None, stream=None) -> None:
    _check(_lib.h2o_prefill_attention(ctypes.byref(cfg), _ptr(Q), _ptr(K), _ptr(V), int(n),
                                      _ptr(workspace), int(ws_bytes), _ptr(out), _ptr(lse_out),
                                      _stream(stream)), "h2o_prefill_attention")


def h2o_prefill_attention_scores(cache, Q, K, V, n, workspace, ws_bytes, out, colsum_out=None,
                                 stream=None) -> None:
    _check(_lib.h2o_prefill_attention_scores(cache, _ptr(Q), _ptr(K), _ptr(V), int(n),
                                             _ptr(workspace), int(ws_bytes), _ptr(out),
                                             _ptr(colsum_out), _stream(stream)),
           "h2o_prefill_attention_scores")


def h2o_prefill_chunk_workspace_bytes(cfg: h2o_config, m: int, with_output: bool = False) -> int:
    return int(_lib.h2o_prefill_chunk_workspace_bytes(ctypes.byref(cfg), int(m), 1 if with_output else 0))


def h2o_prefill_chunk(cache, Q, K, V, m, workspace, ws_bytes, out=None, stream=None) -> None:
    _check(_lib.h2o_prefill_chunk(cache, _ptr(Q), _ptr(K), _ptr(V), int(m), _ptr(workspace),
                                  int(ws_bytes), _ptr(out), _stream(stream)), "h2o_prefill_chunk")


def h2o_decode_step(cache, q, k_new, v_new, out, stream=None) -> None:
    _check(_lib.h2o_decode_step(cache, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                _stream(stream)), "h2o_decode_step")


def h2o_cache_snapshot(cache, pos_out=None, acc_out=None, stream=None) -> None:
    _check(_lib.h2o_cache_snapshot(cache, _ptr(pos_out), _ptr(acc_out), _stream(stream)),
           "h2o_cache_snapshot")


def h2o_cache_restore(cache, K, V, acc, pos, tokens_seen, stream=None) -> None:
    _check(_lib.h2o_cache_restore(cache, _ptr(K), _ptr(V), _ptr(acc), _ptr(pos), int(tokens_seen),
                                  _stream(stream)), "h2o_cache_restore")


def h2o_cache_rolled_positions(cache, rolled_out, stream=None) -> None:
    _check(_lib.h2o_cache_rolled_positions(cache, _ptr(rolled_out), _stream(stream)),
           "h2o_cache_rolled_positions")


def h2o_cache_validate(cache, flags_out, stream=None) -> None:
    _check(_lib.h2o_cache_validate(cache, _ptr(flags_out), _stream(stream)), "h2o_cache_validate")


def h2o_cache_tokens_seen(cache) -> int:
    return int(_lib.h2o_cache_tokens_seen(cache))


def h2o_cache_regions(cache):
    """Device addresses (K, V, acc, pos) of the cache's regions."""
    K, V, A, P = _vp(), _vp(), _vp(), _vp()
    _check(_lib.h2o_cache_regions(cache, ctypes.byref(K), ctypes.byref(V), ctypes.byref(A),
                                  ctypes.byref(P)), "h2o_cache_regions")
    return K.value, V.value, A.value, P.value


class H2OCache:
    """Owns the device memory (a torch byte tensor) and the library handle of
    one cache; methods forward to the entry points of the same name."""

    def __init__(self, batch, heads, head_dim, heavy, recent, dtype=torch.float16, scale=0.0,
                 device="cuda", stream=None, rank=0, kv_bits=0, protect=0, stride=0):
        self.cfg = make_config(batch, heads, head_dim, heavy, recent, dtype, scale, rank, kv_bits,
                               protect, stride)
        self.dtype = dtype if isinstance(dtype, torch.dtype) else TORCH_DTYPES[dtype]
        self.device = torch.device(device)
        self.budget = int(heavy) + int(recent)
        nbytes = h2o_cache_bytes(self.cfg)
        if nbytes == 0:
            raise H2OError(H2O_EINVAL, "h2o_cache_bytes")
        self.nbytes = nbytes
        self.mem = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.handle = h2o_cache_init(self.cfg, self.mem, nbytes, stream)
        self._ws = None

    def close(self):
        if getattr(self, "handle", None):
            _lib.h2o_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: module globals may be gone
            pass

    @property
    def shape_heads(self):
        return self.cfg.batch, self.cfg.heads

    def workspace(self, n: int) -> torch.Tensor:
        need = h2o_prefill_workspace_bytes(self.cfg, n)
        if need == 0:
            raise H2OError(H2O_EUNSUPPORTED, "h2o_prefill_workspace_bytes")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    # -- argument checks: a tensor of the wrong size behind a raw pointer would be an
    # out-of-bounds device access, so the class refuses it on the host
    def _expect(self, x, shape, dtype, what):
        if x is None:
            return
        if not isinstance(x, torch.Tensor):
            raise TypeError("%s: expected a tensor" % what)
        if x.device != self.mem.device:
            raise ValueError("%s lives on %s, the cache on %s" % (what, x.device, self.mem.device))
        if x.dtype != dtype:
            raise ValueError("%s has dtype %s, expected %s" % (what, x.dtype, dtype))
        if tuple(x.shape) != tuple(shape):
            raise ValueError("%s has shape %s, expected %s" % (what, tuple(x.shape), tuple(shape)))
        if not x.is_contiguous():
            raise ValueError("%s must be contiguous" % what)

    def _expect_prompt(self, Q, K, V, names="Q K V"):
        B, Hh = self.shape_heads
        n = (Q if Q is not None else K).shape[-2]
        for x, nm in zip((Q, K, V), names.split()):
            self._expect(x, (B, Hh, n, self.cfg.head_dim), self.dtype, nm)
        return n

    def _stored_row_shape(self):
        B, Hh = self.shape_heads
        if self.cfg.kv_bits == 4:
            return (B, Hh, self.budget, q4_row_bytes(self.cfg.head_dim)), torch.uint8
        return (B, Hh, self.budget, self.cfg.head_dim), self.dtype

    def reset(self, stream=None):
        h2o_cache_reset(self.handle, stream)

    def prefill_scores(self, Q, K, V, colsum_out=None, stream=None):
        n = self._expect_prompt(Q, K, V)
        self._expect(colsum_out, (*self.shape_heads, n), torch.float32, "colsum_out")
        ws = self.workspace(n)
        h2o_prefill_scores(self.handle, Q, K, V, n, ws, ws.numel(), colsum_out, stream)

    def prefill_scores_noalloc(self, Q, K, V, colsum_out=None, stream=None):
        """The same on the library's built-in scratch (no workspace is allocated)."""
        n = self._expect_prompt(Q, K, V)
        self._expect(colsum_out, (*self.shape_heads, n), torch.float32, "colsum_out")
        h2o_prefill_scores_noalloc(self.handle, Q, K, V, n, colsum_out, stream)

    def prefill_chunk(self, Q, K, V, out=None, stream=None):
        """The next Q.shape[-2] prompt tokens as one chunk ([batch, heads, m, head_dim],
        contiguous); `out` (same shape) receives the chunk's attention output if given."""
        m = self._expect_prompt(Q, K, V)
        self._expect(out, Q.shape, self.dtype, "out")
        need = h2o_prefill_chunk_workspace_bytes(self.cfg, m, out is not None)
        if need == 0:
            raise H2OError(H2O_EUNSUPPORTED, "h2o_prefill_chunk_workspace_bytes")
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        h2o_prefill_chunk(self.handle, Q, K, V, m, self._ws, self._ws.numel(), out, stream)

    def prefill_select(self, K, V, score, stream=None):
        n = self._expect_prompt(None, K, V)
        self._expect(score, (*self.shape_heads, n), torch.float32, "score")
        h2o_prefill_select(self.handle, K, V, score, n, stream)

    def decode_step(self, q, k_new, v_new, out, stream=None):
        shape = (*self.shape_heads, self.cfg.head_dim)
        for x, nm in ((q, "q"), (k_new, "k_new"), (v_new, "v_new"), (out, "out")):
            self._expect(x, shape, self.dtype, nm)
        h2o_decode_step(self.handle, q, k_new, v_new, out, stream)

    def snapshot(self, stream=None):
        B, Hh = self.shape_heads
        pos = torch.empty((B, Hh, self.budget), dtype=torch.int32, device=self.device)
        acc = torch.empty((B, Hh, self.budget), dtype=torch.float32, device=self.device)
        h2o_cache_snapshot(self.handle, pos, acc, stream)
        return pos, acc

    def rolled_positions(self, stream=None):
        """int32 [B, Hh, k]: rank of each occupied slot's token among the cached tokens by position."""
        B, Hh = self.shape_heads
        out = torch.empty((B, Hh, self.budget), dtype=torch.int32, device=self.device)
        h2o_cache_rolled_positions(self.handle, out, stream)
        return out

    def validate(self, stream=None) -> torch.Tensor:
        """int32 [B, Hh] (device): 0 for every head whose bookkeeping is consistent, else the
        H2O_BAD_* bits of h2o_cache_validate.  Enqueued; read it after synchronising."""
        flags = torch.empty(self.shape_heads, dtype=torch.int32, device=self.device)
        h2o_cache_validate(self.handle, flags, stream)
        return flags

    def restore(self, K, V, acc, pos, tokens_seen, stream=None, validate=False):
        """Loads a complete state.  validate=True also checks it on the device
        (synchronises) and raises ValueError for a state the steps cannot run on."""
        rshape, rdtype = self._stored_row_shape()
        self._expect(K, rshape, rdtype, "K")
        self._expect(V, rshape, rdtype, "V")
        self._expect(acc, (*self.shape_heads, self.budget), torch.float32, "acc")
        self._expect(pos, (*self.shape_heads, self.budget), torch.int32, "pos")
        h2o_cache_restore(self.handle, K, V, acc, pos, tokens_seen, stream)
        if validate:
            flags = self.validate(stream).cpu()           # the copy synchronises
            if bool(flags.any()):
                bad = flags.nonzero()[0].tolist()
                raise ValueError("restored state is inconsistent: head %s has flags %d (see "
                                 "h2o_cache_validate)" % (tuple(bad), int(flags[tuple(bad)])))

    @property
    def tokens_seen(self) -> int:
        return h2o_cache_tokens_seen(self.handle)

    def views(self):
        """Tensor views (K, V, acc, pos) of the cache's regions: K, V [B, Hh, k, d]
        in the cache dtype (4-bit storage: uint8 [B, Hh, k, row bytes], codes then
        (scale, min) pairs), acc [B, Hh, k] float32, pos [B, Hh, k] int32.  They
        alias the cache memory (for inspection and checkpointing)."""
        B, Hh = self.shape_heads
        d, k = self.cfg.head_dim, self.budget
        kaddr, vaddr, aaddr, paddr = h2o_cache_regions(self.handle)
        base = self.mem.data_ptr()
        es = 4 if self.dtype == torch.float32 else 2
        cnt = B * Hh * k

        def view(addr, nbytes, dtype, shape):
            off = addr - base
            return self.mem[off:off + nbytes].view(dtype).view(shape)
        if self.cfg.kv_bits == 4:
            rowb = q4_row_bytes(d)
            return (view(kaddr, cnt * rowb, torch.uint8, (B, Hh, k, rowb)),
                    view(vaddr, cnt * rowb, torch.uint8, (B, Hh, k, rowb)),
                    view(aaddr, cnt * 4, torch.float32, (B, Hh, k)),
                    view(paddr, cnt * 4, torch.int32, (B, Hh, k)))
        return (view(kaddr, cnt * d * es, self.dtype, (B, Hh, k, d)),
                view(vaddr, cnt * d * es, self.dtype, (B, Hh, k, d)),
                view(aaddr, cnt * 4, torch.float32, (B, Hh, k)),
                view(paddr, cnt * 4, torch.int32, (B, Hh, k)))

    def kv_views(self):
        return self.views()[:2]


def prefill_colsum(cfg: h2o_config, Q, K, stream=None) -> torch.Tensor:
    """Convenience wrapper: allocates workspace and output with torch and calls
    h2o_prefill_colsum.  Q, K: [B, Hh, n, d]."""
    n = Q.shape[-2]
    need = h2o_prefill_workspace_bytes(cfg, n)
    if need == 0:
        raise H2OError(H2O_EUNSUPPORTED, "h2o_prefill_workspace_bytes")
    ws = torch.empty(need, dtype=torch.uint8, device=Q.device)
    out = torch.empty(Q.shape[:-1], dtype=torch.float32, device=Q.device)
    h2o_prefill_colsum(cfg, Q, K, n, ws, need, out, stream)
    return out
