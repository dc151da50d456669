"""Thin ctypes binding of libmixkvq.so.

Argument marshalling only: every step of the hot path runs in the HIP kernels
behind the C ABI (include/mixkvq.h).  torch is used for device allocations and
streams.  There is no CPU fallback: loading fails loudly when the library has
not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmixkvq.so")

PATH_NONE, PATH_MATRIX, PATH_VECTOR = 0, 1, 2

EXPORTS = ("mixkvq_block_layout", "mixkvq_cache_sizes", "mixkvq_cache_create", "mixkvq_cache_destroy",
           "mixkvq_cache_set_block_table", "mixkvq_cache_set_state", "mixkvq_cache_set_state_seq", "mixkvq_cache_reset", "mixkvq_cache_reset_seq", "mixkvq_cache_state", "mixkvq_cache_state_seq",
           "mixkvq_select_channels", "mixkvq_select_channels_seq", "mixkvq_quantize_append", "mixkvq_quantize_append_seq", "mixkvq_prefill",
           "mixkvq_decode_attention", "mixkvq_decode_attention_noalloc", "mixkvq_decode_step", "mixkvq_set_timing_events", "mixkvq_decode_path",
           "mixkvq_strerror")


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "T_max", "Gk", "Gv", "R", "k4", "k16",
                                         "flush_mode", "score_mode", "qacc_reset_on_flush", "policy")] + \
               [("tau16", C.c_double), ("tau4", C.c_double), ("sink", C.c_int32), ("in_dtype", C.c_int32)]


class Sizes(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("blocks", "res_k", "res_v", "qacc", "workspace")]


class Buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("blocks", "res_k", "res_v", "qacc", "workspace")]


class BlockLayout(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("NL", "Wlo", "NLp", "NG", "NVG", "W4", "off_idx", "off_kmax", "off_klo_s",
                                         "off_klo_z",
                                         "off_k4_s", "off_k4_z", "off_klo", "off_k4", "off_k16", "off_v", "off_v_s",
                                         "off_v_z", "rec_bytes", "v_interleave")]


class MixKVQError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"mixkvq error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Load the built shared library; raise if it is missing (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_19206_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    i32, i64p, vp = C.c_int32, C.POINTER(C.c_int64), C.c_void_p
    lib.mixkvq_block_layout.argtypes = [C.POINTER(Config), C.POINTER(BlockLayout)]
    lib.mixkvq_cache_sizes.argtypes = [C.POINTER(Config), C.POINTER(Sizes)]
    lib.mixkvq_cache_create.argtypes = [C.POINTER(Config), C.POINTER(Buffers), C.POINTER(vp)]
    lib.mixkvq_cache_destroy.argtypes = [vp]
    lib.mixkvq_cache_destroy.restype = None
    lib.mixkvq_cache_reset.argtypes = [vp, vp]
    lib.mixkvq_cache_state.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.mixkvq_cache_set_block_table.argtypes = [vp, vp]
    lib.mixkvq_cache_set_state.argtypes = [vp, C.c_int64, i32, i32]
    lib.mixkvq_cache_set_state_seq.argtypes = [vp, i32, C.c_int64, i32, i32]
    lib.mixkvq_cache_reset_seq.argtypes = [vp, i32, vp]
    lib.mixkvq_cache_state_seq.argtypes = [vp, i32, C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.mixkvq_select_channels_seq.argtypes = [vp, i32, vp, i32, i64p, vp, i32, i64p, vp, vp]
    lib.mixkvq_quantize_append_seq.argtypes = [vp, i32, vp, vp, i32, i64p, vp, vp]
    lib.mixkvq_select_channels.argtypes = [vp, vp, i32, i64p, vp, i32, i64p, vp, vp]
    lib.mixkvq_quantize_append.argtypes = [vp, vp, vp, i32, i64p, vp, vp]
    lib.mixkvq_prefill.argtypes = [vp, vp, i32, i64p, vp, vp, i32, i64p, vp, vp]
    lib.mixkvq_decode_attention.argtypes = [vp, vp, vp, vp, C.c_float, i32, vp]
    lib.mixkvq_decode_attention_noalloc.argtypes = [vp, vp, vp, vp, C.c_float, i32, vp]
    lib.mixkvq_decode_step.argtypes = [vp, vp, vp, i64p, vp, vp, vp, C.c_float, i32, vp]
    lib.mixkvq_set_timing_events.argtypes = [vp, vp, vp]
    lib.mixkvq_decode_path.argtypes = [vp]
    lib.mixkvq_strerror.argtypes = [i32]
    lib.mixkvq_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("mixkvq_cache_destroy", "mixkvq_strerror"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise MixKVQError(rc, load_library().mixkvq_strerror(rc).decode())


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _strides3(t: torch.Tensor):
    assert t.dim() == 4 and t.stride(3) == 1, "expected [B, H, L, D] with unit channel stride"
    return (C.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def make_config(**kw) -> Config:
    cfg = Config()
    cfg.tau16 = cfg.tau4 = float("inf")
    for k, v in kw.items():
        setattr(cfg, k, float(v) if k in ("tau16", "tau4") else int(v))
    return cfg


def block_layout(cfg: Config) -> BlockLayout:
    lay = BlockLayout()
    _check(load_library().mixkvq_block_layout(C.byref(cfg), C.byref(lay)))
    return lay


def cache_sizes(cfg: Config) -> Sizes:
    sz = Sizes()
    _check(load_library().mixkvq_cache_sizes(C.byref(cfg), C.byref(sz)))
    return sz


class Cache:
    """Owns the torch device buffers and the library's host handle."""

    def __init__(self, cfg: Config, device="cuda:0"):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.layout = block_layout(cfg)
        sz = cache_sizes(cfg)
        self.sizes = sz
        mk = lambda n: torch.empty(int(n), dtype=torch.uint8, device=self.device)
        self.blocks, self.res_k, self.res_v = mk(sz.blocks), mk(sz.res_k), mk(sz.res_v)
        self.qacc, self.workspace = mk(sz.qacc), mk(sz.workspace)
        bufs = Buffers(self.blocks.data_ptr(), self.res_k.data_ptr(), self.res_v.data_ptr(), self.qacc.data_ptr(),
                       self.workspace.data_ptr())
        h = C.c_void_p()
        _check(self.lib.mixkvq_cache_create(C.byref(cfg), C.byref(bufs), C.byref(h)))
        self.handle = h
        self.reset()

    def __del__(self):
        h = getattr(self, "handle", None)
        if h:
            self.lib.mixkvq_cache_destroy(h)
            self.handle = None

    @property
    def ks(self) -> int:
        return self.cfg.k4 + self.cfg.k16

    def reset(self, stream=None):
        _check(self.lib.mixkvq_cache_reset(self.handle, _stream_ptr(stream)))

    def state(self):
        """(quantized tokens, tokens in the residual window)."""
        nq, r = C.c_int64(), C.c_int32()
        _check(self.lib.mixkvq_cache_state(self.handle, C.byref(nq), C.byref(r), None))
        return nq.value, r.value

    def snapshot(self):
        """Copies of the five device buffers and the token counts of every sequence (everything the cache holds)."""
        bufs = [t.clone() for t in (self.blocks, self.res_k, self.res_v, self.qacc, self.workspace)]
        return bufs, [self.state_seq(b) for b in range(self.cfg.B)]

    def restore(self, snap):
        """Takes a snapshot of a cache of the same configuration back in."""
        bufs, states = snap
        for dst, src in zip((self.blocks, self.res_k, self.res_v, self.qacc, self.workspace), bufs):
            dst.copy_(src)
        if all(st == states[0] for st in states):
            _check(self.lib.mixkvq_cache_set_state(self.handle, *states[0]))
        else:
            for b, st in enumerate(states):
                _check(self.lib.mixkvq_cache_set_state_seq(self.handle, b, *st))

    @property
    def rec_tokens(self) -> int:
        """Tokens per block record: R, except 128 for R = 256 and 32 for R = 96 with Gk = 16 or 32 (a block is then
        stored as two / three records with one channel list)."""
        c = self.cfg
        if c.R > 128:
            return 128
        if c.R == 96 and 32 % c.Gk == 0:
            return 32
        return c.R

    def sink_count(self) -> int:
        n = C.c_int32()
        _check(self.lib.mixkvq_cache_state(self.handle, None, None, C.byref(n)))
        return n.value

    def set_block_table(self, table):
        """table: int32 device tensor [B, T_max/rec_tokens] (kept alive here) or None.  The block buffer becomes the
        pool: B * T_max/rec_tokens slots of Hkv records each."""
        if table is None:
            _check(self.lib.mixkvq_cache_set_block_table(self.handle, None))
        else:
            assert table.dtype == torch.int32 and table.is_contiguous() and table.is_cuda
            _check(self.lib.mixkvq_cache_set_block_table(self.handle, table.data_ptr()))
        self._table = table

    def pool_records(self) -> torch.Tensor:
        """uint8 [slots, Hkv, rec_bytes] view of the block buffer as a pool (paged layout)."""
        slots = self.cfg.B * (self.cfg.T_max // self.rec_tokens)
        n = slots * self.cfg.Hkv * self.layout.rec_bytes
        return self.blocks[:n].view(slots, self.cfg.Hkv, self.layout.rec_bytes)

    # ---- one sequence of the batch (sequences may differ in length) ----
    def reset_seq(self, b: int, stream=None):
        _check(self.lib.mixkvq_cache_reset_seq(self.handle, int(b), _stream_ptr(stream)))

    def state_seq(self, b: int):
        """(quantized tokens, tokens in the residual window, tokens in the sink) of sequence b."""
        nq, r, ns = C.c_int64(), C.c_int32(), C.c_int32()
        _check(self.lib.mixkvq_cache_state_seq(self.handle, int(b), C.byref(nq), C.byref(r), C.byref(ns)))
        return nq.value, r.value, ns.value

    def select_channels_seq(self, b: int, q, k, sel=None, stream=None):
        """q: fp16 [Hq, Lq, D] or None; k: fp16 [Hkv, L, D].  Returns u8 [Hkv, ks] on the device."""
        if sel is None:
            sel = torch.empty((self.cfg.Hkv, self.ks), dtype=torch.uint8, device=self.device)
        s2 = lambda t: (C.c_int64 * 2)(t.stride(0), t.stride(1))
        qp, Lq, qs = (None, 0, None) if q is None else (q.data_ptr(), q.shape[1], s2(q))
        _check(self.lib.mixkvq_select_channels_seq(self.handle, int(b), qp, Lq, qs, k.data_ptr(), k.shape[1], s2(k),
                                                   sel.data_ptr(), _stream_ptr(stream)))
        return sel

    def quantize_append_seq(self, b: int, k_new, v_new, sel=None, stream=None):
        """k_new, v_new: fp16 [Hkv, n, D] with equal strides."""
        assert k_new.dim() == 3 and k_new.stride(2) == 1 and k_new.stride() == v_new.stride()
        st = (C.c_int64 * 2)(k_new.stride(0), k_new.stride(1))
        _check(self.lib.mixkvq_quantize_append_seq(self.handle, int(b), k_new.data_ptr(), v_new.data_ptr(),
                                                   k_new.shape[1], st, None if sel is None else sel.data_ptr(),
                                                   _stream_ptr(stream)))

    def select_channels(self, q, k, sel=None, stream=None):
        """q: fp16 [B, Hq, Lq, D] or None; k: fp16 [B, Hkv, L, D].  Returns u8 [B, Hkv, ks] on the device."""
        if sel is None:
            sel = torch.empty((self.cfg.B, self.cfg.Hkv, self.ks), dtype=torch.uint8, device=self.device)
        qp, Lq, qs = (None, 0, None) if q is None else (q.data_ptr(), q.shape[2], _strides3(q))
        _check(self.lib.mixkvq_select_channels(self.handle, qp, Lq, qs, k.data_ptr(), k.shape[2], _strides3(k),
                                               sel.data_ptr(), _stream_ptr(stream)))
        return sel

    def prefill(self, q, k, v, sel=None, stream=None):
        """q: fp16 [B, Hq, Lq, D] or None; k, v: fp16 [B, Hkv, L, D] with equal strides.  Scoring, selection and
        append of a prompt in one call; returns the selection u8 [B, Hkv, ks]."""
        assert k.stride() == v.stride() and k.shape == v.shape
        if sel is None:
            sel = torch.empty((self.cfg.B, self.cfg.Hkv, self.ks), dtype=torch.uint8, device=self.device)
        qp, Lq, qs = (None, 0, None) if q is None else (q.data_ptr(), q.shape[2], _strides3(q))
        _check(self.lib.mixkvq_prefill(self.handle, qp, Lq, qs, k.data_ptr(), v.data_ptr(), k.shape[2], _strides3(k),
                                       sel.data_ptr(), _stream_ptr(stream)))
        return sel

    def quantize_append(self, k_new, v_new, sel=None, stream=None):
        """k_new, v_new: fp16 [B, Hkv, n, D] with equal strides."""
        assert k_new.stride() == v_new.stride() and k_new.shape == v_new.shape
        _check(self.lib.mixkvq_quantize_append(self.handle, k_new.data_ptr(), v_new.data_ptr(), k_new.shape[2],
                                               _strides3(k_new), None if sel is None else sel.data_ptr(),
                                               _stream_ptr(stream)))

    def decode_attention(self, q, out=None, lse=None, scale=0.0, accumulate_q=False, stream=None):
        """q: fp16 [B, Hq, D] contiguous.  Returns (out fp16 [B, Hq, D], lse fp32 [B, Hq])."""
        assert q.is_contiguous()
        if out is None:
            out = torch.empty_like(q)
        if lse is None:
            lse = torch.empty(q.shape[:2], dtype=torch.float32, device=self.device)
        _check(self.lib.mixkvq_decode_attention(self.handle, q.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                                float(scale), int(bool(accumulate_q)), _stream_ptr(stream)))
        return out, lse

    def decode_attention_noalloc(self, q, out, lse, scale=0.0, accumulate_q=False, stream=None):
        """decode_attention through the entry point that allocates nothing: the caller passes every tensor."""
        assert q.is_contiguous() and out.is_contiguous() and lse.is_contiguous()
        _check(self.lib.mixkvq_decode_attention_noalloc(self.handle, q.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                                        float(scale), int(bool(accumulate_q)), _stream_ptr(stream)))
        return out, lse

    def decode_step(self, k_new, v_new, q, out=None, lse=None, scale=0.0, accumulate_q=False, stream=None):
        """k_new, v_new: fp16 [B, Hkv, 1, D]; q: fp16 [B, Hq, D] contiguous.  Append + attention in one call."""
        assert q.is_contiguous() and k_new.stride() == v_new.stride() and k_new.shape[2] == 1
        if out is None:
            out = torch.empty_like(q)
        if lse is None:
            lse = torch.empty(q.shape[:2], dtype=torch.float32, device=self.device)
        _check(self.lib.mixkvq_decode_step(self.handle, k_new.data_ptr(), v_new.data_ptr(), _strides3(k_new),
                                           q.data_ptr(), out.data_ptr(), lse.data_ptr(), float(scale),
                                           int(bool(accumulate_q)), _stream_ptr(stream)))
        return out, lse

    def set_timing_events(self, start_event, stop_event):
        """start_event, stop_event: raw hipEvent_t handles (ints) or None, None."""
        _check(self.lib.mixkvq_set_timing_events(self.handle, start_event, stop_event))

    def decode_path(self) -> int:
        """Kernel of the last attention call: PATH_NONE, PATH_MATRIX (matrix-core kernel) or PATH_VECTOR (fallback)."""
        return int(self.lib.mixkvq_decode_path(self.handle))

    # helpers for tests: views of the raw buffers
    def block_records(self) -> torch.Tensor:
        """uint8 [P, NB, rec_bytes] view of the block records (NB = T_max / rec_tokens)."""
        P = self.cfg.B * self.cfg.Hkv
        NB = self.cfg.T_max // self.rec_tokens
        n = P * NB * self.layout.rec_bytes
        return self.blocks[:n].view(P, NB, self.layout.rec_bytes)

    def fp16_rows(self):
        """fp16 views [P, sink + R, D] of the key and value rows kept in full precision (sink rows first)."""
        P = self.cfg.B * self.cfg.Hkv
        rows = self.cfg.sink + self.cfg.R
        n = P * rows * self.cfg.D * 2
        shape = (P, rows, self.cfg.D)
        return self.res_k[:n].view(torch.float16).view(shape), self.res_v[:n].view(torch.float16).view(shape)

    def residual(self):
        k, v = self.fp16_rows()
        return k[:, self.cfg.sink:], v[:, self.cfg.sink:]

    def sink(self):
        k, v = self.fp16_rows()
        return k[:, :self.cfg.sink], v[:, :self.cfg.sink]

    def query_accumulator(self):
        P = self.cfg.B * self.cfg.Hkv
        a = self.qacc[:P * (self.cfg.D + 1) * 8].view(torch.int64)
        return a[:P * self.cfg.D].view(P, self.cfg.D), a[P * self.cfg.D:]
