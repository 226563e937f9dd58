"""Thin ctypes binding of libhashattn.so (argument marshalling only).

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/hashattn.h; this module turns torch tensors into device pointers and
passes torch's current HIP stream.  There is no CPU fallback: if the library
has not been built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhashattn.so")

OK, INVALID_ARG, UNSUPPORTED, SCRATCH_TOO_SMALL, HIP_ERROR = 0, 1, 2, 3, 4
STATUS_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "UNSUPPORTED", 3: "SCRATCH_TOO_SMALL", 4: "HIP_ERROR"}


class HashAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"hashattn status {status} ({STATUS_NAMES.get(status, '?')}): {message}")
        self.status = status


class Config(C.Structure):
    _fields_ = [("head_dim", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("bits", C.c_int32), ("page_size", C.c_int32), ("max_batch", C.c_int32),
                ("max_context", C.c_int64), ("max_k", C.c_int64)]


class MlpStruct(C.Structure):
    _fields_ = [("n_heads", C.c_int32), ("n_layers", C.c_int32), ("dims", C.c_int32 * 5),
                ("W", C.c_void_p * 4), ("bias", C.c_void_p * 4)]


class KvStruct(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("codes", C.c_void_p),
                ("page_table", C.c_void_p), ("seq_lens", C.c_void_p), ("n_max", C.c_int64),
                ("n_pages", C.c_int64), ("max_pages_per_seq", C.c_int32), ("max_seq_len", C.c_int32)]


_lib = None


def load() -> C.CDLL:
    """Load libhashattn.so; raises if it was not built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2412_14468_amd.build` "
            "(hipcc --offload-arch=gfx950); the HashAttention path has no CPU fallback")
    # torch goes first: its HIP runtime must be the one this process uses (device memory and streams
    # come from torch), and the library must bind to that same runtime rather than load a second one
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.hashattn_create.restype = i32
    L.hashattn_create.argtypes = [C.POINTER(vp), C.POINTER(Config)]
    L.hashattn_destroy.restype = i32
    L.hashattn_destroy.argtypes = [vp]
    L.hashattn_last_error.restype = C.c_char_p
    L.hashattn_last_error.argtypes = [vp]
    L.hashattn_scratch_bytes.restype = i64
    L.hashattn_scratch_bytes.argtypes = [vp]
    L.hashattn_selftest_set_append_counter.restype = i32
    L.hashattn_selftest_set_append_counter.argtypes = [vp, i32, vp]
    L.hashattn_selftest_set_topk_path.restype = i32
    L.hashattn_selftest_set_topk_path.argtypes = [vp, i32]
    L.hashattn_encode_keys.restype = i32
    L.hashattn_encode_keys.argtypes = [vp, C.POINTER(MlpStruct), vp, vp, i32, i64, C.POINTER(KvStruct), vp]
    L.hashattn_encode_query.restype = i32
    L.hashattn_encode_query.argtypes = [vp, C.POINTER(MlpStruct), vp, i32, vp, vp]
    L.hashattn_score_topk.restype = i32
    L.hashattn_score_topk.argtypes = [vp, vp, C.POINTER(KvStruct), i32, vp, i32, vp, vp, vp, vp]
    L.hashattn_score_topk_window.restype = i32
    L.hashattn_score_topk_window.argtypes = [vp, vp, C.POINTER(KvStruct), i32, vp, i32, i32, i32, vp, vp, vp, vp]
    L.hashattn_encode_score_topk.restype = i32
    L.hashattn_encode_score_topk.argtypes = [vp, C.POINTER(MlpStruct), vp, C.POINTER(KvStruct), i32, vp, i32, i32, i32, vp, vp, vp, vp, vp]
    L.hashattn_decode_step.restype = i32
    L.hashattn_decode_step.argtypes = [vp, C.POINTER(MlpStruct), vp, vp, C.POINTER(MlpStruct), vp, C.POINTER(KvStruct), i32, vp,
                                       i32, i32, i32, C.c_float, vp, vp, vp, vp, vp, vp]
    L.hashattn_gather_attend.restype = i32
    L.hashattn_gather_attend.argtypes = [vp, vp, C.POINTER(KvStruct), vp, vp, i32, i32, C.c_float, vp, vp]
    L.hashattn_gather_attend_noalloc.restype = i32
    L.hashattn_gather_attend_noalloc.argtypes = [i32, i32, i32, vp, C.POINTER(KvStruct), vp, vp, i32, i32, C.c_float, vp, vp]
    L.hashattn_dense_attend.restype = i32
    L.hashattn_dense_attend.argtypes = [vp, vp, C.POINTER(KvStruct), i32, C.c_float, vp, vp]
    _lib = L
    return L


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a tensor-like object, an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def hashattn_gather_attend_noalloc(n_q_heads: int, n_kv_heads: int, page_size: int, q, cache: "KvCache", idx, count,
                                   batch: int, k_max: int, scale: float, out, stream=None) -> None:
    """GATHER-ATT without a context: split partials live in the library's static device array."""
    L = load()
    st = L.hashattn_gather_attend_noalloc(n_q_heads, n_kv_heads, page_size, _ptr(q), C.byref(cache.c), _ptr(idx),
                                          _ptr(count), batch, k_max, float(scale), _ptr(out), _stream(stream))
    if st != OK:
        raise HashAttnError(st, L.hashattn_last_error(None).decode())


class Mlp:
    """Device-resident mapping network: weights[l] is a cuda fp32 tensor [n_heads, dims[l], dims[l+1]]."""

    def __init__(self, weights: Sequence, biases: Optional[Sequence] = None):
        self.weights = list(weights)
        self.biases = list(biases) if biases is not None else [None] * len(self.weights)
        s = MlpStruct()
        s.n_heads = int(self.weights[0].shape[0])
        s.n_layers = len(self.weights)
        for l, w in enumerate(self.weights):
            s.dims[l] = int(w.shape[1])
            s.dims[l + 1] = int(w.shape[2])
            s.W[l] = _ptr(w)
            s.bias[l] = _ptr(self.biases[l])
        self.c = s


class KvCache:
    """Caller-owned KV cache + key-code store (cuda tensors are referenced, never copied)."""

    def __init__(self, k, v, codes, seq_lens, max_seq_len: int, page_table=None):
        self.k, self.v, self.codes, self.seq_lens, self.page_table = k, v, codes, seq_lens, page_table
        s = KvStruct()
        s.k, s.v, s.codes, s.seq_lens = _ptr(k), _ptr(v), _ptr(codes), _ptr(seq_lens)
        s.page_table = _ptr(page_table)
        if page_table is None:
            s.n_max = int(k.shape[2])
            s.n_pages = 0
            s.max_pages_per_seq = 0
        else:
            s.n_max = 0
            s.n_pages = int(k.shape[0])
            s.max_pages_per_seq = int(page_table.shape[1])
        s.max_seq_len = int(max_seq_len)
        self.c = s

    @property
    def max_seq_len(self) -> int:
        return int(self.c.max_seq_len)

    @max_seq_len.setter
    def max_seq_len(self, n: int) -> None:
        self.c.max_seq_len = int(n)


class Context:
    """Owns the library's scratch for one attention-layer shape on the current device."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, max_batch: int, max_context: int, max_k: int,
                 page_size: int = 0, head_dim: int = 128, bits: int = 32):
        L = load()
        cfg = Config(head_dim, n_q_heads, n_kv_heads, bits, page_size, max_batch, max_context, max_k)
        h = C.c_void_p()
        st = L.hashattn_create(C.byref(h), C.byref(cfg))
        if st != OK:
            raise HashAttnError(st, L.hashattn_last_error(None).decode())
        self.h = h
        self.cfg = cfg

    def close(self) -> None:
        if getattr(self, "h", None):
            load().hashattn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int) -> None:
        if st != OK:
            raise HashAttnError(st, load().hashattn_last_error(self.h).decode())

    @property
    def scratch_bytes(self) -> int:
        return int(load().hashattn_scratch_bytes(self.h))

    def hashattn_selftest_set_topk_path(self, path: int) -> None:
        self._check(load().hashattn_selftest_set_topk_path(self.h, int(path)))

    def hashattn_selftest_set_append_counter(self, value: int, stream=None) -> None:
        self._check(load().hashattn_selftest_set_append_counter(self.h, int(value), _stream(stream)))

    # --- the four calls of the path (+ the dense comparison kernel) ---
    def hashattn_encode_keys(self, phi_kv: Mlp, k_new, v_new, batch: int, n_new: int, cache: KvCache,
                             stream=None) -> None:
        self._check(load().hashattn_encode_keys(self.h, C.byref(phi_kv.c), _ptr(k_new), _ptr(v_new),
                                                batch, n_new, C.byref(cache.c), _stream(stream)))

    def hashattn_encode_query(self, phi_q: Mlp, q, batch: int, q_codes, stream=None) -> None:
        self._check(load().hashattn_encode_query(self.h, C.byref(phi_q.c), _ptr(q), batch, _ptr(q_codes),
                                                 _stream(stream)))

    def hashattn_score_topk(self, q_codes, cache: KvCache, batch: int, k_per_seq, k_max: int, idx, count,
                            threshold=None, stream=None) -> None:
        self._check(load().hashattn_score_topk(self.h, _ptr(q_codes), C.byref(cache.c), batch, _ptr(k_per_seq),
                                               k_max, _ptr(idx), _ptr(count), _ptr(threshold), _stream(stream)))

    def hashattn_score_topk_window(self, q_codes, cache: KvCache, batch: int, k_per_seq, k_max: int, n_sink: int,
                                   n_local: int, idx, count, threshold=None, stream=None) -> None:
        self._check(load().hashattn_score_topk_window(self.h, _ptr(q_codes), C.byref(cache.c), batch,
                                                      _ptr(k_per_seq), k_max, n_sink, n_local, _ptr(idx),
                                                      _ptr(count), _ptr(threshold), _stream(stream)))

    def hashattn_encode_score_topk(self, phi_q: Mlp, q, cache: KvCache, batch: int, k_per_seq, k_max: int, n_sink: int,
                                   n_local: int, q_codes, idx, count, threshold=None, stream=None) -> None:
        self._check(load().hashattn_encode_score_topk(self.h, C.byref(phi_q.c), _ptr(q), C.byref(cache.c), batch,
                                                      _ptr(k_per_seq), k_max, n_sink, n_local, _ptr(q_codes), _ptr(idx),
                                                      _ptr(count), _ptr(threshold), _stream(stream)))

    def hashattn_decode_step(self, phi_kv: Optional[Mlp], k_new, v_new, phi_q: Mlp, q, cache: KvCache, batch: int, k_per_seq,
                             k_max: int, n_sink: int, n_local: int, scale: float, q_codes, idx, count, threshold, out,
                             stream=None) -> None:
        self._check(load().hashattn_decode_step(self.h, C.byref(phi_kv.c) if phi_kv is not None else None, _ptr(k_new),
                                                _ptr(v_new), C.byref(phi_q.c), _ptr(q), C.byref(cache.c), batch,
                                                _ptr(k_per_seq), k_max, n_sink, n_local, float(scale), _ptr(q_codes),
                                                _ptr(idx), _ptr(count), _ptr(threshold), _ptr(out), _stream(stream)))

    def hashattn_gather_attend(self, q, cache: KvCache, idx, count, batch: int, k_max: int, scale: float, out,
                               stream=None) -> None:
        self._check(load().hashattn_gather_attend(self.h, _ptr(q), C.byref(cache.c), _ptr(idx), _ptr(count),
                                                  batch, k_max, float(scale), _ptr(out), _stream(stream)))

    def hashattn_dense_attend(self, q, cache: KvCache, batch: int, scale: float, out, stream=None) -> None:
        self._check(load().hashattn_dense_attend(self.h, _ptr(q), C.byref(cache.c), batch, float(scale),
                                                 _ptr(out), _stream(stream)))
