"""ctypes/numpy front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It marshals numpy arrays into hashattn_oracle.c; every step of
the arithmetic is in that C file.  bf16 tensors are uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from .build import build as _build

_lib = None


class _Mlp(C.Structure):
    _fields_ = [("n_heads", C.c_int32), ("n_layers", C.c_int32), ("dims", C.c_int32 * 5),
                ("W", C.c_void_p * 4), ("bias", C.c_void_p * 4)]


class _Cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("codes", C.c_void_p),
                ("page_table", C.c_void_p), ("seq_lens", C.c_void_p), ("n_max", C.c_int64),
                ("max_pages_per_seq", C.c_int32), ("page_size", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32)]


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build(force=False))
        L.ha_oracle_num_threads.restype = C.c_int
        L.ha_oracle_set_threads.restype = None
        L.ha_oracle_set_threads.argtypes = [C.c_int]
        L.ha_oracle_encode_vec.restype = C.c_uint32
        L.ha_oracle_encode_vec.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.ha_oracle_encode_query.restype = None
        L.ha_oracle_encode_query.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                             C.c_void_p, C.c_void_p]
        L.ha_oracle_encode_keys.restype = None
        L.ha_oracle_encode_keys.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int, C.c_int64, C.c_void_p]
        L.ha_oracle_score.restype = C.c_int32
        L.ha_oracle_score.argtypes = [C.c_uint32, C.c_uint32]
        L.ha_oracle_scores.restype = None
        L.ha_oracle_scores.argtypes = [C.c_uint32, C.c_void_p, C.c_int64, C.c_void_p]
        for f in (L.ha_oracle_topk_sort, L.ha_oracle_topk_hist):
            f.restype = C.c_int64
            f.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.ha_oracle_gather_attend.restype = None
        L.ha_oracle_gather_attend.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                              C.c_void_p, C.c_int64, C.c_double, C.c_void_p]
        L.ha_oracle_dense_attend.restype = None
        L.ha_oracle_dense_attend.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                             C.c_int64, C.c_double, C.c_void_p]
        L.ha_oracle_decode_step.restype = None
        L.ha_oracle_decode_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                            C.c_void_p, C.c_int64, C.c_double, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ha_oracle_topk_window.restype = C.c_int64
        L.ha_oracle_topk_window.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                            C.c_void_p, C.c_void_p, C.c_void_p]
        L.ha_oracle_decode_step_window.restype = None
        L.ha_oracle_decode_step_window.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                   C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ha_oracle_token_contributions.restype = None
        L.ha_oracle_token_contributions.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int64,
                                                    C.c_double, C.c_void_p]
        L.ha_oracle_true_topk.restype = C.c_int64
        L.ha_oracle_true_topk.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int64, C.c_int64,
                                          C.c_double, C.c_void_p]
        L.ha_oracle_recall.restype = C.c_double
        L.ha_oracle_recall.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64]
        L.ha_oracle_encode_vec_wide.restype = None
        L.ha_oracle_encode_vec_wide.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.ha_oracle_score_wide.restype = C.c_int32
        L.ha_oracle_score_wide.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.ha_oracle_scores_wide.restype = None
        L.ha_oracle_scores_wide.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        L.ha_oracle_encode_query_wide.restype = None
        L.ha_oracle_encode_query_wide.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.ha_oracle_encode_keys_wide.restype = None
        L.ha_oracle_encode_keys_wide.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                                 C.c_int, C.c_int64, C.c_void_p]
        L.ha_oracle_decode_step_wide.restype = None
        L.ha_oracle_decode_step_wide.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                 C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().ha_oracle_num_threads())


def set_threads(n: int) -> None:
    """Threads for the (sequence, head) loops from now on (used for timing; results do not depend on it)."""
    lib().ha_oracle_set_threads(int(n))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    assert a.dtype == np.dtype(dtype), (a.dtype, dtype)
    assert a.flags["C_CONTIGUOUS"]
    return a


class Mlp:
    """Mapping network F: weights[l] is [n_heads, dims[l], dims[l+1]] fp32 (y = x W)."""

    def __init__(self, weights: Sequence[np.ndarray], biases: Optional[Sequence[Optional[np.ndarray]]] = None):
        assert 1 <= len(weights) <= 4
        self.weights = [_chk(np.ascontiguousarray(w, dtype=np.float32), np.float32) for w in weights]
        self.biases: List[Optional[np.ndarray]] = [None] * len(weights)
        if biases is not None:
            self.biases = [None if b is None else np.ascontiguousarray(b, dtype=np.float32)
                           for b in biases]
        s = _Mlp()
        s.n_heads = self.weights[0].shape[0]
        s.n_layers = len(self.weights)
        for l, w in enumerate(self.weights):
            assert w.shape[0] == s.n_heads
            s.dims[l] = w.shape[1]
            s.dims[l + 1] = w.shape[2]
            if l > 0:
                assert w.shape[1] == self.weights[l - 1].shape[2]
            s.W[l] = w.ctypes.data
            s.bias[l] = _ptr(self.biases[l])
        assert s.dims[s.n_layers] % 32 == 0 and 32 <= s.dims[s.n_layers] <= 512
        self.c = s

    @property
    def n_heads(self) -> int:
        return int(self.c.n_heads)

    @property
    def in_dim(self) -> int:
        return int(self.c.dims[0])


class Cache:
    """KV cache + key-code store in host memory (arrays are referenced, not copied)."""

    def __init__(self, k: np.ndarray, v: np.ndarray, codes: np.ndarray, seq_lens: np.ndarray,
                 page_table: Optional[np.ndarray] = None, page_size: int = 0):
        self.k = _chk(k, np.uint16)
        self.v = _chk(v, np.uint16)
        self.codes = _chk(codes, np.uint32)
        self.seq_lens = _chk(seq_lens, np.int32)
        self.page_table = None if page_table is None else _chk(page_table, np.int32)
        assert k.ndim == 4 and k.shape == v.shape and codes.shape == k.shape[:3]
        s = _Cache()
        s.k, s.v, s.codes = k.ctypes.data, v.ctypes.data, codes.ctypes.data
        s.seq_lens = seq_lens.ctypes.data
        s.n_kv_heads, s.head_dim = k.shape[1], k.shape[3]
        if page_size > 0:
            assert page_table is not None and k.shape[2] == page_size
            s.page_table = page_table.ctypes.data
            s.max_pages_per_seq = page_table.shape[1]
            s.page_size = page_size
            s.n_max = page_table.shape[1] * page_size
        else:
            s.page_table = None
            s.max_pages_per_seq = 0
            s.page_size = 0
            s.n_max = k.shape[2]
        self.c = s

    @property
    def batch(self) -> int:
        return int(self.seq_lens.shape[0])


# ------------------------------------------------------------------ mapping
def encode_vec(mlp: Mlp, head: int, x_bf16: np.ndarray):
    """Code and pre-sign activations of one vector."""
    x = _chk(np.ascontiguousarray(x_bf16), np.uint16)
    assert x.shape == (mlp.in_dim,)
    act = np.zeros(32, dtype=np.float64)
    code = lib().ha_oracle_encode_vec(C.byref(mlp.c), head, x.ctypes.data, act.ctypes.data)
    return np.uint32(code), act


def encode_query(mlp: Mlp, q_bf16: np.ndarray):
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    B, H, d = q.shape
    assert H == mlp.n_heads and d == mlp.in_dim
    codes = np.zeros((B, H), dtype=np.uint32)
    act = np.zeros((B, H, 32), dtype=np.float64)
    lib().ha_oracle_encode_query(C.byref(mlp.c), q.ctypes.data, B, d, codes.ctypes.data, act.ctypes.data)
    return codes, act


def encode_keys(mlp: Mlp, cache: Cache, k_new: Optional[np.ndarray], v_new: Optional[np.ndarray],
                n_new: int, want_act: bool = False):
    """Append (k_new given, [B,Hkv,n_new,d]) or re-encode the last n_new cached rows in place."""
    B, H = cache.batch, int(cache.c.n_kv_heads)
    if k_new is not None:
        k_new = _chk(np.ascontiguousarray(k_new), np.uint16)
        v_new = _chk(np.ascontiguousarray(v_new), np.uint16)
        assert k_new.shape == (B, H, n_new, cache.c.head_dim) and v_new.shape == k_new.shape
    act = np.zeros((B, H, n_new, 32), dtype=np.float64) if want_act else None
    lib().ha_oracle_encode_keys(C.byref(mlp.c), C.byref(cache.c), _ptr(k_new), _ptr(v_new),
                                B, n_new, _ptr(act))
    return act


# ------------------------------------------------------------------ SCORE / TOPK
def score(q_code: int, k_code: int) -> int:
    return int(lib().ha_oracle_score(int(q_code), int(k_code)))


def scores(q_code: int, k_codes: np.ndarray) -> np.ndarray:
    kc = _chk(np.ascontiguousarray(k_codes), np.uint32)
    out = np.zeros(kc.shape[0], dtype=np.int32)
    lib().ha_oracle_scores(int(q_code), kc.ctypes.data, kc.shape[0], out.ctypes.data)
    return out


def _topk(fn, sc: np.ndarray, k: int):
    sc = _chk(np.ascontiguousarray(sc), np.int32)
    n = sc.shape[0]
    idx = np.zeros(max(min(k, n), 1), dtype=np.int32)
    thr = C.c_int32(0)
    cnt = fn(sc.ctypes.data, n, k, idx.ctypes.data, C.byref(thr))
    return idx[:cnt].copy(), int(thr.value)


def topk_sort(sc: np.ndarray, k: int):
    """Definition route: full sort by (score desc, index asc).  Returns (idx ascending, threshold)."""
    return _topk(lib().ha_oracle_topk_sort, sc, k)


def topk_hist(sc: np.ndarray, k: int):
    """Histogram-select route to the same set."""
    return _topk(lib().ha_oracle_topk_hist, sc, k)


def topk_window(sc: np.ndarray, k: int, n_sink: int, n_local: int):
    """TOPK with the first n_sink and last n_local tokens always kept; k counts only the tokens
    retrieved besides them.  Returns (idx ascending, threshold, number retrieved)."""
    sc = _chk(np.ascontiguousarray(sc), np.int32)
    n = sc.shape[0]
    idx = np.zeros(max(n, 1), dtype=np.int32)
    thr = C.c_int32(0)
    got = C.c_int64(0)
    cnt = lib().ha_oracle_topk_window(sc.ctypes.data, n, k, n_sink, n_local, idx.ctypes.data,
                                      C.byref(thr), C.byref(got))
    return idx[:cnt].copy(), int(thr.value), int(got.value)


# ------------------------------------------------------------------ attention
def gather_attend(cache: Cache, b: int, h_kv: int, q_bf16: np.ndarray, idx: np.ndarray,
                  scale: float) -> np.ndarray:
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    idx = _chk(np.ascontiguousarray(idx), np.int32)
    out = np.zeros(cache.c.head_dim, dtype=np.float64)
    lib().ha_oracle_gather_attend(C.byref(cache.c), b, h_kv, q.ctypes.data, idx.ctypes.data,
                                  idx.shape[0], float(scale), out.ctypes.data)
    return out


def dense_attend(cache: Cache, b: int, h_kv: int, q_bf16: np.ndarray, n: int, scale: float) -> np.ndarray:
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    out = np.zeros(cache.c.head_dim, dtype=np.float64)
    lib().ha_oracle_dense_attend(C.byref(cache.c), b, h_kv, q.ctypes.data, n, float(scale),
                                 out.ctypes.data)
    return out


# ------------------------------------------------------------------ quality of a SCORE function
def token_contributions(cache: Cache, b: int, h_kv: int, q_bf16: np.ndarray, n: int, scale: float) -> np.ndarray:
    """a_i * ||v_i||_2 of every token: its contribution to the dense output (section 4.2 lemma)."""
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    out = np.zeros(max(n, 1), dtype=np.float64)
    lib().ha_oracle_token_contributions(C.byref(cache.c), b, h_kv, q.ctypes.data, n, float(scale), out.ctypes.data)
    return out[:n]


def true_topk(cache: Cache, b: int, h_kv: int, q_bf16: np.ndarray, n: int, k: int, scale: float) -> np.ndarray:
    """I_true,k: the k tokens with the largest contribution, ascending."""
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    idx = np.zeros(max(min(k, n), 1), dtype=np.int32)
    cnt = lib().ha_oracle_true_topk(C.byref(cache.c), b, h_kv, q.ctypes.data, n, k, float(scale), idx.ctypes.data)
    return idx[:cnt].copy()


def recall(chosen: np.ndarray, truth: np.ndarray) -> float:
    """|chosen intersect truth| / |truth| (section 4)."""
    a = _chk(np.ascontiguousarray(chosen), np.int32)
    t = _chk(np.ascontiguousarray(truth), np.int32)
    return float(lib().ha_oracle_recall(a.ctypes.data, a.shape[0], t.ctypes.data, t.shape[0]))


# ------------------------------------------------------------------ whole step
def decode_step(phi_q: Optional[Mlp], phi_kv: Optional[Mlp], cache: Cache, q_bf16: np.ndarray,
                k_per_seq: np.ndarray, scale: float, k_new: Optional[np.ndarray] = None,
                v_new: Optional[np.ndarray] = None, q_codes: Optional[np.ndarray] = None,
                n_sink: int = 0, n_local: int = 0):
    """One layer decode step for every (sequence, query head).

    Returns dict(q_codes [B,Hq], idx [B,Hq,pitch], count [B,Hq], threshold [B,Hq], out [B,Hq,d] f64).
    With phi_q None the given q_codes are used.  k_new/v_new [B,Hkv,d] are appended first.
    n_sink / n_local > 0: the first / most recent tokens are always kept and k counts only the
    retrieved ones (pitch = k_max + n_sink + n_local); otherwise pitch = k_max.
    """
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    B, Hq, d = q.shape
    kps = _chk(np.ascontiguousarray(k_per_seq), np.int32)
    k_max = int(kps.max())
    if phi_q is None:
        qc = _chk(np.ascontiguousarray(q_codes).copy(), np.uint32)
    else:
        qc = np.zeros((B, Hq), dtype=np.uint32)
    if k_new is not None:
        k_new = _chk(np.ascontiguousarray(k_new), np.uint16)
        v_new = _chk(np.ascontiguousarray(v_new), np.uint16)
    window = n_sink > 0 or n_local > 0
    idx = np.full((B, Hq, k_max + n_sink + n_local), -1, dtype=np.int32)
    count = np.zeros((B, Hq), dtype=np.int32)
    thr = np.zeros((B, Hq), dtype=np.int32)
    out = np.zeros((B, Hq, d), dtype=np.float64)
    if window:
        lib().ha_oracle_decode_step_window(None if phi_q is None else C.addressof(phi_q.c),
                                           None if phi_kv is None else C.addressof(phi_kv.c),
                                           C.addressof(cache.c), q.ctypes.data, _ptr(k_new), _ptr(v_new),
                                           B, Hq, kps.ctypes.data, k_max, n_sink, n_local, float(scale),
                                           qc.ctypes.data, idx.ctypes.data, count.ctypes.data,
                                           thr.ctypes.data, out.ctypes.data)
        return dict(q_codes=qc, idx=idx, count=count, threshold=thr, out=out)
    lib().ha_oracle_decode_step(None if phi_q is None else C.addressof(phi_q.c),
                                None if phi_kv is None else C.addressof(phi_kv.c),
                                C.addressof(cache.c), q.ctypes.data, _ptr(k_new), _ptr(v_new),
                                B, Hq, kps.ctypes.data, k_max, float(scale), qc.ctypes.data,
                                idx.ctypes.data, count.ctypes.data, thr.ctypes.data, out.ctypes.data)
    return dict(q_codes=qc, idx=idx, count=count, threshold=thr, out=out)


# ------------------------------------------------------------------ wider signatures (words x 32 bits)
def encode_vec_wide(mlp: Mlp, head: int, x_bf16: np.ndarray, words: int):
    """Code words [words] and pre-sign activations [32 words] of one vector."""
    x = _chk(np.ascontiguousarray(x_bf16), np.uint16)
    code = np.zeros(words, dtype=np.uint32)
    act = np.zeros(32 * words, dtype=np.float64)
    lib().ha_oracle_encode_vec_wide(C.byref(mlp.c), head, x.ctypes.data, words, code.ctypes.data, act.ctypes.data)
    return code, act


def score_wide(q_code: np.ndarray, k_code: np.ndarray) -> int:
    q = _chk(np.ascontiguousarray(q_code), np.uint32)
    k = _chk(np.ascontiguousarray(k_code), np.uint32)
    assert q.shape == k.shape and q.ndim == 1
    return int(lib().ha_oracle_score_wide(q.ctypes.data, k.ctypes.data, q.shape[0]))


def scores_wide(q_code: np.ndarray, k_codes: np.ndarray) -> np.ndarray:
    """k_codes [n, words] -> similarities [n]."""
    q = _chk(np.ascontiguousarray(q_code), np.uint32)
    k = _chk(np.ascontiguousarray(k_codes), np.uint32)
    assert k.ndim == 2 and k.shape[1] == q.shape[0]
    out = np.zeros(k.shape[0], dtype=np.int32)
    lib().ha_oracle_scores_wide(q.ctypes.data, k.ctypes.data, k.shape[0], q.shape[0], out.ctypes.data)
    return out


def encode_query_wide(phi_q: Mlp, q_bf16: np.ndarray, words: int):
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    B, H, d = q.shape
    codes = np.zeros((B, H, words), dtype=np.uint32)
    act = np.zeros((B, H, 32 * words), dtype=np.float64)
    lib().ha_oracle_encode_query_wide(C.byref(phi_q.c), q.ctypes.data, B, d, words, codes.ctypes.data, act.ctypes.data)
    return codes, act


def encode_keys_wide(phi_kv: Mlp, cache: Cache, codes: np.ndarray, k_new, v_new, n_new: int, want_act: bool = False):
    """codes: uint32 array shaped like the key cache without d plus a trailing axis of words (updated in place)."""
    codes = _chk(codes, np.uint32)
    words = codes.shape[-1]
    act = None
    if want_act:
        act = np.zeros((cache.batch, cache.c.n_kv_heads, n_new, 32 * words), dtype=np.float64)
    if k_new is not None:
        k_new = _chk(np.ascontiguousarray(k_new), np.uint16)
        v_new = _chk(np.ascontiguousarray(v_new), np.uint16)
    lib().ha_oracle_encode_keys_wide(C.byref(phi_kv.c), C.byref(cache.c), codes.ctypes.data, words, _ptr(k_new),
                                     _ptr(v_new), cache.batch, n_new, _ptr(act))
    return act


def decode_step_wide(phi_q: Optional[Mlp], phi_kv: Optional[Mlp], cache: Cache, codes: np.ndarray, q_bf16: np.ndarray,
                     k_per_seq: np.ndarray, scale: float, k_new=None, v_new=None, q_codes=None,
                     n_sink: int = 0, n_local: int = 0):
    """decode_step with codes of words x 32 bits (codes: trailing axis words; q_codes [B,Hq,words])."""
    codes = _chk(codes, np.uint32)
    words = codes.shape[-1]
    q = _chk(np.ascontiguousarray(q_bf16), np.uint16)
    B, Hq, d = q.shape
    kps = _chk(np.ascontiguousarray(k_per_seq), np.int32)
    k_max = int(kps.max())
    qc = np.zeros((B, Hq, words), dtype=np.uint32) if phi_q is not None else _chk(np.ascontiguousarray(q_codes).copy(), np.uint32)
    if k_new is not None:
        k_new = _chk(np.ascontiguousarray(k_new), np.uint16)
        v_new = _chk(np.ascontiguousarray(v_new), np.uint16)
    idx = np.full((B, Hq, k_max + n_sink + n_local), -1, dtype=np.int32)
    count = np.zeros((B, Hq), dtype=np.int32)
    thr = np.zeros((B, Hq), dtype=np.int32)
    out = np.zeros((B, Hq, d), dtype=np.float64)
    lib().ha_oracle_decode_step_wide(None if phi_q is None else C.addressof(phi_q.c),
                                     None if phi_kv is None else C.addressof(phi_kv.c),
                                     C.addressof(cache.c), codes.ctypes.data, words, q.ctypes.data, _ptr(k_new), _ptr(v_new),
                                     B, Hq, kps.ctypes.data, k_max, n_sink, n_local, float(scale), qc.ctypes.data,
                                     idx.ctypes.data, count.ctypes.data, thr.ctypes.data, out.ctypes.data)
    return dict(q_codes=qc, idx=idx, count=count, threshold=thr, out=out)
