"""numpy-facing wrapper of the CPU oracle (``hata_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this module.  It marshals numpy arrays to the plain-C oracle and adds nothing
to its arithmetic.  bf16 tensors are ``numpy.uint16`` bit patterns.

Function -> passage of the paper:
  hash_encode            Alg. 2 (HashEncode), h(x) = sign(x W_H)
  hamming_score          Alg. 3, S = bitcount(xor(Q_H, K_H^cache)), summed over a GQA group
  topk                   Alg. 3, Idx = TopK(S, N) (k smallest distances, lowest index on ties)
  attention_rows         Alg. 3 Gather + Attention; Eq. 2 third line; scale of Eq. 1
  *_batch / decode_step  the same over the [B, Hkv, L_cap, .] cache layout, Alg. 3 order
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hata_oracle.c")
_LIB = os.path.join(_HERE, "libhata_oracle.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None
_i64 = ctypes.c_int64
_p = ctypes.c_void_p
_dbl = ctypes.c_double


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_round_bf16.argtypes = [_p, _i64, _p]
        lib.oracle_hash_encode.argtypes = [_p, _i64, _i64, _i64, _p, _i64, _p, _p, _dbl, _p]
        lib.oracle_hamming_score.argtypes = [_p, _i64, _p, _i64, _i64, _p]
        lib.oracle_topk.restype = _i64
        lib.oracle_topk.argtypes = [_p, _i64, _i64, _p]
        lib.oracle_attention_rows.argtypes = [_p, _p, _p, _i64, _p, _i64, _i64, _dbl, _p]
        lib.oracle_encode_keys_batch.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _i64, _i64,
                                                 _p, _p, _dbl]
        lib.oracle_encode_keys_bulk.argtypes = lib.oracle_encode_keys_batch.argtypes
        lib.oracle_encode_query_batch.argtypes = [_p, _p, _i64, _i64, _i64, _i64, _i64,
                                                  _p, _p, _dbl]
        lib.oracle_score_batch.argtypes = [_p, _p, _p, _i64, _i64, _i64, _i64, _i64, _p]
        lib.oracle_topk_batch.argtypes = [_p, _p, _p, _i64, _i64, _i64, _i64, _p]
        lib.oracle_sparse_decode_batch.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _i64, _i64,
                                                   _i64, _dbl, _p]
        lib.oracle_dense_decode_batch.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _i64, _i64,
                                                  _dbl, _p]
        lib.oracle_decode_step.argtypes = [_p, _p, _p, _p, _p, _p, _p, ctypes.c_int,
                                           _i64, _i64, _i64, _i64, _i64, _i64, _i64, _dbl,
                                           _p, _p, _p, _p]
        for name in ("oracle_round_bf16", "oracle_hash_encode", "oracle_hamming_score",
                     "oracle_attention_rows", "oracle_encode_keys_batch",
                     "oracle_encode_keys_bulk", "oracle_encode_query_batch",
                     "oracle_score_batch", "oracle_topk_batch", "oracle_sparse_decode_batch",
                     "oracle_dense_decode_batch", "oracle_decode_step",
                     "oracle_set_num_threads"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 bit patterns, round to nearest even."""
    x = _c(x, np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().oracle_round_bf16(x.ctypes.data, x.size, out.ctypes.data)
    return out


def hash_encode(x: np.ndarray, W: np.ndarray, band: float = 1e-4, want_proj: bool = False):
    """x uint16 [n, d], W float32 [d, r] -> (codes u32 [n, r/32], near u32 [n, r/32][, proj f64 [n, r]])."""
    x = _c(x, np.uint16)
    W = _c(W, np.float32)
    n, d = x.shape
    d2, r = W.shape
    assert d == d2 and r % 32 == 0
    codes = np.empty((n, r // 32), dtype=np.uint32)
    near = np.empty((n, r // 32), dtype=np.uint32)
    proj = np.empty((n, r), dtype=np.float64) if want_proj else None
    _load().oracle_hash_encode(x.ctypes.data, n, d, d, W.ctypes.data, r, codes.ctypes.data,
                               near.ctypes.data, band, proj.ctypes.data if want_proj else None)
    return (codes, near, proj) if want_proj else (codes, near)


def hamming_score(qcodes: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """qcodes u32 [G, W], codes u32 [L, W] -> int32 [L] summed Hamming distances."""
    qcodes = _c(qcodes, np.uint32)
    codes = _c(codes, np.uint32)
    G, W = qcodes.shape
    L, W2 = codes.shape
    assert W == W2
    out = np.empty((L,), dtype=np.int32)
    _load().oracle_hamming_score(qcodes.ctypes.data, G, codes.ctypes.data, L, W, out.ctypes.data)
    return out


def topk(scores: np.ndarray, k: int) -> np.ndarray:
    """int32 [L] distances -> ascending indices of the min(k, L) smallest (score, index) pairs."""
    scores = _c(scores, np.int32)
    L = scores.shape[0]
    idx = np.empty((max(min(k, L), 0),), dtype=np.int32)
    cnt = _load().oracle_topk(scores.ctypes.data, L, k, idx.ctypes.data)
    assert cnt == idx.shape[0]
    return idx


def attention_rows(q: np.ndarray, K: np.ndarray, V: np.ndarray, idx, scale: float) -> np.ndarray:
    """q uint16 [d]; K, V uint16 [L, d]; idx int32 [count] or None (all rows) -> f64 [d]."""
    q = _c(q, np.uint16)
    K = _c(K, np.uint16)
    V = _c(V, np.uint16)
    L, d = K.shape
    out = np.empty((d,), dtype=np.float64)
    if idx is None:
        _load().oracle_attention_rows(q.ctypes.data, K.ctypes.data, V.ctypes.data, d, None, L, d,
                                      scale, out.ctypes.data)
    else:
        idx = _c(idx, np.int32)
        _load().oracle_attention_rows(q.ctypes.data, K.ctypes.data, V.ctypes.data, d,
                                      idx.ctypes.data, idx.shape[0], d, scale, out.ctypes.data)
    return out


# ---------------------------------------------------------------- batch drivers

def encode_keys_batch(K, W_H, start, n_new, codes=None, band=1e-4, bulk=False):
    """K uint16 [B,Hkv,L_cap,d]; W_H f32 [Hkv,d,r]; writes rows [start_b, start_b+n_new_b).
    Returns (codes u32 [B,Hkv,L_cap,r/32], near mask of the same shape)."""
    K = _c(K, np.uint16)
    W_H = _c(W_H, np.float32)
    B, Hkv, L_cap, d = K.shape
    r = W_H.shape[2]
    start = _c(start, np.int32)
    n_new = _c(n_new, np.int32)
    if codes is None:
        codes = np.zeros((B, Hkv, L_cap, r // 32), dtype=np.uint32)
    assert codes.flags.c_contiguous and codes.dtype == np.uint32
    near = np.zeros(codes.shape, dtype=np.uint32)
    fn = _load().oracle_encode_keys_bulk if bulk else _load().oracle_encode_keys_batch
    fn(K.ctypes.data, W_H.ctypes.data, start.ctypes.data, n_new.ctypes.data,
       B, Hkv, L_cap, d, r, codes.ctypes.data, near.ctypes.data, band)
    return codes, near


def encode_query_batch(q, W_H, band=1e-4):
    """q uint16 [B,Hq,d] -> (qcodes u32 [B,Hq,r/32], near mask)."""
    q = _c(q, np.uint16)
    W_H = _c(W_H, np.float32)
    B, Hq, d = q.shape
    Hkv, _, r = W_H.shape
    qcodes = np.empty((B, Hq, r // 32), dtype=np.uint32)
    near = np.empty((B, Hq, r // 32), dtype=np.uint32)
    _load().oracle_encode_query_batch(q.ctypes.data, W_H.ctypes.data, B, Hq, Hkv, d, r,
                                      qcodes.ctypes.data, near.ctypes.data, band)
    return qcodes, near


def score_batch(qcodes, codes, seq_len):
    """-> int32 [B,Hkv,L_cap]; rows >= seq_len[b] hold -1."""
    qcodes = _c(qcodes, np.uint32)
    codes = _c(codes, np.uint32)
    seq_len = _c(seq_len, np.int32)
    B, Hq, W = qcodes.shape
    _, Hkv, L_cap, _ = codes.shape
    scores = np.full((B, Hkv, L_cap), -1, dtype=np.int32)
    _load().oracle_score_batch(qcodes.ctypes.data, codes.ctypes.data, seq_len.ctypes.data,
                               B, Hq, Hkv, L_cap, W * 32, scores.ctypes.data)
    return scores


def topk_batch(scores, seq_len, k, k_max):
    """-> int32 [B,Hkv,k_max], ascending, padded with -1."""
    scores = _c(scores, np.int32)
    seq_len = _c(seq_len, np.int32)
    k = _c(k, np.int32)
    B, Hkv, L_cap = scores.shape
    idx = np.empty((B, Hkv, k_max), dtype=np.int32)
    _load().oracle_topk_batch(scores.ctypes.data, seq_len.ctypes.data, k.ctypes.data,
                              B, Hkv, L_cap, k_max, idx.ctypes.data)
    return idx


def sparse_decode_batch(q, K, V, idx, scale):
    """-> f64 [B,Hq,d]."""
    q = _c(q, np.uint16)
    K = _c(K, np.uint16)
    V = _c(V, np.uint16)
    idx = _c(idx, np.int32)
    B, Hq, d = q.shape
    _, Hkv, L_cap, _ = K.shape
    k_max = idx.shape[2]
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().oracle_sparse_decode_batch(q.ctypes.data, K.ctypes.data, V.ctypes.data,
                                       idx.ctypes.data, B, Hq, Hkv, L_cap, d, k_max, scale,
                                       out.ctypes.data)
    return out


def dense_decode_batch(q, K, V, seq_len, scale):
    """Eq. 1 over the whole cache -> f64 [B,Hq,d]."""
    q = _c(q, np.uint16)
    K = _c(K, np.uint16)
    V = _c(V, np.uint16)
    seq_len = _c(seq_len, np.int32)
    B, Hq, d = q.shape
    _, Hkv, L_cap, _ = K.shape
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().oracle_dense_decode_batch(q.ctypes.data, K.ctypes.data, V.ctypes.data,
                                      seq_len.ctypes.data, B, Hq, Hkv, L_cap, d, scale,
                                      out.ctypes.data)
    return out


def decode_step(q, K, V, W_H, codes, seq_len, k, k_max, scale, append=True):
    """One decode step in Alg. 3's order.  ``codes`` is updated in place when ``append``.
    Returns dict(qcodes, scores, idx, out)."""
    q = _c(q, np.uint16)
    K = _c(K, np.uint16)
    V = _c(V, np.uint16)
    W_H = _c(W_H, np.float32)
    seq_len = _c(seq_len, np.int32)
    k = _c(k, np.int32)
    assert codes.flags.c_contiguous and codes.dtype == np.uint32
    B, Hq, d = q.shape
    _, Hkv, L_cap, _ = K.shape
    r = W_H.shape[2]
    qcodes = np.empty((B, Hq, r // 32), dtype=np.uint32)
    scores = np.full((B, Hkv, L_cap), -1, dtype=np.int32)
    idx = np.empty((B, Hkv, k_max), dtype=np.int32)
    out = np.empty((B, Hq, d), dtype=np.float64)
    _load().oracle_decode_step(q.ctypes.data, K.ctypes.data, V.ctypes.data, W_H.ctypes.data,
                               codes.ctypes.data, seq_len.ctypes.data, k.ctypes.data,
                               1 if append else 0, B, Hq, Hkv, L_cap, d, r, k_max, scale,
                               qcodes.ctypes.data, scores.ctypes.data, idx.ctypes.data,
                               out.ctypes.data)
    return dict(qcodes=qcodes, scores=scores, idx=idx, out=out)
