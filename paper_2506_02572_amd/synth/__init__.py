"""Seeded synthetic inputs shaped like the paper's decode workloads.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It contains none of the method's arithmetic: it only draws
reproducible pseudo-random tensors (see ``synth.c``) and describes workload
shapes.  bf16 tensors are returned as ``numpy.uint16`` bit patterns.

Shapes follow the model table of the paper's appendix (32 query / 8 KV heads
or 64 / 8, head_dim 128) and the (context length, token budget) pairs of its
RULER and efficiency sections (32K..128K tokens, about 1.56 %..3.13 % budget).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "synth.c")
_LIB = os.path.join(_HERE, "libhata_synth.so")

DEFAULT_SEED = 20250602

# tensor ids of the independent random streams
TID_Q = 1          # + step index * 16
TID_K = 2
TID_V = 3
TID_WH = 4
TID_LEN = 5
TID_OUTLIER = 6
TID_CODES = 7
TID_MISC = 8


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u64 = ctypes.c_uint64
        lib.synth_u64.restype = u64
        lib.synth_u64.argtypes = [u64, u64, u64]
        lib.synth_normal.restype = ctypes.c_double
        lib.synth_normal.argtypes = [u64, u64, u64]
        lib.synth_fill_bf16.restype = None
        lib.synth_fill_bf16.argtypes = [u64, u64, u64, u64, u64, u64, u64,
                                        ctypes.c_void_p, ctypes.c_void_p]
        lib.synth_fill_f32.restype = None
        lib.synth_fill_f32.argtypes = [u64, u64, u64, u64, ctypes.c_double, ctypes.c_void_p]
        lib.synth_fill_u32.restype = None
        lib.synth_fill_u32.argtypes = [u64, u64, u64, u64, ctypes.c_void_p]
        _lib = lib
    return _lib


def u64(seed: int, tensor_id: int, idx: int) -> int:
    return int(_load().synth_u64(seed, tensor_id, idx))


def normal(seed: int, tensor_id: int, idx: int) -> float:
    return float(_load().synth_normal(seed, tensor_id, idx))


def fill_bf16(seed: int, tensor_id: int, shape, chan_scale: Optional[np.ndarray] = None,
              first: int = 0) -> np.ndarray:
    """bf16 normal tensor of layout [..., heads, rows, d]; optional per-(head, channel) scale."""
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.uint16)
    d = shape[-1]
    rows = shape[-2] if len(shape) >= 2 else 1
    heads = shape[-3] if len(shape) >= 3 else 1
    sc_ptr = None
    if chan_scale is not None:
        chan_scale = np.ascontiguousarray(chan_scale, dtype=np.float32)
        assert chan_scale.shape == (heads, d), (chan_scale.shape, heads, d)
        sc_ptr = chan_scale.ctypes.data
    _load().synth_fill_bf16(seed, tensor_id, first, out.size, d, rows, heads, sc_ptr,
                            out.ctypes.data)
    return out


def fill_f32(seed: int, tensor_id: int, shape, sigma: float, first: int = 0) -> np.ndarray:
    out = np.empty(tuple(int(s) for s in shape), dtype=np.float32)
    _load().synth_fill_f32(seed, tensor_id, first, out.size, float(sigma), out.ctypes.data)
    return out


def fill_u32(seed: int, tensor_id: int, shape, first: int = 0) -> np.ndarray:
    out = np.empty(tuple(int(s) for s in shape), dtype=np.uint32)
    _load().synth_fill_u32(seed, tensor_id, first, out.size, out.ctypes.data)
    return out


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32 (for harness use)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


@dataclass(frozen=True)
class Workload:
    """Shape of one decode-attention workload.  ``L`` and ``k`` are per sequence."""
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    r: int
    L: tuple            # cached length per sequence, including this step's token
    k: tuple            # token budget per sequence
    n_outlier: int = 0  # outlier channels per KV head
    outlier_scale: float = 1.0
    append_steps: int = 0   # extra decode steps that each append one key (L grows by one)
    L_cap: int = 0      # rows allocated per (sequence, KV head); 0 -> max(L) + append_steps
    k_max: int = 0      # 0 -> max(k)

    def __post_init__(self):
        assert len(self.L) == self.B and len(self.k) == self.B
        assert self.Hq % self.Hkv == 0 and self.r % 32 == 0
        if self.L_cap == 0:
            object.__setattr__(self, "L_cap", max(self.L) + self.append_steps)
        if self.k_max == 0:
            object.__setattr__(self, "k_max", max(self.k))

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def W(self) -> int:
        return self.r // 32

    def algorithmic_bytes(self, step: int = 0) -> int:
        """Bytes the method itself must move per decode step: packed codes of every
        cached key + K and V rows of every selected key + q in and out."""
        code = sum((l + step) for l in self.L) * self.Hkv * (self.r // 8)
        rows = sum(min(kk, l + step) for kk, l in zip(self.k, self.L)) * self.Hkv * 2 * self.d * 2
        qo = self.B * self.Hq * self.d * 2 * 2
        return code + rows + qo

    def dense_bytes(self, step: int = 0) -> int:
        return sum((l + step) for l in self.L) * self.Hkv * 2 * self.d * 2 + \
            self.B * self.Hq * self.d * 2 * 2


def budget_2pct(L: int) -> int:
    """Token budget of 2 % of L rounded to the nearest multiple of 64 (at least 64)."""
    return max(64, 64 * int((0.02 * L) / 64 + 0.5))


def config(index: int, seed: int = DEFAULT_SEED) -> Workload:
    """The five benchmark configurations (index 1..5)."""
    if index == 1:
        return Workload("cfg1_tiny", 1, 32, 8, 128, 128, (2048,), (128,), 4, 8.0)
    if index == 2:
        return Workload("cfg2_llama3_8b_32k", 1, 32, 8, 128, 128, (32768,), (512,), 4, 8.0)
    if index == 3:
        B = 16
        L = tuple(8192 + u64(seed, TID_LEN, b) % (32768 - 8192 + 1) for b in range(B))
        k = tuple(budget_2pct(l) for l in L)
        return Workload("cfg3_batched_ragged", B, 32, 8, 128, 128, L, k, 4, 8.0, L_cap=32768)
    if index == 4:
        return Workload("cfg4_long_128k_r256", 1, 32, 8, 128, 256, (131072,), (2048,), 8, 16.0)
    if index == 5:
        return Workload("cfg5_gqa8_append", 4, 64, 8, 128, 128, (65536,) * 4, (1024,) * 4,
                        0, 1.0, append_steps=64)
    raise ValueError("config index must be 1..5")


# Shape sweep with the same kernels: the axes of the paper's efficiency figure and ablations
# (model table: Llama-2 without grouping, Qwen-2.5 with 40 query / 8 KV heads; hash-bit ablation;
# token budgets 0.4 % .. 3.13 %; contexts up to 256K).
SWEEP = {
    "mha32_32k": Workload("mha32_32k", 1, 32, 32, 128, 128, (32768,), (512,), 4, 8.0),
    "g5_40q8kv_32k": Workload("g5_40q8kv_32k", 2, 40, 8, 128, 128, (32768, 20000), (512, 320), 4, 8.0),
    "g16_128q8kv_32k": Workload("g16_128q8kv_32k", 1, 128, 8, 128, 128, (32768,), (512,), 4, 8.0),
    "r64_32k": Workload("r64_32k", 1, 32, 8, 128, 64, (32768,), (512,), 4, 8.0),
    "r32_32k": Workload("r32_32k", 1, 32, 8, 128, 32, (32768,), (512,), 4, 8.0),
    "r256_g8_ragged": Workload("r256_g8_ragged", 2, 64, 8, 128, 256, (24000, 9000), (384, 128), 8, 16.0),
    "budget0p4_32k": Workload("budget0p4_32k", 1, 32, 8, 128, 128, (32768,), (128,), 4, 8.0),
    "budget3p13_32k": Workload("budget3p13_32k", 1, 32, 8, 128, 128, (32768,), (1024,), 4, 8.0),
    "ctx256k": Workload("ctx256k", 1, 32, 8, 128, 128, (262144,), (4096,), 4, 8.0, append_steps=2),
    # the shape the paper's headline ratio is quoted on (Sec. 5.3: batch 8 at 32K tokens, budget 1.56 %)
    "b8_32k": Workload("b8_32k", 8, 32, 8, 128, 128, (32768,) * 8, (512,) * 8, 4, 8.0),
    # a serving-size batch: more (sequence, KV head) units than one launch can keep resident
    "b32_32k": Workload("b32_32k", 32, 32, 8, 128, 128, (32768,) * 32, (512,) * 32, 4, 8.0),
    "b64_32k": Workload("b64_32k", 64, 32, 8, 128, 128, (32768,) * 64, (512,) * 64, 4, 8.0),
}


def workload(name: str) -> Workload:
    """cfg1 .. cfg5 (the benchmark configurations) or a name in SWEEP."""
    if name in SWEEP:
        return SWEEP[name]
    if name.startswith("cfg") and name[3:].isdigit():
        return config(int(name[3:]))
    raise ValueError(f"unknown workload {name!r}")


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def train_vectors(n: int, d: int = 128, latent: int = 8, seed: int = DEFAULT_SEED, tensor_id: int = TID_MISC):
    """Structured stand-in for the q / k vectors of one attention head (the paper samples them from
    real prefills): a few latent directions carry most of the variance, the rest is noise.
    Returns bf16 bit patterns [n, d]; the mixing matrix depends on `seed` only, so queries and keys
    drawn with different tensor ids share it."""
    mix = fill_f32(seed, TID_MISC + 64, (latent, d), 1.0)
    z = fill_f32(seed, tensor_id + 32, (n, latent), 1.0)
    noise = fill_f32(seed, tensor_id + 48, (n, d), 1.0)
    x = (2.0 / np.sqrt(latent)) * (z @ mix) + 0.5 * noise
    return round_to_bf16_bits(x.astype(np.float32))


def massive_direction_vectors(n_keys: int, n_queries: int, d: int = 128, signal: int = 64, massive: int = 4,
                              massive_scale: float = 20.0, noise: float = 0.1, query_scale: float = 4.0,
                              seed: int = DEFAULT_SEED):
    """Stand-in for the q / k vectors of a head whose keys carry a few directions of very large
    magnitude that the queries ignore (LLM keys show such massive, query-irrelevant components; here
    they are rotated away from the channel axes).  In a seeded orthonormal basis, keys have unit
    variance on `signal` directions, `massive_scale` on `massive` further ones and `noise`
    everywhere; queries live on the signal directions (plus the noise) and are scaled to a norm like
    the keys'.  Returns bf16 bit patterns (K [n_keys, d], Q [n_queries, d])."""
    basis, _ = np.linalg.qr(fill_f32(seed, TID_MISC + 80, (d, d), 1.0).astype(np.float64))
    S, M = basis[:, :signal], basis[:, signal:signal + massive]
    zk = fill_f32(seed, TID_K + 96, (n_keys, signal), 1.0).astype(np.float64)
    mk = fill_f32(seed, TID_K + 112, (n_keys, massive), massive_scale).astype(np.float64)
    K = zk @ S.T + mk @ M.T + fill_f32(seed, TID_K + 128, (n_keys, d), noise)
    zq = fill_f32(seed, TID_Q + 96, (n_queries, signal), 1.0).astype(np.float64)
    Q = query_scale * (zq @ S.T + fill_f32(seed, TID_Q + 128, (n_queries, d), noise))
    return round_to_bf16_bits(K.astype(np.float32)), round_to_bf16_bits(Q.astype(np.float32))


def outlier_scales(w: Workload, seed: int) -> np.ndarray:
    """Per-(KV head, channel) scale: ``n_outlier`` distinct channels per head get
    ``outlier_scale``; drawn with a partial Fisher-Yates shuffle of the channel ids."""
    sc = np.ones((w.Hkv, w.d), dtype=np.float32)
    for h in range(w.Hkv):
        ids = list(range(w.d))
        for j in range(w.n_outlier):
            t = j + u64(seed, TID_OUTLIER, h * w.d + j) % (w.d - j)
            ids[j], ids[t] = ids[t], ids[j]
            sc[h, ids[j]] = w.outlier_scale
    return sc


@dataclass
class Inputs:
    w: Workload
    seed: int
    K: np.ndarray        # uint16 [B, Hkv, L_cap, d]
    V: np.ndarray        # uint16 [B, Hkv, L_cap, d]
    W_H: np.ndarray      # float32 [Hkv, d, r]
    seq_len: np.ndarray  # int32 [B]
    k: np.ndarray        # int32 [B]
    chan_scale: np.ndarray  # float32 [Hkv, d]

    def q(self, step: int = 0) -> np.ndarray:
        """Query of decode step ``step``: uint16 [B, Hq, d]; the outlier channels of a
        KV head are scaled in the queries of its whole group as well."""
        w = self.w
        sc_q = np.repeat(self.chan_scale, w.G, axis=0)  # [Hq, d]
        flat = fill_bf16(self.seed, TID_Q + 16 * step, (w.B, w.Hq, 1, w.d), sc_q)
        return flat.reshape(w.B, w.Hq, w.d)


def generate(w: Workload, seed: int = DEFAULT_SEED) -> Inputs:
    """Draw K, V (all L_cap rows, so appended rows exist already), W_H and the
    per-sequence length / budget arrays of a workload."""
    sc = outlier_scales(w, seed)
    K = fill_bf16(seed, TID_K, (w.B, w.Hkv, w.L_cap, w.d), sc)
    V = fill_bf16(seed, TID_V, (w.B, w.Hkv, w.L_cap, w.d), sc)
    W_H = fill_f32(seed, TID_WH, (w.Hkv, w.d, w.r), 128.0 ** -0.5)
    return Inputs(w, seed, K, V, W_H,
                  np.asarray(w.L, dtype=np.int32), np.asarray(w.k, dtype=np.int32), sc)


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (L_cap / k_max re-derived)."""
    kw.setdefault("L_cap", 0)
    kw.setdefault("k_max", 0)
    return replace(w, **kw)
