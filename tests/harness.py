"""Shared helpers of the GPU parity tests: upload seeded inputs, run the oracle beside the
HIP path, compare under the stated tolerances."""
from __future__ import annotations

import math

import numpy as np

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth

# tolerance of the attention output (fp32 result of the kernel against the fp64 oracle):
# |a - b| <= ABS_TOL + REL_TOL * |b|
ABS_TOL = 2e-3
REL_TOL = 1e-3
BAND = 1e-4  # projections closer to zero than this are excluded from bit-exact code comparison


def to_dev(a: np.ndarray):
    """numpy -> device tensor with the same bits (uint16 -> int16, uint32 -> int32)."""
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def to_host(t, dtype=None) -> np.ndarray:
    a = t.detach().cpu().numpy()
    if dtype is not None:
        a = a.view(dtype)
    return a


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in units of bf16 steps between two arrays of bf16 bit patterns."""
    def ordered(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(ordered(a_bits) - ordered(b_bits))


def check_attention(out_f32: np.ndarray, out_bf16_bits: np.ndarray, ref: np.ndarray, what=""):
    err = np.abs(out_f32.astype(np.float64) - ref)
    bound = ABS_TOL + REL_TOL * np.abs(ref)
    worst = float(np.max(err - bound))
    assert worst <= 0, f"{what}: fp32 output off by {float(err.max()):.3e} (max |ref| {float(np.abs(ref).max()):.3f})"
    # the bf16 output is the round-to-nearest-even of the kernel's own fp32 result (bit-exact) ...
    u = out_f32.view(np.uint32)
    rne = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(out_bf16_bits, rne), f"{what}: bf16 output is not RNE(fp32 output)"
    # ... and so lies within the tolerance plus one bf16 rounding (2^-8 relative) of the oracle
    val = (out_bf16_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(np.abs(val - ref) <= bound + 2.0 ** -8 * np.abs(ref)), f"{what}: bf16 output too far"
    return float(err.max()), float((err / np.maximum(np.abs(ref), 1e-30)).max())


def check_codes(got: np.ndarray, ref: np.ndarray, near: np.ndarray, what=""):
    """Bit-exact outside the near-zero band; returns (#bits in band, #bits that differ inside it)."""
    diff = got ^ ref
    outside = diff & ~near
    assert not np.any(outside), f"{what}: {int(np.count_nonzero(outside))} code words differ outside the band"
    in_band = int(sum(bin(int(v)).count("1") for v in near[near != 0]))
    flipped = int(sum(bin(int(v)).count("1") for v in diff[diff != 0]))
    return in_band, flipped


class Case:
    """One workload on the device, with its oracle-side twin on the host."""

    def __init__(self, w: synth.Workload, seed: int = synth.DEFAULT_SEED, oracle_codes: bool = True, **tuning):
        import torch
        from paper_2506_02572_amd import hata
        self.w = w
        self.inp = synth.generate(w, seed)
        self.scale = 1.0 / math.sqrt(w.d)
        self.ctx = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.L_cap, w.k_max, **tuning)
        self.K = to_dev(self.inp.K)
        self.V = to_dev(self.inp.V)
        self.W_H = to_dev(self.inp.W_H)
        self.seq_len = to_dev(self.inp.seq_len)
        self.k = to_dev(self.inp.k)
        self.zero = torch.zeros(w.B, dtype=torch.int32, device="cuda")
        if oracle_codes:
            self.codes_ref, self.near = O.encode_keys_batch(
                self.inp.K, self.inp.W_H, np.zeros(w.B, np.int32), self.inp.seq_len, bulk=True)
        self.torch = torch

    def empty(self, shape, dtype):
        return self.torch.empty(shape, dtype=dtype, device="cuda")

    def sync(self):
        self.torch.cuda.synchronize()
