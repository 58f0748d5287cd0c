"""The allocation-free entry point hata_sparse_decode_static (scratch in the library's device image)
against hata_sparse_decode (scratch in the caller's workspace): same kernels and launch plan, so
the outputs must agree bit for bit -- on two calls in a row, the second with a smaller input that
leaves part of the scratch with the first call's contents."""
import ctypes

import numpy as np
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]

from oracle import hata_oracle as O
from paper_2506_02572_amd import hata, synth
from tests import harness as H


def run_pair(torch, w, seed):
    c = H.Case(w, seed=seed, oracle_codes=False)
    q = c.inp.q(0)
    rng = np.random.default_rng(seed)
    idx = np.full((w.B, w.Hkv, w.k_max), -1, np.int32)
    for b in range(w.B):
        kk = min(int(c.inp.k[b]), int(c.inp.seq_len[b]))
        for h in range(w.Hkv):
            idx[b, h, :kk] = np.sort(rng.choice(int(c.inp.seq_len[b]), size=kk, replace=False))
    ref = O.sparse_decode_batch(q, c.inp.K, c.inp.V, idx, c.scale)
    outs = []
    for static in (False, True):
        out = c.empty((w.B, w.Hq, w.d), torch.int16)
        out32 = c.empty((w.B, w.Hq, w.d), torch.float32)
        out.fill_(0x1234)
        out32.fill_(7.0)
        fn = c.ctx.hata_sparse_decode_static if static else c.ctx.hata_sparse_decode
        fn(H.to_dev(q), c.K, c.V, H.to_dev(idx), c.k, w.B, c.scale, out, out32)
        c.sync()
        outs.append((H.to_host(out32).copy(), H.to_host(out, np.uint16).copy()))
    e = H.check_attention(outs[1][0], outs[1][1], ref, "static scratch")
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32)), "fp32 outputs differ"
    assert np.array_equal(outs[0][1], outs[1][1]), "bf16 outputs differ"
    c.ctx.close()
    return e


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    # many slices per head (partials and counters in use), then a smaller shape right after it
    big = synth.Workload("noalloc_big", 3, 32, 8, 128, 128, (9000, 4097, 6000), (700, 512, 33), 4, 8.0, L_cap=9216,
                         k_max=768)
    small = synth.Workload("noalloc_small", 1, 8, 2, 128, 128, (1500,), (200,), 2, 8.0, L_cap=2048, k_max=256)
    e1 = run_pair(torch, big, 11)
    e2 = run_pair(torch, small, 12)
    print(f"[no-alloc] max abs err vs oracle: {e1[0]:.2e}, {e2[0]:.2e}")


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lib = hata.load_library()
    # 64 sequences x 64 heads x up to 256 slices x 520 B is far beyond 8 MiB
    cfg = hata.hata_config(64, 64, 8, 128, 128, 65536, 65536, 8 * 65536 * 128, 65536 * 128, 128)
    one = ctypes.c_void_p(256)
    rc = lib.hata_sparse_decode_static(ctypes.byref(cfg), one, one, one, one, one, 1, 1.0, one, None, None)
    assert rc == -6 and "scratch" in hata.strerror(rc)
