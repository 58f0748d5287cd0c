"""What the bench advertises beyond the five configurations, at full size against the oracle: a
serving-size batch (B = 32 at L = 32K) in the sliced single-launch form and as one oversubscribed
grid, the KV cache in pinned host memory at the size of configuration 2, and a long run of
identical steps that must reproduce their first result bit for bit (the cross-workgroup hand-offs of
the single-launch step are exercised thousands of times in a row)."""
import math
import time

import numpy as np
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth
from tests import harness as H


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def test_batch_32_at_32k_in_slices_and_as_one_grid(torch_mod):
    torch = torch_mod
    w = synth.SWEEP["b32_32k"]
    t0 = time.time()
    c = H.Case(w, oracle_codes=True)
    print(f"[modes] b32_32k: oracle key codes after {time.time() - t0:.1f}s", flush=True)
    B = w.B
    q = c.inp.q(0)
    seq = c.inp.seq_len
    codes_h = c.codes_ref.copy()
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=True)
    print(f"[modes] b32_32k: oracle step after {time.time() - t0:.1f}s", flush=True)
    out = c.empty((B, w.Hq, w.d), torch.int16)
    out32 = c.empty((B, w.Hq, w.d), torch.float32)
    qd = H.to_dev(q)
    from paper_2506_02572_amd import hata
    # three forms of the same step: the library's own choice (a larger chunk, so that the whole batch
    # is one resident launch), one oversubscribed grid at the plan's chunk (mode 1), and -- on a second
    # context whose chunk is fixed at 4096 keys -- the batch in slices, one resident launch each
    ctx_sliced = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.L_cap, w.k_max, chunk=4096)
    for name, ctx, mode in (("own choice", c.ctx, 0), ("one oversubscribed grid", c.ctx, 1), ("slices", ctx_sliced, 0)):
        ctx.hata_set_step_mode(mode)
        n_sub = ctx.hata_step_sub_batches(B)
        n_launches, chunk, n_chunks = ctx.hata_step_plan(B)
        assert n_launches == 1, "the step is expected in its single-launch form"
        if name == "own choice":
            assert n_sub == 1 and chunk > 4096, "a batch of 32 at 32K is one resident launch at a larger chunk"
        elif name == "slices":
            assert n_sub >= 2 and chunk == 4096, "a batch of 32 at 32K does not fit one resident launch at 4096 keys"
        else:
            assert n_sub == 1
        codes_d = H.to_dev(c.codes_ref)
        out32.zero_()
        ctx.hata_decode_step(qd, c.K, c.V, c.W_H, codes_d, c.seq_len, c.k, B, True, c.scale, out, out32)
        ctx.hata_check()
        qc, _, ix = ctx.hata_step_buffers()
        assert np.array_equal(H.to_host(codes_d, np.uint32), codes_h), f"{name}: code cache"
        assert np.array_equal(H.to_host(qc, np.uint32), ref["qcodes"]), f"{name}: query codes"
        assert np.array_equal(H.to_host(ix), ref["idx"]), f"{name}: index lists"
        e = H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], name)
        print(f"[modes] b32_32k, {name}: {n_sub} launch(es), chunk {chunk} x {n_chunks}, idx exact, "
              f"attention max abs {e[0]:.2e}", flush=True)
    ctx_sliced.close()
    c.ctx.close()


def test_kv_cache_in_host_memory_at_config2_size(torch_mod):
    torch = torch_mod
    w = synth.config(2)
    c = H.Case(w, oracle_codes=True)
    Kh = torch.from_numpy(c.inp.K.view(np.int16)).pin_memory()
    Vh = torch.from_numpy(c.inp.V.view(np.int16)).pin_memory()
    q = c.inp.q(0)
    codes_h = c.codes_ref.copy()
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, c.inp.seq_len, c.inp.k, w.k_max, c.scale,
                        append=True)
    out = c.empty((w.B, w.Hq, w.d), torch.int16)
    out32 = c.empty((w.B, w.Hq, w.d), torch.float32)
    for mode in (0, 3):
        c.ctx.hata_set_step_mode(mode)
        codes_d = H.to_dev(c.codes_ref)
        out32.zero_()
        c.ctx.hata_decode_step(H.to_dev(q), Kh, Vh, c.W_H, codes_d, c.seq_len, c.k, w.B, True, c.scale, out, out32)
        c.ctx.hata_check()
        _, _, ix = c.ctx.hata_step_buffers()
        assert np.array_equal(H.to_host(codes_d, np.uint32), codes_h), "appended key code (key read from host memory)"
        assert np.array_equal(H.to_host(ix), ref["idx"])
        H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], f"host KV at cfg 2, mode {mode}")
    c.ctx.close()


@pytest.mark.parametrize("index", [3, 5])
def test_5000_identical_steps_reproduce_the_first(torch_mod, index):
    """5000 consecutive single-launch steps on fixed inputs: every step's index lists and fp32
    outputs must equal those of step 0 bit for bit (stopping at the first mismatch), and no wait
    may have given up.  Step 0 itself is checked against the oracle by the full-size tests."""
    torch = torch_mod
    w = synth.config(index)
    c = H.Case(w, oracle_codes=False)
    B = w.B
    seq = c.inp.seq_len + (1 if w.append_steps else 0)
    codes_d = torch.zeros((B, w.Hkv, w.L_cap, w.W), dtype=torch.int32, device="cuda")
    c.ctx.hata_encode_keys(c.K, c.W_H, c.zero, H.to_dev(seq), B, int(seq.max()), codes_d)
    qd, seqd = H.to_dev(c.inp.q(0)), H.to_dev(seq)
    assert c.ctx.hata_step_plan(B)[0] == 1
    RING = 50
    outs = c.empty((RING, B, w.Hq, w.d), torch.float32)
    out16 = c.empty((B, w.Hq, w.d), torch.int16)
    _, _, ix = c.ctx.hata_step_buffers()
    idxs = torch.empty((RING,) + tuple(ix.shape), dtype=torch.int32, device="cuda")
    calls = [c.ctx.prepared("hata_decode_step", qd, c.K, c.V, c.W_H, codes_d, seqd, c.k, B, True, c.scale, out16,
                            outs[j]) for j in range(RING)]
    calls[0]()
    c.sync()
    ref_out, ref_idx = outs[0].clone(), ix.clone()
    assert int((ref_idx >= 0).sum()) == int(np.minimum(c.inp.k, seq).sum()) * w.Hkv
    n_steps, done = 5000, 0
    t0 = time.time()
    while done < n_steps:
        for j in range(RING):
            calls[j]()
            idxs[j].copy_(ix)
        c.sync()
        same_out = (outs.view(torch.int32) == ref_out.view(torch.int32).unsqueeze(0)).flatten(1).all(dim=1)
        same_idx = (idxs == ref_idx.unsqueeze(0)).flatten(1).all(dim=1)
        bad = (~(same_out & same_idx)).nonzero()
        assert bad.numel() == 0, f"step {done + int(bad[0])} differs from step 0"
        done += RING
    c.ctx.hata_check()
    print(f"[modes] cfg {index}: {done} identical steps in {time.time() - t0:.1f}s, no wait gave up", flush=True)
    c.ctx.close()
