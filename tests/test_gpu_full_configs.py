"""The five benchmark configurations at FULL size, in the launch configuration bench.py
times (a context of the same shape picks the same launch plan), against the oracle on the
same seeded inputs: bulk key encode, one decode step end to end (appended key code, query
codes, all Hamming scores, the index lists, attention), and for the appended-token
configuration a run of consecutive steps."""
import math
import time

import numpy as np
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(400)]

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth
from tests import harness as H


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def run_config(torch, index, steps_to_check):
    run_workload(torch, synth.config(index), steps_to_check, single_launch=True)


def run_workload(torch, w, steps_to_check, single_launch, dense=True):
    """Bulk key encode, decode steps in both launch forms and the dense baseline of workload `w`,
    each against the oracle.  single_launch: whether the step is expected to be one launch."""
    t_start = time.time()
    index = w.name
    print(f"[full] config {index}: {w.name} B={w.B} Hq={w.Hq} Hkv={w.Hkv} L_cap={w.L_cap} r={w.r} "
          f"k_max={w.k_max}", flush=True)
    c = H.Case(w, oracle_codes=False)
    inp = c.inp
    B = w.B
    # ---- bulk key encode of the prefill rows (the key-code fill of Alg. 1): GPU vs oracle, band counted
    prefill = inp.seq_len.copy()
    codes_ref, near = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(B, np.int32), prefill, bulk=True)
    print(f"[full]   oracle bulk encode done at {time.time() - t_start:.1f}s", flush=True)
    codes_d = torch.zeros((B, w.Hkv, w.L_cap, w.W), dtype=torch.int32, device="cuda")
    c.ctx.hata_encode_keys(c.K, c.W_H, c.zero, H.to_dev(prefill), B, int(prefill.max()), codes_d)
    c.sync()
    got = H.to_host(codes_d, np.uint32)
    diff = got ^ codes_ref
    assert not np.any(diff & ~near), "bulk-encoded key codes differ outside the |projection| < 1e-4 band"
    n_band = int(np.unpackbits(near.view(np.uint8)).sum())
    n_flip = int(np.unpackbits(diff.view(np.uint8)).sum())
    n_proj = int(prefill.sum()) * w.Hkv * w.r
    print(f"[full]   bulk encode: {n_proj} projections, {n_band} inside the band, {n_flip} bits differ there",
          flush=True)
    # the same with the weight planes prepared once (hata_prepare_weights): the key-code writer then
    # runs its fp16-plane form, whose bits may differ from the exact evaluation inside the band only
    if w.r in (32, 64, 128, 256):
        codes_p = torch.zeros_like(codes_d)
        c.ctx.hata_prepare_weights(c.W_H)
        c.ctx.hata_encode_keys(c.K, c.W_H, c.zero, H.to_dev(prefill), B, int(prefill.max()), codes_p)
        c.sync()
        diff_p = H.to_host(codes_p, np.uint32) ^ codes_ref
        assert not np.any(diff_p & ~near), "key codes from prepared weight planes differ outside the band"
        print(f"[full]   bulk encode, prepared planes: {int(np.unpackbits(diff_p.view(np.uint8)).sum())} bits "
              f"differ inside the band", flush=True)
        del diff_p
        # a different tensor at another address must not pick up the prepared planes
        W2 = (c.W_H.view(torch.float32) * 1.0).clone().view(c.W_H.dtype)
        codes_p.zero_()
        c.ctx.hata_encode_keys(c.K, W2, c.zero, H.to_dev(prefill), B, int(prefill.max()), codes_p)
        c.sync()
        assert torch.equal(codes_p, codes_d)
        del codes_p, W2
    # ---- decode steps on the ORACLE's codes (so every later stage is comparable bit for bit)
    codes_h = codes_ref.copy()
    codes_d = H.to_dev(codes_h)
    out = c.empty((B, w.Hq, w.d), torch.int16)
    out32 = c.empty((B, w.Hq, w.d), torch.float32)
    n_steps = max(1, w.append_steps)
    c.ctx.hata_keep_step_scores(True)  # the score array is inspected below
    n_launches, chunk, n_chunks = c.ctx.hata_step_plan(B)
    print(f"[full]   step plan: {n_launches} launch(es), chunk {chunk}, {n_chunks} chunks per unit", flush=True)
    assert n_launches == (1 if single_launch else 3), "unexpected launch form of the decode step"
    for t in range(n_steps):
        seq = inp.seq_len + (t + 1 if w.append_steps else 0)
        append = bool(w.append_steps)
        q = inp.q(t)
        c.ctx.hata_decode_step(H.to_dev(q), c.K, c.V, c.W_H, codes_d, H.to_dev(seq), c.k, B, append,
                               c.scale, out, out32)
        c.ctx.hata_check()
        if t not in steps_to_check:
            # keep the host copy of the code cache in step with the device (oracle-encoded row)
            if append:
                O.encode_keys_batch(inp.K, inp.W_H, (seq - 1).astype(np.int32), np.ones(B, np.int32),
                                    codes=codes_h)
            continue
        ref = O.decode_step(q, inp.K, inp.V, inp.W_H, codes_h, seq, inp.k, w.k_max, c.scale, append=append)
        qc, sc, ix = c.ctx.hata_step_buffers()
        if append:
            rows = np.stack([H.to_host(codes_d[b, :, int(seq[b]) - 1], np.uint32) for b in range(B)])
            want = np.stack([codes_h[b, :, int(seq[b]) - 1] for b in range(B)])
            assert np.array_equal(rows, want), f"step {t}: appended key code"
        assert np.array_equal(H.to_host(qc, np.uint32), ref["qcodes"]), f"step {t}: query codes"
        got_s = H.to_host(sc, np.uint16).astype(np.int32)
        for b in range(B):
            L = int(seq[b])
            assert np.array_equal(got_s[b, :, :L], ref["scores"][b, :, :L]), f"step {t}: scores b={b}"
        assert np.array_equal(H.to_host(ix), ref["idx"]), f"step {t}: index lists"
        e = H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], f"step {t}")
        print(f"[full]   step {t}: codes/scores/idx exact; attention max abs {e[0]:.2e} max rel {e[1]:.2e} "
              f"({time.time() - t_start:.1f}s)", flush=True)
        # the same step in its three-launch form (re-appending the same row is idempotent)
        c.ctx.hata_set_step_mode(3)
        assert c.ctx.hata_step_plan(B)[0] == 3
        out.zero_(); out32.zero_(); ix.fill_(-7)
        c.ctx.hata_decode_step(H.to_dev(q), c.K, c.V, c.W_H, codes_d, H.to_dev(seq), c.k, B, append,
                               c.scale, out, out32)
        c.ctx.hata_check()
        c.ctx.hata_set_step_mode(0)
        assert np.array_equal(H.to_host(ix), ref["idx"]), f"step {t}: index lists (three launches)"
        H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], f"step {t} (three launches)")
    if w.append_steps:
        assert np.array_equal(H.to_host(codes_d, np.uint32)[:, :, :w.L_cap], codes_h), "code cache after the run"
    if not dense:
        c.ctx.close()
        return
    # ---- dense baseline over the whole cache at the same shape (Eq. 1)
    seq = inp.seq_len
    q = inp.q(0)
    ref_d = O.dense_decode_batch(q, inp.K, inp.V, seq, c.scale)
    c.ctx.hata_dense_decode(H.to_dev(q), c.K, c.V, c.seq_len, B, c.scale, out, out32)
    c.sync()
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref_d, "dense")
    c.ctx.close()
    print(f"[full]   config {index} done in {time.time() - t_start:.1f}s", flush=True)


def test_config1_tiny(torch_mod):
    run_config(torch_mod, 1, {0})


def test_config2_llama3_8b_32k(torch_mod):
    run_config(torch_mod, 2, {0})


def test_config3_batched_ragged(torch_mod):
    run_config(torch_mod, 3, {0})


def test_config4_long_128k_r256(torch_mod):
    run_config(torch_mod, 4, {0})


def test_config5_gqa8_append_64_steps(torch_mod):
    # every one of the 64 steps is compared with the oracle (appended code row, query codes, scores,
    # index lists, attention; both launch forms), and the whole code cache once more at the end
    run_config(torch_mod, 5, set(range(64)))
