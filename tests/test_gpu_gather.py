"""hata_gather_rows (the Gather line of Alg. 3 materialised, for the offloading variant of
Sec. 5.3) through the C ABI: the staged rows are byte copies of the selected cache rows; attention
over the staged rows gives the bits of attention over the cache itself; a two-stream pipeline that
fetches the rows of the next layer while the current one attends gives the results of the plain
sequence of calls."""
import math

import numpy as np
import pytest

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def test_gather_rows_is_a_byte_copy_of_the_selected_rows(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    B, Hq, Hkv, d, L, k_max = 3, 8, 2, 128, 700, 200
    pitch = d + 8  # strided cache: padding after every row, poisoned with NaN patterns
    rng = np.random.default_rng(31)
    Kp = np.full((B, Hkv, L, pitch), 0x7FC1, np.uint16)
    Vp = np.full((B, Hkv, L, pitch), 0x7FC2, np.uint16)
    Kp[..., :d] = rng.integers(0, 0x7F00, (B, Hkv, L, d), dtype=np.uint16)
    Vp[..., :d] = rng.integers(0, 0x7F00, (B, Hkv, L, d), dtype=np.uint16)
    idx = np.full((B, Hkv, k_max), -1, np.int32)
    kbud = np.array([200, 137, 0], np.int32)  # full budget, ragged (137 = 2 * 64 + 9), empty
    for b in range(B):
        for h in range(Hkv):
            idx[b, h, :kbud[b]] = np.sort(rng.choice(L, kbud[b], replace=False))
    idx[0, 0, 5] = -1      # holes and out-of-range entries leave their staged rows untouched
    idx[0, 1, 17] = L
    idx[1, 0, 0] = -7
    idx[1, 1, 136] = 1 << 30
    ctx = hata.Context(B, Hq, Hkv, d, 128, L, k_max, kv_strides=(Hkv * L * pitch, L * pitch, pitch))
    for where in ("device", "pinned host"):
        if where == "device":
            Kd, Vd = H.to_dev(Kp), H.to_dev(Vp)
        else:
            Kd = torch.from_numpy(Kp.view(np.int16)).pin_memory()
            Vd = torch.from_numpy(Vp.view(np.int16)).pin_memory()
        Ks = torch.full((B, Hkv, k_max, d), 0x1111, dtype=torch.int16, device="cuda")
        Vs = torch.full((B, Hkv, k_max, d), 0x2222, dtype=torch.int16, device="cuda")
        # (device cache: a workgroup per block of rows; host cache: three workgroups share all blocks)
        ctx.hata_gather_rows(Kd, Vd, H.to_dev(idx), H.to_dev(kbud), B, 0 if where == "device" else 3, Ks, Vs)
        torch.cuda.synchronize()
        gk, gv = H.to_host(Ks, np.uint16), H.to_host(Vs, np.uint16)
        for b in range(B):
            for h in range(Hkv):
                for t in range(k_max):
                    n = int(idx[b, h, t])
                    if t < kbud[b] and 0 <= n < L:
                        assert np.array_equal(gk[b, h, t], Kp[b, h, n, :d]), (where, b, h, t)
                        assert np.array_equal(gv[b, h, t], Vp[b, h, n, :d]), (where, b, h, t)
                    else:
                        assert np.all(gk[b, h, t] == 0x1111) and np.all(gv[b, h, t] == 0x2222), (where, b, h, t)
    # a smaller batch than B_max touches only its own sequences
    Ks = torch.full((B, Hkv, k_max, d), 0x1111, dtype=torch.int16, device="cuda")
    Vs = torch.full((B, Hkv, k_max, d), 0x2222, dtype=torch.int16, device="cuda")
    ctx.hata_gather_rows(H.to_dev(Kp), H.to_dev(Vp), H.to_dev(idx), H.to_dev(kbud), 1, 0, Ks, Vs)
    torch.cuda.synchronize()
    assert np.all(H.to_host(Ks, np.uint16)[1:] == 0x1111)
    with pytest.raises(hata.HataError):
        ctx.hata_gather_rows(H.to_dev(Kp), H.to_dev(Vp), None, H.to_dev(kbud), B, 0, Ks, Vs)
    with pytest.raises(hata.HataError):
        ctx.hata_gather_rows(H.to_dev(Kp), H.to_dev(Vp), H.to_dev(idx), H.to_dev(kbud), B, -1, Ks, Vs)
    ctx.close()


def _staged_setup(torch, w, seed):
    from paper_2506_02572_amd import hata
    c = H.Case(w, seed=seed)
    q = c.inp.q(0)
    qcodes, _ = O.encode_query_batch(q, c.inp.W_H)
    sc = O.score_batch(qcodes, c.codes_ref, c.inp.seq_len)
    idx = O.topk_batch(sc, c.inp.seq_len, c.inp.k, w.k_max)
    ref = O.sparse_decode_batch(q, c.inp.K, c.inp.V, idx, c.scale)
    # attention over the staging buffer: a context whose "cache" has k_max rows, index list 0, 1, 2, ...
    stage_ctx = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.k_max, w.k_max)
    iota = torch.arange(w.k_max, dtype=torch.int32, device="cuda").repeat(w.B, w.Hkv, 1).contiguous()
    return c, q, idx, ref, stage_ctx, iota


def test_attention_over_staged_rows_has_the_bits_of_attention_over_the_cache(torch_mod):
    torch = torch_mod
    w = synth.Workload("stage", 2, 8, 2, 128, 128, (6000, 4500), (128, 96), 4, 8.0)
    c, q, idx, ref, stage_ctx, iota = _staged_setup(torch, w, 778)
    Kh = torch.from_numpy(c.inp.K.view(np.int16)).pin_memory()
    Vh = torch.from_numpy(c.inp.V.view(np.int16)).pin_memory()
    qd, idx_d = H.to_dev(q), H.to_dev(idx)
    out_a, out32_a = c.empty((w.B, w.Hq, w.d), torch.int16), c.empty((w.B, w.Hq, w.d), torch.float32)
    out_b, out32_b = torch.empty_like(out_a), torch.empty_like(out32_a)
    c.ctx.hata_sparse_decode(qd, Kh, Vh, idx_d, c.k, w.B, c.scale, out_a, out32_a)  # zero-copy over the bus
    Ks = torch.zeros((w.B, w.Hkv, w.k_max, w.d), dtype=torch.int16, device="cuda")
    Vs = torch.zeros_like(Ks)
    c.ctx.hata_gather_rows(Kh, Vh, idx_d, c.k, w.B, 32, Ks, Vs)
    stage_ctx.hata_sparse_decode(qd, Ks, Vs, iota, c.k, w.B, c.scale, out_b, out32_b)
    torch.cuda.synchronize()
    H.check_attention(H.to_host(out32_b), H.to_host(out_b, np.uint16), ref, "staged rows")
    assert torch.equal(out32_a, out32_b) and torch.equal(out_a, out_b)
    c.ctx.close()
    stage_ctx.close()


def test_select_step_writes_the_index_lists_of_the_whole_step(torch_mod):
    """hata_select_step against the oracle's step (appended key included), into a caller's buffer."""
    torch = torch_mod
    w = synth.Workload("sel", 3, 8, 2, 128, 128, (9000, 4100, 700), (192, 128, 64), 4, 8.0, append_steps=1)
    c = H.Case(w, seed=780)
    seq = c.inp.seq_len + 1
    codes_h = c.codes_ref.copy()
    for b in range(w.B):
        codes_h[b, :, int(seq[b]) - 1:] = 0xDEADBEEF
    codes_d = H.to_dev(codes_h)
    q = c.inp.q(1)
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=True)
    idx = torch.full((w.B, w.Hkv, w.k_max), 12345, dtype=torch.int32, device="cuda")
    for rep in range(2):
        c.ctx.hata_select_step(H.to_dev(q), c.K, c.W_H, codes_d, H.to_dev(seq), c.k, w.B, True, idx)
        c.ctx.hata_check()
        assert np.array_equal(H.to_host(idx), ref["idx"]), rep
        assert np.array_equal(H.to_host(codes_d, np.uint32), codes_h), "appended code row"
    # without an appended key K may be NULL; with one it may not
    from paper_2506_02572_amd import hata
    c.ctx.hata_select_step(H.to_dev(q), None, c.W_H, codes_d, H.to_dev(seq), c.k, w.B, False, idx)
    c.ctx.hata_check()
    assert np.array_equal(H.to_host(idx), ref["idx"])
    with pytest.raises(hata.HataError):
        c.ctx.hata_select_step(H.to_dev(q), None, c.W_H, codes_d, H.to_dev(seq), c.k, w.B, True, idx)
    c.ctx.close()


def test_two_stream_prefetch_pipeline_matches_the_oracle_steps(torch_mod):
    """The offloading pipeline: per layer, hata_select_step on the main stream, the fetch of the
    selected rows from pinned host memory on a second stream (default priority) into one of three
    staging buffers, attention over the staged rows on the main stream; the selection runs two
    layers ahead of the attention.  Events order select -> fetch -> attend; a staging buffer is
    re-used by a fetch that is enqueued behind a selection that is itself behind the attention
    that last read the buffer."""
    torch = torch_mod
    w = synth.Workload("pipe", 2, 8, 2, 128, 128, (5000, 3100), (128, 64), 4, 8.0)
    c, _, _, _, stage_ctx, iota = _staged_setup(torch, w, 779)
    NL, D = 7, 3
    Kh = torch.from_numpy(c.inp.K.view(np.int16)).pin_memory()
    Vh = torch.from_numpy(c.inp.V.view(np.int16)).pin_memory()
    codes_d = H.to_dev(c.codes_ref)
    qs, refs = [], []
    for l in range(NL):  # per layer another query over the same (host-resident) cache
        ql = c.inp.q(l)
        qs.append(H.to_dev(ql))
        refs.append(O.decode_step(ql, c.inp.K, c.inp.V, c.inp.W_H, c.codes_ref.copy(), c.inp.seq_len, c.inp.k,
                                  w.k_max, c.scale, append=False))
    Ks = [torch.zeros((w.B, w.Hkv, w.k_max, w.d), dtype=torch.int16, device="cuda") for _ in range(D)]
    Vs = [torch.zeros_like(Ks[0]) for _ in range(D)]
    idx = [torch.zeros((w.B, w.Hkv, w.k_max), dtype=torch.int32, device="cuda") for _ in range(D)]
    idx_seen = [torch.zeros_like(idx[0]) for _ in range(NL)]
    outs = [c.empty((w.B, w.Hq, w.d), torch.int16) for _ in range(NL)]
    outs32 = [c.empty((w.B, w.Hq, w.d), torch.float32) for _ in range(NL)]
    main, fetch = torch.cuda.current_stream(), torch.cuda.Stream()
    selected = [torch.cuda.Event() for _ in range(NL)]
    fetched = [torch.cuda.Event() for _ in range(NL)]
    torch.cuda.synchronize()

    def select_and_fetch(l):
        c.ctx.hata_select_step(qs[l], None, c.W_H, codes_d, c.seq_len, c.k, w.B, False, idx[l % D], stream=main)
        selected[l].record(main)
        fetch.wait_event(selected[l])
        c.ctx.hata_gather_rows(Kh, Vh, idx[l % D], c.k, w.B, 2, Ks[l % D], Vs[l % D], stream=fetch)
        idx_seen[l].copy_(idx[l % D])  # (on the main stream, behind the selection)
        fetched[l].record(fetch)

    for rep in range(2):  # twice: the second pass re-uses every buffer and event
        for l in range(min(D - 1, NL)):
            select_and_fetch(l)
        for l in range(NL):
            if l + D - 1 < NL:
                select_and_fetch(l + D - 1)
            main.wait_event(fetched[l])
            stage_ctx.hata_sparse_decode(qs[l], Ks[l % D], Vs[l % D], iota, c.k, w.B, c.scale, outs[l], outs32[l],
                                         stream=main)
        c.ctx.hata_check()
        for l in range(NL):
            assert np.array_equal(H.to_host(idx_seen[l]), refs[l]["idx"]), (rep, l)
            H.check_attention(H.to_host(outs32[l]), H.to_host(outs[l], np.uint16), refs[l]["out"], f"pipeline layer {l}")
            outs32[l].zero_()
    c.ctx.close()
    stage_ctx.close()
