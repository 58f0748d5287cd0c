"""GPU-vs-oracle parity, stage by stage and end to end, through the C ABI.

Bar: bit-exact for hash codes (outside the |projection| < 1e-4 band, which is counted),
Hamming scores and top-k index lists; |a-b| <= 2e-3 + 1e-3 |b| for the fp32 attention
output and at most one bf16 step for the bf16 output.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth
from tests import harness as H

W = synth.Workload
SMALL = {
    "g4_r128_ragged": W("g4_r128_ragged", 2, 8, 2, 128, 128, (5000, 3001), (100, 333), 4, 8.0, L_cap=5120),
    "g8_r128": W("g8_r128", 2, 16, 2, 128, 128, (2500, 4100), (64, 200), 0, 1.0),
    "g4_r256_outl16": W("g4_r256_outl16", 1, 8, 2, 128, 256, (4500,), (250,), 8, 16.0),
    "mha_r128": W("mha_r128", 1, 4, 4, 128, 128, (3000,), (96,), 4, 8.0),
    "g5_r64": W("g5_r64", 1, 10, 2, 128, 64, (2100,), (50,), 0, 1.0),
    "g3_r96_generic": W("g3_r96_generic", 1, 6, 2, 128, 96, (1500,), (33,), 0, 1.0),
    "g16_r32": W("g16_r32", 1, 16, 1, 128, 32, (1100,), (40,), 0, 1.0),
}


@pytest.fixture(scope="module", params=list(SMALL.keys()))
def case(request):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    print(f"[case] {request.param}", flush=True)
    c = H.Case(SMALL[request.param], seed=1234)
    yield c
    c.ctx.close()


def test_encode_query(case):
    import torch
    w = case.w
    q = case.inp.q(0)
    qcodes = case.empty((w.B, w.Hq, w.W), torch.int32)
    case.ctx.hata_encode_query(H.to_dev(q), case.W_H, w.B, qcodes)
    case.sync()
    ref, near = O.encode_query_batch(q, case.inp.W_H, band=H.BAND)
    H.check_codes(H.to_host(qcodes, np.uint32), ref, near, "encode_query")
    # fp64 accumulation: identical even inside the band
    assert np.array_equal(H.to_host(qcodes, np.uint32), ref)


def test_encode_keys_bulk(case):
    import torch
    w = case.w
    codes = torch.full((w.B, w.Hkv, w.L_cap, w.W), -1, dtype=torch.int32, device="cuda")
    case.ctx.hata_encode_keys(case.K, case.W_H, case.zero, case.seq_len, w.B, w.L_cap, codes)
    case.sync()
    got = H.to_host(codes, np.uint32)
    for b in range(w.B):
        L = int(case.inp.seq_len[b])
        in_band, flipped = H.check_codes(got[b, :, :L], case.codes_ref[b, :, :L], case.near[b, :, :L],
                                         f"encode_keys bulk b={b}")
        print(f"  bulk encode b={b}: {in_band} projections in the band, {flipped} bits differ inside it")
        assert np.all(got[b, :, L:] == 0xFFFFFFFF), "rows past the range were written"


def test_encode_keys_partial_range_and_append(case):
    import torch
    w = case.w
    # a sub-range [start, start + n) in bulk mode, then single appended rows
    codes = torch.full((w.B, w.Hkv, w.L_cap, w.W), -1, dtype=torch.int32, device="cuda")
    start = np.array([7 + 3 * b for b in range(w.B)], np.int32)
    n_new = np.array([min(int(case.inp.seq_len[b]) - int(start[b]), 777 + b) for b in range(w.B)], np.int32)
    case.ctx.hata_encode_keys(case.K, case.W_H, H.to_dev(start), H.to_dev(n_new), w.B,
                              int(n_new.max()), codes)
    case.sync()
    got = H.to_host(codes, np.uint32)
    for b in range(w.B):
        s, n = int(start[b]), int(n_new[b])
        H.check_codes(got[b, :, s:s + n], case.codes_ref[b, :, s:s + n], case.near[b, :, s:s + n], "range")
        assert np.all(got[b, :, :s] == 0xFFFFFFFF) and np.all(got[b, :, s + n:] == 0xFFFFFFFF)
    # append: one row per sequence at seq_len - 1 (fp64 path: exact)
    codes.fill_(-1)
    last = (case.inp.seq_len - 1).astype(np.int32)
    ones = np.ones(w.B, np.int32)
    case.ctx.hata_encode_keys(case.K, case.W_H, H.to_dev(last), H.to_dev(ones), w.B, 1, codes)
    case.sync()
    got = H.to_host(codes, np.uint32)
    for b in range(w.B):
        n = int(last[b])
        assert np.array_equal(got[b, :, n], case.codes_ref[b, :, n])
        assert np.all(got[b, :, :n] == 0xFFFFFFFF) and np.all(got[b, :, n + 1:] == 0xFFFFFFFF)


def test_hamming_score(case):
    import torch
    w = case.w
    qcodes, _ = O.encode_query_batch(case.inp.q(0), case.inp.W_H)
    ref = O.score_batch(qcodes, case.codes_ref, case.inp.seq_len)
    scores = torch.full((w.B, w.Hkv, w.L_cap), -1, dtype=torch.int16, device="cuda")
    case.ctx.hata_hamming_score(H.to_dev(qcodes), H.to_dev(case.codes_ref), case.seq_len, w.B, scores)
    case.sync()
    got = H.to_host(scores, np.uint16).astype(np.int32)
    for b in range(w.B):
        L = int(case.inp.seq_len[b])
        assert np.array_equal(got[b, :, :L], ref[b, :, :L])
        assert np.all(got[b, :, L:] == 0xFFFF), "scores past seq_len were written"


def test_topk(case):
    import torch
    w = case.w
    qcodes, _ = O.encode_query_batch(case.inp.q(0), case.inp.W_H)
    sc = O.score_batch(qcodes, case.codes_ref, case.inp.seq_len)
    ref = O.topk_batch(sc, case.inp.seq_len, case.inp.k, w.k_max)
    dev_scores = H.to_dev(np.where(sc < 0, 0xFFFF, sc).astype(np.uint16))
    idx = torch.full((w.B, w.Hkv, w.k_max), -7, dtype=torch.int32, device="cuda")
    case.ctx.hata_topk(dev_scores, case.seq_len, case.k, w.B, idx)
    case.sync()
    assert np.array_equal(H.to_host(idx), ref)


def test_sparse_and_dense_decode(case):
    import torch
    w = case.w
    q = case.inp.q(0)
    qcodes, _ = O.encode_query_batch(q, case.inp.W_H)
    sc = O.score_batch(qcodes, case.codes_ref, case.inp.seq_len)
    idx = O.topk_batch(sc, case.inp.seq_len, case.inp.k, w.k_max)
    ref = O.sparse_decode_batch(q, case.inp.K, case.inp.V, idx, case.scale)
    out = case.empty((w.B, w.Hq, w.d), torch.int16)
    out32 = case.empty((w.B, w.Hq, w.d), torch.float32)
    qd = H.to_dev(q)
    case.ctx.hata_sparse_decode(qd, case.K, case.V, H.to_dev(idx), case.k, w.B, case.scale, out, out32)
    case.sync()
    e = H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref, "sparse_decode")
    print(f"  sparse decode max abs err {e[0]:.2e}, max rel err {e[1]:.2e}")
    # out_f32 is optional
    out_b = case.empty((w.B, w.Hq, w.d), torch.int16)
    case.ctx.hata_sparse_decode(qd, case.K, case.V, H.to_dev(idx), case.k, w.B, case.scale, out_b, None)
    case.sync()
    assert torch.equal(out, out_b)
    # dense (Eq. 1) over the whole cache
    ref_d = O.dense_decode_batch(q, case.inp.K, case.inp.V, case.inp.seq_len, case.scale)
    case.ctx.hata_dense_decode(qd, case.K, case.V, case.seq_len, w.B, case.scale, out, out32)
    case.sync()
    e = H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref_d, "dense_decode")
    print(f"  dense decode max abs err {e[0]:.2e}, max rel err {e[1]:.2e}")


@pytest.mark.parametrize("mode", [0, 3])
def test_decode_step_end_to_end(case, mode):
    """mode 0: the single-launch form where the shape has one; mode 3: three launches."""
    import torch
    w = case.w
    case.ctx.hata_set_step_mode(mode)
    case.ctx.hata_keep_step_scores(True)  # the score array is inspected below
    n_launches, chunk, n_chunks = case.ctx.hata_step_plan(w.B)
    g = w.Hq // w.Hkv
    single_ok = w.r in (32, 64, 128, 256) and (g in (1, 2, 4, 5, 8) or (g == 16 and w.r <= 128))
    assert n_launches == (1 if (mode == 0 and single_ok) else 3), (n_launches, chunk, n_chunks)
    q = case.inp.q(3)
    # host: codes of rows [0, L-1) known, row L-1 is appended by the step
    codes_h = case.codes_ref.copy()
    for b in range(w.B):
        codes_h[b, :, int(case.inp.seq_len[b]) - 1:] = 0xDEADBEEF
    codes_d = H.to_dev(codes_h)
    ref = O.decode_step(q, case.inp.K, case.inp.V, case.inp.W_H, codes_h, case.inp.seq_len,
                        case.inp.k, w.k_max, case.scale, append=True)
    out = case.empty((w.B, w.Hq, w.d), torch.int16)
    out32 = case.empty((w.B, w.Hq, w.d), torch.float32)
    qd = H.to_dev(q)
    try:
        for rep in range(2):  # the second run must reproduce the first bit for bit
            case.ctx.hata_decode_step(qd, case.K, case.V, case.W_H, codes_d, case.seq_len, case.k, w.B,
                                      True, case.scale, out, out32)
            case.ctx.hata_check()  # waits for the stream; raises if an in-kernel wait gave up
            qc, sc, ix = case.ctx.hata_step_buffers()
            assert np.array_equal(H.to_host(codes_d, np.uint32), codes_h), "appended code row"
            assert np.array_equal(H.to_host(qc, np.uint32), ref["qcodes"])
            got_s = H.to_host(sc, np.uint16).astype(np.int32)
            for b in range(w.B):
                L = int(case.inp.seq_len[b])
                assert np.array_equal(got_s[b, :, :L], ref["scores"][b, :, :L])
            assert np.array_equal(H.to_host(ix), ref["idx"])
            H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "decode_step")
            if rep == 0:
                first = (out.clone(), out32.clone())
            else:
                assert torch.equal(out, first[0]) and torch.equal(out32, first[1])
    finally:
        case.ctx.hata_set_step_mode(0)
