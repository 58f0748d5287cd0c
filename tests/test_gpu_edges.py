"""Edge cases of the GPU path against the oracle: ties across chunk boundaries, k >= L,
empty sequences, B < B_max, negative index entries, strided caches, error codes."""
import ctypes
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth
from tests import harness as H


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def run_topk(torch, scores_np, seq_len, k, k_max, Hkv=1):
    from paper_2506_02572_amd import hata
    B, _, L_cap = scores_np.shape
    ctx = hata.Context(B, Hkv * 4, Hkv, 128, 128, L_cap, k_max)
    idx = torch.full((B, Hkv, k_max), -9, dtype=torch.int32, device="cuda")
    ctx.hata_topk(H.to_dev(scores_np.astype(np.uint16)), H.to_dev(np.asarray(seq_len, np.int32)),
                  H.to_dev(np.asarray(k, np.int32)), B, idx)
    torch.cuda.synchronize()
    ref = O.topk_batch(scores_np.astype(np.int32), np.asarray(seq_len, np.int32),
                       np.asarray(k, np.int32), k_max)
    ctx.close()
    return H.to_host(idx), ref


def test_topk_all_equal_scores_take_lowest_rows_across_chunks(torch_mod):
    L = 7000
    s = np.full((1, 1, L), 300, np.int32)
    got, ref = run_topk(torch_mod, s, [L], [2500], 2500)
    assert np.array_equal(got, ref)
    assert np.array_equal(got[0, 0], np.arange(2500))


def test_topk_two_values_threshold_ties_span_chunks(torch_mod):
    rng = np.random.default_rng(8)
    L = 9000
    s = rng.choice([100, 101], size=(2, 2, L)).astype(np.int32)
    got, ref = run_topk(torch_mod, s, [L, 6100], [4000, 333], 4000, Hkv=2)
    assert np.array_equal(got, ref)


def test_topk_k_ge_L_k_zero_len_one_and_len_zero(torch_mod):
    rng = np.random.default_rng(9)
    L_cap = 3000
    s = rng.integers(0, 513, size=(4, 1, L_cap)).astype(np.int32)
    seq = [2000, 1, 0, 3000]
    k = [2500, 5, 7, 0]
    got, ref = run_topk(torch_mod, s, seq, k, 2500)
    assert np.array_equal(got, ref)
    assert np.array_equal(got[0, 0, :2000], np.arange(2000)) and np.all(got[0, 0, 2000:] == -1)
    assert got[1, 0, 0] == 0 and np.all(got[1, 0, 1:] == -1)
    assert np.all(got[2] == -1) and np.all(got[3] == -1)


def test_topk_extreme_score_values(torch_mod):
    # scores at both ends of the range (0 and G*r = 512) and the full range in between
    L = 5000
    s = (np.arange(L) * 7919 % 513).astype(np.int32).reshape(1, 1, L)
    got, ref = run_topk(torch_mod, s, [L], [700], 700)
    assert np.array_equal(got, ref)


def test_step_with_empty_sequence_and_partial_batch(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    w = synth.Workload("edge", 3, 8, 2, 128, 128, (1500, 1, 2048), (64, 64, 3000), 4, 8.0,
                       L_cap=2048, k_max=2048)
    inp = synth.generate(w, seed=77)
    scale = 1.0 / math.sqrt(w.d)
    q = inp.q(0)
    seq = inp.seq_len.copy()
    codes_h, _ = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(3, np.int32), seq)
    # context sized for a larger batch than the call uses
    ctx = hata.Context(5, w.Hq, w.Hkv, w.d, w.r, w.L_cap, w.k_max)
    K, V, WH = H.to_dev(inp.K), H.to_dev(inp.V), H.to_dev(inp.W_H)
    out = torch.empty((3, w.Hq, w.d), dtype=torch.int16, device="cuda")
    out32 = torch.empty((3, w.Hq, w.d), dtype=torch.float32, device="cuda")
    codes_d = H.to_dev(codes_h)
    ctx.hata_decode_step(H.to_dev(q), K, V, WH, codes_d, H.to_dev(seq), H.to_dev(inp.k), 3, False,
                         scale, out, out32)
    torch.cuda.synchronize()
    ref = O.decode_step(q, inp.K, inp.V, inp.W_H, codes_h, seq, inp.k, w.k_max, scale, append=False)
    _, _, ix = ctx.hata_step_buffers()
    assert np.array_equal(H.to_host(ix)[:3], ref["idx"])
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "edge step")
    # sequence 2 has k >= L: the step equals dense attention (the k = L fixed point)
    dense = O.dense_decode_batch(q, inp.K, inp.V, seq, scale)
    assert np.max(np.abs(H.to_host(out32)[2] - dense[2])) < 2e-3
    # sequence 1 has one cached row: output = that V row
    v0 = synth.bf16_to_f32(inp.V[1, :, 0, :])
    got1 = H.to_host(out32)[1].reshape(w.Hkv, w.G, w.d)
    assert np.allclose(got1, v0[:, None, :], rtol=0, atol=1e-6)
    # a zero-length sequence gives zeros and touches nothing else
    seq0 = seq.copy()
    seq0[1] = 0
    ctx.hata_decode_step(H.to_dev(q), K, V, WH, codes_d, H.to_dev(seq0), H.to_dev(inp.k), 3, False,
                         scale, out, out32)
    torch.cuda.synchronize()
    assert np.all(H.to_host(out32)[1] == 0) and np.all(H.to_host(out, np.uint16)[1] == 0)
    ctx.close()


def test_single_launch_wait_gives_up_cleanly_and_is_reported(torch_mod):
    """Error path of the single-launch step, forced from the host: with a wait bound of one poll
    the workgroups give up at once; the kernel still runs to its end, hata_check() reports
    HATA_ETIMEOUT once, and the next step (default bound) is correct again."""
    torch = torch_mod
    from paper_2506_02572_amd import hata
    w = synth.Workload("giveup", 2, 8, 2, 128, 128, (5000, 3001), (100, 333), 4, 8.0, L_cap=5120)
    c = H.Case(w, seed=4321)
    assert c.ctx.hata_step_plan(w.B)[0] == 1 and c.ctx.hata_step_plan(w.B)[2] >= 2
    q = c.inp.q(1)
    codes_h = c.codes_ref.copy()
    codes_d = H.to_dev(codes_h)
    out = c.empty((w.B, w.Hq, w.d), torch.int16)
    out32 = c.empty((w.B, w.Hq, w.d), torch.float32)
    c.ctx.hata_set_wait_limit(1)
    c.ctx.hata_decode_step(H.to_dev(q), c.K, c.V, c.W_H, codes_d, c.seq_len, c.k, w.B, False,
                           c.scale, out, out32)
    with pytest.raises(hata.HataError, match="gave up"):
        c.ctx.hata_check()
    c.ctx.hata_check()  # the flag was cleared by the failed check
    c.ctx.hata_set_wait_limit(0)
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, c.inp.seq_len, c.inp.k, w.k_max,
                        c.scale, append=False)
    # the failure shows in the data: every query head is either NaN in both outputs (a workgroup of
    # its unit gave up a wait) or right; something is NaN
    # (the index lists of such a step are unspecified)
    o32, o16 = H.to_host(out32), H.to_host(out, np.uint16)
    n_nan = 0
    for b in range(w.B):
        for hq in range(w.Hq):
            if np.all(np.isnan(o32[b, hq])):
                assert np.all(o16[b, hq] == 0x7FC0)
                n_nan += 1
            else:
                H.check_attention(o32[b, hq], o16[b, hq], ref["out"][b, hq], "head without a give-up")
    assert n_nan > 0, "a step that gave up a wait must mark its outputs"
    print(f"[edges] forced give-up: {n_nan} of {w.B * w.Hq} heads marked NaN")
    for _ in range(2):
        c.ctx.hata_decode_step(H.to_dev(q), c.K, c.V, c.W_H, codes_d, c.seq_len, c.k, w.B, False,
                               c.scale, out, out32)
        c.ctx.hata_check()
        _, _, ix = c.ctx.hata_step_buffers()
        assert np.array_equal(H.to_host(ix), ref["idx"])
        H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "after give-up")
    c.ctx.close()


def test_kv_cache_in_pinned_host_memory(torch_mod):
    """The offloading variant (Sec. 5.3 of the paper): codes on the GPU, K and V in pinned host
    memory; the step gathers the selected rows over the bus.  Same results as with a device cache."""
    torch = torch_mod
    w = synth.Workload("kvhost", 2, 8, 2, 128, 128, (6000, 4500), (128, 96), 4, 8.0, append_steps=1)
    c = H.Case(w, seed=777)
    Kh = torch.from_numpy(c.inp.K.view(np.int16)).pin_memory()
    Vh = torch.from_numpy(c.inp.V.view(np.int16)).pin_memory()
    seq = c.inp.seq_len + 1
    codes_h = c.codes_ref.copy()
    codes_d = H.to_dev(codes_h)
    q = c.inp.q(0)
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=True)
    out = c.empty((w.B, w.Hq, w.d), torch.int16)
    out32 = c.empty((w.B, w.Hq, w.d), torch.float32)
    for mode in (0, 3):
        c.ctx.hata_set_step_mode(mode)
        out32.zero_()
        c.ctx.hata_decode_step(H.to_dev(q), Kh, Vh, c.W_H, codes_d, H.to_dev(seq), c.k, w.B, True,
                               c.scale, out, out32)
        c.ctx.hata_check()
        _, _, ix = c.ctx.hata_step_buffers()
        assert np.array_equal(H.to_host(ix), ref["idx"])
        assert np.array_equal(H.to_host(codes_d, np.uint32), codes_h), "appended key code (key read from host memory)"
        H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], f"host KV, mode {mode}")
    c.ctx.hata_set_step_mode(0)
    # unpinned host memory is refused on the host side, before any launch
    from paper_2506_02572_amd import hata
    with pytest.raises(hata.HataError):
        c.ctx.hata_decode_step(H.to_dev(q), torch.from_numpy(c.inp.K.view(np.int16)), Vh, c.W_H, codes_d,
                               H.to_dev(seq), c.k, w.B, True, c.scale, out, out32)
    c.ctx.close()


def test_sparse_decode_skips_negative_entries_and_strided_cache(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    B, Hq, Hkv, d, L, k_max = 2, 8, 2, 128, 600, 96
    K = synth.fill_bf16(5, 1, (B, Hkv, L, d))
    V = synth.fill_bf16(5, 2, (B, Hkv, L, d))
    q = synth.fill_bf16(5, 3, (B, Hq, 1, d)).reshape(B, Hq, d)
    scale = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(3)
    idx = np.full((B, Hkv, k_max), -1, np.int32)
    for b in range(B):
        for h in range(Hkv):
            n = 40 + 20 * b + h
            idx[b, h, :n] = np.sort(rng.choice(L, size=n, replace=False))
    ref = O.sparse_decode_batch(q, K, V, idx, scale)
    # cache with padded rows (stride 160 elements) and padded heads
    sn, sh = 160, 160 * (L + 3)
    sb = sh * Hkv + 64
    Kp = np.zeros(B * sb, np.uint16)
    Vp = np.zeros(B * sb, np.uint16)
    for b in range(B):
        for h in range(Hkv):
            for buf, src in ((Kp, K), (Vp, V)):
                view = buf[b * sb + h * sh: b * sb + h * sh + L * sn].reshape(L, sn)
                view[:, :d] = src[b, h]
                view[:, d:] = 0x7FC0  # NaN padding must never be read as data
    ctx = hata.Context(B, Hq, Hkv, d, 128, L, k_max, kv_strides=(sb, sh, sn))
    out = torch.empty((B, Hq, d), dtype=torch.int16, device="cuda")
    out32 = torch.empty((B, Hq, d), dtype=torch.float32, device="cuda")
    kk = H.to_dev(np.full(B, k_max, np.int32))
    ctx.hata_sparse_decode(H.to_dev(q), H.to_dev(Kp), H.to_dev(Vp), H.to_dev(idx), kk, B, scale, out, out32)
    torch.cuda.synchronize()
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref, "strided sparse")
    ctx.close()


def test_huge_logits_do_not_overflow(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    d, L = 128, 300
    qf = np.full((1, 1, d), 16.0, np.float32)
    Kf = np.where((np.arange(L) % 3 == 1)[:, None], -11.0, 11.0).astype(np.float32) * np.ones((L, d), np.float32)
    Vf = (np.arange(L) % 5).astype(np.float32)[:, None] * np.ones((L, d), np.float32)
    bits = lambda x: (x.view(np.uint32) >> 16).astype(np.uint16)
    q, K, V = bits(qf), bits(Kf).reshape(1, 1, L, d), bits(Vf).reshape(1, 1, L, d)
    scale = 1.0 / math.sqrt(d)
    ref = O.dense_decode_batch(q, K, V, np.array([L], np.int32), scale)
    ctx = hata.Context(1, 1, 1, d, 128, L, L)
    out = torch.empty((1, 1, d), dtype=torch.int16, device="cuda")
    out32 = torch.empty((1, 1, d), dtype=torch.float32, device="cuda")
    ctx.hata_dense_decode(H.to_dev(q), H.to_dev(K), H.to_dev(V), H.to_dev(np.array([L], np.int32)), 1,
                          scale, out, out32)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(H.to_host(out32)))
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref, "huge logits")
    ctx.close()


def test_error_codes_on_device_box(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    ctx = hata.Context(2, 8, 2, 128, 128, 1024, 64)
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(hata.HataError):   # B above B_max
        ctx.hata_hamming_score(t, t, t, 3, t)
    with pytest.raises(hata.HataError):   # NULL pointer
        ctx.hata_topk(None, t, t, 1, t)
    with pytest.raises(hata.HataError):   # unsupported head dim
        hata.Context(1, 8, 2, 64, 128, 1024, 64)
    with pytest.raises(hata.HataError):   # k_max above L_cap
        hata.Context(1, 8, 2, 128, 128, 64, 128)
    ctx.close()


def test_decode_steps_replayed_from_a_captured_graph(torch_mod):
    """Three decode steps (three contexts, i.e. three 'layers') captured in one HIP graph and
    replayed with new inputs between replays: every replay must equal the eager result of the same
    inputs.  (A captured launch freezes its arguments, the launch counter of the single-launch form
    included: the kernel retires what it published, so a replay cannot pick up stale words.)"""
    torch = torch_mod
    from paper_2506_02572_amd import hata
    w = synth.Workload("graph", 2, 8, 2, 128, 128, (5000, 3001), (100, 333), 4, 8.0, L_cap=5120)
    cases = [H.Case(w, seed=900 + i) for i in range(3)]
    assert cases[0].ctx.hata_step_plan(w.B)[0] == 1
    codes = [H.to_dev(c.codes_ref) for c in cases]
    qbuf = [torch.zeros((w.B, w.Hq, w.d), dtype=torch.int16, device="cuda") for _ in cases]
    outs = [torch.zeros((w.B, w.Hq, w.d), dtype=torch.int16, device="cuda") for _ in cases]
    outs32 = [torch.zeros((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda") for _ in cases]

    def enqueue():
        for c, cd, qd, o, o32 in zip(cases, codes, qbuf, outs, outs32):
            c.ctx.hata_decode_step(qd, c.K, c.V, c.W_H, cd, c.seq_len, c.k, w.B, False, c.scale, o, o32)

    def set_queries(step):
        for c, qd in zip(cases, qbuf):
            qd.copy_(H.to_dev(c.inp.q(step)))

    # eager references for four different query sets
    eager = []
    for step in range(4):
        set_queries(step)
        enqueue()
        torch.cuda.synchronize()
        eager.append(([o.clone() for o in outs32], [c.ctx.hata_step_buffers()[2].clone() for c in cases]))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        set_queries(0)
        enqueue()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enqueue()
    for step in (1, 3, 0, 2, 2):
        set_queries(step)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, c in enumerate(cases):
            c.ctx.hata_check()
            assert torch.equal(outs32[i], eager[step][0][i]), f"replay with query set {step}, layer {i}: output"
            assert torch.equal(c.ctx.hata_step_buffers()[2], eager[step][1][i]), f"replay {step}, layer {i}: index list"
        outs32[0].add_(1.0)  # eager work between the replays
        torch.cuda.synchronize()
    # and against the oracle once
    c = cases[1]
    ref = O.decode_step(c.inp.q(2), c.inp.K, c.inp.V, c.inp.W_H, c.codes_ref.copy(), c.inp.seq_len, c.inp.k,
                        w.k_max, c.scale, append=False)
    assert np.array_equal(H.to_host(c.ctx.hata_step_buffers()[2]), ref["idx"])
    for c in cases:
        c.ctx.close()


@pytest.mark.parametrize("r", [128, 64])
def test_prefill_write_fills_caches_and_codes_in_one_pass(torch_mod, r):
    """Alg. 1 of the paper in one call: new K / V rows land in the caches at start[b] + i and their
    key codes in the code cache; rows outside the range keep what they held."""
    torch = torch_mod
    w = synth.Workload("prefill", 2, 8, 2, 128, r, (3000, 1700), (64, 64), 4, 8.0, L_cap=3072)
    c = H.Case(w, seed=31, oracle_codes=False)
    B, Hkv, d = w.B, w.Hkv, w.d
    start = np.array([100, 0], np.int32)
    n_new = np.array([2500, 1700], np.int32)
    max_new = 2560
    # new rows = the generator's rows [0, n_new) of each unit, to be stored from row start[b] on
    K_new = np.zeros((B, Hkv, max_new, d), np.uint16)
    V_new = np.zeros((B, Hkv, max_new, d), np.uint16)
    for b in range(B):
        K_new[b, :, :n_new[b]] = c.inp.K[b, :, :n_new[b]]
        V_new[b, :, :n_new[b]] = c.inp.V[b, :, :n_new[b]]
    K_cache = torch.full((B, Hkv, w.L_cap, d), 0x1111, dtype=torch.int16, device="cuda")
    V_cache = torch.full((B, Hkv, w.L_cap, d), 0x2222, dtype=torch.int16, device="cuda")
    codes = torch.full((B, Hkv, w.L_cap, w.W), 0x33333333, dtype=torch.int32, device="cuda")
    c.ctx.hata_prefill_write(H.to_dev(K_new), H.to_dev(V_new), H.to_dev(start), H.to_dev(n_new), B, max_new,
                             K_cache, V_cache, codes, c.W_H)
    c.sync()
    Kc, Vc, cc = H.to_host(K_cache, np.uint16), H.to_host(V_cache, np.uint16), H.to_host(codes, np.uint32)
    # the oracle encodes the rows where they now sit in the cache
    K_host = np.full((B, Hkv, w.L_cap, d), 0x1111, np.uint16)
    for b in range(B):
        K_host[b, :, start[b]:start[b] + n_new[b]] = K_new[b, :, :n_new[b]]
    ref, near = O.encode_keys_batch(K_host, c.inp.W_H, start, n_new, bulk=True)
    for b in range(B):
        lo, hi = int(start[b]), int(start[b] + n_new[b])
        assert np.array_equal(Kc[b, :, lo:hi], K_new[b, :, :n_new[b]]) and np.array_equal(Vc[b, :, lo:hi], V_new[b, :, :n_new[b]])
        assert np.all(Kc[b, :, :lo] == 0x1111) and np.all(Kc[b, :, hi:] == 0x1111)
        assert np.all(Vc[b, :, :lo] == 0x2222) and np.all(Vc[b, :, hi:] == 0x2222)
        assert np.all(cc[b, :, :lo] == 0x33333333) and np.all(cc[b, :, hi:] == 0x33333333)
        diff = (cc[b, :, lo:hi] ^ ref[b, :, lo:hi]) & ~near[b, :, lo:hi]
        assert not np.any(diff), "key codes differ outside the |projection| < 1e-4 band"
    c.ctx.close()


def test_batch_larger_than_one_launch_runs_in_sub_batches(torch_mod):
    """More (sequence, KV head) units than one launch can keep resident: the single-launch form is
    issued once per slice of the batch; every sequence must come out as from the oracle, on the
    contiguous and on the paged layout."""
    torch = torch_mod
    lens = tuple(3000 + 257 * (i % 19) for i in range(20))
    ks = tuple(64 + 16 * (i % 5) for i in range(20))
    w = synth.Workload("bigbatch", 20, 32, 8, 128, 128, lens, ks, 4, 8.0, L_cap=8192, k_max=128)
    c = H.Case(w, seed=61, chunk=1024)  # 8 chunks x 8 KV heads per sequence: 20 sequences = 1280 workgroups
    B = w.B
    n_launches, chunk, n_chunks = c.ctx.hata_step_plan(B)
    n_sub = c.ctx.hata_step_sub_batches(B)
    assert (n_launches, chunk, n_chunks) == (1, 1024, 8) and n_sub >= 2, (n_launches, chunk, n_chunks, n_sub)
    assert c.ctx.hata_step_sub_batches(2) == 1
    q = c.inp.q(5)
    seq = c.inp.seq_len
    codes_h = c.codes_ref.copy()
    for b in range(B):
        codes_h[b, :, int(seq[b]) - 1:] = 0xDEADBEEF
    codes_before = codes_h.copy()
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=True)
    out = c.empty((B, w.Hq, w.d), torch.int16)
    out32 = c.empty((B, w.Hq, w.d), torch.float32)
    codes_d = H.to_dev(codes_before)
    qd = H.to_dev(q)
    c.ctx.hata_keep_step_scores(True)
    c.ctx.hata_decode_step(qd, c.K, c.V, c.W_H, codes_d, c.seq_len, c.k, B, True, c.scale, out, out32)
    c.ctx.hata_check()
    qc, sc, ix = c.ctx.hata_step_buffers()
    assert np.array_equal(H.to_host(codes_d, np.uint32), codes_h), "appended code rows"
    assert np.array_equal(H.to_host(qc, np.uint32), ref["qcodes"])
    got_s = H.to_host(sc, np.uint16).astype(np.int32)
    for b in range(B):
        assert np.array_equal(got_s[b, :, :int(seq[b])], ref["scores"][b, :, :int(seq[b])])
    assert np.array_equal(H.to_host(ix), ref["idx"])
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "sub-batched step")
    first = out32.clone()
    # mode 1: the whole batch in ONE grid that is larger than what is resident at once
    c.ctx.hata_set_step_mode(1)
    assert c.ctx.hata_step_sub_batches(B) == 1
    out32.zero_()
    c.ctx.hata_decode_step(qd, c.K, c.V, c.W_H, H.to_dev(codes_before), c.seq_len, c.k, B, True, c.scale, out, out32)
    c.ctx.hata_check()
    assert np.array_equal(H.to_host(c.ctx.hata_step_buffers()[2]), ref["idx"])
    assert torch.equal(out32, first)
    c.ctx.hata_set_step_mode(0)
    # the paged layout with one page per chunk, identity order: same pools as the contiguous caches
    # seen as [B * 8 pages, Hkv, 1024, .] after moving the block axis in front of the heads
    P, nb = 1024, w.L_cap // 1024
    def pool(t, last):
        return t.view(B, w.Hkv, nb, P, last).permute(0, 2, 1, 3, 4).contiguous().view(B * nb, w.Hkv, P, last)
    table = torch.arange(B * nb, dtype=torch.int32, device="cuda").view(B, nb).contiguous()
    Kp, Vp, Cp = pool(c.K, w.d), pool(c.V, w.d), pool(H.to_dev(codes_before), w.W)
    out32.zero_()
    c.ctx.hata_decode_step_paged(qd, Kp, Vp, c.W_H, Cp, table, nb, P, B * nb, c.seq_len, c.k, B, True, c.scale,
                                 out, out32)
    c.ctx.hata_check()
    assert np.array_equal(H.to_host(c.ctx.hata_step_buffers()[2]), ref["idx"])
    assert torch.equal(out32, first)
    c.ctx.close()


@pytest.mark.parametrize("chunk", [8192, 16384, 32768])
def test_step_with_large_chunks_ties_across_compaction_turns(torch_mod, chunk):
    """Single-launch step with more than 4096 keys per workgroup (the ordered compaction then runs in
    turns of 4096 keys): two-valued scores, so that the threshold's ties span turns and chunks, budgets
    above 4096 and above 8191 selected rows per chunk, ragged lengths incl. one row past a turn boundary."""
    torch = torch_mod
    from paper_2506_02572_amd import hata
    w = synth.Workload("bigchunk", 3, 8, 2, 128, 128, (20000, 13000, 4097), (9000, 5000, 4097), 4, 8.0,
                       L_cap=20000, k_max=9000)
    inp = synth.generate(w, seed=91)
    scale = 1.0 / math.sqrt(w.d)
    q = inp.q(0)
    seq = inp.seq_len.copy()
    rng = np.random.default_rng(92)
    two = rng.integers(0, 2 ** 32, size=(2, w.W), dtype=np.uint64).astype(np.uint32)
    pick = rng.integers(0, 2, size=(w.B, w.Hkv, w.L_cap))
    codes_h = two[pick]  # every key carries one of two codes: its score takes one of two values
    assert codes_h.shape == (w.B, w.Hkv, w.L_cap, w.W)
    ctx = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.L_cap, w.k_max, chunk=chunk)
    n_launches, got_chunk, n_chunks = ctx.hata_step_plan(w.B)
    assert n_launches == 1 and got_chunk == chunk and n_chunks == (w.L_cap + chunk - 1) // chunk
    K, V, WH = H.to_dev(inp.K), H.to_dev(inp.V), H.to_dev(inp.W_H)
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.int16, device="cuda")
    out32 = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
    codes_d = H.to_dev(codes_h)
    ref = O.decode_step(q, inp.K, inp.V, inp.W_H, codes_h.copy(), seq, inp.k, w.k_max, scale, append=False)
    for rep in range(2):  # twice: the control words must be back in their cleared state
        out32.zero_()
        ctx.hata_decode_step(H.to_dev(q), K, V, WH, codes_d, H.to_dev(seq), H.to_dev(inp.k), w.B, False,
                             scale, out, out32)
        ctx.hata_check()
        _, _, ix = ctx.hata_step_buffers()
        assert np.array_equal(H.to_host(ix), ref["idx"]), f"chunk {chunk}, call {rep}: index lists"
        H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], f"chunk {chunk}")
    ctx.close()


def test_overlap_probe_runs_in_its_three_modes(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    buf = torch.randn((8 << 20) // 2, dtype=torch.bfloat16, device="cuda").view(torch.int16)
    for mode in (1, 2, 3):
        hata.hata_probe_mfma_stream(buf, 4, mode)
    torch.cuda.synchronize()
    with pytest.raises(hata.HataError):
        hata.hata_probe_mfma_stream(buf[: 1 << 20], 4, 3)  # 2 MiB: below the probe's minimum

