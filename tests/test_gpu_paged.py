"""Paged (block-table) cache layout: the decode step and the prefill cache fill on pools of pages
against the oracle, which knows only logical rows -- paging is a change of layout, not of the
method, so the test scatters the oracle-side arrays into pages and gathers them back."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth
from tests import harness as H

JUNK16 = 0x7FC0       # bf16 NaN: a read of a row that belongs to nobody poisons the output
JUNK32 = 0x5A5A5A5A


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def make_table(rng, seq_len, page_rows, spare=5, reserve=0):
    """Random assignment of pages to the blocks of each sequence; unused entries hold garbage."""
    B = len(seq_len)
    blocks = [(int(L) + reserve + page_rows - 1) // page_rows for L in seq_len]
    max_blocks = max(max(blocks), 1) + 2
    n_pages = sum(blocks) + spare
    perm = rng.permutation(n_pages)
    table = np.empty((B, max_blocks), np.int32)
    table[:, 0::2] = -1
    table[:, 1::2] = 2 ** 31 - 1
    at = 0
    for b in range(B):
        table[b, :blocks[b]] = perm[at:at + blocks[b]]
        at += blocks[b]
    return table, max_blocks, n_pages, blocks


def scatter(pool, logical, table, blocks, page_rows, seq_len):
    """pool[page, h, r] = logical[b, h, n] for every assigned row."""
    for b in range(logical.shape[0]):
        for blk in range(blocks[b]):
            lo = blk * page_rows
            hi = min(lo + page_rows, logical.shape[2])
            if hi > lo:
                pool[table[b, blk], :, :hi - lo] = logical[b, :, lo:hi]


def gather(pool, table, blocks, page_rows, shape, fill):
    out = np.full(shape, fill, pool.dtype)
    for b in range(shape[0]):
        for blk in range(blocks[b]):
            lo = blk * page_rows
            hi = min(lo + page_rows, shape[2])
            if hi > lo:
                out[b, :, lo:hi] = pool[table[b, blk], :, :hi - lo]
    return out


@pytest.mark.parametrize("page_rows,shape", [
    (16, ("g4_r128", 3, 8, 2, 128, (5000, 1, 3333), (200, 64, 5000), 8192)),
    (256, ("g4_r128", 3, 8, 2, 128, (5000, 1, 3333), (200, 64, 5000), 8192)),
    (2048, ("g8_r256", 2, 16, 2, 256, (7000, 4097), (512, 100), 8192)),
    (64, ("g1_r64", 2, 4, 4, 64, (2500, 900), (128, 128), 4096)),
    (512, ("g16_r128", 1, 32, 2, 128, (6000,), (300,), 8192)),
    # more than 4096 keys per workgroup (the chunk fixed through hata_tuning): up to 2049 page starts per chunk
    (16, ("g4_r128_chunk8k", 2, 8, 2, 128, (20000, 9001), (6000, 300), 20480, 8192)),
    (256, ("g4_r128_chunk16k", 2, 8, 2, 128, (20000, 9001), (6000, 300), 20480, 16384)),
    (16, ("g8_r256_chunk32k", 1, 16, 2, 256, (30001,), (9000,), 32768, 32768)),
])
def test_paged_decode_step_matches_the_oracle_and_the_contiguous_step(torch_mod, page_rows, shape):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    name, B, Hq, Hkv, r, lens, ks, L_cap = shape[:8]
    chunk = shape[8] if len(shape) > 8 else 0
    w = synth.Workload(name, B, Hq, Hkv, 128, r, lens, ks, 4, 8.0, L_cap=L_cap, k_max=min(L_cap, max(ks)))
    c = H.Case(w, seed=9 + page_rows, chunk=chunk)
    if chunk:
        assert c.ctx.hata_step_plan(B)[:2] == (1, chunk)
    rng = np.random.default_rng(page_rows)
    seq = c.inp.seq_len
    table, max_blocks, n_pages, blocks = make_table(rng, seq, page_rows)
    q = c.inp.q(1)
    # host: codes of rows [0, L-1) known, row L-1 is appended by the step
    codes_h = c.codes_ref.copy()
    for b in range(B):
        codes_h[b, :, int(seq[b]) - 1:] = 0xDEADBEEF
    codes_before = codes_h.copy()
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=True)
    K_pool = np.full((n_pages, Hkv, page_rows, 128), JUNK16, np.uint16)
    V_pool = np.full((n_pages, Hkv, page_rows, 128), JUNK16, np.uint16)
    C_pool = np.full((n_pages, Hkv, page_rows, w.W), JUNK32, np.uint32)
    # only rows [0, L) exist in the pools
    Kl, Vl, Cl = c.inp.K.copy(), c.inp.V.copy(), codes_before.copy()
    for b in range(B):
        Kl[b, :, int(seq[b]):] = JUNK16
        Vl[b, :, int(seq[b]):] = JUNK16
        Cl[b, :, int(seq[b]):] = JUNK32
    scatter(K_pool, Kl, table, blocks, page_rows, seq)
    scatter(V_pool, Vl, table, blocks, page_rows, seq)
    scatter(C_pool, Cl, table, blocks, page_rows, seq)
    Kd, Vd, Cd, Td = H.to_dev(K_pool), H.to_dev(V_pool), H.to_dev(C_pool), H.to_dev(table)
    out = c.empty((B, Hq, 128), torch.int16)
    out32 = c.empty((B, Hq, 128), torch.float32)
    qd = H.to_dev(q)
    c.ctx.hata_keep_step_scores(True)
    for rep in range(2):
        c.ctx.hata_decode_step_paged(qd, Kd, Vd, c.W_H, Cd, Td, max_blocks, page_rows, n_pages, c.seq_len,
                                     c.k, B, True, c.scale, out, out32)
        c.ctx.hata_check()
        qc, sc, ix = c.ctx.hata_step_buffers()
        assert np.array_equal(H.to_host(qc, np.uint32), ref["qcodes"])
        got_s = H.to_host(sc, np.uint16).astype(np.int32)
        for b in range(B):
            L = int(seq[b])
            assert np.array_equal(got_s[b, :, :L], ref["scores"][b, :, :L])
        assert np.array_equal(H.to_host(ix), ref["idx"])
        H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "paged step")
        # the code pool: the appended rows hold the oracle's codes, every other word is untouched
        want_pool = C_pool.copy()
        Cl2 = codes_h.copy()
        for b in range(B):
            Cl2[b, :, int(seq[b]):] = JUNK32
        scatter(want_pool, Cl2, table, blocks, page_rows, seq)
        assert np.array_equal(H.to_host(Cd, np.uint32), want_pool)
    # the same step on the contiguous layout gives the same bits
    out_c = c.empty((B, Hq, 128), torch.int16)
    out32_c = c.empty((B, Hq, 128), torch.float32)
    assert c.ctx.hata_step_plan(B)[0] == 1
    c.ctx.hata_decode_step(qd, c.K, c.V, c.W_H, H.to_dev(codes_before), c.seq_len, c.k, B, True, c.scale,
                           out_c, out32_c)
    c.ctx.hata_check()
    assert torch.equal(out32, out32_c) and torch.equal(out, out_c)
    c.ctx.close()


@pytest.mark.parametrize("page_rows,r", [(256, 128), (16, 64), (1024, 256)])
def test_paged_prefill_write_then_decode(torch_mod, page_rows, r):
    """Alg. 1 into pages, then one decode step from those pages: the pools hold exactly the rows the
    table names (everything else untouched), and the step agrees with the oracle."""
    torch = torch_mod
    w = synth.Workload("paged_prefill", 2, 8, 2, 128, r, (3001, 1700), (128, 64), 4, 8.0, L_cap=4096)
    c = H.Case(w, seed=41)
    B, Hkv, d = w.B, w.Hkv, w.d
    rng = np.random.default_rng(7)
    seq = c.inp.seq_len
    table, max_blocks, n_pages, blocks = make_table(rng, seq, page_rows)
    start = np.array([0, 0], np.int32)
    n_first = np.array([2000, 1700], np.int32)     # a first piece of the prompt ...
    start2 = np.array([2000, 1700], np.int32)      # ... and the rest (sequence 1 gets nothing more)
    n_second = np.array([int(seq[0]) - 2000, 0], np.int32)
    K_pool = torch.full((n_pages, Hkv, page_rows, d), 0x1111, dtype=torch.int16, device="cuda")
    V_pool = torch.full((n_pages, Hkv, page_rows, d), 0x2222, dtype=torch.int16, device="cuda")
    C_pool = torch.full((n_pages, Hkv, page_rows, w.W), 0x33333333, dtype=torch.int32, device="cuda")
    Td = H.to_dev(table)
    for st, nn in ((start, n_first), (start2, n_second)):
        max_new = int(nn.max())
        K_new = np.zeros((B, Hkv, max_new, d), np.uint16)
        V_new = np.zeros((B, Hkv, max_new, d), np.uint16)
        for b in range(B):
            K_new[b, :, :nn[b]] = c.inp.K[b, :, st[b]:st[b] + nn[b]]
            V_new[b, :, :nn[b]] = c.inp.V[b, :, st[b]:st[b] + nn[b]]
        c.ctx.hata_prefill_write_paged(H.to_dev(K_new), H.to_dev(V_new), H.to_dev(st), H.to_dev(nn), B, max_new,
                                       K_pool, V_pool, C_pool, Td, max_blocks, page_rows, n_pages, c.W_H)
    c.sync()
    Kp, Vp, Cp = H.to_host(K_pool, np.uint16), H.to_host(V_pool, np.uint16), H.to_host(C_pool, np.uint32)
    shape = (B, Hkv, w.L_cap)
    Kl = gather(Kp, table, blocks, page_rows, shape + (d,), 0x1111)
    Vl = gather(Vp, table, blocks, page_rows, shape + (d,), 0x2222)
    Cl = gather(Cp, table, blocks, page_rows, shape + (w.W,), 0x33333333)
    for b in range(B):
        L = int(seq[b])
        assert np.array_equal(Kl[b, :, :L], c.inp.K[b, :, :L]) and np.array_equal(Vl[b, :, :L], c.inp.V[b, :, :L])
        assert np.all(Kl[b, :, L:] == 0x1111) and np.all(Vl[b, :, L:] == 0x2222) and np.all(Cl[b, :, L:] == 0x33333333)
        diff = (Cl[b, :, :L] ^ c.codes_ref[b, :, :L]) & ~c.near[b, :, :L]
        assert not np.any(diff), "key codes differ outside the |projection| < 1e-4 band"
    # pages nobody owns are untouched
    owned = set(int(p) for b in range(B) for p in table[b, :blocks[b]])
    for p in range(n_pages):
        if p not in owned:
            assert np.all(Kp[p] == 0x1111) and np.all(Vp[p] == 0x2222) and np.all(Cp[p] == 0x33333333)
    # one decode step from the pages; the oracle scores the codes the device wrote (a bit inside
    # the near-zero band may legitimately differ from the exact evaluation)
    q = c.inp.q(2)
    codes_h = np.zeros(shape + (w.W,), np.uint32)
    for b in range(B):
        codes_h[b, :, :int(seq[b])] = Cl[b, :, :int(seq[b])]
    ref = O.decode_step(q, c.inp.K, c.inp.V, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=False)
    out = c.empty((B, w.Hq, d), torch.int16)
    out32 = c.empty((B, w.Hq, d), torch.float32)
    c.ctx.hata_decode_step_paged(H.to_dev(q), K_pool, V_pool, c.W_H, C_pool, Td, max_blocks, page_rows, n_pages,
                                 c.seq_len, c.k, B, False, c.scale, out, out32)
    c.ctx.hata_check()
    _, _, ix = c.ctx.hata_step_buffers()
    assert np.array_equal(H.to_host(ix), ref["idx"])
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "step after paged prefill")
    c.ctx.close()


def test_paged_arguments_are_validated(torch_mod):
    torch = torch_mod
    from paper_2506_02572_amd import hata
    ctx = hata.Context(1, 8, 2, 128, 128, 4096, 256)
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    buf = torch.zeros(1 << 20, dtype=torch.int32, device="cuda")
    args = lambda page_rows, max_blocks, n_pages: (buf, buf, buf, buf, buf, t, max_blocks, page_rows, n_pages, t, t, 1,
                                                   False, 0.1, buf, None)
    for page_rows, max_blocks, n_pages in ((8, 4, 4), (48, 4, 4), (256, 0, 4), (256, 4, 0), (1 << 20, 1 << 11, 4),
                                           (1 << 20, 4, 1 << 11)):
        with pytest.raises(hata.HataError, match="invalid argument"):
            ctx.hata_decode_step_paged(*args(page_rows, max_blocks, n_pages))
    # a shape without a single-launch kernel (r = 96) has no paged step
    ctx96 = hata.Context(1, 8, 2, 128, 96, 4096, 256)
    with pytest.raises(hata.HataError, match="unsupported"):
        ctx96.hata_decode_step_paged(*args(256, 4, 4))
    ctx.close()
    ctx96.close()


def test_two_sequences_share_the_pages_of_a_common_prefix(torch_mod):
    """Prefix sharing: the block tables of two sequences name the SAME pages for their first rows
    (read-only), each has private pages after that, and each appends into a private page.  Both
    must equal the oracle run on the logical caches."""
    torch = torch_mod
    page_rows, shared_blocks = 256, 9
    w = synth.Workload("prefix", 2, 8, 2, 128, 128, (4000, 3100), (160, 96), 4, 8.0, L_cap=4096)
    c = H.Case(w, seed=53, oracle_codes=False)
    B, Hkv, d = w.B, w.Hkv, w.d
    seq = c.inp.seq_len
    # logical caches: sequence 1 starts with the first shared_blocks * page_rows rows of sequence 0
    Kl, Vl = c.inp.K.copy(), c.inp.V.copy()
    n_shared = shared_blocks * page_rows
    Kl[1, :, :n_shared] = Kl[0, :, :n_shared]
    Vl[1, :, :n_shared] = Vl[0, :, :n_shared]
    codes_h, _ = O.encode_keys_batch(Kl, c.inp.W_H, np.zeros(B, np.int32), seq)
    for b in range(B):
        codes_h[b, :, int(seq[b]) - 1:] = 0xDEADBEEF  # row L-1 is appended by the step
    codes_before = codes_h.copy()
    q = c.inp.q(4)
    ref = O.decode_step(q, Kl, Vl, c.inp.W_H, codes_h, seq, c.inp.k, w.k_max, c.scale, append=True)
    # pages: shared prefix pages, then private ones
    blocks = [(int(L) + page_rows - 1) // page_rows for L in seq]
    n_pages = blocks[0] + (blocks[1] - shared_blocks) + 3
    rng = np.random.default_rng(5)
    perm = rng.permutation(n_pages)
    max_blocks = max(blocks)
    table = np.full((B, max_blocks), -7, np.int32)
    table[0, :blocks[0]] = perm[:blocks[0]]
    table[1, :shared_blocks] = table[0, :shared_blocks]
    table[1, shared_blocks:blocks[1]] = perm[blocks[0]:blocks[0] + blocks[1] - shared_blocks]
    assert blocks[0] - 1 >= shared_blocks and blocks[1] - 1 >= shared_blocks  # the appended rows sit in private pages
    K_pool = np.full((n_pages, Hkv, page_rows, d), JUNK16, np.uint16)
    V_pool = np.full((n_pages, Hkv, page_rows, d), JUNK16, np.uint16)
    C_pool = np.full((n_pages, Hkv, page_rows, w.W), JUNK32, np.uint32)
    Kx, Vx, Cx = Kl.copy(), Vl.copy(), codes_before.copy()
    for b in range(B):
        Kx[b, :, int(seq[b]):] = JUNK16
        Vx[b, :, int(seq[b]):] = JUNK16
        Cx[b, :, int(seq[b]):] = JUNK32
    for b in (1, 0):  # (sequence 0 last: it owns the shared pages in full)
        for pool, logical in ((K_pool, Kx), (V_pool, Vx), (C_pool, Cx)):
            scatter(pool, logical[b:b + 1], table[b:b + 1], blocks[b:b + 1], page_rows, seq[b:b + 1])
    Kd, Vd, Cd, Td = H.to_dev(K_pool), H.to_dev(V_pool), H.to_dev(C_pool), H.to_dev(table)
    out = c.empty((B, w.Hq, d), torch.int16)
    out32 = c.empty((B, w.Hq, d), torch.float32)
    c.ctx.hata_decode_step_paged(H.to_dev(q), Kd, Vd, c.W_H, Cd, Td, max_blocks, page_rows, n_pages, c.seq_len,
                                 c.k, B, True, c.scale, out, out32)
    c.ctx.hata_check()
    _, _, ix = c.ctx.hata_step_buffers()
    assert np.array_equal(H.to_host(ix), ref["idx"])
    H.check_attention(H.to_host(out32), H.to_host(out, np.uint16), ref["out"], "prefix-shared pages")
    got = gather(H.to_host(Cd, np.uint32), table[0:1], blocks[0:1], page_rows, (1, Hkv, w.L_cap, w.W), JUNK32)
    L0 = int(seq[0])
    assert np.array_equal(got[0, :, :L0], codes_h[0, :, :L0])
    got1 = gather(H.to_host(Cd, np.uint32), table[1:2], blocks[1:2], page_rows, (1, Hkv, w.L_cap, w.W), JUNK32)
    L1 = int(seq[1])
    assert np.array_equal(got1[0, :, :L1], codes_h[1, :, :L1])
    c.ctx.close()
