"""Pins of the oracle's batch drivers (cache layout, GQA head mapping, ragged lengths,
step order of Alg. 3) against the per-unit oracle functions driven from Python slicing.

The unit functions themselves are pinned in test_oracle_pins.py; here only the
indexing around them is at stake, so each expectation is rebuilt from numpy slices.
"""
import math

import numpy as np

from oracle import hata_oracle as O
from paper_2506_02572_amd import synth


def small_workload():
    return synth.Workload("t", 3, 8, 2, 128, 64, (37, 64, 50), (8, 70, 16), 2, 8.0, L_cap=64)


def test_batch_drivers_match_per_unit_slicing():
    w = small_workload()
    inp = synth.generate(w, seed=9)
    q = inp.q(0)
    G = w.G
    codes, near = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(w.B, np.int32), inp.seq_len)
    qcodes, _ = O.encode_query_batch(q, inp.W_H)
    scores = O.score_batch(qcodes, codes, inp.seq_len)
    idx = O.topk_batch(scores, inp.seq_len, inp.k, w.k_max)
    scale = 1.0 / math.sqrt(w.d)
    out = O.sparse_decode_batch(q, inp.K, inp.V, idx, scale)
    dense = O.dense_decode_batch(q, inp.K, inp.V, inp.seq_len, scale)
    for b in range(w.B):
        L = int(inp.seq_len[b])
        for h in range(w.Hkv):
            c_u, _ = O.hash_encode(inp.K[b, h, :L], inp.W_H[h])
            assert np.array_equal(codes[b, h, :L], c_u)
            assert np.all(codes[b, h, L:] == 0)          # rows past the length are not written
            for g in range(G):
                qc_u, _ = O.hash_encode(q[b, h * G + g][None, :], inp.W_H[h])
                assert np.array_equal(qcodes[b, h * G + g], qc_u[0])
            s_u = O.hamming_score(qcodes[b, h * G:(h + 1) * G], codes[b, h, :L])
            assert np.array_equal(scores[b, h, :L], s_u)
            assert np.all(scores[b, h, L:] == -1)
            i_u = O.topk(s_u, int(inp.k[b]))
            cnt = min(int(inp.k[b]), L)
            assert np.array_equal(idx[b, h, :cnt], i_u)
            assert np.all(idx[b, h, cnt:] == -1)
            for g in range(G):
                o_u = O.attention_rows(q[b, h * G + g], inp.K[b, h], inp.V[b, h], i_u, scale)
                assert np.array_equal(out[b, h * G + g], o_u)
                d_u = O.attention_rows(q[b, h * G + g], inp.K[b, h, :L], inp.V[b, h, :L], None, scale)
                assert np.array_equal(dense[b, h * G + g], d_u)
    # sequence 1 has k >= L: sparse attention over every row equals dense attention (k = L fixed point)
    assert np.allclose(out[1], dense[1], rtol=0, atol=1e-13)
    assert not np.allclose(out[0], dense[0], rtol=0, atol=1e-6)


def test_bulk_encode_equals_batch_encode_and_respects_ranges():
    w = synth.Workload("t", 2, 4, 2, 128, 128, (700, 300), (8, 8), 0, 1.0, L_cap=700)
    inp = synth.generate(w, seed=10)
    start = np.array([5, 0], np.int32)
    n_new = np.array([600, 300], np.int32)
    a, na = O.encode_keys_batch(inp.K, inp.W_H, start, n_new)
    b, nb = O.encode_keys_batch(inp.K, inp.W_H, start, n_new, bulk=True)
    assert np.array_equal(a, b) and np.array_equal(na, nb)
    assert np.all(a[0, :, :5] == 0) and np.all(a[0, :, 605:] == 0) and np.all(a[1, :, 300:] == 0)
    assert np.any(a[0, :, 5:605] != 0)


def test_decode_step_is_the_composition_in_alg3_order():
    # the new key row sits at seq_len-1; its code must be written BEFORE scoring, so that
    # the current token takes part in the selection (decode-stage paragraph of Sec. 3.2)
    w = synth.Workload("t", 2, 8, 2, 128, 128, (129, 200), (16, 32), 4, 8.0, L_cap=256)
    inp = synth.generate(w, seed=12)
    q = inp.q(0)
    scale = 1.0 / math.sqrt(w.d)
    codes, _ = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(w.B, np.int32), inp.seq_len - 1)
    stale = codes.copy()
    res = O.decode_step(q, inp.K, inp.V, inp.W_H, codes, inp.seq_len, inp.k, w.k_max, scale, append=True)
    full, _ = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(w.B, np.int32), inp.seq_len)
    assert np.array_equal(codes, full)                      # append wrote exactly the last row
    assert not np.array_equal(codes, stale)
    qcodes, _ = O.encode_query_batch(q, inp.W_H)
    scores = O.score_batch(qcodes, full, inp.seq_len)
    idx = O.topk_batch(scores, inp.seq_len, inp.k, w.k_max)
    out = O.sparse_decode_batch(q, inp.K, inp.V, idx, scale)
    assert np.array_equal(res["qcodes"], qcodes)
    assert np.array_equal(res["scores"], scores)
    assert np.array_equal(res["idx"], idx)
    assert np.array_equal(res["out"], out)
    # a key identical to the query direction must be selectable in the step it is appended:
    # make the last row of unit (0, 0) equal to q of head 0 -> distance 0 for that head
    K2 = inp.K.copy()
    K2[0, 0, inp.seq_len[0] - 1] = q[0, 0]
    codes2 = stale.copy()
    res2 = O.decode_step(q, K2, inp.V, inp.W_H, codes2, inp.seq_len, inp.k, w.k_max, scale, append=True)
    assert int(inp.seq_len[0] - 1) in set(int(v) for v in res2["idx"][0, 0])


def test_workload_shapes_and_byte_counts():
    # the byte counts of the roofline table follow from the shapes
    assert synth.config(1).algorithmic_bytes() == 262144 + 524288 + 16384
    assert synth.config(2).algorithmic_bytes() == 4194304 + 2097152 + 16384
    assert synth.config(4).algorithmic_bytes() == 33554432 + 8388608 + 16384
    assert synth.config(5).algorithmic_bytes() == 33554432 + 16777216 + 131072
    w3 = synth.config(3)
    assert all(8192 <= l <= 32768 for l in w3.L) and all(kk % 64 == 0 for kk in w3.k)
    assert w3 == synth.config(3)  # seeded draw is reproducible
    assert synth.budget_2pct(32768) == 640 and synth.budget_2pct(8192) == 192


def test_generator_is_counter_based_and_gaussian():
    a = synth.fill_bf16(1, 2, (4, 1000, 128))
    b = synth.fill_bf16(1, 2, (1000, 128), first=2 * 1000 * 128)
    assert np.array_equal(a[2], b)                      # any slice can be regenerated on its own
    x = synth.bf16_to_f32(a).astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs(np.mean(x ** 4) - 3.0) < 0.1
    w = synth.fill_f32(1, 3, (128, 128), 128 ** -0.5)
    assert abs(w.std() * math.sqrt(128) - 1.0) < 0.02
    sc = synth.outlier_scales(synth.config(4), 7)
    assert np.all((sc == 16.0).sum(axis=1) == 8) and np.all((sc == 1.0).sum(axis=1) == 120)


def test_decode_step_against_a_pure_python_brute_force_on_a_tiny_case():
    """The whole step of Alg. 3 written again with nothing but Python numbers -- fractions for the
    projections (so the sign of every hash bit is exact), bin().count for the distances, sorted()
    on (distance, row) for the selection, math.exp for the softmax -- on a case small enough for
    that: every integer result must be identical, the output equal to 1e-12."""
    from fractions import Fraction
    w = synth.Workload("tiny", 2, 4, 2, 128, 32, (9, 5), (3, 7), 2, 8.0, L_cap=12, k_max=7)
    inp = synth.generate(w, seed=3)
    q = inp.q(0)
    scale = 1.0 / math.sqrt(w.d)
    codes, _ = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(w.B, np.int32), inp.seq_len - 1)
    res = O.decode_step(q, inp.K, inp.V, inp.W_H, codes, inp.seq_len, inp.k, w.k_max, scale, append=True)

    def f32(bits):  # bf16 bit pattern -> exact Fraction
        return Fraction(float(np.array([int(bits) << 16], np.uint32).view(np.float32)[0]))

    def code_of(vec_bits, h):  # Alg. 2: bit j set iff the projection on column j is >= 0
        x = [f32(v) for v in vec_bits]
        word = 0
        for j in range(w.r):
            proj = sum(x[c] * Fraction(float(inp.W_H[h, c, j])) for c in range(w.d))
            if proj >= 0:
                word |= 1 << j
        return word

    G = w.Hq // w.Hkv
    for b in range(w.B):
        L, kk = int(inp.seq_len[b]), int(inp.k[b])
        for h in range(w.Hkv):
            kcodes = [code_of(inp.K[b, h, n], h) for n in range(L)]
            got_codes = [int(codes[b, h, n, 0]) for n in range(L)]
            assert kcodes == got_codes, (b, h)
            qcodes = [code_of(q[b, h * G + g], h) for g in range(G)]
            assert qcodes == [int(res["qcodes"][b, h * G + g, 0]) for g in range(G)]
            dist = [sum(bin(qc ^ kc).count("1") for qc in qcodes) for kc in kcodes]
            assert dist == [int(v) for v in res["scores"][b, h, :L]]
            keep = sorted(n for _, n in sorted((dv, n) for n, dv in enumerate(dist))[:min(kk, L)])
            got_idx = [int(v) for v in res["idx"][b, h] if v >= 0]
            assert keep == got_idx, (b, h, keep, got_idx)
            assert all(int(v) == -1 for v in res["idx"][b, h, len(keep):])
            for g in range(G):
                qv = [float(f32(v)) for v in q[b, h * G + g]]
                logits = [scale * sum(qv[c] * float(f32(inp.K[b, h, n, c])) for c in range(w.d)) for n in keep]
                m = max(logits)
                wts = [math.exp(v - m) for v in logits]
                z = sum(wts)
                for c in range(0, w.d, 17):
                    want = sum(wt * float(f32(inp.V[b, h, n, c])) for wt, n in zip(wts, keep)) / z
                    assert abs(res["out"][b, h * G + g, c] - want) <= 1e-12 * max(1.0, abs(want))
