#!/usr/bin/env python3
"""Benchmark of the HATA decode-attention hot path on one MI355X.

A "step" is one whole decode step of Alg. 3 of the paper over one batch: hash-encode the
appended key and the query heads, Hamming-score every cached code, select the budget,
attend over the selected rows -- one call of hata_decode_step().  Inputs are seeded and
synthetic, resident in HBM before the timed region.  Consecutive steps rotate over many
distinct copies ("layers") of the K/V/code caches so that the traffic is HBM traffic and
not Infinity-Cache hits, as a model with tens of layers does for every token.

Prints ONE JSON line.  Beside the step itself it carries separately timed legs of the same
library: the scoring stage alone, the prefill key encode and the fused prefill cache fill, dense
attention (the comparison baseline), 32 layer steps replayed from one HIP graph, the step on the
paged cache layout (--paged), the learning-to-hash training step, and the CPU oracle.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch, from the rocprofv3 --pmc runs summarised in profiles/hbm_traffic_pmc.md:
# FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 (factors from a plain 256 MiB copy in the same runs).
# "step": the single-launch decode step (decode_step_coop_kernel); "score": the scoring kernel
# alone (hata_hamming_score).  None = not measured for that workload.
HBM_TRAFFIC_BYTES = {
    "cfg2_llama3_8b_32k": {"step": 9222963, "score": 5082317},
    "cfg3_batched_ragged": {"step": 72893542, "score": 45563085},
    "cfg4_long_128k_r256": {"step": 48662118, "score": 36862976},
    "cfg5_gqa8_append": {"step": 59414426, "score": 39123354},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="cfg2",
                    help="cfg1 .. cfg5 (the benchmark configurations; default cfg2) or a shape-sweep name "
                         "(paper_2506_02572_amd.synth.SWEEP)")
    ap.add_argument("--layers", type=int, default=0, help="distinct cache copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--kv-host", action="store_true",
                    help="offloading variant (Sec. 5.3 of the paper): K and V in pinned host memory, hash "
                         "codes on the GPU; the selected rows are gathered over the bus")
    ap.add_argument("--no-train", action="store_true", help="skip the learning-to-hash training-step leg")
    ap.add_argument("--graph-layers", type=int, default=32, metavar="N",
                    help="also time N consecutive layer steps captured in ONE HIP graph (a token's pass "
                         "through N attention layers): all hash-aware, and with the first two layers dense "
                         "(the paper keeps them dense, Sec. 5.1); 0 skips the leg")
    ap.add_argument("--step-mode", type=int, default=0, choices=(0, 1, 3),
                    help="hata_set_step_mode: 0 = single-launch form, a batch too large to be resident in "
                         "slices (default); 1 = the whole batch as one grid; 3 = three-launch form")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_ROWS",
                    help="also time the step on the paged (block-table) layout: the caches are re-laid as "
                         "pools of PAGE_ROWS-row pages in a random page order (needs L_cap %% PAGE_ROWS == 0)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--pmc-probe", action="store_true",
                    help="run only a known-size copy kernel, the decode step and the scoring kernel (for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs that calibrate and measure HBM traffic)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2506_02572_amd import hata, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HATA path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    w = synth.workload(args.workload)
    inp = synth.generate(w)
    scale = 1.0 / math.sqrt(w.d)
    n_step_variants = max(1, w.append_steps)

    def dev_bits(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        elif a.dtype == np.uint32:
            a = a.view(np.int32)
        return torch.from_numpy(a).to(dev)

    # ---- device buffers: n_layers copies of (K, V, codes)
    touched = w.algorithmic_bytes()
    layer_bytes = 2 * inp.K.nbytes + inp.K.nbytes // (w.d * 2) * (w.r // 8)
    n_layers = args.layers or max(4, min(int(math.ceil((1 << 30) / touched)), int((96 << 30) // layer_bytes)))
    if args.kv_host:
        # K / V stay in pinned host memory (a few copies: host reads are not cached between steps)
        n_layers = args.layers or 4
        Kh = torch.from_numpy(np.ascontiguousarray(inp.K).view(np.int16))
        Vh = torch.from_numpy(np.ascontiguousarray(inp.V).view(np.int16))
        K_all = torch.empty((n_layers,) + tuple(Kh.shape), dtype=torch.int16, pin_memory=True)
        V_all = torch.empty((n_layers,) + tuple(Vh.shape), dtype=torch.int16, pin_memory=True)
        K_all[:] = Kh
        V_all[:] = Vh
        K_dev0, V_dev0 = Kh.to(dev), Vh.to(dev)  # device copy of one layer for the prefill key encode
        del Kh, Vh
    else:
        K0, V0 = dev_bits(inp.K), dev_bits(inp.V)
        K_all = torch.empty((n_layers,) + tuple(K0.shape), dtype=torch.int16, device=dev)
        V_all = torch.empty_like(K_all)
        K_all[:] = K0
        V_all[:] = V0
        del K0, V0
    codes_all = torch.zeros((n_layers, w.B, w.Hkv, w.L_cap, w.W), dtype=torch.int32, device=dev)
    W_H = dev_bits(inp.W_H)
    kbud = dev_bits(inp.k)
    zero = torch.zeros(w.B, dtype=torch.int32, device=dev)
    # cfg5: the cache grows by one row per step for append_steps steps, then the cycle restarts
    seq_steps = [dev_bits(inp.seq_len + (t + 1 if w.append_steps else 0)) for t in range(n_step_variants)]
    q_steps = [dev_bits(inp.q(t)) for t in range(min(n_step_variants, 8))]
    prefill_len = dev_bits(inp.seq_len + w.append_steps)  # rows a later step appends get codes too
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.int16, device=dev)
    out32 = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
    ctx = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.L_cap, w.k_max)
    ctx.hata_set_step_mode(args.step_mode)
    stream = torch.cuda.current_stream()

    def timed(fn, n, warm):
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for i in range(n):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) / n, wall / n  # ms per call (device events, host wall)

    # ---- prefill-side key-code writer (Alg. 1: the key-code fill of the prefill), every layer once; timed separately
    max_prefill = int(inp.seq_len.max()) + w.append_steps

    # (with the cache in host memory the prefill encode runs from a device copy: every layer here
    # holds the same synthetic keys)
    enc_calls = [ctx.prepared("hata_encode_keys", K_dev0 if args.kv_host else K_all[l], W_H, zero, prefill_len,
                              w.B, max_prefill, codes_all[l], stream=stream) for l in range(n_layers)]

    def enc(i):
        enc_calls[i % n_layers]()

    enc_ms, _ = timed(enc, n_layers, 1)
    enc_keys = int((inp.seq_len + w.append_steps).sum()) * w.Hkv
    enc_bytes = enc_keys * (w.d * 2 + w.r // 8)
    enc_flop = 2.0 * enc_keys * w.d * w.r

    # ---- the same with the cache fill fused in (Alg. 1: KCache <- K, VCache <- V, K_H = HashEncode(K))
    fill_leg = None
    if not args.kv_host and not args.pmc_probe and w.r in (32, 64, 128, 256) and max_prefill == w.L_cap:
        K_dst, V_dst = torch.empty_like(K_all[0]), torch.empty_like(V_all[0])
        codes_dst = torch.empty_like(codes_all[0])
        fill_calls = [ctx.prepared("hata_prefill_write", K_all[l], V_all[l], zero, prefill_len, w.B, w.L_cap,
                                   K_dst, V_dst, codes_dst, W_H, stream=stream) for l in range(n_layers)]
        ms_fill, _ = timed(lambda i: fill_calls[i % n_layers](), n_layers, 1)
        fill_bytes = enc_keys * (4 * w.d * 2 + w.r // 8)  # K and V read and written once, codes written
        fill_leg = {"us_per_layer": round(ms_fill * 1e3, 1), "GBps": round(fill_bytes / (ms_fill * 1e-3) / 1e9, 1)}
        del K_dst, V_dst, codes_dst, fill_calls

    if args.pmc_probe:
        # a plain copy of known size (reads and writes COPY_BYTES each) calibrates the counters;
        # then the decode step and the scoring launch, the same calls the timed legs issue
        COPY_BYTES = 256 << 20
        src = torch.empty(COPY_BYTES // 4, dtype=torch.int32, device=dev).fill_(1)
        dst = torch.empty_like(src)
        qcodes_buf, scores_buf, _ = ctx.hata_step_buffers()
        ctx.hata_encode_query(q_steps[0], W_H, w.B, qcodes_buf, stream)
        torch.cuda.synchronize()
        for i in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        for i in range(40):
            ctx.hata_hamming_score(qcodes_buf, codes_all[i % n_layers], seq_steps[0], w.B, scores_buf, stream)
        torch.cuda.synchronize()
        for i in range(40):
            ctx.hata_decode_step(q_steps[0], K_all[i % n_layers], V_all[i % n_layers], W_H,
                                 codes_all[i % n_layers], seq_steps[0], kbud, w.B, True, scale, out, out32,
                                 stream)
        ctx.hata_check(stream)
        code_bytes = int(inp.seq_len.sum() + (w.B if w.append_steps else 0)) * w.Hkv * (w.r // 8)
        print(json.dumps({"pmc_probe": True, "workload": w.name, "copy_bytes_each_way": COPY_BYTES,
                          "score_code_bytes": code_bytes,
                          "score_write_bytes": code_bytes // (w.r // 8) * 2,
                          "step_algorithmic_bytes": w.algorithmic_bytes(1 if w.append_steps else 0),
                          "step_launches": ctx.hata_step_plan(w.B)[0]}))
        ctx.close()
        return

    # ---- the decode step
    n_combo = n_layers * n_step_variants // math.gcd(n_layers, n_step_variants)
    n_combo = min(n_combo, args.steps + args.warmup)
    step_calls = []
    for i in range(n_combo):
        l, t = i % n_layers, i % n_step_variants
        step_calls.append(ctx.prepared("hata_decode_step", q_steps[t % len(q_steps)], K_all[l], V_all[l],
                                       W_H, codes_all[l], seq_steps[t], kbud, w.B, True, scale, out,
                                       out32, stream=stream))

    def step(i):
        step_calls[i % n_combo]()

    ms_step, ms_wall = timed(step, args.steps, args.warmup)
    ctx.hata_check(stream)  # raises if a single-launch step gave up an in-kernel wait
    us_step = ms_step * 1e3
    n_launches, plan_chunk, plan_n_chunks = ctx.hata_step_plan(w.B)
    n_sub = ctx.hata_step_sub_batches(w.B)  # launches of the single-launch form (batch slices), 0 = three-launch form

    # ---- N layer steps in one HIP graph (launch gaps out of the way), with and without the dense first layers
    graph_leg = None
    if args.graph_layers > 0 and not args.kv_host:
        NL = args.graph_layers

        def enqueue(dense_first):
            for i in range(NL):
                l = i % n_layers
                if i < dense_first:
                    ctx.hata_dense_decode(q_steps[0], K_all[l], V_all[l], seq_steps[0], w.B, scale, out, out32)
                else:
                    ctx.hata_decode_step(q_steps[0], K_all[l], V_all[l], W_H, codes_all[l], seq_steps[0], kbud,
                                         w.B, True, scale, out, out32)

        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            enqueue(2)  # warm-up on a side stream before the capture
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graphs = {}
        for name, dense_first in (("hata_all_layers", 0), ("first_two_dense", 2)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                enqueue(dense_first)
            graphs[name] = g
        reps = max(10, args.steps // NL)
        graph_leg = {"layers": NL, "replays": reps}
        for name, g in graphs.items():
            ms_g, _ = timed(lambda i: g.replay(), reps, 2)
            graph_leg[name + "_us_per_replay"] = round(ms_g * 1e3, 1)
            graph_leg[name + "_us_per_layer"] = round(ms_g * 1e3 / NL, 3)
        ctx.hata_check(stream)
        del graphs

    # ---- the scoring stage alone (the largest stream of bytes of the step)
    qcodes_buf, scores_buf, _ = ctx.hata_step_buffers()

    score_calls = [ctx.prepared("hata_hamming_score", qcodes_buf, codes_all[l], seq_steps[0], w.B,
                                scores_buf, stream=stream) for l in range(n_layers)]

    def score_only(i):
        score_calls[i % n_layers]()

    ms_score, _ = timed(score_only, args.steps, args.warmup)
    code_bytes = int(inp.seq_len.sum() + (w.B if w.append_steps else 0)) * w.Hkv * (w.r // 8)
    score_gbps = code_bytes / (ms_score * 1e-3) / 1e9

    # ---- dense decode over the whole cache (Eq. 1): the comparison baseline, same shapes
    dense_us = None
    if not args.no_dense:
        dense_calls = [ctx.prepared("hata_dense_decode", q_steps[0], K_all[l], V_all[l], seq_steps[0], w.B,
                                    scale, out, out32, stream=stream) for l in range(n_layers)]

        def dense(i):
            dense_calls[i % n_layers]()
        ms_dense, _ = timed(dense, 5 if args.kv_host else max(20, args.steps // 8), 1 if args.kv_host else 5)
        dense_us = ms_dense * 1e3

    # ---- learning-to-hash training step (Sec. 3.1 / App. B): one SGD step on one head's W_H from a
    # 32K-triplet chunk (the chunk size of App. B.2), timed separately
    train_leg = None
    if not args.no_train:
        from paper_2506_02572_amd import train as htrain
        n_tr = 32768
        tctx = htrain.TrainContext(w.d, w.r, n_tr)
        Qt = dev_bits(synth.train_vectors(n_tr, tensor_id=synth.TID_Q))
        Kt = dev_bits(synth.train_vectors(n_tr, tensor_id=synth.TID_K))
        st = torch.full((n_tr,), -1.0, dtype=torch.float32, device=dev)
        st[::10] = 5.0
        Wt = W_H[0].to(torch.float32).contiguous().clone()
        vt = torch.zeros_like(Wt)
        hp = htrain.default_hparams(n_tr)

        def tstep(i):
            tctx.hata_train_step(Qt, Kt, st, n_tr, Wt, vt, hp, None, None, stream)
        ms_tr, _ = timed(tstep, 50, 5)
        flop = 4 * 2.0 * n_tr * w.d * w.r  # two projections + two weight-gradient contractions
        train_leg = {"triplets": n_tr, "r": w.r, "us_per_step": round(ms_tr * 1e3, 1),
                     "TFLOPs": round(flop / (ms_tr * 1e-3) / 1e12, 1),
                     "mfma_issue_TFLOPs": round((3 * 3 + 2 * 3) / 4 * flop / (ms_tr * 1e-3) / 1e12, 1),
                     "launches": 6}
        tctx.close()

    # ---- parity of one step + the oracle timed on this machine's host cores (rank 0, N = 1)
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import hata_oracle as O
        seq0 = inp.seq_len + (1 if w.append_steps else 0)
        # the oracle encodes its own key codes for its own step
        codes_o, _ = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(w.B, np.int32), seq0, bulk=True)
        q0 = inp.q(0)
        t0 = time.perf_counter()
        ref = O.decode_step(q0, inp.K, inp.V, inp.W_H, codes_o, seq0, inp.k, w.k_max, scale, append=True)
        t1 = time.perf_counter() - t0
        reps = int(max(1, min(5000, args.cpu_seconds / max(t1, 1e-6))))
        t0 = time.perf_counter()
        for _ in range(reps):
            O.decode_step(q0, inp.K, inp.V, inp.W_H, codes_o, seq0, inp.k, w.k_max, scale, append=True)
        tn = (time.perf_counter() - t0) / reps
        cpu = {"value": round(tn * 1e6, 1), "unit": "us/step", "cores": O.num_threads(), "kind": "oracle",
               "sample": f"{reps} full decode steps of {w.name} (all {w.B * w.Hkv} units, layer 0, step 0)"}
        # parity of the GPU step on the oracle's codes
        codes_dev = dev_bits(codes_o)
        ctx.hata_decode_step(q_steps[0], K_all[0], V_all[0], W_H, codes_dev, seq_steps[0], kbud, w.B, True,
                             scale, out, out32, stream)
        torch.cuda.synchronize()
        _, _, ix = ctx.hata_step_buffers()
        idx_equal = bool(np.array_equal(ix.cpu().numpy(), ref["idx"]))
        err = np.abs(out32.cpu().numpy().astype(np.float64) - ref["out"])
        ok = bool(np.all(err <= 2e-3 + 1e-3 * np.abs(ref["out"])))
        parity = {"idx_equal": idx_equal, "attn_within_tol": ok, "max_abs_err": float(err.max())}

    # ---- the step on the paged layout (last: the caches are re-laid in place, page order random)
    paged_leg = None
    if args.paged and not args.kv_host and w.L_cap % args.paged == 0 and n_launches == 1:
        P = args.paged
        ctx.hata_decode_step(q_steps[0], K_all[0], V_all[0], W_H, codes_all[0], seq_steps[0], kbud, w.B, True,
                             scale, out, out32, stream)
        torch.cuda.synchronize()
        ref_out = out32.clone()  # the same step on the contiguous layout, for a bit-for-bit comparison
        nb = w.L_cap // P
        n_pages = w.B * nb
        perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(1))  # page of block (b, blk)
        table = perm.view(w.B, nb).to(torch.int32).to(dev)
        inv = torch.argsort(perm).to(dev)                                           # block held by page p

        def to_pool(t, last):  # [B, Hkv, L_cap, last] -> [n_pages, Hkv, P, last] in the same memory
            blocks = t.view(w.B, w.Hkv, nb, P, last).permute(0, 2, 1, 3, 4).reshape(n_pages, w.Hkv, P, last)
            t.view(n_pages, w.Hkv, P, last).copy_(blocks.index_select(0, inv))

        for l in range(n_layers):
            to_pool(K_all[l], w.d)
            to_pool(V_all[l], w.d)
            to_pool(codes_all[l], w.W)
        paged_calls = []
        for i in range(n_combo):
            l, t = i % n_layers, i % n_step_variants
            paged_calls.append(ctx.prepared("hata_decode_step_paged", q_steps[t % len(q_steps)], K_all[l], V_all[l],
                                            W_H, codes_all[l], table, nb, P, n_pages, seq_steps[t], kbud, w.B,
                                            True, scale, out, out32, stream=stream))
        ctx.hata_decode_step_paged(q_steps[0], K_all[0], V_all[0], W_H, codes_all[0], table, nb, P, n_pages,
                                   seq_steps[0], kbud, w.B, True, scale, out, out32, stream)
        torch.cuda.synchronize()
        same = bool(torch.equal(ref_out, out32))
        ms_paged, _ = timed(lambda i: paged_calls[i % n_combo](), args.steps, args.warmup)
        ctx.hata_check(stream)
        paged_leg = {"page_rows": P, "n_pages": n_pages, "us_per_step": round(ms_paged * 1e3, 3),
                     "same_bits_as_contiguous": same}

    alg_bytes = w.algorithmic_bytes(1 if w.append_steps else 0)
    traffic = HBM_TRAFFIC_BYTES.get(w.name, {})
    step_gbps = alg_bytes / (us_step * 1e-6) / 1e9
    score_stage = {"kernel": "score_kernel (hata_hamming_score)", "achieved": round(score_gbps, 1),
                   "unit": "GB/s", "frac": round(score_gbps / HBM_PEAK_GBPS, 4),
                   "traffic": traffic.get("score"), "algorithmic_bytes_per_launch": code_bytes,
                   "avg_launch_us": round(ms_score * 1e3, 3)}
    if n_launches == 1:
        # the whole step is ONE kernel (launched once per slice of a batch too large to be resident at
        # once): it is the dominant kernel, its launches are the step
        roofline = {"bound": "hbm", "kernel": "decode_step_coop_kernel (hata_decode_step: the whole step in one launch)",
                    "achieved": round(step_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(step_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic.get("step"),
                    "algorithmic_bytes_per_launch": alg_bytes // n_sub, "avg_launch_us": round(us_step / n_sub, 3)}
    else:
        roofline = dict(score_stage, bound="hbm", peak=HBM_PEAK_GBPS)
    result = {
        "metric": "hata_decode_attention_us_per_step",
        "value": round(us_step, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 K/V/q with fp32 accumulate; u32 codes; fp64 query/append projection",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d, "r": w.r,
                   "L": list(w.L) if len(set(w.L)) > 1 else w.L[0],
                   "k": list(w.k) if len(set(w.k)) > 1 else w.k[0],
                   "layers_rotated": n_layers, "append_per_step": True,
                   "kv_cache": "pinned host memory (rows gathered over the bus)" if args.kv_host else "HBM",
                   "launches_per_step": n_sub if n_launches == 1 else n_launches, "step_mode": args.step_mode,
                   "chunk": plan_chunk,
                   "chunks_per_unit": plan_n_chunks},
        "achieved_GBps": round(step_gbps, 1),
        "algorithmic_bytes_per_step": alg_bytes,
        "step_roofline_frac": round(step_gbps / HBM_PEAK_GBPS, 4),
        "host_wall_us_per_step": round(ms_wall * 1e3, 3),
        "roofline": roofline,
        "score_stage": score_stage,
        "encode_keys_bulk": {"us_per_layer": round(enc_ms * 1e3, 1), "keys": enc_keys,
                             "GBps": round(enc_bytes / (enc_ms * 1e-3) / 1e9, 1),
                             "TFLOPs": round(enc_flop / (enc_ms * 1e-3) / 1e12, 2)},
        "prefill_write": fill_leg,
        "paged_step": paged_leg,
        "graph_of_layers": graph_leg,
        "dense_decode_us": None if dense_us is None else round(dense_us, 2),
        "speedup_vs_dense": None if dense_us is None else round(dense_us / us_step, 2),
        "train_step": train_leg,
        "cpu_baseline": cpu,
        "parity": parity,
    }
    print(json.dumps(result))
    ctx.close()


if __name__ == "__main__":
    main()
