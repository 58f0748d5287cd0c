#!/usr/bin/env python3
"""Benchmark of the HATA decode-attention hot path on one MI355X.

A "step" is one whole decode step of Alg. 3 of the paper over one batch: hash-encode the
appended key and the query heads, Hamming-score every cached code, select the budget,
attend over the selected rows -- one call of hata_decode_step().  Inputs are seeded and
synthetic, resident in HBM before the timed region.  Consecutive steps rotate over many
distinct copies ("layers") of the K/V/code caches so that the traffic is HBM traffic and
not Infinity-Cache hits, as a model with tens of layers does for every token.

Prints ONE JSON line.  The headline (value, roofline, cpu_baseline) is the workload named by
--workload (default: configuration 2), timed over exactly --steps steps after --warmup.  Beside it
the line carries separately timed legs of the same library (the four stage entry points of the step
each alone -- "stages_alone": query encode, Hamming scoring, top-k, sparse attention --, prefill key
encode and fused prefill cache fill, dense attention, 32 layer steps replayed from one HIP graph,
the paged layout, the KV cache in host memory with and without a staged prefetch, the
learning-to-hash training step), and -- in the default run -- "per_config": the step of
configurations 2, 3, 4 and 5 at full size, each with its own steady-state timing, roofline
fraction, dense comparison and parity against the oracle, and "larger_batch": the same fields for
B = 32 at L = 32K (a serving-size batch, outside the batch range the headline metric names).
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
PER_CONFIG_STEPS = 300   # timed steps of every per_config entry (the headline takes --steps)
PER_CONFIG_WARMUP = 40

# HBM bytes per launch from the rocprofv3 --pmc runs summarised in profiles/hbm_traffic_pmc.md
# (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors from a plain 256 MiB copy in the same runs).  A
# constant of the build the profile names, not a value measured by the run that prints it: the
# "traffic_source" field of the output says so.  "step": the single-launch decode step
# (decode_step_coop_kernel); "score": the scoring kernel alone (hata_hamming_score).
HBM_TRAFFIC_SOURCE = "profiles/hbm_traffic_pmc.md (library of commit 27b79d8; b32_32k: e4b3f88)"
HBM_TRAFFIC_BYTES = {
    "cfg2_llama3_8b_32k": {"step": 9348096, "score": 5082317},
    "cfg3_batched_ragged": {"step": 73044890, "score": 45608141},
    "cfg4_long_128k_r256": {"step": 48791552, "score": 36881203},
    "cfg5_gqa8_append": {"step": 59498394, "score": 39123354},
    "b32_32k": {"step": 209088922, "score": 153628262},
}


GATHER_WGS = 32  # hata_gather_rows from host memory: workgroups with reads outstanding at once


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
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per_config list (configurations 2-5 at full size); it is only produced "
                         "when --workload is the default")
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
    ap.add_argument("--chunk", type=int, default=0, choices=(0, 1024, 2048, 4096, 8192, 16384, 32768),
                    help="hata_tuning.chunk: cached keys per scoring workgroup (0 = the library's choice)")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_ROWS",
                    help="also time the step on the paged (block-table) layout: the caches are re-laid as "
                         "pools of PAGE_ROWS-row pages in a random page order (needs L_cap %% PAGE_ROWS == 0)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--phase-trace", action="store_true",
                    help="print the in-kernel timeline of the single-launch step instead of timing it: per "
                         "checkpoint, when the first / median / last workgroup of the grid passed it.  Needs "
                         "a tuning build of the library (python paper_2506_02572_amd/build.py --trace)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="run only a known-size copy kernel, the decode step and the scoring kernel (for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs that calibrate and measure HBM traffic)")
    ap.add_argument("--overlap-probe", action="store_true",
                    help="run only hata_probe_mfma_stream: a loop of bf16 matrix-core instructions, a 1 GiB "
                         "read, and both in one launch, timed with events (do the two overlap on this device?)")
    return ap.parse_args()


def dev_bits(a, dev):
    import numpy as np
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(dev)


def timed(fn, n, warm, stream):
    """ms per call over exactly n calls after warm untimed ones: (device events, host wall)."""
    import torch
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
    return e0.elapsed_time(e1) / n, wall / n


class Bench:
    """One workload on the device: rotated cache copies, a context, and the legs that time it."""

    def __init__(self, name, args, layers=0, kv_host=False, step_mode=0):
        import numpy as np
        import torch
        from paper_2506_02572_amd import hata, synth
        self.np, self.torch = np, torch
        self.dev = torch.device("cuda:0")
        self.args = args
        w = self.w = synth.workload(name)
        inp = self.inp = synth.generate(w)
        self.scale = 1.0 / math.sqrt(w.d)
        self.kv_host = kv_host
        self.n_step_variants = max(1, w.append_steps)
        dev = self.dev
        touched = w.algorithmic_bytes()
        layer_bytes = 2 * inp.K.nbytes + inp.K.nbytes // (w.d * 2) * (w.r // 8)
        n_layers = layers or max(4, min(int(math.ceil((1 << 30) / touched)), int((96 << 30) // layer_bytes)))
        if kv_host:
            # K / V stay in pinned host memory (a few copies: host reads are not cached between steps)
            n_layers = layers or 4
            Kh = torch.from_numpy(np.ascontiguousarray(inp.K).view(np.int16))
            Vh = torch.from_numpy(np.ascontiguousarray(inp.V).view(np.int16))
            self.K_all = torch.empty((n_layers,) + tuple(Kh.shape), dtype=torch.int16, pin_memory=True)
            self.V_all = torch.empty((n_layers,) + tuple(Vh.shape), dtype=torch.int16, pin_memory=True)
            self.K_all[:] = Kh
            self.V_all[:] = Vh
            self.K_dev0, self.V_dev0 = Kh.to(dev), Vh.to(dev)  # device copy of one layer for the prefill key encode
            del Kh, Vh
        else:
            K0, V0 = dev_bits(inp.K, dev), dev_bits(inp.V, dev)
            self.K_all = torch.empty((n_layers,) + tuple(K0.shape), dtype=torch.int16, device=dev)
            self.V_all = torch.empty_like(self.K_all)
            self.K_all[:] = K0
            self.V_all[:] = V0
            del K0, V0
        self.n_layers = n_layers
        self.codes_all = torch.zeros((n_layers, w.B, w.Hkv, w.L_cap, w.W), dtype=torch.int32, device=dev)
        self.W_H = dev_bits(inp.W_H, dev)
        self.kbud = dev_bits(inp.k, dev)
        self.zero = torch.zeros(w.B, dtype=torch.int32, device=dev)
        # cfg5: the cache grows by one row per step for append_steps steps, then the cycle restarts
        self.seq_steps = [dev_bits(inp.seq_len + (t + 1 if w.append_steps else 0), dev)
                          for t in range(self.n_step_variants)]
        self.q_steps = [dev_bits(inp.q(t), dev) for t in range(min(self.n_step_variants, 8))]
        self.prefill_len = dev_bits(inp.seq_len + w.append_steps, dev)  # rows a later step appends get codes too
        self.max_prefill = int(inp.seq_len.max()) + w.append_steps
        self.out = torch.empty((w.B, w.Hq, w.d), dtype=torch.int16, device=dev)
        self.out32 = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
        self.ctx = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.L_cap, w.k_max, chunk=getattr(args, "chunk", 0))
        self.ctx.hata_set_step_mode(step_mode)
        self.stream = torch.cuda.current_stream()
        # the hash weights are fixed: their fp16 planes for the prefill key encoder are made once
        self.ctx.hata_prepare_weights(self.W_H, self.stream)
        self.alg_bytes = w.algorithmic_bytes(1 if w.append_steps else 0)
        self.code_bytes = int(inp.seq_len.sum() + (w.B if w.append_steps else 0)) * w.Hkv * (w.r // 8)

    def close(self):
        self.ctx.close()
        for n in ("K_all", "V_all", "codes_all", "K_dev0", "V_dev0"):
            if hasattr(self, n):
                delattr(self, n)
        self.torch.cuda.empty_cache()

    # ---- prefill-side key-code writer (Alg. 1: the key-code fill of the prefill), every layer once
    def encode_keys(self):
        w, inp = self.w, self.inp
        calls = [self.ctx.prepared("hata_encode_keys", self.K_dev0 if self.kv_host else self.K_all[l], self.W_H,
                                   self.zero, self.prefill_len, w.B, self.max_prefill, self.codes_all[l],
                                   stream=self.stream) for l in range(self.n_layers)]
        ms, _ = timed(lambda i: calls[i % self.n_layers](), self.n_layers, 1, self.stream)
        keys = int((inp.seq_len + w.append_steps).sum()) * w.Hkv
        nbytes = keys * (w.d * 2 + w.r // 8)
        flop = 2.0 * keys * w.d * w.r
        return {"us_per_layer": round(ms * 1e3, 1), "keys": keys, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "TFLOPs": round(flop / (ms * 1e-3) / 1e12, 2)}

    # ---- the same with the cache fill fused in (Alg. 1: KCache <- K, VCache <- V, K_H = HashEncode(K))
    def prefill_write(self):
        w, torch = self.w, self.torch
        if self.kv_host or w.r not in (32, 64, 128, 256) or self.max_prefill != w.L_cap:
            return None
        K_dst, V_dst = torch.empty_like(self.K_all[0]), torch.empty_like(self.V_all[0])
        codes_dst = torch.empty_like(self.codes_all[0])
        calls = [self.ctx.prepared("hata_prefill_write", self.K_all[l], self.V_all[l], self.zero, self.prefill_len,
                                   w.B, w.L_cap, K_dst, V_dst, codes_dst, self.W_H, stream=self.stream)
                 for l in range(self.n_layers)]
        ms, _ = timed(lambda i: calls[i % self.n_layers](), self.n_layers, 1, self.stream)
        keys = int((self.inp.seq_len + w.append_steps).sum()) * w.Hkv
        fill_bytes = keys * (4 * w.d * 2 + w.r // 8)  # K and V read and written once, codes written
        return {"us_per_layer": round(ms * 1e3, 1), "GBps": round(fill_bytes / (ms * 1e-3) / 1e9, 1)}

    # ---- the decode step
    def step(self, steps, warmup):
        w = self.w
        n_combo = self.n_layers * self.n_step_variants // math.gcd(self.n_layers, self.n_step_variants)
        n_combo = min(n_combo, steps + warmup)
        calls = []
        for i in range(n_combo):
            l, t = i % self.n_layers, i % self.n_step_variants
            calls.append(self.ctx.prepared("hata_decode_step", self.q_steps[t % len(self.q_steps)], self.K_all[l],
                                           self.V_all[l], self.W_H, self.codes_all[l], self.seq_steps[t], self.kbud,
                                           w.B, True, self.scale, self.out, self.out32, stream=self.stream))
        self.step_calls, self.n_combo = calls, n_combo
        # every rotated cache copy is stepped through once before the warm-up (untimed set-up, reported
        # as config.first_pass_untimed): a decode loop revisits its layers' caches every token, and the
        # very first touch of a cache copy costs 1-2 us more than any later one
        for call in calls:
            call()
        self.stream.synchronize()
        ms, wall = timed(lambda i: calls[i % n_combo](), steps, warmup, self.stream)
        self.ctx.hata_check(self.stream)  # raises if a single-launch step gave up an in-kernel wait
        return ms * 1e3, wall * 1e3

    def plan(self):
        n_launches, chunk, n_chunks = self.ctx.hata_step_plan(self.w.B)
        n_sub = self.ctx.hata_step_sub_batches(self.w.B)  # launches of the single-launch form (batch slices), 0 = three-launch form
        return n_launches, chunk, n_chunks, n_sub

    # ---- N layer steps in one HIP graph (launch gaps out of the way), with and without the dense first layers
    def graph_of_layers(self, NL, steps):
        torch, w, ctx = self.torch, self.w, self.ctx

        def enqueue(dense_first):
            for i in range(NL):
                l = i % self.n_layers
                if i < dense_first:
                    ctx.hata_dense_decode(self.q_steps[0], self.K_all[l], self.V_all[l], self.seq_steps[0], w.B,
                                          self.scale, self.out, self.out32)
                else:
                    ctx.hata_decode_step(self.q_steps[0], self.K_all[l], self.V_all[l], self.W_H, self.codes_all[l],
                                         self.seq_steps[0], self.kbud, w.B, True, self.scale, self.out, self.out32)

        side = torch.cuda.Stream()
        side.wait_stream(self.stream)
        with torch.cuda.stream(side):
            enqueue(2)  # warm-up on a side stream before the capture
        self.stream.wait_stream(side)
        torch.cuda.synchronize()
        graphs = {}
        for name, dense_first in (("hata_all_layers", 0), ("first_two_dense", 2)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                enqueue(dense_first)
            graphs[name] = g
        reps = max(10, steps // NL)
        leg = {"layers": NL, "replays": reps}
        for name, g in graphs.items():
            ms_g, _ = timed(lambda i: g.replay(), reps, 2, self.stream)
            leg[name + "_us_per_replay"] = round(ms_g * 1e3, 1)
            leg[name + "_us_per_layer"] = round(ms_g * 1e3 / NL, 3)
        ctx.hata_check(self.stream)
        return leg

    # ---- offloading variant with prefetch (Sec. 5.3): the selected rows of layer l + 1 are fetched from
    # pinned host memory into a double staging buffer on a second stream while layer l attends
    def kv_host_prefetch(self, NL, reps, D=3):
        """Per layer: hata_select_step (codes and q are on the GPU) on the main stream, D - 1 layers
        ahead of the attention; hata_gather_rows of that layer on the fetch stream (same priority)
        once the selection is there, into one of D staging buffers; attention over the staged rows on
        the main stream once the fetch is there.  The queries of all layers are given (synthetic),
        as they are for every other leg; in a model the query of a layer ahead would come from a
        speculated projection or from another request in flight.  Returns us per layer, the bus rate
        of the selected rows, and whether the last layer's output has the bits of attention
        straight over the host-resident cache."""
        from paper_2506_02572_amd import hata
        torch, w, ctx = self.torch, self.w, self.ctx
        stage_ctx = hata.Context(w.B, w.Hq, w.Hkv, w.d, w.r, w.k_max, w.k_max)
        iota = torch.arange(w.k_max, dtype=torch.int32, device=self.dev).repeat(w.B, w.Hkv, 1).contiguous()
        Ks = [torch.zeros((w.B, w.Hkv, w.k_max, w.d), dtype=torch.int16, device=self.dev) for _ in range(D)]
        Vs = [torch.zeros_like(Ks[0]) for _ in range(D)]
        idx = [torch.empty((w.B, w.Hkv, w.k_max), dtype=torch.int32, device=self.dev) for _ in range(D)]
        main, fetch = self.stream, torch.cuda.Stream()
        selected = [torch.cuda.Event() for _ in range(NL)]
        fetched = [torch.cuda.Event() for _ in range(NL)]
        q, seq = self.q_steps[0], self.seq_steps[0]
        sel, gat, att = [], [], []
        for l in range(NL):
            c = l % self.n_layers
            sel.append(ctx.prepared("hata_select_step", q, None, self.W_H, self.codes_all[c], seq, self.kbud, w.B,
                                    False, idx[l % D], stream=main))
            gat.append(ctx.prepared("hata_gather_rows", self.K_all[c], self.V_all[c], idx[l % D], self.kbud, w.B,
                                    GATHER_WGS, Ks[l % D], Vs[l % D], stream=fetch))
            att.append(stage_ctx.prepared("hata_sparse_decode", q, Ks[l % D], Vs[l % D], iota, self.kbud, w.B,
                                          self.scale, self.out, self.out32, stream=main))

        def select_and_fetch(l):
            # (idx[l % D] and staging buffer l % D were last read by the fetch and the attention of
            # layer l - D, both complete before this selection runs on the main stream)
            sel[l]()
            selected[l].record(main)
            fetch.wait_event(selected[l])
            gat[l]()
            fetched[l].record(fetch)

        def token():
            for l in range(min(D - 1, NL)):
                select_and_fetch(l)
            for l in range(NL):
                if l + D - 1 < NL:
                    select_and_fetch(l + D - 1)
                main.wait_event(fetched[l])
                att[l]()

        token()
        torch.cuda.synchronize()
        staged_out = self.out32.clone()
        c_last = (NL - 1) % self.n_layers
        ctx.hata_sparse_decode(q, self.K_all[c_last], self.V_all[c_last], idx[(NL - 1) % D], self.kbud, w.B, self.scale,
                               self.out, self.out32, stream=main)
        torch.cuda.synchronize()
        same = bool(torch.equal(staged_out, self.out32))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(main)
        for _ in range(reps):
            token()
        e1.record(main)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e6 / (reps * NL)
        us = e0.elapsed_time(e1) * 1e3 / (reps * NL)
        ctx.hata_check(main)
        row_bytes = int(self.inp.k.sum()) * w.Hkv * 4 * w.d
        stage_ctx.close()
        return {"layers": NL, "tokens": reps, "staging_buffers": D, "us_per_layer": round(us, 2),
                "host_wall_us_per_layer": round(wall, 2), "bus_bytes_per_layer": row_bytes,
                "bus_GBps": round(row_bytes / (us * 1e-6) / 1e9, 1), "same_bits_as_zero_copy": same}

    # ---- the scoring stage alone (the largest stream of bytes of the step)
    def score(self, steps, warmup):
        qcodes_buf, scores_buf, _ = self.ctx.hata_step_buffers()
        calls = [self.ctx.prepared("hata_hamming_score", qcodes_buf, self.codes_all[l], self.seq_steps[0], self.w.B,
                                   scores_buf, stream=self.stream) for l in range(self.n_layers)]
        ms, _ = timed(lambda i: calls[i % self.n_layers](), steps, warmup, self.stream)
        return ms * 1e3

    # ---- the four stage entry points of Alg. 3, each alone (the step fuses them; these are the
    # stand-alone kernels behind hata_encode_query / hata_hamming_score / hata_topk / hata_sparse_decode)
    def stages(self, steps, warmup):
        w, ctx = self.w, self.ctx
        qcodes_buf, scores_buf, idx_buf = ctx.hata_step_buffers()
        seq, q = self.seq_steps[0], self.q_steps[0]
        enc = ctx.prepared("hata_encode_query", q, self.W_H, w.B, qcodes_buf, stream=self.stream)
        us_enc = timed(lambda i: enc(), steps, warmup, self.stream)[0] * 1e3
        us_score = self.score(steps, warmup)   # leaves the scores of the last layer's codes (all layers hold the same codes)
        topk = ctx.prepared("hata_topk", scores_buf, seq, self.kbud, w.B, idx_buf, stream=self.stream)
        us_topk = timed(lambda i: topk(), steps, warmup, self.stream)[0] * 1e3
        att = [ctx.prepared("hata_sparse_decode", q, self.K_all[l], self.V_all[l], idx_buf, self.kbud, w.B, self.scale,
                            self.out, self.out32, stream=self.stream) for l in range(self.n_layers)]
        us_att = timed(lambda i: att[i % self.n_layers](), steps, warmup, self.stream)[0] * 1e3
        rows = int(self.np.minimum(self.inp.k, self.inp.seq_len).sum()) * w.Hkv
        att_bytes = rows * 2 * w.d * 2 + 2 * w.B * w.Hq * w.d * 2
        score_bytes = self.code_bytes

        def bw(nbytes, us):
            return {"us": round(us, 3), "algorithmic_bytes": nbytes, "GBps": round(nbytes / (us * 1e-6) / 1e9, 1),
                    "frac": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}

        return {"encode_query_us": round(us_enc, 3), "hamming_score": bw(score_bytes, us_score),
                "topk_us": round(us_topk, 3), "sparse_decode": bw(att_bytes, us_att)}

    # ---- dense decode over the whole cache (Eq. 1): the comparison baseline, same shapes
    def dense(self, steps):
        calls = [self.ctx.prepared("hata_dense_decode", self.q_steps[0], self.K_all[l], self.V_all[l],
                                   self.seq_steps[0], self.w.B, self.scale, self.out, self.out32, stream=self.stream)
                 for l in range(self.n_layers)]
        ms, _ = timed(lambda i: calls[i % self.n_layers](), 5 if self.kv_host else max(20, steps // 8),
                      1 if self.kv_host else 5, self.stream)
        return ms * 1e3

    # ---- parity of one step against the oracle, the oracle timed on this machine's host cores
    def oracle(self, cpu_seconds, check_bulk_codes):
        """One step on the ORACLE's own key codes, compared stage by stage; the oracle's step timed.
        check_bulk_codes: also compare the GPU's bulk key codes (layer 0) with the oracle's and count
        the projections inside the |projection| < 1e-4 band and the bits that differ there."""
        from oracle import hata_oracle as O
        np, torch, w, inp, ctx = self.np, self.torch, self.w, self.inp, self.ctx
        seq0 = inp.seq_len + (1 if w.append_steps else 0)
        codes_o, near = O.encode_keys_batch(inp.K, inp.W_H, np.zeros(w.B, np.int32), seq0, bulk=True)
        band = None
        if check_bulk_codes:
            got = self.codes_all[0].cpu().numpy().view(np.uint32)
            diff = got ^ codes_o
            for b in range(w.B):  # rows past the oracle's range (later appended rows) are not compared
                diff[b, :, int(seq0[b]):] = 0
            band = {"projections": int(seq0.sum()) * w.Hkv * w.r,
                    "in_band": int(np.unpackbits(near.view(np.uint8)).sum()),
                    "bits_differ_in_band": int(np.unpackbits((diff & near).view(np.uint8)).sum()),
                    "bits_differ_outside_band": int(np.unpackbits((diff & ~near).view(np.uint8)).sum())}
        q0 = inp.q(0)
        codes_before = codes_o.copy()
        for b in range(w.B):  # the appended row's code is written by the step itself
            codes_before[b, :, int(seq0[b]) - 1] = 0
        t0 = time.perf_counter()
        ref = O.decode_step(q0, inp.K, inp.V, inp.W_H, codes_o, seq0, inp.k, w.k_max, self.scale, append=True)
        t1 = time.perf_counter() - t0
        reps = int(max(1, min(5000, cpu_seconds / max(t1, 1e-6))))
        t0 = time.perf_counter()
        for _ in range(reps):
            O.decode_step(q0, inp.K, inp.V, inp.W_H, codes_o, seq0, inp.k, w.k_max, self.scale, append=True)
        tn = (time.perf_counter() - t0) / reps
        cpu = {"value": round(tn * 1e6, 1), "unit": "us/step", "cores": O.num_threads(), "kind": "oracle",
               "sample": f"{reps} full decode steps of {w.name} (all {w.B * w.Hkv} units, layer 0, step 0)"}
        _, near_q = O.encode_query_batch(q0, inp.W_H)
        codes_dev = dev_bits(codes_before, self.dev)
        ctx.hata_decode_step(self.q_steps[0], self.K_all[0], self.V_all[0], self.W_H, codes_dev, self.seq_steps[0],
                             self.kbud, w.B, True, self.scale, self.out, self.out32, self.stream)
        torch.cuda.synchronize()
        qc, _, ix = ctx.hata_step_buffers()
        err = np.abs(self.out32.cpu().numpy().astype(np.float64) - ref["out"])
        qdiff = qc.cpu().numpy().view(np.uint32) ^ ref["qcodes"]
        parity = {"appended_code_equal": bool(np.array_equal(codes_dev.cpu().numpy().view(np.uint32), codes_o)),
                  "qcodes_equal": bool(not np.any(qdiff)),
                  "idx_equal": bool(np.array_equal(ix.cpu().numpy(), ref["idx"])),
                  "attn_within_tol": bool(np.all(err <= 2e-3 + 1e-3 * np.abs(ref["out"]))),
                  "max_abs_err": float(err.max()),
                  "query_projections_in_band": int(np.unpackbits(near_q.view(np.uint8)).sum()),
                  "query_bits_differ": int(np.unpackbits(qdiff.view(np.uint8)).sum())}
        return cpu, parity, band

    # ---- the step on the paged layout (last: the caches are re-laid in place, page order random)
    def paged(self, P, steps, warmup):
        torch, w, ctx = self.torch, self.w, self.ctx
        ctx.hata_decode_step(self.q_steps[0], self.K_all[0], self.V_all[0], self.W_H, self.codes_all[0],
                             self.seq_steps[0], self.kbud, w.B, True, self.scale, self.out, self.out32, self.stream)
        torch.cuda.synchronize()
        ref_out = self.out32.clone()  # the same step on the contiguous layout, for a bit-for-bit comparison
        nb = w.L_cap // P
        n_pages = w.B * nb
        perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(1))  # page of block (b, blk)
        table = perm.view(w.B, nb).to(torch.int32).to(self.dev)
        inv = torch.argsort(perm).to(self.dev)                                      # block held by page p

        def to_pool(t, last):  # [B, Hkv, L_cap, last] -> [n_pages, Hkv, P, last] in the same memory
            blocks = t.view(w.B, w.Hkv, nb, P, last).permute(0, 2, 1, 3, 4).reshape(n_pages, w.Hkv, P, last)
            t.view(n_pages, w.Hkv, P, last).copy_(blocks.index_select(0, inv))

        for l in range(self.n_layers):
            to_pool(self.K_all[l], w.d)
            to_pool(self.V_all[l], w.d)
            to_pool(self.codes_all[l], w.W)
        calls = []
        for i in range(self.n_combo):
            l, t = i % self.n_layers, i % self.n_step_variants
            calls.append(ctx.prepared("hata_decode_step_paged", self.q_steps[t % len(self.q_steps)], self.K_all[l],
                                      self.V_all[l], self.W_H, self.codes_all[l], table, nb, P, n_pages,
                                      self.seq_steps[t], self.kbud, w.B, True, self.scale, self.out, self.out32,
                                      stream=self.stream))
        ctx.hata_decode_step_paged(self.q_steps[0], self.K_all[0], self.V_all[0], self.W_H, self.codes_all[0], table,
                                   nb, P, n_pages, self.seq_steps[0], self.kbud, w.B, True, self.scale, self.out,
                                   self.out32, self.stream)
        torch.cuda.synchronize()
        same = bool(torch.equal(ref_out, self.out32))
        ms, _ = timed(lambda i: calls[i % self.n_combo](), steps, warmup, self.stream)
        ctx.hata_check(self.stream)
        return {"page_rows": P, "n_pages": n_pages, "us_per_step": round(ms * 1e3, 3),
                "same_bits_as_contiguous": same}

    # checkpoints of decode_step_coop_kernel (slot = number % 32 of the HATA_TRACE_AT calls in csrc/)
    PHASES = [(39, "kernel start"), (40, "sequence length known"), (50, "query codes collected"),
              (41, "chunk scored"), (42, "histogram stores issued"), (43, "histogram stores complete"),
              (44, "arrived at the unit"), (51, "last arriver: threshold search starts"),
              (26, "last arriver: unit histogram loaded and scanned"), (27, "last arriver: threshold known"),
              (28, "last arriver: per-chunk counts"), (29, "last arriver: records published"),
              (45, "record picked up"), (46, "compaction done"), (47, "attention over own rows done"),
              (48, "partial emitted"), (54, "merge done (merging workgroups)")]

    def phase_trace(self, launches=16, repeats=10):
        """Timeline of the single-launch step from a tuning build (-DHATA_TRACE): back-to-back
        launches over the rotated layers; every workgroup stamps the wall clock at each checkpoint
        into its own row, the last launch's stamps stay.  Returns, per checkpoint, the time after
        the first workgroup's start at which the first / 10 % / median / 90 % / last workgroup
        passed it (median over `repeats` traced launches), in us."""
        import ctypes
        from paper_2506_02572_amd import hata
        np, torch, w, ctx = self.np, self.torch, self.w, self.ctx
        lib = hata.load_library()
        if not hasattr(lib, "hata_debug_trace"):
            raise SystemExit("bench.py --phase-trace needs a tuning build: python paper_2506_02572_amd/build.py --trace")
        NW = 4096
        buf = (ctypes.c_ulonglong * (NW * 32))()
        lib.hata_debug_trace_reset()
        rows = []
        for it in range(repeats + 2):
            for j in range(launches):
                l = (it + j) % self.n_layers
                ctx.hata_decode_step(self.q_steps[0], self.K_all[l], self.V_all[l], self.W_H, self.codes_all[l],
                                     self.seq_steps[0], self.kbud, w.B, True, self.scale, self.out, self.out32,
                                     self.stream)
            torch.cuda.synchronize()
            lib.hata_debug_trace(buf)
            rows.append(np.frombuffer(buf, dtype=np.uint64).reshape(NW, 32).astype(np.float64).copy())
        ctx.hata_check(self.stream)
        table = []
        for slot, name in self.PHASES:
            acc, n = [], 0
            for t in rows[2:]:
                e = t[:, 39 & 31]
                newest = e.max()
                base = e[e >= newest - 200 * 100].min()  # stamps of the last launch: within 200 us of the newest start
                v = t[:, slot & 31]
                v = v[v >= base]
                if v.size == 0:
                    continue
                n = int(v.size)
                acc.append([(x - base) / 100.0 for x in (v.min(), np.percentile(v, 10), np.median(v),
                                                         np.percentile(v, 90), v.max())])
            if acc:
                a = np.median(np.array(acc), axis=0)
                table.append({"checkpoint": name, "workgroups": n, "first": round(float(a[0]), 2),
                              "p10": round(float(a[1]), 2), "median": round(float(a[2]), 2),
                              "p90": round(float(a[3]), 2), "last": round(float(a[4]), 2)})
        return {"phase_trace": True, "workload": w.name, "unit": "us after the first workgroup's start",
                "launches_per_sample": launches, "samples": repeats, "checkpoints": table}

    def pmc_probe(self):
        """A plain copy of known size (reads and writes COPY_BYTES each) calibrates the counters; then
        the decode step and the scoring launch, the same calls the timed legs issue."""
        torch, w, ctx = self.torch, self.w, self.ctx
        COPY_BYTES = 256 << 20
        src = torch.empty(COPY_BYTES // 4, dtype=torch.int32, device=self.dev).fill_(1)
        dst = torch.empty_like(src)
        qcodes_buf, scores_buf, _ = ctx.hata_step_buffers()
        ctx.hata_encode_query(self.q_steps[0], self.W_H, w.B, qcodes_buf, self.stream)
        torch.cuda.synchronize()
        for i in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        for i in range(40):
            ctx.hata_hamming_score(qcodes_buf, self.codes_all[i % self.n_layers], self.seq_steps[0], w.B, scores_buf,
                                   self.stream)
        torch.cuda.synchronize()
        for i in range(40):
            l = i % self.n_layers
            ctx.hata_decode_step(self.q_steps[0], self.K_all[l], self.V_all[l], self.W_H, self.codes_all[l],
                                 self.seq_steps[0], self.kbud, w.B, True, self.scale, self.out, self.out32, self.stream)
        ctx.hata_check(self.stream)
        return {"pmc_probe": True, "workload": w.name, "copy_bytes_each_way": COPY_BYTES,
                "score_code_bytes": self.code_bytes, "score_write_bytes": self.code_bytes // (w.r // 8) * 2,
                "step_algorithmic_bytes": self.alg_bytes, "step_launches": ctx.hata_step_plan(w.B)[0]}


def overlap_probe(torch, gib=1, reps=5):
    """Times hata_probe_mfma_stream in its three modes on bf16 N(0,1) data: the matrix-core loop alone
    (sized to take about as long as the read), the read alone, and both in one launch."""
    from paper_2506_02572_amd import hata
    dev = torch.device("cuda:0")
    buf = torch.randn((gib << 30) // 2, dtype=torch.bfloat16, device=dev).view(torch.int16)
    stream = torch.cuda.current_stream()

    def run(mode, iters):
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            hata.hata_probe_mfma_stream(buf, iters, mode, stream)
            e1.record(stream)
            e1.synchronize()
            t = e0.elapsed_time(e1) * 1e3
            best = t if best is None else min(best, t)
        return best

    us_mem = run(2, 0)
    iters = 256
    us_mfma = run(1, iters)
    iters = max(16, int(iters * us_mem / us_mfma))  # a matrix-core loop about as long as the read
    us_mfma = run(1, iters)
    us_both = run(3, iters)
    n_mfma = 16 * iters  # per wave = per SIMD (one matrix-core wave per SIMD on 256 CUs)
    return {"overlap_probe": True, "bytes_read": buf.numel() * 2, "mfma_per_simd": n_mfma,
            "stream_only_us": round(us_mem, 1), "stream_only_TBps": round(buf.numel() * 2 / us_mem / 1e6, 2),
            "mfma_only_us": round(us_mfma, 1),
            "mfma_only_TFLOPs": round(2.0 * 32 * 32 * 16 * n_mfma * 1024 / us_mfma / 1e6, 1),
            "both_us": round(us_both, 1), "sum_of_parts_us": round(us_mem + us_mfma, 1),
            "max_of_parts_us": round(max(us_mem, us_mfma), 1)}


def train_leg(torch, dev, w, W_H, stream):
    """Learning-to-hash training step (Sec. 3.1 / App. B): one SGD step on one head's W_H from a
    32K-triplet chunk (the chunk size of App. B.2)."""
    from paper_2506_02572_amd import synth
    from paper_2506_02572_amd import train as htrain
    n_tr = 32768
    tctx = htrain.TrainContext(w.d, w.r, n_tr)
    Qt = dev_bits(synth.train_vectors(n_tr, tensor_id=synth.TID_Q), dev)
    Kt = dev_bits(synth.train_vectors(n_tr, tensor_id=synth.TID_K), dev)
    st = torch.full((n_tr,), -1.0, dtype=torch.float32, device=dev)
    st[::10] = 5.0
    Wt = W_H[0].to(torch.float32).contiguous().clone()
    vt = torch.zeros_like(Wt)
    hp = htrain.default_hparams(n_tr)
    ms_tr, _ = timed(lambda i: tctx.hata_train_step(Qt, Kt, st, n_tr, Wt, vt, hp, None, None, stream), 50, 5, stream)
    flop = 4 * 2.0 * n_tr * w.d * w.r  # two projections + two weight-gradient contractions
    leg = {"triplets": n_tr, "r": w.r, "us_per_step": round(ms_tr * 1e3, 1),
           "TFLOPs": round(flop / (ms_tr * 1e-3) / 1e12, 1),
           "mfma_issue_TFLOPs": round((3 * 3 + 2 * 3) / 4 * flop / (ms_tr * 1e-3) / 1e12, 1), "launches": 6}
    tctx.close()
    return leg


def per_config_entry(name, args):
    """Configuration `name` at full size: steady-state step time, roofline fraction, the dense
    comparison (measured and at HBM peak) and parity of one step against the oracle."""
    b = Bench(name, args)
    w = b.w
    b.encode_keys()
    us_step, _ = b.step(PER_CONFIG_STEPS, PER_CONFIG_WARMUP)
    n_launches, chunk, n_chunks, n_sub = b.plan()
    stages = b.stages(PER_CONFIG_STEPS, PER_CONFIG_WARMUP)
    us_score = stages["hamming_score"]["us"]
    us_dense = b.dense(PER_CONFIG_STEPS)
    cpu, parity, band = b.oracle(min(args.cpu_seconds, 2.0), True)
    gbps = b.alg_bytes / (us_step * 1e-6) / 1e9
    traffic = HBM_TRAFFIC_BYTES.get(w.name, {}).get("step")
    ideal_dense = w.dense_bytes(1 if w.append_steps else 0) / (HBM_PEAK_GBPS * 1e9) * 1e6
    e = {"workload": w.name, "us_per_step": round(us_step, 3), "steps": PER_CONFIG_STEPS, "warmup": PER_CONFIG_WARMUP,
         "layers_rotated": b.n_layers, "launches_per_step": n_sub if n_launches == 1 else n_launches,
         "chunk": chunk, "chunks_per_unit": n_chunks,
         "algorithmic_bytes_per_step": b.alg_bytes, "achieved_GBps": round(gbps, 1),
         "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
         "traffic_over_algorithmic": None if traffic is None else round(traffic / b.alg_bytes, 3),
         "score_stage_us": round(us_score, 3), "score_stage_GBps": round(b.code_bytes / (us_score * 1e-6) / 1e9, 1),
         "stages_alone": stages,
         "dense_decode_us": round(us_dense, 2), "ideal_dense_us": round(ideal_dense, 2),
         "speedup_vs_dense": round(us_dense / us_step, 2), "speedup_vs_ideal_dense": round(ideal_dense / us_step, 2),
         "parity": parity, "bulk_key_codes": band, "oracle_us_per_step": cpu["value"], "oracle_cores": cpu["cores"]}
    b.close()
    return e


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_02572_amd import hata, synth  # noqa: F401

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HATA path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.overlap_probe:
        print(json.dumps(overlap_probe(torch)))
        return
    default_run = args.workload == "cfg2" and not (args.kv_host or args.paged or args.pmc_probe or args.step_mode or args.chunk)
    b = Bench(args.workload, args, layers=args.layers, kv_host=args.kv_host, step_mode=args.step_mode)
    w = b.w
    enc_leg = b.encode_keys()
    if args.pmc_probe:
        print(json.dumps(b.pmc_probe()))
        b.close()
        return
    if args.phase_trace:
        print(json.dumps(b.phase_trace()))
        b.close()
        return
    fill_leg = b.prefill_write()
    us_step, us_wall = b.step(args.steps, args.warmup)
    n_launches, plan_chunk, plan_n_chunks, n_sub = b.plan()
    graph_leg = b.graph_of_layers(args.graph_layers, args.steps) if args.graph_layers > 0 and not args.kv_host else None
    prefetch_leg = b.kv_host_prefetch(32, max(3, args.steps // 64)) if args.kv_host else None
    stages_alone = None if args.kv_host else b.stages(args.steps, args.warmup)
    us_score = stages_alone["hamming_score"]["us"] if stages_alone else b.score(args.steps, args.warmup)
    score_gbps = b.code_bytes / (us_score * 1e-6) / 1e9
    dense_us = None if args.no_dense else b.dense(args.steps)
    tr_leg = None if args.no_train else train_leg(torch, b.dev, w, b.W_H, b.stream)
    cpu = parity = None
    if not args.no_cpu_baseline:
        cpu, parity, _ = b.oracle(args.cpu_seconds, False)
    paged_leg = None
    if args.paged and not args.kv_host and w.L_cap % args.paged == 0 and n_launches == 1:
        paged_leg = b.paged(args.paged, args.steps, args.warmup)

    traffic = HBM_TRAFFIC_BYTES.get(w.name, {})
    step_gbps = b.alg_bytes / (us_step * 1e-6) / 1e9
    score_stage = {"kernel": "score_kernel (hata_hamming_score)", "achieved": round(score_gbps, 1),
                   "unit": "GB/s", "frac": round(score_gbps / HBM_PEAK_GBPS, 4),
                   "traffic": traffic.get("score"), "algorithmic_bytes_per_launch": b.code_bytes,
                   "avg_launch_us": round(us_score, 3)}
    if n_launches == 1:
        # the whole step is ONE kernel (launched once per slice of a batch too large to be resident at
        # once): it is the dominant kernel, its launches are the step
        roofline = {"bound": "hbm", "kernel": "decode_step_coop_kernel (hata_decode_step: the whole step in one launch)",
                    "achieved": round(step_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(step_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic.get("step"),
                    "traffic_source": HBM_TRAFFIC_SOURCE + " (a constant of that profile's build, not of this run)",
                    "algorithmic_bytes_per_launch": b.alg_bytes // n_sub, "avg_launch_us": round(us_step / n_sub, 3)}
    else:
        roofline = dict(score_stage, bound="hbm", peak=HBM_PEAK_GBPS)
    ideal_dense = w.dense_bytes(1 if w.append_steps else 0) / (HBM_PEAK_GBPS * 1e9) * 1e6
    result = {
        "metric": "hata_decode_attention_us_per_step",
        "value": round(us_step, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(us_step * 1e-3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 K/V/q with fp32 accumulate; u32 codes; fp64 query/append projection",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d, "r": w.r,
                   "L": list(w.L) if len(set(w.L)) > 1 else w.L[0],
                   "k": list(w.k) if len(set(w.k)) > 1 else w.k[0],
                   "layers_rotated": b.n_layers, "first_pass_untimed": b.n_combo, "append_per_step": True,
                   "kv_cache": "pinned host memory (rows gathered over the bus)" if args.kv_host else "HBM",
                   "launches_per_step": n_sub if n_launches == 1 else n_launches, "step_mode": args.step_mode,
                   "chunk": plan_chunk,
                   "chunks_per_unit": plan_n_chunks},
        "achieved_GBps": round(step_gbps, 1),
        "algorithmic_bytes_per_step": b.alg_bytes,
        "step_roofline_frac": round(step_gbps / HBM_PEAK_GBPS, 4),
        "host_wall_us_per_step": round(us_wall, 3),
        "roofline": roofline,
        "score_stage": score_stage,
        "stages_alone": stages_alone,
        "encode_keys_bulk": enc_leg,
        "prefill_write": fill_leg,
        "paged_step": paged_leg,
        "graph_of_layers": graph_leg,
        "kv_host_prefetch": prefetch_leg,
        "dense_decode_us": None if dense_us is None else round(dense_us, 2),
        "ideal_dense_us": round(ideal_dense, 2),
        "speedup_vs_dense": None if dense_us is None else round(dense_us / us_step, 2),
        "speedup_vs_ideal_dense": round(ideal_dense / us_step, 2),
        "train_step": tr_leg,
        "cpu_baseline": cpu,
        "parity": parity,
    }
    b.close()
    del b
    if default_run and not args.no_per_config:
        # configurations 2-5 at full size, each in steady state (the headline above takes the
        # caller's --steps / --warmup, which may be short)
        result["per_config"] = [per_config_entry(n, args) for n in ("cfg2", "cfg3", "cfg4", "cfg5")]
        # a serving-size batch, beyond the batch range the benchmark's metric names (B = 1-16): same fields
        result["larger_batch"] = [per_config_entry("b32_32k", args)]
    print(json.dumps(result))


if __name__ == "__main__":
    main()
