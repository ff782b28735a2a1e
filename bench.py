#!/usr/bin/env python3
"""Benchmark of the W4A8 linear path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: the
linear stack of one LLaMA-13B-shaped decoder layer at M = 1024 tokens (the
context-decoding case), i.e. four per-token activation quantisations (the last
one fused with the SiLU*up glue in front of the down projection) and the four
W4A8 GEMMs with fused dequantisation (QKV 15360x5120, O 5120x5120, gate+up
27648x5120, down 5120x13824): eight kernel launches on one stream.  `value` is the integer GEMM
work of a step (2*M*N*K summed over the four linears) divided by the step time.

The same run also reports the decode side of the metric (M = 1, 4, 16 on the same
four shapes, weights rotated through more than the last-level cache so every byte
comes from HBM), a roofline object for the dominant kernel, the layer stack at
M = 1 .. 2048 replayed from a HIP graph (layer time and GEMM share), the per-GEMM
ratios of the W8A8 comparison variant and of the two ablation variants (unsigned
nibble storage, fine-grained group scales) to W4A8, and the CPU oracle's
throughput on a bounded sample of the workload.  Every GEMM of the run reads the
one tiled copy of the weights, whatever its M.

All inputs are seeded synthetic tensors generated on the host and resident in
HBM before the timed region starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix peak, published (5.0 POP/s)
LAST_LEVEL_CACHE_BYTES = 256 << 20


def gemm_bytes(M, N, K):
    """Algorithmic HBM bytes of one W4A8 GEMM: packed weights + int8 activations + both scale vectors + fp16 output."""
    return N * K // 2 + M * K + 4 * M + 4 * N + 2 * M * N


def gemm_ops(M, N, K):
    return 2 * M * N * K


COPY_CALIBRATION_BYTES = 256 << 20
# L2 fill + write-back bytes per GEMM launch of the default workload (mean over its four linears), from the two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) summarised in profiles/gemm_prefill_tiled_13b_counters.md, each scaled by
# what the counter reads for the 256 MiB copy of --copy-calibration.  Counters cannot be read from inside this
# process, so the figure is carried here and reported only for the workload it was measured on.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {("13b", 1024): 139.5e6}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--M", type=int, default=1024, help="tokens per step (default: the 1024-token context)")
    ap.add_argument("--no-decode", action="store_true", help="skip the M=1,4,16 weight-streaming measurements")
    ap.add_argument("--no-layer-stack", action="store_true", help="skip the graph-replayed layer stack at M=1..2048")
    ap.add_argument("--no-w8a8", action="store_true", help="skip the per-GEMM W4A8 / W8A8 comparison")
    ap.add_argument("--no-achievable", action="store_true", help="skip the probes of achievable HBM and MFMA rates")
    ap.add_argument("--no-medium-m", action="store_true", help="skip the four linears at M = 32 .. 512")
    ap.add_argument("--no-table5", action="store_true", help="skip the GEMM sizes of the paper's Table 5")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy three times: the dispatch of known size against which "
                         "hardware traffic counters are scaled")
    return ap.parse_args()


# One copy of the weights, in the tiled layout, serves every M: the library's tiled entry runs the weight-streaming
# kernels up to M = 16 and the large-M kernel above, with K cut into slices where its tiles alone would not fill the chip.


def prepare_weights(torch, w4a8, synth, model="13b"):
    """Offline weight preparation, on the GPU: quantise and pack, then reorder into the tiled array (the only copy that
    is kept).  Returns name -> (wt, s_w)."""
    out = {}
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).to("cuda")
        wp, s_w = w4a8.w4a8_quantize_weights(w)
        out[name] = (w4a8.w4a8_tile_weights(wp), s_w)
        del w, wp
    return out


class LayerStack:
    """Device buffers of one 13B-shaped decoder layer's linears and the eight launches of a step."""

    def __init__(self, torch, w4a8, synth, M, weights, model="13b"):
        self.torch, self.w4a8, self.M = torch, w4a8, M
        self.shapes = synth.LLAMA_SHAPES[model]
        dev = "cuda"
        self.wp = {k: v[0] for k, v in weights.items()}
        self.s_w = {k: v[1] for k, v in weights.items()}
        H = self.shapes["qkv"][1]
        I = self.shapes["down"][1]
        # fp16 hidden states enter the stack; attention itself is not modelled: the Q slice of the QKV output stands in
        # for its result, and every later linear is fed by the one before it, so the eight launches form one chain
        self.h = torch.from_numpy(synth.activations_fp16(M, H, config_id=3, tag=1)).to(dev)
        e = lambda *s, dt: torch.empty(s, dtype=dt, device=dev)
        self.xq_h, self.sa_h = e(M, H, dt=torch.int8), e(M, dt=torch.float32)
        self.xq_i, self.sa_i = e(M, I, dt=torch.int8), e(M, dt=torch.float32)
        self.out = {name: e(M, N, dt=torch.float16) for name, (N, K) in self.shapes.items()}
        # scratch for the GEMMs whose K the library cuts into slices (medium M; empty where it does not)
        self.ws = {name: e(max(16, w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)), dt=torch.uint8)
                   for name, (N, K) in self.shapes.items()}
        self.gemm_events = []   # (name, start, stop) around GEMM launches, filled when record=True
        # the eight launches with their arguments marshalled once: the timed loop then spends its host time in the
        # library, not in Python
        b = w4a8.bound_call
        self.quant = {"qkv": b("w4a8_quantize_act", self.h, self.xq_h, self.sa_h, M, H),
                      "o": b("w4a8_quantize_act_strided", self.out["qkv"], self.shapes["qkv"][0], self.xq_h, self.sa_h, M, H),
                      "gate_up": b("w4a8_quantize_act", self.out["o"], self.xq_h, self.sa_h, M, H),
                      "down": b("w4a8_silu_mul_quantize", self.out["gate_up"], self.xq_i, self.sa_i, M, I)}
        self.gemm = {}
        for name, (N, K) in self.shapes.items():
            xq, sa = (self.xq_i, self.sa_i) if name == "down" else (self.xq_h, self.sa_h)
            self.gemm[name] = b("w4a8_gemm_tiled_splitk", xq, sa, self.wp[name], self.s_w[name], self.out[name], M, N, K,
                                0, 0, self.ws[name], self.ws[name].numel())

    def _gemm(self, name, record=False):
        if record:
            t = self.torch
            a, b = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
            a.record()
        self.gemm[name]()
        if record:
            b.record()
            self.gemm_events.append((name, a, b))

    def step(self, record=None):
        """One pass over the eight launches; `record` names the GEMM to bracket with timing events (None: none)."""
        for name in ("qkv", "o", "gate_up", "down"):
            self.quant[name]()           # "down": SiLU*up and its quantiser in one pass
            self._gemm(name, record == name)

    def gemms_only(self):
        for name in ("qkv", "o", "gate_up", "down"):
            self.gemm[name]()

    def ops_per_step(self):
        return sum(gemm_ops(self.M, N, K) for N, K in self.shapes.values())


def time_layer_stack(torch, w4a8, synth, weights, Ms=(1, 16, 64, 128, 1024, 2048), steps_per_graph=8, replays=6):
    """The decoder layer's linear stack at several M, replayed from a HIP graph (what a serving loop does; at small M
    the eight launches would otherwise be timed by the interpreter).  Layer time = graph time / steps; the GEMM share
    is the time of a second graph that holds only the four GEMMs, over the layer time.  One layer's weights (158 MB)
    stay resident in the last-level cache across replays: the small-M rows are a warm-cache figure, the HBM-bound
    figure is the `decode` list."""
    rows = []
    for M in Ms:
        stack = LayerStack(torch, w4a8, synth, M, weights)
        for _ in range(3):
            stack.step()
        torch.cuda.synchronize()
        times = {}
        for what, fn in (("layer", stack.step), ("gemms", stack.gemms_only)):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(steps_per_graph):
                    fn()
            graph.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(replays):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            times[what] = a.elapsed_time(b) * 1e3 / (replays * steps_per_graph)
            del graph
        rows.append({"M": M, "layer_us": round(times["layer"], 2), "gemm_us": round(times["gemms"], 2),
                     "gemm_share": round(times["gemms"] / times["layer"], 4),
                     "TOPS": round(stack.ops_per_step() / times["layer"] / 1e6, 2),
                     "weights": "tiled"})
        del stack
        torch.cuda.empty_cache()
    return rows


def time_decode(torch, w4a8, synth, model="13b", Ms=(1, 4, 16), iters=5):
    """Weight-streaming GEMMs: every launch reads a different copy of the weights, the copies together
    exceeding the last-level cache three times, so the weights come from HBM.  Per-launch time is the
    average over back-to-back batches replayed from a HIP graph, between two events on the launch stream
    (the gaps between dependent kernels are included)."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).cuda()
        wp, s_w = w4a8.w4a8_quantize_weights(w)
        wt = w4a8.w4a8_tile_weights(wp)   # the same array the large-M kernel reads
        del w, wp
        wbytes = N * K // 2
        copies = max(2, -(-3 * LAST_LEVEL_CACHE_BYTES // wbytes) + 1)
        wps = [wt] + [wt.clone() for _ in range(copies - 1)]
        for M in Ms:
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            for i in range(min(copies, 4)):
                w4a8.w4a8_gemm_tiled(xq, s_a, wps[i], s_w, out=out)
            torch.cuda.synchronize()
            # One graph holds a back-to-back batch of launches (a decode loop is replayed from a graph as well; launching
            # each 5-15 us kernel from Python would time the interpreter, not the GPU).
            n = max(copies, 24)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(n):
                    w4a8.w4a8_gemm_tiled(xq, s_a, wps[i % copies], s_w, out=out)
            graph.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / (n * iters)
            del graph
            by = gemm_bytes(M, N, K)
            rows.append({"linear": name, "M": M, "N": N, "K": K, "us": round(us, 3),
                         "GBps": round(by / us / 1e3, 1), "hbm_frac": round(by / us / 1e3 / HBM_PEAK_GBS, 4),
                         "weight_copies": copies})
        del wps, wt
        torch.cuda.empty_cache()
    return rows


def time_achievable(torch, w4a8):
    """What the chip sustains, measured with the library's two probes, to set the datasheet fractions against: a
    read-only streaming reduction over 2 GiB (eight times the last-level cache, so every pass comes from HBM) and over
    cold pieces of the sizes of the 13B weight matrices, and a register-resident int8 MFMA loop on constant and on
    random operands, long (about 2 ms) and as short as the GEMM kernels (about 50 us)."""
    out = {}
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    big.fill_(7)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps   # seconds per call

    out["hbm_read_GBps"] = round(big.numel() / timed(lambda: w4a8.w4a8_probe_stream_read(big, sink), 5) / 1e9, 1)
    by_size = {}
    for mb in (13, 39, 71):
        size = mb * 1000 * 1000 // 4096 * 4096
        n = big.numel() // size            # consecutive pieces: each is read once per pass over the 2 GiB
        pieces = [big[i * size:(i + 1) * size] for i in range(n)]
        graph = torch.cuda.CUDAGraph()
        w4a8.w4a8_probe_stream_read(pieces[0], sink)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            for piece in pieces:
                w4a8.w4a8_probe_stream_read(piece, sink)
        by_size[f"{mb}MB"] = round(size * n / timed(graph.replay, 3) / 1e9, 1)
        del graph
    out["hbm_read_GBps_cold_pieces"] = by_size
    del big
    torch.cuda.empty_cache()
    mfma = {}
    for label, iters, pattern, reps in (("constant_2ms", 8000, 0, 3), ("random_2ms", 8000, 1, 3), ("random_50us", 200, 1, 40)):
        ops = [0]

        def run():
            ops[0] = w4a8.w4a8_probe_mfma_int8(sink, iters, pattern)
        t = timed(run, reps)
        mfma[label] = round(ops[0] / t / 1e12, 1)
    out["int8_mfma_TOPS"] = mfma
    return out


def time_medium_m(torch, w4a8, synth, model="13b", Ms=(32, 64, 128, 256, 512), iters=4):
    """Between token generation and context decoding: the four linears at M = 32 .. 512 from cold weights (rotating
    copies as in time_decode), through the one-copy entry with its K slices.  Each row is set against the larger of
    the two roofline times (bytes at the HBM peak, operations at the int8 MFMA peak)."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).cuda()
        wp, s_w = w4a8.w4a8_quantize_weights(w)
        wt = w4a8.w4a8_tile_weights(wp)
        del w, wp
        copies = max(2, -(-3 * LAST_LEVEL_CACHE_BYTES // wt.numel()) + 1)
        wts = [wt] + [wt.clone() for _ in range(copies - 1)]
        for M in Ms:
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            need = w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)
            ws = torch.empty((max(16, need),), dtype=torch.uint8, device="cuda")
            call = lambda i: w4a8.w4a8_gemm_tiled_splitk(xq, s_a, wts[i % copies], s_w, ws=ws, out=out)
            call(0)
            torch.cuda.synchronize()
            n = max(copies, 16)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(n):
                    call(i)
            graph.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / (n * iters)
            del graph
            roof_us = max(gemm_bytes(M, N, K) / HBM_PEAK_GBS / 1e3, gemm_ops(M, N, K) / INT8_PEAK_TOPS / 1e6)
            rows.append({"linear": name, "M": M, "us": round(us, 2), "TOPS": round(gemm_ops(M, N, K) / us / 1e6, 1),
                         "GBps": round(gemm_bytes(M, N, K) / us / 1e3, 1), "roofline_frac": round(roof_us / us, 4),
                         "k_slices": need // (M * N * 4) if need else 1})
        del wts, wt
        torch.cuda.empty_cache()
    return rows


# Latencies the paper prints for its own kernel on an A100-80G (Table 5; unit read as ms), by (M, N, K): context only.
PAPER_TABLE5_A100_MS = {(1024, 4096, 4096): 0.121, (1024, 1024, 8192): 0.073, (1024, 11088, 4096): 0.279,
                        (1024, 5120, 5120): 0.158, (1, 4096, 4096): 0.012, (1, 1024, 8192): 0.019,
                        (1, 11088, 4096): 0.016, (1, 5120, 5120): 0.014}


def time_paper_table5(torch, w4a8, synth, iters=5):
    """The single-GEMM sizes of the paper's Table 5 (M = 1 and 1024, N = 11088 as printed there) through the one-copy
    tiled entry, every launch on a different weight copy (copies exceed the last-level cache three times), batches
    replayed from a HIP graph.  The paper's A100 figures ride along as context, not as a baseline for this chip."""
    rows = []
    for N, K in synth.PAPER_TABLE5_SHAPES:
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=6)).cuda()
        wp, s_w = w4a8.w4a8_quantize_weights(w)
        wt = w4a8.w4a8_tile_weights(wp)
        del w, wp
        copies = max(2, -(-3 * LAST_LEVEL_CACHE_BYTES // wt.numel()) + 1)
        wts = [wt] + [wt.clone() for _ in range(copies - 1)]
        for M in (1, 1024):
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=6, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            ws = torch.empty((max(16, w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)),), dtype=torch.uint8, device="cuda")
            call = lambda i: w4a8.w4a8_gemm_tiled_splitk(xq, s_a, wts[i % copies], s_w, ws=ws, out=out)
            call(0)
            torch.cuda.synchronize()
            n = max(min(copies, 48), 24)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for i in range(n):
                    call(i)
            graph.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(iters):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / (n * iters)
            del graph
            rows.append({"M": M, "N": N, "K": K, "us": round(us, 2), "TOPS": round(gemm_ops(M, N, K) / us / 1e6, 1),
                         "GBps": round(gemm_bytes(M, N, K) / us / 1e3, 1),
                         "paper_a100_us": round(PAPER_TABLE5_A100_MS[(M, N, K)] * 1e3, 1)})
        del wts, wt
        torch.cuda.empty_cache()
    return rows


def time_w4_vs_w8(torch, w4a8, synth, model="13b", Ms=(16, 1024), iters=4):
    """The paper sets its W4A8 against its own W8A8 (Table 4) and its signed storage against the vanilla unsigned one
    ("Asym GEMM", Sec. 6.4) and the fine-grained recipe (group scales, Eq. (2)).  Here, per GEMM: the same large-M kernel
    over tiled int4 (signed), tiled unsigned int4, signed int4 with group scales, and tiled int8 weights of the same
    fp16 matrix, every launch on a different weight copy (copies exceed the last-level
    cache three times, so weights come from HBM), batches replayed from a HIP graph."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).cuda()
        wp, s_w4 = w4a8.w4a8_quantize_weights(w)
        w8, s_w8 = w4a8.w4a8_quantize_act(w)          # per-channel int8: the per-token quantiser on weight rows
        del w
        # "u4": the vanilla unsigned storage, u = w + 8, i.e. bit 3 of every two's-complement nibble flipped
        wt = {4: w4a8.w4a8_tile_weights(wp), 8: w4a8.w8a8_tile_weights(w8), "u4": w4a8.w4a8_tile_weights(wp ^ 0x88)}
        del wp, w8
        # "fg": the fine-grained recipe (one scale per group of 128 k and channel, Eq. (2)) over the signed codes
        s_g = torch.from_numpy(synth.group_scales(N, K, 128, config_id=3)).cuda()
        fmts = (4, "u4", "fg", 8)
        copies = {b: max(2, -(-3 * LAST_LEVEL_CACHE_BYTES // wt[b].numel()) + 1) for b in (4, "u4", 8)}
        wts = {b: [wt[b]] + [wt[b].clone() for _ in range(copies[b] - 1)] for b in (4, "u4", 8)}
        copies["fg"], wts["fg"] = copies[4], wts[4]
        for M in Ms:
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            # all four through the same kernel (the large-M one with the library's tile for the shape), also at M = 16,
            # where w4a8_gemm_tiled itself would hand the signed format to the weight-streaming kernel
            calls = {4: lambda t: w4a8.w4a8_gemm_tuned(xq, s_a, t, s_w4, w4a8.TILING_PREFILL_TILED, 0, N=N, out=out),
                     "u4": lambda t: w4a8.w4a8_gemm_tiled_unsigned(xq, s_a, t, s_w4, out=out),
                     "fg": lambda t: w4a8.w4a8_gemm_fine_grained(xq, s_a, t, s_g, out=out),
                     8: lambda t: w4a8.w8a8_gemm_tiled(xq, s_a, t, s_w8, out=out)}
            graphs, launches = {}, {}
            for b in fmts:
                calls[b](wts[b][0])
                torch.cuda.synchronize()
                launches[b] = max(copies[b], 8)
                graphs[b] = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graphs[b]):
                    for i in range(launches[b]):
                        calls[b](wts[b][i % copies[b]])
                graphs[b].replay()
            torch.cuda.synchronize()
            # the formats take turns, so that drift of the clocks during the measurement touches all alike
            ms = {b: 0.0 for b in fmts}
            for _ in range(iters):
                for b in fmts:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    graphs[b].replay()
                    e1.record()
                    torch.cuda.synchronize()
                    ms[b] += e0.elapsed_time(e1)
            us = {b: ms[b] * 1e3 / (launches[b] * iters) for b in fmts}
            del graphs
            rows.append({"linear": name, "M": M, "w4a8_us": round(us[4], 2), "w4a8_unsigned_us": round(us["u4"], 2),
                         "w4a8_fine_grained_us": round(us["fg"], 2), "w8a8_us": round(us[8], 2),
                         "unsigned_over_w4": round(us["u4"] / us[4], 3),
                         "fine_grained_over_w4": round(us["fg"] / us[4], 3), "w8_over_w4": round(us[8] / us[4], 3)})
        del wts, wt
        torch.cuda.empty_cache()
    return rows


def cpu_baseline(synth, M, target_seconds):
    """The CPU oracle, as it stands, on the first rows of the same step (all four linears, complete N and K)."""
    import numpy as np
    import oracle
    shapes = synth.LLAMA_SHAPES["13b"]
    macs_per_row = sum(N * K for N, K in shapes.values())
    # probe speed on 8 rows of the smallest linear, then size the sample
    N, K = shapes["o"]
    xq, wq, s_a, s_w = synth.uniform_codes(8, N, K, config_id=9)
    wp = oracle.pack_w4(wq)
    t0 = time.perf_counter()
    oracle.gemm(xq, s_a, wp, s_w)
    rate = 8 * N * K / (time.perf_counter() - t0)
    # the probe (8 rows, first touch of the weights) underestimates the oracle's rate on a long run by about a
    # half: the whole step is taken when it is predicted to stay under 30 s, else the rows for the target time
    rows = M if M * macs_per_row / rate <= 30.0 else int(max(8, min(M, target_seconds * rate / macs_per_row)))
    rows -= rows % 8
    prepared = {}
    for name, (N, K) in shapes.items():
        wq, s_w = oracle.quantize_weights_rtn(synth.weights_fp16(N, K, config_id=3))
        prepared[name] = (oracle.pack_w4(wq), s_w)
    H = shapes["qkv"][1]
    x = synth.activations_fp16(M, H, config_id=3, tag=1)[:rows]
    t0 = time.perf_counter()
    out = None
    for name in ("qkv", "o", "gate_up"):   # the same chain as on the GPU: the Q slice feeds O, O feeds gate+up
        xq, s_a = oracle.quantize_act(x)
        _, _, out = oracle.gemm(xq, s_a, *prepared[name])
        x = np.ascontiguousarray(out[:, :H])
    _, act = oracle.silu_mul(out)
    xq, s_a = oracle.quantize_act(act)   # the oracle keeps the two steps apart
    oracle.gemm(xq, s_a, *prepared["down"])
    dt = time.perf_counter() - t0
    ops = 2 * rows * macs_per_row
    return {"value": round(ops / dt / 1e12, 5), "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {rows} of {M} token rows through all four 13B linears (quantise, GEMM, epilogue, SiLU*up), "
                      f"{dt:.1f} s of CPU time",
            "seconds": round(dt, 2)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2311_09550_amd as w4a8
    from paper_2311_09550_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the W4A8 path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    w4a8.lib()
    torch.cuda.set_device(0)
    M = args.M
    if args.copy_calibration:
        src = torch.full((COPY_CALIBRATION_BYTES,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    weights = prepare_weights(torch, w4a8, synth)
    stack = LayerStack(torch, w4a8, synth, M, weights)
    for _ in range(args.warmup):
        stack.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # every step brackets one of its four GEMMs with events, in rotation: each event is a packet of its own in the
    # queue and widens the gap between launches, so instrumenting all four would slow down the step being timed
    names = list(stack.shapes)
    for i in range(args.steps):
        stack.step(record=names[i % len(names)])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    tops = stack.ops_per_step() / (elapsed / args.steps) / 1e12

    # dominant kernel: the LDS-staged GEMM; average launch duration over the timed region from events on its stream
    per = {}
    for name, a, b in stack.gemm_events:
        per.setdefault(name, []).append(a.elapsed_time(b) * 1e3)
    gemm_us = {k: sum(v) / len(v) for k, v in per.items()}
    avg_us = sum(gemm_us.values()) / len(gemm_us)      # mean over the linears of each linear's mean launch
    ops_per_launch = sum(gemm_ops(M, *stack.shapes[k]) for k in gemm_us) / len(gemm_us)
    achieved = ops_per_launch / avg_us / 1e6   # TOPS
    roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved / INT8_PEAK_TOPS, 4), "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(("13b", M)),
                "traffic_unit": "bytes per launch (L2 fills + write-backs)",
                "algorithmic_bytes_per_launch": round(sum(gemm_bytes(M, *stack.shapes[k]) for k in gemm_us) / len(gemm_us)),
                "kernel": "gemm_prefill_tiled_kernel", "avg_launch_us": round(avg_us, 2),
                "per_linear_us": {k: round(v, 2) for k, v in gemm_us.items()},
                "per_linear_tops": {k: round(gemm_ops(M, *stack.shapes[k]) / v / 1e6, 1) for k, v in gemm_us.items()}}

    result = {
        "metric": "W4A8 GEMM TOPS + HBM GB/s vs roofline, LLaMA-13B shapes, M=1..1024",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"LLaMA-13B-shaped decoder-layer linear stack (QKV, O, gate+up, down), M={M} tokens: "
                               "4 per-token int8 quantisations (one fused with SiLU*up) + 4 W4A8 GEMMs with fused dequant; "
                               "weights quantised, packed and reordered into the tiled layout offline",
                   "M": M, "linears": {k: list(v) for k, v in stack.shapes.items()}, "launches_per_step": 8},
        "gemm_share_of_step": round(sum(gemm_us.values()) / (ms_per_step * 1e3), 4),
        "roofline": roofline,
    }
    del stack
    torch.cuda.empty_cache()
    if not args.no_layer_stack:
        result["layer_stack"] = time_layer_stack(torch, w4a8, synth, weights)
    del weights
    torch.cuda.empty_cache()
    if not args.no_decode:
        rows = time_decode(torch, w4a8, synth)
        result["decode"] = rows
        worst = min(rows, key=lambda r: r["hbm_frac"])
        best = max(rows, key=lambda r: r["hbm_frac"])
        mean_us = sum(r["us"] for r in rows) / len(rows)
        mean_bytes = sum(gemm_bytes(r["M"], r["N"], r["K"]) for r in rows) / len(rows)
        result["roofline_decode"] = {"bound": "hbm", "achieved": round(mean_bytes / mean_us / 1e3, 1), "peak": HBM_PEAK_GBS,
                                     "unit": "GB/s", "frac": round(mean_bytes / mean_us / 1e3 / HBM_PEAK_GBS, 4),
                                     "traffic": None, "kernel": "gemm_decode_resident_kernel",
                                     "worst": worst, "best": best}
    if not args.no_achievable:
        ach = time_achievable(torch, w4a8)
        result["achievable"] = ach
        result["roofline"]["frac_of_achievable"] = round(result["roofline"]["achieved"] / ach["int8_mfma_TOPS"]["random_50us"], 4)
        if "roofline_decode" in result:
            # every decode case against the plain read of a cold piece of about its size
            piece = {"o": "13MB", "qkv": "39MB", "down": "39MB", "gate_up": "71MB"}
            for r in result["decode"]:
                rate = ach["hbm_read_GBps_cold_pieces"][piece[r["linear"]]]
                r["frac_of_stream_read"] = round(r["GBps"] / rate, 4)
            result["roofline_decode"]["frac_of_achievable"] = round(
                sum(r["frac_of_stream_read"] for r in result["decode"]) / len(result["decode"]), 4)
    if not args.no_medium_m:
        result["medium_m"] = time_medium_m(torch, w4a8, synth)
    if not args.no_table5:
        result["paper_table5_shapes"] = time_paper_table5(torch, w4a8, synth)
    if not args.no_w8a8:
        result["w4a8_vs_w8a8"] = time_w4_vs_w8(torch, w4a8, synth)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(synth, M, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
