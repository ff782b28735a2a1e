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
comes from HBM), the same for the LLaMA-7B shapes, a sweep of M = 1 .. 4096 over the
LLaMA-70B shapes, the 13B GEMMs at M = 2048 and 4096, the row-major entry
(w4a8_gemm over Wp[N][K/2]) beside the tiled one, a roofline object for the dominant
kernel, the layer stack at M = 1 .. 2048 replayed from a HIP graph (layer time and
GEMM share), the per-GEMM ratios of the W8A8 comparison variant and of the two
ablation variants (unsigned nibble storage, fine-grained group scales) to W4A8, and
the CPU oracle's throughput on a bounded sample of the workload.  Except for the
row-major rows, every GEMM of the run reads the one tiled copy of the weights,
whatever its M.

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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_counters.json")


def kernel_source_hash():
    """Hash of the kernel sources and headers: ties a counter profile to the build it was taken from."""
    from paper_2311_09550_amd.build import source_hash
    return source_hash()


def measured_traffic(key):
    """HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size) of the kernel
    named `key`, from the counter profile written by paper_2311_09550_amd/counters.py.  Counters cannot be read from
    inside this process, so the figure comes from that file, and only if the file was made from the very sources this
    build was made from; otherwise the line says null and why."""
    try:
        prof = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None, "no counter profile (profiles/traffic_counters.json)"
    if prof.get("source_hash") != kernel_source_hash():
        return None, "counter profile is older than the kernel sources"
    entry = prof.get("kernels", {}).get(key)
    if entry is None:
        return None, "kernel not in the counter profile"
    return entry["traffic_bytes_per_launch"], entry.get("summary", "profiles/")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--M", type=int, default=1024, help="tokens per step (default: the 1024-token context)")
    ap.add_argument("--no-decode", action="store_true", help="skip the M=1,4,16 weight-streaming measurements")
    ap.add_argument("--no-layer-stack", action="store_true", help="skip the graph-replayed layer stack at M=1..2048")
    ap.add_argument("--no-w8a8", action="store_true", help="skip the per-GEMM W4A8 / W8A8 comparison")
    ap.add_argument("--no-achievable", action="store_true", help="skip the probes of achievable HBM and MFMA rates")
    ap.add_argument("--no-medium-m", action="store_true", help="skip the four linears at M = 32 .. 512")
    ap.add_argument("--no-table5", action="store_true", help="skip the GEMM sizes of the paper's Table 5")
    ap.add_argument("--no-7b", action="store_true", help="skip the LLaMA-7B decode linears")
    ap.add_argument("--no-70b", action="store_true", help="skip the LLaMA-70B sweep over M")
    ap.add_argument("--no-large-m", action="store_true", help="skip the 13B GEMMs at M = 2048 and 4096")
    ap.add_argument("--no-row-major", action="store_true", help="skip the row-major entry (w4a8_gemm over Wp)")
    ap.add_argument("--only", default="", help="comma-separated sections to run besides the timed step "
                    "(decode, layer_stack, 7b, 70b, large_m, row_major, achievable, medium_m, rowwise, table5, w8a8, cpu); empty = all")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-swiglu-epilogue", action="store_true",
                    help="keep SiLU*up in the quantiser in front of the down projection at every M (default: from 768 "
                         "tokens on it moves into the gate+up GEMM's epilogue, w4a8_gemm_tiled_swiglu)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy three times: the dispatch of known size against which "
                         "hardware traffic counters are scaled")
    return ap.parse_args()


# One copy of the weights, in the tiled layout, serves every M: the library's tiled entry runs the weight-streaming
# kernels up to M = 16 and the large-M kernel above, with K cut into slices where its tiles alone would not fill the chip.


def prepare_weights(torch, w4a8, synth, model="13b"):
    """Offline weight preparation, on the GPU: quantise and pack, then reorder into the tiled array (the only copy that
    is kept).  Returns name -> (wt, s_w); "gate_up_interleaved" holds the gate and up channels of the same matrix
    interleaved, the order the GEMM with the SiLU*up epilogue takes them in (a deployment keeps one of the two orders;
    the benchmark keeps both because it also times the unfused launches)."""
    out = {}
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).to("cuda")
        wp, s_w = w4a8.w4a8_quantize_weights(w)
        out[name] = (w4a8.w4a8_tile_weights(wp), s_w)
        if name == "gate_up":
            wp, s_w = w4a8.w4a8_quantize_weights(w4a8.interleave_gate_up(w))
            out["gate_up_interleaved"] = (w4a8.w4a8_tile_weights(wp), s_w)
        del w, wp
    return out


class LayerStack:
    """Device buffers of one 13B-shaped decoder layer's linears and the launches of a step.

    Eight launches (three per-token quantisers, the fused SiLU*up + quantiser, four GEMMs).  Up to SWIGLU_UP_TO_M and
    from SWIGLU_FROM_M tokens on the gate+up GEMM applies SiLU*up in its epilogue (w4a8_gemm_tiled_swiglu) and a plain
    per-token quantiser follows: still eight launches, but the M x 2I intermediate is neither written nor read.
    M <= FUSE_UP_TO_M with fuse=True: four launches -- every linear quantises its own activations inside the weight-streaming
    GEMM (w4a8_linear_tiled_fp16), and the gate+up one also applies SiLU*up (w4a8_linear_tiled_swiglu_fp16), so that
    the down projection is fed fp16 like the others."""

    # Token count from which the gate+up GEMM takes SiLU*up into its epilogue (None = never; `--no-swiglu-epilogue`).
    # Measured on the 13B layer, both forms in turn on one box: 1.5 to 1.7 % off the step at M = 1024 and 2048 (the GEMM
    # gains 2.7 us of exposed exp2 / reciprocal work at the end of its tiles, the quantiser behind it reads half the
    # bytes and loses 8 us); level at 256 and 512; 1 % slower at 128.
    SWIGLU_FROM_M = 768
    # ... and the token count up to which the weight-streaming kernel does (its epilogue is a few lanes' work)
    SWIGLU_UP_TO_M = 32
    # Token count up to which every linear quantises its own input (w4a8_linear_tiled_fp16 and its SiLU*up form)
    FUSE_UP_TO_M = 3

    def __init__(self, torch, w4a8, synth, M, weights, model="13b", fuse=False, prenorm=False):
        self.torch, self.w4a8, self.M = torch, w4a8, M
        self.shapes = synth.LLAMA_SHAPES[model]
        # measured, the forms timed in turn: 35.3 against 43.5 us per layer at M = 1, 39.9 against 44.8 at M = 2, 44.6
        # against 45.4 at M = 3; at M = 4 the down projection's rows no longer fit LDS twice over
        # (with the norms taken into the linears, prenorm, a third token costs more than the launches save: 49.7 us
        # against about 46 for the eight-launch form with the norm-fused quantisers)
        self.fused = bool(fuse and M <= (2 if prenorm else self.FUSE_UP_TO_M))
        dev = "cuda"
        self.wp = {k: v[0] for k, v in weights.items()}
        self.s_w = {k: v[1] for k, v in weights.items()}
        self.swiglu = (self.SWIGLU_FROM_M is not None and (M >= self.SWIGLU_FROM_M or M <= self.SWIGLU_UP_TO_M)
                       and "gate_up_interleaved" in weights)
        self.fused = self.fused and self.swiglu
        H = self.shapes["qkv"][1]
        I = self.shapes["down"][1]
        # fp16 hidden states enter the stack; attention itself is not modelled: the Q slice of the QKV output stands in
        # for its result, and every later linear is fed by the one before it, so the launches form one chain
        self.h = torch.from_numpy(synth.activations_fp16(M, H, config_id=3, tag=1)).to(dev)
        e = lambda *s, dt: torch.empty(s, dtype=dt, device=dev)
        self.xq_h, self.sa_h = e(M, H, dt=torch.int8), e(M, dt=torch.float32)
        self.xq_i, self.sa_i = e(M, I, dt=torch.int8), e(M, dt=torch.float32)
        self.out = {name: e(M, N, dt=torch.float16) for name, (N, K) in self.shapes.items()}
        # scratch for the GEMMs whose K the library cuts into slices (medium M; empty where it does not)
        self.ws = {name: e(max(16, w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)), dt=torch.uint8)
                   for name, (N, K) in self.shapes.items()}
        self.gemm_events = []   # (name, start, stop) around GEMM launches, filled when record=True
        # the launches with their arguments marshalled once: the timed loop then spends its host time in the
        # library, not in Python
        b = w4a8.bound_call
        self.quant = {"qkv": b("w4a8_quantize_act", self.h, self.xq_h, self.sa_h, M, H),
                      "o": b("w4a8_quantize_act_strided", self.out["qkv"], self.shapes["qkv"][0], self.xq_h, self.sa_h, M, H),
                      "gate_up": b("w4a8_quantize_act", self.out["o"], self.xq_h, self.sa_h, M, H),
                      "down": b("w4a8_silu_mul_quantize", self.out["gate_up"], self.xq_i, self.sa_i, M, I)}
        if prenorm:
            # the two quantisers that sit behind an RMSNorm in a pre-norm decoder layer take it (and, in front of the
            # MLP, the residual addition) into their pass: same launch count, a more faithful layer
            import ctypes
            self.gamma = torch.ones((H,), dtype=torch.float16, device=dev)
            self.resid = e(M, H, dt=torch.float16)
            eps = ctypes.c_float(1e-5)
            self.quant["qkv"] = b("w4a8_add_rmsnorm_quantize", self.h, None, self.gamma, eps, None, None, self.xq_h, self.sa_h, M, H)
            self.quant["gate_up"] = b("w4a8_add_rmsnorm_quantize", self.out["o"], self.h, self.gamma, eps, self.resid, None,
                                      self.xq_h, self.sa_h, M, H)
        self.gemm = {}
        for name, (N, K) in self.shapes.items():
            xq, sa = (self.xq_i, self.sa_i) if name == "down" else (self.xq_h, self.sa_h)
            self.gemm[name] = b("w4a8_gemm_tiled_splitk", xq, sa, self.wp[name], self.s_w[name], self.out[name], M, N, K,
                                0, 0, self.ws[name], self.ws[name].numel())
        if self.swiglu:
            # gate+up with SiLU*up in its epilogue -> h [M][I]; the quantiser in front of the down projection reads h
            self.hmid = e(M, I, dt=torch.float16)
            self.gemm["gate_up"] = b("w4a8_gemm_tiled_swiglu", self.xq_h, self.sa_h, self.wp["gate_up_interleaved"],
                                     self.s_w["gate_up_interleaved"], self.hmid, M, I, self.shapes["gate_up"][1])
            self.quant["down"] = b("w4a8_quantize_act", self.hmid, self.xq_i, self.sa_i, M, I)
        if self.fused:
            src = {"qkv": (self.h, H), "o": (self.out["qkv"], self.shapes["qkv"][0]), "down": (self.hmid, I)}
            self.linear = {name: b("w4a8_linear_tiled_fp16", x, ldx, self.wp[name], self.s_w[name], self.out[name], None,
                                   M, self.shapes[name][0], self.shapes[name][1]) for name, (x, ldx) in src.items()}
            self.linear["gate_up"] = b("w4a8_linear_tiled_swiglu_fp16", self.out["o"], H, self.wp["gate_up_interleaved"],
                                       self.s_w["gate_up_interleaved"], self.hmid, None, M, I, self.shapes["gate_up"][1])
            if prenorm:
                # the two linears behind a norm take it, and the residual addition in front of the MLP, into their launch
                import ctypes
                eps = ctypes.c_float(1e-5)
                self.linear["qkv"] = b("w4a8_linear_tiled_norm_fp16", self.h, H, None, 0, self.gamma, eps, None, None,
                                       self.wp["qkv"], self.s_w["qkv"], self.out["qkv"], None, M, self.shapes["qkv"][0], H, 0)
                self.linear["gate_up"] = b("w4a8_linear_tiled_norm_fp16", self.out["o"], H, self.h, H, self.gamma, eps,
                                           self.resid, None, self.wp["gate_up_interleaved"], self.s_w["gate_up_interleaved"],
                                           self.hmid, None, M, 2 * I, H, 1)
        self.launches_per_step = 4 if self.fused else 8

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
        """One pass over the launches; `record` names the GEMM to bracket with timing events (None: none)."""
        for name in ("qkv", "o", "gate_up", "down"):
            if self.fused:
                self.linear[name]()      # per-token quantiser inside the weight-streaming GEMM
                continue
            self.quant[name]()           # "down": SiLU*up and its quantiser in one pass, or the quantiser of h
            self._gemm(name, record == name)

    def gemms_only(self):
        for name in ("qkv", "o", "gate_up", "down"):
            self.gemm[name]()

    def ops_per_step(self):
        return sum(gemm_ops(self.M, N, K) for N, K in self.shapes.values())


# The chip leaves its idle power state slowly: for the first 20 to 40 ms of work after a pause (and every section here
# starts with host-side set-up) the same kernels run up to 10 % slower than in the steady state that a serving or
# training loop lives in.  Every timed region is therefore preceded by SETTLE_MS of the very work it times.
SETTLE_MS = 30.0
TIMED_MS = 10.0


def settle_and_time(torch, replay, replays):
    """Replays `replay()` untimed for SETTLE_MS of GPU time, then times at least `replays` replays (and at least
    TIMED_MS of them) between two events on the launch stream.  Returns milliseconds per replay."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    replay()
    b.record()
    torch.cuda.synchronize()
    one = max(a.elapsed_time(b), 1e-3)
    for _ in range(min(2000, int(SETTLE_MS / one) + 1)):
        replay()
    n = min(2000, max(replays, int(TIMED_MS / one) + 1))
    a.record()
    for _ in range(n):
        replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


def graph_time_us(torch, fn_of_i, launches, replays):
    """Per-launch time of `launches` calls fn_of_i(0..launches-1) captured in one HIP graph and replayed, after the
    device has settled, at least `replays` times between two events on the launch stream (gaps between dependent
    kernels included)."""
    fn_of_i(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(launches):
            fn_of_i(i)
    graph.replay()
    torch.cuda.synchronize()
    us = settle_and_time(torch, graph.replay, replays) * 1e3 / launches
    del graph
    return us


def cold_copies(torch, wt, at_least=2):
    """Copies of a weight array that together exceed the last-level cache three times: rotating through them, every
    launch finds its weights in HBM."""
    copies = max(at_least, -(-3 * LAST_LEVEL_CACHE_BYTES // wt.numel()) + 1)
    return [wt] + [wt.clone() for _ in range(copies - 1)]


def roofline_row(M, N, K, us):
    by, ops = gemm_bytes(M, N, K), gemm_ops(M, N, K)
    t_mem, t_mfma = by / HBM_PEAK_GBS / 1e3, ops / INT8_PEAK_TOPS / 1e6
    return {"us": round(us, 2), "TOPS": round(ops / us / 1e6, 1), "GBps": round(by / us / 1e3, 1),
            "bound": "hbm" if t_mem >= t_mfma else "mfma", "roofline_frac": round(max(t_mem, t_mfma) / us, 4)}


def time_layer_stack(torch, w4a8, synth, weights, Ms=(1, 2, 3, 16, 64, 128, 1024, 2048), steps_per_graph=8, replays=6):
    """The decoder layer's linear stack at several M, replayed from a HIP graph (what a serving loop does; at small M
    the launches would otherwise be timed by the interpreter).  Layer time = graph time / steps; the GEMM share is the
    time of a second graph that holds only the four plain GEMMs (pre-quantised inputs), over the layer time.  At
    M <= 3 the layer runs with the quantisers folded into the GEMMs (4 launches), and the unfused form (8 launches)
    is timed beside it.  One layer's weights (158 MB) stay resident in the last-level cache across replays: the small-M
    rows are a warm-cache figure, the HBM-bound figure is the `decode` list.  `prenorm_layer_us`: the same layer with an
    RMSNorm in front of QKV and the residual addition + RMSNorm in front of gate+up, as in a pre-norm decoder layer, taken
    into the quantisers (eight-launch rows) or into the self-quantising linears (four-launch rows): same launch counts."""
    rows = []
    for M in Ms:
        stack = LayerStack(torch, w4a8, synth, M, weights, fuse=True)
        plain = LayerStack(torch, w4a8, synth, M, weights, fuse=False) if stack.fused else None
        times = {}
        todo = [("layer", stack.step), ("gemms", stack.gemms_only)]
        if plain is not None:
            todo.append(("unfused", plain.step))
        for what, fn in todo:
            for _ in range(3):
                fn()
            times[what] = graph_time_us(torch, lambda i: fn(), steps_per_graph, replays)
        pre = LayerStack(torch, w4a8, synth, M, weights, fuse=stack.fused, prenorm=True)
        for _ in range(3):
            pre.step()
        times["prenorm"] = graph_time_us(torch, lambda i: pre.step(), steps_per_graph, replays)
        del pre
        row = {"M": M, "layer_us": round(times["layer"], 2), "gemm_us": round(times["gemms"], 2),
               "gemm_share": round(times["gemms"] / times["layer"], 4),
               "TOPS": round(stack.ops_per_step() / times["layer"] / 1e6, 2),
               "launches": stack.launches_per_step, "weights": "tiled"}
        if plain is not None:
            row["unfused_layer_us"] = round(times["unfused"], 2)
        if "prenorm" in times:
            row["prenorm_layer_us"] = round(times["prenorm"], 2)
        rows.append(row)
        del stack, plain
        torch.cuda.empty_cache()
    return rows


def quantised_tiled(torch, w4a8, w):
    wp, s_w = w4a8.w4a8_quantize_weights(w)
    return w4a8.w4a8_tile_weights(wp), wp, s_w


def time_decode(torch, w4a8, synth, model="13b", Ms=(1, 4, 16), iters=5):
    """Weight-streaming GEMMs: every launch reads a different copy of the weights, the copies together
    exceeding the last-level cache three times, so the weights come from HBM.  Per-launch time is the
    average over back-to-back batches replayed from a HIP graph, between two events on the launch stream
    (the gaps between dependent kernels are included)."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).cuda()
        wt, wp, s_w = quantised_tiled(torch, w4a8, w)   # wt: the same array the large-M kernel reads
        del w, wp
        wts = cold_copies(torch, wt)
        copies = len(wts)
        for M in Ms:
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            for i in range(min(copies, 4)):
                w4a8.w4a8_gemm_tiled(xq, s_a, wts[i], s_w, out=out)
            # One graph holds a back-to-back batch of launches (a decode loop is replayed from a graph as well; launching
            # each 5-15 us kernel from Python would time the interpreter, not the GPU).
            us = graph_time_us(torch, lambda i: w4a8.w4a8_gemm_tiled(xq, s_a, wts[i % copies], s_w, out=out),
                               max(copies, 24), iters)
            by = gemm_bytes(M, N, K)
            rows.append({"linear": name, "M": M, "N": N, "K": K, "us": round(us, 3),
                         "GBps": round(by / us / 1e3, 1), "hbm_frac": round(by / us / 1e3 / HBM_PEAK_GBS, 4),
                         "weight_copies": copies})
        del wts, wt
        torch.cuda.empty_cache()
    return rows


def decode_roofline(rows, kernel):
    worst = min(rows, key=lambda r: r["hbm_frac"])
    best = max(rows, key=lambda r: r["hbm_frac"])
    mean_us = sum(r["us"] for r in rows) / len(rows)
    mean_bytes = sum(gemm_bytes(r["M"], r["N"], r["K"]) for r in rows) / len(rows)
    return {"bound": "hbm", "achieved": round(mean_bytes / mean_us / 1e3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(mean_bytes / mean_us / 1e3 / HBM_PEAK_GBS, 4),
            "mean_of_row_fracs": round(sum(r["hbm_frac"] for r in rows) / len(rows), 4),
            "algorithmic_bytes_per_launch": round(mean_bytes), "kernel": kernel, "worst": worst, "best": best}


def device_weights_fp16(torch, N, K, seed, sigma=0.02):
    """fp16 N(0, sigma) weights drawn on the device from a seeded generator (the 70B matrices are too large to draw on
    the host within the run's time): same distribution as synth.weights_fp16, another stream."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    w = torch.empty((N, K), dtype=torch.float16, device="cuda")
    rows = max(1, (64 << 20) // K)
    for r0 in range(0, N, rows):
        r1 = min(N, r0 + rows)
        w[r0:r1] = (torch.randn((r1 - r0, K), generator=g, device="cuda", dtype=torch.float32) * sigma).to(torch.float16)
    return w


def device_activations_fp16(torch, synth, M, K, seed):
    """fp16 N(0,1) activations with the fixed outlier channels of the workload x50, drawn on the device."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32)
    x[:, torch.from_numpy(synth.outlier_channels(K, 4)).cuda()] *= 50.0
    return x.to(torch.float16)


def time_llama70b_sweep(torch, w4a8, synth, Ms=(1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096)):
    """The four LLaMA-70B-shaped linears (GQA: 64 query and 8 KV heads of 128) over M = 1 .. 4096 through the one-copy
    entry, cold weights (rotating copies), one graph-replayed timing per point.  Each row is set against the larger of
    its two roofline times."""
    rows = []
    for idx, (name, (N, K)) in enumerate(synth.LLAMA_SHAPES["70b"].items()):
        w = device_weights_fp16(torch, N, K, seed=7000 + idx)
        wt, wp, s_w = quantised_tiled(torch, w4a8, w)
        del w, wp
        wts = cold_copies(torch, wt)
        copies = len(wts)
        for M in Ms:
            x = device_activations_fp16(torch, synth, M, K, seed=7100 + idx)
            xq, s_a = w4a8.w4a8_quantize_act(x)
            del x
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            ws = torch.empty((max(16, w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)),), dtype=torch.uint8, device="cuda")
            us = graph_time_us(torch, lambda i: w4a8.w4a8_gemm_tiled_splitk(xq, s_a, wts[i % copies], s_w, ws=ws, out=out),
                               max(copies, 4 if M >= 1024 else 12), 2)
            rows.append({"linear": name, "M": M, "N": N, "K": K, **roofline_row(M, N, K, us)})
            del xq, s_a, out, ws
        del wts, wt
        torch.cuda.empty_cache()
    return rows


def time_large_m(torch, w4a8, synth, weights, Ms=(2048, 4096)):
    """The 13B linears as single GEMMs at M = 2048 and 4096 (warm weights: at these sizes the operands are re-read
    from cache many times within one launch anyway)."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES["13b"].items():
        wt, s_w = weights[name]
        for M in Ms:
            x = device_activations_fp16(torch, synth, M, K, seed=1300 + M)
            xq, s_a = w4a8.w4a8_quantize_act(x)
            del x
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            us = graph_time_us(torch, lambda i: w4a8.w4a8_gemm_tiled(xq, s_a, wt, s_w, out=out), 4, 3)
            rows.append({"linear": name, "M": M, "N": N, "K": K, **roofline_row(M, N, K, us)})
            del xq, s_a, out
        torch.cuda.empty_cache()
    return rows


def time_row_major(torch, w4a8, synth, Ms=(1, 16, 1024)):
    """The entry the problem statement names, w4a8_gemm over the row-major packed array Wp[N][K/2], beside the tiled
    entry on the same codes: what a caller pays for not reordering the weights offline.  Cold weights, graph replay."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES["13b"].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).cuda()
        wt, wp, s_w = quantised_tiled(torch, w4a8, w)
        del w
        wps, wts = cold_copies(torch, wp), cold_copies(torch, wt)
        copies = len(wps)
        for M in Ms:
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            n = max(copies, 24) if M <= 16 else max(copies, 8)
            us_row = graph_time_us(torch, lambda i: w4a8.w4a8_gemm(xq, s_a, wps[i % copies], s_w, out=out), n, 3)
            us_tiled = graph_time_us(torch, lambda i: w4a8.w4a8_gemm_tiled(xq, s_a, wts[i % copies], s_w, out=out), n, 3)
            rows.append({"linear": name, "M": M, "N": N, "K": K, "row_major": roofline_row(M, N, K, us_row),
                         "tiled_us": round(us_tiled, 2), "row_major_over_tiled": round(us_row / us_tiled, 3)})
        del wps, wts, wp, wt
        torch.cuda.empty_cache()
    return rows


READ_PATTERNS = {0: "grid-wide stride, global loads", 1: "one contiguous run per workgroup, global loads",
                 2: "grid-wide stride, buffer loads", 3: "one run per workgroup, buffer loads",
                 4: "grid-wide stride, buffer loads, non-temporal", 5: "one run per workgroup, buffer loads, non-temporal"}


def time_achievable(torch, w4a8):
    """What the chip sustains, measured with the library's probes, to set the datasheet fractions against.
    Reads: a streaming reduction over 2 GiB (eight times the last-level cache, so every pass comes from HBM) in a
    handful of access patterns (grid-wide stride or one run per workgroup; plain or non-temporal loads; 4 / 8 / 16 loads
    in flight per thread; 1 .. 8 workgroups per compute unit), the best of which is the read ceiling, and the same best
    pattern over cold pieces of the sizes of the 13B weight matrices, launched back to back from a graph (what one
    weight-streaming GEMM launch could reach at most).  An independent figure: a plain 256 MiB device-to-device copy
    (read + write).  Matrix cores: a register-resident int8 MFMA loop on constant and on random operands."""
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

    variants = [(p, l, g) for p in (0, 1, 4, 5) for l in (4, 8, 16) for g in (1, 2, 8)]
    rates = {v: big.numel() / timed(lambda: w4a8.w4a8_probe_read_pattern(big, sink, *v), 2) / 1e9 for v in variants}
    best = max(rates, key=rates.get)
    out["hbm_read_GBps"] = round(rates[best], 1)
    out["hbm_read_pattern"] = {"pattern": READ_PATTERNS[best[0]], "loads_in_flight_per_thread": best[1],
                               "workgroups_per_cu": best[2]}
    out["hbm_read_GBps_by_pattern"] = {READ_PATTERNS[p]: round(max(r for v, r in rates.items() if v[0] == p), 1)
                                       for p in (0, 1, 4, 5)}
    out["hbm_read_GBps_plain_probe"] = round(big.numel() / timed(lambda: w4a8.w4a8_probe_stream_read(big, sink), 3) / 1e9, 1)
    by_size = {}
    for mb in (13, 39, 71):
        size = mb * 1000 * 1000 // 4096 * 4096
        n = big.numel() // size            # consecutive pieces: each is read once per pass over the 2 GiB
        pieces = [big[i * size:(i + 1) * size] for i in range(n)]
        best_rate = 0.0
        for v in ((4, 8, 2), (4, 4, 2), (5, 8, 2), (5, 4, 8)):
            w4a8.w4a8_probe_read_pattern(pieces[0], sink, *v)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for piece in pieces:
                    w4a8.w4a8_probe_read_pattern(piece, sink, *v)
            best_rate = max(best_rate, size * n / timed(graph.replay, 2) / 1e9)
            del graph
        by_size[f"{mb}MB"] = round(best_rate, 1)
    out["hbm_read_GBps_cold_pieces"] = by_size
    # one workgroup per compute unit reading 512 KB: from memory, from L2, and half and half (the situation of a GEMM
    # at a hundred or so tokens: activations re-read from cache while the weights stream); graph of launches over
    # rotating cold windows, figures per launch including the 1.4 us between kernels
    hot = torch.full((640 << 10,), 5, dtype=torch.uint8, device="cuda")
    window = 128 << 20
    n = big.numel() // window
    mixed = {}
    for mode, name in ((2, "memory_only"), (3, "l2_only"), (0, "half_and_half_same_waves"), (1, "half_and_half_separate_waves")):
        span = window if mode == 2 else window // 2     # 512 KB (mode 2) or 256 KB of cold data per compute unit
        per_cu = w4a8.w4a8_probe_mixed_read(big[:span], hot, sink, mode)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(n):
                w4a8.w4a8_probe_mixed_read(big[i * window:i * window + span], hot, sink, mode)
        us = timed(graph.replay, 3) * 1e6 / n
        mixed[name] = {"us": round(us, 2), "KB_per_us_per_cu": round(per_cu / 1024 / us, 1)}
        del graph
    out["per_cu_read_512KB"] = mixed
    del big, hot
    torch.cuda.empty_cache()
    src = torch.full((COPY_CALIBRATION_BYTES,), 3, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    out["copy_256MiB_read_plus_write_GBps"] = round(2 * COPY_CALIBRATION_BYTES / timed(lambda: dst.copy_(src), 5) / 1e9, 1)
    del src, dst
    mfma = {}
    for label, iters, pattern, reps in (("constant_2ms", 8000, 0, 3), ("random_2ms", 8000, 1, 3), ("random_50us", 200, 1, 40)):
        ops = [0]

        def run():
            ops[0] = w4a8.w4a8_probe_mfma_int8(sink, iters, pattern)
        t = timed(run, reps)
        mfma[label] = round(ops[0] / t / 1e12, 1)
    out["int8_mfma_TOPS"] = mfma
    return out


def time_rowwise(torch, w4a8, synth, Ms=(1, 16, 1024), K=5120):
    """The row-wise kernels in front of a linear, replayed back to back from a HIP graph (1.4 us of every figure is the
    gap between kernels): the per-token quantiser alone and fused behind residual addition + RMSNorm, with the bytes
    each moves (quantiser: 2 K in, K out per token; fused: x and the residual in, the new residual and the codes out)."""
    rows = []
    gamma = torch.ones((K,), dtype=torch.float16, device="cuda")
    for M in Ms:
        x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=6)).cuda()
        res = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=7)).cuda()
        r = torch.empty_like(x)
        xq = torch.empty((M, K), dtype=torch.int8, device="cuda")
        s_a = torch.empty((M,), dtype=torch.float32, device="cuda")
        quant = w4a8.bound_call("w4a8_quantize_act", x, xq, s_a, M, K)
        import ctypes
        fused = w4a8.bound_call("w4a8_add_rmsnorm_quantize", x, res, gamma, ctypes.c_float(1e-5), r, None, xq, s_a, M, K)
        t_q = graph_time_us(torch, lambda i: quant(), 16, 6)
        t_f = graph_time_us(torch, lambda i: fused(), 16, 6)
        rows.append({"M": M, "K": K, "quantize_act_us": round(t_q, 2), "quantize_act_GBps": round(3 * M * K / t_q / 1e3, 1),
                     "add_rmsnorm_quantize_us": round(t_f, 2), "add_rmsnorm_quantize_GBps": round(7 * M * K / t_f / 1e3, 1)})
    return rows


def time_medium_m(torch, w4a8, synth, model="13b", Ms=(32, 64, 128, 256, 512), iters=4):
    """Between token generation and context decoding: the four linears at M = 32 .. 512 from cold weights (rotating
    copies as in time_decode), through the one-copy entry with its K slices.  Each row is set against the larger of
    the two roofline times (bytes at the HBM peak, operations at the int8 MFMA peak)."""
    rows = []
    for name, (N, K) in synth.LLAMA_SHAPES[model].items():
        w = torch.from_numpy(synth.weights_fp16(N, K, config_id=3)).cuda()
        wt, wp, s_w = quantised_tiled(torch, w4a8, w)
        del w, wp
        wts = cold_copies(torch, wt)
        copies = len(wts)
        for M in Ms:
            x = torch.from_numpy(synth.activations_fp16(M, K, config_id=3, tag=4)).cuda()
            xq, s_a = w4a8.w4a8_quantize_act(x)
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            need = w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)
            ws = torch.empty((max(16, need),), dtype=torch.uint8, device="cuda")
            us = graph_time_us(torch, lambda i: w4a8.w4a8_gemm_tiled_splitk(xq, s_a, wts[i % copies], s_w, ws=ws, out=out),
                               max(copies, 16), iters)
            rows.append({"linear": name, "M": M, **roofline_row(M, N, K, us),
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
            us = settle_and_time(torch, graph.replay, iters) * 1e3 / n
            del graph
            rows.append({"M": M, "N": N, "K": K, "us": round(us, 2), "TOPS": round(gemm_ops(M, N, K) / us / 1e6, 1),
                         "GBps": round(gemm_bytes(M, N, K) / us / 1e3, 1),
                         "paper_a100_us": round(PAPER_TABLE5_A100_MS[(M, N, K)] * 1e3, 1)})
        del wts, wt
        torch.cuda.empty_cache()
    return rows


def time_w4_vs_w8(torch, w4a8, synth, model="13b", Ms=(16, 1024), iters=4):
    """The paper sets its W4A8 against its own W8A8 (Table 4) and its signed storage against the vanilla unsigned one
    ("Asym GEMM", Sec. 7.2) and the fine-grained recipe (group scales, Eq. (5)).  Here, per GEMM: the same large-M kernel
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
        # "fg": the fine-grained recipe (one scale per group of 128 k and channel, Eq. (5)) over the signed codes
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
            settle_and_time(torch, lambda: [graphs[b].replay() for b in fmts], 1)
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
    w4a8.w4a8_init()
    only = {s for s in args.only.split(",") if s}

    def wanted(section, disabled):
        return not disabled and (not only or section in only)

    M = args.M
    if args.copy_calibration:
        src = torch.full((COPY_CALIBRATION_BYTES,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.no_swiglu_epilogue:
        LayerStack.SWIGLU_FROM_M = None
    weights = prepare_weights(torch, w4a8, synth)
    stack = LayerStack(torch, w4a8, synth, M, weights)
    # set-up ends with the device out of its idle power state (see SETTLE_MS); then the warm-up steps asked for
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < 2 * SETTLE_MS:
        for _ in range(10):
            stack.step()
        torch.cuda.synchronize()
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
    traffic, traffic_note = measured_traffic(f"gemm_prefill_tiled_kernel@13b,M={M}")

    def launch_bytes(k):   # the gate+up GEMM with the SiLU*up epilogue writes M x I values instead of M x 2I
        by = gemm_bytes(M, *stack.shapes[k])
        return by - M * stack.shapes[k][0] if (k == "gate_up" and stack.swiglu) else by

    roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved / INT8_PEAK_TOPS, 4), "traffic": traffic,
                "traffic_unit": "bytes per launch (L2 fills + write-backs)", "traffic_source": traffic_note,
                "algorithmic_bytes_per_launch": round(sum(launch_bytes(k) for k in gemm_us) / len(gemm_us)),
                "kernel": "gemm_prefill_tiled_kernel", "avg_launch_us": round(avg_us, 2),
                "per_linear_us": {k: round(v, 2) for k, v in gemm_us.items()},
                "per_linear_tops": {k: round(gemm_ops(M, *stack.shapes[k]) / v / 1e6, 1) for k, v in gemm_us.items()},
                "per_linear_frac": {k: round(gemm_ops(M, *stack.shapes[k]) / v / 1e6 / INT8_PEAK_TOPS, 4)
                                    for k, v in gemm_us.items()}}

    result = {
        "metric": "W4A8 GEMM TOPS + HBM GB/s vs roofline, LLaMA-13B shapes, M=1..1024",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"LLaMA-13B-shaped decoder-layer linear stack (QKV, O, gate+up, down), M={M} tokens: "
                               "4 per-token int8 quantisations + 4 W4A8 GEMMs with fused dequant, SiLU*up "
                               + ("in the gate+up GEMM's epilogue; " if stack.swiglu else "fused with the quantiser behind it; ")
                               + "weights quantised, packed and reordered into the tiled layout offline",
                   "silu_mul": "gemm epilogue" if stack.swiglu else "quantiser",
                   "M": M, "linears": {k: list(v) for k, v in stack.shapes.items()}, "launches_per_step": 8},
        "settle_ms_before_warmup": 2 * SETTLE_MS,
        "gemm_share_of_step": round(sum(gemm_us.values()) / (ms_per_step * 1e3), 4),
        "kernel_source_hash": kernel_source_hash(),
        "roofline": roofline,
    }
    del stack
    torch.cuda.empty_cache()
    if wanted("layer_stack", args.no_layer_stack):
        result["layer_stack"] = time_layer_stack(torch, w4a8, synth, weights)
    if wanted("large_m", args.no_large_m):
        result["llama13b_large_m"] = time_large_m(torch, w4a8, synth, weights)
    del weights
    torch.cuda.empty_cache()
    if wanted("decode", args.no_decode):
        rows = time_decode(torch, w4a8, synth)
        result["decode"] = rows
        result["roofline_decode"] = decode_roofline(rows, "gemm_decode_resident_kernel")
        t, note = measured_traffic("gemm_decode_resident_kernel@13b,M=1..16")
        result["roofline_decode"]["traffic"] = t
        result["roofline_decode"]["traffic_source"] = note
    if wanted("7b", args.no_7b):
        rows = time_decode(torch, w4a8, synth, model="7b")
        result["llama7b_decode"] = rows
        result["roofline_llama7b_decode"] = decode_roofline(rows, "gemm_decode_resident_kernel")
    if wanted("70b", args.no_70b):
        result["llama70b_sweep"] = time_llama70b_sweep(torch, w4a8, synth)
    if wanted("row_major", args.no_row_major):
        result["row_major"] = time_row_major(torch, w4a8, synth)
    if wanted("achievable", args.no_achievable):
        ach = time_achievable(torch, w4a8)
        result["achievable"] = ach
        result["roofline"]["frac_of_achievable"] = round(result["roofline"]["achieved"] / ach["int8_mfma_TOPS"]["random_2ms"], 4)
        if "roofline_decode" in result:
            # every decode case against the best plain read of a cold piece of about its size
            piece = {"o": "13MB", "qkv": "39MB", "down": "39MB", "gate_up": "71MB"}
            for r in result["decode"]:
                rate = ach["hbm_read_GBps_cold_pieces"][piece[r["linear"]]]
                r["frac_of_stream_read"] = round(r["GBps"] / rate, 4)
            result["roofline_decode"]["frac_of_achievable"] = round(
                sum(r["frac_of_stream_read"] for r in result["decode"]) / len(result["decode"]), 4)
    if wanted("medium_m", args.no_medium_m):
        result["medium_m"] = time_medium_m(torch, w4a8, synth)
    if wanted("rowwise", False):
        result["rowwise"] = time_rowwise(torch, w4a8, synth)
    if wanted("table5", args.no_table5):
        result["paper_table5_shapes"] = time_paper_table5(torch, w4a8, synth)
    if wanted("w8a8", args.no_w8a8):
        result["w4a8_vs_w8a8"] = time_w4_vs_w8(torch, w4a8, synth)
    if wanted("cpu", args.no_cpu_baseline):
        result["cpu_baseline"] = cpu_baseline(synth, M, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
