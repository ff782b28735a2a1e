"""The entry points under HIP graph capture: captured once after w4a8_init (which makes every per-device preparation up
front, so that no launch has to make one while a capture is open), replayed several times with new input contents and
with eager work and synchronisations between the replays; every replay must reproduce the eager result bit for bit."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

pytestmark = pytest.mark.gpu


def _linear(t, M, wt, s_w, x, xq, s_a, out, how, ws):
    if how == "fused":
        w4a8.w4a8_linear_tiled_fp16(x, wt, s_w, out=out)
        return
    w4a8.w4a8_quantize_act(x, xq, s_a)
    if how == "tiled":
        w4a8.w4a8_gemm_tiled(xq, s_a, wt, s_w, out=out)
    elif how == "splitk":
        w4a8.w4a8_gemm_tiled_splitk(xq, s_a, wt, s_w, ws=ws, out=out)
    else:
        w4a8.w4a8_gemm_tiled_splitk_static(xq, s_a, wt, s_w, out)


# (M, N, K, entry): whole-row staging, fused quantiser, per-wave windows, K slices of the weight-streaming kernel (slabs in a
# workspace and in the static array), K slices of the large-M kernel, the two-phase large-M launch
CASES = [(3, 520, 2080, "tiled"), (2, 520, 2080, "fused"), (16, 1000, 5120, "tiled"), (48, 300, 13824, "splitk"),
         (48, 300, 13824, "static"), (130, 520, 8192, "splitk"), (130, 520, 8192, "static"), (300, 17000, 160, "tiled")]


@pytest.mark.parametrize("M,N,K,how", CASES)
def test_graph_replays_match_eager(gpu, oracle, M, N, K, how):
    t = gpu
    w4a8.w4a8_init()
    w = t.from_numpy(synth.weights_fp16(N, K, config_id=90)).cuda()
    wp, s_w = w4a8.w4a8_quantize_weights(w)
    wt = w4a8.w4a8_tile_weights(wp)
    xs = [t.from_numpy(synth.activations_fp16(M, K, config_id=90, tag=10 + i)).cuda() for i in range(4)]
    x = xs[0].clone()
    xq = t.empty((M, K), dtype=t.int8, device="cuda")
    s_a = t.empty((M,), dtype=t.float32, device="cuda")
    out = t.empty((M, N), dtype=t.float16, device="cuda")
    ws = t.empty((max(16, 8 * M * N * 4),), dtype=t.uint8, device="cuda")

    eager = []
    for xi in xs:
        x.copy_(xi)
        _linear(t, M, wt, s_w, x, xq, s_a, out, how, ws)
        eager.append(out.clone())
    t.cuda.synchronize()

    x.copy_(xs[0])
    side = t.cuda.Stream()
    side.wait_stream(t.cuda.current_stream())
    graph = t.cuda.CUDAGraph()
    with t.cuda.stream(side):
        with t.cuda.graph(graph):
            _linear(t, M, wt, s_w, x, xq, s_a, out, how, ws)
    t.cuda.current_stream().wait_stream(side)
    for rnd in range(2):
        for i, xi in enumerate(xs):
            x.copy_(xi)                      # eager work between the replays
            out.fill_(7.0)
            ws[: min(ws.numel(), 1 << 16)].fill_(0x5A)
            graph.replay()
            t.cuda.synchronize()
            assert bool((out.view(t.int16) == eager[i].view(t.int16)).all()), f"replay {rnd}.{i} of {how} M={M} differs from eager"
    # and the eager result is the oracle's
    xq_o, s_a_o = oracle.quantize_act(xs[3].cpu().numpy())
    wq_o, s_w_o = oracle.quantize_weights_rtn(w.cpu().numpy())
    acc_o, y32, _ = oracle.gemm(xq_o, s_a_o, oracle.pack_w4(wq_o), s_w_o)
    got = eager[3].cpu().numpy().astype(np.float64)
    y = y32.astype(np.float64)
    assert np.all(np.abs(got - y) <= np.maximum(2.0 ** -10 * np.abs(y), 2.0 ** -24))


@pytest.mark.parametrize("M,I,K,how", [(2, 256, 2080, "fused"), (16, 512, 5120, "tiled"), (48, 160, 5120, "tiled"),
                                       (300, 8512, 160, "tiled")])
def test_graph_replays_of_the_swiglu_entries_match_eager(gpu, M, I, K, how):
    """The entries with SiLU*up in the GEMM's epilogue, captured and replayed the same way (their eager results are
    checked against the oracle in test_gpu_swiglu.py; here against the chain of separate calls)."""
    t = gpu
    w4a8.w4a8_init()
    w = t.from_numpy(synth.weights_fp16(2 * I, K, config_id=91)).cuda()
    wp_i, s_w_i = w4a8.w4a8_quantize_weights(w4a8.interleave_gate_up(w))
    wt_i = w4a8.w4a8_tile_weights(wp_i)
    wp, s_w = w4a8.w4a8_quantize_weights(w)
    wt = w4a8.w4a8_tile_weights(wp)
    xs = [t.from_numpy(synth.activations_fp16(M, K, config_id=91, tag=20 + i)).cuda() for i in range(3)]
    x = xs[0].clone()
    xq = t.empty((M, K), dtype=t.int8, device="cuda")
    s_a = t.empty((M,), dtype=t.float32, device="cuda")
    h = t.empty((M, I), dtype=t.float16, device="cuda")

    def launch():
        if how == "fused":
            w4a8.w4a8_linear_tiled_swiglu_fp16(x, wt_i, s_w_i, h=h)
        else:
            w4a8.w4a8_quantize_act(x, xq, s_a)
            w4a8.w4a8_gemm_tiled_swiglu(xq, s_a, wt_i, s_w_i, h=h)

    eager = []
    for xi in xs:
        x.copy_(xi)
        launch()
        eager.append(h.clone())
        q, sa = w4a8.w4a8_quantize_act(x)
        chain = w4a8.w4a8_silu_mul(w4a8.w4a8_gemm_tiled(q, sa, wt, s_w))
        assert bool((eager[-1].view(t.int16) == chain.view(t.int16)).all()), "eager result differs from the separate calls"
    t.cuda.synchronize()
    x.copy_(xs[0])
    side = t.cuda.Stream()
    side.wait_stream(t.cuda.current_stream())
    graph = t.cuda.CUDAGraph()
    with t.cuda.stream(side):
        with t.cuda.graph(graph):
            launch()
    t.cuda.current_stream().wait_stream(side)
    for rnd in range(2):
        for i, xi in enumerate(xs):
            x.copy_(xi)
            h.fill_(7.0)
            graph.replay()
            t.cuda.synchronize()
            assert bool((h.view(t.int16) == eager[i].view(t.int16)).all()), f"replay {rnd}.{i} of {how} M={M} differs from eager"


@pytest.mark.parametrize("M,K", [(3, 5120), (300, 1056)])
def test_graph_replays_of_the_fused_norm_quantiser_match_eager(gpu, M, K):
    """w4a8_add_rmsnorm_quantize with the residual stream updated in place, captured and replayed the same way (its
    eager results are checked against the oracle in test_gpu_rmsnorm.py)."""
    t = gpu
    xs = [t.from_numpy(synth.activations_fp16(M, K, config_id=92, tag=30 + i)).cuda() for i in range(3)]
    res0 = t.from_numpy(synth.activations_fp16(M, K, config_id=92, tag=40)).cuda()
    g = t.from_numpy(np.linspace(0.5, 1.5, K).astype(np.float16)).cuda()
    x, res = xs[0].clone(), res0.clone()
    xq = t.empty((M, K), dtype=t.int8, device="cuda")
    s_a = t.empty((M,), dtype=t.float32, device="cuda")
    eager = []
    for xi in xs:
        x.copy_(xi)
        res.copy_(res0)
        w4a8.w4a8_add_rmsnorm_quantize(x, res, g, 1e-5, r_out=res, xq=xq, s_a=s_a)
        eager.append((xq.clone(), s_a.clone(), res.clone()))
    t.cuda.synchronize()
    side = t.cuda.Stream()
    side.wait_stream(t.cuda.current_stream())
    graph = t.cuda.CUDAGraph()
    with t.cuda.stream(side):
        with t.cuda.graph(graph):
            w4a8.w4a8_add_rmsnorm_quantize(x, res, g, 1e-5, r_out=res, xq=xq, s_a=s_a)
    t.cuda.current_stream().wait_stream(side)
    for rnd in range(2):
        for i, xi in enumerate(xs):
            x.copy_(xi)
            res.copy_(res0)
            xq.fill_(5)
            graph.replay()
            t.cuda.synchronize()
            assert bool((xq == eager[i][0]).all()) and bool((s_a.view(t.int32) == eager[i][1].view(t.int32)).all()), f"replay {rnd}.{i}"
            assert bool((res.view(t.int16) == eager[i][2].view(t.int16)).all()), f"replay {rnd}.{i}: residual"


@pytest.mark.parametrize("swiglu", [False, True])
def test_graph_replays_of_the_norm_linear_match_eager(gpu, swiglu):
    """w4a8_linear_tiled_norm_fp16 captured and replayed with new inputs (eager results checked in test_gpu_rmsnorm.py)."""
    t = gpu
    w4a8.w4a8_init()
    M, N, K = 2, 512, 5120
    w = t.from_numpy(synth.weights_fp16(N, K, config_id=93)).cuda()
    wp, s_w = w4a8.w4a8_quantize_weights(w4a8.interleave_gate_up(w) if swiglu else w)
    wt = w4a8.w4a8_tile_weights(wp)
    xs = [t.from_numpy(synth.activations_fp16(M, K, config_id=93, tag=50 + i)).cuda() for i in range(3)]
    res = t.from_numpy(synth.activations_fp16(M, K, config_id=93, tag=60)).cuda()
    g = t.from_numpy(np.linspace(0.5, 1.5, K).astype(np.float16)).cuda()
    x = xs[0].clone()
    out = t.empty((M, N // 2 if swiglu else N), dtype=t.float16, device="cuda")
    r_out = t.empty((M, K), dtype=t.float16, device="cuda")
    eager = []
    for xi in xs:
        x.copy_(xi)
        w4a8.w4a8_linear_tiled_norm_fp16(x, res, g, 1e-5, wt, s_w, swiglu=swiglu, out=out, r_out=r_out)
        eager.append((out.clone(), r_out.clone()))
    t.cuda.synchronize()
    side = t.cuda.Stream()
    side.wait_stream(t.cuda.current_stream())
    graph = t.cuda.CUDAGraph()
    with t.cuda.stream(side):
        with t.cuda.graph(graph):
            w4a8.w4a8_linear_tiled_norm_fp16(x, res, g, 1e-5, wt, s_w, swiglu=swiglu, out=out, r_out=r_out)
    t.cuda.current_stream().wait_stream(side)
    for rnd in range(2):
        for i, xi in enumerate(xs):
            x.copy_(xi)
            out.fill_(7.0)
            r_out.fill_(7.0)
            graph.replay()
            t.cuda.synchronize()
            assert bool((out.view(t.int16) == eager[i][0].view(t.int16)).all()), f"replay {rnd}.{i}: output"
            assert bool((r_out.view(t.int16) == eager[i][1].view(t.int16)).all()), f"replay {rnd}.{i}: residual"
