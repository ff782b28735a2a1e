"""GPU parity of the token-generation linear that quantises its own activations (w4a8_linear_tiled_fp16): against the
CPU oracle's two steps (per-token quantiser, then GEMM with the epilogue of Eq. (6),(7)) and, bit for bit, against the
library's own two calls, through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu


def _check(t, oracle, x, w, what, view=None):
    """x: numpy fp16 [M][K] (the logical input); view: optional device view of a wider matrix holding the same rows."""
    M, K = x.shape
    N = w.shape[0]
    xq_o, s_a_o = oracle.quantize_act(x)
    wq_o, s_w_o = oracle.quantize_weights_rtn(w)
    wp = oracle.pack_w4(wq_o)
    acc_o, y32, _ = oracle.gemm(xq_o, s_a_o, wp, s_w_o)
    dx = t.from_numpy(x).cuda() if view is None else view
    dwt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    dsw = t.from_numpy(s_w_o).cuda()
    s_a = t.full((M,), -1.0, dtype=t.float32, device="cuda")
    out = w4a8.w4a8_linear_tiled_fp16(dx, dwt, dsw, s_a_out=s_a)
    xq2, sa2 = w4a8.w4a8_quantize_act_strided(dx)
    ref = w4a8.w4a8_gemm_tiled(xq2, sa2, dwt, dsw)
    t.cuda.synchronize()
    assert_equal_bits(s_a.cpu().numpy().view(np.uint32), s_a_o.view(np.uint32), what + " s_a")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what + " out")
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), what + " vs two calls")


@pytest.mark.parametrize("M", [1, 2, 3, 4])
@pytest.mark.parametrize("N,K", [(16, 32), (100, 160), (520, 2080), (1001, 4096), (5120, 5120), (300, 8192), (136, 11008),
                                 (200, 13824)])
def test_fused_linear_matches_oracle_and_two_calls(gpu, oracle, M, N, K):
    if M * K > 45000:
        pytest.skip("the rows do not fit in LDS twice over: refused (see test_fused_linear_refuses_what_it_cannot_hold)")
    x = synth.activations_fp16(M, K, config_id=2, tag=70)
    w = synth.weights_fp16(N, K, config_id=70)
    _check(gpu, oracle, x, w, f"fused linear M={M} N={N} K={K}")


def test_fused_linear_rounding_ties_zero_rows_and_strided_input(gpu, oracle):
    t = gpu
    M, N, K = 4, 264, 1024
    x = synth.activations_fp16(M, K, config_id=2, tag=71)
    x[0, :] = 0                        # an all-zero token: scale 0, codes 0, output 0
    x[1, :] = 0
    x[1, 5], x[1, 6], x[1, 7], x[1, 8], x[1, 9] = 127.0, 0.5, 1.5, 2.5, -3.5   # scale 1: exact halves, round to even
    x[2, :] = np.float16(1e-7)         # fp16 subnormals
    x[3, :] = np.linspace(-63.5, 63.5, K).astype(np.float16)
    x[3, 0] = 127.0                    # scale 1 again: many quotients on or near halves
    w = synth.weights_fp16(N, K, config_id=71)
    _check(t, oracle, x, w, "fused linear special rows")
    # the same rows as a column slice of a wider matrix (ldx > K)
    wide = np.zeros((M, 3 * K), np.float16)
    wide[:, K:2 * K] = x
    dwide = t.from_numpy(wide).cuda()
    _check(t, oracle, x, w, "fused linear strided input", view=dwide[:, K:2 * K])


def test_fused_linear_refuses_what_it_cannot_hold(gpu):
    t = gpu
    for M, N, K in [(5, 64, 1024), (4, 64, 16384), (4, 136, 13824), (3, 64, 28672)]:
        x = t.zeros((M, K), dtype=t.float16, device="cuda")
        wt = t.zeros((w4a8.w4a8_tiled_weight_bytes(N, K),), dtype=t.uint8, device="cuda")
        s_w = t.ones((N,), dtype=t.float32, device="cuda")
        with pytest.raises(w4a8.W4A8Error) as e:
            w4a8.w4a8_linear_tiled_fp16(x, wt, s_w)
        assert e.value.code == -7


@pytest.mark.parametrize("M", [1, 4])
@pytest.mark.parametrize("name", ["qkv", "o", "gate_up"])
def test_fused_linear_llama13b_shapes_sampled(gpu, oracle, name, M):
    """Full size: all M rows, a seeded sample of output channels against the oracle; everything against the two calls."""
    t = gpu
    N, K = synth.LLAMA_SHAPES["13b"][name]
    x = synth.activations_fp16(M, K, config_id=3, tag=72)
    w = synth.weights_fp16(N, K, config_id=3)
    dw = t.from_numpy(w).cuda()
    wp, s_w = w4a8.w4a8_quantize_weights(dw)
    wt = w4a8.w4a8_tile_weights(wp)
    dx = t.from_numpy(x).cuda()
    out = w4a8.w4a8_linear_tiled_fp16(dx, wt, s_w)
    xq2, sa2 = w4a8.w4a8_quantize_act(dx)
    ref = w4a8.w4a8_gemm_tiled(xq2, sa2, wt, s_w)
    t.cuda.synchronize()
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), f"{name} M={M} vs two calls")
    cols = np.sort(np.random.default_rng(72).choice(N, 256, replace=False))
    xq_o, s_a_o = oracle.quantize_act(x)
    wq_o, s_w_o = oracle.quantize_weights_rtn(np.ascontiguousarray(w[cols]))
    acc_o, y32, _ = oracle.gemm(xq_o, s_a_o, oracle.pack_w4(wq_o), s_w_o)
    assert_fp16_close(out.cpu().numpy()[:, cols], y32, acc_o, f"{name} M={M} sampled channels")
