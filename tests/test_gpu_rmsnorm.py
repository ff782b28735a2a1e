"""GPU parity of the per-token quantiser fused behind the residual addition and RMSNorm (w4a8_add_rmsnorm_quantize),
stage by stage against the CPU oracle: r bit-exact, y within an fp16 rounding of the fp64 value, codes and scales
bit-exact on the y the GPU computed (the decision that makes integers is taken on the same fp16 values on both sides),
through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits

pytestmark = pytest.mark.gpu


def _gain(K, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(0.25, 2.0, K).astype(np.float16)


def _check(t, oracle, x, res, g, eps, what):
    M, K = x.shape
    dx, dg = t.from_numpy(x).cuda(), t.from_numpy(g).cuda()
    dres = None if res is None else t.from_numpy(res).cuda()
    r_out = t.empty((M, K), dtype=t.float16, device="cuda")
    y_out = t.empty((M, K), dtype=t.float16, device="cuda")
    xq, s_a = w4a8.w4a8_add_rmsnorm_quantize(dx, dres, dg, eps, r_out=r_out, y_out=y_out)
    xq2, s_a2 = w4a8.w4a8_add_rmsnorm_quantize(dx, dres, dg, eps)      # production form: neither r nor y written
    t.cuda.synchronize()
    r_o, y64, _ = oracle.add_rmsnorm(x, res, g, eps)
    assert_equal_bits(r_out.cpu().numpy().view(np.uint16), r_o.view(np.uint16), what + " r")
    y = y_out.cpu().numpy()
    big = np.abs(y64) >= 2.0 ** -14
    assert np.all(np.abs(y.astype(np.float64) - y64)[big] <= 2.0 ** -10 * np.abs(y64)[big]), what + " y"
    assert np.all(np.abs(y.astype(np.float64) - y64)[~big] <= 2.0 ** -24), what + " y (subnormal range)"
    xq_o, s_a_o = oracle.quantize_act(y)                                # the oracle's quantiser on the GPU's y
    assert_equal_bits(s_a.cpu().numpy().view(np.uint32), s_a_o.view(np.uint32), what + " s_a")
    assert_equal_bits(xq.cpu().numpy(), xq_o, what + " xq")
    assert_equal_bits(xq2.cpu().numpy(), xq_o, what + " xq without r / y outputs")
    assert_equal_bits(s_a2.cpu().numpy().view(np.uint32), s_a_o.view(np.uint32), what + " s_a without r / y outputs")
    return dx, dres, dg, r_out, xq, s_a


@pytest.mark.parametrize("with_res", [False, True])
@pytest.mark.parametrize("M,K", [(1, 32), (3, 96), (1, 4096), (16, 5120), (5, 8192), (2, 16384), (2, 16416), (3, 28672),
                                 (1, 65536), (130, 1024), (1024, 5120)])
def test_add_rmsnorm_quantize_stage_wise(gpu, oracle, M, K, with_res):
    x = synth.activations_fp16(M, K, config_id=2, tag=95)
    res = synth.activations_fp16(M, K, config_id=2, tag=96) if with_res else None
    _check(gpu, oracle, x, res, _gain(K, K), 1e-5, f"M={M} K={K} res={with_res}")


def test_add_rmsnorm_quantize_special_rows_and_in_place_residual(gpu, oracle):
    t = gpu
    M, K = 6, 16416                    # longer than what a thread keeps in registers: the later passes read r back
    x = synth.activations_fp16(M, K, config_id=2, tag=97)
    res = synth.activations_fp16(M, K, config_id=2, tag=98)
    x[0, :] = 0
    res[0, :] = 0                      # an all-zero row: y = 0, scale 0, codes 0 (eps > 0)
    res[1, :] = -x[1, :]               # cancels to a zero row
    x[2, :] = np.float16(2048)
    res[2, :] = np.float16(3)          # every sum is a tie in fp16 (2051 -> 2052)
    x[3, :] = np.float16(6e-8)
    res[3, :] = 0                      # fp16 subnormals: the mean square is far below eps
    x[4, :] = np.float16(60000)
    res[4, :] = np.float16(5000)       # sums near the top of the fp16 range (65000 rounds to 64992)
    g = _gain(K, 7)
    dx, dres, dg, r_ref, xq_ref, sa_ref = _check(t, oracle, x, res, g, 1e-5, "special rows")
    # the residual stream updated in place: r_out is the residual buffer itself
    res_buf = dres.clone()
    xq, s_a = w4a8.w4a8_add_rmsnorm_quantize(dx, res_buf, dg, 1e-5, r_out=res_buf)
    t.cuda.synchronize()
    assert bool((res_buf.view(t.int16) == r_ref.view(t.int16)).all()), "in-place residual differs"
    assert bool((xq == xq_ref).all()) and bool((s_a.view(t.int32) == sa_ref.view(t.int32)).all()), "in-place: codes differ"


def test_add_rmsnorm_quantize_refuses_bad_arguments(gpu):
    t = gpu
    x = t.zeros((2, 64), dtype=t.float16, device="cuda")
    g = t.ones((64,), dtype=t.float16, device="cuda")
    for eps in (-1.0, float("nan"), float("inf")):
        with pytest.raises(w4a8.W4A8Error) as e:
            w4a8.w4a8_add_rmsnorm_quantize(x, None, g, eps)
        assert e.value.code == -7
    with pytest.raises(w4a8.W4A8Error) as e:
        w4a8.w4a8_add_rmsnorm_quantize(t.zeros((2, 40), dtype=t.float16, device="cuda"), None,
                                       t.ones((40,), dtype=t.float16, device="cuda"), 1e-5)
    assert e.value.code == -2


@pytest.mark.parametrize("swiglu", [False, True])
@pytest.mark.parametrize("with_res", [False, True])
@pytest.mark.parametrize("M,N,K", [(1, 64, 32), (2, 192, 160), (3, 1024, 1056), (1, 2560, 5120), (4, 512, 4096), (2, 320, 8192),
                                   (1, 15360, 5120)])
def test_norm_linear_stage_wise(gpu, oracle, M, N, K, with_res, swiglu):
    """w4a8_linear_tiled_norm_fp16: r bit-exact and y within an fp16 rounding of the oracle; the output, bit for bit,
    what the linear without the norm gives on the y this call computed (which is itself checked against the oracle's
    quantiser and GEMM in test_gpu_fused_linear.py / test_gpu_swiglu.py)."""
    t = gpu
    if M * K > 27000:
        pytest.skip("the rows do not fit in LDS three times over: refused")
    x = synth.activations_fp16(M, K, config_id=2, tag=101)
    res = synth.activations_fp16(M, K, config_id=2, tag=102) if with_res else None
    g = _gain(K, K + 1)
    w = t.from_numpy(synth.weights_fp16(N, K, config_id=101)).cuda()
    wp, s_w = w4a8.w4a8_quantize_weights(w4a8.interleave_gate_up(w) if swiglu else w)
    wt = w4a8.w4a8_tile_weights(wp)
    dx, dg = t.from_numpy(x).cuda(), t.from_numpy(g).cuda()
    dres = None if res is None else t.from_numpy(res).cuda()
    r_out = t.empty((M, K), dtype=t.float16, device="cuda")
    y_out = t.empty((M, K), dtype=t.float16, device="cuda")
    s_a = t.empty((M,), dtype=t.float32, device="cuda")
    out = w4a8.w4a8_linear_tiled_norm_fp16(dx, dres, dg, 1e-5, wt, s_w, swiglu=swiglu, r_out=r_out, y_out=y_out, s_a_out=s_a)
    out2 = w4a8.w4a8_linear_tiled_norm_fp16(dx, dres, dg, 1e-5, wt, s_w, swiglu=swiglu)   # nothing but the output written
    ref = w4a8.w4a8_linear_tiled_swiglu_fp16(y_out, wt, s_w) if swiglu else w4a8.w4a8_linear_tiled_fp16(y_out, wt, s_w)
    t.cuda.synchronize()
    what = f"M={M} N={N} K={K} res={with_res} swiglu={swiglu}"
    r_o, y64, _ = oracle.add_rmsnorm(x, res, g, 1e-5)
    assert_equal_bits(r_out.cpu().numpy().view(np.uint16), r_o.view(np.uint16), what + " r")
    y = y_out.cpu().numpy()
    big = np.abs(y64) >= 2.0 ** -14
    assert np.all(np.abs(y.astype(np.float64) - y64)[big] <= 2.0 ** -10 * np.abs(y64)[big]), what + " y"
    assert np.all(np.abs(y.astype(np.float64) - y64)[~big] <= 2.0 ** -24), what + " y (subnormal range)"
    _, s_a_o = oracle.quantize_act(y)
    assert_equal_bits(s_a.cpu().numpy().view(np.uint32), s_a_o.view(np.uint32), what + " s_a")
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), what + " out vs the linear on y")
    assert_equal_bits(out2.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), what + " out without r / y outputs")


def test_norm_linear_strided_inputs_zero_rows_and_refusals(gpu, oracle):
    t = gpu
    M, N, K = 3, 264, 2080
    x = synth.activations_fp16(M, K, config_id=2, tag=103)
    res = synth.activations_fp16(M, K, config_id=2, tag=104)
    x[1, :] = 0
    res[1, :] = 0                                     # a zero row: y = 0, scale 0, output 0
    g = _gain(K, 3)
    w = t.from_numpy(synth.weights_fp16(N, K, config_id=103)).cuda()
    wp, s_w = w4a8.w4a8_quantize_weights(w)
    wt = w4a8.w4a8_tile_weights(wp)
    dg = t.from_numpy(g).cuda()
    dense = w4a8.w4a8_linear_tiled_norm_fp16(t.from_numpy(x).cuda(), t.from_numpy(res).cuda(), dg, 1e-5, wt, s_w)
    wide_x = t.zeros((M, 3 * K), dtype=t.float16, device="cuda")
    wide_r = t.zeros((M, 2 * K + 8), dtype=t.float16, device="cuda")
    wide_x[:, K:2 * K] = t.from_numpy(x).cuda()
    wide_r[:, 8:8 + K] = t.from_numpy(res).cuda()
    strided = w4a8.w4a8_linear_tiled_norm_fp16(wide_x[:, K:2 * K], wide_r[:, 8:8 + K], dg, 1e-5, wt, s_w)
    t.cuda.synchronize()
    assert_equal_bits(strided.cpu().numpy().view(np.uint16), dense.cpu().numpy().view(np.uint16), "strided inputs")
    assert bool((dense[1] == 0).all()), "zero row"
    for bad in (dict(M=5, K=1024), dict(M=1, K=8224)):            # beyond four tokens; beyond the hidden sizes it serves
        xb = t.zeros((bad["M"], bad["K"]), dtype=t.float16, device="cuda")
        wtb = t.zeros((w4a8.w4a8_tiled_weight_bytes(64, bad["K"]),), dtype=t.uint8, device="cuda")
        with pytest.raises(w4a8.W4A8Error) as e:
            w4a8.w4a8_linear_tiled_norm_fp16(xb, None, t.ones((bad["K"],), dtype=t.float16, device="cuda"), 1e-5, wtb,
                                             t.ones((64,), dtype=t.float32, device="cuda"))
        assert e.value.code == -7
