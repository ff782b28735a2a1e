"""GPU parity of the row-wise kernels (activation quantiser, weight quantiser +
packer, SiLU*up glue) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, SUBNORMAL_STEP, FP16_MIN_NORMAL, REL_TOL

pytestmark = pytest.mark.gpu


def _quant_act_gpu(torch, x):
    xq, s_a = w4a8.w4a8_quantize_act(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    return xq.cpu().numpy(), s_a.cpu().numpy()


@pytest.mark.parametrize("M,K", [(1, 32), (3, 96), (1, 4096), (16, 5120), (5, 11008), (33, 13824), (2, 16384),
                                 (2, 16416), (3, 28672), (1, 65536), (257, 1024), (128, 13824), (129, 5120), (256, 16416),
                                 (300, 28672)])
def test_quantize_act_bit_exact(gpu, oracle, M, K):
    x = synth.activations_fp16(M, K, tag=11)
    xq, s_a = _quant_act_gpu(gpu, x)
    xq_o, s_o = oracle.quantize_act(x)
    assert_equal_bits(s_a.view(np.uint32), s_o.view(np.uint32), f"s_a M={M} K={K}")
    assert_equal_bits(xq, xq_o, f"xq M={M} K={K}")


def test_quantize_act_ties_zero_rows_and_scales(gpu, oracle):
    K = 256
    g = synth.rng(920)
    x = (g.standard_normal((12, K)) * 3).astype(np.float16)
    x[0, :] = 0                                       # all-zero token
    x[1, :] = 0; x[1, 7] = np.float16(-3.0)           # single non-zero
    x[2, :10] = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 126.5, -126.5], np.float16)
    x[2, 10:] = 0                                     # scale exactly 1: ties decide the codes
    x[3, :] = np.float16(6e-8)                        # smallest subnormal everywhere
    x[4, :] = np.float16(65504.0); x[4, 1] = np.float16(-65504.0)
    x[5, :] *= np.float16(1e-3)
    x[6, :] *= np.float16(300.0)
    xq, s_a = _quant_act_gpu(gpu, x)
    xq_o, s_o = oracle.quantize_act(x)
    assert_equal_bits(s_a.view(np.uint32), s_o.view(np.uint32), "s_a")
    assert_equal_bits(xq, xq_o, "xq")
    assert list(xq[2, :10]) == [127, 0, 2, 2, 0, -2, -2, 4, 126, -126]
    assert s_a[0] == 0 and not xq[0].any()


def test_quantize_act_where_division_and_reciprocal_differ(gpu, oracle):
    """Rows on which x * (1/s) would give another code than x / s (Eq. (2) divides)."""
    g = synth.rng(904)
    rows = []
    for _ in range(400):
        x = (g.standard_normal(256) * g.uniform(0.1, 30)).astype(np.float16)
        xf = x.astype(np.float32)
        s = np.float32(np.abs(xf).max() / np.float32(127.0))
        if (np.rint(xf / s) != np.rint(xf * (np.float32(1.0) / s))).any():
            rows.append(x)
    assert len(rows) >= 3
    x = np.stack(rows)
    xq, s_a = _quant_act_gpu(gpu, x)
    xq_o, s_o = oracle.quantize_act(x)
    assert_equal_bits(s_a.view(np.uint32), s_o.view(np.uint32), "s_a")
    assert_equal_bits(xq, xq_o, "xq")


@pytest.mark.parametrize("N,K", [(1, 32), (7, 96), (64, 4096), (33, 5120), (4, 28672)])
def test_quantize_weights_bit_exact(gpu, oracle, N, K):
    w = synth.weights_fp16(N, K)
    if N > 2:
        w[1, :] = 0
        w[2, 0] = np.float16(-1.0)
    wp, s_w = w4a8.w4a8_quantize_weights(gpu.from_numpy(w).cuda())
    gpu.cuda.synchronize()
    wq_o, s_o = oracle.quantize_weights_rtn(w)
    assert_equal_bits(s_w.cpu().numpy().view(np.uint32), s_o.view(np.uint32), "s_w")
    assert_equal_bits(wp.cpu().numpy(), oracle.pack_w4(wq_o), "wp")


@pytest.mark.parametrize("N,K", [(1, 32), (7, 96), (64, 4096), (33, 5120), (4, 28672)])
def test_quantize_weights_clipped_bit_exact(gpu, oracle, N, K):
    """Eq. (8),(9) with per-channel clipping strengths: codes (saturating at -8 / 7) and scales bit-exact."""
    g = synth.rng(924, N, K)
    w = synth.weights_fp16(N, K, config_id=8)
    if N > 2:
        w[1, :] = 0
        w[2, 0] = np.float16(-1.0)
    gamma = g.uniform(0.25, 1.0, N).astype(np.float32)
    beta = g.uniform(0.25, 1.0, N).astype(np.float32)
    dw = gpu.from_numpy(w).cuda()
    for ga, be in ((gamma, beta), (gamma, None), (None, beta), (None, None)):
        wp, s_w = w4a8.w4a8_quantize_weights_clipped(dw, None if ga is None else gpu.from_numpy(ga).cuda(),
                                                     None if be is None else gpu.from_numpy(be).cuda())
        gpu.cuda.synchronize()
        wq_o, s_o = oracle.quantize_weights_clip(w, ga, be)
        assert_equal_bits(s_w.cpu().numpy().view(np.uint32), s_o.view(np.uint32), "s_w")
        assert_equal_bits(wp.cpu().numpy(), oracle.pack_w4(wq_o), "wp")
    if N >= 33:
        assert wq_o.min() == -7                      # last pass had no clipping: plain RTN never reaches -8
        wq_c, _ = oracle.quantize_weights_clip(w, gamma, beta)
        assert wq_c.min() == -8 and wq_c.max() == 7  # the clipped one saturates
    # the unclipped call is the plain quantiser
    wp0, s0 = w4a8.w4a8_quantize_weights(dw)
    gpu.cuda.synchronize()
    assert_equal_bits(wp.cpu().numpy(), wp0.cpu().numpy(), "clipped(None, None) vs plain: wp")
    assert_equal_bits(s_w.cpu().numpy().view(np.uint32), s0.cpu().numpy().view(np.uint32), "clipped(None, None) vs plain: s_w")


@pytest.mark.parametrize("M,I", [(1, 8), (3, 104), (16, 13824), (130, 1024)])
def test_silu_mul_close(gpu, oracle, M, I):
    g = synth.rng(921, M, I)
    gu = (g.standard_normal((M, 2 * I)) * 4).astype(np.float16)
    gu[0, 0] = 0
    gu[0, 1] = np.float16(-65504.0)
    gu[0, 2] = np.float16(65504.0); gu[0, I + 2] = np.float16(1.0)
    gu[0, 3] = np.float16(-20.0)
    h = w4a8.w4a8_silu_mul(gpu.from_numpy(gu).cuda())
    gpu.cuda.synchronize()
    y64, _ = oracle.silu_mul(gu)
    o = h.cpu().numpy().astype(np.float64)
    finite = np.abs(y64) < 65520.0
    assert np.all(np.isinf(o[~finite])) and np.all(np.isfinite(o[finite]))
    err = np.abs(o - y64)
    normal = finite & (np.abs(y64) >= FP16_MIN_NORMAL)
    assert np.all(err[normal] <= REL_TOL * np.abs(y64[normal]))
    assert np.all(err[finite & ~normal] <= SUBNORMAL_STEP)


@pytest.mark.parametrize("M,I", [(1, 32), (3, 96), (16, 13824), (130, 1024), (2, 16416)])
def test_silu_mul_quantize_equals_the_two_kernels_and_the_oracle(gpu, oracle, M, I):
    """Stage-wise parity of the fused glue + quantiser: its codes and scales are those of quantising the GPU's own
    fp16 intermediate (bit-exact against the oracle's quantiser fed that intermediate)."""
    g = synth.rng(922, M, I)
    gu = (g.standard_normal((M, 2 * I)) * 3).astype(np.float16)
    gu[0, :8] = 0
    d = gpu.from_numpy(gu).cuda()
    h = w4a8.w4a8_silu_mul(d)
    xq2, sa2 = w4a8.w4a8_quantize_act(h)
    xq, sa = w4a8.w4a8_silu_mul_quantize(d)
    gpu.cuda.synchronize()
    assert_equal_bits(xq.cpu().numpy(), xq2.cpu().numpy(), "fused vs two kernels: codes")
    assert_equal_bits(sa.cpu().numpy().view(np.uint32), sa2.cpu().numpy().view(np.uint32), "fused vs two kernels: scales")
    xq_o, sa_o = oracle.quantize_act(h.cpu().numpy())
    assert_equal_bits(xq.cpu().numpy(), xq_o, "codes vs oracle on the GPU's intermediate")
    assert_equal_bits(sa.cpu().numpy().view(np.uint32), sa_o.view(np.uint32), "scales vs oracle")


def test_quantizers_on_adversarial_quotients(gpu, oracle):
    """Rows built so that many quotients x / s_a sit exactly on, or within an ulp of, a half-integer: the shortcut
    of the quantiser must fall back to the division there."""
    g = synth.rng(923)
    rows = []
    for amax in (127.0, 63.5, 254.0, 31.75, 1016.0, 0.9921875):
        s = amax / 127.0
        ks = g.integers(-126, 127, size=255).astype(np.float64) + 0.5
        x = np.concatenate([[amax], ks * s]).astype(np.float16)
        rows.append(x)
        x2 = x.copy(); x2[1:] = np.nextafter(x2[1:], np.float16(np.inf)); rows.append(x2)
        x3 = x.copy(); x3[1:] = np.nextafter(x3[1:], np.float16(-np.inf)); rows.append(x3)
    x = np.stack(rows)
    xq, s_a = _quant_act_gpu(gpu, x)
    xq_o, s_o = oracle.quantize_act(x)
    assert_equal_bits(s_a.view(np.uint32), s_o.view(np.uint32), "s_a")
    assert_equal_bits(xq, xq_o, "xq")
    w = np.stack([np.concatenate([[7.0 * sc], (g.integers(-7, 7, size=255) + 0.5) * sc]).astype(np.float16) for sc in (1.0, 0.5, 0.03125, 3.0)])
    wp, s_w = w4a8.w4a8_quantize_weights(gpu.from_numpy(w).cuda())
    gpu.cuda.synchronize()
    wq_o, sw_o = oracle.quantize_weights_rtn(w)
    assert_equal_bits(s_w.cpu().numpy().view(np.uint32), sw_o.view(np.uint32), "s_w")
    assert_equal_bits(wp.cpu().numpy(), oracle.pack_w4(wq_o), "wp")


@pytest.mark.parametrize("M,K,ld,col0", [(1, 32, 96, 32), (5, 160, 480, 160), (16, 5120, 15360, 0), (130, 1024, 3080, 1032)])
def test_quantize_act_strided_column_block(gpu, oracle, M, K, ld, col0):
    """A block of K columns of a wider fp16 matrix, quantised in place: bit-exact against the oracle on that block."""
    wide = synth.activations_fp16(M, ld, config_id=97, tag=5)
    d = gpu.from_numpy(wide).cuda()
    xq, s_a = w4a8.w4a8_quantize_act_strided(d[:, col0:col0 + K])
    gpu.cuda.synchronize()
    xq_o, s_a_o = oracle.quantize_act(np.ascontiguousarray(wide[:, col0:col0 + K]))
    assert_equal_bits(xq.cpu().numpy(), xq_o, "strided quantiser codes")
    assert_equal_bits(s_a.cpu().numpy().view(np.uint32), s_a_o.view(np.uint32), "strided quantiser scales")
