"""GPU parity of the W4A8 GEMM against the CPU oracle, through the C ABI:
raw int32 sums bit-exact, fp16 outputs within 2^-10 relative of the oracle's
fp32 epilogue value."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu

RESIDENT, STREAM, PREFILL = w4a8.TILING_DECODE_RESIDENT, w4a8.TILING_DECODE_STREAM, w4a8.TILING_PREFILL


def _codes(M, N, K, tag=1):
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=tag)
    return xq, wq, s_a, s_w


def _run_both(torch, oracle, xq, wq, s_a, s_w, tiling, variant, what):
    """Run the forced tiling on the GPU (raw sums and fp16 output) and compare with the oracle."""
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    d = dict(xq=torch.from_numpy(xq).cuda(), s_a=torch.from_numpy(s_a).cuda(),
             wp=torch.from_numpy(wp).cuda(), s_w=torch.from_numpy(s_w).cuda())
    acc = w4a8.w4a8_gemm_tuned(d["xq"], None, d["wp"], None, tiling, variant, want_acc=True)
    out = w4a8.w4a8_gemm_tuned(d["xq"], d["s_a"], d["wp"], d["s_w"], tiling, variant)
    torch.cuda.synchronize()
    assert_equal_bits(acc.cpu().numpy(), acc_o, what + " acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what + " out")


def test_config1_full_parity(gpu, oracle):
    """M=8, N=1024, K=1024, uniform codes, seed 0: the whole matrix, default tiling choice."""
    xq, wq, s_a, s_w = _codes(8, 1024, 1024)
    wp = oracle.pack_w4(wq)
    assert np.array_equal(w4a8.w4a8_pack_weights_host(wq), wp)
    acc_o, y32, out_o = oracle.gemm(xq, s_a, wp, s_w)
    t = gpu
    dxq, dsa = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda()
    dwp, dsw = t.from_numpy(wp).cuda(), t.from_numpy(s_w).cuda()
    acc = w4a8.w4a8_gemm_acc_i32(dxq, dwp)
    out = w4a8.w4a8_gemm(dxq, dsa, dwp, dsw)
    t.cuda.synchronize()
    assert_equal_bits(acc.cpu().numpy(), acc_o, "config 1 acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, "config 1 out")
    # same fp32 epilogue arithmetic on both sides: the fp16 bits agree as well
    assert np.mean(out.cpu().numpy().view(np.uint16) == out_o.view(np.uint16)) > 0.999


@pytest.mark.parametrize("M", [1, 2, 3, 5, 7, 8, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64])
def test_stream_tiling_all_m(gpu, oracle, M):
    xq, wq, s_a, s_w = _codes(M, 200, 1056, tag=30)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, STREAM, 0, f"stream M={M}")


@pytest.mark.parametrize("variant", [104, 108, 204, 208])
@pytest.mark.parametrize("M", [3, 16, 40, 64])
def test_stream_tiling_variants(gpu, oracle, M, variant):
    if M > 48 and variant == 208:
        pytest.skip("4 column tiles x 2 row tiles x 8 waves exceeds LDS; the library rejects it")
    xq, wq, s_a, s_w = _codes(M, 328, 2080, tag=34)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, STREAM, variant, f"stream variant={variant} M={M}")


@pytest.mark.parametrize("N,K", [(1, 32), (16, 32), (17, 64), (24, 96), (1000, 128), (1001, 160), (30, 4128),
                                 (4096, 1024), (520, 11008), (40, 28672)])
@pytest.mark.parametrize("M", [1, 16, 37])
def test_stream_tiling_ragged_shapes(gpu, oracle, M, N, K):
    xq, wq, s_a, s_w = _codes(M, N, K, tag=31)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, STREAM, 0, f"stream M={M} N={N} K={K}")


@pytest.mark.parametrize("M", [1, 2, 3, 5, 7, 8, 15, 16])
@pytest.mark.parametrize("N,K", [(1, 32), (16, 32), (17, 64), (24, 96), (1000, 128), (1001, 160), (30, 4128), (4096, 1024),
                                 (8200, 2048), (520, 5120), (300, 11008), (520, 13824), (40, 16384)])
def test_resident_tiling_m_up_to_16(gpu, oracle, M, N, K):
    xq, wq, s_a, s_w = _codes(M, N, K, tag=35)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, RESIDENT, 0, f"resident M={M} N={N} K={K}")


@pytest.mark.parametrize("M", [17, 24, 31, 32])
@pytest.mark.parametrize("N,K", [(16, 32), (1001, 160), (520, 5120), (700, 8192), (30, 4128)])
def test_resident_tiling_m_up_to_32(gpu, oracle, M, N, K):
    xq, wq, s_a, s_w = _codes(M, N, K, tag=36)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, RESIDENT, 0, f"resident M={M} N={N} K={K}")


@pytest.mark.parametrize("waves,grid", [(8, 1), (8, 7), (8, 512), (16, 1), (16, 3), (16, 100), (16, 256), (16, 4096)])
@pytest.mark.parametrize("M,N,K", [(1, 5120, 512), (16, 1000, 2080), (9, 130, 5120)])
def test_resident_tiling_grid_and_wave_variants(gpu, oracle, M, N, K, waves, grid):
    """Any persistent grid size gives the same bits: few workgroups walk many row blocks each, many walk one."""
    xq, wq, s_a, s_w = _codes(M, N, K, tag=37)
    if -(-N // grid) > 512:
        # more than 512 output channels per workgroup are refused (their scales are staged in LDS)
        with pytest.raises(w4a8.W4A8Error) as e:
            w4a8.w4a8_gemm_tuned(gpu.from_numpy(xq).cuda(), None, gpu.from_numpy(oracle.pack_w4(wq)).cuda(), None,
                                 RESIDENT, waves * 100000 + grid, want_acc=True)
        assert e.value.code == -7
        return
    _run_both(gpu, oracle, xq, wq, s_a, s_w, RESIDENT, waves * 100000 + grid, f"resident {waves}w grid={grid} M={M} N={N} K={K}")


def test_back_to_back_calls_share_nothing(gpu, oracle):
    """Calls of different shapes in a row on one stream, no synchronisation in between."""
    t = gpu
    jobs = []
    for i, (M, N, K) in enumerate([(16, 1024, 4096), (3, 520, 2048), (1, 48, 512), (16, 1024, 4096), (40, 4096, 1024),
                                   (200, 300, 1024)]):
        xq, wq, s_a, s_w = _codes(M, N, K, tag=33 + i)
        wp = oracle.pack_w4(wq)
        jobs.append((t.from_numpy(xq).cuda(), t.from_numpy(wp).cuda(), oracle.gemm_acc_i32(xq, wp)))
    accs = [w4a8.w4a8_gemm_acc_i32(dx, dw) for dx, dw, _ in jobs for _ in range(2)]
    t.cuda.synchronize()
    for i, acc in enumerate(accs):
        assert_equal_bits(acc.cpu().numpy(), jobs[i // 2][2], f"call {i}")


PREFILL_TILES = [1, 2, 3, 4, 5, 6, 7, 8]   # register-staged 128x256 (1x4 waves), 128x128, 128x160, 128x256 (2x2 waves); 5..8: the same four shapes, LDS-direct loads


@pytest.mark.parametrize("tile", PREFILL_TILES)
@pytest.mark.parametrize("M", [1, 17, 64, 65, 127, 128, 129, 300])
def test_prefill_tiling_all_m(gpu, oracle, M, tile):
    xq, wq, s_a, s_w = _codes(M, 520, 1056, tag=40)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, PREFILL, tile, f"prefill tile={tile} M={M}")


@pytest.mark.parametrize("M,N,K", [(130, 1, 32), (128, 255, 64), (256, 256, 96), (100, 257, 128), (200, 1001, 160),
                                   (70, 1000, 4128), (1024, 512, 1024), (384, 300, 5120)])
@pytest.mark.parametrize("tile", PREFILL_TILES)
def test_prefill_tiling_ragged_shapes(gpu, oracle, M, N, K, tile):
    xq, wq, s_a, s_w = _codes(M, N, K, tag=41)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, PREFILL, tile, f"prefill tile={tile} M={M} N={N} K={K}")


@pytest.mark.parametrize("tiling,M", [(STREAM, 2), (STREAM, 40), (PREFILL, 130)])
def test_extreme_codes_at_max_k_do_not_overflow(gpu, oracle, tiling, M):
    """a = -128, w = -8 along all of K = 65536: the sixteen-fold sum is 2^30, inside int32 (Sec. 5.3)."""
    K, N = 65536, 48
    xq = np.full((M, K), -128, np.int8)
    xq[1, :] = 127
    wq = np.full((N, K), -8, np.int8)
    wq[1, :] = 7
    wq[2, ::2] = 0
    s_a = np.full(M, 2.0 ** -12, np.float32)
    s_w = np.full(N, 2.0 ** -12, np.float32)
    _run_both(gpu, oracle, xq, wq, s_a, s_w, tiling, 0, "extremes")


def test_invariants_on_gpu(gpu, oracle):
    """Zero weights give zero output; a single +-1 weight selects an activation column; doubling a scale doubles O."""
    t = gpu
    M, N, K = 16, 64, 256
    g = synth.rng(950)
    xq = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    dxq = t.from_numpy(xq).cuda()
    s_a = g.uniform(1e-3, 1e-2, M).astype(np.float32)
    s_w = g.uniform(1e-3, 1e-2, N).astype(np.float32)
    zero = w4a8.w4a8_gemm(dxq, t.from_numpy(s_a).cuda(), t.zeros((N, K // 2), dtype=t.uint8, device="cuda"),
                          t.from_numpy(s_w).cuda())
    assert not zero.any().item()
    wq = np.zeros((N, K), np.int8)
    ks = g.integers(0, K, N)
    sg = g.choice([-1, 1], N).astype(np.int8)
    wq[np.arange(N), ks] = sg
    dwp = t.from_numpy(w4a8.w4a8_pack_weights_host(wq)).cuda()
    acc = w4a8.w4a8_gemm_acc_i32(dxq, dwp).cpu().numpy()
    assert np.array_equal(acc, xq[:, ks].astype(np.int32) * sg.astype(np.int32))
    wq = g.integers(-8, 8, size=(N, K), dtype=np.int8)
    dwp = t.from_numpy(w4a8.w4a8_pack_weights_host(wq)).cuda()
    o1 = w4a8.w4a8_gemm(dxq, t.from_numpy(s_a).cuda(), dwp, t.from_numpy(s_w).cuda()).float()
    o2 = w4a8.w4a8_gemm(dxq, t.from_numpy(2 * s_a).cuda(), dwp, t.from_numpy(s_w).cuda()).float()
    o3 = w4a8.w4a8_gemm(dxq, t.from_numpy(s_a).cuda(), dwp, t.from_numpy(4 * s_w).cuda()).float()
    assert t.equal(o2, 2 * o1) and t.equal(o3, 4 * o1)


def _layer_inputs(oracle, M, N, K, tag):
    """Config 2/3 recipe: fp16 activations with outlier channels and fp16 N(0, 0.02) weights, quantised by the oracle."""
    x = synth.activations_fp16(M, K, tag=tag)
    w = synth.weights_fp16(N, K)
    xq, s_a = oracle.quantize_act(x)
    wq, s_w = oracle.quantize_weights_rtn(w)
    return x, w, xq, s_a, oracle.pack_w4(wq), s_w


@pytest.mark.parametrize("M", [1, 4, 16])
@pytest.mark.parametrize("N,K", [(4096, 4096), (4096, 11008)])
def test_llama7b_decode_shapes_full_parity(gpu, oracle, M, N, K):
    t = gpu
    x, w, xq, s_a, wp, s_w = _layer_inputs(oracle, M, N, K, tag=2)
    dxq, dsa = w4a8.w4a8_quantize_act(t.from_numpy(x).cuda())
    dwp, dsw = w4a8.w4a8_quantize_weights(t.from_numpy(w).cuda())
    assert_equal_bits(dxq.cpu().numpy(), xq, "xq")
    assert_equal_bits(dwp.cpu().numpy(), wp, "wp")
    acc = w4a8.w4a8_gemm_acc_i32(dxq, dwp)
    out = w4a8.w4a8_gemm(dxq, dsa, dwp, dsw)
    t.cuda.synchronize()
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    assert_equal_bits(acc.cpu().numpy(), acc_o, "acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, "out")


@pytest.mark.parametrize("M", [1, 16, 1024])
@pytest.mark.parametrize("name", ["qkv", "o", "gate_up", "down"])
def test_llama13b_full_size_sampled_parity(gpu, oracle, M, name):
    """Full LLaMA-13B shapes in the launch configuration the benchmark times; the oracle checks a seeded
    sample of output rows/columns (complete K sums), since the whole matrix would take it minutes."""
    t = gpu
    N, K = synth.LLAMA_SHAPES["13b"][name]
    x = synth.activations_fp16(M, K, tag=3)
    w = synth.weights_fp16(N, K, config_id=3)
    dxq, dsa = w4a8.w4a8_quantize_act(t.from_numpy(x).cuda())
    dwp, dsw = w4a8.w4a8_quantize_weights(t.from_numpy(w).cuda())
    acc = w4a8.w4a8_gemm_acc_i32(dxq, dwp)
    out = w4a8.w4a8_gemm(dxq, dsa, dwp, dsw)
    t.cuda.synchronize()
    g = synth.rng(960, M, N, K)
    rows = np.sort(g.choice(M, size=min(M, 24), replace=False))
    # columns: a few whole 16-wide tiles, the last columns, and scattered singles
    cols = np.unique(np.concatenate([np.arange(0, 32), np.arange(N - 16, N), g.choice(N, size=200, replace=False)]))
    xq_o, s_a_o = oracle.quantize_act(x[rows])
    wq_o, s_w_o = oracle.quantize_weights_rtn(np.ascontiguousarray(w[cols]))
    acc_o, y32, _ = oracle.gemm(xq_o, s_a_o, oracle.pack_w4(wq_o), s_w_o)
    assert_equal_bits(dxq.cpu().numpy()[rows], xq_o, "xq")
    assert_equal_bits(acc.cpu().numpy()[np.ix_(rows, cols)], acc_o, "acc sample")
    assert_fp16_close(out.cpu().numpy()[np.ix_(rows, cols)], y32, acc_o, "out sample")
    # properties that hold at any size: O = fp16(acc * s_a * s_w) recomputed from the GPU's own integers
    a = acc.cpu().numpy().astype(np.float32)
    y = a * (dsa.cpu().numpy()[:, None] * dsw.cpu().numpy()[None, :])
    assert_fp16_close(out.cpu().numpy(), y, None, "epilogue of full matrix")
