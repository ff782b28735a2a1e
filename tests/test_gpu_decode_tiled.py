"""GPU parity of the weight-streaming (token-generation) kernels reading the TILED weight array, so that one copy of
the weights serves every M: raw int32 sums bit-exact and fp16 within 2^-10 against the CPU oracle, and the bits of the
same kernels over the row-major array, through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu

RESIDENT_T, STREAM_T, AUTO_T = w4a8.TILING_DECODE_RESIDENT_TILED, w4a8.TILING_DECODE_STREAM_TILED, w4a8.TILING_AUTO_TILED


def _run(torch, oracle, M, N, K, tiling, variant, tag, what):
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=tag)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    dxq, dsa, dsw = torch.from_numpy(xq).cuda(), torch.from_numpy(s_a).cuda(), torch.from_numpy(s_w).cuda()
    wt = w4a8.w4a8_tile_weights(torch.from_numpy(wp).cuda())
    acc = w4a8.w4a8_gemm_tuned(dxq, None, wt, None, tiling, variant, want_acc=True, N=N)
    out = w4a8.w4a8_gemm_tuned(dxq, dsa, wt, dsw, tiling, variant, N=N)
    torch.cuda.synchronize()
    assert_equal_bits(acc.cpu().numpy(), acc_o, what + " acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what + " out")


@pytest.mark.parametrize("M", [1, 2, 3, 5, 7, 8, 15, 16])
@pytest.mark.parametrize("N,K", [(1, 32), (16, 32), (17, 64), (24, 96), (1000, 128), (1001, 160), (30, 4128), (4096, 1024),
                                 (8200, 2048), (520, 5120), (300, 11008), (520, 13824), (40, 16384)])
def test_resident_over_tiled_weights(gpu, oracle, M, N, K):
    _run(gpu, oracle, M, N, K, RESIDENT_T, 0, 90, f"resident/tiled M={M} N={N} K={K}")


@pytest.mark.parametrize("M", [17, 24, 32])
@pytest.mark.parametrize("N,K", [(16, 32), (1001, 160), (520, 5120), (700, 8192)])
def test_resident_over_tiled_weights_two_column_tiles(gpu, oracle, M, N, K):
    _run(gpu, oracle, M, N, K, RESIDENT_T, 0, 91, f"resident/tiled M={M} N={N} K={K}")


@pytest.mark.parametrize("waves,grid", [(8, 1), (8, 7), (16, 3), (16, 256), (16, 4096)])
@pytest.mark.parametrize("M,N,K", [(1, 5120, 512), (16, 1000, 2080), (9, 130, 5120)])
def test_resident_over_tiled_weights_grid_and_wave_variants(gpu, oracle, M, N, K, waves, grid):
    if -(-N // grid) > 512:
        pytest.skip("more than 512 channels per workgroup: refused (covered for the row-major array)")
    _run(gpu, oracle, M, N, K, RESIDENT_T, waves * 100000 + grid, 92, f"resident/tiled {waves}w grid={grid}")


@pytest.mark.parametrize("N,K", [(1, 32), (17, 64), (1001, 160), (30, 4128), (4096, 1024), (520, 11008), (40, 28672)])
@pytest.mark.parametrize("M", [1, 16, 37, 64])
def test_stream_over_tiled_weights(gpu, oracle, M, N, K):
    _run(gpu, oracle, M, N, K, STREAM_T, 0, 93, f"stream/tiled M={M} N={N} K={K}")


@pytest.mark.parametrize("variant", [104, 108, 204, 208])
@pytest.mark.parametrize("M", [3, 16, 40])
def test_stream_over_tiled_weights_variants(gpu, oracle, M, variant):
    _run(gpu, oracle, M, 328, 2080, STREAM_T, variant, 94, f"stream/tiled variant={variant} M={M}")


@pytest.mark.parametrize("M,N,K", [(1, 700, 2080), (16, 700, 2080), (17, 700, 2080), (4, 40, 28672), (300, 330, 1056)])
def test_one_weight_copy_serves_every_m(gpu, oracle, M, N, K):
    """w4a8_gemm_tiled (library's choice over the tiled array) returns the bits of w4a8_gemm over the row-major one,
    whichever kernel either of them picks; the split entry agrees as well."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=95)
    wp = oracle.pack_w4(wq)
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    dwp = t.from_numpy(wp).cuda()
    wt = w4a8.w4a8_tile_weights(dwp)
    a = w4a8.w4a8_gemm(dxq, dsa, dwp, dsw)
    b = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, dsw)
    c = w4a8.w4a8_gemm_tiled_splitk(dxq, dsa, wt, dsw)
    d = w4a8.w4a8_gemm_tuned(dxq, dsa, wt, dsw, AUTO_T, 0, N=N)
    t.cuda.synchronize()
    for name, other in (("tiled", b), ("tiled split entry", c), ("tuned, library's choice", d)):
        assert_equal_bits(other.cpu().numpy().view(np.uint16), a.cpu().numpy().view(np.uint16), f"{name} M={M}")
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    assert_fp16_close(b.cpu().numpy(), y32, acc_o, f"tiled entry M={M}")


def test_llama13b_decode_shapes_over_tiled_weights(gpu, oracle):
    """Full-size 13B linears at M = 16 through w4a8_gemm_tiled: output channels sampled against the oracle."""
    t = gpu
    M = 16
    for name, (N, K) in synth.LLAMA_SHAPES["13b"].items():
        xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=96)
        wp = oracle.pack_w4(wq)
        wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
        out = w4a8.w4a8_gemm_tiled(t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), wt, t.from_numpy(s_w).cuda())
        t.cuda.synchronize()
        cols = sorted({0, 1, 31, 32, 33, N // 2, N - 33, N - 32, N - 1} | set(range(4097, N, 977)))
        acc_o, y32, _ = oracle.gemm(xq, s_a, wp[cols], s_w[cols])
        assert_fp16_close(out.cpu().numpy()[:, cols], y32, acc_o, f"13B {name} M=16 over tiled weights")


@pytest.mark.parametrize("M", [8, 1024])
@pytest.mark.parametrize("N,K", synth.PAPER_TABLE5_SHAPES)
def test_paper_table5_shapes_over_tiled_weights(gpu, oracle, M, N, K):
    """The GEMM sizes the paper itself times (Table 5; N = 11088 is not a multiple of 32, so the last weight block is
    partly padding) at a token-generation and a context-decoding M, through the one-copy entry; rows sampled."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=98)
    wp = oracle.pack_w4(wq)
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    ws = t.empty((max(16, w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)),), dtype=t.uint8, device="cuda")
    out = w4a8.w4a8_gemm_tiled_splitk(t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), wt, t.from_numpy(s_w).cuda(), ws=ws)
    t.cuda.synchronize()
    rows = sorted({0, 1, M // 2, M - 1})
    acc_o, y32, _ = oracle.gemm(xq[rows], s_a[rows], wp, s_w)
    assert_fp16_close(out.cpu().numpy()[rows], y32, acc_o, f"Table 5 shape N={N} K={K} M={M}")
