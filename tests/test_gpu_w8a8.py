"""GPU parity of the W8A8 comparison variant (int8 weight codes, same kernels without the int4 conversion) against
the CPU oracle's plain int8 x int8 definition, through the C ABI: tiled layout byte for byte, raw int32 sums
bit-exact, fp16 outputs within 2^-10 relative."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu

TILES = [1, 2, 3, 4, 5, 6, 7, 8]


def _codes8(M, N, K, tag):
    g = synth.rng(980, tag, M, N, K)
    xq = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    w8 = g.integers(-128, 128, size=(N, K), dtype=np.int8)
    s_a = g.uniform(1e-3, 1e-2, M).astype(np.float32)
    s_w = g.uniform(1e-4, 1e-3, N).astype(np.float32)
    return xq, w8, s_a, s_w


def tiled_layout8(w8):
    """The tiled int8 array straight from the layout's definition."""
    N, K = w8.shape
    NB, KB = (N + 31) // 32, (K + 127) // 128
    pad = np.zeros((NB * 32, KB * 128), np.int8)
    pad[:N, :K] = w8
    blocks = pad.reshape(NB, 32, KB, 8, 16).transpose(0, 2, 3, 1, 4)      # nb, kb, c, r, 16 codes
    return np.ascontiguousarray(blocks).view(np.uint8).reshape(-1)


@pytest.mark.parametrize("N,K", [(1, 32), (32, 128), (33, 160), (100, 96), (257, 4128), (64, 65536)])
def test_tile_weights8_matches_the_layout_definition(gpu, N, K):
    _, w8, _, _ = _codes8(1, N, K, 1)
    wt = w4a8.w8a8_tile_weights(gpu.from_numpy(w8).cuda())
    gpu.cuda.synchronize()
    expect = tiled_layout8(w8)
    assert wt.numel() == expect.size == w4a8.w8a8_tiled_weight_bytes(N, K)
    assert_equal_bits(wt.cpu().numpy(), expect, f"tiled int8 layout N={N} K={K}")


def _run(torch, oracle, xq, w8, s_a, s_w, tile, what):
    N = w8.shape[0]
    acc_o, y32, _ = oracle.gemm_w8(xq, s_a, w8, s_w)
    dxq, dsa, dsw = torch.from_numpy(xq).cuda(), torch.from_numpy(s_a).cuda(), torch.from_numpy(s_w).cuda()
    wt = w4a8.w8a8_tile_weights(torch.from_numpy(w8).cuda())
    acc = w4a8.w8a8_gemm_tiled(dxq, None, wt, None, N=N, variant=tile, want_acc=True)
    out = w4a8.w8a8_gemm_tiled(dxq, dsa, wt, dsw, variant=tile)
    torch.cuda.synchronize()
    assert_equal_bits(acc.cpu().numpy(), acc_o, what + " acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what + " out")


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("M", [1, 17, 64, 65, 128, 129, 256, 300])
def test_w8a8_all_m(gpu, oracle, M, tile):
    xq, w8, s_a, s_w = _codes8(M, 520, 1056, 2)
    _run(gpu, oracle, xq, w8, s_a, s_w, tile, f"w8a8 tile={tile} M={M}")


@pytest.mark.parametrize("M,N,K", [(130, 1, 32), (128, 255, 64), (256, 256, 96), (100, 257, 128), (200, 1001, 160),
                                   (70, 1000, 4128), (1024, 512, 1024), (384, 300, 5120), (513, 161, 384)])
@pytest.mark.parametrize("tile", TILES)
def test_w8a8_ragged_shapes(gpu, oracle, M, N, K, tile):
    xq, w8, s_a, s_w = _codes8(M, N, K, 3)
    _run(gpu, oracle, xq, w8, s_a, s_w, tile, f"w8a8 tile={tile} M={M} N={N} K={K}")


def test_w8a8_extremes_at_max_k(gpu, oracle):
    """a = -128, w = -128 along all of K = 65536: the sum is 2^30, inside int32."""
    M, K, N = 130, 65536, 48
    xq = np.full((M, K), -128, np.int8)
    xq[1, :] = 127
    w8 = np.full((N, K), -128, np.int8)
    w8[1, :] = 127
    w8[2, ::2] = 0
    s_a = np.full(M, 2.0 ** -14, np.float32)
    s_w = np.full(N, 2.0 ** -14, np.float32)
    _run(gpu, oracle, xq, w8, s_a, s_w, 0, "w8a8 extremes")


def test_w8a8_on_int4_codes_equals_w4a8(gpu, oracle):
    """Weight codes that fit four bits give, through the int8 path, the bits the W4A8 path gives for the same codes."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(200, 700, 2080, config_id=55)
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    wt4 = w4a8.w4a8_tile_weights(t.from_numpy(oracle.pack_w4(wq)).cuda())
    wt8 = w4a8.w8a8_tile_weights(t.from_numpy(wq).cuda())
    a = w4a8.w4a8_gemm_tiled(dxq, dsa, wt4, dsw)
    b = w4a8.w8a8_gemm_tiled(dxq, dsa, wt8, dsw)
    t.cuda.synchronize()
    assert_equal_bits(b.cpu().numpy().view(np.uint16), a.cpu().numpy().view(np.uint16), "int8 path on int4 codes")


@pytest.mark.parametrize("M", [16, 1024])
def test_w8a8_llama13b_sampled(gpu, oracle, M):
    """Full-size LLaMA-13B QKV shape, weights from the 8-bit per-channel quantiser (the per-token quantiser applied
    to weight rows), default tile: sampled rows and channels against the oracle."""
    t = gpu
    N, K = synth.LLAMA_SHAPES["13b"]["qkv"]
    x = synth.activations_fp16(M, K, config_id=6, tag=1)
    w = synth.weights_fp16(N, K, config_id=6)
    dxq, dsa = w4a8.w4a8_quantize_act(t.from_numpy(x).cuda())
    dw8, dsw = w4a8.w4a8_quantize_act(t.from_numpy(w).cuda())           # Eq. (8),(9) with 8 bits
    wt = w4a8.w8a8_tile_weights(dw8)
    acc = w4a8.w8a8_gemm_tiled(dxq, None, wt, None, N=N, want_acc=True)
    out = w4a8.w8a8_gemm_tiled(dxq, dsa, wt, dsw)
    t.cuda.synchronize()
    g = synth.rng(981, M)
    rows = np.unique(np.concatenate([g.choice(M, size=min(M, 16), replace=False), [0, M - 1]]))
    cols = np.unique(np.concatenate([np.arange(32), np.arange(N - 32, N), g.choice(N, size=300, replace=False)]))
    ri, ci = t.from_numpy(rows).cuda(), t.from_numpy(cols).cuda()
    w8_o, s_w_o = oracle.quantize_weights_rtn8(np.ascontiguousarray(w[cols]))
    xq_o, s_a_o = oracle.quantize_act(x[rows])
    assert_equal_bits(dw8[ci].cpu().numpy(), w8_o, "int8 weight codes")
    assert_equal_bits(dsw[ci].cpu().numpy().view(np.uint32), s_w_o.view(np.uint32), "s_w")
    acc_o, y32, _ = oracle.gemm_w8(xq_o, s_a_o, w8_o, s_w_o)
    assert_equal_bits(acc[ri][:, ci].cpu().numpy(), acc_o, "acc sample")
    assert_fp16_close(out[ri][:, ci].cpu().numpy(), y32, acc_o, "out sample")
