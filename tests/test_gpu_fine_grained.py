"""GPU parity of the fine-grained (group-wise scales) ablation kernel against the CPU oracle, through the C ABI.

Two bars: (1) against the definition in fp64, |O - y64| <= 2^-10 |y64| + (G + 2) 2^-24 mag, where G is the number of
groups and mag the sum of the absolute group terms (one fp32 rounding per fused multiply-add of the chain, one for
the product with s_a, then the fp16 rounding); (2) bit for bit against the oracle's fp32 evaluation of the same chain
in the same order, which the kernel follows exactly."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits

pytestmark = pytest.mark.gpu

TILES = [1, 2, 3, 4, 5, 6]   # 128x256, 256x128, 128x128, 64x128, 64x64, 32x128


def _pad_scales(s_g):
    """[G][N] -> [G][ldg] with ldg the next multiple of 4 (the padding is never used)."""
    G, N = s_g.shape
    ldg = (N + 3) // 4 * 4
    out = np.full((G, ldg), np.float32(777.0))
    out[:, :N] = s_g
    return out


def _check(torch, oracle, xq, wq, s_a, s_g, tile, what):
    N, K = wq.shape
    wp = oracle.pack_w4(wq)
    y64, y32, out_o, mag = oracle.gemm_fine_grained(xq, s_a, wp, s_g)
    wt = w4a8.w4a8_tile_weights(torch.from_numpy(wp).cuda())
    out = w4a8.w4a8_gemm_fine_grained(torch.from_numpy(xq).cuda(), torch.from_numpy(s_a).cuda(), wt,
                                      torch.from_numpy(_pad_scales(s_g)).cuda(), N=N, variant=tile)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    err = np.abs(o.astype(np.float64) - y64)
    bound = 2.0 ** -10 * np.abs(y64) + (K // 128 + 2) * 2.0 ** -24 * mag + 2.0 ** -24
    assert np.all(err <= bound), f"{what}: {np.sum(err > bound)} outputs outside the fp64 bound"
    assert_equal_bits(o.view(np.uint16), out_o.view(np.uint16), what + " vs the fp32 chain")


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("M", [1, 17, 64, 65, 129, 257, 300])
def test_fine_grained_all_m(gpu, oracle, M, tile):
    N, K = 520, 1152
    xq, wq, s_a, _ = synth.uniform_codes(M, N, K, config_id=70)
    _check(gpu, oracle, xq, wq, s_a, synth.group_scales(N, K, 128, config_id=70), tile, f"fine tile={tile} M={M}")


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("M,N,K", [(130, 1, 128), (128, 255, 256), (100, 257, 128), (200, 1001, 384), (70, 1000, 4096),
                                   (1024, 512, 1024), (384, 300, 5120), (260, 330, 256), (513, 161, 640)])
def test_fine_grained_ragged_shapes(gpu, oracle, M, N, K, tile):
    xq, wq, s_a, _ = synth.uniform_codes(M, N, K, config_id=71)
    _check(gpu, oracle, xq, wq, s_a, synth.group_scales(N, K, 128, config_id=71), tile,
           f"fine tile={tile} M={M} N={N} K={K}")


def test_fine_grained_extreme_codes_at_max_k(gpu, oracle):
    """a = -128, w = -8 in every position of K = 65536 (512 groups): every group's sum is 2^17, exactly convertible."""
    M, K, N = 70, 65536, 40
    xq = np.full((M, K), -128, np.int8)
    xq[1, :] = 127
    wq = np.full((N, K), -8, np.int8)
    wq[1, :] = 7
    wq[2, ::2] = 0
    s_a = np.full(M, 2.0 ** -12, np.float32)
    _check(gpu, oracle, xq, wq, s_a, synth.group_scales(N, K, 128, config_id=72) * np.float32(2.0 ** -6), 0, "fine extremes")


def test_fine_grained_with_equal_group_scales_tracks_the_per_channel_kernel(gpu, oracle):
    """With the same scale in every group of a channel the result is the per-channel one up to the fp32 roundings of
    the chain; with power-of-two scales those roundings vanish for sums below 2^24 and the bits are equal."""
    t = gpu
    M, N, K = 200, 520, 1152
    xq, wq, s_a, _ = synth.uniform_codes(M, N, K, config_id=73)
    s_w = (2.0 ** -(8 + np.arange(N) % 5)).astype(np.float32)
    wp = oracle.pack_w4(wq)
    dxq, dsa = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda()
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    per_channel = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, t.from_numpy(s_w).cuda())
    fine = w4a8.w4a8_gemm_fine_grained(dxq, dsa, wt, t.from_numpy(np.tile(s_w, (K // 128, 1))).cuda())
    t.cuda.synchronize()
    acc = oracle.gemm_acc_i32(xq, wp)
    assert np.abs(acc).max() < 2 ** 24
    # per-channel rounds float(acc) * (s_a * s_w), fine-grained (float(acc) * s_w) * s_a: s_w is a power of two, so
    # both are float(acc) * s_a * s_w rounded once
    assert_equal_bits(fine.cpu().numpy().view(np.uint16), per_channel.cpu().numpy().view(np.uint16), "fine vs per-channel")


def test_fine_grained_llama13b_sampled(gpu, oracle):
    """Full-size LLaMA-13B down projection (K = 13824: 108 groups) at M = 1024 in the default tile, and the QKV shape
    at M = 16; sampled rows against the oracle."""
    t = gpu
    for M, (N, K), rows in ((1024, synth.LLAMA_SHAPES["13b"]["down"], [0, 1, 127, 128, 511, 777, 1023]),
                            (16, synth.LLAMA_SHAPES["13b"]["qkv"], list(range(16)))):
        xq, wq, s_a, _ = synth.uniform_codes(M, N, K, config_id=74)
        s_g = synth.group_scales(N, K, 128, config_id=74)
        wp = oracle.pack_w4(wq)
        wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
        out = w4a8.w4a8_gemm_fine_grained(t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), wt, t.from_numpy(s_g).cuda())
        t.cuda.synchronize()
        _, _, out_o, _ = oracle.gemm_fine_grained(xq[rows], s_a[rows], wp, s_g)
        assert_equal_bits(out.cpu().numpy()[rows].view(np.uint16), out_o.view(np.uint16), f"13B fine-grained M={M}")
