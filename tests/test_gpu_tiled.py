"""GPU parity of the tiled weight layout and of the large-M kernel that reads it: the reordering is checked byte for
byte against the layout's definition written out here in numpy, the GEMM against the CPU oracle (raw int32 sums
bit-exact, fp16 within 2^-10 relative), through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu

TILED = w4a8.TILING_PREFILL_TILED
BASE_TILES = [1, 2, 3, 4, 5, 6, 7, 8]   # 256x256 (2x4 waves), 256x256 (4x2), 128x256, 128x160, 128x128, 64x128, 64x64, 32x128
TILES = BASE_TILES + [9, 10, 11, 12]    # signed int4 only: 128x160 and 128x128 with two wave sets splitting each stage's k; 256x192;
                                        # 128x256 on 8 waves


def tiled_layout(wq):
    """The tiled array from the codes wq [N][K] in [-8, 7], straight from the layout's definition."""
    N, K = wq.shape
    NB, KB = (N + 31) // 32, (K + 127) // 128
    pad = np.zeros((NB * 32, KB * 128), np.int8)
    pad[:N, :K] = wq
    nib = (pad.astype(np.uint8) & 15).reshape(NB, 32, KB, 4, 4, 8)      # nb, r, kb, c, dword, code k0..k7
    order = [0, 4, 1, 5, 2, 6, 3, 7]                                   # nibble position i holds code order[i]
    dwords = np.zeros(nib.shape[:-1], np.uint32)
    for i, k in enumerate(order):
        dwords |= nib[..., k].astype(np.uint32) << np.uint32(4 * i)
    blocks = dwords.transpose(0, 2, 3, 1, 4)                            # nb, kb, c, r, dword
    return np.ascontiguousarray(blocks).astype("<u4").view(np.uint8).reshape(-1)


@pytest.mark.parametrize("N,K", [(1, 32), (32, 128), (33, 160), (100, 96), (257, 4128), (1000, 1056), (64, 65536)])
def test_tile_weights_matches_the_layout_definition(gpu, oracle, N, K):
    _, wq, _, _ = synth.uniform_codes(1, N, K, config_id=50)
    wp = oracle.pack_w4(wq)
    wt = w4a8.w4a8_tile_weights(gpu.from_numpy(wp).cuda())
    gpu.cuda.synchronize()
    expect = tiled_layout(wq)
    assert wt.numel() == expect.size == w4a8.w4a8_tiled_weight_bytes(N, K)
    assert_equal_bits(wt.cpu().numpy(), expect, f"tiled layout N={N} K={K}")


def _run_tiled(torch, oracle, xq, wq, s_a, s_w, tile, what):
    N = wq.shape[0]
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    dxq, dsa, dsw = torch.from_numpy(xq).cuda(), torch.from_numpy(s_a).cuda(), torch.from_numpy(s_w).cuda()
    wt = w4a8.w4a8_tile_weights(torch.from_numpy(wp).cuda())
    acc = w4a8.w4a8_gemm_tuned(dxq, None, wt, None, TILED, tile, want_acc=True, N=N)
    out = w4a8.w4a8_gemm_tuned(dxq, dsa, wt, dsw, TILED, tile, N=N)
    torch.cuda.synchronize()
    assert_equal_bits(acc.cpu().numpy(), acc_o, what + " acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what + " out")


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("M", [1, 17, 64, 65, 127, 128, 129, 255, 256, 257, 300])
def test_tiled_all_m(gpu, oracle, M, tile):
    xq, wq, s_a, s_w = synth.uniform_codes(M, 520, 1056, config_id=51)
    _run_tiled(gpu, oracle, xq, wq, s_a, s_w, tile, f"tiled tile={tile} M={M}")


@pytest.mark.parametrize("M,N,K", [(130, 1, 32), (128, 255, 64), (256, 256, 96), (100, 257, 128), (200, 1001, 160),
                                   (70, 1000, 4128), (1024, 512, 1024), (384, 300, 5120), (260, 330, 256), (513, 161, 384)])
@pytest.mark.parametrize("tile", TILES)
def test_tiled_ragged_shapes(gpu, oracle, M, N, K, tile):
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=52)
    _run_tiled(gpu, oracle, xq, wq, s_a, s_w, tile, f"tiled tile={tile} M={M} N={N} K={K}")


def test_tiled_extreme_codes_at_max_k(gpu, oracle):
    """a = -128, w = -8 along all of K = 65536: the sixteen-fold sum is 2^30, inside int32 (Sec. 5.3)."""
    M, K, N = 130, 65536, 48
    xq = np.full((M, K), -128, np.int8)
    xq[1, :] = 127
    wq = np.full((N, K), -8, np.int8)
    wq[1, :] = 7
    wq[2, ::2] = 0
    s_a = np.full(M, 2.0 ** -12, np.float32)
    s_w = np.full(N, 2.0 ** -12, np.float32)
    _run_tiled(gpu, oracle, xq, wq, s_a, s_w, 0, "tiled extremes")


def test_gemm_tiled_entry_equals_row_major_entry(gpu, oracle):
    """w4a8_gemm_tiled over the reordered weights returns the bits w4a8_gemm returns over the row-major ones (same
    arithmetic, same rounding), for a decode-sized and a prefill-sized M; repeated calls agree with themselves."""
    for M in (4, 200):
        xq, wq, s_a, s_w = synth.uniform_codes(M, 700, 2080, config_id=53)
        wp = oracle.pack_w4(wq)
        t = gpu
        dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
        dwp = t.from_numpy(wp).cuda()
        wt = w4a8.w4a8_tile_weights(dwp)
        a = w4a8.w4a8_gemm(dxq, dsa, dwp, dsw)
        b = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, dsw)
        c = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, dsw)
        t.cuda.synchronize()
        assert_equal_bits(b.cpu().numpy().view(np.uint16), a.cpu().numpy().view(np.uint16), f"tiled vs row-major M={M}")
        assert_equal_bits(c.cpu().numpy().view(np.uint16), b.cpu().numpy().view(np.uint16), f"repeat M={M}")
        acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
        assert_fp16_close(b.cpu().numpy(), y32, acc_o, f"tiled entry M={M}")


@pytest.mark.parametrize("tile", BASE_TILES)
@pytest.mark.parametrize("M,N,K", [(1, 520, 1056), (65, 520, 1056), (300, 520, 1056), (200, 1001, 160), (384, 300, 5120)])
def test_unsigned_storage_variant(gpu, oracle, M, N, K, tile):
    """The storage ablation (unsigned nibbles u = w + 8, 8 subtracted in registers) against the oracle's definition of
    it, and bit-identical to the signed format on the same codes."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=56)
    up = oracle.pack_u4(wq.astype(np.int16) + 8)
    acc_o, y32, _ = oracle.gemm_u4(xq, s_a, up, s_w)
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    ut = w4a8.w4a8_tile_weights(t.from_numpy(up).cuda())
    acc = w4a8.w4a8_gemm_tiled_unsigned(dxq, None, ut, None, N=N, variant=tile, want_acc=True)
    out = w4a8.w4a8_gemm_tiled_unsigned(dxq, dsa, ut, dsw, variant=tile)
    wt = w4a8.w4a8_tile_weights(t.from_numpy(oracle.pack_w4(wq)).cuda())
    ref = w4a8.w4a8_gemm_tuned(dxq, dsa, wt, dsw, TILED, tile, N=N)
    t.cuda.synchronize()
    assert_equal_bits(acc.cpu().numpy(), acc_o, f"unsigned tile={tile} acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, f"unsigned tile={tile} out")
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), "unsigned vs signed storage")


@pytest.mark.parametrize("M,N,K", [(256, 27648, 160), (512, 15360, 160), (2048, 5120, 160), (1024, 27648, 128)])
def test_library_tile_choice_exists_for_every_weight_format(gpu, oracle, M, N, K):
    """Shapes for which the signed int4 format is given one of its own tiles (128 x 256 on 8 waves, 256 x 192, the
    two-phase launch): the unsigned storage and the int8 weights, which lack those tiles, must be given one they have.
    Same codes, so all three outputs have the same bits; sampled rows against the oracle."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=57)
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    wp = oracle.pack_w4(wq)
    signed = w4a8.w4a8_gemm_tiled(dxq, dsa, w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda()), dsw)
    ut = w4a8.w4a8_tile_weights(t.from_numpy(oracle.pack_u4(wq.astype(np.int16) + 8)).cuda())
    unsigned = w4a8.w4a8_gemm_tiled_unsigned(dxq, dsa, ut, dsw)
    w8 = w4a8.w8a8_gemm_tiled(dxq, dsa, w4a8.w8a8_tile_weights(t.from_numpy(wq).cuda()), dsw)
    t.cuda.synchronize()
    assert_equal_bits(unsigned.cpu().numpy().view(np.uint16), signed.cpu().numpy().view(np.uint16), "unsigned vs signed")
    assert_equal_bits(w8.cpu().numpy().view(np.uint16), signed.cpu().numpy().view(np.uint16), "int8 weights vs signed int4")
    rows = [0, M // 3, M - 1]
    acc_o, y32, _ = oracle.gemm(xq[rows], s_a[rows], wp, s_w)
    assert_fp16_close(signed.cpu().numpy()[rows], y32, acc_o, f"library tile M={M} N={N} K={K}")


def test_tiled_llama13b_prefill_sampled(gpu, oracle):
    """Full-size LLaMA-13B gate/up shape at M = 1024 in the default tile: rows of the output sampled and checked
    against the oracle one by one (raw sums bit-exact)."""
    M, N, K = 1024, 27648, 5120
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=54)
    wp = oracle.pack_w4(wq)
    t = gpu
    dxq = t.from_numpy(xq).cuda()
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    acc = w4a8.w4a8_gemm_tuned(dxq, None, wt, None, TILED, 0, want_acc=True, N=N)
    out = w4a8.w4a8_gemm_tiled(dxq, t.from_numpy(s_a).cuda(), wt, t.from_numpy(s_w).cuda())
    t.cuda.synchronize()
    rows = [0, 1, 127, 128, 255, 256, 511, 777, 1023]
    acc_o, y32, _ = oracle.gemm(xq[rows], s_a[rows], wp, s_w)
    assert_equal_bits(acc.cpu().numpy()[rows], acc_o, "13B gate_up sampled rows acc")
    assert_fp16_close(out.cpu().numpy()[rows], y32, acc_o, "13B gate_up sampled rows out")
