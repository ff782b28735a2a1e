"""GPU parity of the persistent weight-streaming kernel over all its knobs (depth of the weight prefetch, evenly split
chunks or chunks of 16, wave count, grid, cache policy, activations staged in LDS or read directly): raw int32 sums bit-exact and fp16 within 2^-10 against the CPU oracle, over the row-major and
over the tiled weight array, for every prefetch depth, both wave counts, both chunkings and the non-temporal loads,
through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu

EPOCH, EPOCH_T = w4a8.TILING_DECODE_RESIDENT, w4a8.TILING_DECODE_RESIDENT_TILED


def variant(grid=0, waves=0, prefetch=0, whole16=False, nt=None, x_direct=False, window=False):
    flags = (1 if whole16 else 0) + (0 if nt is None else 2 if nt else 8) + (4 if x_direct else 0) + (16 if window else 0)
    return grid + 100000 * waves + 10000000 * prefetch + 100000000 * flags


def _run(torch, oracle, M, N, K, tiled, var, tag, what, acc_too=True):
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=tag)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    dxq, dsa, dsw = torch.from_numpy(xq).cuda(), torch.from_numpy(s_a).cuda(), torch.from_numpy(s_w).cuda()
    w = torch.from_numpy(wp).cuda()
    tiling = EPOCH
    if tiled:
        w, tiling = w4a8.w4a8_tile_weights(w), EPOCH_T
    try:
        out = w4a8.w4a8_gemm_tuned(dxq, dsa, w, dsw, tiling, var, N=N)
        acc = w4a8.w4a8_gemm_tuned(dxq, None, w, None, tiling, var, want_acc=True, N=N) if acc_too else None
    except w4a8.W4A8Error as e:
        if e.code == -7:
            pytest.skip("the library refuses this variant for this shape (registers or LDS)")
        raise
    torch.cuda.synchronize()
    if acc is not None:
        assert_equal_bits(acc.cpu().numpy(), acc_o, what + " acc")
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what + " out")


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("M", [1, 3, 8, 16])
@pytest.mark.parametrize("N,K", [(1, 32), (16, 32), (17, 64), (24, 96), (1000, 128), (1001, 160), (30, 4128), (4096, 1024),
                                 (8200, 2048), (5120, 5120), (300, 11008), (520, 13824), (40, 16384)])
def test_persistent_kernel_librarys_choice(gpu, oracle, M, N, K, tiled):
    _run(gpu, oracle, M, N, K, tiled, 0, 60, f"epoch tiled={tiled} M={M} N={N} K={K}")


@pytest.mark.parametrize("tiled", [False, True])
@pytest.mark.parametrize("M", [17, 24, 32])
@pytest.mark.parametrize("N,K", [(16, 32), (1001, 160), (520, 5120), (700, 8192)])
def test_persistent_kernel_two_column_tiles(gpu, oracle, M, N, K, tiled):
    _run(gpu, oracle, M, N, K, tiled, 0, 61, f"epoch tiled={tiled} M={M} N={N} K={K}")


@pytest.mark.parametrize("prefetch", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("waves", [8, 16])
@pytest.mark.parametrize("grid", [1, 7, 64, 256, 1000])
@pytest.mark.parametrize("M,N,K", [(1, 5120, 512), (16, 1000, 2080), (9, 1300, 5120), (4, 516, 8192)])
def test_persistent_kernel_prefetch_wave_and_grid_variants(gpu, oracle, M, N, K, waves, grid, prefetch):
    """Ranges of 4 .. N channels per workgroup: one-shot walks (no more chunks than the prefetch holds), walks of several
    epochs that alternate between the two sets of LDS slots, ranges that end in a partial chunk."""
    if -(-N // grid) > 512:
        pytest.skip("more than 512 channels per workgroup: outside this kernel's reach")
    for whole16 in (False, True):
        _run(gpu, oracle, M, N, K, True, variant(grid, waves, prefetch, whole16), 62,
             f"epoch {waves}w grid={grid} P={prefetch} whole16={whole16} M={M} N={N} K={K}", acc_too=not whole16)


@pytest.mark.parametrize("M,N,K", [(1, 700, 2080), (16, 5120, 5120), (5, 130, 13824)])
def test_persistent_kernel_cache_policies_and_activation_paths(gpu, oracle, M, N, K):
    for nt in (True, False):
        for x_direct in (False, True):
            _run(gpu, oracle, M, N, K, True, variant(nt=nt, x_direct=x_direct), 63,
                 f"nt={nt} x_direct={x_direct} M={M} N={N} K={K}", acc_too=False)
    _run(gpu, oracle, M, N, K, True, variant(256, 0, 2, False, True), 63, f"nt P=2 M={M} N={N} K={K}", acc_too=False)
    _run(gpu, oracle, M, N, K, False, variant(100, 0, 2, False, False, True), 63, f"row-major P=2 direct M={M} N={N} K={K}")


def test_persistent_kernel_extreme_codes_at_the_longest_k(gpu, oracle):
    """All activations -128 and all weights -8 at the longest K the kernel takes with registers to spare: the
    sixteen-fold sums stay inside int32 (Sec. 5.3) and come back exact."""
    t = gpu
    M, N, K = 2, 40, 16384
    xq = np.full((M, K), -128, np.int8)
    wq = np.full((N, K), -8, np.int8)
    wt = w4a8.w4a8_tile_weights(t.from_numpy(oracle.pack_w4(wq)).cuda())
    acc = w4a8.w4a8_gemm_tuned(t.from_numpy(xq).cuda(), None, wt, None, EPOCH_T, 0, want_acc=True, N=N)
    t.cuda.synchronize()
    assert np.all(acc.cpu().numpy() == 128 * 8 * K)


# ---- every wave stages its own k steps through a window of LDS (tiled weights; the only form beyond 32 tokens and the
# library's choice from five tokens on)

WINDOW_SHAPES = [(16, 32), (17, 64), (1001, 160), (300, 1024), (520, 4096), (520, 5120), (130, 7168), (700, 8192)]


@pytest.mark.parametrize("M", [1, 5, 16, 17, 31, 32, 33, 47, 48, 49, 64])
@pytest.mark.parametrize("N,K", WINDOW_SHAPES + [(520, 13824), (40, 16384)])
def test_window_form_librarys_choice(gpu, oracle, M, N, K):
    """Two to four column tiles, one and several windows per wave, ranges of one chunk and of many, ragged N and a K
    that ends inside a k step; shapes whose K does not fit a wave's registers are refused (and skipped here: they are
    served in K slices, below)."""
    _run(gpu, oracle, M, N, K, True, variant(window=True), 64, f"window M={M} N={N} K={K}")


@pytest.mark.parametrize("prefetch", [1, 2])
@pytest.mark.parametrize("grid", [1, 7, 64, 256, 1000])
@pytest.mark.parametrize("M,N,K", [(20, 5120, 512), (33, 1000, 2080), (64, 1300, 5120), (40, 516, 4128)])
def test_window_form_grid_and_prefetch_variants(gpu, oracle, M, N, K, grid, prefetch):
    if -(-N // grid) > 512:
        pytest.skip("more than 512 channels per workgroup: outside this kernel's reach")
    _run(gpu, oracle, M, N, K, True, variant(grid, 0, prefetch, window=True), 65,
         f"window grid={grid} P={prefetch} M={M} N={N} K={K}")


@pytest.mark.parametrize("M", [4, 5, 9, 16, 17, 32, 48, 64])
@pytest.mark.parametrize("N,K", [(520, 5120), (1001, 160), (200, 13824)])
def test_one_weight_array_serves_medium_m_too(gpu, oracle, M, N, K):
    """w4a8_gemm_tiled routes 5 to 64 tokens to the window form when all of K fits a wave's registers (and to the
    large-M kernel when it does not)."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=66)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    out = w4a8.w4a8_gemm_tiled(t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), wt, t.from_numpy(s_w).cuda())
    t.cuda.synchronize()
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, f"gemm_tiled M={M} N={N} K={K}")


@pytest.mark.parametrize("M,N,K,splits", [(64, 520, 13824, 3), (64, 520, 13824, 0), (32, 300, 13824, 2), (48, 1001, 8192, 2),
                                          (33, 130, 28672, 0), (64, 200, 5120, 4), (17, 40, 4096, 8), (33, 77, 4128, 3),
                                          (50, 1001, 2080, 5), (20, 24, 65536, 0)])
def test_window_form_in_k_slices(gpu, oracle, M, N, K, splits):
    """A K too long for a wave's registers (or a forced slice count) is cut over workgroups: one slab of raw sums per
    slice, added up and dequantised by the slab epilogue.  Integer sums: the bits of the unsliced result."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=67)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    if splits == 0:
        need = w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)
        assert need > 0 and need % (M * N * 4) == 0
        ws = t.empty((need,), dtype=t.uint8, device="cuda")
        out = w4a8.w4a8_gemm_tiled_splitk(dxq, dsa, wt, dsw, ws=ws)
    else:
        out = w4a8.w4a8_gemm_tiled_splitk(dxq, dsa, wt, dsw, splits=splits)
    ref = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, dsw)
    t.cuda.synchronize()
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, f"sliced M={M} N={N} K={K} splits={splits}")
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), "sliced vs w4a8_gemm_tiled")


def _random_shapes(count, seed):
    g = synth.rng(4242, seed)
    shapes = []
    for _ in range(count):
        M = int(g.integers(1, 65))
        N = int(g.integers(1, 2500))
        K = 32 * int(g.integers(1, 257))          # 32 .. 8192, any multiple of 32 (ragged against the 128-wide k steps)
        shapes.append((M, N, K))
    return shapes


@pytest.mark.parametrize("M,N,K", _random_shapes(48, 1))
def test_one_copy_entries_on_seeded_random_shapes(gpu, oracle, M, N, K):
    """Seeded random (M <= 64, N, K) through both one-copy entries: whichever kernel the library picks (whole-row
    staging, per-wave windows, K slices, or the large-M kernel where K does not fit), the raw sums behind the fp16
    output are the oracle's."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=68)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    a = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, dsw)
    b = w4a8.w4a8_gemm_tiled_splitk(dxq, dsa, wt, dsw)
    t.cuda.synchronize()
    assert_fp16_close(a.cpu().numpy(), y32, acc_o, f"gemm_tiled M={M} N={N} K={K}")
    assert_equal_bits(b.cpu().numpy().view(np.uint16), a.cpu().numpy().view(np.uint16), "splitk entry vs gemm_tiled")
