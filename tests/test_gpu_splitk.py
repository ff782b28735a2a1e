"""GPU parity of the tiled GEMM with K split over workgroups (raw int32 slabs + a second kernel for Eq. (6),(7)):
against the CPU oracle, and bit for bit against the unsplit tiled kernel, through the C ABI."""
import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu


def _inputs(torch, oracle, M, N, K, config_id):
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=config_id)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    d = dict(xq=torch.from_numpy(xq).cuda(), s_a=torch.from_numpy(s_a).cuda(), s_w=torch.from_numpy(s_w).cuda(),
             wt=w4a8.w4a8_tile_weights(torch.from_numpy(wp).cuda()))
    return d, acc_o, y32


@pytest.mark.parametrize("splits", [1, 2, 3, 5, 8, 64])
@pytest.mark.parametrize("M,N,K,tile", [(1, 520, 1056, 8), (33, 520, 1056, 6), (100, 257, 2080, 7), (129, 1001, 1056, 5),
                                        (64, 300, 5120, 0), (200, 161, 4128, 4), (70, 130, 160, 6), (96, 512, 13824, 0)])
def test_forced_split_matches_oracle_and_unsplit_kernel(gpu, oracle, M, N, K, tile, splits):
    d, acc_o, y32 = _inputs(gpu, oracle, M, N, K, 80)
    out = w4a8.w4a8_gemm_tiled_splitk(d["xq"], d["s_a"], d["wt"], d["s_w"], variant=tile, splits=splits)
    ref = w4a8.w4a8_gemm_tiled(d["xq"], d["s_a"], d["wt"], d["s_w"])
    gpu.cuda.synchronize()
    what = f"split-K M={M} N={N} K={K} tile={tile} splits={splits}"
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, what)
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), what + " vs unsplit")


@pytest.mark.parametrize("M,N,K", [(32, 5120, 5120), (128, 5120, 13824), (64, 15360, 5120), (256, 5120, 5120), (1024, 5120, 5120)])
def test_library_choice_on_llama13b_shapes(gpu, oracle, M, N, K):
    """splits = 0 with a workspace of exactly the advertised size; rows sampled against the oracle, everything
    against the unsplit kernel; two calls in a row reuse the workspace."""
    t = gpu
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=81)
    wp = oracle.pack_w4(wq)
    need = w4a8.w4a8_gemm_tiled_workspace_bytes(M, N, K)
    assert need % (M * N * 4) == 0 and need // (M * N * 4) in (0, 2, 3, 4, 5, 6, 7, 8)
    if (M, N) == (128, 5120):
        assert need > 0          # 80 tiles on 256 compute units: the library splits
    if (M, N) == (32, 5120):
        assert need == 0         # all of K fits a wave's registers: the weight-streaming kernel, no slabs
    if M == 1024:
        assert need == 0         # large M is never split
    ws = t.empty((max(need, 16),), dtype=t.uint8, device="cuda")
    dxq, dsa, dsw = t.from_numpy(xq).cuda(), t.from_numpy(s_a).cuda(), t.from_numpy(s_w).cuda()
    wt = w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda())
    ref = w4a8.w4a8_gemm_tiled(dxq, dsa, wt, dsw)
    a = w4a8.w4a8_gemm_tiled_splitk(dxq, dsa, wt, dsw, ws=ws)
    b = w4a8.w4a8_gemm_tiled_splitk(dxq, dsa, wt, dsw, ws=ws)
    t.cuda.synchronize()
    assert_equal_bits(a.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), f"library split M={M} N={N} K={K}")
    assert_equal_bits(b.cpu().numpy().view(np.uint16), a.cpu().numpy().view(np.uint16), "second call")
    rows = sorted({0, 1, M // 2, M - 1})
    acc_o, y32, _ = oracle.gemm(xq[rows], s_a[rows], wp, s_w)
    assert_fp16_close(a.cpu().numpy()[rows], y32, acc_o, f"library split rows M={M} N={N} K={K}")


def test_workspace_too_small_is_refused(gpu, oracle):
    d, _, _ = _inputs(gpu, oracle, 64, 256, 1024, 82)
    ws = gpu.empty((2 * 64 * 256 * 4 - 16,), dtype=gpu.uint8, device="cuda")
    with pytest.raises(w4a8.W4A8Error) as e:
        w4a8.w4a8_gemm_tiled_splitk(d["xq"], d["s_a"], d["wt"], d["s_w"], splits=2, ws=ws)
    assert e.value.code == -4


def test_bound_call_launches_what_the_plain_binding_launches(gpu, oracle):
    """The pre-marshalled launch used by tight loops goes through the same C entry points: same bits out, and an error
    code still raises."""
    t = gpu
    M, N, K = 48, 300, 2080
    d, _, _ = _inputs(t, oracle, M, N, K, 83)
    ref = w4a8.w4a8_gemm_tiled(d["xq"], d["s_a"], d["wt"], d["s_w"])
    out = t.zeros((M, N), dtype=t.float16, device="cuda")
    ws = t.empty((3 * M * N * 4,), dtype=t.uint8, device="cuda")
    call = w4a8.bound_call("w4a8_gemm_tiled_splitk", d["xq"], d["s_a"], d["wt"], d["s_w"], out, M, N, K, 0, 3, ws, ws.numel())
    call()
    call()
    t.cuda.synchronize()
    assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), "bound call")
    bad = w4a8.bound_call("w4a8_gemm_tiled_splitk", d["xq"], d["s_a"], d["wt"], d["s_w"], out, M, N, K, 0, 3, ws, 16)
    with pytest.raises(w4a8.W4A8Error) as e:
        bad()
    assert e.value.code == -4
