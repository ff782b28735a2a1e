"""GPU test of the entry point that allocates nothing (w4a8_gemm_tiled_splitk_static): through the C ABI, against the
entry point it is a variant of (w4a8_gemm_tiled_splitk with a caller-provided workspace), bit for bit, and against the
CPU oracle; two calls in a row, the second with a smaller input, so that what the first call left in the library's
scratch array must not leak into the second result."""
import ctypes

import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

from parity import assert_equal_bits, assert_fp16_close

pytestmark = pytest.mark.gpu


def _case(t, oracle, M, N, K, config_id):
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=config_id)
    wp = oracle.pack_w4(wq)
    acc_o, y32, _ = oracle.gemm(xq, s_a, wp, s_w)
    dev = dict(xq=t.from_numpy(xq).cuda(), s_a=t.from_numpy(s_a).cuda(), s_w=t.from_numpy(s_w).cuda(),
               wt=w4a8.w4a8_tile_weights(t.from_numpy(wp).cuda()))
    return dev, acc_o, y32


def _static_call(t, d, out, M, N, K, variant, splits):
    """Straight through the C ABI: raw pointers, no marshalling helper in between."""
    vp = ctypes.c_void_p
    code = w4a8.lib().w4a8_gemm_tiled_splitk_static(vp(d["xq"].data_ptr()), vp(d["s_a"].data_ptr()), vp(d["wt"].data_ptr()),
                                                    vp(d["s_w"].data_ptr()), vp(out.data_ptr()), M, N, K, variant, splits,
                                                    vp(t.cuda.current_stream().cuda_stream))
    return code


@pytest.mark.parametrize("first,second", [((96, 520, 4128, 6, 5), (33, 260, 2080, 6, 3)),
                                          ((128, 5120, 5120, 0, 0), (32, 5120, 5120, 0, 0)),
                                          ((200, 161, 4128, 4, 8), (70, 130, 160, 6, 2))])
def test_static_scratch_entry_matches_workspace_entry(gpu, oracle, first, second):
    t = gpu
    for i, (M, N, K, variant, splits) in enumerate((first, second)):
        d, acc_o, y32 = _case(t, oracle, M, N, K, 90 + i)
        ref = w4a8.w4a8_gemm_tiled_splitk(d["xq"], d["s_a"], d["wt"], d["s_w"], variant=variant, splits=splits)
        out = t.full((M, N), float("nan"), dtype=t.float16, device="cuda")
        assert _static_call(t, d, out, M, N, K, variant, splits) == 0
        t.cuda.synchronize()
        what = f"static scratch call {i}: M={M} N={N} K={K} tile={variant} splits={splits}"
        assert_equal_bits(out.cpu().numpy().view(np.uint16), ref.cpu().numpy().view(np.uint16), what + " vs workspace entry")
        assert_fp16_close(out.cpu().numpy(), y32, acc_o, what)


def test_static_scratch_entry_token_generation_and_limit(gpu, oracle):
    t = gpu
    # M <= 16 streams the weights and uses no slabs at all
    d, acc_o, y32 = _case(t, oracle, 4, 1024, 2048, 93)
    out = t.full((4, 1024), float("nan"), dtype=t.float16, device="cuda")
    assert _static_call(t, d, out, 4, 1024, 2048, 0, 0) == 0
    t.cuda.synchronize()
    assert_fp16_close(out.cpu().numpy(), y32, acc_o, "static scratch entry, M = 4")
    # slabs beyond the array: refused, nothing launched, the output untouched
    M, N, K = 512, 4096, 1024
    assert 8 * M * N * 4 > w4a8.STATIC_SCRATCH_BYTES
    dummy = dict(xq=t.zeros((M, K), dtype=t.int8, device="cuda"), s_a=t.ones((M,), dtype=t.float32, device="cuda"),
                 s_w=t.ones((N,), dtype=t.float32, device="cuda"),
                 wt=t.zeros((w4a8.w4a8_tiled_weight_bytes(N, K),), dtype=t.uint8, device="cuda"))
    out = t.full((M, N), 3.0, dtype=t.float16, device="cuda")
    assert _static_call(t, dummy, out, M, N, K, 6, 8) == -4
    t.cuda.synchronize()
    assert bool((out == 3.0).all())
    assert w4a8.lib().w4a8_init() == 0
