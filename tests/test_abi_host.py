"""CPU-only checks of the C-ABI library: it loads, exports what the header
declares, validates arguments before touching the GPU, and its host packing
helper agrees with the oracle.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2311_09550_amd as w4a8
from paper_2311_09550_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", h) for h in ("w4a8.h", "w4a8_tuning.h")]


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(w4a8.LIB_PATH):
        from paper_2311_09550_amd.build import build_library
        build_library(force=True)
    return w4a8.lib()


def declared_symbols():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(w[48]a8_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(L):
    syms = declared_symbols()
    assert {"w4a8_quantize_act", "w4a8_gemm", "w4a8_gemm_acc_i32", "w4a8_gemm_workspace_bytes",
            "w4a8_pack_weights_host", "w4a8_strerror", "w4a8_version"} <= set(syms)
    for s in syms:
        assert hasattr(L, s), s


def test_version_and_strerror(L):
    assert L.w4a8_version() >= 100
    seen = set()
    for code in range(0, -8, -1):
        msg = w4a8.w4a8_strerror(code)
        assert msg and msg not in seen
        seen.add(msg)
    assert "unknown" in w4a8.w4a8_strerror(-99)
    # no entry point has returned W4A8_ERR_LAUNCH on this thread: validation errors never reach HIP
    assert L.w4a8_last_hip_error() == b"hipSuccess"


def test_workspace_bytes_is_a_pure_function_of_shape(L):
    # partial sums meet in LDS: no tiling needs scratch memory, for valid and invalid shapes alike
    for shape in [(16, 5120, 5120), (1024, 27648, 5120), (0, 16, 32), (1, 16, 48)]:
        assert w4a8.w4a8_gemm_workspace_bytes(*shape) == w4a8.w4a8_gemm_workspace_bytes(*shape) == 0


def test_argument_validation_happens_before_any_launch(L):
    # fake, aligned, non-NULL "device" addresses: validation must reject these calls without dereferencing anything
    p = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    null = ctypes.c_void_p(0)
    big = ctypes.c_size_t(1 << 40)
    g = L.w4a8_gemm
    assert g(null, p, p, p, p, 1, 16, 32, p, big, null) == -1
    assert g(p, p, p, p, null, 1, 16, 32, p, big, null) == -1
    assert g(p, p, p, p, p, 0, 16, 32, p, big, null) == -2
    assert g(p, p, p, p, p, 1, 0, 32, p, big, null) == -2
    assert g(p, p, p, p, p, 1, 16, 16, p, big, null) == -2
    assert g(p, p, p, p, p, 1, 16, 48, p, big, null) == -2
    assert g(p, p, p, p, p, 1, 16, 65536 + 32, p, big, null) == -2
    assert g(odd, p, p, p, p, 1, 16, 32, p, big, null) == -3
    assert g(p, p, odd, p, p, 1, 16, 32, p, big, null) == -3
    t = L.w4a8_gemm_tuned
    assert t(p, p, p, p, p, null, 1, 16, 1024, 10, 0, p, big, null) == -7      # unknown tiling
    assert t(p, p, p, p, p, null, 1, 16, 1024, 2, 303, p, big, null) == -7     # stream: 3 row tiles / 3 waves do not exist
    assert t(p, p, p, p, p, null, 1, 16, 1024, 3, 9, p, big, null) == -7       # prefill: unknown tile id
    assert t(p, p, p, p, p, null, 65, 16, 1024, 2, 0, p, big, null) == -7      # decode tilings are for M <= 64
    assert t(p, p, p, p, p, null, 65, 16, 1024, 1, 0, p, big, null) == -7
    assert t(p, p, p, p, p, null, 16, 16, 32768, 1, 0, p, big, null) == -7     # resident: activations would not fit in registers
    assert t(p, p, p, p, p, null, 48, 16, 1024, 1, 0, p, big, null) == -7      # resident: M <= 32 only
    assert t(p, p, p, p, p, p, 1, 16, 1024, 0, 0, p, big, null) == -1         # both outputs given
    assert t(p, p, p, p, null, null, 1, 16, 1024, 0, 0, p, big, null) == -1   # no output given
    q = L.w4a8_quantize_act
    assert q(null, p, p, 1, 32, null) == -1
    assert q(p, p, p, 0, 32, null) == -2
    assert q(p, p, p, 1, 40, null) == -2
    assert q(odd, p, p, 1, 32, null) == -3
    qs = L.w4a8_quantize_act_strided
    assert qs(null, 64, p, p, 1, 32, null) == -1
    assert qs(p, 24, p, p, 1, 32, null) == -2      # rows would overlap
    assert qs(p, 36, p, p, 1, 32, null) == -2      # rows would not start 16-byte aligned
    assert qs(p, 64, p, p, 1, 40, null) == -2
    assert qs(odd, 64, p, p, 1, 32, null) == -3
    assert L.w4a8_quantize_weights(p, p, null, 4, 32, null) == -1
    assert L.w4a8_quantize_weights(p, p, p, 4, 33, null) == -2
    assert L.w4a8_quantize_weights_clipped(p, null, null, p, null, 4, 32, null) == -1
    assert L.w4a8_quantize_weights_clipped(p, p, p, p, p, 4, 48, null) == -2
    assert L.w4a8_quantize_weights_clipped(odd, null, null, p, p, 4, 32, null) == -3
    assert L.w4a8_silu_mul(p, null, 1, 8, null) == -1
    assert L.w4a8_silu_mul(p, p, 1, 12, null) == -2
    assert L.w4a8_silu_mul_quantize(p, null, p, 1, 32, null) == -1
    assert L.w4a8_silu_mul_quantize(p, p, p, 1, 24, null) == -2
    assert t(p, p, p, p, p, null, 1, 16, 1024, 4, 13, p, big, null) == -7      # tiled layout: unknown tile id
    f = L.w4a8_linear_tiled_fp16
    assert f(null, 1024, p, p, p, null, 1, 16, 1024, null) == -1
    assert f(p, 1024, p, p, null, null, 1, 16, 1024, null) == -1
    assert f(p, 1000, p, p, p, null, 1, 16, 1024, null) == -2                   # rows would overlap
    assert f(p, 1028, p, p, p, null, 1, 16, 1024, null) == -2                   # rows not 16-byte aligned
    assert f(odd, 1024, p, p, p, null, 1, 16, 1024, null) == -3
    assert f(p, 1024, p, p, p, null, 17, 16, 1024, null) == -7                  # M beyond token generation
    assert f(p, 16384, p, p, p, null, 4, 16, 16384, null) == -7                 # K beyond what a wave can hold
    nq = L.w4a8_add_rmsnorm_quantize
    eps = ctypes.c_float(1e-5)
    assert nq(null, null, p, eps, null, null, p, p, 1, 64, null) == -1
    assert nq(p, null, null, eps, null, null, p, p, 1, 64, null) == -1
    assert nq(p, null, p, eps, null, null, p, null, 1, 64, null) == -1
    assert nq(p, null, p, eps, null, null, p, p, 1, 40, null) == -2
    assert nq(p, odd, p, eps, null, null, p, p, 1, 64, null) == -3
    assert nq(p, null, p, eps, odd, null, p, p, 1, 64, null) == -3
    assert nq(p, null, p, ctypes.c_float(-1.0), null, null, p, p, 1, 64, null) == -7
    mr = L.w4a8_probe_mixed_read
    assert mr(null, big, p, ctypes.c_size_t(1 << 20), p, 0, null) == -1
    assert mr(p, big, p, ctypes.c_size_t(1 << 20), p, 4, null) == -7
    assert mr(p, ctypes.c_size_t(1024), p, ctypes.c_size_t(1 << 20), p, 0, null) == -2      # less than one iteration per compute unit
    assert mr(odd, big, p, ctypes.c_size_t(1 << 20), p, 0, null) == -3
    nl = L.w4a8_linear_tiled_norm_fp16
    assert nl(p, 1024, null, 0, null, eps, null, null, p, p, p, null, 1, 64, 1024, 0, null) == -1     # no gain vector
    assert nl(p, 1024, p, 1000, p, eps, null, null, p, p, p, null, 1, 64, 1024, 0, null) == -2        # residual rows would overlap
    assert nl(p, 1024, null, 0, odd, eps, null, null, p, p, p, null, 1, 64, 1024, 0, null) == -3
    assert nl(p, 1024, null, 0, p, ctypes.c_float(-1.0), null, null, p, p, p, null, 1, 64, 1024, 0, null) == -7
    assert nl(p, 1024, null, 0, p, eps, null, null, p, p, p, null, 1, 64, 1024, 2, null) == -7         # swiglu is 0 or 1
    assert nl(p, 1024, null, 0, p, eps, null, null, p, p, p, null, 1, 96, 1024, 1, null) == -2         # N = 2 I, I % 32 == 0
    assert nl(p, 1024, null, 0, p, eps, null, null, p, p, p, null, 5, 64, 1024, 0, null) == -7
    assert nl(p, 16384, null, 0, p, eps, null, null, p, p, p, null, 1, 64, 16384, 0, null) == -7      # K beyond 8192
    fs = L.w4a8_linear_tiled_swiglu_fp16
    assert fs(p, 1024, p, p, null, null, 1, 32, 1024, null) == -1
    assert fs(p, 1024, p, p, p, null, 1, 40, 1024, null) == -2                  # I follows the K contract
    assert fs(p, 1000, p, p, p, null, 1, 32, 1024, null) == -2
    assert fs(odd, 1024, p, p, p, null, 1, 32, 1024, null) == -3
    assert fs(p, 1024, p, p, p, null, 5, 32, 1024, null) == -7
    sg = L.w4a8_gemm_tiled_swiglu
    assert sg(p, p, p, null, p, 4, 64, 64, null) == -1
    assert sg(p, p, p, p, p, 4, 40, 64, null) == -2                            # I follows the K contract
    assert sg(p, p, p, p, p, 4, 64, 48, null) == -2
    assert sg(p, p, p, p, odd, 4, 64, 64, null) == -3
    g2 = L.w4a8_gemm_tiled_splitk_static
    assert g2(null, p, p, p, p, 64, 512, 1024, 0, 0, null) == -1
    assert g2(p, p, p, p, p, 64, 512, 1000, 0, 0, null) == -2
    assert g2(p, p, p, p, p, 64, 512, 1024, 99, 0, null) == -7
    assert g2(p, p, p, p, p, 512, 4096, 1024, 6, 8, null) == -4                  # slabs beyond the static array
    assert L.w4a8_tile_weights(null, p, 32, 128, null) == -1
    assert L.w4a8_tile_weights(p, p, 32, 100, null) == -2
    assert L.w4a8_tile_weights(p, odd, 32, 128, null) == -3
    assert L.w4a8_gemm_tiled(p, p, p, p, null, 1, 16, 32, null) == -1
    assert L.w4a8_gemm_tiled(p, p, p, p, p, 1, 16, 48, null) == -2
    assert L.w4a8_gemm_tiled_unsigned(p, p, null, p, p, null, 1, 16, 32, 0, null) == -1
    assert L.w4a8_gemm_tiled_unsigned(p, p, p, p, p, null, 1, 16, 32, 9, null) == -7
    sk = L.w4a8_gemm_tiled_splitk
    assert sk(p, p, p, p, null, 1, 16, 256, 0, 0, p, big, null) == -1
    assert sk(p, p, p, p, p, 1, 16, 48, 0, 0, p, big, null) == -2
    assert sk(p, p, p, p, p, 1, 16, 256, 13, 0, p, big, null) == -7          # unknown tile
    assert sk(p, p, p, p, p, 1, 16, 256, 0, 65, p, big, null) == -7          # too many slices
    assert sk(p, p, p, p, p, 1, 16, 256, 0, 2, null, big, null) == -1        # two slices need a workspace
    assert sk(p, p, p, p, p, 1, 16, 256, 0, 2, p, ctypes.c_size_t(127), null) == -4
    assert sk(p, p, p, p, p, 1, 16, 256, 0, 2, odd, big, null) == -3
    fg = L.w4a8_gemm_fine_grained
    assert fg(p, p, p, null, 16, p, 1, 16, 128, 0, null) == -1
    assert fg(p, p, p, p, 16, p, 1, 16, 160, 0, null) == -2      # K must be whole groups of 128
    assert fg(p, p, p, p, 12, p, 1, 16, 128, 0, null) == -2      # pitch of the scales below N
    assert fg(p, p, p, p, 18, p, 1, 16, 128, 0, null) == -2      # pitch not a multiple of 4
    assert fg(p, p, p, p, 16, p, 1, 16, 128, 7, null) == -7      # unknown tile
    assert fg(p, p, p, odd, 16, p, 1, 16, 128, 0, null) == -3
    assert L.w8a8_tile_weights(null, p, 32, 128, null) == -1
    assert L.w8a8_tile_weights(p, p, 32, 100, null) == -2
    assert L.w8a8_gemm_tiled(p, p, p, p, p, p, 1, 16, 32, 0, null) == -1        # both outputs
    assert L.w8a8_gemm_tiled(p, p, p, p, null, null, 1, 16, 32, 0, null) == -1  # no output
    assert L.w8a8_gemm_tiled(p, p, p, p, p, null, 1, 16, 48, 0, null) == -2
    assert L.w8a8_gemm_tiled(p, p, p, p, p, null, 1, 16, 32, 9, null) == -7
    assert L.w8a8_gemm_tiled(p, p, odd, p, p, null, 1, 16, 32, 0, null) == -3
    assert w4a8.w8a8_tiled_weight_bytes(32, 128) == 4096 and w4a8.w8a8_tiled_weight_bytes(33, 160) == 4 * 4096


def test_tiled_weight_bytes_counts_whole_blocks(L):
    f = w4a8.w4a8_tiled_weight_bytes
    assert f(32, 128) == 2048 and f(1, 32) == 2048 and f(33, 160) == 4 * 2048
    assert f(15360, 5120) == 15360 * 5120 // 2            # whole blocks: same size as the row-major array
    assert f(5120, 13824) == 5120 * 13824 // 2
    assert f(16, 48) == 0 and f(0, 128) == 0              # outside the contract


def test_host_packing_matches_oracle_and_rejects_bad_codes(L, oracle):
    _, wq, _, _ = synth.uniform_codes(2, 64, 96)
    assert np.array_equal(w4a8.w4a8_pack_weights_host(wq), oracle.pack_w4(wq))
    # all 256 nibble pairs
    pairs = np.array([[a, c] for a in range(-8, 8) for c in range(-8, 8)], np.int8).reshape(1, -1)
    assert np.array_equal(w4a8.w4a8_pack_weights_host(pairs), oracle.pack_w4(pairs))
    # the paper's worked value: -7 is stored as nibble 1001
    assert w4a8.w4a8_pack_weights_host(np.array([[-7, 0]], np.int8))[0, 0] == 0b1001
    bad = wq.copy(); bad[3, 5] = 8
    with pytest.raises(w4a8.W4A8Error) as e:
        w4a8.w4a8_pack_weights_host(bad)
    assert e.value.code == -6


def test_split_workspace_is_a_pure_function_of_shape(L):
    f = w4a8.w4a8_gemm_tiled_workspace_bytes
    assert f(1024, 15360, 5120) == 0                      # 240 tiles of 256 x 256: no split
    assert f(16, 48, 40) == 0 and f(0, 16, 32) == 0       # outside the contract
    for shape in [(32, 5120, 13824), (128, 5120, 13824), (64, 4096, 11008), (100, 5120, 5120)]:
        n = f(*shape)
        assert n == f(*shape) and n % (shape[0] * shape[1] * 4) == 0 and 2 <= n // (shape[0] * shape[1] * 4) <= 8
    # 17 to 64 tokens with a K that fits a wave's registers: the weight-streaming kernel in one slice, no slabs
    assert f(32, 5120, 5120) == 0 and f(64, 4096, 4096) == 0 and f(64, 15360, 5120) == 0


def test_probe_arguments(L):
    p, null, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0), ctypes.c_void_p(0x1008)
    assert L.w4a8_probe_stream_read(null, ctypes.c_size_t(1 << 20), p, null) == -1
    assert L.w4a8_probe_stream_read(p, ctypes.c_size_t(8), p, null) == -2
    assert L.w4a8_probe_stream_read(odd, ctypes.c_size_t(1 << 20), p, null) == -3
    assert L.w4a8_probe_mfma_int8(null, 10, 0, null) == -1
    assert L.w4a8_probe_mfma_int8(p, 0, 0, null) == -7
    assert L.w4a8_probe_mfma_int8(p, 10, 2, null) == -7
