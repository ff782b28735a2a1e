"""ctypes binding of the CPU oracle (``w4a8_oracle.c``).

Test infrastructure only: the tests, the smoke check and the CPU-baseline leg
of the benchmark may import this module; the GPU library never does.  The
binding only marshals numpy arrays; every bit of arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w4a8_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-shared",
               "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_selftest(out_dir: str | None = None) -> str:
    """Compile the oracle together with its sanitizer driver (`selftest.c`) under AddressSanitizer and
    UndefinedBehaviorSanitizer, host only; returns the executable's path.  Running it exercises every exported
    function on ragged shapes with exact-size heap buffers."""
    exe = os.path.join(out_dir or _HERE, "oracle_selftest")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-ffp-contract=off", "-Wall", "-Wextra", "-o", exe,
           os.path.join(_HERE, "selftest.c"), _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_pack_w4.restype = ctypes.c_int
        _lib.oracle_gemm.restype = ctypes.c_int
        _lib.oracle_nibble_in_high_half_as_int8.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def half_to_float(h):
    h = _c(h, np.uint16)
    f = np.empty(h.shape, np.float32)
    _load().oracle_half_to_float(_p(h), _p(f), ctypes.c_size_t(h.size))
    return f


def float_to_half(f):
    f = _c(f, np.float32)
    h = np.empty(f.shape, np.uint16)
    _load().oracle_float_to_half(_p(f), _p(h), ctypes.c_size_t(f.size))
    return h


def double_to_half(d):
    d = _c(d, np.float64)
    h = np.empty(d.shape, np.uint16)
    _load().oracle_double_to_half(_p(d), _p(h), ctypes.c_size_t(d.size))
    return h


def pack_w4(wq):
    """int8 [N][K] in [-8,7] -> uint8 [N][K/2], low nibble = even k."""
    wq = _c(wq, np.int8)
    N, K = wq.shape
    wp = np.empty((N, K // 2), np.uint8)
    if _load().oracle_pack_w4(_p(wq), _p(wp), N, K) != 0:
        raise ValueError("weights out of [-8,7] or K odd")
    return wp


def unpack_w4(wp):
    wp = _c(wp, np.uint8)
    N, K2 = wp.shape
    wq = np.empty((N, 2 * K2), np.int8)
    _load().oracle_unpack_w4(_p(wp), _p(wq), N, 2 * K2)
    return wq


def nibble_in_high_half_as_int8(nib: int) -> int:
    return int(_load().oracle_nibble_in_high_half_as_int8(ctypes.c_uint(nib)))


def quantize_act(x_half):
    """fp16 bits [M][K] (uint16 or float16) -> (int8 [M][K], float32 [M])."""
    x = np.ascontiguousarray(x_half)
    if x.dtype == np.float16:
        x = x.view(np.uint16)
    x = _c(x, np.uint16)
    M, K = x.shape
    xq = np.empty((M, K), np.int8)
    s_a = np.empty(M, np.float32)
    _load().oracle_quantize_act(_p(x), _p(xq), _p(s_a), M, K)
    return xq, s_a


def quantize_weights_rtn(w_half):
    """fp16 [N][K] -> (int8 codes [N][K] in [-8,7], float32 scales [N])."""
    w = np.ascontiguousarray(w_half)
    if w.dtype == np.float16:
        w = w.view(np.uint16)
    w = _c(w, np.uint16)
    N, K = w.shape
    wq = np.empty((N, K), np.int8)
    s_w = np.empty(N, np.float32)
    _load().oracle_quantize_weights_rtn(_p(w), _p(wq), _p(s_w), N, K)
    return wq, s_w


def quantize_weights_clip(w_half, gamma=None, beta=None):
    """fp16 [N][K], per-channel clipping strengths (float32 [N] or None = 1) -> (int8 codes in [-8,7], float32 scales)."""
    w = np.ascontiguousarray(w_half)
    if w.dtype == np.float16:
        w = w.view(np.uint16)
    w = _c(w, np.uint16)
    N, K = w.shape
    g = None if gamma is None else _c(np.asarray(gamma, np.float32), np.float32)
    b = None if beta is None else _c(np.asarray(beta, np.float32), np.float32)
    wq = np.empty((N, K), np.int8)
    s_w = np.empty(N, np.float32)
    _load().oracle_quantize_weights_clip(_p(w), None if g is None else _p(g), None if b is None else _p(b), _p(wq), _p(s_w),
                                         N, K)
    return wq, s_w


def gemm_acc_i32(xq, wp):
    xq = _c(xq, np.int8)
    wp = _c(wp, np.uint8)
    M, K = xq.shape
    N, K2 = wp.shape
    if 2 * K2 != K:
        raise ValueError("shape mismatch")
    acc = np.empty((M, N), np.int32)
    _load().oracle_gemm_acc_i32(_p(xq), _p(wp), _p(acc), M, N, K)
    return acc


def epilogue(acc, s_a, s_w):
    """-> (y32 float32 [M][N], out fp16 bits as float16 [M][N])."""
    acc = _c(acc, np.int32)
    s_a = _c(s_a, np.float32)
    s_w = _c(s_w, np.float32)
    M, N = acc.shape
    if s_a.shape != (M,) or s_w.shape != (N,):
        raise ValueError("scale shape mismatch")
    y32 = np.empty((M, N), np.float32)
    out = np.empty((M, N), np.uint16)
    _load().oracle_epilogue(_p(acc), _p(s_a), _p(s_w), _p(y32), _p(out), M, N)
    return y32, out.view(np.float16)


def gemm(xq, s_a, wp, s_w):
    """Whole quantised linear -> (acc int32, y32 float32, out float16)."""
    acc = gemm_acc_i32(xq, wp)
    y32, out = epilogue(acc, s_a, s_w)
    return acc, y32, out


def pack_u4(u):
    """Unsigned codes [N][K] in [0, 15] -> uint8 [N][K/2], low nibble = even k (the vanilla unsigned storage)."""
    u = np.ascontiguousarray(u)
    if u.min() < 0 or u.max() > 15 or u.shape[1] % 2:
        raise ValueError("codes outside [0, 15] or odd K")
    u = u.astype(np.uint8)
    return np.ascontiguousarray(u[:, 0::2] | (u[:, 1::2] << 4))


def gemm_acc_i32_u4(xq, up):
    """sum_k xq * (u - 8) over unsigned nibbles u."""
    xq = _c(xq, np.int8)
    up = _c(up, np.uint8)
    M, K = xq.shape
    N, K2 = up.shape
    if 2 * K2 != K:
        raise ValueError("shape mismatch")
    acc = np.empty((M, N), np.int32)
    _load().oracle_gemm_acc_i32_u4(_p(xq), _p(up), _p(acc), M, N, K)
    return acc


def gemm_u4(xq, s_a, up, s_w):
    acc = gemm_acc_i32_u4(xq, up)
    y32, out = epilogue(acc, s_a, s_w)
    return acc, y32, out


def gemm_acc_i32_w8(xq, w8):
    xq = _c(xq, np.int8)
    w8 = _c(w8, np.int8)
    M, K = xq.shape
    N, K2 = w8.shape
    if K2 != K:
        raise ValueError("shape mismatch")
    acc = np.empty((M, N), np.int32)
    _load().oracle_gemm_acc_i32_w8(_p(xq), _p(w8), _p(acc), M, N, K)
    return acc


def gemm_w8(xq, s_a, w8, s_w):
    """The W8A8 linear (int8 weight codes [N][K]) -> (acc int32, y32 float32, out float16)."""
    acc = gemm_acc_i32_w8(xq, w8)
    y32, out = epilogue(acc, s_a, s_w)
    return acc, y32, out


def quantize_weights_rtn8(w_half):
    """fp16 [N][K] -> (int8 codes [N][K], float32 scales [N]), scale absmax / 127."""
    w = np.ascontiguousarray(w_half)
    if w.dtype == np.float16:
        w = w.view(np.uint16)
    w = _c(w, np.uint16)
    N, K = w.shape
    wq = np.empty((N, K), np.int8)
    s_w = np.empty(N, np.float32)
    _load().oracle_quantize_weights_rtn8(_p(w), _p(wq), _p(s_w), N, K)
    return wq, s_w


def add_rmsnorm(x_half, res_half, gamma_half, eps):
    """fp16 [M][K] x, fp16 [M][K] residual or None, fp16 [K] gain, eps -> (r float16 [M][K], y64 float64 [M][K],
    y float16 [M][K]): r = fp16(res + x), y = r / sqrt(mean r^2 + eps) * gain (see the C source)."""
    def bits(a):
        a = np.ascontiguousarray(a)
        return _c(a.view(np.uint16) if a.dtype == np.float16 else a, np.uint16)
    x = bits(x_half)
    M, K = x.shape
    res = None if res_half is None else bits(res_half)
    g = bits(gamma_half)
    if g.shape != (K,) or (res is not None and res.shape != (M, K)):
        raise ValueError("shape mismatch")
    r = np.empty((M, K), np.uint16)
    y64 = np.empty((M, K), np.float64)
    y = np.empty((M, K), np.uint16)
    _load().oracle_add_rmsnorm(_p(x), None if res is None else _p(res), _p(g), ctypes.c_double(eps), _p(r), _p(y64), _p(y), M, K)
    return r.view(np.float16), y64, y.view(np.float16)


def silu_mul(gate_up_half):
    """fp16 [M][2I] -> (y64 float64 [M][I], h float16 [M][I])."""
    g = np.ascontiguousarray(gate_up_half)
    if g.dtype == np.float16:
        g = g.view(np.uint16)
    g = _c(g, np.uint16)
    M, I2 = g.shape
    I = I2 // 2
    y64 = np.empty((M, I), np.float64)
    h = np.empty((M, I), np.uint16)
    _load().oracle_silu_mul(_p(g), _p(y64), _p(h), M, I)
    return y64, h.view(np.float16)


def quantize_weights_groups(w_half, group=128):
    """fp16 [N][K] -> (int8 codes [N][K] in [-7, 7], float32 group scales [K/group][N]): round-to-nearest with one
    scale per run of `group` consecutive k of a channel."""
    w = np.ascontiguousarray(w_half)
    if w.dtype == np.float16:
        w = w.view(np.uint16)
    w = _c(w, np.uint16)
    N, K = w.shape
    if group <= 0 or K % group:
        raise ValueError("K must be a multiple of the group size")
    wq = np.empty((N, K), np.int8)
    s_g = np.empty((K // group, N), np.float32)
    if _load().oracle_quantize_weights_groups(_p(w), group, _p(wq), _p(s_g), N, K) != 0:
        raise ValueError("bad group size")
    return wq, s_g


def gemm_fine_grained(xq, s_a, wp, s_g, group=128):
    """The fine-grained (group-wise) W4A8 linear: s_g is float32 [K/group][N].
    -> (y64 float64: the definition, y32 float32: the same in fp32 in ascending group order, out float16 = y32 rounded,
        mag float64: the sum of the absolute group terms, what a rounding bound is relative to)."""
    xq = _c(xq, np.int8)
    wp = _c(wp, np.uint8)
    s_a = _c(s_a, np.float32)
    s_g = _c(s_g, np.float32)
    M, K = xq.shape
    N, K2 = wp.shape
    if 2 * K2 != K or group <= 0 or K % group or s_g.shape != (K // group, N) or s_a.shape != (M,):
        raise ValueError("shape mismatch")
    y64 = np.empty((M, N), np.float64)
    y32 = np.empty((M, N), np.float32)
    out = np.empty((M, N), np.uint16)
    mag = np.empty((M, N), np.float64)
    lib = _load()
    lib.oracle_gemm_fine_grained.restype = ctypes.c_int
    if lib.oracle_gemm_fine_grained(_p(xq), _p(s_a), _p(wp), _p(s_g), group, _p(y64), _p(y32), _p(out), _p(mag),
                                    M, N, K) != 0:
        raise ValueError("bad group size")
    return y64, y32, out.view(np.float16), mag
