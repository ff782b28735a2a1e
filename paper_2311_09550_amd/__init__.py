"""Thin Python binding of the MI355X W4A8 library (``libw4a8.so``).

Only argument marshalling happens here: torch supplies device memory and the
current HIP stream, every step of the path runs in the HIP kernels behind the C
ABI declared in ``include/w4a8.h`` and ``include/w4a8_tuning.h``.  There is no CPU fallback: if the library
has not been built (``python -m paper_2311_09550_amd.build`` or
``__graft_entry__.build()``), the first call raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libw4a8.so")

TILING_AUTO, TILING_DECODE_RESIDENT, TILING_DECODE_STREAM, TILING_PREFILL, TILING_PREFILL_TILED = 0, 1, 2, 3, 4
TILING_DECODE_RESIDENT_TILED, TILING_DECODE_STREAM_TILED, TILING_AUTO_TILED = 5, 6, 7
_TILED_TILINGS = (TILING_PREFILL_TILED, TILING_DECODE_RESIDENT_TILED, TILING_DECODE_STREAM_TILED, TILING_AUTO_TILED)

_lib = None


class W4A8Error(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"w4a8 error {code}: {what}")
        self.code = code


def lib():
    """Load libw4a8.so (once).  Fails loudly when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build the HIP library first "
                "(python -m paper_2311_09550_amd.build); there is no fallback path")
        # torch first: it ships its own HIP runtime, and the one loaded first serves the whole process.  Loaded the
        # other way round, this library's kernels are registered with a runtime that torch's streams and memory do
        # not belong to, and every launch is rejected.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.w4a8_version.restype = i
        L.w4a8_strerror.restype = ctypes.c_char_p
        L.w4a8_strerror.argtypes = [i]
        L.w4a8_quantize_act.argtypes = [vp, vp, vp, i, i, vp]
        L.w4a8_quantize_act_strided.restype = i
        L.w4a8_quantize_act_strided.argtypes = [vp, ctypes.c_longlong, vp, vp, i, i, vp]
        L.w4a8_gemm_workspace_bytes.restype = sz
        L.w4a8_gemm_workspace_bytes.argtypes = [i, i, i]
        L.w4a8_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp, sz, vp]
        L.w4a8_gemm_acc_i32.argtypes = [vp, vp, vp, i, i, i, vp, sz, vp]
        L.w4a8_gemm_tuned.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
        L.w4a8_quantize_weights.argtypes = [vp, vp, vp, i, i, vp]
        L.w4a8_quantize_weights_clipped.argtypes = [vp, vp, vp, vp, vp, i, i, vp]
        L.w4a8_silu_mul.argtypes = [vp, vp, i, i, vp]
        L.w4a8_silu_mul_quantize.argtypes = [vp, vp, vp, i, i, vp]
        L.w4a8_pack_weights_host.argtypes = [vp, vp, i, i]
        L.w4a8_tiled_weight_bytes.restype = sz
        L.w4a8_tiled_weight_bytes.argtypes = [i, i]
        L.w4a8_tile_weights.argtypes = [vp, vp, i, i, vp]
        L.w4a8_gemm_tiled.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp]
        L.w8a8_tiled_weight_bytes.restype = sz
        L.w8a8_tiled_weight_bytes.argtypes = [i, i]
        L.w8a8_tile_weights.argtypes = [vp, vp, i, i, vp]
        L.w8a8_gemm_tiled.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
        L.w8a8_tile_weights.restype = i
        L.w8a8_gemm_tiled.restype = i
        L.w4a8_gemm_tiled_unsigned.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
        L.w4a8_gemm_tiled_workspace_bytes.restype = sz
        L.w4a8_gemm_tiled_workspace_bytes.argtypes = [i, i, i]
        L.w4a8_gemm_tiled_splitk.restype = i
        L.w4a8_gemm_tiled_splitk.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp]
        L.w4a8_gemm_tiled_splitk_static.restype = i
        L.w4a8_gemm_tiled_splitk_static.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp]
        L.w4a8_gemm_tiled_swiglu.restype = i
        L.w4a8_gemm_tiled_swiglu.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp]
        L.w4a8_linear_tiled_fp16.restype = i
        L.w4a8_linear_tiled_fp16.argtypes = [vp, ctypes.c_longlong, vp, vp, vp, vp, i, i, i, vp]
        L.w4a8_linear_tiled_norm_fp16.restype = i
        L.w4a8_linear_tiled_norm_fp16.argtypes = [vp, ctypes.c_longlong, vp, ctypes.c_longlong, vp, ctypes.c_float, vp, vp, vp, vp,
                                                  vp, vp, i, i, i, i, vp]
        L.w4a8_add_rmsnorm_quantize.restype = i
        L.w4a8_add_rmsnorm_quantize.argtypes = [vp, vp, vp, ctypes.c_float, vp, vp, vp, vp, i, i, vp]
        L.w4a8_linear_tiled_swiglu_fp16.restype = i
        L.w4a8_linear_tiled_swiglu_fp16.argtypes = [vp, ctypes.c_longlong, vp, vp, vp, vp, i, i, i, vp]
        L.w4a8_init.restype = i
        L.w4a8_init.argtypes = []
        L.w4a8_probe_stream_read.restype = i
        L.w4a8_probe_stream_read.argtypes = [vp, sz, vp, vp]
        L.w4a8_probe_mixed_read.restype = i
        L.w4a8_probe_mixed_read.argtypes = [vp, sz, vp, sz, vp, i, vp]
        L.w4a8_probe_read_pattern.restype = i
        L.w4a8_probe_read_pattern.argtypes = [vp, sz, vp, i, i, i, vp]
        L.w4a8_probe_mfma_int8.restype = i
        L.w4a8_probe_mfma_int8.argtypes = [vp, i, i, vp]
        L.w4a8_gemm_fine_grained.restype = i
        L.w4a8_gemm_fine_grained.argtypes = [vp, vp, vp, vp, i, vp, i, i, i, i, vp]
        L.w4a8_gemm_tiled_unsigned.restype = i
        for name in ("w4a8_quantize_act", "w4a8_gemm", "w4a8_gemm_acc_i32", "w4a8_gemm_tuned",
                     "w4a8_quantize_weights", "w4a8_quantize_weights_clipped", "w4a8_silu_mul", "w4a8_silu_mul_quantize", "w4a8_pack_weights_host",
                     "w4a8_tile_weights", "w4a8_gemm_tiled"):
            getattr(L, name).restype = i
        L.w4a8_last_hip_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(code: int):
    if code != 0:
        detail = f" ({lib().w4a8_last_hip_error().decode()})" if code == -5 else ""
        raise W4A8Error(code, lib().w4a8_strerror(code).decode() + detail)


def _torch():
    import torch
    return torch


def _stream():
    """torch's current stream on the current device: the library launches on the device that is current when it is
    called, and `_on_current_device` holds every tensor argument to that device."""
    torch = _torch()
    return ctypes.c_void_p(torch.cuda.current_stream(torch.cuda.current_device()).cuda_stream)


def _on_current_device(t, what):
    torch = _torch()
    if not t.is_cuda:
        raise TypeError(f"{what}: expected a device tensor")
    if t.device.index != torch.cuda.current_device():
        raise ValueError(f"{what} is on {t.device} but the current device is cuda:{torch.cuda.current_device()}: "
                         "call under torch.cuda.device(...) of the tensors' device")


def _dev(t, dtype, what):
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what}: expected a contiguous device tensor of {dtype}")
    _on_current_device(t, what)
    return ctypes.c_void_p(t.data_ptr())


def _shaped(t, shape, what):
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def bound_call(name: str, *args):
    """A launch with its arguments marshalled once, for loops that repeat the same call: `name` is an entry point of
    the C ABI, `args` its arguments in the C order without the trailing stream (device tensors, ints, or None for a
    NULL pointer).  Returns a function of no arguments that launches on torch's current stream of the tensors' device
    (which the caller keeps current) and raises on an error code.  The tensors are kept alive by the returned
    function; shapes and dtypes are the caller's responsibility here (the C side still validates pointers, sizes and
    alignment)."""
    torch = _torch()
    fn = getattr(lib(), name)
    keep = [a for a in args if isinstance(a, torch.Tensor)]
    for t in keep:
        if not (t.is_cuda and t.is_contiguous()):
            raise TypeError(f"{name}: expected contiguous device tensors")
    if len({t.device for t in keep}) > 1:
        raise ValueError(f"{name}: the tensors are on different devices")
    device = keep[0].device if keep else torch.device("cuda", torch.cuda.current_device())
    cargs = [ctypes.c_void_p(a.data_ptr()) if isinstance(a, torch.Tensor) else a for a in args]
    current_stream = torch.cuda.current_stream

    def call(_keep=keep):
        code = fn(*cargs, ctypes.c_void_p(current_stream(device).cuda_stream))
        if code != 0:
            _check(code)
    return call


def w4a8_probe_stream_read(buf, sink):
    """Read-only streaming reduction over a uint8 device buffer (a probe of the achievable read rate)."""
    torch = _torch()
    _check(lib().w4a8_probe_stream_read(_dev(buf, torch.uint8, "buf"), buf.numel(), _dev(sink, torch.int32, "sink"), _stream()))


def w4a8_probe_read_pattern(buf, sink, pattern: int, loads: int, workgroups_per_cu: int):
    """The read probe with the access pattern, loads in flight and workgroups per compute unit chosen by the caller."""
    torch = _torch()
    _check(lib().w4a8_probe_read_pattern(_dev(buf, torch.uint8, "buf"), buf.numel(), _dev(sink, torch.int32, "sink"),
                                         pattern, loads, workgroups_per_cu, _stream()))


def w4a8_probe_mixed_read(cold, hot, sink, mode: int):
    """The read probe with a cold (read once) and a hot (cache-resident, shared) buffer; returns the bytes every
    compute unit reads in this launch (cold + hot)."""
    torch = _torch()
    _check(lib().w4a8_probe_mixed_read(_dev(cold, torch.uint8, "cold"), cold.numel(), _dev(hot, torch.uint8, "hot"), hot.numel(),
                                       _dev(sink, torch.int32, "sink"), mode, _stream()))
    cus = torch.cuda.get_device_properties(sink.device).multi_processor_count
    per_iter = (4096 if mode == 2 else 2048) * 16
    iters = cold.numel() // cus // per_iter
    return iters * 4096 * 16


def w4a8_probe_mfma_int8(sink, iters: int, pattern: int = 1):
    """Register-resident int8 MFMA loop on every compute unit; returns the operations it performs."""
    torch = _torch()
    _check(lib().w4a8_probe_mfma_int8(_dev(sink, torch.int32, "sink"), iters, pattern, _stream()))
    cus = torch.cuda.get_device_properties(sink.device).multi_processor_count
    return cus * 8 * iters * 8 * 65536


def w4a8_version() -> int:
    return int(lib().w4a8_version())


def w4a8_strerror(code: int) -> str:
    return lib().w4a8_strerror(code).decode()


def w4a8_gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().w4a8_gemm_workspace_bytes(M, N, K))


_workspaces = {}


def workspace(M: int, N: int, K: int, device=None):
    """A zero-filled workspace tensor large enough for (M, N, K), cached per device and stream."""
    torch = _torch()
    device = torch.device("cuda", torch.cuda.current_device()) if device is None else torch.device(device)
    need = max(w4a8_gemm_workspace_bytes(M, N, K), 256)
    key = (device.index, torch.cuda.current_stream(device).cuda_stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.zeros(need, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def w4a8_quantize_act(x, xq=None, s_a=None):
    """fp16 [M][K] -> (int8 [M][K], fp32 [M])."""
    torch = _torch()
    M, K = x.shape
    xq = torch.empty((M, K), dtype=torch.int8, device=x.device) if xq is None else _shaped(xq, (M, K), "xq")
    s_a = torch.empty((M,), dtype=torch.float32, device=x.device) if s_a is None else _shaped(s_a, (M,), "s_a")
    _check(lib().w4a8_quantize_act(_dev(x, torch.float16, "x"), _dev(xq, torch.int8, "xq"),
                                   _dev(s_a, torch.float32, "s_a"), M, K, _stream()))
    return xq, s_a


def w4a8_quantize_act_strided(x, xq=None, s_a=None):
    """fp16 [M][K] view whose rows are x.stride(0) elements apart (a column block of a wider matrix) -> (int8, fp32)."""
    torch = _torch()
    M, K = x.shape
    if not (x.is_cuda and x.dtype == torch.float16 and x.stride(1) == 1):
        raise TypeError("x: expected a device fp16 view with unit column stride")
    _on_current_device(x, "x")
    xq = torch.empty((M, K), dtype=torch.int8, device=x.device) if xq is None else _shaped(xq, (M, K), "xq")
    s_a = torch.empty((M,), dtype=torch.float32, device=x.device) if s_a is None else _shaped(s_a, (M,), "s_a")
    _check(lib().w4a8_quantize_act_strided(ctypes.c_void_p(x.data_ptr()), x.stride(0), _dev(xq, torch.int8, "xq"),
                                           _dev(s_a, torch.float32, "s_a"), M, K, _stream()))
    return xq, s_a


def w4a8_gemm(xq, s_a, wp, s_w, out=None, ws=None):
    """int8 [M][K], fp32 [M], uint8 [N][K/2], fp32 [N] -> fp16 [M][N]."""
    torch = _torch()
    M, K = xq.shape
    N = wp.shape[0]
    if wp.shape[1] * 2 != K or s_a.shape != (M,) or s_w.shape != (N,):
        raise ValueError("shape mismatch")
    out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    ws = workspace(M, N, K, xq.device) if ws is None else ws
    _check(lib().w4a8_gemm(_dev(xq, torch.int8, "xq"), _dev(s_a, torch.float32, "s_a"), _dev(wp, torch.uint8, "wp"),
                           _dev(s_w, torch.float32, "s_w"), _dev(out, torch.float16, "out"), M, N, K,
                           _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()))
    return out


def w4a8_gemm_acc_i32(xq, wp, acc=None, ws=None):
    """int8 [M][K], uint8 [N][K/2] -> int32 [M][N] raw sums."""
    torch = _torch()
    M, K = xq.shape
    N = wp.shape[0]
    if wp.shape[1] * 2 != K:
        raise ValueError("shape mismatch")
    acc = torch.empty((M, N), dtype=torch.int32, device=xq.device) if acc is None else acc
    if acc.shape != (M, N):
        raise ValueError("acc shape mismatch")
    ws = workspace(M, N, K, xq.device) if ws is None else ws
    _check(lib().w4a8_gemm_acc_i32(_dev(xq, torch.int8, "xq"), _dev(wp, torch.uint8, "wp"), _dev(acc, torch.int32, "acc"),
                                   M, N, K, _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()))
    return acc


def w4a8_gemm_tuned(xq, s_a, wp, s_w, tiling: int, variant: int = 0, want_acc: bool = False, out=None, ws=None, N=None):
    """Forced tiling / variant; returns fp16 [M][N], or int32 [M][N] when want_acc.  With a tiling over the tiled
    layout (TILING_*_TILED), wp is the flat tiled array of w4a8_tile_weights and N must be given."""
    torch = _torch()
    M, K = xq.shape
    if tiling in _TILED_TILINGS:
        if N is None or wp.numel() != w4a8_tiled_weight_bytes(N, K):
            raise ValueError("tiled weights: N missing or array size mismatch")
    else:
        N = wp.shape[0]
        if wp.shape[1] * 2 != K:
            raise ValueError("shape mismatch")
    ws = workspace(M, N, K, xq.device) if ws is None else ws
    if want_acc:
        out = torch.empty((M, N), dtype=torch.int32, device=xq.device) if out is None else out
        o16, o32 = None, _dev(out, torch.int32, "acc")
        sa = None if s_a is None else _dev(s_a, torch.float32, "s_a")
        sw = None if s_w is None else _dev(s_w, torch.float32, "s_w")
    else:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
        o16, o32 = _dev(out, torch.float16, "out"), None
        sa, sw = _dev(s_a, torch.float32, "s_a"), _dev(s_w, torch.float32, "s_w")
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    _check(lib().w4a8_gemm_tuned(_dev(xq, torch.int8, "xq"), sa, _dev(wp, torch.uint8, "wp"), sw, o16, o32, M, N, K,
                                 tiling, variant, _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()))
    return out


def w4a8_tiled_weight_bytes(N: int, K: int) -> int:
    return int(lib().w4a8_tiled_weight_bytes(N, K))


def w4a8_tile_weights(wp, wt=None):
    """uint8 [N][K/2] packed int4 -> flat uint8 array in the tiled layout for large M."""
    torch = _torch()
    N, K = wp.shape[0], wp.shape[1] * 2
    nbytes = w4a8_tiled_weight_bytes(N, K)
    if nbytes == 0:
        _check(-2)
    wt = torch.empty((nbytes,), dtype=torch.uint8, device=wp.device) if wt is None else wt
    if wt.numel() != nbytes:
        raise ValueError("wt size mismatch")
    _check(lib().w4a8_tile_weights(_dev(wp, torch.uint8, "wp"), _dev(wt, torch.uint8, "wt"), N, K, _stream()))
    return wt


def w4a8_gemm_tiled(xq, s_a, wt, s_w, out=None):
    """int8 [M][K], fp32 [M], tiled weights of N = len(s_w) channels, fp32 [N] -> fp16 [M][N]."""
    torch = _torch()
    M, K = xq.shape
    N = s_w.shape[0]
    if wt.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    _check(lib().w4a8_gemm_tiled(_dev(xq, torch.int8, "xq"), _dev(s_a, torch.float32, "s_a"), _dev(wt, torch.uint8, "wt"),
                                 _dev(s_w, torch.float32, "s_w"), _dev(out, torch.float16, "out"), M, N, K, _stream()))
    return out


def w8a8_tiled_weight_bytes(N: int, K: int) -> int:
    return int(lib().w8a8_tiled_weight_bytes(N, K))


def w8a8_tile_weights(w8, wt=None):
    """int8 [N][K] weight codes -> flat uint8 array in the tiled layout of the W8A8 variant."""
    torch = _torch()
    N, K = w8.shape
    nbytes = w8a8_tiled_weight_bytes(N, K)
    if nbytes == 0:
        _check(-2)
    wt = torch.empty((nbytes,), dtype=torch.uint8, device=w8.device) if wt is None else wt
    if wt.numel() != nbytes:
        raise ValueError("wt size mismatch")
    _check(lib().w8a8_tile_weights(_dev(w8, torch.int8, "w8"), _dev(wt, torch.uint8, "wt"), N, K, _stream()))
    return wt


def w8a8_gemm_tiled(xq, s_a, wt, s_w, N=None, variant: int = 0, want_acc: bool = False, out=None):
    """W8A8 linear over tiled int8 weights -> fp16 [M][N], or the raw int32 sums when want_acc."""
    torch = _torch()
    M, K = xq.shape
    N = s_w.shape[0] if N is None else N
    if wt.numel() != w8a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    if want_acc:
        out = torch.empty((M, N), dtype=torch.int32, device=xq.device) if out is None else out
        o16, o32 = None, _dev(out, torch.int32, "acc")
        sa = None if s_a is None else _dev(s_a, torch.float32, "s_a")
        sw = None if s_w is None else _dev(s_w, torch.float32, "s_w")
    else:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
        o16, o32 = _dev(out, torch.float16, "out"), None
        sa, sw = _dev(s_a, torch.float32, "s_a"), _dev(s_w, torch.float32, "s_w")
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    _check(lib().w8a8_gemm_tiled(_dev(xq, torch.int8, "xq"), sa, _dev(wt, torch.uint8, "wt"), sw, o16, o32, M, N, K, variant,
                                 _stream()))
    return out


def w4a8_gemm_tiled_unsigned(xq, s_a, ut, s_w, N=None, variant: int = 0, want_acc: bool = False, out=None):
    """The storage ablation: tiled unsigned nibbles u = w + 8 -> fp16 [M][N], or the raw int32 sums when want_acc."""
    torch = _torch()
    M, K = xq.shape
    N = s_w.shape[0] if N is None else N
    if ut.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    if want_acc:
        out = torch.empty((M, N), dtype=torch.int32, device=xq.device) if out is None else out
        o16, o32 = None, _dev(out, torch.int32, "acc")
        sa = None if s_a is None else _dev(s_a, torch.float32, "s_a")
        sw = None if s_w is None else _dev(s_w, torch.float32, "s_w")
    else:
        out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
        o16, o32 = _dev(out, torch.float16, "out"), None
        sa, sw = _dev(s_a, torch.float32, "s_a"), _dev(s_w, torch.float32, "s_w")
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    _check(lib().w4a8_gemm_tiled_unsigned(_dev(xq, torch.int8, "xq"), sa, _dev(ut, torch.uint8, "ut"), sw, o16, o32, M, N, K,
                                          variant, _stream()))
    return out


def w4a8_gemm_tiled_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().w4a8_gemm_tiled_workspace_bytes(M, N, K))


def w4a8_gemm_tiled_splitk(xq, s_a, wt, s_w, variant: int = 0, splits: int = 0, ws=None, out=None):
    """w4a8_gemm_tiled with K cut into slices over workgroups when the tiles alone would not fill the chip.  ws: a
    uint8 device buffer of at least w4a8_gemm_tiled_workspace_bytes(M, N, K) bytes (splits = 0) or splits * M * N * 4
    (forced); allocated here when None."""
    torch = _torch()
    M, K = xq.shape
    N = s_w.shape[0]
    if wt.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    if ws is None:
        need = w4a8_gemm_tiled_workspace_bytes(M, N, K) if splits == 0 else max(splits, 1) * M * N * 4
        ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=xq.device)
    _check(lib().w4a8_gemm_tiled_splitk(_dev(xq, torch.int8, "xq"), _dev(s_a, torch.float32, "s_a"), _dev(wt, torch.uint8, "wt"),
                                        _dev(s_w, torch.float32, "s_w"), _dev(out, torch.float16, "out"), M, N, K, variant,
                                        splits, _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()))
    return out


def w4a8_gemm_tiled_swiglu(xq, s_a, wt_gu, s_w_gu, h=None):
    """int8 [M][K], fp32 [M], tiled weights of the 2 I interleaved gate / up channels, fp32 [2 I] -> h = fp16 [M][I],
    silu(gate) * up applied in the GEMM's epilogue."""
    torch = _torch()
    M, K = xq.shape
    N = s_w_gu.shape[0]
    if N % 2 or wt_gu.numel() != w4a8_tiled_weight_bytes(N, K) or tuple(s_a.shape) != (M,):
        raise ValueError("shape mismatch")
    I = N // 2
    h = torch.empty((M, I), dtype=torch.float16, device=xq.device) if h is None else _shaped(h, (M, I), "h")
    _check(lib().w4a8_gemm_tiled_swiglu(_dev(xq, torch.int8, "xq"), _dev(s_a, torch.float32, "s_a"), _dev(wt_gu, torch.uint8, "wt_gu"),
                                        _dev(s_w_gu, torch.float32, "s_w_gu"), _dev(h, torch.float16, "h"), M, I, K, _stream()))
    return h


def interleave_gate_up(w_gate_up):
    """[2 I][...] rows (gate rows, then up rows) -> rows interleaved gate_0, up_0, gate_1, up_1, ...: the order
    w4a8_gemm_tiled_swiglu expects its channels in (a view operation on the caller's weights, before quantisation)."""
    I = w_gate_up.shape[0] // 2
    return w_gate_up.reshape(2, I, *w_gate_up.shape[1:]).transpose(0, 1).reshape(w_gate_up.shape).contiguous()


def w4a8_linear_tiled_fp16(x, wt, s_w, out=None, s_a_out=None):
    """fp16 [M][K] view (unit column stride, rows x.stride(0) apart), tiled weights, fp32 [N] -> fp16 [M][N]: per-token
    quantisation and W4A8 GEMM in one launch (M <= 4, rows small enough for LDS).  s_a_out (fp32 [M]) also receives the scales."""
    torch = _torch()
    M, K = x.shape
    N = s_w.shape[0]
    if not (x.is_cuda and x.dtype == torch.float16 and x.stride(1) == 1):
        raise TypeError("x: expected a device fp16 view with unit column stride")
    _on_current_device(x, "x")
    if wt.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    out = torch.empty((M, N), dtype=torch.float16, device=x.device) if out is None else out
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    if s_a_out is not None and tuple(s_a_out.shape) != (M,):
        raise ValueError("s_a_out shape mismatch")
    _check(lib().w4a8_linear_tiled_fp16(ctypes.c_void_p(x.data_ptr()), x.stride(0), _dev(wt, torch.uint8, "wt"),
                                        _dev(s_w, torch.float32, "s_w"), _dev(out, torch.float16, "out"),
                                        None if s_a_out is None else _dev(s_a_out, torch.float32, "s_a_out"), M, N, K,
                                        _stream()))
    return out


def w4a8_add_rmsnorm_quantize(x, res, gamma, eps: float, r_out=None, y_out=None, xq=None, s_a=None):
    """fp16 [M][K] x, fp16 [M][K] residual or None, fp16 [K] gain -> (xq int8 [M][K], s_a fp32 [M]) of
    y = rmsnorm(res + x) * gamma, in one launch; r_out / y_out (fp16 [M][K] or None) receive res + x and y."""
    torch = _torch()
    M, K = x.shape
    for name, t, shape in (("res", res, (M, K)), ("gamma", gamma, (K,)), ("r_out", r_out, (M, K)), ("y_out", y_out, (M, K))):
        if t is not None and tuple(t.shape) != shape:
            raise ValueError(f"{name} shape mismatch")
    xq = torch.empty((M, K), dtype=torch.int8, device=x.device) if xq is None else xq
    s_a = torch.empty((M,), dtype=torch.float32, device=x.device) if s_a is None else s_a
    if tuple(xq.shape) != (M, K) or tuple(s_a.shape) != (M,):
        raise ValueError("xq / s_a shape mismatch")
    opt = lambda t, name: None if t is None else _dev(t, torch.float16, name)
    _check(lib().w4a8_add_rmsnorm_quantize(_dev(x, torch.float16, "x"), opt(res, "res"), _dev(gamma, torch.float16, "gamma"),
                                           float(eps), opt(r_out, "r_out"), opt(y_out, "y_out"), _dev(xq, torch.int8, "xq"),
                                           _dev(s_a, torch.float32, "s_a"), M, K, _stream()))
    return xq, s_a


def w4a8_linear_tiled_norm_fp16(x, res, gamma, eps: float, wt, s_w, swiglu: bool = False, out=None, r_out=None, y_out=None,
                                s_a_out=None):
    """fp16 [M][K] views x and res (or None), fp16 [K] gain, tiled weights -> the linear of rmsnorm(res + x) * gamma in
    one launch: fp16 [M][N], or h = fp16 [M][N / 2] with swiglu (interleaved gate / up channels).  r_out / y_out (dense
    fp16 [M][K] or None) receive res + x and the normalised rows."""
    torch = _torch()
    M, K = x.shape
    N = s_w.shape[0]
    for name, t in (("x", x), ("res", res)):
        if t is not None and not (t.is_cuda and t.dtype == torch.float16 and t.stride(1) == 1 and tuple(t.shape) == (M, K)):
            raise TypeError(f"{name}: expected a device fp16 [M][K] view with unit column stride")
    _on_current_device(x, "x")
    if wt.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    cols = N // 2 if swiglu else N
    out = torch.empty((M, cols), dtype=torch.float16, device=x.device) if out is None else out
    if tuple(out.shape) != (M, cols):
        raise ValueError("out shape mismatch")
    for name, t in (("r_out", r_out), ("y_out", y_out)):
        if t is not None and tuple(t.shape) != (M, K):
            raise ValueError(f"{name} shape mismatch")
    if s_a_out is not None and tuple(s_a_out.shape) != (M,):
        raise ValueError("s_a_out shape mismatch")
    opt = lambda t, dt, name: None if t is None else _dev(t, dt, name)
    _check(lib().w4a8_linear_tiled_norm_fp16(ctypes.c_void_p(x.data_ptr()), x.stride(0),
                                             None if res is None else ctypes.c_void_p(res.data_ptr()),
                                             0 if res is None else res.stride(0), _dev(gamma, torch.float16, "gamma"),
                                             float(eps), opt(r_out, torch.float16, "r_out"), opt(y_out, torch.float16, "y_out"),
                                             _dev(wt, torch.uint8, "wt"), _dev(s_w, torch.float32, "s_w"),
                                             _dev(out, torch.float16, "out"), opt(s_a_out, torch.float32, "s_a_out"), M, N, K,
                                             1 if swiglu else 0, _stream()))
    return out


def w4a8_linear_tiled_swiglu_fp16(x, wt_gu, s_w_gu, h=None, s_a_out=None):
    """fp16 [M][K] view, tiled weights of the 2 I interleaved gate / up channels, fp32 [2 I] -> h = fp16 [M][I]:
    per-token quantisation, W4A8 GEMM and SiLU(gate) * up in one launch (M <= 4, rows small enough for LDS)."""
    torch = _torch()
    M, K = x.shape
    N = s_w_gu.shape[0]
    if N % 2:
        raise ValueError("s_w_gu holds the scales of 2 I interleaved channels")
    if not (x.is_cuda and x.dtype == torch.float16 and x.stride(1) == 1):
        raise TypeError("x: expected a device fp16 view with unit column stride")
    _on_current_device(x, "x")
    if wt_gu.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (2 I, K)")
    h = torch.empty((M, N // 2), dtype=torch.float16, device=x.device) if h is None else h
    if h.shape != (M, N // 2):
        raise ValueError("h shape mismatch")
    if s_a_out is not None and tuple(s_a_out.shape) != (M,):
        raise ValueError("s_a_out shape mismatch")
    _check(lib().w4a8_linear_tiled_swiglu_fp16(ctypes.c_void_p(x.data_ptr()), x.stride(0), _dev(wt_gu, torch.uint8, "wt_gu"),
                                               _dev(s_w_gu, torch.float32, "s_w_gu"), _dev(h, torch.float16, "h"),
                                               None if s_a_out is None else _dev(s_a_out, torch.float32, "s_a_out"), M,
                                               N // 2, K, _stream()))
    return h


STATIC_SCRATCH_BYTES = 16 << 20


def w4a8_init():
    """Per-device set-up (LDS allowances, address of the static scratch array) for torch's current device."""
    _check(lib().w4a8_init())


def w4a8_gemm_tiled_splitk_static(xq, s_a, wt, s_w, out, variant: int = 0, splits: int = 0):
    """w4a8_gemm_tiled_splitk without a workspace argument: the slabs live in the library's static scratch array.
    `out` (fp16 [M][N]) is the caller's; nothing is allocated here or in the library."""
    torch = _torch()
    M, K = xq.shape
    N = s_w.shape[0]
    if wt.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    _check(lib().w4a8_gemm_tiled_splitk_static(_dev(xq, torch.int8, "xq"), _dev(s_a, torch.float32, "s_a"),
                                               _dev(wt, torch.uint8, "wt"), _dev(s_w, torch.float32, "s_w"),
                                               _dev(out, torch.float16, "out"), M, N, K, variant, splits, _stream()))
    return out


def w4a8_gemm_fine_grained(xq, s_a, wt, s_g, N=None, variant: int = 0, out=None):
    """The granularity ablation: tiled signed int4 weights with group scales s_g fp32 [K/128][ldg] (ldg >= N, a
    multiple of 4; columns past N are ignored) -> fp16 [M][N]."""
    torch = _torch()
    M, K = xq.shape
    G, ldg = s_g.shape
    N = ldg if N is None else N
    if G * 128 != K:
        raise ValueError("s_g must have K / 128 rows")
    if wt.numel() != w4a8_tiled_weight_bytes(N, K):
        raise ValueError("tiled weight array does not match (N, K)")
    out = torch.empty((M, N), dtype=torch.float16, device=xq.device) if out is None else out
    if out.shape != (M, N):
        raise ValueError("out shape mismatch")
    _check(lib().w4a8_gemm_fine_grained(_dev(xq, torch.int8, "xq"), _dev(s_a, torch.float32, "s_a"), _dev(wt, torch.uint8, "wt"),
                                        _dev(s_g, torch.float32, "s_g"), ldg, _dev(out, torch.float16, "out"), M, N, K,
                                        variant, _stream()))
    return out


def w4a8_quantize_weights(w, wp=None, s_w=None):
    """fp16 [N][K] -> (uint8 [N][K/2] packed int4, fp32 [N])."""
    torch = _torch()
    N, K = w.shape
    wp = torch.empty((N, K // 2), dtype=torch.uint8, device=w.device) if wp is None else wp
    s_w = torch.empty((N,), dtype=torch.float32, device=w.device) if s_w is None else s_w
    _check(lib().w4a8_quantize_weights(_dev(w, torch.float16, "w"), _dev(wp, torch.uint8, "wp"),
                                       _dev(s_w, torch.float32, "s_w"), N, K, _stream()))
    return wp, s_w


def w4a8_quantize_weights_clipped(w, gamma=None, beta=None, wp=None, s_w=None):
    """fp16 [N][K], clipping strengths fp32 [N] (None = 1) -> (uint8 [N][K/2] packed int4, fp32 [N])."""
    torch = _torch()
    N, K = w.shape
    wp = torch.empty((N, K // 2), dtype=torch.uint8, device=w.device) if wp is None else wp
    s_w = torch.empty((N,), dtype=torch.float32, device=w.device) if s_w is None else s_w
    for v, what in ((gamma, "gamma"), (beta, "beta")):
        if v is not None and tuple(v.shape) != (N,):
            raise ValueError(f"{what}: expected {N} values")
    _check(lib().w4a8_quantize_weights_clipped(_dev(w, torch.float16, "w"),
                                               None if gamma is None else _dev(gamma, torch.float32, "gamma"),
                                               None if beta is None else _dev(beta, torch.float32, "beta"),
                                               _dev(wp, torch.uint8, "wp"), _dev(s_w, torch.float32, "s_w"), N, K, _stream()))
    return wp, s_w


def w4a8_silu_mul(gate_up, h=None):
    """fp16 [M][2I] -> fp16 [M][I]."""
    torch = _torch()
    M, I2 = gate_up.shape
    I = I2 // 2
    h = torch.empty((M, I), dtype=torch.float16, device=gate_up.device) if h is None else h
    _check(lib().w4a8_silu_mul(_dev(gate_up, torch.float16, "gate_up"), _dev(h, torch.float16, "h"), M, I, _stream()))
    return h


def w4a8_silu_mul_quantize(gate_up, xq=None, s_a=None):
    """fp16 [M][2I] -> (int8 [M][I], fp32 [M]): SiLU*up and the per-token quantiser in one pass."""
    torch = _torch()
    M, I2 = gate_up.shape
    I = I2 // 2
    xq = torch.empty((M, I), dtype=torch.int8, device=gate_up.device) if xq is None else xq
    s_a = torch.empty((M,), dtype=torch.float32, device=gate_up.device) if s_a is None else s_a
    _check(lib().w4a8_silu_mul_quantize(_dev(gate_up, torch.float16, "gate_up"), _dev(xq, torch.int8, "xq"),
                                        _dev(s_a, torch.float32, "s_a"), M, I, _stream()))
    return xq, s_a


def w4a8_pack_weights_host(wq):
    """numpy int8 [N][K] codes in [-8,7] -> numpy uint8 [N][K/2] (host helper, no GPU)."""
    import numpy as np
    wq = np.ascontiguousarray(wq)
    if wq.dtype != np.int8 or wq.ndim != 2:
        raise TypeError("wq: expected a 2-D int8 array")
    N, K = wq.shape
    wp = np.empty((N, K // 2), np.uint8)
    _check(lib().w4a8_pack_weights_host(wq.ctypes.data_as(ctypes.c_void_p), wp.ctypes.data_as(ctypes.c_void_p), N, K))
    return wp
