"""Thin ctypes binding over the C ABI declared in include/w2mm.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libw2mm.so.  torch is used for device memory and streams.  There is no CPU
fallback: if the shared library is missing or fails to load, importing this
module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libw2mm.so")

CODEC_INT2, CODEC_TERNARY = 0, 1
DT_F32, DT_BF16 = 0, 1
VARIANT_AUTO, VARIANT_DOT4, VARIANT_SMALLM, VARIANT_TILED, VARIANT_MIDM, VARIANT_SCALED16 = 0, 1, 2, 3, 4, 5
VARIANT_GEMV = 6

OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED_SHAPE, ERR_MISALIGNED = -1, -2, -3
ERR_BUFFER_TOO_SMALL, ERR_HIP, ERR_BAD_CODE = -4, -5, -6

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2508_06753_amd.build` "
        "(there is no CPU fallback)")

_lib = ctypes.CDLL(LIB_PATH)

_i64, _int, _sz, _vp = ctypes.c_int64, ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
_SIGS = {
    "w2_packed_size": [_i64, _i64, _int, ctypes.POINTER(_sz)],
    "w2_prepack": [_vp, _vp, _i64, _i64, _int, _int, _vp, _sz, _vp, _vp],
    "w2_quantize_rows": [_vp, _int, _i64, _i64, _i64, _int, _vp, _vp, _vp, _vp],
    "w2_matmul_a8": [_vp, _i64, _i64, _int, _vp, _vp, _i64, _vp, _i64, _vp, _sz, _vp],
    "w2_matmul_a8_ex": [_vp, _i64, _i64, _int, _vp, _vp, _i64, _vp, _i64, _vp, _sz, _vp, _vp],
    "w2_matmul_a8_fused": [_vp, _i64, _i64, _int, _vp, _int, _i64, _i64, _vp, _i64, _vp, _sz, _vp],
    "w2_init": [],
    "w2_matmul_a8_fused_noalloc": [_vp, _i64, _i64, _int, _vp, _int, _i64, _i64, _vp, _i64, _vp],
    "w2_matmul_a16": [_vp, _i64, _i64, _int, _vp, _i64, _i64, _vp, _i64, _vp, _sz, _vp],
    "w2_matmul_a16_ex": [_vp, _i64, _i64, _int, _vp, _i64, _i64, _vp, _i64, _vp, _sz, _vp, _vp],
    "w2_workspace_size": [_i64, _i64, _i64, _int, _int, ctypes.POINTER(_sz)],
    "w2_debug_group_acc_a8": [_vp, _i64, _i64, _int, _vp, _i64, _vp, _vp, _vp],
    "w2_debug_unpack": [_vp, _i64, _i64, _int, _int, _vp, _vp, _vp],
    "w2_debug_stream_read": [_vp, _sz, _vp, _vp, _vp],
    "w2_debug_int8_gemv": [_vp, _i64, _i64, _vp, _vp, _vp],
    "w2_matmul_a8_epi": [_vp, _i64, _i64, _int, _vp, _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp, _vp],
    "w2_matmul_a16_epi": [_vp, _i64, _i64, _int, _vp, _i64, _i64, _vp, _i64, _vp, _vp, _sz, _vp, _vp],
    "w2_matmul_a8_fused_epi": [_vp, _i64, _i64, _int, _vp, _int, _i64, _i64, _vp, _i64, _vp, _vp, _sz, _vp, _vp],
}
for _name, _args in _SIGS.items():
    _f = getattr(_lib, _name)
    _f.argtypes = _args
    _f.restype = _int
_lib.w2_status_string.argtypes = [_int]
_lib.w2_status_string.restype = ctypes.c_char_p
_lib.w2_last_error.argtypes = []
_lib.w2_last_error.restype = ctypes.c_char_p

EXPORTED = sorted(list(_SIGS) + ["w2_status_string", "w2_last_error"])


class W2Error(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        detail = _lib.w2_last_error().decode()
        super().__init__(f"{fn}: {_lib.w2_status_string(status).decode()} ({status}): {detail}")


def raw():
    """The ctypes library object (tests call entry points with raw pointers)."""
    return _lib


def _check(fn, status):
    if status != OK:
        raise W2Error(fn, status)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t


def packed_size(K, N, G):
    out = _sz(0)
    _check("w2_packed_size", _lib.w2_packed_size(K, N, G, ctypes.byref(out)))
    return out.value


def workspace_size(M, K, N, G, a16=False):
    out = _sz(0)
    _check("w2_workspace_size", _lib.w2_workspace_size(M, K, N, G, int(a16), ctypes.byref(out)))
    return out.value


def prepack(codes, scales, G, codec=CODEC_INT2, bad_codes=None):
    """codes uint8 [K,N], scales bf16 bits (int16/uint16 storage) [K/G,N], both on device.
    Returns the packed blob (uint8 tensor)."""
    _dev(codes, torch.uint8, "codes")
    K, N = codes.shape
    if scales.dtype not in (torch.int16, torch.uint16, torch.bfloat16) or not scales.is_cuda:
        raise ValueError("scales must be a 16-bit device tensor")
    if tuple(scales.shape) != (K // G, N):
        raise ValueError("scales must be [K/G, N]")
    codes, scales = codes.contiguous(), scales.contiguous()
    nbytes = packed_size(K, N, G)
    packed = torch.empty(nbytes, dtype=torch.uint8, device=codes.device)
    _check("w2_prepack", _lib.w2_prepack(_ptr(codes), _ptr(scales), K, N, G, codec, _ptr(packed),
                                         nbytes, _ptr(bad_codes), _stream()))
    return packed


def quantize_rows(X, G=128, want_gsum=False):
    """X fp32 or bf16 [M,K] on device (row stride may exceed K).  Returns (xq, sx, gsum|None)."""
    if X.dtype == torch.float32:
        dt = DT_F32
    elif X.dtype == torch.bfloat16:
        dt = DT_BF16
    else:
        raise ValueError("X must be float32 or bfloat16")
    if not X.is_cuda or X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be a 2-D device tensor with unit inner stride")
    M, K = X.shape
    xq = torch.empty((M, K), dtype=torch.int8, device=X.device)
    sx = torch.empty((M,), dtype=torch.float32, device=X.device)
    gsum = torch.empty((M, K // G), dtype=torch.int32, device=X.device) if want_gsum else None
    ldx = X.stride(0) if M > 1 else K
    _check("w2_quantize_rows", _lib.w2_quantize_rows(_ptr(X), dt, M, K, ldx, G, _ptr(xq), _ptr(sx),
                                                     _ptr(gsum), _stream()))
    return xq, sx, gsum


class Tuning(ctypes.Structure):
    """w2_tuning_t: overrides for tests and sweeps; every field 0 = the library's own rule."""
    _fields_ = [(n, ctypes.c_int) for n in (
        "variant", "dot4_max_m", "midm_min_m", "midm_max_m", "small_waves", "small_cbw", "small_kc", "gemv_window",
        "gemv_max_m", "midm_cbw", "tiled_bm", "tiled_bn", "tiled_kw", "tiled_wd", "tiled_group_m", "splitk", "splitk_min_tiles", "stream_unroll", "stream_blocks",
        "gemv_cbw", "gemv_ks", "fused_rows")]


def _tune(variant=VARIANT_AUTO, tune=None):
    """NULL when nothing is overridden, else a Tuning (kept alive by the caller's frame)."""
    if tune is None and variant == VARIANT_AUTO:
        return None
    t = Tuning()
    if isinstance(tune, Tuning):
        ctypes.memmove(ctypes.byref(t), ctypes.byref(tune), ctypes.sizeof(t))
    elif tune:
        for k, v in tune.items():
            if not hasattr(t, k):
                raise ValueError(f"w2_tuning_t has no field {k}")
            setattr(t, k, int(v))
    if variant != VARIANT_AUTO:
        t.variant = int(variant)
    return t


def _tp(t):
    return None if t is None else ctypes.byref(t)


def _ws(workspace):
    if workspace is None:
        return None, 0
    _dev(workspace, torch.uint8, "workspace")
    return _ptr(workspace), workspace.numel()


def matmul_a8(packed, K, N, G, xq, sx, out=None, variant=VARIANT_AUTO, workspace=None, tune=None):
    """Y bf16 [M,N] = dequant-fused int8 matmul.  xq int8 [M,K], sx fp32 [M].  `workspace`: optional uint8
    device tensor; with workspace_size(M, K, N, G) bytes the tiled kernel may split K across workgroups."""
    _dev(xq, torch.int8, "xq")
    _dev(sx, torch.float32, "sx")
    M = xq.shape[0]
    if tuple(xq.shape) != (M, K) or not xq.is_contiguous() or tuple(sx.shape) != (M,):
        raise ValueError("xq must be contiguous [M,K], sx [M]")
    Y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=xq.device)
    ldy = Y.stride(0) if M > 1 else N
    wp, wb = _ws(workspace)
    t = _tune(variant, tune)
    _check("w2_matmul_a8", _lib.w2_matmul_a8_ex(_ptr(packed), K, N, G, _ptr(xq), _ptr(sx), M,
                                                _ptr(Y), ldy, wp, wb, _tp(t), _stream()))
    return Y


ACT_NONE, ACT_SILU, ACT_SILU_MUL = 0, 1, 2


class _Epilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("act", ctypes.c_int)]


def _epi(bias, act, N):
    if bias is not None:
        if bias.dtype not in (torch.int16, torch.bfloat16) or bias.numel() != N or not bias.is_cuda:
            raise ValueError("bias must be a device tensor of N bf16 values")
    return _Epilogue(bias.data_ptr() if bias is not None else None, int(act))


def matmul_a8_epi(packed, K, N, G, xq, sx, bias=None, act=ACT_NONE, out=None, variant=VARIANT_AUTO, workspace=None,
                  tune=None):
    """matmul_a8 with the fused epilogue: bias (bf16 [N]) and activation; ACT_SILU_MUL gives N/2 columns."""
    _dev(xq, torch.int8, "xq")
    _dev(sx, torch.float32, "sx")
    M = xq.shape[0]
    if tuple(xq.shape) != (M, K) or not xq.is_contiguous() or tuple(sx.shape) != (M,):
        raise ValueError("xq must be contiguous [M,K], sx [M]")
    n_out = N // 2 if act == ACT_SILU_MUL else N
    Y = out if out is not None else torch.empty((M, n_out), dtype=torch.bfloat16, device=xq.device)
    ldy = Y.stride(0) if M > 1 else n_out
    e = _epi(bias, act, N)
    wp, wb = _ws(workspace)
    t = _tune(variant, tune)
    _check("w2_matmul_a8_epi", _lib.w2_matmul_a8_epi(_ptr(packed), K, N, G, _ptr(xq), _ptr(sx), M, _ptr(Y), ldy,
                                                     ctypes.byref(e), wp, wb, _tp(t), _stream()))
    return Y


def matmul_a8_fused_epi(packed, K, N, G, X, bias=None, act=ACT_NONE, out=None, workspace=None, tune=None):
    """matmul_a8_fused with the fused epilogue."""
    if X.dtype == torch.float32:
        dt = DT_F32
    elif X.dtype == torch.bfloat16:
        dt = DT_BF16
    else:
        raise ValueError("X must be float32 or bfloat16")
    if not X.is_cuda or X.dim() != 2 or X.shape[1] != K or X.stride(1) != 1:
        raise ValueError("X must be a device tensor [M,K] with unit inner stride")
    M = X.shape[0]
    n_out = N // 2 if act == ACT_SILU_MUL else N
    Y = out if out is not None else torch.empty((M, n_out), dtype=torch.bfloat16, device=X.device)
    ldx = X.stride(0) if M > 1 else K
    ldy = Y.stride(0) if M > 1 else n_out
    e = _epi(bias, act, N)
    wp, wb = _ws(workspace)
    t = _tune(VARIANT_AUTO, tune)
    _check("w2_matmul_a8_fused_epi", _lib.w2_matmul_a8_fused_epi(_ptr(packed), K, N, G, _ptr(X), dt, ldx, M,
                                                                 _ptr(Y), ldy, ctypes.byref(e), wp, wb, _tp(t),
                                                                 _stream()))
    return Y


def matmul_a16_epi(packed, K, N, G, X, bias=None, act=ACT_NONE, out=None, variant=VARIANT_AUTO, workspace=None,
                   tune=None):
    """matmul_a16 with the fused epilogue."""
    _dev(X, torch.bfloat16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K or X.stride(1) != 1:
        raise ValueError("X must be [M,K] with unit inner stride")
    n_out = N // 2 if act == ACT_SILU_MUL else N
    Y = out if out is not None else torch.empty((M, n_out), dtype=torch.bfloat16, device=X.device)
    ldx = X.stride(0) if M > 1 else K
    ldy = Y.stride(0) if M > 1 else n_out
    e = _epi(bias, act, N)
    wp, wb = _ws(workspace)
    t = _tune(variant, tune)
    _check("w2_matmul_a16_epi", _lib.w2_matmul_a16_epi(_ptr(packed), K, N, G, _ptr(X), ldx, M, _ptr(Y), ldy,
                                                       ctypes.byref(e), wp, wb, _tp(t), _stream()))
    return Y


def matmul_a8_fused(packed, K, N, G, X, out=None, workspace=None):
    """Y bf16 [M,N] from unquantised X (fp32 or bf16); `workspace`: a uint8 device tensor of
    workspace_size(M, K, N, G) bytes, needed for M > 4."""
    if X.dtype == torch.float32:
        dt = DT_F32
    elif X.dtype == torch.bfloat16:
        dt = DT_BF16
    else:
        raise ValueError("X must be float32 or bfloat16")
    if not X.is_cuda or X.dim() != 2 or X.shape[1] != K or X.stride(1) != 1:
        raise ValueError("X must be a device tensor [M,K] with unit inner stride")
    M = X.shape[0]
    Y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    ldx = X.stride(0) if M > 1 else K
    ldy = Y.stride(0) if M > 1 else N
    ws, ws_bytes = (None, 0) if workspace is None else (_ptr(workspace), workspace.numel() * workspace.element_size())
    _check("w2_matmul_a8_fused", _lib.w2_matmul_a8_fused(_ptr(packed), K, N, G, _ptr(X), dt, ldx, M,
                                                         _ptr(Y), ldy, ws, ws_bytes, _stream()))
    return Y


NOALLOC_SCRATCH_BYTES = 24 << 20


def init():
    """Resolves the built-in scratch buffer's address on the current device (optional; see the header)."""
    _check("w2_init", _lib.w2_init())


def matmul_a8_fused_noalloc(packed, K, N, G, X, out):
    """matmul_a8_fused out of the library's built-in scratch buffer: the call allocates nothing, so `out`
    (bf16 [M,N]) is required."""
    if X.dtype == torch.float32:
        dt = DT_F32
    elif X.dtype == torch.bfloat16:
        dt = DT_BF16
    else:
        raise ValueError("X must be float32 or bfloat16")
    if not X.is_cuda or X.dim() != 2 or X.shape[1] != K or X.stride(1) != 1:
        raise ValueError("X must be a device tensor [M,K] with unit inner stride")
    M = X.shape[0]
    _dev(out, torch.bfloat16, "out")
    ldx = X.stride(0) if M > 1 else K
    ldy = out.stride(0) if M > 1 else N
    _check("w2_matmul_a8_fused_noalloc", _lib.w2_matmul_a8_fused_noalloc(_ptr(packed), K, N, G, _ptr(X), dt, ldx, M,
                                                                         _ptr(out), ldy, _stream()))
    return out


def matmul_a16(packed, K, N, G, X, out=None, variant=VARIANT_AUTO, workspace=None, tune=None):
    """Y bf16 [M,N] from bf16 activations X [M,K] (unquantised).  `workspace`: as for matmul_a8
    (workspace_size(..., a16=True) bytes)."""
    _dev(X, torch.bfloat16, "X")
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != K or X.stride(1) != 1:
        raise ValueError("X must be [M,K] with unit inner stride")
    Y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    ldx = X.stride(0) if M > 1 else K
    ldy = Y.stride(0) if M > 1 else N
    wp, wb = _ws(workspace)
    t = _tune(variant, tune)
    _check("w2_matmul_a16", _lib.w2_matmul_a16_ex(_ptr(packed), K, N, G, _ptr(X), ldx, M, _ptr(Y),
                                                  ldy, wp, wb, _tp(t), _stream()))
    return Y


def debug_group_acc_a8(packed, K, N, G, xq, variant=VARIANT_AUTO, tune=None):
    _dev(xq, torch.int8, "xq")
    M = xq.shape[0]
    acc = torch.empty((M, K // G, N), dtype=torch.int32, device=xq.device)
    t = _tune(variant, tune)
    _check("w2_debug_group_acc_a8", _lib.w2_debug_group_acc_a8(_ptr(packed), K, N, G, _ptr(xq), M,
                                                               _tp(t), _ptr(acc), _stream()))
    return acc


def debug_unpack(packed, K, N, G, codec=CODEC_INT2):
    codes = torch.empty((K, N), dtype=torch.uint8, device=packed.device)
    scales = torch.empty((K // G, N), dtype=torch.int16, device=packed.device)
    _check("w2_debug_unpack", _lib.w2_debug_unpack(_ptr(packed), K, N, G, codec, _ptr(codes),
                                                   _ptr(scales), _stream()))
    return codes, scales


def debug_int8_gemv(W8, xq, out=None):
    """Comparator: out int32 [N] = W8 int8 [N,K] @ xq int8 [K], exact."""
    _dev(W8, torch.int8, "W8")
    _dev(xq, torch.int8, "xq")
    N, K = W8.shape
    if not W8.is_contiguous() or xq.numel() != K:
        raise ValueError("W8 must be contiguous [N,K] and xq [K]")
    if out is None:
        out = torch.empty(N, dtype=torch.int32, device=W8.device)
    _check("w2_debug_int8_gemv", _lib.w2_debug_int8_gemv(_ptr(W8), K, N, _ptr(xq), _ptr(out), _stream()))
    return out


def debug_stream_read(buf, sink=None, tune=None):
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    t = _tune(VARIANT_AUTO, tune)
    _check("w2_debug_stream_read", _lib.w2_debug_stream_read(_ptr(buf), buf.numel() * buf.element_size(),
                                                             _ptr(sink), _tp(t), _stream()))
    return sink
