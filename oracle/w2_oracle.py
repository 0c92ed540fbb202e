"""ctypes marshalling for ``w2_oracle.c``.  No arithmetic lives here."""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "w2_oracle.c")
_LIB = os.path.join(_HERE, "libw2oracle.so")

CODEC_INT2 = 0      # q = c - 2
CODEC_TERNARY = 1   # q = c - 1, code 3 illegal
ERR_BAD_CODE = -6


class OracleError(RuntimeError):
    def __init__(self, fn, rc):
        super().__init__(f"{fn} returned {rc}")
        self.rc = rc


def build(force=False):
    """Compile the oracle with gcc (plain C, no intrinsics)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-Wall", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.w2o_bf16_to_f32.restype = ctypes.c_float
        _lib.w2o_bf16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.w2o_f64_to_bf16.restype = ctypes.c_uint16
        _lib.w2o_f64_to_bf16.argtypes = [ctypes.c_double]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _i64(v):
    return ctypes.c_int64(int(v))


def _chk(fn, rc):
    if rc != 0:
        raise OracleError(fn, rc)


def bf16_to_f32(bits):
    """bf16 bit patterns (uint16 array) -> float32 array, exact."""
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    f = lib().w2o_bf16_to_f32
    flat_in, flat_out = bits.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = f(int(flat_in[i]))
    return out


def f64_to_bf16(v):
    """fp64 array -> bf16 bit patterns (uint16), one RNE rounding."""
    v = _c(v, np.float64)
    out = np.empty(v.shape, np.uint16)
    lib().w2o_f64_to_bf16_array(_p(v), _i64(v.size), _p(out))
    return out


def check_codes(codes, codec):
    codes = _c(codes, np.uint8)
    K, N = codes.shape
    return lib().w2o_check_codes(_p(codes), _i64(K), _i64(N), int(codec))


def quantize_rows(X, G, x_is_bf16=False, want_gsum=True):
    """Per-token int8 quantisation.  X: float32 [M,K], or bf16 bits uint16 [M,K]."""
    X = _c(X, np.uint16 if x_is_bf16 else np.float32)
    M, K = X.shape
    xq = np.empty((M, K), np.int8)
    sx = np.empty((M,), np.float32)
    gs = np.empty((M, K // G), np.int32) if want_gsum else None
    _chk("w2o_quantize_rows",
         lib().w2o_quantize_rows(_p(X), int(bool(x_is_bf16)), _i64(M), _i64(K), _i64(K),
                                 int(G), _p(xq), _p(sx), _p(gs)))
    return xq, sx, gs


def group_acc(codes, G, codec, xq):
    codes = _c(codes, np.uint8)
    xq = _c(xq, np.int8)
    K, N = codes.shape
    M = xq.shape[0]
    assert xq.shape == (M, K)
    acc = np.empty((M, K // G, N), np.int32)
    _chk("w2o_group_acc",
         lib().w2o_group_acc(_p(codes), _i64(K), _i64(N), int(G), int(codec), _p(xq), _i64(M),
                             _p(acc)))
    return acc


def matmul_a8(codes, scales, G, codec, xq, sx):
    """Returns (Y bf16 bits [M,N], y64 unrounded [M,N])."""
    codes = _c(codes, np.uint8)
    scales = _c(scales, np.uint16)
    xq = _c(xq, np.int8)
    sx = _c(sx, np.float32)
    K, N = codes.shape
    M = xq.shape[0]
    assert scales.shape == (K // G, N) and xq.shape == (M, K) and sx.shape == (M,)
    Y = np.empty((M, N), np.uint16)
    y64 = np.empty((M, N), np.float64)
    _chk("w2o_matmul_a8",
         lib().w2o_matmul_a8(_p(codes), _p(scales), _i64(K), _i64(N), int(G), int(codec),
                             _p(xq), _p(sx), _i64(M), _p(Y), _p(y64)))
    return Y, y64


def a8_term_magnitude(codes, scales, G, codec, xq, sx):
    codes = _c(codes, np.uint8)
    scales = _c(scales, np.uint16)
    xq = _c(xq, np.int8)
    sx = _c(sx, np.float32)
    K, N = codes.shape
    M = xq.shape[0]
    mag = np.empty((M, N), np.float64)
    _chk("w2o_a8_term_magnitude",
         lib().w2o_a8_term_magnitude(_p(codes), _p(scales), _i64(K), _i64(N), int(G),
                                     int(codec), _p(xq), _p(sx), _i64(M), _p(mag)))
    return mag


def matmul_a16(codes, scales, G, codec, X_bf16):
    """Returns (Y bf16 bits, y64 unrounded, sum_k |x*w|)."""
    codes = _c(codes, np.uint8)
    scales = _c(scales, np.uint16)
    X = _c(X_bf16, np.uint16)
    K, N = codes.shape
    M = X.shape[0]
    assert X.shape == (M, K) and scales.shape == (K // G, N)
    Y = np.empty((M, N), np.uint16)
    y64 = np.empty((M, N), np.float64)
    mag = np.empty((M, N), np.float64)
    _chk("w2o_matmul_a16",
         lib().w2o_matmul_a16(_p(codes), _p(scales), _i64(K), _i64(N), int(G), int(codec),
                              _p(X), _i64(K), _i64(M), _p(Y), _p(y64), _p(mag)))
    return Y, y64, mag


def epilogue(y64, bias=None, act=0):
    """Fused epilogue on the unrounded result.  Returns (Y bf16 bits, out64), [M, N or N/2]."""
    y64 = _c(y64, np.float64)
    M, N = y64.shape
    bias = None if bias is None else _c(bias, np.uint16)
    n_out = N // 2 if act == 2 else N
    Y = np.empty((M, n_out), np.uint16)
    out64 = np.empty((M, n_out), np.float64)
    _chk("w2o_epilogue", lib().w2o_epilogue(_p(y64), _i64(M), _i64(N), _p(bias), int(act), _p(Y), _p(out64)))
    return Y, out64


def bruteforce_a8(codes, scales, G, codec, xq, sx):
    codes = _c(codes, np.uint8)
    scales = _c(scales, np.uint16)
    xq = _c(xq, np.int8)
    sx = _c(sx, np.float32)
    K, N = codes.shape
    M = xq.shape[0]
    y64 = np.empty((M, N), np.float64)
    _chk("w2o_bruteforce_a8",
         lib().w2o_bruteforce_a8(_p(codes), _p(scales), _i64(K), _i64(N), int(G), int(codec),
                                 _p(xq), _p(sx), _i64(M), _p(y64)))
    return y64


def num_threads():
    return int(lib().w2o_num_threads())
