"""ctypes front end of the C oracle (oracle/hikonv_oracle.c).  Test infrastructure only.

Every function takes and returns numpy arrays; the arithmetic is in the C file, which
cites the passages of the paper it follows.
"""
import ctypes as C

import numpy as np

from .build_oracle import build

_lib = C.CDLL(build())

_i8p = np.ctypeslib.ndpointer(dtype=np.int8, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")

_lib.oracle_num_threads.restype = C.c_int
_lib.oracle_set_num_threads.argtypes = [C.c_int]
_lib.oracle_conv1d.argtypes = [_i8p, C.c_int, C.c_int64, C.c_int64, _i8p, C.c_int, C.c_int, C.c_int, _i32p]
_lib.oracle_conv1d.restype = C.c_int
_lib.oracle_conv2d.argtypes = [_i8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _i8p, C.c_int, C.c_int,
                               C.c_int, C.c_int, C.c_int, C.c_int, _i32p]
_lib.oracle_conv2d.restype = C.c_int
_lib.oracle_conv3d.argtypes = [_i8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _i8p, C.c_int, C.c_int,
                               C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _i32p]
_lib.oracle_conv3d.restype = C.c_int
_lib.oracle_relu_requant.argtypes = [_i32p, C.c_int64, C.c_int, C.c_int, _i8p]
_lib.oracle_maxpool2x2.argtypes = [_i8p, C.c_int, C.c_int, C.c_int, C.c_int, _i8p]
_lib.oracle_container_bits.argtypes = [C.c_int]
_lib.oracle_container_bits.restype = C.c_int
_lib.oracle_bitdense_row_bytes.argtypes = [C.c_int64, C.c_int]
_lib.oracle_bitdense_row_bytes.restype = C.c_int64
_lib.oracle_bitdense_pack.argtypes = [_i8p, C.c_int64, C.c_int64, C.c_int, _u8p]

FULL, VALID = 0, 1


def num_threads() -> int:
    return int(_lib.oracle_num_threads())


def set_num_threads(n: int) -> None:
    _lib.oracle_set_num_threads(int(n))


def _bytes(a: np.ndarray):
    """(int8 view, is_unsigned): uint8 arrays are read as 0..255, everything else as int8."""
    a = np.asarray(a)
    if a.dtype == np.uint8:
        return np.ascontiguousarray(a).view(np.int8), 1
    return np.ascontiguousarray(a, dtype=np.int8), 0


def conv1d(f: np.ndarray, g: np.ndarray, mode: int = FULL) -> np.ndarray:
    """y[r][m] = sum_k h_r[m-k] g[k]; f is [rows][len], g is [K] (shared); int8 or uint8."""
    if np.asarray(f).ndim == 1:
        return conv1d(np.asarray(f)[None, :], g, mode)[0]
    f, fu = _bytes(f)
    g, gu = _bytes(g)
    rows, length = f.shape
    K = g.shape[0]
    out_len = length + K - 1 if mode == FULL else max(length - K + 1, 0)
    y = np.zeros((rows, out_len), dtype=np.int32)
    rc = _lib.oracle_conv1d(f, fu, rows, length, g, gu, K, mode, y)
    if rc != 0:
        raise OverflowError("1-D convolution result does not fit int32")
    return y


def conv2d(x: np.ndarray, w: np.ndarray, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Cross-correlation layer on NCHW x and [Co][C][Kh][Kw] w (int8 or uint8), int32 NCHW out."""
    x, xu = _bytes(x)
    w, wu = _bytes(w)
    n, c, h, wd = x.shape
    co, c2, kh, kw = w.shape
    assert c == c2
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    y = np.zeros((n, co, max(ho, 0), max(wo, 0)), dtype=np.int32)
    rc = _lib.oracle_conv2d(x, xu, n, c, h, wd, w, wu, co, kh, kw, stride, pad, y)
    if rc != 0:
        raise OverflowError("2-D convolution result does not fit int32")
    return y


def conv3d(x: np.ndarray, w: np.ndarray, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Cross-correlation layer on NCDHW x and [Co][C][Kd][Kh][Kw] w (int8 or uint8), int32 NCDHW out."""
    x, xu = _bytes(x)
    w, wu = _bytes(w)
    n, c, d, h, wd = x.shape
    co, c2, kd, kh, kw = w.shape
    assert c == c2
    do = (d + 2 * pad - kd) // stride + 1
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    y = np.zeros((n, co, max(do, 0), max(ho, 0), max(wo, 0)), dtype=np.int32)
    rc = _lib.oracle_conv3d(x, xu, n, c, d, h, wd, w, wu, co, kd, kh, kw, stride, pad, y)
    if rc != 0:
        raise OverflowError("3-D convolution result does not fit int32")
    return y


def relu_requant(acc: np.ndarray, shift: int, qmax: int) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    q = np.zeros(acc.shape, dtype=np.int8)
    _lib.oracle_relu_requant(acc, acc.size, shift, qmax, q)
    return q


def maxpool2x2(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int8)
    n, c, h, w = x.shape
    y = np.zeros((n, c, h // 2, w // 2), dtype=np.int8)
    _lib.oracle_maxpool2x2(x, n, c, h, w, y)
    return y


def container_bits(bits: int) -> int:
    return int(_lib.oracle_container_bits(bits))


def bitdense_row_bytes(length: int, bits: int) -> int:
    return int(_lib.oracle_bitdense_row_bytes(length, bits))


def bitdense_pack(v: np.ndarray, bits: int) -> np.ndarray:
    """[rows][len] int8 -> [rows][row_bytes] uint8 bit-dense container stream."""
    v, _ = _bytes(v)
    rows, length = v.shape
    out = np.zeros((rows, bitdense_row_bytes(length, bits)), dtype=np.uint8)
    _lib.oracle_bitdense_pack(v, rows, length, bits, out)
    return out
