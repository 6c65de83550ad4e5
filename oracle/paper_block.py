"""ctypes access to the oracle of the paper's self-contained block (oracle/ecco_paper_block.cpp).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes as C

import numpy as np

from .oracle import lib

GROUP, CENTROIDS, SYMBOLS, BOOKS, BLOCK_BYTES = 128, 15, 16, 4, 64


class _Model(C.Structure):
    _fields_ = [("S", C.c_int), ("texp", C.c_int), ("cent", C.c_void_p), ("lens", C.c_void_p), ("kp_lens", C.c_void_p)]


class Model:
    """cent [S,15] fp16 bits, lens [S,4,16], kp_lens [S], texp."""

    def __init__(self, cent, lens, kp_lens, texp):
        self.cent = np.ascontiguousarray(cent, dtype=np.uint16).reshape(-1, CENTROIDS)
        self.S = self.cent.shape[0]
        self.lens = np.ascontiguousarray(lens, dtype=np.uint8).reshape(self.S, BOOKS, SYMBOLS)
        self.kp_lens = np.ascontiguousarray(kp_lens, dtype=np.uint8).reshape(self.S)
        self.texp = int(texp)
        self.c = _Model(self.S, self.texp, self.cent.ctypes.data, self.lens.ctypes.data, self.kp_lens.ctypes.data)


def fp8_value(b: int) -> float:
    L = lib()
    L.pb_fp8_value.restype = C.c_double
    L.pb_fp8_value.argtypes = [C.c_uint8]
    return float(L.pb_fp8_value(b))


def fp8_round(v: float) -> int:
    L = lib()
    L.pb_fp8_round.restype = C.c_uint8
    L.pb_fp8_round.argtypes = [C.c_double]
    return int(L.pb_fp8_round(v))


def verify_model(m: Model) -> int:
    return int(lib().pb_verify_model(C.byref(m.c)))


def quantize_group(m: Model, x_u16):
    x = np.ascontiguousarray(x_u16, dtype=np.uint16).reshape(-1)
    assert x.size == GROUP
    a, p, h, s8 = C.c_int(0), C.c_int(0), C.c_int(0), C.c_uint8(0)
    idx = np.zeros(GROUP, np.uint8)
    lib().pb_quantize_group(C.byref(m.c), x.ctypes.data_as(C.c_void_p), C.byref(a), C.byref(s8), C.byref(p), C.byref(h),
                            idx.ctypes.data_as(C.c_void_p))
    return int(a.value), int(s8.value), int(p.value), int(h.value), idx


def encode(m: Model, src_u16):
    src = np.ascontiguousarray(src_u16, dtype=np.uint16).reshape(-1)
    assert src.size % GROUP == 0
    n = src.size // GROUP
    blocks = np.zeros((n, BLOCK_BYTES), np.uint8)
    lib().pb_encode(C.byref(m.c), src.ctypes.data_as(C.c_void_p), C.c_size_t(n), blocks.ctypes.data_as(C.c_void_p))
    return blocks


def decode(m: Model, blocks):
    blocks = np.ascontiguousarray(blocks, dtype=np.uint8).reshape(-1, BLOCK_BYTES)
    n = blocks.shape[0]
    dst = np.zeros((n, GROUP), np.uint16)
    n_coded = np.zeros(n, np.uint8)
    n_out = np.zeros(n, np.uint8)
    lib().pb_decode(C.byref(m.c), blocks.ctypes.data_as(C.c_void_p), C.c_size_t(n), dst.ctypes.data_as(C.c_void_p),
                    n_coded.ctypes.data_as(C.c_void_p), n_out.ctypes.data_as(C.c_void_p))
    return dst, n_coded, n_out


def gemv(m: Model, blocks, rows: int, cols: int, x_u16):
    blocks = np.ascontiguousarray(blocks, dtype=np.uint8).reshape(-1, BLOCK_BYTES)
    x = np.ascontiguousarray(x_u16, dtype=np.uint16).reshape(-1)
    assert cols % GROUP == 0 and x.size == cols and blocks.shape[0] == rows * (cols // GROUP)
    y = np.zeros(rows, np.float64)
    lib().pb_gemv(C.byref(m.c), blocks.ctypes.data_as(C.c_void_p), C.c_int(rows), C.c_int(cols), x.ctypes.data_as(C.c_void_p),
                  y.ctypes.data_as(C.c_void_p))
    return y
