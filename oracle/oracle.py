"""ctypes access to the CPU oracle (oracle/ecco_oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Argument marshalling and nothing else: every function below forwards numpy arrays to the C++
routine of the same name.  Imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

GROUP, K, BLOCK_BYTES, MAX_LEN = 128, 16, 64, 12

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.oracle_h2f.restype = C.c_float
        _lib.oracle_h2f.argtypes = [C.c_uint16]
        _lib.oracle_f2h.restype = C.c_uint16
        _lib.oracle_f2h.argtypes = [C.c_float]
        _lib.oracle_dequant.restype = C.c_uint16
        _lib.oracle_dequant.argtypes = [C.c_uint16, C.c_uint16]
        _lib.oracle_map_values.argtypes = [C.c_void_p, C.c_int, C.c_uint16, C.c_void_p, C.c_void_p]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def set_threads(n: int) -> int:
    return lib().oracle_set_threads(C.c_int(n))


def h2f(h: int) -> float:
    return float(lib().oracle_h2f(h))


def f2h(f: float) -> int:
    return int(lib().oracle_f2h(C.c_float(f)))


def dequant(c: int, s: int) -> int:
    return int(lib().oracle_dequant(c, s))


def huffman_lengths(counts) -> np.ndarray:
    counts = _c(counts, np.uint64)
    lens = np.zeros(len(counts), np.uint8)
    rc = lib().oracle_huffman_lengths(_p(counts), C.c_int(len(counts)), _p(lens))
    assert rc == 0, rc
    return lens


def limited_lengths(counts, max_len: int) -> np.ndarray:
    counts = _c(counts, np.uint64)
    lens = np.zeros(len(counts), np.uint8)
    rc = lib().oracle_limited_lengths(_p(counts), C.c_int(len(counts)), C.c_int(max_len), _p(lens))
    if rc != 0:
        raise ValueError(f"oracle_limited_lengths rc={rc}")
    return lens


def canonical_codes(lens) -> np.ndarray:
    lens = _c(lens, np.uint8)
    codes = np.zeros(len(lens), np.uint16)
    lib().oracle_canonical_codes(_p(lens), C.c_int(len(lens)), _p(codes))
    return codes


def verify_model(centroids, lens) -> int:
    centroids = _c(centroids, np.uint16)
    lens = _c(lens, np.uint8)
    S = centroids.size // K
    return int(lib().oracle_verify_model(_p(centroids), _p(lens), C.c_int(S)))


def kmeans_1d(v, Kc: int, max_iter: int = 25):
    v = _c(v, np.float32)
    cent = np.zeros(Kc, np.float64)
    obj = np.zeros(max_iter + 2, np.float64)
    it = lib().oracle_kmeans_1d(_p(v), C.c_int(v.size), C.c_int(Kc), C.c_int(max_iter), _p(cent), _p(obj))
    return cent, obj[: it + 1], it


def fit(data_u16, S: int, max_len: int = MAX_LEN, seed: int = 0):
    data = _c(data_u16, np.uint16).reshape(-1)
    cent = np.zeros((S, K), np.uint16)
    lens = np.zeros((S, K), np.uint8)
    hist = np.zeros((S, K), np.uint64)
    nfit = C.c_size_t(0)
    rc = lib().oracle_fit(_p(data), C.c_size_t(data.size), C.c_int(S), C.c_int(max_len), C.c_uint64(seed),
                          _p(cent), _p(lens), _p(hist), C.byref(nfit))
    if rc != 0:
        raise ValueError(f"oracle_fit rc={rc}")
    return cent, lens, hist, int(nfit.value)


def fit_trace(data_u16, S: int, max_len: int = MAX_LEN, seed: int = 0):
    """oracle_fit_trace: the fit plus the picked group indices, the per-group patterns and the step-4 objective."""
    data = _c(data_u16, np.uint16).reshape(-1)
    n_all = data.size // GROUP
    n_cap = min(n_all, 65536)
    cent = np.zeros((S, K), np.uint16)
    lens = np.zeros((S, K), np.uint8)
    hist = np.zeros((S, K), np.uint64)
    pick = np.zeros(n_cap, np.uint64)
    pats = np.zeros((n_cap, K), np.float64)
    obj = np.zeros(50, np.float64)
    nfit, nobj = C.c_size_t(0), C.c_int(0)
    rc = lib().oracle_fit_trace(_p(data), C.c_size_t(data.size), C.c_int(S), C.c_int(max_len), C.c_uint64(seed),
                                _p(cent), _p(lens), _p(hist), C.byref(nfit), _p(pick), _p(pats), _p(obj), C.byref(nobj))
    if rc != 0:
        raise ValueError(f"oracle_fit_trace rc={rc}")
    n = int(nfit.value)
    return dict(cent=cent, lens=lens, hist=hist, n_fit=n, pick=pick[:n].astype(np.int64), patterns=pats[:n],
                objective=obj[: int(nobj.value)].copy())


def quantize_group(centroids, x_u16):
    centroids = _c(centroids, np.uint16)
    S = centroids.size // K
    x = _c(x_u16, np.uint16).reshape(-1)
    assert x.size == GROUP
    scale = C.c_uint16(0)
    pat = C.c_int(0)
    idx = np.zeros(GROUP, np.uint8)
    sse = np.zeros(S, np.float32)
    lib().oracle_quantize_group(_p(centroids), C.c_int(S), _p(x), C.byref(scale), C.byref(pat), _p(idx), _p(sse))
    return int(scale.value), int(pat.value), idx, sse


def encode(centroids, lens, src_u16):
    centroids = _c(centroids, np.uint16)
    lens = _c(lens, np.uint8)
    S = centroids.size // K
    src = _c(src_u16, np.uint16).reshape(-1)
    assert src.size % GROUP == 0
    n = src.size // GROUP
    blocks = np.zeros((n, BLOCK_BYTES), np.uint8)
    meta = np.zeros(n, np.uint32)
    lib().oracle_encode(_p(centroids), _p(lens), C.c_int(S), _p(src), C.c_size_t(n), _p(blocks), _p(meta))
    return blocks, meta


def select_minmax(centroids, x_u16):
    centroids = _c(centroids, np.uint16)
    S = centroids.size // K
    x = _c(x_u16, np.uint16).reshape(-1)
    assert x.size == GROUP
    scale = C.c_uint16(0)
    pat = C.c_int(0)
    fit_ = np.zeros(S, np.float32)
    lib().oracle_select_minmax(_p(centroids), C.c_int(S), _p(x), C.byref(scale), C.byref(pat), _p(fit_))
    return int(scale.value), int(pat.value), fit_


def map_values(centroids, p: int, scale: int, x_u16):
    centroids = _c(centroids, np.uint16)
    x = _c(x_u16, np.uint16).reshape(-1)
    assert x.size == GROUP and 0 <= p < centroids.size // K
    idx = np.zeros(GROUP, np.uint8)
    lib().oracle_map_values(_p(centroids), C.c_int(p), C.c_uint16(scale), _p(x), _p(idx))
    return idx


def encode_minmax(centroids, lens, src_u16):
    centroids = _c(centroids, np.uint16)
    lens = _c(lens, np.uint8)
    S = centroids.size // K
    src = _c(src_u16, np.uint16).reshape(-1)
    assert src.size % GROUP == 0
    n = src.size // GROUP
    blocks = np.zeros((n, BLOCK_BYTES), np.uint8)
    meta = np.zeros(n, np.uint32)
    lib().oracle_encode_minmax(_p(centroids), _p(lens), C.c_int(S), _p(src), C.c_size_t(n), _p(blocks), _p(meta))
    return blocks, meta


def decode_indices(lens, S: int, blocks, meta):
    lens = _c(lens, np.uint8)
    blocks = _c(blocks, np.uint8).reshape(-1, BLOCK_BYTES)
    meta = _c(meta, np.uint32).reshape(-1)
    n = meta.size
    assert blocks.shape[0] == n
    idx = np.zeros((n, GROUP), np.uint8)
    used = np.zeros(n, np.uint16)
    lib().oracle_decode_indices(_p(lens), C.c_int(S), _p(blocks), _p(meta), C.c_size_t(n), _p(idx), _p(used))
    return idx, used


def decode(centroids, lens, blocks, meta):
    centroids = _c(centroids, np.uint16)
    lens = _c(lens, np.uint8)
    S = centroids.size // K
    blocks = _c(blocks, np.uint8).reshape(-1, BLOCK_BYTES)
    meta = _c(meta, np.uint32).reshape(-1)
    n = meta.size
    assert blocks.shape[0] == n
    dst = np.zeros((n, GROUP), np.uint16)
    lib().oracle_decode(_p(centroids), _p(lens), C.c_int(S), _p(blocks), _p(meta), C.c_size_t(n), _p(dst))
    return dst


def gemv(centroids, lens, blocks, meta, rows: int, cols: int, x_u16):
    centroids = _c(centroids, np.uint16)
    lens = _c(lens, np.uint8)
    S = centroids.size // K
    blocks = _c(blocks, np.uint8).reshape(-1, BLOCK_BYTES)
    meta = _c(meta, np.uint32).reshape(-1)
    x = _c(x_u16, np.uint16).reshape(-1, cols)
    batch = x.shape[0]
    assert cols % GROUP == 0 and meta.size == rows * (cols // GROUP) == blocks.shape[0]
    y = np.zeros((batch, rows), np.float64)
    lib().oracle_gemv(_p(centroids), _p(lens), C.c_int(S), _p(blocks), _p(meta), C.c_int(rows), C.c_int(cols),
                      _p(x), C.c_int(batch), _p(y))
    return y


def kv_append(ck, lk, cv, lv, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max, minmax=False):
    """In place on the numpy caches (k_blocks [B,H,T_max,64] u8, k_meta [B,H,T_max] u32, ...)."""
    ck, cv = _c(ck, np.uint16), _c(cv, np.uint16)
    lk, lv = _c(lk, np.uint8), _c(lv, np.uint8)
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    seq_len = _c(seq_len, np.int32)
    for a in (k_blocks, k_meta, v_blocks, v_meta):
        assert a.flags["C_CONTIGUOUS"]
    fn = lib().oracle_kv_append_minmax if minmax else lib().oracle_kv_append
    fn(_p(ck), _p(lk), C.c_int(ck.size // K), _p(cv), _p(lv), C.c_int(cv.size // K),
                           _p(k_new), _p(v_new), _p(k_blocks), _p(k_meta), _p(v_blocks), _p(v_meta),
                           _p(seq_len), C.c_int(B), C.c_int(H), C.c_int(T_max))


def kv_attend(ck, lk, cv, lv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max):
    ck, cv = _c(ck, np.uint16), _c(cv, np.uint16)
    lk, lv = _c(lk, np.uint8), _c(lv, np.uint8)
    q = _c(q, np.uint16)
    seq_len = _c(seq_len, np.int32)
    k_blocks, v_blocks = _c(k_blocks, np.uint8), _c(v_blocks, np.uint8)
    k_meta, v_meta = _c(k_meta, np.uint32), _c(v_meta, np.uint32)
    out = np.zeros((B, H, GROUP), np.float64)
    lib().oracle_kv_attend(_p(ck), _p(lk), C.c_int(ck.size // K), _p(cv), _p(lv), C.c_int(cv.size // K),
                           _p(q), _p(k_blocks), _p(k_meta), _p(v_blocks), _p(v_meta), _p(seq_len),
                           C.c_int(B), C.c_int(H), C.c_int(T_max), _p(out))
    return out


def kv_attend_gqa(ck, lk, cv, lv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max):
    assert Hq % Hkv == 0
    ck, cv = _c(ck, np.uint16), _c(cv, np.uint16)
    lk, lv = _c(lk, np.uint8), _c(lv, np.uint8)
    q = _c(q, np.uint16)
    seq_len = _c(seq_len, np.int32)
    k_blocks, v_blocks = _c(k_blocks, np.uint8), _c(v_blocks, np.uint8)
    k_meta, v_meta = _c(k_meta, np.uint32), _c(v_meta, np.uint32)
    assert q.size == B * Hq * GROUP and k_meta.size == B * Hkv * T_max == v_meta.size
    out = np.zeros((B, Hq, GROUP), np.float64)
    lib().oracle_kv_attend_gqa(_p(ck), _p(lk), C.c_int(ck.size // K), _p(cv), _p(lv), C.c_int(cv.size // K),
                               _p(q), _p(k_blocks), _p(k_meta), _p(v_blocks), _p(v_meta), _p(seq_len),
                               C.c_int(B), C.c_int(Hq), C.c_int(Hkv), C.c_int(T_max), _p(out))
    return out


ACT_GROUP = 64


def act_dequant(q: int, s_bits: int, z_bits: int) -> int:
    L = lib()
    L.oracle_act_dequant.restype = C.c_uint16
    L.oracle_act_dequant.argtypes = [C.c_int, C.c_uint16, C.c_uint16]
    return int(L.oracle_act_dequant(q, s_bits, z_bits))


def act_params(x_u16):
    x = _c(x_u16, np.uint16).reshape(-1)
    assert x.size == ACT_GROUP
    s, z = C.c_uint16(0), C.c_uint16(0)
    lib().oracle_act_params(_p(x), C.byref(s), C.byref(z))
    return int(s.value), int(z.value)


def act_encode(src_u16):
    src = _c(src_u16, np.uint16).reshape(-1)
    assert src.size % ACT_GROUP == 0
    n = src.size // ACT_GROUP
    blocks = np.zeros((n, BLOCK_BYTES), np.uint8)
    lib().oracle_act_encode(_p(src), C.c_size_t(n), _p(blocks))
    return blocks


def act_decode(blocks):
    blocks = _c(blocks, np.uint8).reshape(-1, BLOCK_BYTES)
    n = blocks.shape[0]
    dst = np.zeros((n, ACT_GROUP), np.uint16)
    lib().oracle_act_decode(_p(blocks), C.c_size_t(n), _p(dst))
    return dst
