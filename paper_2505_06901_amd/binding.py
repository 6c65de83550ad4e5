"""Thin ctypes binding of libecco's C ABI (include/ecco.h): argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing else);
every step of the path runs in the library's HIP kernels.  There is no CPU fallback: if the
library is not built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

GROUP, BLOCK_BYTES, K, MAX_LEN, MAX_S = 128, 64, 16, 12, 64
_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libecco.so")
_lib = None

EXPORTS = [
    "ecco_strerror", "ecco_fit_patterns", "ecco_model_create", "ecco_model_save", "ecco_model_load",
    "ecco_model_S", "ecco_model_centroids", "ecco_model_code_lens", "ecco_model_to_device", "ecco_model_free",
    "ecco_encode", "ecco_decode", "ecco_decode_indices", "ecco_decode_gemv", "ecco_kv_append", "ecco_kv_attend",
    "ecco_encode_minmax", "ecco_kv_append_minmax", "ecco_act_encode", "ecco_act_decode",
    "ecco_kv_attend_gqa", "ecco_kv_attend_gqa_workspace", "ecco_kv_attend_gqa_splits", "ecco_kv_attend_gqa_noalloc", "ecco_read_stream", "ecco_device_info",
    "ecco_pb_fit", "ecco_pb_model_create", "ecco_pb_model_S", "ecco_pb_model_texp", "ecco_pb_model_centroids",
    "ecco_pb_model_code_lens", "ecco_pb_model_kp_lens", "ecco_pb_model_to_device", "ecco_pb_model_free",
    "ecco_pb_encode", "ecco_pb_decode", "ecco_pb_decode_gemv", "ecco_pb_model_save", "ecco_pb_model_load",
]


class EccoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_06901_amd.build`")
        L = C.CDLL(_LIB_PATH)
        L.ecco_strerror.restype = C.c_char_p
        L.ecco_strerror.argtypes = [C.c_int]
        L.ecco_model_centroids.restype = C.POINTER(C.c_uint16)
        L.ecco_model_code_lens.restype = C.POINTER(C.c_uint8)
        for name in ("ecco_model_S", "ecco_model_centroids", "ecco_model_code_lens", "ecco_model_free"):
            getattr(L, name).argtypes = [C.c_void_p]
        L.ecco_model_free.restype = None
        vp, sz, i32, u64 = C.c_void_p, C.c_size_t, C.c_int, C.c_uint64
        L.ecco_fit_patterns.argtypes = [vp, sz, i32, i32, u64, C.POINTER(vp)]
        L.ecco_model_create.argtypes = [vp, vp, i32, C.POINTER(vp)]
        L.ecco_model_save.argtypes = [vp, vp, sz, C.POINTER(sz)]
        L.ecco_model_load.argtypes = [vp, sz, C.POINTER(vp)]
        L.ecco_model_to_device.argtypes = [vp, i32]
        L.ecco_encode.argtypes = [vp, vp, sz, vp, vp, vp]
        L.ecco_encode_minmax.argtypes = [vp, vp, sz, vp, vp, vp]
        L.ecco_decode.argtypes = [vp, vp, vp, sz, vp, vp]
        L.ecco_decode_indices.argtypes = [vp, vp, vp, sz, vp, vp]
        L.ecco_decode_gemv.argtypes = [vp, vp, vp, i32, i32, vp, i32, vp, vp]
        L.ecco_kv_append.argtypes = [vp] * 9 + [i32, i32, i32, vp]
        L.ecco_kv_append_minmax.argtypes = [vp] * 9 + [i32, i32, i32, vp]
        L.ecco_kv_attend.argtypes = [vp] * 8 + [i32, i32, i32, vp, vp]
        L.ecco_act_encode.argtypes = [vp, sz, vp, vp]
        L.ecco_read_stream.argtypes = [vp, sz, vp, vp]
        L.ecco_kv_attend_gqa.argtypes = [vp] * 8 + [i32, i32, i32, i32, i32, vp, vp, vp]
        L.ecco_kv_attend_gqa_noalloc.argtypes = [vp] * 8 + [i32, i32, i32, i32, i32, vp, vp]
        L.ecco_kv_attend_gqa_workspace.argtypes = [i32, i32, i32]
        L.ecco_kv_attend_gqa_workspace.restype = sz
        L.ecco_kv_attend_gqa_splits.argtypes = [i32, i32, i32, i32]
        L.ecco_kv_attend_gqa_splits.restype = i32
        L.ecco_device_info.argtypes = [i32, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.ecco_device_info.restype = i32
        L.ecco_pb_fit.argtypes = [vp, sz, i32, u64, C.POINTER(vp)]
        L.ecco_pb_model_create.argtypes = [vp, vp, vp, i32, i32, C.POINTER(vp)]
        for name in ("ecco_pb_model_S", "ecco_pb_model_texp", "ecco_pb_model_centroids", "ecco_pb_model_code_lens",
                     "ecco_pb_model_kp_lens", "ecco_pb_model_free"):
            getattr(L, name).argtypes = [vp]
        L.ecco_pb_model_centroids.restype = C.POINTER(C.c_uint16)
        L.ecco_pb_model_code_lens.restype = C.POINTER(C.c_uint8)
        L.ecco_pb_model_kp_lens.restype = C.POINTER(C.c_uint8)
        L.ecco_pb_model_free.restype = None
        L.ecco_pb_model_to_device.argtypes = [vp, i32]
        L.ecco_pb_model_save.argtypes = [vp, vp, sz, C.POINTER(sz)]
        L.ecco_pb_model_load.argtypes = [vp, sz, C.POINTER(vp)]
        L.ecco_pb_encode.argtypes = [vp, vp, sz, vp, vp]
        L.ecco_pb_decode.argtypes = [vp, vp, sz, vp, vp]
        L.ecco_pb_decode_gemv.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.ecco_act_decode.argtypes = [vp, sz, vp, vp]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().ecco_strerror(status).decode()


def _check(status: int, where: str):
    if status != 0:
        raise EccoError(status, where)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dp(t):
    """Device pointer of a contiguous torch tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


class Model:
    """Owner of an ecco_model handle."""

    def __init__(self, handle):
        self._h = C.c_void_p(handle)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.ecco_model_free(h)

    @property
    def handle(self):
        return self._h

    @property
    def S(self) -> int:
        return int(lib().ecco_model_S(self._h))

    @property
    def centroids(self) -> np.ndarray:
        """[S,16] uint16 (FP16 bit patterns), a copy."""
        return np.ctypeslib.as_array(lib().ecco_model_centroids(self._h), shape=(self.S, K)).copy()

    @property
    def code_lens(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().ecco_model_code_lens(self._h), shape=(self.S, K)).copy()


def ecco_fit_patterns(data, S: int, max_code_len: int = MAX_LEN, seed: int = 0) -> Model:
    """data: numpy array of FP16 (or their uint16 bit patterns), size % 128 == 0, on the host."""
    a = np.ascontiguousarray(data)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("FP16 data expected")
    out = C.c_void_p(0)
    _check(lib().ecco_fit_patterns(a.ctypes.data_as(C.c_void_p), a.size, S, max_code_len, seed, C.byref(out)),
           "ecco_fit_patterns")
    return Model(out.value)


def ecco_model_create(centroids, code_lens) -> Model:
    c = np.ascontiguousarray(centroids)
    if c.dtype == np.float16:
        c = c.view(np.uint16)
    c = np.ascontiguousarray(c, dtype=np.uint16)
    l = np.ascontiguousarray(code_lens, dtype=np.uint8)
    out = C.c_void_p(0)
    _check(lib().ecco_model_create(c.ctypes.data_as(C.c_void_p), l.ctypes.data_as(C.c_void_p), c.size // K, C.byref(out)),
           "ecco_model_create")
    return Model(out.value)


def ecco_model_save(m: Model) -> bytes:
    n = C.c_size_t(0)
    _check(lib().ecco_model_save(m.handle, None, 0, C.byref(n)), "ecco_model_save")
    buf = C.create_string_buffer(n.value)
    _check(lib().ecco_model_save(m.handle, buf, n.value, C.byref(n)), "ecco_model_save")
    return buf.raw[: n.value]


def ecco_model_load(blob: bytes) -> Model:
    out = C.c_void_p(0)
    _check(lib().ecco_model_load(blob, len(blob), C.byref(out)), "ecco_model_load")
    return Model(out.value)


def ecco_model_to_device(m: Model, device: int = 0) -> Model:
    _check(lib().ecco_model_to_device(m.handle, device), "ecco_model_to_device")
    return m


def _encode(name: str, m: Model, src, blocks, meta):
    import torch
    n = src.numel() // GROUP
    assert src.numel() % GROUP == 0 and src.dtype == torch.float16
    if blocks is None:
        blocks = torch.empty((n, BLOCK_BYTES), dtype=torch.uint8, device=src.device)
    if meta is None:
        meta = torch.empty((n,), dtype=torch.int32, device=src.device)
    _check(getattr(lib(), name)(m.handle, _dp(src), n, _dp(blocks), _dp(meta), _stream()), name)
    return blocks, meta


def ecco_encode(m: Model, src, blocks=None, meta=None):
    """src: CUDA FP16 tensor with numel % 128 == 0.  Returns (blocks uint8 [n,64], meta int32 [n])."""
    return _encode("ecco_encode", m, src, blocks, meta)


def ecco_encode_minmax(m: Model, src, blocks=None, meta=None):
    """As ecco_encode, with the min/max pattern selector."""
    return _encode("ecco_encode_minmax", m, src, blocks, meta)


def ecco_decode(m: Model, blocks, meta, dst=None):
    import torch
    n = meta.numel()
    if dst is None:
        dst = torch.empty((n, GROUP), dtype=torch.float16, device=blocks.device)
    _check(lib().ecco_decode(m.handle, _dp(blocks), _dp(meta), n, _dp(dst), _stream()), "ecco_decode")
    return dst


def ecco_decode_indices(m: Model, blocks, meta, idx=None):
    import torch
    n = meta.numel()
    if idx is None:
        idx = torch.empty((n, GROUP), dtype=torch.uint8, device=blocks.device)
    _check(lib().ecco_decode_indices(m.handle, _dp(blocks), _dp(meta), n, _dp(idx), _stream()), "ecco_decode_indices")
    return idx


def ecco_decode_gemv(m: Model, blocks, meta, rows: int, cols: int, x, y=None):
    """x: CUDA FP16 [batch, cols]; returns y FP32 [batch, rows]."""
    import torch
    batch = x.shape[0] if x.dim() == 2 else 1
    if y is None:
        y = torch.empty((batch, rows), dtype=torch.float32, device=x.device)
    _check(lib().ecco_decode_gemv(m.handle, _dp(blocks), _dp(meta), rows, cols, _dp(x), batch, _dp(y), _stream()),
           "ecco_decode_gemv")
    return y


def ecco_kv_append(mk: Model, mv: Model, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max):
    _check(lib().ecco_kv_append(mk.handle, mv.handle, _dp(k_new), _dp(v_new), _dp(k_blocks), _dp(k_meta),
                                _dp(v_blocks), _dp(v_meta), _dp(seq_len), B, H, T_max, _stream()), "ecco_kv_append")


def ecco_kv_append_minmax(mk: Model, mv: Model, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max):
    _check(lib().ecco_kv_append_minmax(mk.handle, mv.handle, _dp(k_new), _dp(v_new), _dp(k_blocks), _dp(k_meta),
                                       _dp(v_blocks), _dp(v_meta), _dp(seq_len), B, H, T_max, _stream()),
           "ecco_kv_append_minmax")


def ecco_kv_attend(mk: Model, mv: Model, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max, out=None):
    import torch
    if out is None:
        out = torch.empty((B, H, GROUP), dtype=torch.float32, device=q.device)
    _check(lib().ecco_kv_attend(mk.handle, mv.handle, _dp(q), _dp(k_blocks), _dp(k_meta), _dp(v_blocks), _dp(v_meta),
                                _dp(seq_len), B, H, T_max, _dp(out), _stream()), "ecco_kv_attend")
    return out


def ecco_device_info(device: int = 0):
    """(compute units, memory clock in kHz, memory bus width in bits) as the runtime reports them."""
    cu, clk, bits = C.c_int(0), C.c_int(0), C.c_int(0)
    _check(lib().ecco_device_info(device, C.byref(cu), C.byref(clk), C.byref(bits)), "ecco_device_info")
    return cu.value, clk.value, bits.value


def ecco_kv_attend_gqa_splits(device: int, B: int, Hkv: int, tokens: int) -> int:
    n = int(lib().ecco_kv_attend_gqa_splits(device, B, Hkv, tokens))
    _check(min(n, 0), "ecco_kv_attend_gqa_splits")
    return n


def ecco_kv_attend_gqa(mk: Model, mv: Model, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max,
                       n_splits: int = 1, workspace=None, out=None):
    """q [B, Hq, 128] FP16; caches [B, Hkv, T_max]; workspace: uint8/float tensor of ecco_kv_attend_gqa_workspace bytes."""
    import torch
    if out is None:
        out = torch.empty((B, Hq, GROUP), dtype=torch.float32, device=q.device)
    if n_splits > 1 and workspace is None:
        workspace = torch.empty((int(lib().ecco_kv_attend_gqa_workspace(B, Hq, n_splits)),), dtype=torch.uint8, device=q.device)
    _check(lib().ecco_kv_attend_gqa(mk.handle, mv.handle, _dp(q), _dp(k_blocks), _dp(k_meta), _dp(v_blocks), _dp(v_meta),
                                    _dp(seq_len), B, Hq, Hkv, T_max, n_splits, _dp(workspace), _dp(out), _stream()),
           "ecco_kv_attend_gqa")
    return out


GQA_SCRATCH_BYTES = 8 << 20  # ECCO_GQA_SCRATCH_BYTES of include/ecco.h


def ecco_kv_attend_gqa_noalloc(mk: Model, mv: Model, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max, n_splits, out):
    """ecco_kv_attend_gqa with the splits' partial results in the library's static device array: the caller passes
    every buffer (`out` included) and nothing is allocated, here or in the library."""
    _check(lib().ecco_kv_attend_gqa_noalloc(mk.handle, mv.handle, _dp(q), _dp(k_blocks), _dp(k_meta), _dp(v_blocks), _dp(v_meta),
                                            _dp(seq_len), B, Hq, Hkv, T_max, n_splits, _dp(out), _stream()),
           "ecco_kv_attend_gqa_noalloc")
    return out


def ecco_read_stream(src, out):
    """Reads every byte of the CUDA tensor src once (measurement aid); out: CUDA int32 tensor with at least 256 elements."""
    _check(lib().ecco_read_stream(_dp(src), src.numel() * src.element_size(), _dp(out), _stream()), "ecco_read_stream")


ACT_GROUP = 64


def ecco_act_encode(src, blocks=None):
    """src: CUDA FP16 tensor with numel % 64 == 0.  Returns blocks uint8 [n, 64]."""
    import torch
    assert src.dtype == torch.float16 and src.numel() % ACT_GROUP == 0
    n = src.numel() // ACT_GROUP
    if blocks is None:
        blocks = torch.empty((n, BLOCK_BYTES), dtype=torch.uint8, device=src.device)
    _check(lib().ecco_act_encode(_dp(src), n, _dp(blocks), _stream()), "ecco_act_encode")
    return blocks


def ecco_act_decode(blocks, dst=None):
    import torch
    n = blocks.numel() // BLOCK_BYTES
    if dst is None:
        dst = torch.empty((n, ACT_GROUP), dtype=torch.float16, device=blocks.device)
    _check(lib().ecco_act_decode(_dp(blocks), n, _dp(dst), _stream()), "ecco_act_decode")
    return dst


# ---- the self-contained block format (include/ecco_paper_block.h) ------------------------------------------------
class PbModel:
    """Owner of an ecco_pb_model handle."""

    def __init__(self, handle):
        self._h = C.c_void_p(handle)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.ecco_pb_model_free(h)

    @property
    def handle(self):
        return self._h

    @property
    def S(self) -> int:
        return int(lib().ecco_pb_model_S(self._h))

    @property
    def texp(self) -> int:
        return int(lib().ecco_pb_model_texp(self._h))

    @property
    def centroids(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().ecco_pb_model_centroids(self._h), shape=(self.S, 15)).copy()

    @property
    def code_lens(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().ecco_pb_model_code_lens(self._h), shape=(self.S, 4, 16)).copy()

    @property
    def kp_lens(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().ecco_pb_model_kp_lens(self._h), shape=(self.S,)).copy()


def ecco_pb_fit(data, S: int, seed: int = 0) -> PbModel:
    a = np.ascontiguousarray(data)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("FP16 data expected")
    out = C.c_void_p(0)
    _check(lib().ecco_pb_fit(a.ctypes.data_as(C.c_void_p), a.size, S, seed, C.byref(out)), "ecco_pb_fit")
    return PbModel(out.value)


def ecco_pb_model_create(centroids, code_lens, kp_lens, texp: int) -> PbModel:
    c = np.ascontiguousarray(centroids)
    if c.dtype == np.float16:
        c = c.view(np.uint16)
    c = np.ascontiguousarray(c, dtype=np.uint16)
    l = np.ascontiguousarray(code_lens, dtype=np.uint8)
    k = np.ascontiguousarray(kp_lens, dtype=np.uint8)
    out = C.c_void_p(0)
    _check(lib().ecco_pb_model_create(c.ctypes.data_as(C.c_void_p), l.ctypes.data_as(C.c_void_p), k.ctypes.data_as(C.c_void_p),
                                      c.size // 15, int(texp), C.byref(out)), "ecco_pb_model_create")
    return PbModel(out.value)


def ecco_pb_model_save(m: PbModel) -> bytes:
    n = C.c_size_t(0)
    _check(lib().ecco_pb_model_save(m.handle, None, 0, C.byref(n)), "ecco_pb_model_save")
    buf = C.create_string_buffer(n.value)
    _check(lib().ecco_pb_model_save(m.handle, buf, n.value, C.byref(n)), "ecco_pb_model_save")
    return buf.raw[: n.value]


def ecco_pb_model_load(blob: bytes) -> PbModel:
    out = C.c_void_p(0)
    _check(lib().ecco_pb_model_load(blob, len(blob), C.byref(out)), "ecco_pb_model_load")
    return PbModel(out.value)


def ecco_pb_model_to_device(m: PbModel, device: int = 0) -> PbModel:
    _check(lib().ecco_pb_model_to_device(m.handle, device), "ecco_pb_model_to_device")
    return m


def ecco_pb_encode(m: PbModel, src, blocks=None):
    import torch
    assert src.dtype == torch.float16 and src.numel() % GROUP == 0
    n = src.numel() // GROUP
    if blocks is None:
        blocks = torch.empty((n, BLOCK_BYTES), dtype=torch.uint8, device=src.device)
    _check(lib().ecco_pb_encode(m.handle, _dp(src), n, _dp(blocks), _stream()), "ecco_pb_encode")
    return blocks


def ecco_pb_decode(m: PbModel, blocks, dst=None):
    import torch
    n = blocks.numel() // BLOCK_BYTES
    if dst is None:
        dst = torch.empty((n, GROUP), dtype=torch.float16, device=blocks.device)
    _check(lib().ecco_pb_decode(m.handle, _dp(blocks), n, _dp(dst), _stream()), "ecco_pb_decode")
    return dst


def ecco_pb_decode_gemv(m: PbModel, blocks, rows: int, cols: int, x, y=None):
    """x: CUDA FP16 [cols]; returns y FP32 [rows]."""
    import torch
    if y is None:
        y = torch.empty((rows,), dtype=torch.float32, device=x.device)
    _check(lib().ecco_pb_decode_gemv(m.handle, _dp(blocks), rows, cols, _dp(x), _dp(y), _stream()), "ecco_pb_decode_gemv")
    return y
