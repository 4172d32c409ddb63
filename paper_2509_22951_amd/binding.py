"""ctypes binding for libtq.so.  Function names mirror include/tq.h; pointers are passed as integers
(e.g. ``tensor.data_ptr()``, ``torch.cuda.current_stream().cuda_stream``) so no torch type crosses the ABI."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

TQ_MAX_BATCH = 16
TQ_MAX_ENTRIES_DEVICE = 30719
TQ_MAX_LMAX = 4
TQ_DEFAULT_SEG_COLS = 256

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[ctypes.CDLL] = None

EXPORTS = [
    "tq_encode", "tq_encode_quantized", "tq_free_blob", "tq_validate_blob", "tq_create_from_encoded", "tq_matvec",
    "tq_matvec_multi", "tq_decompress", "tq_decompress_multi", "tq_get_info", "tq_destroy", "tq_last_error_string",
    "tq_encode_gate_up", "tq_matvec_gate_up", "tq_matvec_gate_up_multi",
    "tq_set_ring_min_bands_per_cu",
    "tq_matvec_multi_static", "tq_step_create_staged", "tq_step_set_spin_limit",
    "tq_step_create", "tq_step_launch", "tq_step_get_info", "tq_step_destroy",
    "tq_listing_build_table", "tq_listing_compress", "tq_listing_create", "tq_listing_decompress", "tq_listing_get_info",
    "tq_listing_destroy",
]


class TqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"tq error {code}: {msg}")
        self.code = code


class TqEncodeOpts(ctypes.Structure):
    _fields_ = [("max_entries", ctypes.c_uint32), ("lmax", ctypes.c_uint32), ("n_threads", ctypes.c_uint32),
                ("seg_cols", ctypes.c_uint32), ("dict_from", ctypes.c_void_p), ("dict_from_bytes", ctypes.c_uint64),
                ("dictionary", ctypes.c_uint32), ("bits", ctypes.c_uint32), ("packing", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


class TqStepInfo(ctypes.Structure):
    _fields_ = [("n_matrices", ctypes.c_uint32), ("n_launches", ctypes.c_uint32), ("table_bytes", ctypes.c_uint64),
                ("n_stages", ctypes.c_uint32), ("persistent", ctypes.c_uint32), ("fault", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class TqInfo(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_uint32), ("cols", ctypes.c_uint32), ("seg_cols", ctypes.c_uint32),
                ("n_panels", ctypes.c_uint32), ("n_entries", ctypes.c_uint32), ("lmax", ctypes.c_uint32),
                ("n_units", ctypes.c_uint64), ("n_codes", ctypes.c_uint64), ("n_real_codes", ctypes.c_uint64),
                ("dict_bytes", ctypes.c_uint64),
                ("offset_bytes", ctypes.c_uint64), ("code_bytes", ctypes.c_uint64), ("scale_bytes", ctypes.c_uint64),
                ("compressed_bytes", ctypes.c_uint64), ("lane_spread", ctypes.c_uint32), ("packing", ctypes.c_uint32)]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class TqListingInfo(ctypes.Structure):
    _fields_ = [("n_values", ctypes.c_uint64), ("n_words", ctypes.c_uint64), ("n_tokens", ctypes.c_uint64),
                ("n_escapes", ctypes.c_uint64), ("n_table", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_ if n != "reserved"}


def lib_path() -> str:
    return os.environ.get("TQ_LIB_PATH") or os.path.join(_HERE, "libtq.so")


def load() -> ctypes.CDLL:
    """Load libtq.so.  Raises if it has not been built (python -m paper_2509_22951_amd.build)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python paper_2509_22951_amd/build.py` "
                                "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, sz, ci, u32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_uint32
    lib.tq_encode.restype = ci
    lib.tq_encode.argtypes = [vp, u32, u32, ctypes.POINTER(TqEncodeOpts), ctypes.POINTER(vp), ctypes.POINTER(sz)]
    lib.tq_encode_quantized.restype = ci
    lib.tq_encode_quantized.argtypes = [vp, vp, u32, u32, ctypes.POINTER(TqEncodeOpts), ctypes.POINTER(vp), ctypes.POINTER(sz)]
    lib.tq_free_blob.restype = None
    lib.tq_free_blob.argtypes = [vp]
    lib.tq_validate_blob.restype = ci
    lib.tq_validate_blob.argtypes = [vp, sz, ctypes.POINTER(TqInfo)]
    lib.tq_create_from_encoded.restype = ci
    lib.tq_create_from_encoded.argtypes = [vp, sz, ctypes.POINTER(vp)]
    lib.tq_matvec.restype = ci
    lib.tq_matvec.argtypes = [vp, vp, vp, ci, vp]
    lib.tq_set_ring_min_bands_per_cu.restype = ci
    lib.tq_set_ring_min_bands_per_cu.argtypes = [u32]
    lib.tq_encode_gate_up.restype = ci
    lib.tq_encode_gate_up.argtypes = [vp, vp, u32, u32, ctypes.POINTER(TqEncodeOpts), ctypes.POINTER(vp), ctypes.POINTER(sz)]
    lib.tq_matvec_gate_up.restype = ci
    lib.tq_matvec_gate_up.argtypes = [vp, vp, vp, ci, vp]
    lib.tq_matvec_gate_up_multi.restype = ci
    lib.tq_matvec_gate_up_multi.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp]
    lib.tq_matvec_multi.restype = ci
    lib.tq_matvec_multi.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp]
    lib.tq_matvec_multi_static.restype = ci
    lib.tq_matvec_multi_static.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp]
    lib.tq_step_create.restype = ci
    lib.tq_step_create.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ci, u32, ctypes.POINTER(vp)]
    lib.tq_step_create_staged.restype = ci
    lib.tq_step_create_staged.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(ci), ci, u32,
                                          ctypes.POINTER(vp)]
    lib.tq_step_set_spin_limit.restype = ci
    lib.tq_step_set_spin_limit.argtypes = [vp, u32]
    lib.tq_step_launch.restype = ci
    lib.tq_step_launch.argtypes = [vp, vp]
    lib.tq_step_get_info.restype = ci
    lib.tq_step_get_info.argtypes = [vp, ctypes.POINTER(TqStepInfo)]
    lib.tq_step_destroy.restype = ci
    lib.tq_step_destroy.argtypes = [vp]
    lib.tq_decompress.restype = ci
    lib.tq_decompress.argtypes = [vp, vp, vp]
    lib.tq_decompress_multi.restype = ci
    lib.tq_decompress_multi.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), vp]
    lib.tq_get_info.restype = ci
    lib.tq_get_info.argtypes = [vp, ctypes.POINTER(TqInfo)]
    lib.tq_destroy.restype = ci
    lib.tq_destroy.argtypes = [vp]
    lib.tq_last_error_string.restype = ctypes.c_char_p
    lib.tq_last_error_string.argtypes = []
    u64 = ctypes.c_uint64
    lib.tq_listing_build_table.restype = ci
    lib.tq_listing_build_table.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(u64), u32, u32, ctypes.POINTER(vp), ctypes.POINTER(u32)]
    lib.tq_listing_compress.restype = ci
    lib.tq_listing_compress.argtypes = [vp, u64, vp, u32, ctypes.POINTER(vp), ctypes.POINTER(u64)]
    lib.tq_listing_create.restype = ci
    lib.tq_listing_create.argtypes = [vp, u64, vp, u32, ctypes.POINTER(vp)]
    lib.tq_listing_decompress.restype = ci
    lib.tq_listing_decompress.argtypes = [vp, vp, vp]
    lib.tq_listing_get_info.restype = ci
    lib.tq_listing_get_info.argtypes = [vp, ctypes.POINTER(TqListingInfo)]
    lib.tq_listing_destroy.restype = ci
    lib.tq_listing_destroy.argtypes = [vp]
    _LIB = lib
    return lib


def tq_last_error_string() -> str:
    return load().tq_last_error_string().decode()


def _check(rc: int):
    if rc != 0:
        raise TqError(rc, tq_last_error_string())


DICTIONARY_KINDS = {"lzw": 0, "frequency": 1}


def _opts(max_entries: int, lmax: int, n_threads: int, seg_cols: int, dict_from: Optional[bytes],
          dictionary: str = "lzw", bits: int = 0, pack: bool = False) -> TqEncodeOpts:
    o = TqEncodeOpts()
    o.max_entries, o.lmax, o.n_threads, o.seg_cols = max_entries, lmax, n_threads, seg_cols
    o.bits = bits
    o.packing = 1 if pack else 0
    o.dictionary = DICTIONARY_KINDS[dictionary]
    if dict_from is not None:
        o.dict_from = ctypes.cast(ctypes.c_char_p(dict_from), ctypes.c_void_p)   # the caller's bytes object outlives the call
        o.dict_from_bytes = len(dict_from)
    return o


def _take_blob(ptr: ctypes.c_void_p, n: ctypes.c_size_t) -> bytes:
    try:
        return ctypes.string_at(ptr.value, n.value)
    finally:
        load().tq_free_blob(ptr)


def tq_encode(w: np.ndarray, max_entries: int = 0, lmax: int = 0, n_threads: int = 0, seg_cols: int = 0,
              dict_from: Optional[bytes] = None, dictionary: str = "lzw", bits: int = 0, pack: bool = False) -> bytes:
    """fp32 [rows, cols] host array -> container bytes.  dict_from: a container made earlier whose dictionary LZW
    continues from (one dictionary over a sequence of matrices).  bits: quantization width, 2..8 (0 = 8).
    pack (bits 2..4): two values per stored byte (TQ_PACK_NIBBLES)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    assert w.ndim == 2
    ptr, n = ctypes.c_void_p(), ctypes.c_size_t()
    o = _opts(max_entries, lmax, n_threads, seg_cols, dict_from, dictionary, bits, pack)
    _check(load().tq_encode(w.ctypes.data, w.shape[0], w.shape[1], ctypes.byref(o), ctypes.byref(ptr), ctypes.byref(n)))
    return _take_blob(ptr, n)


def tq_encode_quantized(q: np.ndarray, scales: np.ndarray, max_entries: int = 0, lmax: int = 0, n_threads: int = 0,
                        seg_cols: int = 0, dict_from: Optional[bytes] = None, dictionary: str = "lzw", pack: bool = False) -> bytes:
    q = np.ascontiguousarray(q, dtype=np.int8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    assert q.ndim == 2 and scales.shape == (q.shape[0],)
    ptr, n = ctypes.c_void_p(), ctypes.c_size_t()
    o = _opts(max_entries, lmax, n_threads, seg_cols, dict_from, dictionary, 0, pack)
    _check(load().tq_encode_quantized(q.ctypes.data, scales.ctypes.data, q.shape[0], q.shape[1], ctypes.byref(o),
                                      ctypes.byref(ptr), ctypes.byref(n)))
    return _take_blob(ptr, n)


def tq_encode_gate_up(w_gate: np.ndarray, w_up: np.ndarray, max_entries: int = 0, lmax: int = 0, n_threads: int = 0,
                      seg_cols: int = 0, dict_from: Optional[bytes] = None, dictionary: str = "lzw", bits: int = 0,
                      pack: bool = False) -> bytes:
    """Two fp32 [rows, cols] host arrays -> one container of 2 * rows rows, gate and up rows interleaved."""
    g = np.ascontiguousarray(w_gate, dtype=np.float32)
    u = np.ascontiguousarray(w_up, dtype=np.float32)
    assert g.ndim == 2 and g.shape == u.shape
    ptr, n = ctypes.c_void_p(), ctypes.c_size_t()
    o = _opts(max_entries, lmax, n_threads, seg_cols, dict_from, dictionary, bits, pack)
    _check(load().tq_encode_gate_up(g.ctypes.data, u.ctypes.data, g.shape[0], g.shape[1], ctypes.byref(o), ctypes.byref(ptr),
                                    ctypes.byref(n)))
    return _take_blob(ptr, n)


def tq_validate_blob(blob: bytes) -> dict:
    info = TqInfo()
    _check(load().tq_validate_blob(blob, len(blob), ctypes.byref(info)))
    return info.as_dict()


def tq_create_from_encoded(blob: bytes) -> int:
    """Returns the opaque handle (an integer).  Needs a GPU."""
    h = ctypes.c_void_p()
    _check(load().tq_create_from_encoded(blob, len(blob), ctypes.byref(h)))
    return h.value


def tq_matvec(handle: int, x_ptr: int, y_ptr: int, batch: int, stream: int = 0) -> None:
    _check(load().tq_matvec(handle, x_ptr, y_ptr, batch, stream))


def tq_set_ring_min_bands_per_cu(bands_per_cu: int) -> None:
    _check(load().tq_set_ring_min_bands_per_cu(bands_per_cu))


def tq_matvec_gate_up(handle: int, x_ptr: int, y_ptr: int, batch: int, stream: int = 0) -> None:
    _check(load().tq_matvec_gate_up(handle, x_ptr, y_ptr, batch, stream))


def tq_matvec_gate_up_multi(handles, x_ptrs, y_ptrs, batch: int, stream: int = 0) -> None:
    n = len(handles)
    assert n == len(x_ptrs) == len(y_ptrs) and n >= 1
    arr = ctypes.c_void_p * n
    _check(load().tq_matvec_gate_up_multi(n, arr(*handles), arr(*x_ptrs), arr(*y_ptrs), batch, stream))


class MultiCall:
    """Pre-marshalled argument arrays for tq_matvec_multi (built once, launched many times)."""

    def __init__(self, handles, x_ptrs, y_ptrs, batch: int):
        n = len(handles)
        assert n == len(x_ptrs) == len(y_ptrs) and n >= 1
        arr = ctypes.c_void_p * n
        self.n, self.batch = n, batch
        self.hs, self.xs, self.ys = arr(*handles), arr(*x_ptrs), arr(*y_ptrs)

    def launch(self, stream: int = 0) -> None:
        _check(load().tq_matvec_multi(self.n, self.hs, self.xs, self.ys, self.batch, stream))


def tq_matvec_multi(handles, x_ptrs, y_ptrs, batch: int, stream: int = 0) -> None:
    MultiCall(handles, x_ptrs, y_ptrs, batch).launch(stream)


TQ_STATIC_MAX_MATRICES = 896


def tq_matvec_multi_static(handles, x_ptrs, y_ptrs, batch: int, stream: int = 0) -> None:
    n = len(handles)
    assert n == len(x_ptrs) == len(y_ptrs) and n >= 1
    arr = ctypes.c_void_p * n
    _check(load().tq_matvec_multi_static(n, arr(*handles), arr(*x_ptrs), arr(*y_ptrs), batch, stream))


TQ_STEP_GATE_UP = 1
TQ_STEP_DECOMPRESS = 2


def tq_step_create(handles, x_ptrs, y_ptrs, batch: int, flags: int = 0) -> int:
    """x_ptrs may be None with TQ_STEP_DECOMPRESS (y_ptrs are then the int8 output matrices)."""
    n = len(handles)
    assert n == len(y_ptrs) and n >= 1 and (x_ptrs is None or len(x_ptrs) == n)
    arr = ctypes.c_void_p * n
    out = ctypes.c_void_p()
    xs = arr(*x_ptrs) if x_ptrs is not None else None
    _check(load().tq_step_create(n, arr(*handles), xs, arr(*y_ptrs), batch, flags, ctypes.byref(out)))
    return out.value


def tq_step_create_staged(handles, x_ptrs, y_ptrs, stages, batch: int, flags: int = 0) -> int:
    """stages[i]: the stage product i belongs to (from 0, never decreasing, never skipping)."""
    n = len(handles)
    assert n == len(x_ptrs) == len(y_ptrs) == len(stages) and n >= 1
    arr = ctypes.c_void_p * n
    out = ctypes.c_void_p()
    _check(load().tq_step_create_staged(n, arr(*handles), arr(*x_ptrs), arr(*y_ptrs), (ctypes.c_int * n)(*stages), batch, flags,
                                        ctypes.byref(out)))
    return out.value


def tq_step_set_spin_limit(step: int, polls: int) -> None:
    _check(load().tq_step_set_spin_limit(step, polls))


def tq_step_launch(step: int, stream: int = 0) -> None:
    _check(load().tq_step_launch(step, stream))


def tq_step_get_info(step: int) -> dict:
    info = TqStepInfo()
    _check(load().tq_step_get_info(step, ctypes.byref(info)))
    return {n: int(getattr(info, n)) for n, _ in info._fields_}


def tq_step_destroy(step) -> None:
    _check(load().tq_step_destroy(step))


class Step:
    """Owning wrapper around a prepared step (marshalling only): tq_matvec_multi for fixed matrices and buffers."""

    def __init__(self, handles, x_ptrs, y_ptrs, batch: int = 1, gate_up: bool = False, decompress: bool = False, stages=None):
        flags = (TQ_STEP_GATE_UP if gate_up else 0) | (TQ_STEP_DECOMPRESS if decompress else 0)
        if stages is not None:      # products that depend on each other: tq_step_create_staged
            self.handle = tq_step_create_staged(handles, x_ptrs, y_ptrs, stages, batch, flags)
        else:
            self.handle = tq_step_create(handles, x_ptrs, y_ptrs, batch, flags)
        self.info = tq_step_get_info(self.handle)

    def launch(self, stream: int = 0) -> None:
        tq_step_launch(self.handle, stream)

    def close(self) -> None:
        h, self.handle = self.handle, None
        tq_step_destroy(h)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tq_decompress(handle: int, out_ptr: int, stream: int = 0) -> None:
    _check(load().tq_decompress(handle, out_ptr, stream))


def tq_decompress_multi(handles, out_ptrs, stream: int = 0) -> None:
    n = len(handles)
    assert n == len(out_ptrs) and n >= 1
    arr = ctypes.c_void_p * n
    _check(load().tq_decompress_multi(n, arr(*handles), arr(*out_ptrs), stream))


def tq_get_info(handle: int) -> dict:
    info = TqInfo()
    _check(load().tq_get_info(handle, ctypes.byref(info)))
    return info.as_dict()


def tq_destroy(handle: Optional[int]) -> None:
    if handle:
        _check(load().tq_destroy(handle))


class Matrix:
    """Owning convenience wrapper around a handle (marshalling only)."""

    def __init__(self, blob: bytes):
        self.handle = tq_create_from_encoded(blob)
        self.info = tq_get_info(self.handle)

    def matvec(self, x_ptr: int, y_ptr: int, batch: int, stream: int = 0) -> None:
        tq_matvec(self.handle, x_ptr, y_ptr, batch, stream)

    def decompress(self, out_ptr: int, stream: int = 0) -> None:
        tq_decompress(self.handle, out_ptr, stream)

    def close(self) -> None:
        h, self.handle = self.handle, None
        tq_destroy(h)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- the stream format of the paper's section 4 listings (marshalling only) ----

def tq_listing_build_table(params, top_k: int = 65534) -> np.ndarray:
    """params: sequence of uint8 arrays (one per parameter).  Returns uint8 [n, 4]; row i is codeword i + 1."""
    arrs = [np.ascontiguousarray(p, dtype=np.uint8).reshape(-1) for p in params]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[a.ctypes.data for a in arrs])
    lens = (ctypes.c_uint64 * max(n, 1))(*[a.size for a in arrs])
    table, n_table = ctypes.c_void_p(), ctypes.c_uint32()
    _check(load().tq_listing_build_table(ptrs, lens, n, top_k, ctypes.byref(table), ctypes.byref(n_table)))
    try:
        raw = ctypes.string_at(table.value, n_table.value * 4) if n_table.value else b""
    finally:
        load().tq_free_blob(table)
    return np.frombuffer(raw, dtype=np.uint8).reshape(-1, 4).copy()


def tq_listing_compress(values: np.ndarray, table: np.ndarray) -> np.ndarray:
    """One parameter's byte values -> its uint16 words."""
    v = np.ascontiguousarray(values, dtype=np.uint8).reshape(-1)
    t = np.ascontiguousarray(table, dtype=np.uint8).reshape(-1, 4)
    words, n_words = ctypes.c_void_p(), ctypes.c_uint64()
    _check(load().tq_listing_compress(v.ctypes.data, v.size, t.ctypes.data, t.shape[0], ctypes.byref(words), ctypes.byref(n_words)))
    try:
        raw = ctypes.string_at(words.value, n_words.value * 2) if n_words.value else b""
    finally:
        load().tq_free_blob(words)
    return np.frombuffer(raw, dtype=np.uint16).copy()


class Listing:
    """Owning wrapper around a tq_listing handle (a compressed parameter and its table in device memory)."""

    def __init__(self, words: np.ndarray, table: np.ndarray):
        w = np.ascontiguousarray(words, dtype=np.uint16).reshape(-1)
        t = np.ascontiguousarray(table, dtype=np.uint8).reshape(-1, 4)
        h = ctypes.c_void_p()
        _check(load().tq_listing_create(w.ctypes.data, w.size, t.ctypes.data, t.shape[0], ctypes.byref(h)))
        self.handle = h.value
        info = TqListingInfo()
        _check(load().tq_listing_get_info(self.handle, ctypes.byref(info)))
        self.info = info.as_dict()

    def decompress(self, out_ptr: int, stream: int = 0) -> None:
        _check(load().tq_listing_decompress(self.handle, out_ptr, stream))

    def close(self) -> None:
        h, self.handle = self.handle, None
        if h:
            _check(load().tq_listing_destroy(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
