"""CPU oracle for the fused dictionary-decode + dequantize + matrix-vector path.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``; the product package never imports it and the two share no code.
Everything here is the plain definition (or the paper's algorithm step by step) in numpy / plain C:

* ``quantize_rows``   per-row symmetric absmax int8 (the 8-bit choice of the paper's section 3; rounding
                      primitive = round-half-to-even as in Listing 1's ``torch.round``; per-row symmetric
                      granularity is the benchmark configuration's, not the listing's per-tensor min/max).
* ``serialize``       the fixed byte order in which a matrix is handed to the codec (format rule, no maths).
* ``lzw_encode``      LZW as described in the paper's Background, "Compression" (C, see tq_oracle.c).
* ``lzw_decode``      table lookup decompression, section 4: reproduces the quantized bytes exactly.
* ``gemv_f64``        y = diag(s) Q x in float64, the definition the fused kernel must reach.
* ``build_blob`` / ``parse_blob``  writer and reader of the container format, written from the format
                      description independently of the product's encoder.

Pins (tests/test_oracle_*.py): quantizer closed forms and invariances; serialization special cases that
reduce to numpy slicing; LZW against a published worked example, closed-form all-equal inputs, a
brute-force longest-match parser on tiny alphabets, round-trip identity and the zeroth-order entropy
bound; GEMV against numpy float64 matmul and unit-vector probes.  No function here is unpinned.
"""
from __future__ import annotations

import ctypes
import os
import struct
import subprocess
from dataclasses import dataclass

import numpy as np

TILE_ROWS = 16      # rows per micro-tile
MT_COLS = 8         # columns per micro-tile
GROUP_COLS = 256    # columns per restart group (32 micro-tiles)
GROUP_BYTES = TILE_ROWS * GROUP_COLS
CODE_ALIGN = 8      # each group's code run is padded to a multiple of this many codes (one 16-byte lane load)
LCAP = 16           # must equal TQO_LCAP in tq_oracle.c
MAGIC = b"TQMOEv1\0"
HEADER_BYTES = 256
SECTION_ALIGN = 256

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def build_oracle_lib(force: bool = False) -> str:
    """Compile tq_oracle.c with gcc into oracle/_build/ (idempotent)."""
    src = os.path.join(_HERE, "tq_oracle.c")
    out_dir = os.path.join(_HERE, "_build")
    out = os.path.join(out_dir, "libtqoracle.so")
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        os.makedirs(out_dir, exist_ok=True)
        tmp = out + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", tmp, src])
        os.replace(tmp, out)
    return out


def _lib():
    global _LIB
    if _LIB is None:
        lib = ctypes.CDLL(build_oracle_lib())
        ll, vp, ci = ctypes.c_longlong, ctypes.c_void_p, ctypes.c_int
        lib.tqo_lzw_encode.restype = ll
        lib.tqo_lzw_encode.argtypes = [vp, ll, ll, ci, ci, vp, vp, vp, vp, ctypes.POINTER(ci)]
        lib.tqo_lzw_decode.restype = ll
        lib.tqo_lzw_decode.argtypes = [vp, vp, ll, ll, ll, vp, vp, ci, ci, vp]
        lib.tqo_gemv_f64.restype = None
        lib.tqo_gemv_f64.argtypes = [vp, vp, vp, ll, ll, ll, vp]
        _LIB = lib
    return _LIB


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------- quantizer

def quantize_rows(W: np.ndarray):
    """Per-row symmetric absmax int8.  All arithmetic in IEEE fp32, in this order:
    amax = max_j |W[r,j]|;  s[r] = amax / 127;  Q[r,j] = clamp(rne(W[r,j] / s[r]), -127, 127).
    A row of zeros gets s = 0 and Q = 0.  Dequantized weight = s[r] * Q[r,j].
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    amax = np.max(np.abs(W), axis=1).astype(np.float32)
    s = (amax / np.float32(127.0)).astype(np.float32)
    safe = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    t = (W / safe[:, None]).astype(np.float32)
    q = np.clip(np.rint(t), -127.0, 127.0)
    q = np.where(s[:, None] > 0, q, 0.0)
    return q.astype(np.int8), s


# --------------------------------------------------------------------------- serialization

def padded_shape(rows: int, cols: int):
    rp = -(-rows // TILE_ROWS) * TILE_ROWS
    cp = -(-cols // GROUP_COLS) * GROUP_COLS
    return rp, cp


def serialize(Q: np.ndarray) -> np.ndarray:
    """Matrix -> codec byte string.  Q is zero-padded to multiples of (16, 256); the string lists
    16x8 micro-tiles (each row-major), micro-tiles left to right, 16-row bands top to bottom.
    int8 -> byte by two's complement."""
    Q = np.ascontiguousarray(Q, dtype=np.int8)
    rows, cols = Q.shape
    rp, cp = padded_shape(rows, cols)
    P = np.zeros((rp, cp), dtype=np.int8)
    P[:rows, :cols] = Q
    # (band, i, microtile, c) -> (band, microtile, i, c)
    S = P.reshape(rp // TILE_ROWS, TILE_ROWS, cp // MT_COLS, MT_COLS).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(S).reshape(-1).view(np.uint8)


def deserialize(S: np.ndarray, rows: int, cols: int) -> np.ndarray:
    rp, cp = padded_shape(rows, cols)
    S = np.ascontiguousarray(S, dtype=np.uint8)
    assert S.size == rp * cp
    P = S.view(np.int8).reshape(rp // TILE_ROWS, cp // MT_COLS, TILE_ROWS, MT_COLS).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(P).reshape(rp, cp)[:rows, :cols].copy()


# --------------------------------------------------------------------------- codec

@dataclass
class Dictionary:
    ent_bytes: np.ndarray   # uint8 [n_entries, LCAP]; bytes beyond ent_len are zero
    ent_len: np.ndarray     # uint8 [n_entries]

    @property
    def n_entries(self) -> int:
        return int(self.ent_len.size)

    def entry(self, e: int) -> bytes:
        return bytes(self.ent_bytes[e, : self.ent_len[e]])


def lzw_encode(S: np.ndarray, group_bytes: int = GROUP_BYTES, max_entries: int = 32000, lmax: int = 3):
    """Returns (codes uint16 [n_codes] without padding, group_ncodes uint32 [n_groups], Dictionary)."""
    S = np.ascontiguousarray(S, dtype=np.uint8)
    n = int(S.size)
    n_groups = -(-n // group_bytes) if n else 0
    codes = np.zeros(max(n, 1), dtype=np.uint16)
    gnc = np.zeros(max(n_groups, 1), dtype=np.uint32)
    eb = np.zeros((max_entries, LCAP), dtype=np.uint8)
    el = np.zeros(max_entries, dtype=np.uint8)
    ne = ctypes.c_int(0)
    nc = _lib().tqo_lzw_encode(_ptr(S), n, group_bytes, max_entries, lmax, _ptr(codes), _ptr(gnc), _ptr(eb), _ptr(el),
                               ctypes.byref(ne))
    if nc < 0:
        raise ValueError("tqo_lzw_encode: bad arguments")
    return codes[:nc].copy(), gnc[:n_groups].copy(), Dictionary(eb[: ne.value].copy(), el[: ne.value].copy())


def pad_stream(codes: np.ndarray, group_ncodes: np.ndarray, pad_code: int, align: int = CODE_ALIGN):
    """Lay the per-group code runs out with each run padded to a multiple of `align` codes.
    Returns (stream uint16, goff uint32 [n_groups+1])."""
    padded = (-(-group_ncodes.astype(np.int64) // align)) * align
    goff = np.zeros(group_ncodes.size + 1, dtype=np.int64)
    np.cumsum(padded, out=goff[1:])
    stream = np.full(int(goff[-1]), pad_code, dtype=np.uint16)
    src = np.zeros(group_ncodes.size + 1, dtype=np.int64)
    np.cumsum(group_ncodes.astype(np.int64), out=src[1:])
    # destination index of every real code
    grp = np.repeat(np.arange(group_ncodes.size), group_ncodes.astype(np.int64))
    dst = np.arange(codes.size, dtype=np.int64) - src[grp] + goff[grp]
    stream[dst] = codes
    assert goff[-1] < 2 ** 32
    return stream, goff.astype(np.uint32)


def lzw_decode(stream: np.ndarray, goff: np.ndarray, d: Dictionary, n_bytes: int, pad_code: int,
               group_bytes: int = GROUP_BYTES) -> np.ndarray:
    stream = np.ascontiguousarray(stream, dtype=np.uint16)
    goff = np.ascontiguousarray(goff, dtype=np.uint32)
    n_groups = goff.size - 1
    assert n_groups == (-(-n_bytes // group_bytes) if n_bytes else 0)
    out = np.zeros(n_bytes, dtype=np.uint8)
    eb = np.ascontiguousarray(d.ent_bytes, dtype=np.uint8)
    el = np.ascontiguousarray(d.ent_len, dtype=np.uint8)
    rc = _lib().tqo_lzw_decode(_ptr(stream), _ptr(goff), n_groups, group_bytes, n_bytes, _ptr(eb), _ptr(el),
                               d.n_entries, pad_code, _ptr(out))
    if rc != 0:
        raise ValueError(f"stream inconsistent in group {-rc - 1}")
    return out


# --------------------------------------------------------------------------- GEMV

def gemv_f64(Q: np.ndarray, s: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y[b, r] = s[r] * sum_j Q[r, j] * x[b, j], float64, natural order.  x: fp32 [B, K]."""
    Q = np.ascontiguousarray(Q, dtype=np.int8)
    s = np.ascontiguousarray(s, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim == 1:
        x = x[None, :]
    R, K = Q.shape
    B = x.shape[0]
    assert x.shape[1] == K and s.size == R
    y = np.zeros((B, R), dtype=np.float64)
    _lib().tqo_gemv_f64(_ptr(Q), _ptr(s), _ptr(x), R, K, B, _ptr(y))
    return y


# --------------------------------------------------------------------------- whole-matrix encode + container

@dataclass
class Encoded:
    rows: int
    cols: int
    lmax: int
    max_entries: int
    Q: np.ndarray           # int8 [rows, cols]
    scales: np.ndarray      # fp32 [rows]
    dictionary: Dictionary
    stream: np.ndarray      # uint16, padded
    goff: np.ndarray        # uint32 [n_groups + 1]
    n_real_codes: int

    @property
    def pad_code(self) -> int:
        return self.dictionary.n_entries


def encode_quantized(Q: np.ndarray, scales: np.ndarray, max_entries: int = 32000, lmax: int = 3) -> Encoded:
    rows, cols = Q.shape
    S = serialize(Q)
    codes, gnc, d = lzw_encode(S, GROUP_BYTES, max_entries, lmax)
    stream, goff = pad_stream(codes, gnc, d.n_entries)
    return Encoded(rows, cols, lmax, max_entries, Q, np.asarray(scales, np.float32), d, stream, goff, int(codes.size))


def encode_matrix(W: np.ndarray, max_entries: int = 32000, lmax: int = 3) -> Encoded:
    Q, s = quantize_rows(W)
    return encode_quantized(Q, s, max_entries, lmax)


def dict_slots(d: Dictionary) -> np.ndarray:
    """Device dictionary words: bytes 0..2 = run (unused bytes zero), byte 3 = run length in bits (8, 16
    or 24); one extra all-zero word at index n_entries is the pad code's entry (length 0).  Needs lmax <= 3."""
    assert int(d.ent_len.max()) <= 3
    eb = d.ent_bytes.astype(np.uint32)
    w = eb[:, 0] | (eb[:, 1] << 8) | (eb[:, 2] << 16) | ((8 * d.ent_len.astype(np.uint32)) << 24)
    return np.concatenate([w, np.zeros(1, np.uint32)]).astype(np.uint32)


def _align(n: int, a: int = SECTION_ALIGN) -> int:
    return -(-n // a) * a


_HDR = struct.Struct("<8sII" "II" "II" "IIII" "IIII" "QQ" "QQ" "QQ" "QQ" "QQ" "Q" "I")


def build_blob(e: Encoded) -> bytes:
    rp, cp = padded_shape(e.rows, e.cols)
    slots = dict_slots(e.dictionary)
    scales = np.zeros(rp, np.float32)
    scales[: e.rows] = e.scales
    n_groups = (rp // TILE_ROWS) * (cp // GROUP_COLS)
    assert e.goff.size == n_groups + 1
    sec = [slots.tobytes(), e.goff.astype(np.uint32).tobytes(), e.stream.astype(np.uint16).tobytes(), scales.tobytes()]
    offs, pos = [], HEADER_BYTES
    for b in sec:
        offs.append(pos)
        pos = _align(pos + len(b))
    total = pos
    hdr = _HDR.pack(MAGIC, 1, HEADER_BYTES, e.rows, e.cols, rp, cp, TILE_ROWS, MT_COLS, GROUP_COLS, GROUP_BYTES,
                    e.dictionary.n_entries, e.lmax, e.max_entries, e.pad_code, n_groups, int(e.stream.size),
                    offs[0], len(sec[0]), offs[1], len(sec[1]), offs[2], len(sec[2]), offs[3], len(sec[3]),
                    total, CODE_ALIGN)
    out = bytearray(total)
    out[: len(hdr)] = hdr
    for o, b in zip(offs, sec):
        out[o: o + len(b)] = b
    return bytes(out)


def parse_blob(blob: bytes) -> dict:
    (magic, version, hbytes, rows, cols, rp, cp, tr, mc, gc, gb, n_entries, lmax, max_entries, pad_code, n_groups,
     n_codes, o_d, b_d, o_g, b_g, o_c, b_c, o_s, b_s, total, calign) = _HDR.unpack_from(blob, 0)
    assert magic == MAGIC and version == 1 and hbytes == HEADER_BYTES
    assert (tr, mc, gc, gb, calign) == (TILE_ROWS, MT_COLS, GROUP_COLS, GROUP_BYTES, CODE_ALIGN)
    assert total == len(blob) and pad_code == n_entries
    buf = np.frombuffer(blob, dtype=np.uint8)
    slots = buf[o_d: o_d + b_d].view(np.uint32)
    goff = buf[o_g: o_g + b_g].view(np.uint32)
    stream = buf[o_c: o_c + b_c].view(np.uint16)
    scales = buf[o_s: o_s + b_s].view(np.float32)
    assert slots.size == n_entries + 1 and goff.size == n_groups + 1 and stream.size == n_codes and scales.size == rp
    assert np.all((slots[:n_entries] >> 24) % 8 == 0)
    el = ((slots[:n_entries] >> 24) // 8).astype(np.uint8)
    eb = np.zeros((n_entries, LCAP), np.uint8)
    for k in range(3):
        eb[:, k] = (slots[:n_entries] >> (8 * k)) & 0xFF
    return dict(rows=rows, cols=cols, rows_pad=rp, cols_pad=cp, n_entries=n_entries, lmax=lmax,
                max_entries=max_entries, pad_code=pad_code, n_groups=n_groups, n_codes=n_codes,
                dictionary=Dictionary(eb, el), slots=slots, goff=goff, stream=stream, scales=scales,
                compressed_bytes=int(b_d + b_g + b_c + b_s), stream_bytes=int(b_c))


def decode_blob(blob: bytes):
    """Container -> (Q int8 [rows, cols], scales fp32 [rows]) through the oracle's own decoder."""
    p = parse_blob(blob)
    S = lzw_decode(p["stream"], p["goff"], p["dictionary"], p["rows_pad"] * p["cols_pad"], p["pad_code"])
    return deserialize(S, p["rows"], p["cols"]), p["scales"][: p["rows"]].copy()


def matvec_from_blob(blob: bytes, x: np.ndarray) -> np.ndarray:
    Q, s = decode_blob(blob)
    return gemv_f64(Q, s, x)
