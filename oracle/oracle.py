"""CPU oracle for the fused dictionary-decode + dequantize + matrix-vector path.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``; the product package never imports it and the two share no code.
Everything here is the plain definition (or the paper's algorithm step by step) in numpy / plain C:

* ``quantize_rows``   per-row symmetric absmax int8 (the 8-bit choice of the paper's section 3; rounding
                      primitive = round-half-to-even as in Listing 1's ``torch.round``; per-row symmetric
                      granularity is the benchmark configuration's, not the listing's per-tensor min/max).
* ``serialize``       the fixed byte order in which a matrix is handed to the codec (format rule, no maths).
* ``lzw_encode``      LZW as described in the paper's Background, "Compression" (C, see tq_oracle.c).
* ``frequency_dictionary``  entries picked by frequency, as section 4 picks its table (runs of 2; numpy).
* ``sort_code_space`` the codes renumbered so that a code's place tells its run length (format rule, a permutation).
* ``lzw_decode``      table lookup decompression, section 4: reproduces the quantized bytes exactly.
* ``gemv_f64``        y = diag(s) Q x in float64, the definition the fused kernel must reach.
* ``build_blob`` / ``parse_blob``  writer and reader of the container format, written from the format
                      description independently of the product's encoder.

Pins (tests/test_oracle_*.py): quantizer closed forms and invariances; serialization special cases that
reduce to numpy slicing; LZW against a published worked example, closed-form all-equal inputs, a
brute-force longest-match parser on tiny alphabets, round-trip identity and the zeroth-order entropy
bound; the frequency dictionary against hand-counted inputs and against a plain counting loop; GEMV against numpy float64 matmul and unit-vector probes.  No function here is unpinned.
tests/test_oracle_pins_catch_mistakes.py plants mistakes here (wrong rounding, index, sign, order) and expects the pins to fail.
"""
from __future__ import annotations

import ctypes
import os
import struct
import subprocess
from dataclasses import dataclass

import numpy as np

UNIT_ROWS = 16      # rows of a unit (lane & 15)
UNIT_PANELS = 4     # column panels of a unit (lane >> 4)
CHUNK_CODES = 4     # codes per lane and chunk
CHUNK_WORDS = 64 * CHUNK_CODES
DEFAULT_SEG_COLS = 256
LCAP = 16           # must equal TQO_LCAP in tq_oracle.c
MAGIC = b"TQMOEv3\0"
UNIT_BUDGET = 30716  # dictionary storage the device path offers when runs may be longer than 2 bytes: units of one
                     # 32-bit word of the product kernel's LDS image, 1 per entry of up to 2 bytes, 2 per longer entry,
                     # 4 more kept for the padding code's entry and alignment (120 KB in all)
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
        lib.tqo_lzw_encode.argtypes = [vp, ll, vp, ll, ci, ci, ll, ci, vp, vp, vp, vp, ctypes.POINTER(ci)]
        lib.tqo_lzw_decode.restype = ll
        lib.tqo_lzw_decode.argtypes = [vp, vp, vp, ll, vp, vp, ci, ci, vp]
        lib.tqo_gemv_f64.restype = None
        lib.tqo_gemv_f64.argtypes = [vp, vp, vp, ll, ll, ll, vp]
        _LIB = lib
    return _LIB


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


# --------------------------------------------------------------------------- quantizer

def quantize_rows(W: np.ndarray, bits: int = 8):
    """Per-row symmetric absmax quantization to `bits` bits (paper section 3: a fixed range of discrete levels set by
    the number of bits; 2..8).  qmax = 2^(bits-1) - 1 (127 at 8 bits, 1 at 2 bits: ternary).  All arithmetic in IEEE
    fp32, in this order:
    amax = max_j |W[r,j]|;  s[r] = amax / qmax;  Q[r,j] = clamp(rne(W[r,j] / s[r]), -qmax, qmax).
    A row of zeros gets s = 0 and Q = 0.  Dequantized weight = s[r] * Q[r,j].  Q is kept one value per int8.
    """
    if not 2 <= bits <= 8:
        raise ValueError("bits must be in [2, 8]")
    qmax = np.float32((1 << (bits - 1)) - 1)
    W = np.ascontiguousarray(W, dtype=np.float32)
    amax = np.max(np.abs(W), axis=1).astype(np.float32)
    s = (amax / qmax).astype(np.float32)
    safe = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    t = (W / safe[:, None]).astype(np.float32)
    q = np.clip(np.rint(t), -qmax, qmax)
    q = np.where(s[:, None] > 0, q, 0.0)
    return q.astype(np.int8), s


# --------------------------------------------------------------------------- serialization

def geometry(rows: int, cols: int, seg_cols: int = DEFAULT_SEG_COLS):
    """(n_bands, n_panels, n_quads) of a rows x cols matrix cut into segments of seg_cols columns."""
    assert seg_cols % 16 == 0 and 16 <= seg_cols <= 1024
    n_bands = -(-rows // UNIT_ROWS)
    n_panels = -(-cols // seg_cols)
    n_quads = -(-n_panels // UNIT_PANELS)
    return n_bands, n_panels, n_quads


def segment_table(rows: int, cols: int, seg_cols: int = DEFAULT_SEG_COLS):
    """The segments in stream order.  A segment is seg_cols consecutive columns of one row (the last panel of a
    row may be shorter).  They come in units of 64 = 16 consecutive rows (a band) x 4 consecutive panels (a quad),
    units ordered band-major then quad; inside a unit, lane l owns row 16*band + (l & 15), panel 4*quad + (l >> 4).
    Segments past the matrix edge exist with length 0.  Returns (row, col0, length) int64 arrays [n_units * 64]."""
    n_bands, n_panels, n_quads = geometry(rows, cols, seg_cols)
    band, quad, lane = np.meshgrid(np.arange(n_bands), np.arange(n_quads), np.arange(64), indexing="ij")
    row = (UNIT_ROWS * band + (lane & 15)).reshape(-1).astype(np.int64)
    panel = (UNIT_PANELS * quad + (lane >> 4)).reshape(-1).astype(np.int64)
    col0 = panel * seg_cols
    length = np.where((row < rows) & (panel < n_panels), np.minimum(seg_cols, cols - col0), 0).astype(np.int64)
    length = np.maximum(length, 0)
    return row, col0, length


def serialize(Q: np.ndarray, seg_cols: int = DEFAULT_SEG_COLS):
    """Matrix -> (codec byte string, segment lengths): the segments of segment_table() back to back;
    int8 -> byte by two's complement."""
    Q = np.ascontiguousarray(Q, dtype=np.int8)
    rows, cols = Q.shape
    row, col0, length = segment_table(rows, cols, seg_cols)
    start = np.zeros(length.size + 1, np.int64)
    np.cumsum(length, out=start[1:])
    seg = np.repeat(np.arange(length.size), length)
    within = np.arange(int(start[-1]), dtype=np.int64) - start[seg]
    S = Q[row[seg], col0[seg] + within]
    return np.ascontiguousarray(S).view(np.uint8), length.astype(np.uint32)


def deserialize(S: np.ndarray, rows: int, cols: int, seg_cols: int = DEFAULT_SEG_COLS) -> np.ndarray:
    S = np.ascontiguousarray(S, dtype=np.uint8)
    row, col0, length = segment_table(rows, cols, seg_cols)
    assert S.size == int(length.sum()) == rows * cols
    start = np.zeros(length.size + 1, np.int64)
    np.cumsum(length, out=start[1:])
    seg = np.repeat(np.arange(length.size), length)
    within = np.arange(S.size, dtype=np.int64) - start[seg]
    Q = np.zeros((rows, cols), np.int8)
    Q[row[seg], col0[seg] + within] = S.view(np.int8)
    return Q


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


def lzw_encode(S: np.ndarray, seg_len, max_entries: int = 30719, lmax: int = 2, carry: "Dictionary | None" = None,
               unit_budget: int = 0):
    """LZW over the segments of S (a match never crosses a segment end).  `seg_len` is the array of segment
    lengths, or one integer = equal-length segments (the last may be short).  `carry` = the dictionary a previous
    call returned: the parse starts with those entries instead of the 256 singles alone.  `unit_budget` (0 = none):
    an entry is added only while the dictionary stays within that many units (1 per entry of up to 2 bytes, 2 per
    longer one).
    Returns (codes uint16 [n_codes], seg_ncodes uint32 [n_segs], Dictionary)."""
    S = np.ascontiguousarray(S, dtype=np.uint8)
    n = int(S.size)
    if np.isscalar(seg_len):
        g = int(seg_len)
        k = -(-n // g) if n else 0
        seg_len = np.full(k, g, np.uint32)
        if k:
            seg_len[-1] = n - g * (k - 1)
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint32)
    n_segs = int(seg_len.size)
    codes = np.zeros(max(n, 1), dtype=np.uint16)
    snc = np.zeros(max(n_segs, 1), dtype=np.uint32)
    eb = np.zeros((max_entries, LCAP), dtype=np.uint8)
    el = np.zeros(max_entries, dtype=np.uint8)
    n_init = 0
    if carry is not None:
        n_init = carry.n_entries
        eb[:n_init] = carry.ent_bytes
        el[:n_init] = carry.ent_len
    ne = ctypes.c_int(0)
    nc = _lib().tqo_lzw_encode(_ptr(S), n, _ptr(seg_len), n_segs, max_entries, lmax, unit_budget, n_init, _ptr(codes),
                               _ptr(snc), _ptr(eb), _ptr(el), ctypes.byref(ne))
    if nc < 0:
        raise ValueError("tqo_lzw_encode: bad arguments")
    return codes[:nc].copy(), snc[:n_segs].copy(), Dictionary(eb[: ne.value].copy(), el[: ne.value].copy())


def sort_code_space(codes: np.ndarray, d: Dictionary):
    """Renumber the codes so that the entries come in order of run length (all 1-byte entries, then the 2-byte ones,
    ...), entries of equal length keeping the order LZW created them in: a code's place in the code space then tells its
    length.  The single bytes keep code == byte.  Returns (renumbered codes, reordered dictionary, class_end) with
    class_end[k] = number of entries of at most k + 1 bytes, k = 0..3 (runs are at most 4 bytes here).
    LZW adds a run only after the run it extends, so every entry still follows the entry it extends."""
    assert int(d.ent_len.max()) <= 4
    order = np.argsort(d.ent_len, kind="stable")           # order[new] = old
    new_of_old = np.empty(order.size, np.int64)
    new_of_old[order] = np.arange(order.size)
    sorted_len = d.ent_len[order]
    class_end = np.array([int((sorted_len <= k + 1).sum()) for k in range(4)], np.uint32)
    return new_of_old[codes].astype(np.uint16), Dictionary(d.ent_bytes[order].copy(), sorted_len.copy()), class_end


def interleave(codes: np.ndarray, seg_ncodes: np.ndarray, pad_code: int):
    """Lay the code runs of the segments out as lane streams: segments come in units of 64 (segment g = lane g % 64
    of unit g // 64; the last unit is completed with empty segments); every lane stream of a unit is padded with
    pad_code to the unit's length = longest lane stream rounded up to whole chunks of 4 codes; code k of lane l of
    unit u goes to stream[(uoff[u] + k // 4) * 256 + l * 4 + k % 4].  Returns (stream uint16, uoff uint32 [n_units+1],
    in chunks)."""
    n_segs = int(seg_ncodes.size)
    n_units = -(-n_segs // 64)
    cnt = np.zeros(n_units * 64, np.int64)
    cnt[:n_segs] = seg_ncodes
    unit_chunks = -(-cnt.reshape(n_units, 64).max(axis=1) // CHUNK_CODES) if n_units else np.zeros(0, np.int64)
    uoff = np.zeros(n_units + 1, np.int64)
    np.cumsum(unit_chunks, out=uoff[1:])
    assert uoff[-1] * CHUNK_WORDS < 2 ** 32
    stream = np.full(int(uoff[-1]) * CHUNK_WORDS, pad_code, dtype=np.uint16)
    src = np.zeros(cnt.size + 1, np.int64)
    np.cumsum(cnt, out=src[1:])
    seg = np.repeat(np.arange(cnt.size), cnt)
    k = np.arange(codes.size, dtype=np.int64) - src[seg]
    dst = (uoff[seg // 64] + k // CHUNK_CODES) * CHUNK_WORDS + (seg % 64) * CHUNK_CODES + k % CHUNK_CODES
    stream[dst] = codes
    return stream, uoff.astype(np.uint32)


def lzw_decode(stream: np.ndarray, uoff: np.ndarray, seg_len: np.ndarray, d: Dictionary, pad_code: int) -> np.ndarray:
    """Inverse of lzw_encode + interleave: returns the byte string (segments back to back)."""
    stream = np.ascontiguousarray(stream, dtype=np.uint16)
    uoff = np.ascontiguousarray(uoff, dtype=np.uint32)
    seg_len = np.ascontiguousarray(seg_len, dtype=np.uint32)
    n_segs = int(seg_len.size)
    assert uoff.size - 1 == -(-n_segs // 64)
    assert stream.size == int(uoff[-1]) * CHUNK_WORDS
    out = np.zeros(max(int(seg_len.sum()), 1), dtype=np.uint8)
    eb = np.ascontiguousarray(d.ent_bytes, dtype=np.uint8)
    el = np.ascontiguousarray(d.ent_len, dtype=np.uint8)
    rc = _lib().tqo_lzw_decode(_ptr(stream), _ptr(uoff), _ptr(seg_len), n_segs, _ptr(eb), _ptr(el), d.n_entries,
                               pad_code, _ptr(out))
    if rc != 0:
        raise ValueError(f"stream inconsistent in segment {-rc - 1}")
    return out[: int(seg_len.sum())]


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


def gate_up_f64(Qg: np.ndarray, sg: np.ndarray, Qu: np.ndarray, su: np.ndarray, x: np.ndarray) -> np.ndarray:
    """The gated pair of a feed-forward block by its definition, in float64: silu(g) * u with g, u the two
    matrix-vector products and silu(g) = g / (1 + exp(-g))."""
    g = gemv_f64(Qg, sg, x)
    u = gemv_f64(Qu, su, x)
    return g / (1.0 + np.exp(-g)) * u


def interleave_rows(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Rows a[0], b[0], a[1], b[1], ... (the row order of a gate/up container)."""
    assert a.shape == b.shape
    out = np.empty((2 * a.shape[0],) + a.shape[1:], dtype=a.dtype)
    out[0::2] = a
    out[1::2] = b
    return out


# --------------------------------------------------------------------------- whole-matrix encode + container

@dataclass
class Encoded:
    rows: int
    cols: int
    seg_cols: int
    lmax: int
    max_entries: int
    Q: np.ndarray           # int8 [rows, cols]
    scales: np.ndarray      # fp32 [rows]
    dictionary: Dictionary
    stream: np.ndarray      # uint16, interleaved and padded
    uoff: np.ndarray        # uint32 [n_units + 1], in chunks
    n_real_codes: int
    class_end: np.ndarray   # uint32 [4]: entries of at most 1, 2, 3, 4 bytes (the code space is sorted by run length)
    packing: int = 0        # 1: Q holds two 4-bit values per byte (pack_nibbles), the weight matrix is rows x 2 cols

    @property
    def pad_code(self) -> int:
        return self.dictionary.n_entries


def frequency_dictionary(S: np.ndarray, seg_len: np.ndarray, max_entries: int = 30719, lmax: int = 2) -> Dictionary:
    """Dictionary chosen by frequency, the way the paper's section 4 picks its table entries (most frequent sequences
    first; equally frequent ones in order of first appearance), for runs of 2: the 256 single bytes, then the most
    frequent pairs of neighbouring bytes, counted at every offset inside a segment and never across two segments, as
    many as max_entries leaves room for.  lmax 1: the singles alone."""
    assert lmax in (1, 2)
    S = np.ascontiguousarray(S, dtype=np.uint8)
    eb = np.zeros((256, LCAP), np.uint8)
    eb[:, 0] = np.arange(256)
    el = np.ones(256, np.uint8)
    room = max_entries - 256
    if lmax < 2 or room <= 0 or S.size < 2:
        return Dictionary(eb, el)
    inside = np.ones(S.size - 1, bool)                       # pair (i, i + 1) lies inside one segment
    ends = np.cumsum(np.asarray(seg_len, dtype=np.int64))
    cut = ends[(ends > 0) & (ends < S.size)]
    inside[cut - 1] = False
    keys = (S[:-1].astype(np.uint32) << 8 | S[1:])[inside]
    if keys.size == 0:
        return Dictionary(eb, el)
    uniq, first, count = np.unique(keys, return_index=True, return_counts=True)
    order = np.lexsort((first, -count.astype(np.int64)))[:room]
    pairs = np.zeros((order.size, LCAP), np.uint8)
    pairs[:, 0] = uniq[order] >> 8
    pairs[:, 1] = uniq[order] & 0xFF
    return Dictionary(np.concatenate([eb, pairs]), np.concatenate([el, np.full(order.size, 2, np.uint8)]))


def pack_nibbles(Q: np.ndarray) -> np.ndarray:
    """Two 4-bit values per byte: byte j of a row = (Q[r, 2j] mod 16) + 16 * (Q[r, 2j+1] mod 16), the values in 4-bit two's
    complement (-8..7).  Returned as int8 [rows, cols / 2]: the byte matrix that is then coded like any other."""
    Q = np.asarray(Q, dtype=np.int64)
    if Q.shape[1] % 2 or Q.min(initial=0) < -8 or Q.max(initial=0) > 7:
        raise ValueError("pack_nibbles: an even number of columns of values in [-8, 7]")
    lo, hi = Q[:, 0::2] % 16, Q[:, 1::2] % 16
    return (lo + 16 * hi).astype(np.uint8).view(np.int8)


def unpack_nibbles(P: np.ndarray) -> np.ndarray:
    """Inverse of pack_nibbles: int8 [rows, 2 * cols] from the byte matrix."""
    b = np.asarray(P).view(np.uint8).astype(np.int64)
    lo, hi = b % 16, b // 16
    Q = np.empty((b.shape[0], 2 * b.shape[1]), np.int64)
    Q[:, 0::2] = np.where(lo >= 8, lo - 16, lo)
    Q[:, 1::2] = np.where(hi >= 8, hi - 16, hi)
    return Q.astype(np.int8)


def encode_quantized(Q: np.ndarray, scales: np.ndarray, max_entries: int = 30719, lmax: int = 2,
                     seg_cols: int = DEFAULT_SEG_COLS, carry: "Dictionary | None" = None, dictionary: str = "lzw") -> Encoded:
    """dictionary "lzw": LZW growth with freeze (the paper's Background).  "frequency": the dictionary is fixed before
    the parse - the carried one if given, else frequency_dictionary of this matrix - and the parse is the same greedy
    longest match.  Runs are at most lmax <= 4 bytes; beyond 2 the dictionary also has to stay within UNIT_BUDGET."""
    assert 1 <= lmax <= 4
    budget = UNIT_BUDGET if lmax > 2 else 0
    rows, cols = Q.shape
    S, seg_len = serialize(Q, seg_cols)
    if dictionary == "frequency":
        fixed = carry if carry is not None else frequency_dictionary(S, seg_len, max_entries, lmax)
        codes, snc, d = lzw_encode(S, seg_len, fixed.n_entries, lmax, fixed)     # full from the start: nothing is added
        assert d.n_entries == fixed.n_entries
    else:
        assert dictionary == "lzw"
        codes, snc, d = lzw_encode(S, seg_len, max_entries, lmax, carry, budget)
    codes, d, class_end = sort_code_space(codes, d)
    stream, uoff = interleave(codes, snc, d.n_entries)
    return Encoded(rows, cols, seg_cols, lmax, max_entries, Q, np.asarray(scales, np.float32), d, stream, uoff,
                   int(codes.size), class_end)


def encode_matrix(W: np.ndarray, max_entries: int = 30719, lmax: int = 2, seg_cols: "int | None" = None,
                  carry: "Dictionary | None" = None, dictionary: str = "lzw", bits: int = 8, pack: bool = False) -> Encoded:
    """pack (widths of at most 4 bits): two values share a byte (pack_nibbles) and the byte matrix, half as wide, is what
    gets coded; seg_cols then counts bytes.  seg_cols None: 256, or 128 bytes (256 weights again) when packing."""
    if seg_cols is None:
        seg_cols = DEFAULT_SEG_COLS // 2 if pack else DEFAULT_SEG_COLS
    Q, s = quantize_rows(W, bits)
    if not pack:
        return encode_quantized(Q, s, max_entries, lmax, seg_cols, carry, dictionary)
    if bits > 4:
        raise ValueError("packing takes widths of at most 4 bits")
    e = encode_quantized(pack_nibbles(Q), s, max_entries, lmax, seg_cols, carry, dictionary)
    e.packing = 1
    return e


def dict_slots(d: Dictionary) -> np.ndarray:
    """Container dictionary words: the run's bytes, first byte lowest, unused bytes zero (the run's length follows from
    the code's place in the sorted code space); one extra all-zero word at index n_entries is the pad code's entry.
    Needs lmax <= 4."""
    assert int(d.ent_len.max()) <= 4
    eb = d.ent_bytes.astype(np.uint32)
    w = eb[:, 0] | (eb[:, 1] << 8) | (eb[:, 2] << 16) | (eb[:, 3] << 24)
    return np.concatenate([w, np.zeros(1, np.uint32)]).astype(np.uint32)


def _align(n: int, a: int = SECTION_ALIGN) -> int:
    return -(-n // a) * a


# magic, version, header_bytes | rows, cols | seg_cols, unit_rows, unit_panels, chunk_codes | n_bands, n_panels,
# n_quads | n_entries, lmax, max_entries, pad_code, packing | n_units, n_chunks, n_real_codes |
# (offset, size) of dictionary, unit offsets, codes, scales | total | class_end[4]
_HDR = struct.Struct("<8sII" "II" "IIII" "III" "IIIII" "QQQ" "QQ" "QQ" "QQ" "QQ" "Q" "IIII")


def build_blob(e: Encoded) -> bytes:
    n_bands, n_panels, n_quads = geometry(e.rows, e.cols, e.seg_cols)
    n_units = n_bands * n_quads
    slots = dict_slots(e.dictionary)
    scales = np.zeros(n_bands * UNIT_ROWS, np.float32)
    scales[: e.rows] = e.scales
    assert e.uoff.size == n_units + 1
    n_chunks = int(e.uoff[-1])
    assert e.stream.size == n_chunks * CHUNK_WORDS
    sec = [slots.tobytes(), e.uoff.astype(np.uint32).tobytes(), e.stream.astype(np.uint16).tobytes(), scales.tobytes()]
    offs, pos = [], HEADER_BYTES
    for b in sec:
        offs.append(pos)
        pos = _align(pos + len(b))
    total = pos
    hdr = _HDR.pack(MAGIC, 3, HEADER_BYTES, e.rows, e.cols, e.seg_cols, UNIT_ROWS, UNIT_PANELS, CHUNK_CODES,
                    n_bands, n_panels, n_quads, e.dictionary.n_entries, e.lmax, e.max_entries, e.pad_code, e.packing,
                    n_units, n_chunks, e.n_real_codes,
                    offs[0], len(sec[0]), offs[1], len(sec[1]), offs[2], len(sec[2]), offs[3], len(sec[3]), total,
                    *[int(c) for c in e.class_end])
    out = bytearray(total)
    out[: len(hdr)] = hdr
    for o, b in zip(offs, sec):
        out[o: o + len(b)] = b
    return bytes(out)


def parse_blob(blob: bytes) -> dict:
    (magic, version, hbytes, rows, cols, seg_cols, ur, up, cc, n_bands, n_panels, n_quads, n_entries, lmax,
     max_entries, pad_code, packing, n_units, n_chunks, n_real, o_d, b_d, o_u, b_u, o_c, b_c, o_s, b_s,
     total, ce0, ce1, ce2, ce3) = _HDR.unpack_from(blob, 0)
    assert magic == MAGIC and version == 3 and hbytes == HEADER_BYTES
    assert (ur, up, cc) == (UNIT_ROWS, UNIT_PANELS, CHUNK_CODES)
    assert (n_bands, n_panels, n_quads) == geometry(rows, cols, seg_cols) and n_units == n_bands * n_quads
    assert total == len(blob) and pad_code == n_entries and packing in (0, 1)
    buf = np.frombuffer(blob, dtype=np.uint8)
    slots = buf[o_d: o_d + b_d].view(np.uint32)
    uoff = buf[o_u: o_u + b_u].view(np.uint32)
    stream = buf[o_c: o_c + b_c].view(np.uint16)
    scales = buf[o_s: o_s + b_s].view(np.float32)
    assert slots.size == n_entries + 1 and uoff.size == n_units + 1 and stream.size == n_chunks * CHUNK_WORDS
    assert scales.size == n_bands * UNIT_ROWS and int(uoff[-1]) == n_chunks
    class_end = np.array([ce0, ce1, ce2, ce3], np.uint32)
    assert ce0 == 256 and ce0 <= ce1 <= ce2 <= ce3 == n_entries and 1 <= lmax <= 4 and class_end[lmax - 1] == n_entries
    code = np.arange(n_entries)
    el = (1 + (code >= ce0) + (code >= ce1) + (code >= ce2)).astype(np.uint8)      # the run length follows from the code
    eb = np.zeros((n_entries, LCAP), np.uint8)
    for k in range(4):
        eb[:, k] = (slots[:n_entries] >> (8 * k)) & 0xFF
    assert not np.any(eb[np.arange(LCAP)[None, :] >= el[:, None]])                   # nothing past an entry's length
    return dict(rows=rows, cols=cols, seg_cols=seg_cols, n_bands=n_bands, n_panels=n_panels, n_quads=n_quads,
                n_entries=n_entries, lmax=lmax, max_entries=max_entries, pad_code=pad_code, packing=packing, n_units=n_units,
                n_chunks=n_chunks, n_codes=n_chunks * CHUNK_WORDS, n_real_codes=n_real,
                dictionary=Dictionary(eb, el), class_end=class_end, slots=slots, uoff=uoff, stream=stream, scales=scales,
                compressed_bytes=int(b_d + b_u + b_c + b_s), stream_bytes=int(b_c))


def decode_blob(blob: bytes):
    """Container -> (Q int8 [rows, K], scales fp32 [rows]) through the oracle's own decoder; K is the header's cols, twice
    that for a container of packed 4-bit values."""
    p = parse_blob(blob)
    _, _, seg_len = segment_table(p["rows"], p["cols"], p["seg_cols"])
    S = lzw_decode(p["stream"], p["uoff"], seg_len.astype(np.uint32), p["dictionary"], p["pad_code"])
    Q = deserialize(S, p["rows"], p["cols"], p["seg_cols"])
    return (unpack_nibbles(Q) if p["packing"] else Q), p["scales"][: p["rows"]].copy()


def matvec_from_blob(blob: bytes, x: np.ndarray) -> np.ndarray:
    Q, s = decode_blob(blob)
    return gemv_f64(Q, s, x)
