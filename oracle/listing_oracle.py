"""CPU oracle for the stream format the paper's section 4 listings define ("listing format").

TEST INFRASTRUCTURE ONLY.  Imported by tests/ only; the product package never imports it and the two share no code.

What the listings of section 4 compute, restated:

* Table ("Finding Frequent Sequences"): every window of 4 consecutive byte values of every parameter, taken at every
  offset (stride 1) and never across two parameters, is counted; the ``top_k`` most frequent windows, most frequent
  first and, among equally frequent ones, in order of first appearance (parameters in their given order), get the
  codewords 1, 2, 3, ...
* Compression ("Compressing Model Weights"), per parameter, a sequence of 16-bit words: the values are cut into
  groups of 4 from the start (stride 4); a group that is in the table becomes its codeword; any other group becomes
  the marker 0xFFFF followed by its 4 values, one word each; fewer than 4 values left over at the end become the
  marker followed by those values.
* Decompression ("Decompressing Model Weights"): words are read in order; a codeword yields its table entry; the
  marker yields the next (up to) 4 words as values.  The output equals the input values exactly (section 4).

Reading taken where the listings collide with themselves: with the printed default ``top_k = 2**16 - 1`` the last
codeword would be 65535 = 0xFFFF, the marker.  Here ``top_k`` is at most 65534, so no codeword equals the marker;
codeword 0 is never assigned and never valid.

Pins (tests/test_listing_format.py): a hand-evaluated example of the three listings, the window-count ranking of a
hand-counted input, closed forms (all values equal; no group in the table), round-trip identity, and a brute-force
word-by-word reader on small random inputs.  No function here is unpinned.
"""
from __future__ import annotations

import numpy as np

SEQ = 4                 # values per table entry (the listings' sequence_length)
MARKER = 0xFFFF         # "what follows is raw" (the listings' special codeword)
MAX_TOP_K = 0xFFFE      # largest table that keeps every codeword different from the marker


def _keys(values: np.ndarray) -> np.ndarray:
    """The windows of 4 consecutive values at every offset, each as one integer (first value in the low byte)."""
    v = np.ascontiguousarray(values, dtype=np.uint8).astype(np.uint32)
    if v.size < SEQ:
        return np.zeros(0, np.uint32)
    n = v.size - SEQ + 1
    return v[0:n] | v[1:n + 1] << 8 | v[2:n + 2] << 16 | v[3:n + 3] << 24


def build_table(params, top_k: int = MAX_TOP_K) -> np.ndarray:
    """Section 4, first listing.  params: sequence of uint8 arrays.  Returns uint8 [n, 4]: row i is codeword i + 1."""
    assert 0 <= top_k <= MAX_TOP_K
    keys = np.concatenate([_keys(p) for p in params]) if len(params) else np.zeros(0, np.uint32)
    if keys.size == 0 or top_k == 0:
        return np.zeros((0, SEQ), np.uint8)
    uniq, first, count = np.unique(keys, return_index=True, return_counts=True)
    order = np.lexsort((first, -count.astype(np.int64)))[:top_k]      # most frequent first, then first seen first
    chosen = uniq[order]
    return np.stack([(chosen >> (8 * k)) & 0xFF for k in range(SEQ)], axis=1).astype(np.uint8)


def compress(values: np.ndarray, table: np.ndarray) -> np.ndarray:
    """Section 4, second listing, for one parameter.  Returns the uint16 words."""
    v = np.ascontiguousarray(values, dtype=np.uint8)
    n_groups, tail = divmod(v.size, SEQ)
    groups = v[: n_groups * SEQ].reshape(n_groups, SEQ).astype(np.uint32)
    gkeys = groups[:, 0] | groups[:, 1] << 8 | groups[:, 2] << 16 | groups[:, 3] << 24
    t = np.ascontiguousarray(table, dtype=np.uint8).astype(np.uint32).reshape(-1, SEQ)
    tkeys = t[:, 0] | t[:, 1] << 8 | t[:, 2] << 16 | t[:, 3] << 24
    code_of = {int(k): i + 1 for i, k in enumerate(tkeys)}
    assert len(code_of) == tkeys.size, "table entries must be distinct"
    out = []
    for g, k in zip(groups, gkeys):
        c = code_of.get(int(k))
        if c is None:
            out.append(MARKER)
            out.extend(int(x) for x in g)
        else:
            out.append(c)
    if tail:
        out.append(MARKER)
        out.extend(int(x) for x in v[n_groups * SEQ:])
    return np.array(out, dtype=np.uint16)


def decompress(words: np.ndarray, table: np.ndarray) -> np.ndarray:
    """Section 4, third listing, for one parameter.  Returns the uint8 values."""
    w = np.ascontiguousarray(words, dtype=np.uint16)
    t = np.ascontiguousarray(table, dtype=np.uint8).reshape(-1, SEQ)
    out = []
    i = 0
    while i < w.size:
        c = int(w[i])
        i += 1
        if c == MARKER:
            raw = w[i: i + SEQ]
            assert np.all(raw <= 0xFF), "a raw value does not fit a byte"
            out.extend(int(x) for x in raw)
            i += SEQ
        else:
            assert 1 <= c <= t.shape[0], f"codeword {c} is not in the table"
            out.extend(int(x) for x in t[c - 1])
    return np.array(out, dtype=np.uint8)
