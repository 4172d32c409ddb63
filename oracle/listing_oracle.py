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
    """Section 4, "Decompressing Model Weights", for one parameter.  Returns the uint8 values.

    Written as a whole-array computation rather than a reader that walks the words: a raw value is at most 0xFF and a
    codeword at most 0xFFFE (the reading above), so every word equal to the marker IS a marker, wherever it stands.
    The (up to) 4 words after a marker are raw values; every other word is a codeword and yields its table entry."""
    w = np.ascontiguousarray(words, dtype=np.uint16).astype(np.int64)
    t = np.ascontiguousarray(table, dtype=np.uint8).reshape(-1, SEQ)
    n = w.size
    pos = np.arange(n)
    markers = pos[w == MARKER]
    # how far behind the nearest earlier marker each word stands (0 = the marker itself; n = no marker before it)
    last = np.full(n, -1, np.int64)
    last[markers] = markers
    last = np.maximum.accumulate(last)
    behind = np.where(last >= 0, pos - last, n)
    assert markers.size < 2 or np.all(np.diff(markers) > SEQ), "a marker inside the raw values of another"
    raw = (behind >= 1) & (behind <= SEQ)
    code = ~raw & (w != MARKER)
    assert np.all(w[raw] <= 0xFF), "a raw value does not fit a byte"
    assert np.all((w[code] >= 1) & (w[code] <= t.shape[0])), "a codeword is not in the table"
    # values each word contributes, then their place in the output
    yields = np.where(raw, 1, np.where(code, SEQ, 0))
    start = np.cumsum(yields) - yields
    out = np.zeros(int(yields.sum()), np.uint8)
    out[start[raw]] = w[raw]
    if code.any():
        out[(start[code][:, None] + np.arange(SEQ)[None, :]).reshape(-1)] = t[w[code] - 1].reshape(-1)
    return out
