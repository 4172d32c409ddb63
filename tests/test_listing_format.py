"""Pins of the listing-format oracle (paper section 4) and, further down, the library's host side against it."""
import os

import numpy as np
import pytest

from oracle import listing_oracle as L

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "listing_hand_example.txt")


def _golden_lines():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    return [np.array([int(x) for x in r]) for r in rows]


def test_hand_evaluated_example_of_the_three_listings():
    values, entry, words, _, _ = _golden_lines()
    table = entry.astype(np.uint8).reshape(1, 4)
    assert np.array_equal(L.compress(values.astype(np.uint8), table), words.astype(np.uint16))
    assert np.array_equal(L.decompress(words.astype(np.uint16), table), values.astype(np.uint8))


def test_window_counts_rank_by_frequency_then_first_appearance():
    _, _, _, values, want = _golden_lines()
    assert np.array_equal(L.build_table([values.astype(np.uint8)], top_k=3), want.astype(np.uint8).reshape(3, 4))
    # windows never span two parameters: cutting the input in two removes the windows across the cut
    a, b = values[:5].astype(np.uint8), values[5:].astype(np.uint8)
    t = L.build_table([a, b], top_k=10)
    assert [tuple(r) for r in t] == [(1, 2, 3, 4), (2, 3, 4, 1), (2, 3, 4, 9)]


def test_closed_forms():
    # all values equal, length a multiple of 4, that window in the table: one codeword per group
    v = np.full(40, 77, np.uint8)
    t = L.build_table([v])
    assert t.tolist() == [[77, 77, 77, 77]]
    assert L.compress(v, t).tolist() == [1] * 10
    # empty table: every group costs 5 words, a tail of k values k + 1
    v = np.arange(11, dtype=np.uint8)
    w = L.compress(v, np.zeros((0, 4), np.uint8))
    assert w.size == 5 + 5 + 4 and w[0] == 0xFFFF and w[5] == 0xFFFF and w[10] == 0xFFFF
    assert w[[1, 2, 3, 4, 6, 7, 8, 9, 11, 12, 13]].tolist() == list(range(11))
    assert L.compress(np.zeros(0, np.uint8), t).size == 0


def _read_word_by_word(words, table):
    """Brute force: a reader with an explicit two-state machine, no slicing."""
    out, raw_left = [], 0
    for w in words.tolist():
        if raw_left:
            out.append(w)
            raw_left -= 1
        elif w == 0xFFFF:
            raw_left = 4
        else:
            out.extend(table[w - 1].tolist())
    return np.array(out, np.uint8)


@pytest.mark.parametrize("seed,n,alphabet,top_k", [(0, 1, 3, 4), (1, 3, 2, 100), (2, 64, 2, 5), (3, 257, 3, 20), (4, 1000, 4, 65534),
                                                   (5, 4096, 256, 50)])
def test_round_trip_and_brute_force_reader(seed, n, alphabet, top_k):
    rng = np.random.default_rng(seed)
    params = [rng.integers(0, alphabet, size=m, dtype=np.uint8) for m in (n, max(n // 3, 1), 7)]
    table = L.build_table(params, top_k)
    assert table.shape[0] <= top_k and len({tuple(r) for r in table}) == table.shape[0]
    for p in params:
        w = L.compress(p, table)
        assert np.array_equal(L.decompress(w, table), p)            # section 4: reconstructed exactly
        assert np.array_equal(_read_word_by_word(w, table), p)
        groups, tail = divmod(p.size, 4)
        hits = int(np.sum((w != 0xFFFF) & ~_covered(w)))
        assert w.size == hits + 5 * (groups - hits) + (tail + 1 if tail else 0)


def _covered(w):
    """Words that are raw values: the up to 4 words after each marker."""
    c = np.zeros(w.size, bool)
    for i in np.flatnonzero(w == 0xFFFF):
        c[i + 1: i + 5] = True
    return c
