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


# ---- the library's host side against the oracle (no GPU) ----

import paper_2509_22951_amd as tq  # noqa: E402
from inputs import make_weights, small_case  # noqa: E402
from oracle import oracle as O  # noqa: E402


def _quantized_bytes(rows, cols, seed, dist="normal"):
    Q, _ = O.quantize_rows(make_weights(small_case(rows, cols, seed=seed, dist=dist)))
    return Q.view(np.uint8).reshape(-1)


@pytest.mark.parametrize("top_k", [0, 1, 7, 1000, 65534])
def test_library_table_and_stream_equal_the_oracles(top_k):
    rng = np.random.default_rng(11)
    params = [rng.integers(0, 3, size=5000, dtype=np.uint8), _quantized_bytes(64, 256, 5, "student_t4"), np.array([1, 2, 3], np.uint8),
              np.zeros(0, np.uint8), rng.integers(0, 2, size=1001, dtype=np.uint8)]
    want = L.build_table(params, top_k)
    got = tq.tq_listing_build_table(params, top_k)
    assert np.array_equal(got, want)
    for p in params:
        assert np.array_equal(tq.tq_listing_compress(p, got), L.compress(p, want))


def test_library_reproduces_the_hand_evaluated_example():
    values, entry, words, values2, table2 = _golden_lines()
    assert np.array_equal(tq.tq_listing_compress(values.astype(np.uint8), entry.astype(np.uint8).reshape(1, 4)), words.astype(np.uint16))
    assert np.array_equal(tq.tq_listing_build_table([values2.astype(np.uint8)], 3), table2.astype(np.uint8).reshape(3, 4))


def test_library_rejects_a_table_that_would_reach_the_markers_value():
    with pytest.raises(tq.TqError):
        tq.tq_listing_build_table([np.zeros(16, np.uint8)], 65535)
    with pytest.raises(tq.TqError):   # entries must be distinct
        tq.tq_listing_compress(np.zeros(8, np.uint8), np.zeros((2, 4), np.uint8))


def test_create_rejects_invalid_streams_before_touching_the_device():
    table = np.array([[1, 2, 3, 4]], np.uint8)
    for bad in ([2], [0], [0xFFFF], [1, 0xFFFF, 1, 2, 300, 4], [0xFFFF, 1, 0xFFFF, 1, 2]):   # the last: a marker where a raw value must be
        with pytest.raises(tq.TqError) as e:
            tq.Listing(np.array(bad, np.uint16), table)
        assert e.value.code == -2, bad


# ---- device decompression against the oracle ----

def _gpu_round_trip(values, table, dev, misalign=False):
    import torch
    words = L.compress(values, table)                      # the oracle's stream goes to the device
    assert np.array_equal(tq.tq_listing_compress(values, table), words)
    h = tq.Listing(words, table)
    try:
        assert h.info["n_values"] == values.size and h.info["n_words"] == words.size
        assert h.info["n_escapes"] == int(np.sum(words == 0xFFFF))
        buf = torch.full((values.size + 16,), 0xAB, dtype=torch.uint8, device=dev)
        off = 1 if misalign else 0
        out = buf[off: off + values.size]
        h.decompress(out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got = buf.cpu().numpy()
        assert np.array_equal(got[off: off + values.size], values)          # section 4: exactly the original values
        assert np.all(got[:off] == 0xAB) and np.all(got[off + values.size:] == 0xAB)   # nothing outside is written
    finally:
        h.close()


@pytest.mark.gpu
@pytest.mark.parametrize("n,alphabet,top_k", [(0, 2, 10), (1, 2, 10), (3, 2, 10), (4, 2, 10), (4099, 2, 3), (100001, 3, 40), (300002, 4, 65534),
                                              (65536, 256, 100), (1 << 20, 2, 65534)])
def test_device_decompression_is_exact(n, alphabet, top_k):
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(n + alphabet)
    values = rng.integers(0, alphabet, size=n, dtype=np.uint8)
    table = L.build_table([values], top_k)
    _gpu_round_trip(values, table, dev)
    _gpu_round_trip(values, table, dev, misalign=True)
    _gpu_round_trip(values, np.zeros((0, 4), np.uint8), dev)    # no table at all: every group escaped


@pytest.mark.gpu
def test_device_decompression_of_quantized_weights():
    """The benchmark's weight distributions through the listings' format: Gaussian int8 weights hardly ever repeat a
    window of 4, so nearly every group is escaped; Student-t weights hit the table more often."""
    import torch
    dev = torch.device("cuda:0")
    for dist in ("normal", "student_t4"):
        values = _quantized_bytes(512, 2048, 21, dist)
        table = tq.tq_listing_build_table([values])
        assert np.array_equal(table, L.build_table([values]))
        _gpu_round_trip(values, table, dev)
