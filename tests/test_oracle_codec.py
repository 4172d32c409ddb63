"""Pins for the oracle's LZW codec (paper Background, "Compression"; section 4 exact reconstruction)."""
import os

import numpy as np
import pytest

from inputs import make_weights, small_case
from oracle import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force_lzw(S: bytes, group_bytes: int, max_entries: int, lmax: int, entries=None, unit_budget: int = 0):
    """Independent restatement used only as a pin: the dictionary is a plain Python list of byte strings and
    the longest match is found by trying every entry at every position (no trie, no incremental walk).
    unit_budget (0 = none): an entry is added only if the dictionary then takes at most that many units, entries of up
    to 2 bytes counting 1 and longer ones 2."""
    entries = [bytes([b]) for b in range(256)] if entries is None else list(entries)

    def units(es):
        return sum(1 if len(e) <= 2 else 2 for e in es)
    codes, per_group = [], []
    for gs in range(0, len(S), group_bytes):
        ge = min(gs + group_bytes, len(S))
        i, cnt = gs, 0
        while i < ge:
            best = None
            for code, ent in enumerate(entries):
                if len(ent) <= lmax and S[i:i + len(ent)] == ent and i + len(ent) <= ge:
                    if best is None or len(ent) > len(entries[best]):
                        best = code
            m = len(entries[best])
            codes.append(best)
            cnt += 1
            if len(entries) < max_entries and m < lmax and i + m < ge:
                if not unit_budget or units(entries + [S[i:i + m + 1]]) <= unit_budget:
                    entries.append(S[i:i + m + 1])
            i += m
        per_group.append(cnt)
    return codes, per_group, entries


def test_published_worked_example():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "lzw_classic_example.txt")) if l.strip() and not l.startswith("#")]
    text, want = lines[0].encode(), [int(t) for t in lines[1].split()]
    codes, gnc, d = O.lzw_encode(np.frombuffer(text, np.uint8), seg_len=1 << 20, max_entries=65536, lmax=16)
    assert codes.tolist() == want
    assert d.n_entries == 271
    assert d.entry(256) == b"TO" and d.entry(265) == b"TOB" and d.entry(268) == b"TOBE" and d.entry(270) == b"RNO"


def test_triangular_growth_on_equal_bytes():
    # six equal bytes: phrases of length 1, 2, 3 (the classic triangular growth)
    codes, gnc, d = O.lzw_encode(np.full(6, 1, np.uint8), seg_len=64, max_entries=65536, lmax=8)
    assert codes.tolist() == [1, 256, 257]
    assert [d.entry(c) for c in (256, 257)] == [b"\x01\x01", b"\x01\x01\x01"]


@pytest.mark.parametrize("lmax", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("group", [64, 100, 4096])
def test_all_zero_closed_form(lmax, group):
    n = 3 * group + 17
    codes, gnc, d = O.lzw_encode(np.zeros(n, np.uint8), seg_len=group, max_entries=65536, lmax=lmax)
    # closed form: first group grows 1,2,..,lmax then stays at lmax with a remainder run; later groups use lmax runs
    exp_lens = []
    have = 1  # longest all-zero phrase in the dictionary
    for gs in range(0, n, group):
        left = min(group, n - gs)
        while left > 0:
            m = min(have, left, lmax)
            exp_lens.append(m)
            if m == have and have < lmax and left - m > 0:
                have += 1
            left -= m
    got_lens = [len(d.entry(c)) for c in codes]
    assert got_lens == exp_lens
    assert all(set(d.entry(c)) == {0} for c in codes)
    assert d.n_entries == 256 + lmax - 1      # 00, 000, ... up to lmax zeros (first group is long enough)
    assert int(gnc.sum()) == codes.size


@pytest.mark.parametrize("seed", range(6))
def test_against_brute_force_small_alphabet(seed):
    rng = np.random.default_rng(seed)
    alphabet = np.array([0, 1, 255, 128][: 2 + seed % 3], np.uint8)
    n = int(rng.integers(40, 400))
    S = alphabet[rng.integers(0, alphabet.size, n)]
    group = int(rng.choice([16, 37, 128]))
    lmax = int(rng.choice([2, 3, 4, 8]))
    max_entries = int(rng.choice([258, 262, 300, 65536]))
    codes, gnc, d = O.lzw_encode(S, seg_len=group, max_entries=max_entries, lmax=lmax)
    bc, bg, be = brute_force_lzw(S.tobytes(), group, max_entries, lmax)
    assert codes.tolist() == bc
    assert gnc.tolist() == bg
    # the same input cut into ragged segments given one by one
    seg_len = []
    left = n
    while left:
        seg_len.append(min(left, int(rng.integers(0, 40))))
        left -= seg_len[-1]
    codes2, snc2, d2 = O.lzw_encode(S, seg_len=np.array(seg_len, np.uint32), max_entries=max_entries, lmax=lmax)
    entries = [bytes([b]) for b in range(256)]
    want, pos = [], 0
    for L in seg_len:      # brute force segment by segment, carrying the entries
        c, _, entries = brute_force_lzw(S.tobytes()[pos:pos + L], max(L, 1), max_entries, lmax, entries=entries)
        want.append(c)
        pos += L
    assert codes2.tolist() == [c for seg in want for c in seg] and snc2.tolist() == [len(c) for c in want]
    assert [d.entry(e) for e in range(d.n_entries)] == be


def test_freeze_when_full_and_no_reset():
    rng = np.random.default_rng(7)
    S = rng.integers(0, 256, 20000, dtype=np.uint8)
    codes, gnc, d = O.lzw_encode(S, seg_len=4096, max_entries=300, lmax=3)
    assert d.n_entries == 300            # filled, then frozen
    assert int(codes.max()) < 300
    # entries were created by the first 44 codes only (one entry per code while not full)
    first = O.lzw_encode(S[:200], seg_len=4096, max_entries=300, lmax=3)[2]
    assert [first.entry(e) for e in range(300)] == [d.entry(e) for e in range(300)]


def _ragged_segments(rng, n_segs, lo, hi, empty_every=0):
    seg_len = rng.integers(lo, hi, n_segs).astype(np.uint32)
    if empty_every:
        seg_len[::empty_every] = 0
    return seg_len


@pytest.mark.parametrize("lmax,max_entries", [(3, 32000), (3, 4096), (8, 65536), (2, 1000), (2, 30719)])
def test_round_trip_identity(lmax, max_entries):
    rng = np.random.default_rng(11)
    seg_len = _ragged_segments(rng, 300, 1, 400, empty_every=7)        # 4 full units and a ragged fifth one
    S = np.clip(np.rint(rng.standard_normal(int(seg_len.sum())) * 35), -127, 127).astype(np.int8).view(np.uint8)
    codes, snc, d = O.lzw_encode(S, seg_len=seg_len, max_entries=max_entries, lmax=lmax)
    assert np.all(snc[seg_len == 0] == 0)
    stream, uoff = O.interleave(codes, snc, d.n_entries)
    assert uoff.size == 5 + 1 and stream.size == int(uoff[-1]) * O.CHUNK_WORDS
    back = O.lzw_decode(stream, uoff, seg_len, d, d.n_entries)
    assert np.array_equal(back, S)
    # matches never cross a segment end: every segment decodes to exactly its own bytes (checked inside
    # lzw_decode) and no run is longer than lmax
    assert int(d.ent_len.max()) <= lmax


def test_interleave_layout_by_hand():
    """Three segments with 5, 0 and 2 codes: one unit of two chunks; lane l's code k sits at (k // 4) * 256 + 4 l + k % 4,
    everything else is the pad code."""
    codes = np.array([10, 11, 12, 13, 14, 20, 21], np.uint16)
    stream, uoff = O.interleave(codes, np.array([5, 0, 2], np.uint32), pad_code=999)
    assert uoff.tolist() == [0, 2] and stream.size == 512
    want = np.full(512, 999, np.uint16)
    want[0:4] = [10, 11, 12, 13]
    want[256] = 14
    want[8:10] = [20, 21]
    assert np.array_equal(stream, want)


def test_decode_rejects_inconsistent_stream():
    S = np.arange(256, dtype=np.uint8).repeat(2)
    seg_len = np.full(4, 128, np.uint32)
    codes, snc, d = O.lzw_encode(S, seg_len=seg_len, max_entries=400, lmax=3)
    stream, uoff = O.interleave(codes, snc, d.n_entries)
    bad = stream.copy()
    bad[0] = d.n_entries + 5           # not an entry and not the pad code
    with pytest.raises(ValueError):
        O.lzw_decode(bad, uoff, seg_len, d, d.n_entries)
    bad = stream.copy()
    bad[1] = d.n_entries               # a pad code before real codes
    with pytest.raises(ValueError):
        O.lzw_decode(bad, uoff, seg_len, d, d.n_entries)
    wrong = seg_len.copy()
    wrong[0] -= 1                      # segment 0 now decodes to one byte too many
    with pytest.raises(ValueError):
        O.lzw_decode(stream, uoff, wrong, d, d.n_entries)
    assert np.array_equal(O.lzw_decode(stream, uoff, seg_len, d, d.n_entries), S)
    # Padding only ever ends a lane stream: a real code after a pad code is an error even when the lengths still add up.
    two = np.array([7, 9], np.uint8)
    codes, snc, d = O.lzw_encode(two, seg_len=np.array([2], np.uint32), max_entries=256, lmax=2)
    stream, uoff = O.interleave(codes, snc, d.n_entries)
    assert list(stream[:4]) == [7, 9, 256, 256] and np.array_equal(O.lzw_decode(stream, uoff, [2], d, 256), two)
    stream[:4] = [7, 256, 9, 256]
    with pytest.raises(ValueError):
        O.lzw_decode(stream, uoff, [2], d, 256)


def test_dictionary_carried_over_equals_one_run_over_the_concatenation():
    """LZW state is only the dictionary, so encoding B with the dictionary A left behind gives the codes that
    encoding A followed by B in one go gives for B (section 4 builds one table over all parameters)."""
    rng = np.random.default_rng(21)
    A = rng.integers(0, 7, 3000).astype(np.uint8)
    B = rng.integers(0, 7, 2000).astype(np.uint8)
    for max_entries, lmax in ((400, 3), (65536, 4), (300, 2)):
        ca, _, da = O.lzw_encode(A, seg_len=100, max_entries=max_entries, lmax=lmax)
        cb, _, db = O.lzw_encode(B, seg_len=100, max_entries=max_entries, lmax=lmax, carry=da)
        call, _, dall = O.lzw_encode(np.concatenate([A, B]), seg_len=100, max_entries=max_entries, lmax=lmax)
        assert np.array_equal(np.concatenate([ca, cb]), call)
        assert [db.entry(e) for e in range(db.n_entries)] == [dall.entry(e) for e in range(dall.n_entries)]
        # and against the brute-force parser started from A's entries
        bc, _, be = brute_force_lzw(B.tobytes(), 100, max_entries, lmax, entries=[da.entry(e) for e in range(da.n_entries)])
        assert cb.tolist() == bc and [db.entry(e) for e in range(db.n_entries)] == be


def test_singles_only_dictionary_is_identity_code():
    rng = np.random.default_rng(3)
    S = rng.integers(0, 256, 5000, dtype=np.uint8)
    codes, gnc, d = O.lzw_encode(S, seg_len=4096, max_entries=256, lmax=3)
    assert np.array_equal(codes, S.astype(np.uint16))     # code == byte
    codes1, _, _ = O.lzw_encode(S, seg_len=4096, max_entries=65536, lmax=1)
    assert np.array_equal(codes1, S.astype(np.uint16))


def test_information_bound_on_iid_input():
    """A lossless coder cannot beat the zeroth-order entropy on i.i.d. symbols: 16 bits per code must carry
    at most 16/H symbols on average (finite-sample slack 2 %)."""
    rng = np.random.default_rng(5)
    S = np.clip(np.rint(rng.standard_normal(1 << 20) * 34.0), -127, 127).astype(np.int8).view(np.uint8)
    p = np.bincount(S, minlength=256) / S.size
    H = -(p[p > 0] * np.log2(p[p > 0])).sum()
    for max_entries in (32000, 65536):
        codes, gnc, d = O.lzw_encode(S, seg_len=4096, max_entries=max_entries, lmax=3)
        sym_per_code = S.size / codes.size
        assert sym_per_code < 16.0 / H * 1.02
        assert sym_per_code > 1.5          # and it does find pairs


# ---- dictionary picked by frequency (how the paper's section 4 picks its table), runs of 2 ----

def _pairs_of(d):
    return [tuple(int(x) for x in d.ent_bytes[e, :2]) for e in range(256, d.n_entries)]


def test_frequency_dictionary_on_hand_counted_input():
    # one segment 1 2 1 2 1 2 3 1 2: (1,2) x4, (2,1) x2, (2,3) x1, (3,1) x1
    S = np.array([1, 2, 1, 2, 1, 2, 3, 1, 2], np.uint8)
    d = O.frequency_dictionary(S, np.array([9], np.uint32), max_entries=300)
    assert d.n_entries == 260 and np.all(d.ent_len[:256] == 1) and np.all(d.ent_len[256:] == 2)
    assert [d.entry(e) for e in (0, 65, 255)] == [b"\x00", b"A", b"\xff"]
    assert _pairs_of(d) == [(1, 2), (2, 1), (2, 3), (3, 1)]
    assert _pairs_of(O.frequency_dictionary(S, np.array([9], np.uint32), max_entries=258)) == [(1, 2), (2, 1)]
    assert O.frequency_dictionary(S, np.array([9], np.uint32), max_entries=256).n_entries == 256
    assert O.frequency_dictionary(S, np.array([9], np.uint32), max_entries=300, lmax=1).n_entries == 256
    # with the two best pairs the greedy parse is 12 12 12 3 12 (hand-derived)
    e = O.encode_quantized(S.view(np.int8).reshape(1, 9), np.ones(1, np.float32), max_entries=258, seg_cols=16, dictionary="frequency")
    codes = e.stream.reshape(-1, 64, 4)[:, 0, :].reshape(-1)          # lane 0 holds the only segment
    assert codes[: e.n_real_codes].tolist() == [256, 256, 256, 3, 256]


def test_frequency_dictionary_never_counts_across_segments_and_breaks_ties_by_first_appearance():
    # segments 1 2 1 | 2 1 2: inside them (1,2) (2,1) | (2,1) (1,2); the pair (1,2) across the cut is not counted
    S = np.array([1, 2, 1, 2, 1, 2], np.uint8)
    assert _pairs_of(O.frequency_dictionary(S, np.array([3, 3], np.uint32), 300)) == [(1, 2), (2, 1)]
    # as one segment the same bytes give (1,2) x3, (2,1) x2
    assert _pairs_of(O.frequency_dictionary(S, np.array([6], np.uint32), 300)) == [(1, 2), (2, 1)]
    S = np.array([7, 7, 9, 9, 7, 7], np.uint8)
    assert _pairs_of(O.frequency_dictionary(S, np.array([2, 2, 2], np.uint32), 300)) == [(7, 7), (9, 9)]
    assert _pairs_of(O.frequency_dictionary(S, np.array([0, 6, 0], np.uint32), 300)) == [(7, 7), (7, 9), (9, 9), (9, 7)]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_frequency_dictionary_against_a_counting_loop(seed):
    rng = np.random.default_rng(seed)
    seg_len = rng.integers(0, 9, size=40).astype(np.uint32)
    S = rng.integers(0, 4, size=int(seg_len.sum()), dtype=np.uint8)
    count, first, pos, t = {}, {}, 0, 0
    for n in seg_len:
        seg = S[pos: pos + n]
        for a, b in zip(seg[:-1], seg[1:]):
            k = (int(a), int(b))
            count[k] = count.get(k, 0) + 1
            first.setdefault(k, t)
            t += 1
        pos += int(n)
    want = sorted(count, key=lambda k: (-count[k], first[k]))
    for room in (0, 3, 100):
        assert _pairs_of(O.frequency_dictionary(S, seg_len, 256 + room)) == want[:room]


def test_frequency_dictionary_round_trip_and_gain_over_lzw():
    W = make_weights(small_case(256, 2048, seed=12))
    Q, s = O.quantize_rows(W)
    f = O.encode_quantized(Q, s, dictionary="frequency")
    l = O.encode_quantized(Q, s, dictionary="lzw")
    S, seg_len = O.serialize(Q)
    assert np.array_equal(O.lzw_decode(f.stream, f.uoff, seg_len, f.dictionary, f.pad_code), S)
    assert f.dictionary.n_entries == 30719 and f.n_real_codes < l.n_real_codes       # the better-chosen pairs cover more


def test_unit_budget_closed_form_on_equal_bytes():
    """20 zero bytes, runs of up to 4: LZW wants to add 00 (1 unit), 000 (2 units), 0000 (2 units) on top of the 256
    units of the single bytes.  Budget 261 or none: all three, runs 1 2 3 4 4 4 2.  Budget 259: 0000 does not fit, runs
    1 2 3 3 3 3 3 2.  Budget 258: 000 does not fit either (and is offered again at every later match of 00, in vain):
    runs 1 2 2 ... 2 1.  Budget 256: nothing but the single bytes."""
    S = np.zeros(20, np.uint8)
    for budget, want_entries, want_runs in ((0, 259, [1, 2, 3, 4, 4, 4, 2]), (261, 259, [1, 2, 3, 4, 4, 4, 2]),
                                            (260, 258, [1, 2, 3, 3, 3, 3, 3, 2]), (259, 258, [1, 2, 3, 3, 3, 3, 3, 2]),
                                            (258, 257, [1] + [2] * 9 + [1]), (256, 256, [1] * 20)):
        codes, _, d = O.lzw_encode(S, seg_len=64, max_entries=65536, lmax=4, unit_budget=budget)
        assert d.n_entries == want_entries, budget
        assert [int(d.ent_len[c]) for c in codes] == want_runs, budget


def test_unit_budget_against_the_brute_force_parser():
    rng = np.random.default_rng(77)
    for _ in range(12):
        n = int(rng.integers(50, 400))
        S = rng.integers(0, int(rng.choice([2, 3, 5])), n).astype(np.uint8)
        group = int(rng.choice([7, 16, 64, 1000]))
        lmax = int(rng.choice([3, 4]))
        budget = 256 + int(rng.integers(0, 40))
        max_entries = int(rng.choice([262, 280, 65536]))
        codes, gnc, d = O.lzw_encode(S, seg_len=group, max_entries=max_entries, lmax=lmax, unit_budget=budget)
        bc, bg, be = brute_force_lzw(S.tobytes(), group, max_entries, lmax, unit_budget=budget)
        assert list(codes) == bc and list(gnc) == bg
        assert [d.entry(e) for e in range(d.n_entries)] == be
        assert sum(1 if len(e) <= 2 else 2 for e in be) <= budget


def test_sorted_code_space_hand_example():
    """"aaabaabab", runs of up to 4, one segment, by hand: a | aa | b | aab | a | b with the entries created in the order
    256 aa, 257 aab, 258 ba, 259 aaba, 260 ab.  Sorted by length, equal lengths in order of creation: 256 aa, 257 ba,
    258 ab, 259 aab, 260 aaba, so the stream 97 256 98 257 97 98 becomes 97 256 98 259 97 98."""
    S = np.frombuffer(b"aaabaabab", np.uint8)
    codes, _, d = O.lzw_encode(S, seg_len=64, max_entries=65536, lmax=4)
    assert list(codes) == [97, 256, 98, 257, 97, 98]
    assert [d.entry(e) for e in range(256, d.n_entries)] == [b"aa", b"aab", b"ba", b"aaba", b"ab"]
    codes2, d2, class_end = O.sort_code_space(codes, d)
    assert list(codes2) == [97, 256, 98, 259, 97, 98]
    assert [d2.entry(e) for e in range(256, d2.n_entries)] == [b"aa", b"ba", b"ab", b"aab", b"aaba"]
    assert list(class_end) == [256, 259, 260, 261]
    assert all(d2.entry(b) == bytes([b]) for b in range(256))


def test_sorted_code_space_is_a_relabelling():
    """The renumbered stream with the reordered dictionary spells the same bytes; lengths never decrease along the code
    space; every entry of two or more bytes still follows the entry it extends (what lets a later matrix go on from it)."""
    rng = np.random.default_rng(5)
    S = rng.integers(0, 4, 3000).astype(np.uint8)
    seg_len = np.full(30, 100, np.uint32)
    codes, snc, d = O.lzw_encode(S, seg_len=seg_len, max_entries=700, lmax=4, unit_budget=900)
    codes2, d2, class_end = O.sort_code_space(codes, d)
    assert b"".join(d.entry(c) for c in codes) == b"".join(d2.entry(c) for c in codes2) == S.tobytes()
    assert np.all(np.diff(d2.ent_len.astype(int)) >= 0) and class_end[3] == d2.n_entries and class_end[0] == 256
    where = {d2.entry(e): e for e in range(d2.n_entries)}
    assert all(where[d2.entry(e)[:-1]] < e for e in range(256, d2.n_entries))
    again = O.lzw_encode(S, seg_len=seg_len, max_entries=700, lmax=4, carry=d2, unit_budget=900)   # a carried, sorted dictionary
    assert again[2].n_entries >= d2.n_entries
    stream, uoff = O.interleave(codes2, snc, d2.n_entries)
    assert np.array_equal(O.lzw_decode(stream, uoff, seg_len, d2, d2.n_entries), S)
