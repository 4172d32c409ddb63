"""Pins for the oracle's LZW codec (paper Background, "Compression"; section 4 exact reconstruction)."""
import os

import numpy as np
import pytest

from oracle import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force_lzw(S: bytes, group_bytes: int, max_entries: int, lmax: int):
    """Independent restatement used only as a pin: the dictionary is a plain Python list of byte strings and
    the longest match is found by trying every entry at every position (no trie, no incremental walk)."""
    entries = [bytes([b]) for b in range(256)]
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
                entries.append(S[i:i + m + 1])
            i += m
        per_group.append(cnt)
    return codes, per_group, entries


def test_published_worked_example():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "lzw_classic_example.txt")) if l.strip() and not l.startswith("#")]
    text, want = lines[0].encode(), [int(t) for t in lines[1].split()]
    codes, gnc, d = O.lzw_encode(np.frombuffer(text, np.uint8), group_bytes=1 << 20, max_entries=65536, lmax=16)
    assert codes.tolist() == want
    assert d.n_entries == 271
    assert d.entry(256) == b"TO" and d.entry(265) == b"TOB" and d.entry(268) == b"TOBE" and d.entry(270) == b"RNO"


def test_triangular_growth_on_equal_bytes():
    # six equal bytes: phrases of length 1, 2, 3 (the classic triangular growth)
    codes, gnc, d = O.lzw_encode(np.full(6, 1, np.uint8), group_bytes=64, max_entries=65536, lmax=8)
    assert codes.tolist() == [1, 256, 257]
    assert [d.entry(c) for c in (256, 257)] == [b"\x01\x01", b"\x01\x01\x01"]


@pytest.mark.parametrize("lmax", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("group", [64, 100, 4096])
def test_all_zero_closed_form(lmax, group):
    n = 3 * group + 17
    codes, gnc, d = O.lzw_encode(np.zeros(n, np.uint8), group_bytes=group, max_entries=65536, lmax=lmax)
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
    codes, gnc, d = O.lzw_encode(S, group_bytes=group, max_entries=max_entries, lmax=lmax)
    bc, bg, be = brute_force_lzw(S.tobytes(), group, max_entries, lmax)
    assert codes.tolist() == bc
    assert gnc.tolist() == bg
    assert [d.entry(e) for e in range(d.n_entries)] == be


def test_freeze_when_full_and_no_reset():
    rng = np.random.default_rng(7)
    S = rng.integers(0, 256, 20000, dtype=np.uint8)
    codes, gnc, d = O.lzw_encode(S, group_bytes=4096, max_entries=300, lmax=3)
    assert d.n_entries == 300            # filled, then frozen
    assert int(codes.max()) < 300
    # entries were created by the first 44 codes only (one entry per code while not full)
    first = O.lzw_encode(S[:200], group_bytes=4096, max_entries=300, lmax=3)[2]
    assert [first.entry(e) for e in range(300)] == [d.entry(e) for e in range(300)]


@pytest.mark.parametrize("lmax,max_entries", [(3, 32000), (3, 4096), (8, 65536), (2, 1000)])
def test_round_trip_identity(lmax, max_entries):
    rng = np.random.default_rng(11)
    S = np.clip(np.rint(rng.standard_normal(70000) * 35), -127, 127).astype(np.int8).view(np.uint8)
    codes, gnc, d = O.lzw_encode(S, group_bytes=4096, max_entries=max_entries, lmax=lmax)
    stream, goff = O.pad_stream(codes, gnc, d.n_entries)
    assert all(int(x) % O.CODE_ALIGN == 0 for x in goff)
    assert stream.size - codes.size < O.CODE_ALIGN * gnc.size
    back = O.lzw_decode(stream, goff, d, S.size, d.n_entries)
    assert np.array_equal(back, S)
    # matches never cross a restart boundary: every group decodes to exactly its own bytes (checked inside
    # lzw_decode) and no run is longer than lmax
    assert int(d.ent_len.max()) <= lmax


def test_decode_rejects_inconsistent_stream():
    S = np.arange(256, dtype=np.uint8).repeat(2)
    codes, gnc, d = O.lzw_encode(S, group_bytes=128, max_entries=400, lmax=3)
    stream, goff = O.pad_stream(codes, gnc, d.n_entries)
    bad = stream.copy()
    bad[0] = d.n_entries + 5           # not an entry and not the pad code
    with pytest.raises(ValueError):
        O.lzw_decode(bad, goff, d, S.size, d.n_entries, group_bytes=128)
    short = goff.copy()
    short[1] -= O.CODE_ALIGN           # group 0 loses codes -> wrong length
    with pytest.raises(ValueError):
        O.lzw_decode(stream, short, d, S.size, d.n_entries, group_bytes=128)
    assert np.array_equal(O.lzw_decode(stream, goff, d, S.size, d.n_entries, group_bytes=128), S)


def test_singles_only_dictionary_is_identity_code():
    rng = np.random.default_rng(3)
    S = rng.integers(0, 256, 5000, dtype=np.uint8)
    codes, gnc, d = O.lzw_encode(S, group_bytes=4096, max_entries=256, lmax=3)
    assert np.array_equal(codes, S.astype(np.uint16))     # code == byte
    codes1, _, _ = O.lzw_encode(S, group_bytes=4096, max_entries=65536, lmax=1)
    assert np.array_equal(codes1, S.astype(np.uint16))


def test_information_bound_on_iid_input():
    """A lossless coder cannot beat the zeroth-order entropy on i.i.d. symbols: 16 bits per code must carry
    at most 16/H symbols on average (finite-sample slack 2 %)."""
    rng = np.random.default_rng(5)
    S = np.clip(np.rint(rng.standard_normal(1 << 20) * 34.0), -127, 127).astype(np.int8).view(np.uint8)
    p = np.bincount(S, minlength=256) / S.size
    H = -(p[p > 0] * np.log2(p[p > 0])).sum()
    for max_entries in (32000, 65536):
        codes, gnc, d = O.lzw_encode(S, group_bytes=4096, max_entries=max_entries, lmax=3)
        sym_per_code = S.size / codes.size
        assert sym_per_code < 16.0 / H * 1.02
        assert sym_per_code > 1.5          # and it does find pairs
