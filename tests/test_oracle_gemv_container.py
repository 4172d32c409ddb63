"""Pins for the oracle's float64 GEMV, its byte serialization and its container reader/writer."""
import numpy as np
import pytest

from inputs import make_activations, make_weights, small_case
from oracle import oracle as O


def _rand_q(rng, r, k):
    return rng.integers(-127, 128, (r, k), dtype=np.int8), (rng.random(r).astype(np.float32) + 0.1)


def test_gemv_equals_numpy_float64_matmul():
    rng = np.random.default_rng(0)
    Q, s = _rand_q(rng, 37, 301)
    x = rng.standard_normal((3, 301)).astype(np.float32)
    y = O.gemv_f64(Q, s, x)
    ref = (x.astype(np.float64) @ Q.astype(np.float64).T) * s.astype(np.float64)[None, :]
    assert y.shape == (3, 37)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-9)


def test_gemv_unit_vectors_and_ones():
    rng = np.random.default_rng(1)
    Q, s = _rand_q(rng, 16, 64)
    for j in (0, 5, 63):
        e = np.zeros((1, 64), np.float32)
        e[0, j] = 1.0
        assert np.array_equal(O.gemv_f64(Q, s, e)[0], s.astype(np.float64) * Q[:, j])
    ones = np.ones((1, 64), np.float32)
    assert np.array_equal(O.gemv_f64(Q, s, ones)[0], s.astype(np.float64) * Q.sum(axis=1, dtype=np.int64))
    # a transposed operand or a dropped scale would fail these: non-square, distinct scales
    assert O.gemv_f64(Q, s, ones).shape == (1, 16)


def test_serialize_special_cases_reduce_to_slicing():
    rng = np.random.default_rng(2)
    # one full unit: 16 rows x 4 panels of 16 columns; lane l = row l % 16, panel l // 16
    Q = rng.integers(-127, 128, (16, 64), dtype=np.int8)
    S, seg_len = O.serialize(Q, seg_cols=16)
    assert seg_len.tolist() == [16] * 64
    for lane in (0, 1, 15, 16, 37, 63):
        assert np.array_equal(S[16 * lane: 16 * lane + 16].view(np.int8), Q[lane % 16, 16 * (lane // 16): 16 * (lane // 16) + 16])
    # two bands, two quads (8 panels): units in the order (band 0, quad 0), (band 0, quad 1), (band 1, quad 0), ...
    Q = rng.integers(-127, 128, (32, 128), dtype=np.int8)
    S, seg_len = O.serialize(Q, seg_cols=16)
    unit = 64 * 16
    assert np.array_equal(S[1 * unit + 16 * 17: 1 * unit + 16 * 18].view(np.int8), Q[1, 64 + 16: 64 + 32])      # band 0, quad 1, lane 17
    assert np.array_equal(S[2 * unit + 16 * 63: 3 * unit].view(np.int8), Q[16 + 15, 48:64])                      # band 1, quad 0, lane 63
    # ragged: 5 x 40 with panels of 16 -> 3 panels (16, 16, 8 columns) in one quad, rows 5..15 and panel 3 are empty
    Q = rng.integers(-127, 128, (5, 40), dtype=np.int8)
    S, seg_len = O.serialize(Q, seg_cols=16)
    want = np.zeros((4, 16), np.uint32)
    want[0, :5] = 16
    want[1, :5] = 16
    want[2, :5] = 8
    assert np.array_equal(seg_len.reshape(4, 16), want)
    assert np.array_equal(S[:16].view(np.int8), Q[0, :16]) and np.array_equal(S[-8:].view(np.int8), Q[4, 32:])


@pytest.mark.parametrize("shape,seg_cols", [((16, 256), 64), ((5, 7), 16), ((33, 300), 32), ((48, 512), 256), ((1, 1), 16),
                                            ((17, 257), 256), ((40, 3000), 1024)])
def test_serialize_is_a_permutation_and_inverts(shape, seg_cols):
    rng = np.random.default_rng(3)
    Q = rng.integers(-127, 128, shape, dtype=np.int8)
    S, seg_len = O.serialize(Q, seg_cols)
    n_bands, n_panels, n_quads = O.geometry(shape[0], shape[1], seg_cols)
    assert seg_len.size == 64 * n_bands * n_quads and S.size == Q.size == int(seg_len.sum())
    assert np.array_equal(np.sort(S), np.sort(Q.view(np.uint8).reshape(-1)))
    assert np.array_equal(O.deserialize(S, shape[0], shape[1], seg_cols), Q)
    assert O.serialize(np.array([[-1]], np.int8), 16)[0][0] == 0xFF      # two's complement byte


@pytest.mark.parametrize("shape,max_entries,seg_cols", [((64, 512), 30719, 256), ((33, 300), 1000, 64), ((16, 8), 256, 16),
                                                        ((200, 1024), 4096, 128)])
def test_container_round_trip(shape, max_entries, seg_cols):
    spec = small_case(shape[0], shape[1], seed=42)
    W = make_weights(spec)
    enc = O.encode_matrix(W, max_entries=max_entries, lmax=2, seg_cols=seg_cols)
    blob = O.build_blob(enc)
    p = O.parse_blob(blob)
    assert (p["rows"], p["cols"]) == shape and p["n_entries"] == enc.dictionary.n_entries
    assert p["n_codes"] == enc.stream.size and p["pad_code"] == enc.dictionary.n_entries and p["seg_cols"] == seg_cols
    assert p["slots"][-1] == 0                                    # the pad entry is empty
    assert np.array_equal(p["slots"][:256], np.arange(256, dtype=np.uint32))               # singles: code == byte
    assert list(p["class_end"]) == [256] + [p["n_entries"]] * 3                           # no run longer than 2 here
    Q, s = O.decode_blob(blob)
    assert np.array_equal(Q, enc.Q) and np.array_equal(s, enc.scales)
    Qq, sq = O.quantize_rows(W)
    assert np.array_equal(Q, Qq)
    bits, x = make_activations(spec, 2)
    y = O.matvec_from_blob(blob, x)
    ref = (x.astype(np.float64) @ Qq.astype(np.float64).T) * sq.astype(np.float64)[None, :]
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("lmax", [3, 4])
def test_container_with_longer_runs(lmax):
    """Runs of up to 4 bytes: the container word of an entry holds its bytes, first byte lowest; the length is told by
    the code's place (class_end); the round trip through writer, reader and decoder is exact; the dictionary stays
    within the unit budget."""
    spec = small_case(96, 640, seed=9, dist="student_t4")
    W = make_weights(spec)
    W[:, 100:300] = 0                                   # a stretch of equal values, so that long runs do get used
    enc = O.encode_matrix(W, lmax=lmax, seg_cols=128)
    assert int(enc.dictionary.ent_len.max()) == lmax
    p = O.parse_blob(O.build_blob(enc))
    assert list(p["class_end"]) == list(enc.class_end) and p["class_end"][lmax - 1] == p["n_entries"]
    assert np.array_equal(p["dictionary"].ent_len, enc.dictionary.ent_len)
    assert np.array_equal(p["dictionary"].ent_bytes, enc.dictionary.ent_bytes)
    e = int(p["class_end"][1])                          # the first 3-byte entry, written out by hand
    b = enc.dictionary.entry(e)
    assert len(b) == 3 and int(p["slots"][e]) == b[0] | b[1] << 8 | b[2] << 16
    n12, n34 = int(p["class_end"][1]), p["n_entries"] - int(p["class_end"][1])
    assert n12 + 2 * n34 <= O.UNIT_BUDGET
    Q, s = O.decode_blob(O.build_blob(enc))
    assert np.array_equal(Q, O.quantize_rows(W)[0]) and np.array_equal(s, enc.scales)
    assert enc.n_real_codes < O.encode_matrix(W, lmax=2, seg_cols=128).n_real_codes      # the longer runs do pay here


def test_measured_ratio_config1_like():
    """On config-1-like input the stream is close to the size of raw int8 (i.i.d. Gaussian symbols carry about
    7.2 bits each); the measured ratio must sit under the entropy bound and above a sanity floor."""
    spec = small_case(512, 2048, seed=1)
    W = make_weights(spec)
    enc = O.encode_matrix(W, max_entries=30719, lmax=2)
    weights_per_code = (512 * 2048) / enc.n_real_codes
    p = np.bincount(enc.Q.view(np.uint8).reshape(-1), minlength=256) / enc.Q.size
    H = -(p[p > 0] * np.log2(p[p > 0])).sum()
    assert 1.5 < weights_per_code < 16.0 / H * 1.02


def test_gate_up_definition_on_textbook_values():
    """silu(1) = 0.7310585786300049, silu(2) = 1.7615941559557649, silu(-2) = -0.2384058440442351, silu(0) = 0."""
    Qg = np.array([[1, 0], [2, 0], [-2, 0], [0, 5]], np.int8)
    Qu = np.array([[3, 0], [3, 0], [3, 0], [3, 0]], np.int8)
    ones = np.ones(4, np.float32)
    x = np.array([[1.0, 0.0]], np.float32)
    y = O.gate_up_f64(Qg, ones, Qu, ones, x)
    assert np.allclose(y[0], [3 * 0.7310585786300049, 3 * 1.7615941559557649, 3 * -0.2384058440442351, 0.0], rtol=0, atol=1e-15)
    # scales enter each product separately: halving the gate scale halves g, not y
    y2 = O.gate_up_f64(Qg, np.float32(0.5) * ones, Qu, np.float32(2) * ones, x)
    assert np.allclose(y2[0, :2], [6 * 0.5 / (1 + np.exp(-0.5)), 6 * 0.7310585786300049], rtol=0, atol=1e-15)
    # large gate: silu(g) -> g; large negative gate: -> 0
    big = O.gate_up_f64(np.array([[127], [-127]], np.int8), np.ones(2, np.float32), np.array([[1], [1]], np.int8), np.ones(2, np.float32),
                        np.array([[1.0]], np.float32))
    assert abs(big[0, 0] - 127.0) < 1e-12 and abs(big[0, 1]) < 1e-12
    assert O.interleave_rows(np.array([[1], [2]]), np.array([[7], [8]])).ravel().tolist() == [1, 7, 2, 8]


# ----- two 4-bit values per byte

def test_nibble_packing_by_hand():
    # column 2j in bits 0..3, column 2j + 1 in bits 4..7, 4-bit two's complement: -1 = 0xF, -8 = 0x8
    Q = np.array([[1, 2, -1, 0, 7, -8, -7, 3]], np.int8)
    P = O.pack_nibbles(Q)
    assert P.dtype == np.int8 and P.shape == (1, 4)
    assert P.view(np.uint8).tolist() == [[0x21, 0x0F, 0x87, 0x39]]
    assert np.array_equal(O.unpack_nibbles(P), Q)


def test_nibble_packing_round_trips_every_byte_and_rejects_what_does_not_fit():
    P = np.arange(256, dtype=np.uint8).reshape(2, 128).view(np.int8)
    Q = O.unpack_nibbles(P)
    assert Q.shape == (2, 256) and Q.min() == -8 and Q.max() == 7
    assert np.array_equal(O.pack_nibbles(Q), P)
    for v in range(256):                                 # arithmetic definition of the two fields
        lo, hi = int(Q.reshape(-1)[2 * v]), int(Q.reshape(-1)[2 * v + 1])
        assert (lo % 16) + 16 * (hi % 16) == v
    with pytest.raises(ValueError):
        O.pack_nibbles(np.array([[8, 0]], np.int8))
    with pytest.raises(ValueError):
        O.pack_nibbles(np.array([[0, -9]], np.int8))
    with pytest.raises(ValueError):
        O.pack_nibbles(np.zeros((2, 3), np.int8))


def test_packed_container_decodes_to_the_quantized_matrix_and_is_half_as_wide():
    W = make_weights(small_case(40, 1000, seed=23))
    for bits in (4, 3, 2):
        e = O.encode_matrix(W, seg_cols=64, bits=bits, pack=True)
        assert e.packing == 1 and e.cols == 500
        blob = O.build_blob(e)
        p = O.parse_blob(blob)
        assert p["packing"] == 1 and p["cols"] == 500
        Q, s = O.decode_blob(blob)
        Qo, so = O.quantize_rows(W, bits=bits)
        assert Q.shape == (40, 1000) and np.array_equal(Q, Qo) and np.array_equal(s, so)
        _, x = make_activations(small_case(40, 1000, seed=23), 2)
        assert np.array_equal(O.matvec_from_blob(blob, x), O.gemv_f64(Qo, so, x))
    with pytest.raises(ValueError):
        O.encode_matrix(W, bits=6, pack=True)
    # more weights per code than one value per byte can reach (2)
    packed, plain = O.parse_blob(O.build_blob(O.encode_matrix(W, bits=4, pack=True))), O.parse_blob(O.build_blob(O.encode_matrix(W, bits=4)))
    assert W.size / packed["n_real_codes"] > 2.5 > 2.0 >= W.size / plain["n_real_codes"]
    assert packed["n_real_codes"] < 0.8 * plain["n_real_codes"]
