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
    # one micro-tile: 16 x 8 -> the string starts with the matrix in row-major order, rest is zero padding
    Q = rng.integers(-127, 128, (16, 8), dtype=np.int8)
    S = O.serialize(Q)
    assert S.size == 16 * 256
    assert np.array_equal(S[:128].view(np.int8), Q.reshape(-1))
    assert not S[128:].any()
    # two micro-tiles side by side
    Q = rng.integers(-127, 128, (16, 16), dtype=np.int8)
    S = O.serialize(Q).view(np.int8)
    assert np.array_equal(S[:128], Q[:, :8].reshape(-1)) and np.array_equal(S[128:256], Q[:, 8:].reshape(-1))
    # two bands, two groups: band-major, then groups left to right, then micro-tiles
    Q = rng.integers(-127, 128, (32, 512), dtype=np.int8)
    S = O.serialize(Q).view(np.int8)
    g = 4096
    assert np.array_equal(S[0:128], Q[0:16, 0:8].reshape(-1))
    assert np.array_equal(S[g + 128 * 3: g + 128 * 4], Q[0:16, 256 + 24: 256 + 32].reshape(-1))
    assert np.array_equal(S[2 * g: 2 * g + 128], Q[16:32, 0:8].reshape(-1))
    assert np.array_equal(S[3 * g + 128 * 31: 4 * g], Q[16:32, 504:512].reshape(-1))


@pytest.mark.parametrize("shape", [(16, 256), (5, 7), (33, 300), (48, 512), (1, 1), (17, 257)])
def test_serialize_is_a_padded_permutation_and_inverts(shape):
    rng = np.random.default_rng(3)
    Q = rng.integers(-127, 128, shape, dtype=np.int8)
    S = O.serialize(Q)
    rp, cp = O.padded_shape(*shape)
    assert S.size == rp * cp and rp % 16 == 0 and cp % 256 == 0
    assert np.array_equal(np.sort(S[S != 0]), np.sort(Q.view(np.uint8)[Q != 0].reshape(-1)))
    assert np.array_equal(O.deserialize(S, *shape), Q)
    assert O.serialize(np.array([[-1]], np.int8))[0] == 0xFF      # two's complement byte


@pytest.mark.parametrize("shape,max_entries", [((64, 512), 32000), ((33, 300), 1000), ((16, 8), 256), ((200, 1024), 4096)])
def test_container_round_trip(shape, max_entries):
    spec = small_case(shape[0], shape[1], seed=42)
    W = make_weights(spec)
    enc = O.encode_matrix(W, max_entries=max_entries, lmax=3)
    blob = O.build_blob(enc)
    p = O.parse_blob(blob)
    assert (p["rows"], p["cols"]) == shape and p["n_entries"] == enc.dictionary.n_entries
    assert p["n_codes"] == enc.stream.size and p["pad_code"] == enc.dictionary.n_entries
    assert p["slots"][-1] == 0                                    # the pad entry has length 0
    assert np.array_equal(p["slots"][:256], np.arange(256, dtype=np.uint32) | (8 << 24))   # singles: code == byte, 8 bits long
    Q, s = O.decode_blob(blob)
    assert np.array_equal(Q, enc.Q) and np.array_equal(s, enc.scales)
    Qq, sq = O.quantize_rows(W)
    assert np.array_equal(Q, Qq)
    bits, x = make_activations(spec, 2)
    y = O.matvec_from_blob(blob, x)
    ref = (x.astype(np.float64) @ Qq.astype(np.float64).T) * sq.astype(np.float64)[None, :]
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_measured_ratio_config1_like():
    """On config-1-like input the stream is close to the size of raw int8 (i.i.d. Gaussian symbols carry about
    7.2 bits each); the measured ratio must sit under the entropy bound and above a sanity floor."""
    spec = small_case(512, 2048, seed=1)
    W = make_weights(spec)
    enc = O.encode_matrix(W, max_entries=32000, lmax=3)
    weights_per_code = (512 * 2048) / enc.n_real_codes
    p = np.bincount(enc.Q.view(np.uint8).reshape(-1), minlength=256) / enc.Q.size
    H = -(p[p > 0] * np.log2(p[p > 0])).sum()
    assert 1.5 < weights_per_code < 16.0 / H * 1.02
