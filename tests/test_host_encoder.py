"""Host-side checks of libtq that need no GPU: the C ABI exports, the encoder against the oracle, and
container validation."""
import ctypes
import os
import re
import struct

import numpy as np
import pytest

import paper_2509_22951_amd as tq
from inputs import make_weights, small_case
from oracle import oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tq.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tq_[a-z_]+)\s*\(", hdr))
    assert {"tq_create_from_encoded", "tq_matvec", "tq_decompress", "tq_destroy", "tq_encode"} <= declared
    lib = ctypes.CDLL(tq.lib_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(tq.binding.EXPORTS)


@pytest.mark.parametrize("shape,max_entries,lmax,dist", [
    ((64, 512), 32000, 3, "normal"),
    ((33, 300), 1000, 3, "normal"),
    ((16, 8), 256, 3, "normal"),
    ((200, 1024), 4096, 2, "student_t4"),
    ((512, 2048), 32000, 3, "student_t4"),
    ((48, 256), 300, 1, "normal"),
])
def test_encoder_container_is_byte_identical_to_the_oracles(shape, max_entries, lmax, dist):
    W = make_weights(small_case(shape[0], shape[1], seed=7, dist=dist))
    blob = tq.tq_encode(W, max_entries=max_entries, lmax=lmax)
    ref = O.build_blob(O.encode_matrix(W, max_entries=max_entries, lmax=lmax))
    assert blob == ref
    info = tq.tq_validate_blob(blob)
    p = O.parse_blob(blob)
    assert info["rows"] == shape[0] and info["cols"] == shape[1] and info["n_codes"] == p["n_codes"]
    assert info["compressed_bytes"] == p["compressed_bytes"]
    Q, s = O.decode_blob(blob)
    Qo, so = O.quantize_rows(W)
    assert np.array_equal(Q, Qo) and np.array_equal(s, so)


@pytest.mark.parametrize("dist", ["normal", "student_t4"])
def test_auto_lmax_keeps_the_smaller_container(dist):
    W = make_weights(small_case(512, 2048, seed=21, dist=dist))
    auto = tq.tq_encode(W)                       # lmax = 0: auto
    cands = {l: O.build_blob(O.encode_matrix(W, max_entries=tq.TQ_DEFAULT_MAX_ENTRIES, lmax=l)) for l in (2, 3)}
    want = cands[2] if len(cands[2]) < len(cands[3]) else cands[3]
    assert auto == want
    assert tq.tq_validate_blob(auto)["lmax"] == (2 if dist == "normal" else 3)


def test_encoder_is_deterministic_across_thread_counts():
    W = make_weights(small_case(256, 2048, seed=9))
    a = tq.tq_encode(W, max_entries=2000, n_threads=1)
    b = tq.tq_encode(W, max_entries=2000, n_threads=7)
    assert a == b


def test_encode_quantized_accepts_any_byte_and_matches_oracle():
    rng = np.random.default_rng(0)
    Q = rng.integers(-128, 128, (40, 520), dtype=np.int8)
    Q[3, :] = -128
    Q[5, :] = 0
    s = rng.random(40).astype(np.float32)
    blob = tq.tq_encode_quantized(Q, s, max_entries=5000, lmax=3)
    assert blob == O.build_blob(O.encode_quantized(Q, s, max_entries=5000, lmax=3))
    Qd, sd = O.decode_blob(blob)
    assert np.array_equal(Qd, Q) and np.array_equal(sd, s)


def test_quantizer_ties_match_oracle():
    W = np.array([[-127.0, 0.0, 62.5, 63.5, 127.0, 0.5, 1.5, 2.5]], np.float32)
    Q, s = O.decode_blob(tq.tq_encode(W))
    assert Q.tolist() == [[-127, 0, 62, 64, 127, 0, 2, 2]] and s.tolist() == [1.0]


def test_encode_argument_errors():
    W = np.zeros((4, 4), np.float32)
    for kw in (dict(max_entries=100), dict(max_entries=tq.TQ_MAX_ENTRIES_DEVICE + 1), dict(lmax=4)):
        with pytest.raises(tq.TqError) as ei:
            tq.tq_encode(W, **kw)
        assert ei.value.code == -1


def _mutate(blob: bytes, offset: int, fmt: str, value) -> bytes:
    b = bytearray(blob)
    struct.pack_into(fmt, b, offset, value)
    return bytes(b)


def test_validation_rejects_malformed_containers():
    W = make_weights(small_case(64, 512, seed=3))
    blob = tq.tq_encode(W, max_entries=2000)
    p = O.parse_blob(blob)
    (o_d, _, o_g, _, o_c, _) = struct.unpack_from("<QQQQQQ", blob, 80)
    assert tq.tq_validate_blob(blob)["n_entries"] == p["n_entries"]
    bad = {
        "magic": _mutate(blob, 0, "<B", 0x55),
        "truncated": blob[:-256],
        "rows": _mutate(blob, 16, "<I", 65),
        "code out of range": _mutate(blob, o_c, "<H", p["n_entries"] + 1),
        "group length": _mutate(blob, o_c, "<H", 256 if p["stream"][0] < 256 else 0),
        "offset not monotone": _mutate(blob, o_g + 4, "<I", 0xFFFFFFF0),
        "offset misaligned": _mutate(blob, o_g + 4, "<I", int(p["goff"][1]) + 1),
        "entry length": _mutate(blob, o_d + 4 * 300, "<I", (32 << 24) | 0x010203),
        "entry length not whole bytes": _mutate(blob, o_d + 4 * 300, "<I", (12 << 24) | 0x0102),
        "single byte entry": _mutate(blob, o_d + 4 * 7, "<I", (8 << 24) | 8),
        "pad entry": _mutate(blob, o_d + 4 * p["n_entries"], "<I", 8 << 24),
    }
    # a pad code in the middle of a group (before real codes)
    mid = bytearray(blob)
    struct.pack_into("<H", mid, o_c + 2, p["pad_code"])
    bad["pad inside group"] = bytes(mid)
    for why, b in bad.items():
        with pytest.raises(tq.TqError) as ei:
            tq.tq_validate_blob(b)
        assert ei.value.code == -2, why
