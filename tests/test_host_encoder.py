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


@pytest.mark.parametrize("shape,max_entries,lmax,seg_cols,dist", [
    ((64, 512), 30719, 2, 256, "normal"),
    ((33, 300), 1000, 2, 64, "normal"),
    ((16, 8), 256, 2, 16, "normal"),
    ((200, 1024), 4096, 2, 128, "student_t4"),
    ((512, 2048), 30719, 2, 256, "student_t4"),
    ((48, 256), 300, 1, 256, "normal"),
    ((100, 3000), 30719, 2, 1024, "normal"),
    ((200, 1024), 30719, 3, 128, "student_t4"),      # runs of up to 3 and 4 bytes: sorted code space, unit budget
    ((512, 2048), 30719, 4, 256, "student_t4"),
    ((64, 512), 700, 4, 64, "normal"),
    ((33, 300), 30719, 4, 32, "student_t4"),
])
def test_encoder_container_is_byte_identical_to_the_oracles(shape, max_entries, lmax, seg_cols, dist):
    W = make_weights(small_case(shape[0], shape[1], seed=7, dist=dist))
    blob = tq.tq_encode(W, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols)
    ref = O.build_blob(O.encode_matrix(W, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols))
    assert blob == ref
    info = tq.tq_validate_blob(blob)
    p = O.parse_blob(blob)
    assert info["rows"] == shape[0] and info["cols"] == shape[1] and info["n_codes"] == p["n_codes"]
    assert info["n_real_codes"] == p["n_real_codes"] and info["seg_cols"] == seg_cols
    assert info["compressed_bytes"] == p["compressed_bytes"]
    Q, s = O.decode_blob(blob)
    Qo, so = O.quantize_rows(W)
    assert np.array_equal(Q, Qo) and np.array_equal(s, so)


def test_longer_runs_on_low_entropy_matrices_and_over_a_sequence():
    """Runs of up to 4 bytes where they pay: 4-bit levels one per byte and a matrix that is mostly zeros (the unit budget
    binds there: every 4-byte run takes two units), containers identical to the oracle's, also when a second matrix
    goes on from the first one's dictionary; both store well under 0.7 bytes per weight."""
    rng = np.random.default_rng(3)
    W4 = make_weights(small_case(512, 2048, seed=8))
    Ws = make_weights(small_case(512, 2048, seed=9)) * (rng.random((512, 2048)) < 0.1)      # 90 % zeros
    for W, bits in ((W4, 4), (Ws, 8)):
        blob = tq.tq_encode(W, lmax=4, bits=0 if bits == 8 else bits)
        enc = O.encode_matrix(W, lmax=4, bits=bits)
        assert blob == O.build_blob(enc)
        info = tq.tq_validate_blob(blob)
        assert info["lmax"] == 4 and info["compressed_bytes"] < 0.7 * W.size
        assert np.array_equal(O.decode_blob(blob)[0], O.quantize_rows(W, bits)[0])
        W2 = np.roll(W, 7, axis=1)
        blob2 = tq.tq_encode(W2, lmax=4, bits=0 if bits == 8 else bits, dict_from=blob)
        enc2 = O.encode_matrix(W2, lmax=4, bits=bits, carry=enc.dictionary)
        assert blob2 == O.build_blob(enc2)
        p = O.parse_blob(blob2)
        assert int(p["class_end"][1]) + 2 * (p["n_entries"] - int(p["class_end"][1])) <= O.UNIT_BUDGET


def test_defaults_are_the_documented_ones():
    W = make_weights(small_case(64, 512, seed=21))
    assert tq.tq_encode(W) == O.build_blob(O.encode_matrix(W, max_entries=tq.TQ_MAX_ENTRIES_DEVICE, lmax=2, seg_cols=256))


def test_dictionary_carried_over_a_sequence_of_matrices():
    """dict_from: LZW goes on from the earlier container's dictionary; once it is full the later containers hold
    byte-identical dictionary sections."""
    Ws = [make_weights(small_case(r, c, seed=30 + k)) for k, (r, c) in enumerate([(512, 2048), (256, 3072), (64, 768)])]
    blobs, encs = [], []
    for k, W in enumerate(Ws):
        blobs.append(tq.tq_encode(W, dict_from=blobs[-1] if blobs else None, seg_cols=192 if k else 256))
        encs.append(O.encode_matrix(W, seg_cols=192 if k else 256, carry=encs[-1].dictionary if encs else None))
        assert blobs[-1] == O.build_blob(encs[-1])
    ps = [O.parse_blob(b) for b in blobs]
    assert ps[0]["n_entries"] == tq.TQ_MAX_ENTRIES_DEVICE          # the first matrix fills the dictionary
    assert np.array_equal(ps[0]["slots"], ps[1]["slots"]) and np.array_equal(ps[1]["slots"], ps[2]["slots"])
    for W, b in zip(Ws, blobs):
        assert np.array_equal(O.decode_blob(b)[0], O.quantize_rows(W)[0])
    # a small dictionary keeps growing over the sequence
    small = [tq.tq_encode(Ws[2][:2, :32], max_entries=400, seg_cols=16)]
    small.append(tq.tq_encode(Ws[2][16:32, :64], max_entries=400, seg_cols=16, dict_from=small[0]))
    n0, n1 = (O.parse_blob(b)["n_entries"] for b in small)
    assert 256 < n0 < n1 <= 400
    with pytest.raises(tq.TqError):      # the earlier dictionary does not fit the new cap
        tq.tq_encode(Ws[2], max_entries=300, dict_from=small[1])


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
    blob = tq.tq_encode_quantized(Q, s, max_entries=5000, seg_cols=64)
    assert blob == O.build_blob(O.encode_quantized(Q, s, max_entries=5000, seg_cols=64))
    Qd, sd = O.decode_blob(blob)
    assert np.array_equal(Qd, Q) and np.array_equal(sd, s)


def test_quantizer_ties_match_oracle():
    W = np.array([[-127.0, 0.0, 62.5, 63.5, 127.0, 0.5, 1.5, 2.5]], np.float32)
    Q, s = O.decode_blob(tq.tq_encode(W))
    assert Q.tolist() == [[-127, 0, 62, 64, 127, 0, 2, 2]] and s.tolist() == [1.0]


def test_lower_widths_give_the_oracles_container():
    W = make_weights(small_case(48, 640, seed=17))
    for bits, dictionary in ((6, "lzw"), (4, "lzw"), (2, "lzw"), (4, "frequency")):
        blob = tq.tq_encode(W, seg_cols=64, bits=bits, dictionary=dictionary)
        assert blob == O.build_blob(O.encode_matrix(W, seg_cols=64, bits=bits, dictionary=dictionary)), (bits, dictionary)
        Q, s = O.decode_blob(blob)
        Qo, so = O.quantize_rows(W, bits=bits)
        assert np.array_equal(Q, Qo) and np.array_equal(s, so)
    W4 = np.array([[-7.0, 0.0, 2.5, 3.5, 7.0, -6.5, 0.49, 6.51]], np.float32)
    Q, s = O.decode_blob(tq.tq_encode(W4, bits=4))
    assert Q.tolist() == [[-7, 0, 2, 4, 7, -6, 0, 7]] and s.tolist() == [1.0]
    assert tq.tq_encode(W, seg_cols=64, bits=8) == tq.tq_encode(W, seg_cols=64) == tq.tq_encode(W, seg_cols=64, bits=0)


def test_packed_containers_match_the_oracle():
    W = make_weights(small_case(48, 640, seed=19))
    for bits, dictionary, seg in ((4, "lzw", 64), (3, "lzw", 32), (2, "lzw", 16), (4, "frequency", 64)):
        blob = tq.tq_encode(W, seg_cols=seg, bits=bits, dictionary=dictionary, pack=True)
        assert blob == O.build_blob(O.encode_matrix(W, seg_cols=seg, bits=bits, dictionary=dictionary, pack=True)), (bits, dictionary)
        info = tq.tq_validate_blob(blob)
        assert info["packing"] == 1 and info["cols"] == 640 and info["rows"] == 48
        Q, s = O.decode_blob(blob)
        Qo, so = O.quantize_rows(W, bits=bits)
        assert np.array_equal(Q, Qo) and np.array_equal(s, so)
    # already quantized values, any nibble
    rng = np.random.default_rng(5)
    Q = rng.integers(-8, 8, (20, 96), dtype=np.int8)
    s = (rng.random(20) + 0.5).astype(np.float32)
    blob = tq.tq_encode_quantized(Q, s, seg_cols=16, pack=True)
    assert blob == O.build_blob(_packed_encoded(Q, s, 16))
    assert np.array_equal(O.decode_blob(blob)[0], Q)
    assert tq.tq_validate_blob(tq.tq_encode(W, seg_cols=64))["packing"] == 0


def _packed_encoded(Q, s, seg_cols):
    e = O.encode_quantized(O.pack_nibbles(Q), s, seg_cols=seg_cols)
    e.packing = 1
    return e


def test_packing_argument_errors():
    W = np.zeros((4, 8), np.float32)
    for kw in (dict(pack=True), dict(pack=True, bits=6), dict(pack=True, bits=8)):
        with pytest.raises(tq.TqError) as ei:
            tq.tq_encode(W, **kw)
        assert ei.value.code == -1
    with pytest.raises(tq.TqError):
        tq.tq_encode(np.zeros((4, 7), np.float32), bits=4, pack=True)          # odd number of columns
    with pytest.raises(tq.TqError):
        tq.tq_encode_quantized(np.full((2, 4), 8, np.int8), np.ones(2, np.float32), pack=True)   # 8 does not fit 4 bits


def test_four_bit_values_all_pair_up():
    # 15 levels: every pair of neighbouring values gets a dictionary entry early on, so nearly every code stands for two weights
    W = make_weights(small_case(256, 1024, seed=18))
    info = tq.tq_validate_blob(tq.tq_encode(W, bits=4))
    assert info["n_entries"] <= 256 + 15 * 15
    assert 256 * 1024 / info["n_real_codes"] > 1.99


def test_encode_argument_errors():
    W = np.zeros((4, 4), np.float32)
    for kw in (dict(max_entries=100), dict(max_entries=tq.TQ_MAX_ENTRIES_DEVICE + 1), dict(lmax=5), dict(lmax=3, dictionary="frequency"),
               dict(seg_cols=24), dict(seg_cols=2048), dict(bits=1), dict(bits=9)):
        with pytest.raises(tq.TqError) as ei:
            tq.tq_encode(W, **kw)
        assert ei.value.code == -1


def _mutate(blob: bytes, offset: int, fmt: str, value) -> bytes:
    b = bytearray(blob)
    struct.pack_into(fmt, b, offset, value)
    return bytes(b)


def test_validation_rejects_malformed_containers():
    W = make_weights(small_case(64, 512, seed=3))
    blob = tq.tq_encode(W, max_entries=2000, seg_cols=64)
    p = O.parse_blob(blob)
    (o_d, _, o_u, _, o_c, _) = struct.unpack_from("<QQQQQQ", blob, 96)
    assert tq.tq_validate_blob(blob)["n_entries"] == p["n_entries"]
    assert o_d == 256 and np.array_equal(np.frombuffer(blob, np.uint32, 3, o_u), p["uoff"][:3])
    last = int(np.flatnonzero(p["stream"][:256].reshape(64, 4)[0] != p["pad_code"]).max())   # lane 0, first chunk
    bad = {
        "magic": _mutate(blob, 0, "<B", 0x55),
        "truncated": blob[:-256],
        "rows": _mutate(blob, 16, "<I", 65),
        "segment width": _mutate(blob, 24, "<I", 48),
        "code out of range": _mutate(blob, o_c, "<H", p["n_entries"] + 1),
        "segment length": _mutate(blob, o_c, "<H", 256 if p["stream"][0] < 256 else 0),
        "offset not monotone": _mutate(blob, o_u + 4, "<I", 0xFFFFFFF0),
        "offset shifted": _mutate(blob, o_u + 4, "<I", int(p["uoff"][1]) + 1),
        "entry longer than its place in the code space says": _mutate(blob, o_d + 4 * 300, "<I", 0x010203),
        "entry bytes past its length": _mutate(blob, o_d + 4 * 7, "<I", 0x0107),
        "single byte entry": _mutate(blob, o_d + 4 * 7, "<I", 8),
        "pad entry": _mutate(blob, o_d + 4 * p["n_entries"], "<I", 5),
        "classes not monotone": _mutate(blob, 168 + 8, "<I", 255),
        "classes beyond the entries": _mutate(blob, 168 + 4, "<I", p["n_entries"] + 1),
        "classes say longer runs than lmax": _mutate(blob, 168 + 4, "<I", p["n_entries"] - 1),
        "singles class": _mutate(blob, 168, "<I", 255),
        "count of real codes": _mutate(blob, 88, "<Q", p["n_real_codes"] + 1),
    }
    # a pad code in the middle of a lane stream (before real codes)
    assert last >= 1
    bad["pad inside a lane stream"] = _mutate(blob, o_c, "<H", p["pad_code"])
    for why, b in bad.items():
        with pytest.raises(tq.TqError) as ei:
            tq.tq_validate_blob(b)
        assert ei.value.code == -2, why


def _lane_spread_from_the_stream(blob: bytes) -> int:
    """Largest difference between the columns two still incomplete lanes of one unit have reached after the same
    number of chunks, counted directly from the parsed container."""
    p = O.parse_blob(blob)
    _, _, seg_len = O.segment_table(p["rows"], p["cols"], p["seg_cols"])
    lens = np.concatenate([p["dictionary"].ent_len.astype(np.int64), [0]])   # the pad code adds nothing
    worst = 0
    for u in range(p["n_units"]):
        lo, hi = int(p["uoff"][u]), int(p["uoff"][u + 1])
        codes = p["stream"][lo * 256: hi * 256].reshape(hi - lo, 64, 4)
        reached = np.cumsum(lens[codes].sum(axis=2), axis=0)                     # [chunk, lane]
        want = np.zeros(64, np.int64)
        segs = seg_len[u * 64: (u + 1) * 64]
        want[: segs.size] = segs
        for r in reached:
            busy = r < want
            if busy.sum() >= 2:
                worst = max(worst, int(r[busy].max() - r[busy].min()))
    return worst


@pytest.mark.parametrize("rows,cols,seg_cols,max_entries", [(64, 512, 64, 1000), (40, 300, 32, 300), (48, 1024, 256, 30719),
                                                            (17, 257, 256, 400)])
def test_validation_reports_the_lane_spread(rows, cols, seg_cols, max_entries):
    first = tq.tq_encode(make_weights(small_case(rows, cols, seed=31)), max_entries=max_entries, seg_cols=seg_cols)
    second = tq.tq_encode(make_weights(small_case(rows, cols, seed=32)), max_entries=max_entries, seg_cols=seg_cols, dict_from=first)
    for blob in (first, second):
        assert tq.tq_validate_blob(blob)["lane_spread"] == _lane_spread_from_the_stream(blob)
    Q = np.zeros((32, 512), np.int8)
    Q[1::2] = np.random.default_rng(3).integers(-127, 128, size=(16, 512), dtype=np.int8)
    blob = tq.tq_encode_quantized(Q, np.ones(32, np.float32), max_entries=300, seg_cols=256)
    spread = tq.tq_validate_blob(blob)["lane_spread"]
    assert spread == _lane_spread_from_the_stream(blob) and spread > 65


@pytest.mark.parametrize("shape,max_entries,lmax,seg_cols,dist", [
    ((64, 512), 30719, 2, 256, "normal"),
    ((33, 300), 1000, 2, 64, "normal"),
    ((16, 8), 256, 2, 16, "normal"),
    ((200, 1024), 4096, 2, 128, "student_t4"),
    ((48, 256), 300, 1, 256, "normal"),
])
def test_frequency_dictionary_container_is_byte_identical_to_the_oracles(shape, max_entries, lmax, seg_cols, dist):
    W = make_weights(small_case(shape[0], shape[1], seed=8, dist=dist))
    blob = tq.tq_encode(W, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols, dictionary="frequency")
    enc = O.encode_matrix(W, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols, dictionary="frequency")
    assert blob == O.build_blob(enc)
    tq.tq_validate_blob(blob)
    assert np.array_equal(O.decode_blob(blob)[0], O.quantize_rows(W)[0])
    # carried over to the next matrix the dictionary stays as it is, in both kinds of encoder run
    W2 = make_weights(small_case(shape[0], shape[1], seed=9, dist=dist))
    blob2 = tq.tq_encode(W2, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols, dictionary="frequency", dict_from=blob)
    enc2 = O.encode_matrix(W2, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols, dictionary="frequency", carry=enc.dictionary)
    assert blob2 == O.build_blob(enc2)
    assert np.array_equal(O.parse_blob(blob2)["slots"], O.parse_blob(blob)["slots"])


def test_gate_up_container_is_the_row_interleaved_matrix():
    Wg = make_weights(small_case(24, 300, seed=41))
    Wu = make_weights(small_case(24, 300, seed=42))
    blob = tq.tq_encode_gate_up(Wg, Wu, max_entries=1000, seg_cols=64)
    assert blob == O.build_blob(O.encode_matrix(O.interleave_rows(Wg, Wu), max_entries=1000, seg_cols=64))
    assert tq.tq_validate_blob(blob)["rows"] == 48


def test_null_arguments_are_refused_before_any_device_work():
    """Every entry point checks its pointers first: a null handle, buffer or output is TQ_E_INVALID_ARG with a message,
    on a machine without a GPU too; destroying nothing is not an error; a malformed container is refused by the host
    validation that precedes the first device call."""
    import ctypes

    from paper_2509_22951_amd import binding
    lib = tq.load()
    null = ctypes.c_void_p(None)
    some = ctypes.c_void_p(0x1000)      # never dereferenced: the handle next to it is null
    arr1 = (ctypes.c_void_p * 1)(None)
    out = ctypes.c_void_p()
    info = binding.TqInfo()
    words = (ctypes.c_uint16 * 1)(1)
    calls = [
        ("tq_matvec", lambda: lib.tq_matvec(null, some, some, 1, None)),
        ("tq_matvec_gate_up", lambda: lib.tq_matvec_gate_up(null, some, some, 1, None)),
        ("tq_decompress", lambda: lib.tq_decompress(null, some, None)),
        ("tq_matvec_multi n = 0", lambda: lib.tq_matvec_multi(0, arr1, arr1, arr1, 1, None)),
        ("tq_matvec_multi null lists", lambda: lib.tq_matvec_multi(1, None, None, None, 1, None)),
        ("tq_matvec_multi null handle", lambda: lib.tq_matvec_multi(1, arr1, arr1, arr1, 1, None)),
        ("tq_matvec_gate_up_multi null handle", lambda: lib.tq_matvec_gate_up_multi(1, arr1, arr1, arr1, 1, None)),
        ("tq_decompress_multi null handle", lambda: lib.tq_decompress_multi(1, arr1, arr1, None)),
        ("tq_get_info null handle", lambda: lib.tq_get_info(null, ctypes.byref(info))),
        ("tq_step_create n = 0", lambda: lib.tq_step_create(0, arr1, arr1, arr1, 1, 0, ctypes.byref(out))),
        ("tq_step_create null handle", lambda: lib.tq_step_create(1, arr1, arr1, arr1, 1, 0, ctypes.byref(out))),
        ("tq_step_create null output", lambda: lib.tq_step_create(1, arr1, arr1, arr1, 1, 0, None)),
        ("tq_step_launch null", lambda: lib.tq_step_launch(null, None)),
        ("tq_step_get_info null", lambda: lib.tq_step_get_info(null, ctypes.byref(binding.TqStepInfo()))),
        ("tq_create_from_encoded null container", lambda: lib.tq_create_from_encoded(None, 0, ctypes.byref(out))),
        ("tq_create_from_encoded null output", lambda: lib.tq_create_from_encoded(b"x" * 512, 512, None)),
        ("tq_listing_create null output", lambda: lib.tq_listing_create(words, 1, None, 0, None)),
        ("tq_listing_create null words", lambda: lib.tq_listing_create(None, 1, None, 0, ctypes.byref(out))),
        ("tq_listing_decompress null handle", lambda: lib.tq_listing_decompress(null, some, None)),
        ("tq_listing_get_info null handle", lambda: lib.tq_listing_get_info(null, ctypes.byref(binding.TqListingInfo()))),
        ("tq_listing_build_table null outputs", lambda: lib.tq_listing_build_table(None, None, 0, 10, None, None)),
        ("tq_listing_compress null outputs", lambda: lib.tq_listing_compress(None, 0, None, 0, None, None)),
    ]
    for what, call in calls:
        assert call() == -1, what                                  # TQ_E_INVALID_ARG
        assert tq.tq_last_error_string(), what
    assert lib.tq_destroy(null) == 0 and lib.tq_step_destroy(null) == 0 and lib.tq_listing_destroy(null) == 0
    blob = tq.tq_encode(make_weights(small_case(32, 64, seed=5)), seg_cols=16)
    for bad in (blob[:-1], blob[:100], b"\0" * len(blob)):
        out = ctypes.c_void_p(0x55)
        assert lib.tq_create_from_encoded(bad, len(bad), ctypes.byref(out)) == -2      # TQ_E_BAD_BLOB
        assert out.value is None                                                       # the output is cleared on failure


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message before it touches a device: the path is a single-GPU kernel."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()


def test_bench_launch_plans_group_what_a_layer_can_run_side_by_side():
    """The launch plans of bench.py on the 3B sweep (28 layers of q, k, v, o, gate, up, down, then lm_head): one group, one
    per layer, one per set of products with a common input (q,k,v | o | gate,up | down: the stages of the staged step),
    one per matrix; every plan keeps the order of the sweep and covers every matrix once."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    from inputs import config_matrices
    specs = config_matrices(4)
    assert len(specs) == 197
    sizes = {fuse: [len(g) for g in bench.launch_groups(specs, fuse)] for fuse in ("sweep", "layer", "independent", "none")}
    assert sizes["sweep"] == [197]
    assert sizes["layer"] == [7] * 28 + [1]
    assert sizes["independent"] == [3, 1, 2, 1] * 28 + [1] and len(sizes["independent"]) == 113
    assert sizes["none"] == [1] * 197
    for fuse in sizes:
        flat = [i for g in bench.launch_groups(specs, fuse) for i in g]
        assert flat == list(range(197))
    first = bench.launch_groups(specs, "independent")[:4]
    assert [[specs[i].name.split(".")[-1] for i in g] for g in first] == [["q_proj", "k_proj", "v_proj"], ["o_proj"], ["gate_proj", "up_proj"], ["down_proj"]]
