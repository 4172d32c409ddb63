"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Decoded weights must be bit-exact; outputs within 1e-3 of the float64 oracle, measured as
max_r |y - y_ref| <= 1e-3 * max_r |y_ref| per (matrix, batch row)."""
import numpy as np
import pytest

import paper_2509_22951_amd as tq
from inputs import make_activations, make_weights, small_case
from oracle import oracle as O

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (no CPU fallback exists)")
    tq.load()
    return torch.device("cuda:0")


RING_MIN_BANDS_DEFAULT = 24


@pytest.fixture
def ring_for_small_launches(dev):
    """The library keeps the ring kernel for launches with many bands per CU; this lets a small matrix through."""
    tq.tq_set_ring_min_bands_per_cu(0)
    yield
    tq.tq_set_ring_min_bands_per_cu(RING_MIN_BANDS_DEFAULT)


@pytest.fixture(autouse=True)
def _default_ring_threshold_afterwards():
    """Tests that change the library's ring-kernel threshold leave the default behind."""
    yield
    tq.tq_set_ring_min_bands_per_cu(24)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def gpu_decompress(m: tq.Matrix, dev):
    out = torch.full((m.info["rows"], m.info["cols"]), 77, dtype=torch.int8, device=dev)
    m.decompress(out.data_ptr(), _stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_matvec(m: tq.Matrix, bits: np.ndarray, dev, misalign: bool = False):
    batch = bits.shape[0]
    flat = torch.from_numpy(bits.view(np.int16).reshape(-1).copy())
    if misalign:   # same values at a 2-byte-aligned but not 16-byte-aligned address
        buf = torch.zeros(flat.numel() + 8, dtype=torch.int16, device=dev)
        buf[1:1 + flat.numel()] = flat.to(dev)
        x = buf[1:1 + flat.numel()]
    else:
        x = flat.to(dev)
    y = torch.full((batch, m.info["rows"]), float("nan"), dtype=torch.float32, device=dev)
    m.matvec(x.data_ptr(), y.data_ptr(), batch, _stream())
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check_outputs(y, ref, tol=1e-3):
    assert y.shape == ref.shape and np.isfinite(y).all()
    for b in range(ref.shape[0]):
        scale = np.abs(ref[b]).max()
        err = np.abs(y[b].astype(np.float64) - ref[b]).max()
        assert err <= tol * max(scale, 1e-30), (b, err, scale)
    return max(np.abs(y[b] - ref[b]).max() / max(np.abs(ref[b]).max(), 1e-30) for b in range(ref.shape[0]))


CASES = [
    # rows, cols, max_entries, lmax, seg_cols, dist
    (64, 512, 30719, 2, 64, "normal"),          # several units, dictionary not full
    (16, 8, 256, 2, 16, "normal"),              # one short segment per row, singles only
    (33, 300, 1000, 2, 32, "normal"),           # ragged rows and columns, last quad partly empty
    (17, 257, 300, 2, 256, "student_t4"),       # ragged, tiny dictionary, one-column last panel
    (48, 256, 300, 1, 48, "normal"),            # lmax 1: code == byte; segment width not a multiple of 32
    (200, 1024, 4096, 2, 128, "student_t4"),
    (512, 2048, 30719, 2, 256, "normal"),       # dictionary full and frozen; several bands per workgroup
    (1040, 768, 30719, 2, 192, "student_t4"),   # one quad per band
    (300, 3000, 30719, 2, 1024, "normal"),      # widest segments
    (4128, 1024, 30719, 2, 64, "normal"),       # more bands than CUs
    (2048, 2048, 30719, 2, 256, "normal"),      # config 1
]


@pytest.mark.parametrize("rows,cols,max_entries,lmax,seg_cols,dist", CASES)
def test_decompress_bit_exact_and_matvec(dev, rows, cols, max_entries, lmax, seg_cols, dist):
    spec = small_case(rows, cols, seed=rows * 7 + cols, dist=dist)
    W = make_weights(spec)
    Qo, so = O.quantize_rows(W)
    blob = tq.tq_encode(W, max_entries=max_entries, lmax=lmax, seg_cols=seg_cols)
    m = tq.Matrix(blob)
    try:
        Q = gpu_decompress(m, dev)
        assert np.array_equal(Q, Qo)
        for batch in (1, 3, 8, 16):
            bits, x = make_activations(spec, batch)
            y = gpu_matvec(m, bits, dev)
            ref = O.gemv_f64(Qo, so, x)
            worst = check_outputs(y, ref)
            assert worst < 1e-5      # fp32 accumulation of exact products: far inside the 1e-3 bar
    finally:
        m.close()


LONG_RUN_CASES = [
    # rows, cols, lmax, seg_cols, width, pack, what the weights are
    (64, 512, 3, 64, 8, False, "student"),
    (200, 1024, 4, 128, 8, False, "sparse"),          # 90 % zeros: runs of 4 zeros carry most of the matrix
    (33, 300, 4, 32, 8, False, "sparse"),             # ragged rows and columns
    (512, 2048, 4, 256, 4, False, "normal"),          # 4-bit levels one per byte: 15 distinct bytes
    (100, 768, 3, 64, 6, False, "normal"),
    (48, 1024, 4, 128, 4, True, "normal"),            # packed nibbles and long runs: the batched kernels at every batch
    (1040, 768, 4, 192, 8, False, "zero rows"),
    (17, 257, 4, 256, 8, False, "sparse"),            # one-column last panel
]


@pytest.mark.parametrize("rows,cols,lmax,seg_cols,width,pack,what", LONG_RUN_CASES)
def test_runs_of_three_and_four_bytes(dev, rows, cols, lmax, seg_cols, width, pack, what):
    """Containers whose dictionary holds runs of up to 4 bytes (sorted code space, two LDS slots per long entry):
    expansion bit-exact, products within the tolerance at batch 1 (the dot-product kernel's long form), 2, 3, 8 and 16
    (whole-strip kernels), aligned and misaligned activations, alone and as a prepared step."""
    spec = small_case(rows, cols, seed=rows * 11 + cols, dist="student_t4" if what == "student" else "normal")
    W = make_weights(spec)
    rng = np.random.default_rng(rows)
    if what == "sparse":
        W *= rng.random(W.shape) < 0.1
    if what == "zero rows":
        W[5] = 0
        W[rows - 1] = 0
        W[100:140] = 0
    Qo, so = O.quantize_rows(W, width)
    blob = tq.tq_encode(W, lmax=lmax, seg_cols=seg_cols, bits=0 if width == 8 else width, pack=pack)
    assert blob == O.build_blob(O.encode_matrix(W, lmax=lmax, seg_cols=seg_cols, bits=width, pack=pack))
    m = tq.Matrix(blob)
    try:
        assert m.info["lmax"] == lmax
        assert np.array_equal(gpu_decompress(m, dev), Qo)
        for batch in (1, 2, 3, 8, 16):
            bits, x = make_activations(spec, batch)
            ref = O.gemv_f64(Qo, so, x)
            assert check_outputs(gpu_matvec(m, bits, dev), ref) < 1e-5
            assert check_outputs(gpu_matvec(m, bits, dev, misalign=True), ref) < 1e-5
            xd = torch.from_numpy(bits.view(np.int16).copy()).to(dev)
            y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=dev)
            step = tq.Step([m.handle], [xd.data_ptr()], [y.data_ptr()], batch)
            step.launch(_stream())
            torch.cuda.synchronize()
            step.close()
            assert check_outputs(y.cpu().numpy(), ref) < 1e-5
        # unit vectors: every output is one weight times its scale, exactly; checks the column position of every run
        for j in (0, 1, 2, 3, cols // 2, cols - 2, cols - 1):
            xb = np.zeros((1, cols), np.float32)
            xb[0, j] = 1.0
            from inputs.synth import f32_to_bf16_bits
            y1 = gpu_matvec(m, f32_to_bf16_bits(xb), dev)
            assert np.array_equal(y1[0], (Qo[:, j].astype(np.float32) * so).astype(np.float32)), j
    finally:
        m.close()


def test_one_call_with_long_run_and_ordinary_matrices(dev):
    """A call that mixes containers with runs of up to 4 bytes, ordinary ones and packed ones is split by kind;
    every product and every expansion still comes out right, directly and as prepared steps."""
    shapes = [(64, 512, 4, False), (48, 256, 2, False), (80, 768, 3, False), (32, 512, 2, True), (96, 512, 4, True)]
    mats, xs, refs, Qs = [], [], [], []
    batch = 1
    for k, (rows, cols, lmax, pack) in enumerate(shapes):
        spec = small_case(rows, cols, seed=400 + k)
        W = make_weights(spec) * (np.random.default_rng(k).random((rows, cols)) < 0.3)
        width = 4 if pack else 8
        mats.append(tq.Matrix(tq.tq_encode(W, lmax=lmax, seg_cols=64, bits=0 if width == 8 else width, pack=pack)))
        Q, s = O.quantize_rows(W, width)
        bits, x = make_activations(spec, batch)
        xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
        refs.append(O.gemv_f64(Q, s, x))
        Qs.append(Q)
    hs = [m.handle for m in mats]
    try:
        for use_step in (False, True):
            ys = [torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev) for r, _, _, _ in shapes]
            outs = [torch.full((r, c), 77, dtype=torch.int8, device=dev) for r, c, _, _ in shapes]
            if use_step:
                st = tq.Step(hs, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch)
                sd = tq.Step(hs, None, [o.data_ptr() for o in outs], decompress=True)
                st.launch(_stream())
                sd.launch(_stream())
                torch.cuda.synchronize()
                st.close()
                sd.close()
            else:
                tq.tq_matvec_multi(hs, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch, _stream())
                tq.tq_decompress_multi(hs, [o.data_ptr() for o in outs], _stream())
                torch.cuda.synchronize()
            for y, ref, o, Q in zip(ys, refs, outs, Qs):
                check_outputs(y.cpu().numpy(), ref)
                assert np.array_equal(o.cpu().numpy(), Q)
    finally:
        for m in mats:
            m.close()


def test_oracle_made_container_decodes_on_gpu(dev):
    spec = small_case(96, 768, seed=5)
    W = make_weights(spec)
    enc = O.encode_matrix(W, max_entries=3000, seg_cols=64)
    m = tq.Matrix(O.build_blob(enc))
    try:
        assert np.array_equal(gpu_decompress(m, dev), enc.Q)
    finally:
        m.close()


def test_unit_vectors_probe_every_column_position(dev):
    """x = e_j gives y[r] = s[r] * Q[r, j] exactly: checks the column each decoded run lands on."""
    spec = small_case(32, 520, seed=11)
    W = make_weights(spec)
    Qo, so = O.quantize_rows(W)
    m = tq.Matrix(tq.tq_encode(W, max_entries=2000, seg_cols=64))
    try:
        cols = [0, 1, 7, 8, 63, 64, 65, 127, 128, 255, 256, 300, 511, 512, 519]
        for c0 in range(0, len(cols), 16):
            js = cols[c0:c0 + 16]
            x = np.zeros((len(js), 520), np.float32)
            for b, j in enumerate(js):
                x[b, j] = 1.0
            bits = (x.view(np.uint32) >> 16).astype(np.uint16)
            y = gpu_matvec(m, bits, dev)
            for b, j in enumerate(js):
                want = (so.astype(np.float64) * Qo[:, j]).astype(np.float32)
                assert np.array_equal(y[b], want), j
    finally:
        m.close()


def test_ones_vector_gives_exact_row_sums(dev):
    spec = small_case(64, 2048, seed=13)
    W = make_weights(spec)
    Qo, so = O.quantize_rows(W)
    m = tq.Matrix(tq.tq_encode(W))
    try:
        bits = np.full((1, 2048), 0x3F80, np.uint16)      # bf16 1.0
        y = gpu_matvec(m, bits, dev)
        want = (so.astype(np.float64) * Qo.sum(axis=1, dtype=np.int64)).astype(np.float32)
        np.testing.assert_allclose(y[0], want, rtol=2e-7, atol=0)
    finally:
        m.close()


def test_unaligned_activation_pointer_and_odd_columns(dev):
    for rows, cols in ((40, 300), (64, 512)):
        spec = small_case(rows, cols, seed=17)
        W = make_weights(spec)
        Qo, so = O.quantize_rows(W)
        m = tq.Matrix(tq.tq_encode(W, max_entries=1500))
        try:
            bits, x = make_activations(spec, 5)
            y = gpu_matvec(m, bits, dev, misalign=True)
            check_outputs(y, O.gemv_f64(Qo, so, x))
        finally:
            m.close()


def test_byte_transparent_including_minus_128(dev):
    rng = np.random.default_rng(2)
    Q = rng.integers(-128, 128, (48, 512), dtype=np.int8)
    Q[0, :] = -128
    Q[1, :] = 0
    Q[2, :] = 127
    s = (rng.random(48) + 0.5).astype(np.float32)
    m = tq.Matrix(tq.tq_encode_quantized(Q, s, max_entries=4000))
    try:
        assert np.array_equal(gpu_decompress(m, dev), Q)
        spec = small_case(48, 512, seed=19)
        bits, x = make_activations(spec, 2)
        check_outputs(gpu_matvec(m, bits, dev), O.gemv_f64(Q, s, x))
    finally:
        m.close()


def test_repeated_calls_are_deterministic_and_overwrite(dev):
    spec = small_case(128, 1024, seed=23)
    W = make_weights(spec)
    m = tq.Matrix(tq.tq_encode(W))
    try:
        bits, _ = make_activations(spec, 4)
        a = gpu_matvec(m, bits, dev)
        b = gpu_matvec(m, bits, dev)
        assert np.array_equal(a, b)
    finally:
        m.close()


def _multi_case(dev, shapes, batch, shared_dictionary, max_entries=3000):
    mats, xs, ys, refs, singles = [], [], [], [], []
    prev = None
    for k, (r, c, seg) in enumerate(shapes):
        spec = small_case(r, c, seed=100 + k)
        W = make_weights(spec)
        Qo, so = O.quantize_rows(W)
        blob = tq.tq_encode(W, max_entries=max_entries, seg_cols=seg, dict_from=prev if shared_dictionary else None)
        prev = blob
        m = tq.Matrix(blob)
        bits, x = make_activations(spec, batch)
        xd = torch.from_numpy(bits.view(np.int16).copy()).to(dev)
        mats.append(m)
        xs.append(xd)
        ys.append(torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev))
        refs.append(O.gemv_f64(Qo, so, x))
        singles.append(gpu_matvec(m, bits, dev))
    tq.tq_matvec_multi([m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch, _stream())
    torch.cuda.synchronize()
    for y, ref, one in zip(ys, refs, singles):
        got = y.cpu().numpy()
        check_outputs(got, ref)
        assert np.abs(got - one).max() <= 1e-5 * np.abs(ref).max()   # another split of the rows over the wavefronts
    for m in mats:
        m.close()


@pytest.mark.parametrize("shared_dictionary", [False, True])
def test_multi_launch_matches_single_launches_and_oracle(dev, shared_dictionary):
    """q/k/v/o/gate/down-like set of different shapes in one launch."""
    shapes = [(192, 768, 64), (64, 768, 64), (64, 768, 192), (48, 768, 64), (512, 768, 192), (192, 2048, 256)]
    for batch in (1, 8):
        _multi_case(dev, shapes, batch, shared_dictionary)


def test_multi_launch_splits_into_ring_and_whole_strip_launches(dev, ring_for_small_launches):
    """One call whose matrices go partly to the ring kernel (inherited dictionary, whole units, aligned activations) and
    partly to the whole-strip kernel (300 columns: no whole units)."""
    shapes = [(192, 768, 64), (64, 768, 64), (64, 768, 192), (40, 300, 32), (512, 768, 192), (192, 2048, 256), (100, 1024, 128)]
    for batch in (3, 8, 16):
        _multi_case(dev, shapes, batch, True)


def test_multi_launch_of_more_matrices_than_one_kernel_takes(dev):
    shapes = [(16 * (1 + k % 5), 256 + 64 * (k % 3), 64) for k in range(70)]
    _multi_case(dev, shapes, 2, True, max_entries=600)


def test_decompress_multi_is_bit_exact(dev):
    shapes = [(192, 768, 64), (40, 300, 32), (64, 768, 192), (48, 2048, 256), (512, 768, 192), (17, 257, 256)] * 25   # 150 > 128
    mats, outs, want = [], [], []
    prev = None
    for k, (r, c, seg) in enumerate(shapes):
        W = make_weights(small_case(r, c, seed=300 + k))
        prev = tq.tq_encode(W, max_entries=900, seg_cols=seg, dict_from=prev if k % 7 else None)
        mats.append(tq.Matrix(prev))
        outs.append(torch.full((r, c), 77, dtype=torch.int8, device=dev))
        want.append(O.quantize_rows(W)[0])
    tq.tq_decompress_multi([m.handle for m in mats], [o.data_ptr() for o in outs], _stream())
    torch.cuda.synchronize()
    for o, w in zip(outs, want):
        assert np.array_equal(o.cpu().numpy(), w)
    # the same expansion as a prepared step: 150 matrices in one launch instead of two
    step = tq.Step([m.handle for m in mats], None, [o.data_ptr() for o in outs], decompress=True)
    assert step.info["n_launches"] == 1 and step.info["n_matrices"] == len(mats)
    for o in outs:
        o.fill_(55)
    step.launch(_stream())
    torch.cuda.synchronize()
    for o, w in zip(outs, want):
        assert np.array_equal(o.cpu().numpy(), w)
    step.close()
    with pytest.raises(tq.TqError):
        tq.tq_step_create([mats[0].handle], None, [outs[0].data_ptr()], 1, tq.TQ_STEP_DECOMPRESS | tq.TQ_STEP_GATE_UP)
    with pytest.raises(tq.TqError):
        tq.tq_step_create([mats[0].handle], None, [outs[0].data_ptr()], 1, 0)        # products need activations
    for m in mats:
        m.close()


def _oracle_by_row_blocks(fn, n_rows, threads=16, block=4096):
    """The oracle, as it stands, on blocks of rows spread over host threads (rows are independent: quantization is per
    row, and so is every output of the product); returns the per-block results in row order."""
    from concurrent.futures import ThreadPoolExecutor
    cuts = [(a, min(n_rows, a + block)) for a in range(0, n_rows, block)]
    with ThreadPoolExecutor(threads) as pool:
        return list(pool.map(lambda ab: fn(*ab), cuts))


@pytest.mark.parametrize("config,width,pack,batches", [(4, 8, False, (1, 8)), (4, 8, False, (4, 16)), (4, 4, True, (1, 2, 4, 8, 16)),
                                                       (5, 8, False, (1, 16)), (3, 8, False, (1,)), (2, 8, False, (1,))])
def test_full_size_shapes_in_the_benchmarks_launch_configuration_every_row(dev, config, width, pack, batches):
    """Config-4 shapes at full size (one 3B layer plus lm_head 128256 x 3072), encoded as bench.py encodes them (one
    dictionary over the sequence, default options) and launched as bench.py launches them (all matrices in one
    tq_matvec_multi / tq_decompress_multi call, and as the prepared step), batch 1, 4, 8 and 16 (dot-product kernel,
    ring kernel with 11, 10 and 8 wavefronts: the call brings 9,744 bands, enough for the ring kernel).  Every row of
    every matrix is compared: the expansion with the oracle's quantized matrix byte for byte, every output with the
    oracle's float64 product.  Third case: the same shapes as packed 4-bit weights (bench.py --bits 4 --pack).  Then
    config 5 (the same shapes with Student-t weights, batch 1 and 16), config 3 (one LLaMA-3.2-1B layer plus its lm_head
    128256 x 2048) and config 2 (the 1B layer alone: a launch too small for the ring kernel)."""
    from inputs import config_matrices
    specs = [s for s in config_matrices(config) if config == 2 or s.name.startswith("L00.") or s.name == "lm_head"]
    assert len(specs) == (7 if config == 2 else 8) and (config == 2 or specs[-1].rows == 128256)
    mats, q_ref, s_ref = [], [], []
    prev = None
    for spec in specs:
        W = make_weights(spec)
        prev = tq.tq_encode(W, dict_from=prev, bits=0 if width == 8 else width, pack=pack)
        mats.append(tq.Matrix(prev))
        parts = _oracle_by_row_blocks(lambda a, b: O.quantize_rows(W[a:b], bits=width), spec.rows)
        q_ref.append(np.concatenate([p[0] for p in parts]))
        s_ref.append(np.concatenate([p[1] for p in parts]))
        del W
    if pack:
        assert all(m.info["packing"] == 1 and m.info["seg_cols"] == 128 for m in mats)
    else:
        assert mats[-1].info["n_entries"] == tq.TQ_MAX_ENTRIES_DEVICE and mats[-1].info["seg_cols"] == 256
    handles = [m.handle for m in mats]
    try:
        outs = [torch.full((sp.rows, sp.cols), 77, dtype=torch.int8, device=dev) for sp in specs]
        tq.tq_decompress_multi(handles, [o.data_ptr() for o in outs], _stream())
        torch.cuda.synchronize()
        for o, Qs in zip(outs, q_ref):
            assert torch.equal(o, torch.from_numpy(Qs).to(dev))          # the whole matrix, bit for bit
        del outs
        if config == 4 and not pack:
            assert all(m.info["lane_spread"] <= 113 for m in mats)   # none of them needs the whole-strip kernel
        for batch in batches:
            xs, ys, refs = [], [], []
            for sp, Qs, ss in zip(specs, q_ref, s_ref):
                bits, x = make_activations(sp, batch)
                xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
                ys.append(torch.full((batch, sp.rows), float("nan"), dtype=torch.float32, device=dev))
                refs.append(np.concatenate(_oracle_by_row_blocks(lambda a, b: O.gemv_f64(Qs[a:b], ss[a:b], x), sp.rows), axis=1))
            step = tq.Step(handles, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch)   # what bench.py times
            for through_step in (False, True):
                for y in ys:
                    y.fill_(float("nan"))
                if through_step:
                    step.launch(_stream())
                else:
                    tq.tq_matvec_multi(handles, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch, _stream())
                torch.cuda.synchronize()
                for y, ref in zip(ys, refs):
                    got = y.cpu().numpy()
                    assert got.shape == ref.shape and np.isfinite(got).all()
                    scale = np.abs(ref).max(axis=1, keepdims=True)
                    assert (np.abs(got - ref) <= 1e-3 * scale).all()
                    assert (np.abs(got - ref) <= 1e-5 * scale).all()   # what fp32 accumulation of exact products gives
            step.close()
    finally:
        for m in mats:
            m.close()


RING_SPREAD_LIMIT = 65   # lane_spread up to which the batched product keeps a 128-byte ring per lane instead of the whole segment


def test_batched_product_ring_and_whole_strip_kernels_agree(dev, ring_for_small_launches):
    """A matrix encoded with an inherited, full dictionary keeps its 64 lanes close together (lane_spread small): with
    16-byte aligned activations its batched product runs on the ring kernel, with misaligned ones on the whole-strip
    kernel.  Both must match the oracle, for every batch size that takes these kernels, over several bands, several
    quads, rows past the last band's end, and 1, 2 and 8 windows per segment."""
    first = tq.tq_encode(make_weights(small_case(256, 1024, seed=900)), max_entries=3000, seg_cols=64)
    for rows, cols, seg in [(200, 2048, 256), (1000, 512, 64), (96, 1024, 128), (40, 256, 32)]:
        spec = small_case(rows, cols, seed=901 + rows)
        W = make_weights(spec)
        blob = tq.tq_encode(W, max_entries=3000, seg_cols=seg, dict_from=first)
        info = tq.tq_validate_blob(blob)
        assert info["lane_spread"] <= RING_SPREAD_LIMIT and cols % (4 * seg) == 0, info
        Qo, so = O.quantize_rows(W)
        m = tq.Matrix(blob)
        try:
            for batch in (3, 5, 8, 16):        # (batch 2 of these matrices runs on the dot-product kernel)
                bits, x = make_activations(spec, batch)
                ref = O.gemv_f64(Qo, so, x)
                ring = gpu_matvec(m, bits, dev)
                strip = gpu_matvec(m, bits, dev, misalign=True)
                check_outputs(ring, ref)
                check_outputs(strip, ref)
                assert np.abs(ring - strip).max() <= 1e-5 * np.abs(ref).max()
                assert np.array_equal(ring, gpu_matvec(m, bits, dev))   # the atomic adds come in a fixed order
        finally:
            m.close()


def test_matrix_that_starts_a_dictionary_takes_the_careful_ring_mode(dev, ring_for_small_launches):
    """The first segments of a matrix that starts from the 256 single bytes are nearly all singles, later ones nearly all
    pairs: the lanes of the first units are further apart than the ring absorbs in groups of 4 windows, but not further
    than it absorbs window by window."""
    spec = small_case(128, 1024, seed=950)
    W = make_weights(spec)
    blob = tq.tq_encode(W, seg_cols=256)
    spread = tq.tq_validate_blob(blob)["lane_spread"]
    assert RING_SPREAD_LIMIT < spread <= 113, spread
    Qo, so = O.quantize_rows(W)
    m = tq.Matrix(blob)
    try:
        for batch in (2, 8, 16):
            bits, x = make_activations(spec, batch)
            ref = O.gemv_f64(Qo, so, x)
            ring = gpu_matvec(m, bits, dev)
            check_outputs(ring, ref)
            assert np.abs(ring - gpu_matvec(m, bits, dev, misalign=True)).max() <= 1e-5 * np.abs(ref).max()
    finally:
        m.close()


@pytest.mark.parametrize("width", [6, 4, 2])
def test_lower_quantization_widths_through_the_same_path(dev, ring_for_small_launches, width):
    """Paper section 3: 6-, 4- and 2-bit (ternary) levels.  One value per byte, same container and kernels: the expansion
    is the oracle's quantized matrix bit for bit, the products match its float64 definition."""
    spec = small_case(272, 2048, seed=960 + width)
    W = make_weights(spec)
    Qo, so = O.quantize_rows(W, bits=width)
    m = tq.Matrix(tq.tq_encode(W, bits=width))
    try:
        assert np.array_equal(gpu_decompress(m, dev), Qo)
        for batch in (1, 3, 16):
            bits, x = make_activations(spec, batch)
            check_outputs(gpu_matvec(m, bits, dev), O.gemv_f64(Qo, so, x))
    finally:
        m.close()


PACKED_CASES = [
    # rows, cols, bits, seg_cols (bytes), dictionary
    (64, 1024, 4, 64, "lzw"),            # whole units
    (16, 32, 4, 16, "lzw"),              # one segment per row
    (33, 600, 4, 32, "lzw"),             # ragged rows, last quad partly empty, cols / 2 not a multiple of 8
    (17, 514, 3, 256, "lzw"),            # one-byte last panel
    (272, 2048, 4, 128, "frequency"),    # the default segment width, several bands per wavefront
    (100, 4096, 2, 128, "lzw"),          # ternary
    (1027, 1536, 4, 128, "lzw"),         # more bands than wavefronts
]


@pytest.mark.parametrize("rows,cols,width,seg_cols,dictionary", PACKED_CASES)
def test_packed_four_bit_weights(dev, rows, cols, width, seg_cols, dictionary):
    """Two 4-bit values per stored byte: the expansion gives the oracle's quantized matrix bit for bit (one int8 per weight),
    the products match its float64 definition, at batch 1 (fp8 dictionary image, two dot products per code) and at
    batches on the MFMA kernel, with aligned and misaligned activations."""
    spec = small_case(rows, cols, seed=970 + rows)
    W = make_weights(spec)
    Qo, so = O.quantize_rows(W, bits=width)
    m = tq.Matrix(tq.tq_encode(W, bits=width, seg_cols=seg_cols, dictionary=dictionary, pack=True))
    try:
        assert m.info["packing"] == 1 and (m.info["rows"], m.info["cols"]) == (rows, cols)
        assert np.array_equal(gpu_decompress(m, dev), Qo)
        for batch in (1, 2, 5, 16):
            bits, x = make_activations(spec, batch)
            ref = O.gemv_f64(Qo, so, x)
            check_outputs(gpu_matvec(m, bits, dev), ref)
            check_outputs(gpu_matvec(m, bits, dev, misalign=True), ref)
    finally:
        m.close()


def test_packed_weights_on_the_ring_kernel(dev, ring_for_small_launches):
    """Whole units of packed bytes with the lanes close together: aligned activations take the ring kernel (two MFMA steps
    per 8-byte piece), misaligned ones the whole-strip kernel; both match the oracle.  The first matrix starts its
    dictionary (lanes further apart: careful mode or whole strips), the others inherit a full one."""
    first_spec = small_case(256, 1024, seed=995)
    first = tq.tq_encode(make_weights(first_spec), bits=4, seg_cols=64, pack=True)
    cases = [(first_spec, first)]
    for rows, cols, seg in [(200, 2048, 128), (1000, 512, 64), (96, 1024, 128), (40, 256, 32)]:
        spec = small_case(rows, cols, seed=996 + rows)
        cases.append((spec, tq.tq_encode(make_weights(spec), bits=4, seg_cols=seg, pack=True, dict_from=first)))
    spreads = []
    for spec, blob in cases:
        info = tq.tq_validate_blob(blob)
        spreads.append(info["lane_spread"])
        assert (spec.cols // 2) % (4 * info["seg_cols"]) == 0
        Qo, so = O.quantize_rows(make_weights(spec), bits=4)
        m = tq.Matrix(blob)
        try:
            for batch in (2, 5, 8, 16):
                bits, x = make_activations(spec, batch)
                ref = O.gemv_f64(Qo, so, x)
                ring = gpu_matvec(m, bits, dev)
                strip = gpu_matvec(m, bits, dev, misalign=True)
                check_outputs(ring, ref)
                check_outputs(strip, ref)
                assert np.abs(ring - strip).max() <= 1e-5 * np.abs(ref).max()
                assert np.array_equal(ring, gpu_matvec(m, bits, dev))
        finally:
            m.close()
    assert min(spreads[1:]) <= RING_SPREAD_LIMIT, spreads       # at least these run in groups of four pieces


def test_two_activation_rows_on_the_dot_product_kernel(dev):
    """Batch 2 of one-weight-per-byte matrices: both rows in the LDS image, one dot product per row and code.  Unit
    vectors in either row land on the right column of the right output row; ragged shapes, an odd number of columns
    (second row misaligned), shared bands, gate/up pairs."""
    for rows, cols, seg in [(64, 512, 64), (33, 301, 32), (17, 257, 256), (1027, 2048, 256), (200, 768, 192)]:
        spec = small_case(rows, cols, seed=940 + rows)
        W = make_weights(spec)
        Qo, so = O.quantize_rows(W)
        m = tq.Matrix(tq.tq_encode(W, seg_cols=seg, max_entries=4000))
        try:
            bits, x = make_activations(spec, 2)
            ref = O.gemv_f64(Qo, so, x)
            for mis in (False, True):
                got = gpu_matvec(m, bits, dev, misalign=mis)
                check_outputs(got, ref)
                assert (np.abs(got - ref) <= 1e-5 * np.abs(ref).max(axis=1, keepdims=True)).all()
            one = np.stack([gpu_matvec(m, bits[b:b + 1], dev)[0] for b in range(2)])      # each row alone, batch-1 kernel
            assert np.abs(gpu_matvec(m, bits, dev) - one).max() <= 1e-5 * np.abs(ref).max()
            e = np.zeros((2, cols), np.float32)
            for j0, j1 in ((0, cols - 1), (1, 2), (cols // 2, cols // 2 + 1)):
                e[:] = 0
                e[0, j0], e[1, j1] = 1.0, -2.0
                y = gpu_matvec(m, (e.view(np.uint32) >> 16).astype(np.uint16), dev)
                assert np.array_equal(y[0], so * Qo[:, j0].astype(np.float32)), (rows, cols, j0)
                assert np.array_equal(y[1], so * (-2.0 * Qo[:, j1].astype(np.float32))), (rows, cols, j1)
        finally:
            m.close()
    sg, su = small_case(120, 640, seed=946), small_case(120, 640, seed=947)
    Wg, Wu = make_weights(sg), make_weights(su)
    m = tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, seg_cols=64))
    try:
        bits, x = make_activations(sg, 2)
        check_outputs(_gpu_gate_up(m, bits, dev, 120), O.gate_up_f64(*O.quantize_rows(Wg), *O.quantize_rows(Wu), x))
    finally:
        m.close()


def test_two_activation_rows_of_packed_weights(dev):
    """Batch 2 of packed 4-bit matrices on the dot-product kernel (two dwords per byte column in the LDS image): ragged
    shapes, misaligned activations, shared bands, unit vectors in either row, every nibble value; a row too long for the
    doubled image goes to the batched kernels and gives the same result."""
    for rows, cols, seg in [(64, 512, 64), (33, 302, 32), (17, 258, 128), (1027, 2048, 128), (200, 768, 96), (32, 49152, 128)]:
        spec = small_case(rows, cols, seed=960 + rows)
        W = make_weights(spec)
        Qo, so = O.quantize_rows(W, 4)
        m = tq.Matrix(tq.tq_encode(W, seg_cols=seg, max_entries=4000, bits=4, pack=True))
        try:
            assert np.array_equal(gpu_decompress(m, dev), Qo)
            bits, x = make_activations(spec, 2)
            ref = O.gemv_f64(Qo, so, x)
            for mis in (False, True):
                got = gpu_matvec(m, bits, dev, misalign=mis)
                check_outputs(got, ref)
                assert (np.abs(got - ref) <= 1e-5 * np.abs(ref).max(axis=1, keepdims=True)).all()
            one = np.stack([gpu_matvec(m, bits[b:b + 1], dev)[0] for b in range(2)])      # each row alone, batch-1 kernel
            assert np.abs(gpu_matvec(m, bits, dev) - one).max() <= 1e-5 * np.abs(ref).max()
            e = np.zeros((2, cols), np.float32)
            for j0, j1 in ((0, cols - 1), (1, 2), (cols // 2, cols // 2 + 1), (3, 0)):
                e[:] = 0
                e[0, j0], e[1, j1] = 1.0, -2.0
                y = gpu_matvec(m, (e.view(np.uint32) >> 16).astype(np.uint16), dev)
                assert np.array_equal(y[0], so * Qo[:, j0].astype(np.float32)), (rows, cols, j0)
                assert np.array_equal(y[1], so * (-2.0 * Qo[:, j1].astype(np.float32))), (rows, cols, j1)
        finally:
            m.close()
    rng = np.random.default_rng(13)
    Q = rng.integers(-8, 8, (48, 512), dtype=np.int8)
    Q[0, :16] = np.arange(-8, 8)
    s = (rng.random(48) + 0.5).astype(np.float32)
    m = tq.Matrix(tq.tq_encode_quantized(Q, s, seg_cols=64, pack=True))
    try:
        bits, x = make_activations(small_case(48, 512, seed=972), 2)
        check_outputs(gpu_matvec(m, bits, dev), O.gemv_f64(Q, s, x), tol=1e-5)
    finally:
        m.close()
    sg, su = small_case(120, 640, seed=948), small_case(120, 640, seed=949)
    Wg, Wu = make_weights(sg), make_weights(su)
    m = tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, seg_cols=64, bits=4, pack=True))
    try:
        bits, x = make_activations(sg, 2)
        check_outputs(_gpu_gate_up(m, bits, dev, 120), O.gate_up_f64(*O.quantize_rows(Wg, 4), *O.quantize_rows(Wu, 4), x))
    finally:
        m.close()


def test_rows_too_long_for_the_activation_image_run_on_the_batched_kernels(dev, monkeypatch):
    """A row whose LDS image does not fit beside the dictionary is not refused: batch 1 and 2 then run on the kernels that
    serve the larger batches (whole-strip, or ring when the launch is large enough).  Alone, as a prepared step, mixed
    with ordinary matrices in one call (the call is split), as a gate/up pair, packed."""
    cases = [(96, 28672, 256, 12000, 8, False), (64, 65536, 256, 2000, 8, False), (48, 98304, 128, 4000, 4, True)]
    for rows, cols, seg, me, width, pack in cases:
        spec = small_case(rows, cols, seed=7000 + rows)
        W = make_weights(spec)
        Qo, so = O.quantize_rows(W, width)
        m = tq.Matrix(tq.tq_encode(W, seg_cols=seg, max_entries=me, bits=0 if width == 8 else width, pack=pack))
        small = small_case(80, 512, seed=7100 + rows)
        Ws = make_weights(small)
        Qs, ss = O.quantize_rows(Ws, width)
        m_small = tq.Matrix(tq.tq_encode(Ws, seg_cols=64, max_entries=me, bits=0 if width == 8 else width, pack=pack))
        try:
            assert np.array_equal(gpu_decompress(m, dev), Qo)
            for ring_min in (24, 0):        # 0: the ring kernel takes the launch whatever its size
                tq.tq_set_ring_min_bands_per_cu(ring_min)
                for batch in (1, 2, 8):
                    bits, x = make_activations(spec, batch)
                    ref = O.gemv_f64(Qo, so, x)
                    check_outputs(gpu_matvec(m, bits, dev), ref)
                    check_outputs(gpu_matvec(m, bits, dev, misalign=True), ref)
                    bs, xsm = make_activations(small, batch)
                    xd = [torch.from_numpy(b.view(np.int16).copy()).to(dev) for b in (bs, bits, bs)]
                    yd = [torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev) for r in (80, rows, 80)]
                    hs = [m_small.handle, m.handle, m_small.handle]
                    tq.tq_matvec_multi(hs, [t.data_ptr() for t in xd], [t.data_ptr() for t in yd], batch, _stream())
                    torch.cuda.synchronize()
                    for y, r in zip(yd, (O.gemv_f64(Qs, ss, xsm), ref, O.gemv_f64(Qs, ss, xsm))):
                        check_outputs(y.cpu().numpy(), r)
                    step = tq.Step(hs, [t.data_ptr() for t in xd], [t.data_ptr() for t in yd], batch)
                    try:
                        for y in yd:
                            y.fill_(float("nan"))
                        step.launch(_stream())
                        torch.cuda.synchronize()
                    finally:
                        step.close()
                    for y, r in zip(yd, (O.gemv_f64(Qs, ss, xsm), ref, O.gemv_f64(Qs, ss, xsm))):
                        check_outputs(y.cpu().numpy(), r)
        finally:
            m.close()
            m_small.close()
    sg, su = small_case(40, 65536, seed=7201), small_case(40, 65536, seed=7202)
    Wg, Wu = make_weights(sg), make_weights(su)
    m = tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, max_entries=2000))
    try:
        for batch in (1, 2):
            bits, x = make_activations(sg, batch)
            check_outputs(_gpu_gate_up(m, bits, dev, 40), O.gate_up_f64(*O.quantize_rows(Wg), *O.quantize_rows(Wu), x))
    finally:
        m.close()


def test_packed_weights_take_every_nibble_value(dev):
    """All 16 nibble values, -8 included (the quantizer never makes it, a container may hold it): the batch-1 kernel's fp8
    image and the MFMA kernel's conversion are exact for each."""
    rng = np.random.default_rng(12)
    Q = rng.integers(-8, 8, (48, 512), dtype=np.int8)
    Q[0, :16] = np.arange(-8, 8)
    s = (rng.random(48) + 0.5).astype(np.float32)
    m = tq.Matrix(tq.tq_encode_quantized(Q, s, seg_cols=64, pack=True))
    try:
        assert np.array_equal(gpu_decompress(m, dev), Q)
        spec = small_case(48, 512, seed=971)
        for batch in (1, 4):
            bits, x = make_activations(spec, batch)
            check_outputs(gpu_matvec(m, bits, dev), O.gemv_f64(Q, s, x), tol=1e-5)
        e = np.zeros((1, 512), np.float32)          # unit vectors: every column lands where it belongs
        for j in (0, 1, 2, 15, 127, 128, 129, 511):
            e[:] = 0
            e[0, j] = 1.0
            bits = (e.view(np.uint32) >> 16).astype(np.uint16)
            y = gpu_matvec(m, bits, dev)
            assert np.array_equal(y[0], s * Q[:, j].astype(np.float32)), j      # one fp32 product per row: exact
    finally:
        m.close()


def test_one_call_with_packed_and_plain_matrices(dev):
    shapes = [(192, 768, 4, True), (64, 768, 8, False), (64, 1024, 4, True), (48, 768, 6, False), (512, 768, 2, True)]
    for batch in (1, 8):
        mats, xs, ys, refs = [], [], [], []
        for k, (r, c, width, pack) in enumerate(shapes):
            spec = small_case(r, c, seed=980 + k)
            W = make_weights(spec)
            Qo, so = O.quantize_rows(W, bits=width)
            mats.append(tq.Matrix(tq.tq_encode(W, bits=width, seg_cols=64, pack=pack)))
            bits, x = make_activations(spec, batch)
            refs.append(O.gemv_f64(Qo, so, x))
            xs.append(torch.from_numpy(bits.view(np.int16).reshape(-1).copy()).to(dev))
            ys.append(torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev))
        tq.tq_matvec_multi([m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch, _stream())
        torch.cuda.synchronize()
        for y, ref in zip(ys, refs):
            check_outputs(y.cpu().numpy(), ref)
        outs = [torch.full((r, c), 77, dtype=torch.int8, device=dev) for (r, c, _, _) in shapes]
        tq.tq_decompress_multi([m.handle for m in mats], [o.data_ptr() for o in outs], _stream())
        torch.cuda.synchronize()
        for k, (r, c, width, _) in enumerate(shapes):
            assert np.array_equal(outs[k].cpu().numpy(), O.quantize_rows(make_weights(small_case(r, c, seed=980 + k)), bits=width)[0])
        for m in mats:
            m.close()


def test_packed_gate_up(dev):
    sg, su = small_case(200, 768, seed=990), small_case(200, 768, seed=991)
    Wg, Wu = make_weights(sg), make_weights(su)
    m = tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, bits=4, pack=True))
    try:
        for batch in (1, 6):
            bits, x = make_activations(sg, batch)
            ref = O.gate_up_f64(*O.quantize_rows(Wg, bits=4), *O.quantize_rows(Wu, bits=4), x)
            check_outputs(_gpu_gate_up(m, bits, dev, 200), ref)
    finally:
        m.close()


def _gpu_gate_up(m, bits, dev, rows):
    batch = bits.shape[0]
    x = torch.from_numpy(bits.view(np.int16).reshape(-1).copy()).to(dev)
    y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=dev)
    tq.tq_matvec_gate_up(m.handle, x.data_ptr(), y.data_ptr(), batch, _stream())
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("rows,cols,seg_cols", [(8, 64, 16), (100, 768, 64), (1027, 2048, 256), (520, 1000, 128)])
def test_gate_up_product_with_fused_silu(dev, rows, cols, seg_cols):
    """silu(W_gate x) * (W_up x) from one container of interleaved rows, against the float64 definition: batch 1
    (dot-product kernel) and batched (whole-strip MFMA kernel), bands that end in the middle of a pair's band included."""
    sg, su = small_case(rows, cols, seed=70), small_case(rows, cols, seed=71)
    Wg, Wu = make_weights(sg), make_weights(su)
    Qg, scg = O.quantize_rows(Wg)
    Qu, scu = O.quantize_rows(Wu)
    m = tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, seg_cols=seg_cols))
    try:
        assert m.info["rows"] == 2 * rows
        assert np.array_equal(gpu_decompress(m, dev), O.interleave_rows(Qg, Qu))
        for batch in (1, 3, 16):
            bits, x = make_activations(sg, batch)
            got = _gpu_gate_up(m, bits, dev, rows)
            check_outputs(got, O.gate_up_f64(Qg, scg, Qu, scu, x))
            assert np.array_equal(got, _gpu_gate_up(m, bits, dev, rows))
    finally:
        m.close()


def test_gate_up_multi_and_argument_errors(dev):
    pairs = [(64, 512, 64), (200, 768, 192), (48, 2048, 256)]
    mats, refs, xs, ys = [], [], [], []
    batch = 4
    for k, (r, c, seg) in enumerate(pairs):
        sg, su = small_case(r, c, seed=80 + 2 * k), small_case(r, c, seed=81 + 2 * k)
        Wg, Wu = make_weights(sg), make_weights(su)
        mats.append(tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, seg_cols=seg, max_entries=2000)))
        bits, x = make_activations(sg, batch)
        xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
        ys.append(torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev))
        refs.append(O.gate_up_f64(*O.quantize_rows(Wg), *O.quantize_rows(Wu), x))
    tq.tq_matvec_gate_up_multi([m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch, _stream())
    torch.cuda.synchronize()
    for y, ref in zip(ys, refs):
        check_outputs(y.cpu().numpy(), ref)
    odd = tq.Matrix(tq.tq_encode(make_weights(small_case(17, 64, seed=90)), seg_cols=16))
    with pytest.raises(tq.TqError) as e:
        tq.tq_matvec_gate_up(odd.handle, xs[0].data_ptr(), ys[0].data_ptr(), 1, _stream())
    assert e.value.code == -1
    for m in mats + [odd]:
        m.close()


def test_frequency_dictionary_containers_on_the_device(dev, ring_for_small_launches):
    """Same container, same kernels: a dictionary picked by frequency decodes bit-exactly and multiplies within
    tolerance (dot-product kernel, ring kernel - such a matrix has no start-up phase of single bytes, its lanes stay
    close - and whole-strip kernel through misaligned activations)."""
    spec = small_case(256, 2048, seed=61)
    W = make_weights(spec)
    blob = tq.tq_encode(W, dictionary="frequency")
    lzw = tq.tq_validate_blob(tq.tq_encode(W))
    info = tq.tq_validate_blob(blob)
    assert info["lane_spread"] <= RING_SPREAD_LIMIT < lzw["lane_spread"] and info["n_real_codes"] < lzw["n_real_codes"]
    Qo, so = O.quantize_rows(W)
    m = tq.Matrix(blob)
    try:
        assert np.array_equal(gpu_decompress(m, dev), Qo)
        for batch in (1, 8, 16):
            bits, x = make_activations(spec, batch)
            ref = O.gemv_f64(Qo, so, x)
            check_outputs(gpu_matvec(m, bits, dev), ref)
            check_outputs(gpu_matvec(m, bits, dev, misalign=True), ref)
    finally:
        m.close()


def test_lanes_far_apart_fall_back_to_the_whole_strip_kernel(dev):
    """All-zero rows (every code a pair once the dictionary knows the pair of zeros) next to rows of values the small
    frozen dictionary has no pairs for (every code a single): the lanes of a unit drift far apart, lane_spread exceeds
    what a ring can absorb, and the batched product must still be exact through the whole-strip kernel."""
    rng = np.random.default_rng(5)
    rows, cols = 64, 2048
    Q = rng.integers(-127, 128, size=(rows, cols), dtype=np.int8)
    Q[::2] = 0
    scales = rng.uniform(0.5, 2.0, rows).astype(np.float32)
    blob = tq.tq_encode_quantized(Q, scales, max_entries=300, seg_cols=256)
    info = tq.tq_validate_blob(blob)
    assert info["lane_spread"] > 113, info   # more than the ring absorbs even window by window
    spec = small_case(rows, cols, seed=77)
    m = tq.Matrix(blob)
    try:
        assert np.array_equal(gpu_decompress(m, dev), Q)
        for batch in (1, 8):
            bits, x = make_activations(spec, batch)
            check_outputs(gpu_matvec(m, bits, dev), O.gemv_f64(Q, scales, x))
    finally:
        m.close()


def test_launches_can_be_captured_in_a_hip_graph_and_replayed(dev):
    """The launch calls allocate nothing and do not synchronise: a captured step replays to the eager results, every
    time, with eager work of the same kernels in between."""
    shapes = [(192, 768, 64), (64, 768, 192), (48, 2048, 256)]
    for batch in (1, 4):
        mats, xs, ys = [], [], []
        prev = None
        for k, (r, c, seg) in enumerate(shapes):
            spec = small_case(r, c, seed=400 + k)
            prev = tq.tq_encode(make_weights(spec), max_entries=2000, seg_cols=seg, dict_from=prev)
            mats.append(tq.Matrix(prev))
            bits, _ = make_activations(spec, batch)
            xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
            ys.append(torch.zeros((batch, r), dtype=torch.float32, device=dev))
        hs, xp, yp = [m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
        out = torch.zeros((48, 2048), dtype=torch.int8, device=dev)
        tq.tq_matvec_multi(hs, xp, yp, batch, _stream())
        mats[2].decompress(out.data_ptr(), _stream())
        torch.cuda.synchronize()
        want_y, want_q = [y.clone() for y in ys], out.clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            cap = torch.cuda.current_stream().cuda_stream
            tq.tq_matvec_multi(hs, xp, yp, batch, cap)
            tq.tq_matvec(hs[0], xp[0], yp[0], batch, cap)
            tq.tq_decompress(hs[2], out.data_ptr(), cap)
        for _ in range(3):
            for y in ys:
                y.fill_(-1.0)          # fill kernels, not memsets
            out.fill_(9)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for y, w in zip(ys[1:], want_y[1:]):
                assert torch.equal(y, w)
            assert torch.equal(out, want_q)
            check = torch.zeros_like(ys[0])
            tq.tq_matvec(hs[0], xp[0], check.data_ptr(), batch, _stream())    # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(ys[0], check)
        del graph
        for m in mats:
            m.close()


def _step_case(dev, shapes, batch, max_entries=900, widths=None):
    """The same matrices through tq_matvec_multi and through a prepared step; both against the oracle."""
    mats, xs, ys, y2, refs = [], [], [], [], []
    prev = {}
    for k, (r, c, seg) in enumerate(shapes):
        spec = small_case(r, c, seed=600 + k)
        W = make_weights(spec)
        width, pack = widths[k % len(widths)] if widths else (8, False)
        Qo, so = O.quantize_rows(W, bits=width)
        blob = tq.tq_encode(W, max_entries=max_entries, seg_cols=seg // 2 if pack else seg, dict_from=prev.get(pack) if k % 9 else None,
                            bits=0 if width == 8 else width, pack=pack)
        prev[pack] = blob
        mats.append(tq.Matrix(blob))
        bits, x = make_activations(spec, batch)
        xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
        ys.append(torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev))
        y2.append(torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev))
        refs.append(O.gemv_f64(Qo, so, x))
    hs, xp = [m.handle for m in mats], [x.data_ptr() for x in xs]
    step = tq.Step(hs, xp, [y.data_ptr() for y in ys], batch)
    assert step.info["n_matrices"] == len(shapes) and step.info["table_bytes"] % len(shapes) == 0
    tq.tq_matvec_multi(hs, xp, [y.data_ptr() for y in y2], batch, _stream())
    for _ in range(2):                       # a step can be launched again and again
        for y in ys:
            y.fill_(float("nan"))
        step.launch(_stream())
        torch.cuda.synchronize()
        for y, other, ref in zip(ys, y2, refs):
            got = y.cpu().numpy()
            check_outputs(got, ref)
            assert np.abs(got - other.cpu().numpy()).max() <= 1e-5 * np.abs(ref).max()
    n_launches = step.info["n_launches"]
    step.close()
    for m in mats:
        m.close()
    return n_launches


def test_prepared_step_serves_more_matrices_per_launch_than_the_kernel_arguments_hold(dev):
    shapes = [(16 * (1 + k % 5), 256 + 64 * (k % 3), 64) for k in range(150)]
    assert _step_case(dev, shapes, 1) == 1                      # tq_matvec_multi needs two launches for 150 matrices
    assert _step_case(dev, shapes, 4) == 1


def test_prepared_step_with_ring_whole_strip_and_packed_matrices(dev, ring_for_small_launches):
    """One step whose matrices go to different kernels: ring (whole units), whole strip (300 columns), packed 4-bit."""
    shapes = [(192, 768, 64), (64, 768, 64), (64, 768, 192), (40, 300, 32), (512, 768, 192), (192, 2048, 256), (100, 1024, 128)]
    for batch in (1, 3, 16):
        n = _step_case(dev, shapes, batch, max_entries=3000, widths=[(8, False), (8, False), (4, True)])
        assert n >= 2


def test_prepared_step_of_gate_up_pairs_in_a_hip_graph(dev):
    pairs = [(64, 512, 64), (200, 768, 192), (48, 2048, 256)]
    for batch in (1, 4):
        mats, refs, xs, ys = [], [], [], []
        for k, (r, c, seg) in enumerate(pairs):
            sg, su = small_case(r, c, seed=680 + 2 * k), small_case(r, c, seed=681 + 2 * k)
            Wg, Wu = make_weights(sg), make_weights(su)
            mats.append(tq.Matrix(tq.tq_encode_gate_up(Wg, Wu, seg_cols=seg, max_entries=2000)))
            bits, x = make_activations(sg, batch)
            xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
            ys.append(torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev))
            refs.append(O.gate_up_f64(*O.quantize_rows(Wg), *O.quantize_rows(Wu), x))
        step = tq.Step([m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], batch, gate_up=True)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step.launch(torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            for y in ys:
                y.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for y, ref in zip(ys, refs):
                check_outputs(y.cpu().numpy(), ref)
            step.launch(_stream())           # eager work between the replays
            torch.cuda.synchronize()
        del graph
        step.close()
        for m in mats:
            m.close()


def _staged_case(dev, batch, shapes_by_stage, seed, pack=False):
    mats, xs, ys, refs, stages, prev = [], [], [], [], [], None
    for st, shapes in enumerate(shapes_by_stage):
        for rows, cols in shapes:
            spec = small_case(rows, cols, seed=seed + len(mats))
            W = make_weights(spec)
            prev = tq.tq_encode(W, seg_cols=64, max_entries=4000, dict_from=prev, bits=4 if pack else 0, pack=pack)
            mats.append(tq.Matrix(prev))
            bits, x = make_activations(spec, batch)
            xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
            ys.append(torch.full((batch, rows), float("nan"), dtype=torch.float32, device=dev))
            Q, s = O.quantize_rows(W, 4 if pack else 8)
            refs.append(O.gemv_f64(Q, s, x))
            stages.append(st)
    return mats, xs, ys, refs, stages


@pytest.mark.parametrize("batch,pack", [(1, False), (2, False), (1, True)])
def test_staged_step_runs_dependent_products_in_one_launch(dev, batch, pack):
    """Products in stages (the shapes of two small transformer layers: q,k,v | o | gate,up | down, then a head): one
    kernel launch walks the stages with a device-side hand-over between them; every product against the oracle, on
    repeated launches, and equal to the plain prepared step bit for bit (same kernels, same split per stage or not,
    the sums of a row are the same numbers: checked to the tolerance, and for determinism against itself)."""
    layer = [[(256, 512), (64, 512), (64, 512)], [(256, 256)], [(1024, 256), (1024, 256)], [(256, 1024)]]
    mats, xs, ys, refs, stages = _staged_case(dev, batch, layer + layer + [[(4000, 256)]], 12000, pack)
    hs, xp, yp = [m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
    step = tq.Step(hs, xp, yp, batch, stages=stages)
    try:
        assert step.info["persistent"] == 1 and step.info["n_launches"] == 1 and step.info["n_stages"] == 9
        first = None
        for rep in range(3):
            for y in ys:
                y.fill_(float("nan"))
            step.launch(_stream())
            torch.cuda.synchronize()
            got = [y.cpu().numpy() for y in ys]
            for g, ref in zip(got, refs):
                assert check_outputs(g, ref) < 1e-5
            if first is None:
                first = got
            assert all(np.array_equal(a, b) for a, b in zip(first, got))
        assert tq.tq_step_get_info(step.handle)["fault"] == 0
    finally:
        step.close()
        for m in mats:
            m.close()


def test_staged_step_in_a_hip_graph(dev):
    """The staged launch (a fill kernel for the stage counters, then the persistent kernel) captured into a graph and
    replayed, with eager launches of the same step between the replays: every replay against the oracle."""
    layer = [[(256, 512), (64, 512), (64, 512)], [(256, 256)], [(1024, 256), (1024, 256)], [(256, 1024)]]
    mats, xs, ys, refs, stages = _staged_case(dev, 1, layer + layer, 15000)
    hs, xp, yp = [m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
    step = tq.Step(hs, xp, yp, 1, stages=stages)
    try:
        assert step.info["persistent"] == 1
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step.launch(torch.cuda.current_stream().cuda_stream)
        for _ in range(4):
            for y in ys:
                y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for y, ref in zip(ys, refs):
                assert check_outputs(y.cpu().numpy(), ref) < 1e-5
            step.launch(_stream())           # eager work between the replays
            torch.cuda.synchronize()
            for y, ref in zip(ys, refs):
                assert check_outputs(y.cpu().numpy(), ref) < 1e-5
        assert tq.tq_step_get_info(step.handle)["fault"] == 0
        del graph
    finally:
        step.close()
        for m in mats:
            m.close()


def test_staged_step_falls_back_to_one_set_of_launches_per_stage(dev):
    """Batch 8 goes to the MFMA kernels, which have no staged form: the step then holds the launches of every stage in
    order (the stream orders them); results as before.  Argument errors of the staged form."""
    layer = [[(256, 512), (64, 512)], [(256, 256)], [(512, 256)]]
    mats, xs, ys, refs, stages = _staged_case(dev, 8, layer, 13000)
    hs, xp, yp = [m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
    step = tq.Step(hs, xp, yp, 8, stages=stages)
    try:
        assert step.info["persistent"] == 0 and step.info["n_launches"] == 3 and step.info["n_stages"] == 3
        step.launch(_stream())
        torch.cuda.synchronize()
        for y, ref in zip(ys, refs):
            check_outputs(y.cpu().numpy(), ref)
        for bad in ([1, 1, 2, 3], [0, 2, 2, 3], [0, 1, 0, 1]):
            with pytest.raises(tq.TqError):
                tq.tq_step_create_staged(hs, xp, yp, bad, 8)
    finally:
        step.close()
        for m in mats:
            m.close()


def test_staged_step_reports_a_hand_over_that_gave_up(dev):
    """The wait at a hand-over is bounded.  With the bound set to zero polls from the host, every workgroup that arrives
    before the last one gives up at once: the kernel still ends normally, the step reports the fault, and later launches
    are refused.  The first stage is one band of a long row: one workgroup works on it for microseconds while all others
    have nothing to do there and reach the wait for it at once."""
    layer = [[(16, 16384)], [(2048, 512)], [(2048, 512)]]
    mats, xs, ys, refs, stages = _staged_case(dev, 1, layer, 14000)
    hs, xp, yp = [m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
    step = tq.Step(hs, xp, yp, 1, stages=stages)
    try:
        assert step.info["persistent"] == 1
        tq.tq_step_set_spin_limit(step.handle, 0)
        step.launch(_stream())
        torch.cuda.synchronize()
        assert tq.tq_step_get_info(step.handle)["fault"] == 1
        with pytest.raises(tq.TqError) as ei:
            step.launch(_stream())
        assert ei.value.code == -5
    finally:
        step.close()
        for m in mats:
            m.close()


def test_prepared_step_argument_errors(dev):
    m = tq.Matrix(tq.tq_encode(make_weights(small_case(17, 64, seed=690)), seg_cols=16))
    x = torch.zeros(64, dtype=torch.int16, device=dev)
    y = torch.zeros(17, dtype=torch.float32, device=dev)
    for kw in (dict(batch=0), dict(batch=17), dict(batch=1, flags=4), dict(batch=1, flags=3),
               dict(batch=1, flags=tq.TQ_STEP_GATE_UP)):   # unknown flag, two forms at once, odd rows: no pairs
        with pytest.raises(tq.TqError):
            tq.tq_step_create([m.handle], [x.data_ptr()], [y.data_ptr()], **kw)
    with pytest.raises(tq.TqError):
        tq.tq_step_create([m.handle], [0], [y.data_ptr()], 1)
    with pytest.raises(tq.TqError):
        tq.tq_step_launch(None)
    tq.tq_step_destroy(None)
    m.close()


def test_argument_errors(dev):
    spec = small_case(16, 256, seed=29)
    m = tq.Matrix(tq.tq_encode(make_weights(spec)))
    try:
        y = torch.zeros((17, 16), dtype=torch.float32, device=dev)
        x = torch.zeros((17, 256), dtype=torch.int16, device=dev)
        for batch in (0, 17, -1):
            with pytest.raises(tq.TqError) as ei:
                m.matvec(x.data_ptr(), y.data_ptr(), batch, _stream())
            assert ei.value.code == -3
        with pytest.raises(tq.TqError) as ei:
            m.matvec(0, y.data_ptr(), 1, _stream())
        assert ei.value.code == -1
    finally:
        m.close()
    with pytest.raises(tq.TqError) as ei:
        tq.tq_create_from_encoded(b"\0" * 1024)
    assert ei.value.code == -2
