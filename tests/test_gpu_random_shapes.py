"""Seeded random shapes, segment widths, dictionary sizes, widths and batches through every kernel, each case against
the oracle: containers byte for byte, expansion bit for bit, products within the tolerance of the other parity tests."""
import numpy as np
import pytest
import torch

import paper_2509_22951_amd as tq
from inputs import make_activations, make_weights, small_case
from oracle import oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available()
    return torch.device("cuda:0")


@pytest.fixture(autouse=True)
def _default_ring_threshold_afterwards():
    """Tests that change the library's ring-kernel threshold leave the default behind."""
    yield
    tq.tq_set_ring_min_bands_per_cu(24)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _draw_matrix(rng, gate_up=False):
    pack = bool(rng.integers(0, 3) == 0)
    width = int(rng.choice([2, 3, 4])) if pack else int(rng.choice([8, 8, 8, 6, 4]))
    seg = int(rng.choice([16, 32, 64, 96, 128, 256]))
    rows = int(rng.integers(1, 300)) * (2 if gate_up else 1)
    cols = int(rng.integers(1, 40)) * int(rng.choice([2, 8, 16, 64, 128]))
    if rng.integers(0, 3) == 0:
        cols = (4 * seg * (2 if pack else 1)) * int(rng.integers(1, 5))     # whole units: what the ring kernel takes
    spec = small_case(rows, cols, seed=int(rng.integers(0, 1 << 30)), dist=str(rng.choice(["normal", "student_t4"])))
    return spec, pack, width, seg


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_single_matrices(dev, seed, monkeypatch):
    rng = np.random.default_rng(seed)
    for _ in range(40):
        spec, pack, width, seg = _draw_matrix(rng)
        me = int(rng.choice([256, 300, 1000, 5000, 30719]))
        kind = str(rng.choice(["lzw", "frequency"]))
        lmax = 2 if kind == "frequency" else int(rng.choice([2, 2, 3, 4]))     # runs of up to 3 and 4 bytes now and then
        tq.tq_set_ring_min_bands_per_cu(int(rng.choice([0, 24])))
        W = make_weights(spec)
        if rng.integers(0, 5) == 0:
            W[rng.integers(0, spec.rows)] = 0           # an all-zero row
        if lmax > 2 and rng.integers(0, 2):
            W *= rng.random(W.shape) < 0.2              # mostly zeros: the long runs get used
        case = dict(rows=spec.rows, cols=spec.cols, seg=seg, entries=me, width=width, pack=pack, dist=spec.dist, kind=kind, lmax=lmax)
        blob = tq.tq_encode(W, max_entries=me, lmax=lmax, seg_cols=seg, bits=0 if width == 8 else width, pack=pack, dictionary=kind)
        assert blob == O.build_blob(O.encode_matrix(W, max_entries=me, lmax=lmax, seg_cols=seg, bits=width, pack=pack, dictionary=kind)), case
        Q, s = O.quantize_rows(W, bits=width)
        m = tq.Matrix(blob)
        try:
            out = torch.full((spec.rows, spec.cols), 77, dtype=torch.int8, device=dev)
            m.decompress(out.data_ptr(), _stream())
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), Q), case
            for batch in (1, int(rng.integers(2, 9)), int(rng.integers(9, 17))):
                bits, x = make_activations(spec, batch)
                ref = O.gemv_f64(Q, s, x)
                flat = torch.from_numpy(bits.view(np.int16).reshape(-1).copy())
                off = int(rng.integers(0, 4) == 0)                      # now and then a 2-byte aligned x
                buf = torch.zeros(flat.numel() + 8, dtype=torch.int16, device=dev)
                buf[off:off + flat.numel()] = flat.to(dev)
                y = torch.full((batch, spec.rows), float("nan"), dtype=torch.float32, device=dev)
                if rng.integers(0, 2):
                    m.matvec(buf[off:].data_ptr(), y.data_ptr(), batch, _stream())
                else:
                    step = tq.Step([m.handle], [buf[off:].data_ptr()], [y.data_ptr()], batch)
                    step.launch(_stream())
                    torch.cuda.synchronize()
                    step.close()
                torch.cuda.synchronize()
                got = y.cpu().numpy()
                assert np.isfinite(got).all(), (case, batch)
                assert (np.abs(got - ref) <= 1e-3 * np.maximum(np.abs(ref).max(axis=1, keepdims=True), 1e-30)).all(), (case, batch)
        finally:
            m.close()


@pytest.mark.parametrize("seed", [21, 22])
def test_calls_with_several_matrices(dev, seed, monkeypatch):
    rng = np.random.default_rng(seed)
    for _ in range(12):
        n = int(rng.integers(2, 14))
        batch = int(rng.choice([1, 1, 2, 5, 8, 9, 16]))
        gate_up = bool(rng.integers(0, 5) == 0)
        tq.tq_set_ring_min_bands_per_cu(int(rng.choice([0, 0, 24])))
        mats, xs, ys, refs, outs, Qs = [], [], [], [], [], []
        chain, entries = {}, {}
        for _k in range(n):
            spec, pack, width, seg = _draw_matrix(rng, gate_up)
            W = make_weights(spec)
            key = (pack, width)
            me = entries.setdefault(key, int(rng.choice([600, 3000, 30719])))
            blob = tq.tq_encode(W, max_entries=me, seg_cols=seg, bits=0 if width == 8 else width, pack=pack,
                                dict_from=chain.get(key) if rng.integers(0, 3) else None)
            chain[key] = blob
            Q, s = O.quantize_rows(W, bits=width)
            bits, x = make_activations(spec, batch)
            refs.append(O.gate_up_f64(Q[0::2], s[0::2], Q[1::2], s[1::2], x) if gate_up else O.gemv_f64(Q, s, x))
            mats.append(tq.Matrix(blob))
            Qs.append(Q)
            xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
            ys.append(torch.full(refs[-1].shape, float("nan"), dtype=torch.float32, device=dev))
            outs.append(torch.full((spec.rows, spec.cols), 77, dtype=torch.int8, device=dev))
        hs, xp, yp = [m.handle for m in mats], [x.data_ptr() for x in xs], [y.data_ptr() for y in ys]
        try:
            for how in ("call", "step"):
                for y in ys:
                    y.fill_(float("nan"))
                if how == "call":
                    (tq.tq_matvec_gate_up_multi if gate_up else tq.tq_matvec_multi)(hs, xp, yp, batch, _stream())
                else:
                    step = tq.Step(hs, xp, yp, batch, gate_up=gate_up)
                    step.launch(_stream())
                    torch.cuda.synchronize()
                    step.close()
                torch.cuda.synchronize()
                for y, ref in zip(ys, refs):
                    got = y.cpu().numpy()
                    assert np.isfinite(got).all(), (how, n, batch, gate_up)
                    assert (np.abs(got - ref) <= 1e-3 * np.maximum(np.abs(ref).max(axis=1, keepdims=True), 1e-30)).all(), (how, n, batch)
            tq.tq_decompress_multi(hs, [o.data_ptr() for o in outs], _stream())
            torch.cuda.synchronize()
            for o, Q in zip(outs, Qs):
                assert np.array_equal(o.cpu().numpy(), Q)
        finally:
            for m in mats:
                m.close()
