"""tq_matvec_multi_static, the entry point that allocates no device memory (its job table lives in a static array of the
library's device image), against the existing entry point whose kernels use the same kind of table, the prepared step:
same matrices, same buffers, two calls in a row, the second with a smaller input.  Both also against the oracle."""
import numpy as np
import pytest

import paper_2509_22951_amd as tq
from inputs import make_activations, make_weights, small_case
from oracle import oracle as O

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _case(dev, shapes, batch, seed):
    mats, xs, refs, prev = [], [], [], None
    for k, (rows, cols) in enumerate(shapes):
        spec = small_case(rows, cols, seed=seed + k)
        W = make_weights(spec)
        prev = tq.tq_encode(W, seg_cols=64, max_entries=3000, dict_from=prev)
        mats.append(tq.Matrix(prev))
        bits, x = make_activations(spec, batch)
        xs.append(torch.from_numpy(bits.view(np.int16).copy()).to(dev))
        Q, s = O.quantize_rows(W)
        refs.append(O.gemv_f64(Q, s, x))
    return mats, xs, refs


@pytest.mark.parametrize("batch", [1, 8])
def test_static_job_table_matches_the_prepared_step_on_two_calls_in_a_row(batch):
    assert torch.cuda.is_available()
    tq.load()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    # first call: 200 matrices (more than the 128 that fit a launch's arguments, more than one writer launch);
    # second call: 37 of other shapes, so the table keeps 163 stale entries of the first call beyond its own
    big = [(int(rng.integers(1, 9)) * 16, int(rng.integers(1, 5)) * 256) for _ in range(200)]
    small = [(int(rng.integers(1, 6)) * 16 + 3, int(rng.integers(1, 4)) * 256) for _ in range(37)]
    for shapes, seed in ((big, 9000), (small, 9500)):
        mats, xs, refs = _case(dev, shapes, batch, seed)
        hs, xp = [m.handle for m in mats], [x.data_ptr() for x in xs]
        y_step = [torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev) for r, _ in shapes]
        y_stat = [torch.full((batch, r), float("nan"), dtype=torch.float32, device=dev) for r, _ in shapes]
        step = tq.Step(hs, xp, [y.data_ptr() for y in y_step], batch)
        step.launch(_stream())
        tq.tq_matvec_multi_static(hs, xp, [y.data_ptr() for y in y_stat], batch, _stream())
        torch.cuda.synchronize()
        for a, b, ref in zip(y_step, y_stat, refs):
            got, want = b.cpu().numpy(), a.cpu().numpy()
            assert np.isfinite(got).all()
            scale = np.abs(ref).max(axis=1, keepdims=True)
            assert (np.abs(got - want) <= 1e-3 * scale).all()      # the bar of the other product tests
            assert np.array_equal(got, want)                        # same plan, same kernels: the same bits
            assert (np.abs(got - ref) <= 1e-3 * scale).all()
        step.close()
        for m in mats:
            m.close()


def test_static_job_table_refuses_more_matrices_than_it_holds():
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    spec = small_case(16, 256, seed=1)
    m = tq.Matrix(tq.tq_encode(make_weights(spec)))
    bits, _ = make_activations(spec, 1)
    x = torch.from_numpy(bits.view(np.int16).copy()).to(dev)
    y = torch.zeros((1, 16), dtype=torch.float32, device=dev)
    n = tq.TQ_STATIC_MAX_MATRICES + 1
    with pytest.raises(tq.TqError) as ei:
        tq.tq_matvec_multi_static([m.handle] * n, [x.data_ptr()] * n, [y.data_ptr()] * n, 1, _stream())
    assert ei.value.code == -3 and "static job table" in str(ei.value)
    m.close()
