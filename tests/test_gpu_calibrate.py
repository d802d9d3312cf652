"""GPU parity of lstm_int_calibrate: the statistics run of Sec. 4 (float LSTM
of Sec. 2 in double precision on the GPU) against the oracle's float LSTM.

Both sides compute the same real-valued recursion in double; they differ in
the order of the sums (matrix products, layer-norm means), so the comparison
is to a relative 1e-9, far above the rounding of sums of a few thousand
doubles and far below anything that moves a quantization scale."""
import numpy as np
import pytest

import lstm_workloads as wl

pytestmark = pytest.mark.gpu

VARIANTS = [0, wl.LAYER_NORM, wl.PEEPHOLE, wl.PROJECTION, wl.CIFG,
            wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM,
            wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION]
RTOL = 1e-9


def _close(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape
    assert np.all(np.abs(a - b) <= RTOL * np.maximum(1.0, np.abs(b))), (a, b)


def _compare(orc, layers, x):
    import torch
    from paper_2101_05453_amd import binding

    y_ref, st_ref = orc.float_forward(layers, x)
    xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    st, y = binding.calibrate(layers, xd, want_output=True, apply=False)
    torch.cuda.synchronize()
    _close(y.cpu().numpy(), y_ref)
    assert len(st) == len(st_ref)
    for got, ref in zip(st, st_ref):
        for k in ("x_min", "x_max", "h_min", "h_max", "m_min", "m_max", "c_absmax"):
            _close(got[k], ref[k])
        _close(got["g_absmax"], ref["g_absmax"])
    return st, st_ref


@pytest.mark.parametrize("flags", VARIANTS)
def test_statistics_and_float_output_every_variant(orc, flags):
    # two stacked layers; sizes that are no multiples of the kernels' tiles (16 rows, 64 columns, 32 k)
    layers, x = wl.make_custom([24, 40 if flags & wl.PROJECTION else 72], 72, 40, flags, 5, 7, seed=3)
    _compare(orc, layers, x)


def test_single_row_single_step(orc):
    layers, x = wl.make_custom([8], 16, 16, wl.LAYER_NORM, 1, 1, seed=5)
    _compare(orc, layers, x)


def test_c2_statistics_give_the_same_integer_model(orc):
    """At C2's shape the GPU statistics lead prepare to the very model the
    oracle's statistics lead to: every scale, multiplier and quantized tensor."""
    import torch
    from paper_2101_05453_amd import binding

    layers, x = wl.make_workload("C2")
    rows = np.ascontiguousarray(x[:, :16])
    st, st_ref = _compare(orc, layers, rows)
    orc.apply_stats(layers, st_ref)
    ref = binding.prepare(layers, device=-1).get_quant(0)
    xd = torch.from_numpy(rows.astype(np.float32)).cuda()
    binding.calibrate(layers, xd)  # writes the statistics into the specs
    got = binding.prepare(layers, device=-1).get_quant(0)
    assert got.keys() == ref.keys()
    for k in ref:
        if isinstance(ref[k], np.ndarray):
            assert np.array_equal(got[k], ref[k]), k
        else:
            assert got[k] == ref[k], k


def test_c4_stack_statistics(orc):
    """The 8-layer stack of the headline configuration, on its 16 calibration rows."""
    layers, x = wl.make_workload("C4")
    _compare(orc, layers, np.ascontiguousarray(x[:, :16]))


def test_argument_errors():
    import torch
    from paper_2101_05453_amd import binding

    layers, x = wl.make_custom([8], 16, 16, 0, 2, 2, seed=1)
    xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    layers[0].W[1] = None  # a missing gate matrix
    with pytest.raises(binding.LstmIntError):
        binding.calibrate(layers, xd)
