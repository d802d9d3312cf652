"""lstm_int_forward_bidirectional: a forward stack and a backward stack (option "reverse") over the same input,
outputs side by side (Sec. 7: the bidirectional LSTM as two loops over the cell), against the oracle's two runs."""
import numpy as np
import pytest

import lstm_workloads as wl
from parity_util import assert_equal, calibrate_on_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", [
    (0, [24], 40, 40, 5, 7),
    (wl.LAYER_NORM | wl.PROJECTION, [48, 24], 64, 24, 37, 6),
    (wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE, [64], 128, 128, 16, 9),
])
def test_bidirectional_outputs_side_by_side(orc, case):
    import torch
    from paper_2101_05453_amd import binding

    flags, inputs, N, H, B, T = case
    lay_f, x = wl.make_custom(inputs, N, H, flags, B, T, seed=31)
    lay_b, _ = wl.make_custom(inputs, N, H, flags, B, T, seed=77)  # the other direction has its own parameters
    xd = calibrate_on_gpu(lay_f, x)
    calibrate_on_gpu(lay_b, x)
    # the backward direction's statistics belong to the flipped sequence; the ranges of x are the same either way
    fwd, bwd = binding.prepare(lay_f, device=0), binding.prepare(lay_b, device=0)
    bwd.set_option("reverse", 1)
    of, ob = orc.prepare(lay_f), orc.prepare(lay_b)
    xq = fwd.quantize_input(xd)
    dims_f, dims_b = fwd.dims(), bwd.dims()
    rng = np.random.Generator(np.random.PCG64(3))
    st = {}
    for name, dims in (("f", dims_f), ("b", dims_b)):
        st[name] = (rng.integers(-128, 128, sum(B * d[2] for d in dims), dtype=np.int8),
                    rng.integers(-2000, 2000, sum(B * d[1] for d in dims), dtype=np.int16))
    dev = {k: (torch.from_numpy(v[0].copy()).cuda(), torch.from_numpy(v[1].copy()).cuda()) for k, v in st.items()}
    y = binding.forward_bidirectional(fwd, bwd, xq, state_fwd=dev["f"], state_bwd=dev["b"])
    torch.cuda.synchronize()
    assert fwd.device_status() == 0 and bwd.device_status() == 0
    xh = xq.cpu().numpy()
    hf, cf = st["f"][0].copy(), st["f"][1].copy()
    hb, cb = st["b"][0].copy(), st["b"][1].copy()
    yf = orc.forward(of, xh, h_state=hf, c_state=cf)
    yb = orc.forward(ob, xh, h_state=hb, c_state=cb, reverse=True)
    assert_equal("bidi.y", y.cpu().numpy(), np.concatenate([yf, yb], axis=2))
    for name, got, want in (("h_f", dev["f"][0], hf), ("c_f", dev["f"][1], cf), ("h_b", dev["b"][0], hb), ("c_b", dev["b"][1], cb)):
        assert_equal("bidi." + name, got.cpu().numpy(), want)
    # stateless call, caller-provided output and workspace
    ws = torch.empty(binding.bidirectional_workspace_bytes(fwd, bwd, T, B), dtype=torch.uint8, device="cuda")
    y2 = torch.full((T, B, dims_f[-1][2] + dims_b[-1][2]), 99, dtype=torch.int8, device="cuda")
    binding.forward_bidirectional(fwd, bwd, xq, y=y2, workspace=ws)
    torch.cuda.synchronize()
    assert_equal("bidi.y0", y2.cpu().numpy(), np.concatenate([orc.forward(of, xh), orc.forward(ob, xh, reverse=True)], axis=2))


def test_bidirectional_argument_checks(orc):
    import torch
    from paper_2101_05453_amd import binding

    lay_f, x = wl.make_custom([24], 40, 40, 0, 3, 4, seed=1)
    lay_b, _ = wl.make_custom([24], 40, 40, 0, 3, 4, seed=2)
    xd = calibrate_on_gpu(lay_f, x)
    calibrate_on_gpu(lay_b, x)
    fwd, bwd = binding.prepare(lay_f, device=0), binding.prepare(lay_b, device=0)
    xq = fwd.quantize_input(xd)
    with pytest.raises(binding.LstmIntError) as e:  # the backward model must have "reverse" set
        binding.forward_bidirectional(fwd, bwd, xq)
    assert e.value.code == binding.E_INVALID_ARG
    bwd.set_option("reverse", 1)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.LstmIntError) as e:
        binding.forward_bidirectional(fwd, bwd, xq, workspace=small)
    assert e.value.code == binding.E_WORKSPACE
    lay_c, x2 = wl.make_custom([32], 40, 40, 0, 3, 4, seed=2)  # another input width
    calibrate_on_gpu(lay_c, x2)
    other = binding.prepare(lay_c, device=0)
    other.set_option("reverse", 1)
    with pytest.raises(binding.LstmIntError) as e:
        binding.forward_bidirectional(fwd, other, xq)
    assert e.value.code == binding.E_INVALID_ARG
    assert binding.forward_bidirectional(fwd, bwd, xq[:0]).shape == (0, 3, 80)
    torch.cuda.synchronize()
