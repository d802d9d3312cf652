"""GPU parity of the integer SRU (sru_int_forward through the C ABI) against the CPU oracle's
(oracle/sru_int_oracle.c) on the same seeded inputs: every integer tensor of every layer and step,
bit for bit, on both forms of the input matmul.  The recipe itself is this build's (Sec. 7 of the
paper names the SRU and gives none); the calibration statistics are inputs of both sides."""
import numpy as np
import pytest

import lstm_workloads as wl

pytestmark = pytest.mark.gpu

FIELDS = ("tx", "tv", "act", "c", "h16", "y")


@pytest.fixture(scope="module")
def sru(orc):
    from oracle import sru as s

    s.lib()
    return s


def both(sru, layers):
    from paper_2101_05453_amd import binding

    return binding.sru_prepare(layers, device=0), sru.SruModel(layers)


def quantize_x(x, q):
    return np.clip(np.floor(x.astype(np.float64) / q["s_x"] + 0.5) + q["zp_x"], -128, 127).astype(np.int8)


def equal(name, got, want):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape and got.dtype == want.dtype, (name, got.shape, want.shape, got.dtype, want.dtype)
    if not (got == want).all():
        bad = np.argwhere(got != want)
        first = tuple(bad[0])
        raise AssertionError(f"{name}: {len(bad)} of {got.size} differ; first at {first}: gpu={got[first]} oracle={want[first]}")


def state_rows(buf, layers, B, sel):
    out, off = [], 0
    for s in layers:
        n = s.num_cells
        out.append(buf[off:off + B * n].reshape(B, n)[sel])
        off += B * n
    return out


def compare_all(sru, layers, x, name, rows=None, calibration_rows=None):
    """Every traced tensor of every layer, the output and the carried state; then the untraced call (which may
    take the register-resident matmul and the tile-ordered scan) with and without a state buffer, and the
    same with that matmul switched off."""
    import torch

    sru.calibrate(layers, x if calibration_rows is None else np.ascontiguousarray(x[:, :calibration_rows]), threads=8)
    lib_m, orc_m = both(sru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    T, B, _ = xq.shape
    xd = torch.from_numpy(xq).cuda()
    sel = np.arange(B) if rows is None else np.asarray(rows)
    Ntot = sum(s.num_cells for s in layers)
    rng = np.random.default_rng(7)
    c0 = rng.integers(-20000, 20000, size=B * Ntot).astype(np.int16)  # a state to start from
    c0_o = np.concatenate([r.ravel() for r in state_rows(c0, layers, B, sel)])
    for l in range(len(layers)):
        cs = torch.from_numpy(c0.copy()).cuda()
        y, tr = lib_m.forward(xd, c_state=cs, trace_layer=l)
        torch.cuda.synchronize()
        cs_o = c0_o.copy()
        yo, tro = orc_m.forward(xq[:, sel], c_state=cs_o, trace_layer=l, threads=8)
        for f in FIELDS:
            equal(f"{name}.layer{l}.{f}", tr[f].cpu().numpy()[:, sel], tro[f])
        equal(f"{name}.y", y.cpu().numpy()[:, sel], yo)
        for a, b in zip(state_rows(cs.cpu().numpy(), layers, B, sel), state_rows(cs_o, layers, len(sel), np.arange(len(sel)))):
            equal(f"{name}.c_state", a, b)
    y0, _ = orc_m.forward(xq[:, sel], threads=8)
    for reg in (1, 0):
        lib_m.set_option("register_gemm", reg)
        cs = torch.from_numpy(c0.copy()).cuda()
        equal(f"{name}.y_untraced[{reg}]", lib_m.forward(xd, c_state=cs).cpu().numpy()[:, sel], yo)
        for a, b in zip(state_rows(cs.cpu().numpy(), layers, B, sel), state_rows(cs_o, layers, len(sel), np.arange(len(sel)))):
            equal(f"{name}.c_state_untraced[{reg}]", a, b)
        equal(f"{name}.y_nostate[{reg}]", lib_m.forward(xd).cpu().numpy()[:, sel], y0)


@pytest.mark.parametrize("case", [
    ([24], 40, 3, 6, 0.2, None),           # ragged: I, N no multiples of the tiles; W_s
    ([64, 64], 64, 16, 5, 0.2, None),      # exact tiles, x read in place, the input as the highway term
    ([37, 37, 37], 37, 5, 7, 0.3, None),   # N not a multiple of 4, three layers without W_s
    ([32, 128], 128, 33, 9, 0.1, None),    # two row blocks, the last with one row; W_s then none
    ([100], 200, 1, 12, 0.15, None),       # a single row
    ([48, 48], 48, 40, 3, 0.2, True),      # W_s although the sizes agree; fewer steps than the prefetch depth
    ([16], 8, 70, 1, 0.3, None),           # one step, one tile of cells, three row blocks
])
def test_every_tensor_small_shapes(sru, case):
    inputs, N, B, T, wp, hw = case
    layers, x = wl.make_sru(inputs, N, B, T, seed=21, weight_param=wp, input_param=1.5, highway_matrix=hw)
    compare_all(sru, layers, x, f"sru{inputs}x{N}")


def test_saturating_inputs_and_clipped_ranges(sru):
    import torch

    layers, x = wl.make_sru([48, 96], 96, 6, 8, seed=5, weight_param=0.5, input_dist="uniform", input_param=3.0)
    sru.calibrate(layers, x)
    layers[0].x_min, layers[0].x_max = -1.0, 2.0  # inputs beyond the range saturate; zero point off centre
    for s in layers:
        s.b[0] = s.b[0] * 40        # gate sums into the Q3.12 clamps
        s.v[1] = s.v[1] * 30
        s.c_absmax *= 0.25          # candidate, state and highway term into the int16 clamps
        s.h_min, s.h_max = 0.3 * s.h_min, 0.2 * s.h_max  # outputs into the int8 clamps
    lib_m, orc_m = both(sru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    xd = torch.from_numpy(xq).cuda()
    for l in range(2):
        y, tr = lib_m.forward(xd, trace_layer=l)
        yo, tro = orc_m.forward(xq, trace_layer=l)
        for f in FIELDS:
            equal(f"sat.layer{l}.{f}", tr[f].cpu().numpy(), tro[f])
        equal("sat.y", y.cpu().numpy(), yo)
        assert (np.abs(tro["tx"].astype(np.int32)) >= 32767).any() and (tro["y"] == 127).any() and (tro["y"] == -128).any()
    equal("sat.y_untraced", lib_m.forward(xd).cpu().numpy(), yo)


def test_speech_encoder_shapes_sampled_rows(sru):
    """Layers of the benchmark's width: N = 2048 at B = 256 (input 512, then 2048 = the general matmul and the
    input as the highway term) on rows spread over the row blocks, N = 1024 at B = 64 whole."""
    layers, x = wl.make_sru([512, 2048], 2048, 256, 6, seed=3, weight_param=0.03)
    compare_all(sru, layers, x, "sru2048", rows=[0, 15, 16, 100, 127, 128, 200, 255])
    layers, x = wl.make_sru([256, 1024], 1024, 64, 10, seed=4, weight_param=0.04)
    compare_all(sru, layers, x, "sru1024")


def test_benchmark_configuration_sampled_rows(sru):
    """The configuration bench.py --sru times, two of its four layers (2048 cells, input 512 then 2048, B = 256,
    T = 64: 16384-row matmuls on the register-resident GEMM and on the general matmul's widest tile, both forms of
    the scan) on three rows of different row blocks."""
    layers, x = wl.make_sru([512, 2048], 2048, 256, 64, seed=0, weight_param=0.03)
    compare_all(sru, layers, x, "sru_bench", rows=[0, 100, 255], calibration_rows=16)  # statistics from 16 rows (Sec. 4)


def test_split_sequence_and_long_run(sru):
    import torch

    layers, x = wl.make_sru([32, 64], 64, 5, 300, seed=8, weight_param=0.12)
    sru.calibrate(layers, x, threads=5)
    lib_m, orc_m = both(sru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    xd = torch.from_numpy(xq).cuda()
    cs = torch.zeros(2 * 5 * 64, dtype=torch.int16, device="cuda")
    parts = [lib_m.forward(xd[a:b].contiguous(), c_state=cs).cpu().numpy() for a, b in ((0, 1), (1, 120), (120, 300))]
    cs_o = np.zeros(2 * 5 * 64, dtype=np.int16)
    yo, _ = orc_m.forward(xq, c_state=cs_o, threads=5)
    equal("split.y", np.concatenate(parts), yo)
    equal("split.c_state", cs.cpu().numpy(), cs_o)


def test_empty_calls_and_workspace_checks(sru):
    import ctypes as C

    import torch

    from paper_2101_05453_amd import binding

    layers, x = wl.make_sru([16], 24, 3, 4, seed=1)
    sru.calibrate(layers, x)
    lib_m, orc_m = both(sru, layers)
    xq = torch.from_numpy(quantize_x(x, orc_m.get_quant(0))).cuda()
    L = binding.sru_lib()
    y = torch.full((4, 3, 24), 77, dtype=torch.int8, device="cuda")
    ws = torch.empty(lib_m.workspace_bytes(4, 3), dtype=torch.uint8, device="cuda")
    for T, B in ((0, 3), (4, 0)):  # no-ops: nothing is written
        assert L.sru_int_forward(lib_m._h, xq.data_ptr(), T, B, y.data_ptr(), None, ws.data_ptr(), ws.numel(), None, None) == 0
    torch.cuda.synchronize()
    assert (y == 77).all()
    assert L.sru_int_forward(lib_m._h, xq.data_ptr(), 4, 3, y.data_ptr(), None, ws.data_ptr(), ws.numel() - 1, None, None) == binding.E_WORKSPACE
    assert L.sru_int_forward(lib_m._h, xq.data_ptr(), 4, 3, y.data_ptr(), None, ws.data_ptr() + 16, ws.numel(), None, None) == binding.E_WORKSPACE
    assert L.sru_int_forward(lib_m._h, None, 4, 3, y.data_ptr(), None, ws.data_ptr(), ws.numel(), None, None) == binding.E_INVALID_ARG
    tr = binding.SruTrace()
    tr.layer = 1
    assert L.sru_int_forward(lib_m._h, xq.data_ptr(), 4, 3, y.data_ptr(), None, ws.data_ptr(), ws.numel(), None, C.byref(tr)) == binding.E_INVALID_ARG


def test_forward_captured_in_a_hip_graph(sru):
    """The call launches kernels only: captured once, replayed with new inputs in the same buffers, every replay
    equal to the oracle."""
    import torch

    layers, x = wl.make_sru([64, 128], 128, 32, 12, seed=6, weight_param=0.1)
    sru.calibrate(layers, x, threads=8)
    lib_m, orc_m = both(sru, layers)
    q0 = orc_m.get_quant(0)
    xd = torch.zeros((12, 32, 64), dtype=torch.int8, device="cuda")
    y = torch.zeros((12, 32, 128), dtype=torch.int8, device="cuda")
    cs = torch.zeros(2 * 32 * 128, dtype=torch.int16, device="cuda")
    ws = torch.empty(lib_m.workspace_bytes(12, 32), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        lib_m.forward(xd, y=y, c_state=cs, workspace=ws)  # warm-up outside the capture
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            lib_m.forward(xd, y=y, c_state=cs, workspace=ws)
    cs_o = np.zeros(2 * 32 * 128, dtype=np.int16)
    rng = np.random.default_rng(3)
    for rep in range(3):
        xq = quantize_x(x * rng.uniform(0.5, 1.0), q0)
        xd.copy_(torch.from_numpy(xq))
        if rep == 0:
            cs.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        yo, _ = orc_m.forward(xq, c_state=cs_o, threads=8)
        equal(f"graph.replay{rep}.y", y.cpu().numpy(), yo)
        equal(f"graph.replay{rep}.c_state", cs.cpu().numpy(), cs_o)
        _ = (y.float().sum() + 1).item()  # eager work between the replays
