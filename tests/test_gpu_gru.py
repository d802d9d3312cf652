"""GPU parity of the integer GRU (gru_int_forward through the C ABI) against the CPU oracle's
(oracle/gru_int_oracle.c) on the same seeded inputs: every integer tensor of every layer and step,
bit for bit.  The recipe itself is this build's (Sec. 7 of the paper names the GRU and gives none)."""
import numpy as np
import pytest

import lstm_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gru(orc):
    from oracle import gru as g

    g.lib()
    return g


def both(gru, layers):
    from paper_2101_05453_amd import binding

    return binding.gru_prepare(layers, device=0), gru.GruModel(layers)


def quantize_x(x, q):
    return np.clip(np.floor(x.astype(np.float64) / q["s_x"] + 0.5) + q["zp_x"], -128, 127).astype(np.int8)


def equal(name, got, want):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape and got.dtype == want.dtype, (name, got.shape, want.shape, got.dtype, want.dtype)
    if not (got == want).all():
        bad = np.argwhere(got != want)
        first = tuple(bad[0])
        raise AssertionError(f"{name}: {len(bad)} of {got.size} differ; first at {first}: gpu={got[first]} oracle={want[first]}")


def compare_all(gru, layers, x, name, rows=None):
    """Every traced tensor of every layer, the output and the carried state."""
    import torch

    lib_m, orc_m = both(gru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    T, B, _ = xq.shape
    xd = torch.from_numpy(xq).cuda()
    sel = np.arange(B) if rows is None else np.asarray(rows)
    Ntot = sum(s.num_cells for s in layers)
    for l in range(len(layers)):
        hs = torch.zeros(B * Ntot, dtype=torch.int16, device="cuda")
        y, tr = lib_m.forward(xd, h_state=hs, trace_layer=l)
        torch.cuda.synchronize()
        hs_o = np.zeros(len(sel) * Ntot, dtype=np.int16)
        yo, tro = orc_m.forward(xq[:, sel], h_state=hs_o, trace_layer=l, threads=8)
        for f in ("tx", "th", "act", "h16", "h8"):
            equal(f"{name}.layer{l}.{f}", tr[f].cpu().numpy()[:, sel], tro[f])
        equal(f"{name}.y", y.cpu().numpy()[:, sel], yo)
        off_g = off_o = 0
        for s in layers:
            n = s.num_cells
            equal(f"{name}.h_state", hs.cpu().numpy()[off_g:off_g + B * n].reshape(B, n)[sel],
                  hs_o[off_o:off_o + len(sel) * n].reshape(len(sel), n))
            off_g += B * n
            off_o += len(sel) * n
    y2 = lib_m.forward(xd)  # no state buffer, no trace: the same output from zeros
    equal(f"{name}.y_nostate", y2.cpu().numpy()[:, sel], yo)


@pytest.mark.parametrize("case", [
    ([24], 40, 3, 6, 0.2),          # ragged: I, N no multiples of the tiles
    ([64], 64, 16, 5, 0.2),         # exact tiles, x read in place
    ([17, 37, 37], 37, 5, 7, 0.3),  # N not a multiple of 4, three layers
    ([32, 128], 128, 33, 9, 0.1),   # three row tiles, the last with one row
    ([100], 200, 1, 12, 0.15),      # a single row
])
def test_every_tensor_small_shapes(gru, case):
    inputs, N, B, T, wp = case
    layers, x = wl.make_gru(inputs, N, B, T, seed=21, weight_param=wp, input_param=1.5)
    compare_all(gru, layers, x, f"gru{inputs}x{N}")


def test_saturating_inputs_and_clipped_range(gru):
    layers, x = wl.make_gru([48], 96, 6, 8, seed=5, weight_param=0.5, input_dist="uniform", input_param=3.0)
    layers[0].x_min, layers[0].x_max = -1.0, 2.0  # inputs beyond the range saturate; zero point off centre
    for s in layers:  # large biases drive gate sums into the Q3.12 clamps
        s.bx[1] = s.bx[1] * 80
        s.bh[2] = s.bh[2] * 60
    compare_all(gru, layers, x, "gru_sat")


def test_speech_encoder_shapes_sampled_rows(gru):
    """Layers of the benchmark's width: N = 2048 at B = 256 (two layers, T = 6) on rows spread over the row
    tiles, N = 1024 at B = 64 whole."""
    layers, x = wl.make_gru([512, 2048], 2048, 256, 6, seed=3, weight_param=0.03)
    compare_all(gru, layers, x, "gru2048", rows=[0, 15, 16, 100, 127, 128, 200, 255])
    layers, x = wl.make_gru([256], 1024, 64, 10, seed=4, weight_param=0.04)
    compare_all(gru, layers, x, "gru1024")


def test_large_products_take_the_wide_matmul_tile(gru):
    """T * B = 2100 rows by 3 * 400 = 1200 output columns (padded to 1280 = 5 blocks of 256): with a trace the input
    term comes from the general matmul, which gives products of this size to its 256 x 256 tile -- a ragged last row
    block, columns beyond the real ones, input depths 100 and 400."""
    layers, x = wl.make_gru([100, 400], 400, 70, 30, seed=12, weight_param=0.08)
    compare_all(gru, layers, x, "gru_tile256")
    # a depth of one k tile (48 -> 64 bytes): that tile's four-deep load pipeline runs on repeats of the only tile
    layers, x = wl.make_gru([48], 400, 70, 30, seed=13, weight_param=0.1)
    compare_all(gru, layers, x, "gru_tile256_k64")


def test_benchmark_configuration_sampled_rows(gru):
    """The configuration bench.py --gru times (2 x 2048 cells, input 512, B = 256, T = 64: 16384-row matmuls on the
    register-resident GEMM and on the general matmul's widest tile, 128 step launches) on three rows of different
    row tiles: every traced tensor, the output and the carried state."""
    layers, x = wl.make_gru([512, 2048], 2048, 256, 64, seed=0, weight_param=0.03)
    compare_all(gru, layers, x, "gru_bench", rows=[0, 100, 255])


def test_split_sequence_and_long_run(gru):
    import torch

    layers, x = wl.make_gru([32, 64], 64, 5, 300, seed=8, weight_param=0.12)
    lib_m, orc_m = both(gru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    xd = torch.from_numpy(xq).cuda()
    hs = torch.zeros(2 * 5 * 64, dtype=torch.int16, device="cuda")
    parts = [lib_m.forward(xd[a:b].contiguous(), h_state=hs).cpu().numpy() for a, b in ((0, 1), (1, 120), (120, 300))]
    hs_o = np.zeros(2 * 5 * 64, dtype=np.int16)
    yo, _ = orc_m.forward(xq, h_state=hs_o, threads=5)
    equal("gru_split.y", np.concatenate(parts), yo)
    equal("gru_split.h_state", hs.cpu().numpy(), hs_o)


def test_empty_inputs_and_workspace_checks(gru):
    import torch
    from paper_2101_05453_amd import binding

    layers, x = wl.make_gru([16], 32, 2, 3, seed=1)
    m = binding.gru_prepare(layers, device=0)
    xd = torch.zeros((0, 2, 16), dtype=torch.int8, device="cuda")
    assert m.forward(xd).shape == (0, 2, 32)
    xd = torch.zeros((3, 2, 16), dtype=torch.int8, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.LstmIntError) as e:
        m.forward(xd, workspace=small)
    assert e.value.code == binding.E_WORKSPACE
    big = torch.empty(m.workspace_bytes(3, 2) + 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.LstmIntError) as e:
        m.forward(xd, workspace=big[1:])  # misaligned
    assert e.value.code == binding.E_WORKSPACE
    torch.cuda.synchronize()


def test_forward_captured_in_a_hip_graph(gru):
    """gru_int_forward allocates nothing, never synchronizes and launches only kernels: a caller can capture a
    whole multi-step call (two layers x eight steps = 20 kernel nodes) in a HIP graph.  Replays with new inputs and
    carried state, with the program's own eager work and synchronization in between, give what the oracle gives."""
    import torch

    layers, x = wl.make_gru([40, 96], 96, 12, 24, seed=17, weight_param=0.15)
    lib_m, orc_m = both(gru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    T, B = 8, 12
    xin = torch.from_numpy(np.ascontiguousarray(xq[:T])).cuda()
    y = torch.empty((T, B, 96), dtype=torch.int8, device="cuda")
    hs = torch.zeros(2 * B * 96, dtype=torch.int16, device="cuda")
    ws = torch.empty(lib_m.workspace_bytes(T, B), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # one call outside the capture first
        lib_m.forward(xin, y=y, h_state=hs, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lib_m.forward(xin, y=y, h_state=hs, workspace=ws)
    for rep in range(2):
        hs.zero_()
        hs_o = np.zeros(2 * B * 96, dtype=np.int16)
        for part in range(3):  # the 24 steps as three replays of the captured 8-step call
            xin.copy_(torch.from_numpy(np.ascontiguousarray(xq[part * T:(part + 1) * T])))
            graph.replay()
            torch.cuda.synchronize()
            want, _ = orc_m.forward(xq[part * T:(part + 1) * T], h_state=hs_o)
            equal(f"gru_graph.rep{rep}.part{part}.y", y.cpu().numpy(), want)
            equal(f"gru_graph.rep{rep}.part{part}.h", hs.cpu().numpy(), hs_o)


def run_both_paths(gru, layers, x, name, rows=None, splits=None):
    """Untraced forward with carried state on the persistent launch (default) and with option "persistent" = 0 (one
    launch per step): both against the oracle, device status 0."""
    import torch

    lib_m, orc_m = both(gru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    T, B, _ = xq.shape
    sel = np.arange(B) if rows is None else np.asarray(rows)
    Ntot = sum(s.num_cells for s in layers)
    xd = torch.from_numpy(xq).cuda()
    hs_o = np.zeros(len(sel) * Ntot, dtype=np.int16)
    want, _ = orc_m.forward(xq[:, sel], h_state=hs_o, threads=8)
    for persistent in (1, 0):
        lib_m.set_option("persistent", persistent)
        hs = torch.zeros(B * Ntot, dtype=torch.int16, device="cuda")
        parts = []
        for a, b in (splits or [(0, T)]):
            parts.append(lib_m.forward(xd[a:b].contiguous(), h_state=hs).cpu().numpy())
        torch.cuda.synchronize()
        assert lib_m.device_status() == 0
        equal(f"{name}.p{persistent}.y", np.concatenate(parts)[:, sel], want)
        off_g = off_o = 0
        for s in layers:
            n = s.num_cells
            equal(f"{name}.p{persistent}.h_state", hs.cpu().numpy()[off_g:off_g + B * n].reshape(B, n)[sel],
                  hs_o[off_o:off_o + len(sel) * n].reshape(len(sel), n))
            off_g += B * n
            off_o += len(sel) * n
    return lib_m


@pytest.mark.parametrize("case", [
    ([24], 40, 3, 6, 0.2),            # two cell tiles, the second ragged
    ([64], 32, 16, 5, 0.2),           # a group of one workgroup
    ([17, 37, 37], 37, 5, 7, 0.3),    # N not a multiple of 4, three layers
    ([32, 128], 128, 33, 9, 0.1),     # two groups of rows, the second with one row
    ([100], 200, 1, 12, 0.15),        # a single row
    ([48, 96], 96, 70, 40, 0.12),     # three groups, 40 steps
])
def test_persistent_launch_small_shapes(gru, case):
    inputs, N, B, T, wp = case
    layers, x = wl.make_gru(inputs, N, B, T, seed=23, weight_param=wp, input_param=1.5)
    run_both_paths(gru, layers, x, f"gru_seq{inputs}x{N}", splits=[(0, 1), (1, T)] if T > 6 else None)


def test_persistent_launch_full_chip_and_beyond(gru):
    """N = 1024 at B = 256: 8 groups x 32 workgroups = every compute unit; N = 512 at B = 300: 10 groups of 16
    workgroups; N = 1024 at B = 288 does not fit one launch and runs one launch per step."""
    layers, x = wl.make_gru([256, 1024], 1024, 256, 10, seed=6, weight_param=0.04)
    run_both_paths(gru, layers, x, "gru_seq1024", rows=[0, 31, 32, 100, 127, 128, 200, 224, 255])
    layers, x = wl.make_gru([128], 512, 300, 8, seed=7, weight_param=0.05)
    run_both_paths(gru, layers, x, "gru_seq512", rows=[0, 15, 31, 32, 159, 160, 287, 288, 299])
    layers, x = wl.make_gru([64], 1024, 288, 4, seed=8, weight_param=0.04)
    run_both_paths(gru, layers, x, "gru_1024_b288", rows=[0, 100, 255, 256, 287])


def test_persistent_wait_gives_up_and_model_recovers(gru):
    """The kernel's waits are bounded: with the test hook every barrier waits for an arrival that never comes, each
    wait ends at its (small) limit, the kernel exits normally and the status word says so; after a reset the same
    model computes the right result.  (That the status becomes 1 also shows that the persistent launch ran.)"""
    import torch

    layers, x = wl.make_gru([32], 96, 40, 5, seed=9, weight_param=0.2)
    lib_m, orc_m = both(gru, layers)
    xq = quantize_x(x, orc_m.get_quant(0))
    xd = torch.from_numpy(xq).cuda()
    lib_m.set_option("spin_limit", 64)
    lib_m.set_option("barrier_never_completes", 1)
    lib_m.forward(xd)
    torch.cuda.synchronize()
    assert lib_m.device_status() == 1
    lib_m.set_option("barrier_never_completes", 0)
    lib_m.set_option("spin_limit", 1 << 21)
    lib_m.set_option("reset_status", 1)
    assert lib_m.device_status() == 0
    y = lib_m.forward(xd)
    torch.cuda.synchronize()
    want, _ = orc_m.forward(xq, threads=8)
    assert lib_m.device_status() == 0
    equal("gru_recovered.y", y.cpu().numpy(), want)


def test_tile_ordered_input_terms_on_both_recurrent_kernels(gru):
    """With 8192 and more (t, b) rows the launch-per-step path also takes its input terms from the register-resident
    input GEMM in that kernel's tile order (the persistent launch always does): 512 rows x 16 steps, two layers, a
    ragged variant with 515 rows."""
    layers, x = wl.make_gru([64, 128], 128, 512, 16, seed=12, weight_param=0.15)
    run_both_paths(gru, layers, x, "gru_tx2")
    layers, x = wl.make_gru([40, 96], 96, 515, 16, seed=13, weight_param=0.15)
    run_both_paths(gru, layers, x, "gru_tx2_ragged", splits=[(0, 5), (5, 16)])
