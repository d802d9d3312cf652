"""GPU parity: the HIP library against the CPU oracle, bit for bit, through
the C ABI.  Small shapes (several tiles, ragged tails, every variant) compare
every intermediate integer tensor of every layer and step; the benchmark
configurations C3-C5 run at full size on the GPU and are compared on sampled
batch rows (rows never interact, so the oracle computes exactly those rows)."""
import numpy as np
import pytest

import lstm_workloads as wl
from parity_util import assert_equal, compare_traces, prepare_both, run_and_compare

pytestmark = pytest.mark.gpu

VARIANTS = [0, wl.LAYER_NORM, wl.PEEPHOLE, wl.PROJECTION, wl.CIFG,
            wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM,
            wl.CIFG | wl.PEEPHOLE | wl.PROJECTION,
            wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION]


@pytest.fixture(scope="module", autouse=True)
def gpu():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05453_amd import binding

    binding.lib()  # fails loudly if liblstm_int.so is not built
    yield


@pytest.mark.parametrize("flags", VARIANTS)
def test_variants_every_tensor(orc, flags):
    """Ragged everything: I = 72 and H = 136 are not multiples of 64, N = 200
    is not a multiple of the 256-thread row loop, B = 37 straddles tiles."""
    H = 136 if flags & wl.PROJECTION else 200
    print(f"variant flags={flags}", flush=True)
    layers, x = wl.make_custom([72, H], 200, H, flags, 37, 5, seed=flags + 11, weight_param=0.08)
    run_and_compare(orc, layers, x, f"variant{flags}")


@pytest.mark.parametrize("flags", [wl.LAYER_NORM | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE])
def test_cooperative_launch(orc, flags):
    """Option "cooperative_launch": the persistent kernel launched through the
    runtime's cooperative path (the default is a plain launch); 4 workgroups per
    group, 3 groups, two layers."""
    H = 136 if flags & wl.PROJECTION else 200
    print(f"cooperative flags={flags}", flush=True)
    layers, x = wl.make_custom([72, H], 200, H, flags, 70, 6, seed=flags + 31, weight_param=0.08)
    run_and_compare(orc, layers, x, f"coop{flags}", trace=False, options={"cooperative_launch": 1})


@pytest.mark.parametrize("flags", [0, wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM])
def test_odd_sizes(orc, flags):
    """N = 203 makes G*N odd (scalar int16 stores), I = 7, B = 1."""
    H = 29 if flags & wl.PROJECTION else 203
    print(f"odd flags={flags}", flush=True)
    layers, x = wl.make_custom([7], 203, H, flags, 1, 4, seed=flags + 50, weight_param=0.2)
    run_and_compare(orc, layers, x, f"odd{flags}")


def test_c1_full(orc):
    layers, x = wl.make_workload("C1")
    run_and_compare(orc, layers, x, "C1")


def test_c2_full(orc):
    layers, x = wl.make_workload("C2")
    run_and_compare(orc, layers, x, "C2", trace=True)


def group_edge_rows(B, rows_pg):
    """First and last batch row of every group of rows_pg rows."""
    rows = set()
    for r0 in range(0, B, rows_pg):
        rows.update((r0, min(B, r0 + rows_pg) - 1))
    return sorted(rows)


@pytest.mark.parametrize("name,rows_pg", [("C3", 16), ("C4", 32), ("C5", 32)])
def test_benchmark_configs_full_size_sampled_rows(orc, name, rows_pg):
    """The benchmark configurations at full size in the launch configuration bench.py
    times, compared on the first and the last batch row of every group of rows of the
    recurrent kernel that runs them (C3: 8 groups of 16 rows; C4: 8 groups of 32, one
    per XCD; C5: two launches of 16 groups of 32) -- every group, hence every XCD and
    every launch, has rows under comparison."""
    layers, x = wl.make_workload(name)
    rows = group_edge_rows(x.shape[1], rows_pg)
    print(f"{name} full size, oracle on {len(rows)} rows {rows}", flush=True)
    run_and_compare(orc, layers, x, name, trace=False, rows=rows)


def test_c3_layer_at_256_rows_on_the_32_row_kernel(orc):
    """The peephole + layer norm + projection layer of C3 at B = 256 with option
    "rows16" off: eight groups of 32 rows, one per XCD, two statistics rounds per
    step; first and last row of every group compared."""
    flags = wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION
    print("C3 layer, B=256, rows16=0", flush=True)
    layers, x = wl.make_custom([640], 2048, 640, flags, 256, 4, seed=91, weight_param=0.03)
    run_and_compare(orc, layers, x, "c3layer256", trace=False, rows=group_edge_rows(256, 32), options={"rows16": 0})


@pytest.mark.parametrize("case", [
    # (inputs, N, H, flags, B, T): batches beyond 32 rows x the groups of one launch at a k depth below 32
    # take two row tiles (64 rows) per group; the last group is ragged, its second tile empty
    ([64], 1024, 512, wl.LAYER_NORM | wl.PROJECTION, 520, 3),
    ([64], 512, 512, 0, 1100, 3),
    ([64], 512, 512, wl.LAYER_NORM | wl.PEEPHOLE, 1090, 3),
])
def test_two_row_tiles_per_group(orc, case):
    import torch

    inputs, N, H, flags, B, T = case
    print(f"two row tiles: N={N} H={H} flags={flags} B={B}", flush=True)
    layers, x = wl.make_custom(inputs, N, H, flags, B, T, seed=N + B, weight_param=0.04)
    last0 = (B - 1) // 64 * 64  # first row of the last group
    rows = sorted({0, 31, 32, 63, 64, 95, 96, 127, last0 - 64, last0 - 33, last0 - 32, last0 - 1, last0, B - 1})
    lib_model, y = run_and_compare(orc, layers, x, f"rt2_{N}_{B}", trace=False, rows=rows, options={"rows16": 0})
    lib_model.profile_begin()
    lib_model.forward(torch.zeros((T, B, inputs[0]), dtype=torch.int8, device="cuda"))
    prof = lib_model.profile_end()
    assert prof["recurrent"]["launches"] == 1 and prof["cell"]["launches"] == 0, prof  # one launch: 64 rows per group


@pytest.mark.parametrize("rows16", [1, 0])
@pytest.mark.parametrize("flags", [wl.LAYER_NORM | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE,
                                   wl.PEEPHOLE | wl.PROJECTION])
def test_persistent_path_every_step_and_layer(orc, flags, rows16):
    """The persistent kernels dump no intermediate tensors, so their state is
    checked step by step instead: the sequence runs as one-step calls with h and c
    carried in the state buffers, and after every call the h and c of EVERY layer
    are compared with the oracle's traces of that layer at that step."""
    import torch

    print(f"every step and layer: flags={flags} rows16={rows16}", flush=True)
    H = 136 if flags & wl.PROJECTION else 200
    layers, x = wl.make_custom([72, H, H], 200, H, flags, 37, 6, seed=flags + 71, weight_param=0.08)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    lib_model.set_option("rows16", rows16)
    lib_model.set_option("stack", 0)  # one layer after the other (the stacked launch has its own test)
    T, B, _ = xq.shape
    dims = lib_model.dims()
    traces = [orc.forward(orc_model, xq, trace_layer=l)[1] for l in range(len(layers))]
    want_y = orc.forward(orc_model, xq)
    hs = torch.cat([torch.full((B * d[2],), lib_model.get_quant(l)["zp_h"], dtype=torch.int8)
                    for l, d in enumerate(dims)]).cuda()
    cs = torch.zeros(sum(B * d[1] for d in dims), dtype=torch.int16).cuda()
    xd = torch.from_numpy(xq).cuda()
    lib_model.profile_begin()
    for t in range(T):
        y = lib_model.forward(xd[t:t + 1].contiguous(), h_state=hs, c_state=cs)
        torch.cuda.synchronize()
        assert_equal(f"y[{t}]", y.cpu().numpy()[0], want_y[t])
        h_np, c_np = hs.cpu().numpy(), cs.cpu().numpy()
        ho = co = 0
        for l, (I, N, Hl) in enumerate(dims):
            assert_equal(f"h[{t}] layer {l}", h_np[ho:ho + B * Hl].reshape(B, Hl), traces[l]["h"][t])
            assert_equal(f"c[{t}] layer {l}", c_np[co:co + B * N].reshape(B, N), traces[l]["c"][t])
            ho, co = ho + B * Hl, co + B * N
    prof = lib_model.profile_end()
    assert prof["cell"]["launches"] == 0 and prof["recurrent"]["launches"] == T * len(layers), prof
    assert lib_model.device_status() == 0


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_benchmark_configs_take_the_persistent_path(name):
    """Every benchmark configuration must fit the persistent kernel (its LDS
    budget at C4 is within a KB of the limit): no per-step cell kernel may run."""
    import torch

    from paper_2101_05453_amd import binding
    from parity_util import calibrate_on_gpu

    layers, x = wl.make_workload(name, batch=None, steps=2, num_layers=2 if name == "C4" else None)
    xf = calibrate_on_gpu(layers, x)
    model = binding.prepare(layers, device=0)
    xd = model.quantize_input(xf)
    model.profile_begin()
    model.forward(xd)
    prof = model.profile_end()
    assert prof["recurrent"]["launches"] > 0 and prof["cell"]["launches"] == 0, prof
    assert model.device_status() == 0


@pytest.mark.parametrize("rows16", [1, 0])
def test_wait_gives_up_and_model_recovers(orc, rows16):
    """A barrier that cannot complete (option "barrier_never_completes": it waits for
    one arrival more than will come) and a small spin limit make the waits inside
    the persistent kernel give up: every workgroup leaves the kernel (no hang),
    the status word says so, and after a reset the same model computes the right
    answer again.  On both kernels of the one-layer path."""
    import torch

    print("bounded waits", flush=True)
    layers, x = wl.make_custom([40], 512, 512, wl.LAYER_NORM, 40, 6, seed=31, weight_param=0.05)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    xd = torch.from_numpy(xq).cuda()
    lib_model.set_option("rows16", rows16)
    lib_model.set_option("spin_limit", 64)
    lib_model.set_option("barrier_never_completes", 1)
    lib_model.forward(xd)
    torch.cuda.synchronize()
    assert lib_model.device_status() == 1
    lib_model.set_option("spin_limit", 1 << 21)
    lib_model.set_option("barrier_never_completes", 0)
    lib_model.set_option("reset_status", 1)
    assert lib_model.device_status() == 0
    y = lib_model.forward(xd)
    torch.cuda.synchronize()
    assert lib_model.device_status() == 0
    assert_equal("recovered", y.cpu().numpy(), orc.forward(orc_model, xq))


def test_batch_beyond_one_launch(orc):
    """N = 2048 with a projection: 8 groups of 64 rows per launch (two row tiles per
    group), so B = 600 runs in two launches, the second with a ragged last group
    whose second row tile is empty; still on the persistent path."""
    import torch

    print("batch beyond one launch", flush=True)
    layers, x = wl.make_custom([64], 2048, 640, wl.LAYER_NORM | wl.PROJECTION, 600, 3, seed=21, weight_param=0.03)
    lib_model, y = run_and_compare(orc, layers, x, "b600", trace=False,
                                   rows=[0, 31, 32, 63, 64, 255, 256, 511, 512, 543, 544, 575, 576, 599])
    lib_model.profile_begin()
    lib_model.forward(torch.zeros((3, 600, 64), dtype=torch.int8, device="cuda"))
    prof = lib_model.profile_end()
    assert prof["recurrent"]["launches"] == 2 and prof["cell"]["launches"] == 0, prof


def test_split_sequence_carries_state(orc):
    import torch

    layers, x = wl.make_custom([40, 24], 96, 24, wl.LAYER_NORM | wl.PROJECTION, 9, 12, seed=77)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    B = xq.shape[1]
    dims = lib_model.dims()
    xd = torch.from_numpy(xq).cuda()
    y = lib_model.forward(xd)
    hs = torch.cat([torch.full((B * d[2],), lib_model.get_quant(l)["zp_h"], dtype=torch.int8)
                    for l, d in enumerate(dims)]).cuda()
    cs = torch.zeros(sum(B * d[1] for d in dims), dtype=torch.int16).cuda()
    junk = lambda T: torch.randint(0, 256, (lib_model.workspace_bytes(T, B),), dtype=torch.uint8, device="cuda")
    ya = lib_model.forward(xd[:5].contiguous(), h_state=hs, c_state=cs, workspace=junk(5))
    yb = lib_model.forward(xd[5:].contiguous(), h_state=hs, c_state=cs, workspace=junk(7))
    torch.cuda.synchronize()
    assert_equal("split", torch.cat([ya, yb]).cpu().numpy(), y.cpu().numpy())
    assert_equal("split vs oracle", y.cpu().numpy(), orc.forward(orc_model, xq))


@pytest.mark.parametrize("path", [0, 1])
@pytest.mark.parametrize("flags", [0, wl.LAYER_NORM | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION])
def test_reverse_direction(orc, flags, path):
    """Option "reverse": the recursion runs from t = T - 1 down to 0 (the backward
    half of a bidirectional layer, Sec. 7), on both paths, two stacked layers,
    states carried in and out, every traced tensor at its position in time."""
    import torch

    print(f"reverse flags {flags} path {path}", flush=True)
    H = 40 if flags & wl.PROJECTION else 72
    layers, x = wl.make_custom([24, H], 72, 40, flags, 37, 5, seed=11 + flags)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    lib_model.set_option("reverse", 1)
    lib_model.set_option("path", path)
    T, B, _ = xq.shape
    dims = lib_model.dims()
    rng = np.random.Generator(np.random.PCG64(5))
    h0 = rng.integers(-128, 128, sum(B * d[2] for d in dims), dtype=np.int8)
    c0 = rng.integers(-3000, 3000, sum(B * d[1] for d in dims), dtype=np.int16)
    xd = torch.from_numpy(xq).cuda()
    for layer in range(2):
        hs, cs = torch.from_numpy(h0.copy()).cuda(), torch.from_numpy(c0.copy()).cuda()
        y, gtr = lib_model.forward(xd, h_state=hs, c_state=cs, trace_layer=layer)
        torch.cuda.synchronize()
        assert lib_model.device_status() == 0
        ohs, ocs = h0.copy(), c0.copy()
        yo, otr = orc.forward(orc_model, xq, h_state=ohs, c_state=ocs, trace_layer=layer, reverse=True)
        assert_equal("rev.y", y.cpu().numpy(), yo)
        assert_equal("rev.h_state", hs.cpu().numpy(), ohs)
        assert_equal("rev.c_state", cs.cpu().numpy(), ocs)
        compare_traces(f"rev.l{layer}", gtr, otr, flags)
    # without a trace the persistent kernel runs (path 0): same outputs
    hs, cs = torch.from_numpy(h0.copy()).cuda(), torch.from_numpy(c0.copy()).cuda()
    y2 = lib_model.forward(xd, h_state=hs, c_state=cs)
    torch.cuda.synchronize()
    assert lib_model.device_status() == 0
    assert_equal("rev.y untraced", y2.cpu().numpy(), yo)
    assert_equal("rev.h_state untraced", hs.cpu().numpy(), ohs)
    assert_equal("rev.c_state untraced", cs.cpu().numpy(), ocs)


@pytest.mark.parametrize("I", [40, 300, 520, 700, 1100])
def test_input_gemm_k_depths(orc, I):
    """One input size per register-depth class of the weight-resident input
    GEMM (k up to 256, 512, 640, 1024 bytes) and one beyond it, which takes the
    tiled GEMM; B = 70 leaves a ragged last block of rows."""
    print(f"input size {I}", flush=True)
    layers, x = wl.make_custom([I], 64, 64, 0, 70, 3, seed=I, weight_param=0.05)
    run_and_compare(orc, layers, x, f"in{I}", trace=False)


@pytest.mark.parametrize("steps", [8, 16, 24, 32, 40, 48])
def test_input_gemm_blocks_per_workgroup(orc, steps):
    """N = 2048 gives 32 column blocks, so the rows are split into 8 parts and a
    workgroup streams steps/8 blocks of 32 rows: 1 to 6, covering the start-up
    and the drain of its load and store pipeline."""
    print(f"steps {steps}", flush=True)
    layers, x = wl.make_custom([64], 2048, 64, wl.PROJECTION | wl.LAYER_NORM, 32, steps, seed=steps,
                               weight_param=0.05)
    run_and_compare(orc, layers, x, f"blocks{steps}", trace=False)


@pytest.mark.parametrize("N", [64, 128, 192, 256, 512, 1024])
def test_input_gemm_work_splits(orc, N):
    """The input GEMM spreads (row part, column block) pairs over the eight XCDs;
    the number of column blocks (N / 64) decides which split applies: 1, 2 and 3
    column blocks fall back to the plain split, 4, 8 and 16 take the grouped one
    with 64, 32 and 16 row parts.  42 steps x 48 rows = 63 blocks of 32 rows, so
    parts get one block, or two, or none."""
    print(f"cells {N}", flush=True)
    layers, x = wl.make_custom([96], N, N, 0, 48, 42, seed=N, weight_param=0.05)
    run_and_compare(orc, layers, x, f"split{N}", trace=False)


def test_small_shifts(orc):
    """Large weights push the effective scales of the gate terms to 1/4 and
    above, i.e. rescale shifts below 33, where the one-product form of rescale
    pre-shifts (and clamps) its operand."""
    print("small shifts", flush=True)
    from paper_2101_05453_amd import binding
    from parity_util import calibrate_on_gpu

    layers, x = wl.make_custom([48], 128, 128, wl.PEEPHOLE, 40, 6, seed=77, weight_param=0.6)
    calibrate_on_gpu(layers, x)
    q = binding.prepare(layers, device=0).get_quant(0)
    shifts = [31 - e for e in q["ex"] + q["eh"]]
    assert min(shifts) < 33, shifts
    run_and_compare(orc, layers, x, "small_shifts")


def test_saturating_ranges(orc):
    """Calibration ranges far too small: every clamp on the path is hit."""
    import torch

    layers, x = wl.make_custom([64], 128, 64, wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, 8, 6, seed=5,
                               weight_param=0.3)
    from paper_2101_05453_amd import binding
    from parity_util import calibrate_on_gpu

    xf = calibrate_on_gpu(layers, x)
    s = layers[0]
    s.g_absmax = [v * 0.05 for v in s.g_absmax]
    s.m_min, s.m_max, s.h_min, s.h_max, s.c_absmax = -0.02, 0.03, -0.05, 0.02, 0.4
    lib_model = binding.prepare(layers, device=0)
    orc_model = orc.prepare(layers)
    q0 = orc_model.layer(0)
    xq = lib_model.quantize_input((xf * 4).contiguous()).cpu().numpy()  # features beyond the calibrated range
    assert xq.min() == -128 and xq.max() == 127
    assert_equal("sat.xq", xq, orc.quantize_input(x * np.float32(4), q0["s_x"], q0["zp_x"]))
    y, gtr = lib_model.forward(torch.from_numpy(xq).cuda(), trace_layer=0)
    torch.cuda.synchronize()
    yo, otr = orc.forward(orc_model, xq, trace_layer=0)
    assert otr["g"].min() == -32767 and otr["g"].max() == 32767 and otr["m"].min() == -128 and otr["m"].max() == 127
    assert_equal("sat.y", y.cpu().numpy(), yo)
    for f in ("tx", "th", "g", "ln", "act", "c", "m", "h"):
        assert_equal(f"sat.{f}", gtr[f].cpu().numpy(), otr[f])


def test_empty_and_error_paths(orc):
    import torch

    from paper_2101_05453_amd import binding

    layers, x = wl.make_custom([64], 64, 64, 0, 4, 3, seed=2)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    xd = torch.from_numpy(xq).cuda()
    assert lib_model.forward(xd[:0].contiguous()).shape == (0, 4, 64)
    assert lib_model.forward(xd[:, :0].contiguous()).shape == (3, 0, 64)
    ws = torch.empty(lib_model.workspace_bytes(3, 4) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.LstmIntError) as ei:
        lib_model.forward(xd, workspace=ws)
    assert ei.value.code == binding.E_WORKSPACE
    # an input pointer that is not 16-byte aligned takes the padded-copy route
    big = torch.zeros(xd.numel() + 16, dtype=torch.int8, device="cuda")
    off = big[3:3 + xd.numel()].view(xd.shape)
    off.copy_(xd)
    y = lib_model.forward(off)
    torch.cuda.synchronize()
    assert_equal("unaligned", y.cpu().numpy(), orc.forward(orc_model, xq))


@pytest.mark.parametrize("T,flags,with_state,rows16", [
    (1 << 14, wl.LAYER_NORM, True, 1), ((1 << 14) + 1, wl.LAYER_NORM, True, 1),
    ((1 << 14) + 1, wl.LAYER_NORM | wl.PROJECTION, False, 1),
    (1 << 14, wl.LAYER_NORM, True, 0), ((1 << 14) + 1, wl.LAYER_NORM | wl.PROJECTION, False, 0)])
def test_longest_sequences(orc, T, flags, with_state, rows16):
    """2^14 steps is the most one launch of the persistent kernel takes (its
    layer-norm statistics words count up over the launch); one step more and
    the layer runs in two pieces, h and c carried from one to the next (c through
    the caller's state buffer, or through the workspace when there is none).  Two
    workgroups per group, so the words are in use.  On the 16-row kernel and,
    with option "rows16" off, on the kernel with groups of 32 rows."""
    print(f"T {T} rows16 {rows16}", flush=True)
    layers, x = wl.make_custom([16], 128, 64, flags, 3, T, seed=21)
    run_and_compare(orc, layers, x, f"long{T}", trace=False, with_state=with_state, options={"rows16": rows16})


def test_maximum_sizes(orc):
    """Layer norm at its row limit N = 4096; accumulation depth 2^15."""
    print("max sizes", flush=True)
    layers, x = wl.make_custom([16], 4096, 4096, wl.LAYER_NORM, 2, 2, seed=8, weight_param=0.02)
    run_and_compare(orc, layers, x, "ln4096", trace=True)
    layers, x = wl.make_custom([32768], 16, 16, 0, 3, 2, seed=9, weight_param=0.01)
    run_and_compare(orc, layers, x, "depth32768", trace=True)


@pytest.mark.parametrize("case", [
    # (inputs, N, H, flags, B, T, rows)
    ([72, 200], 200, 200, wl.LAYER_NORM, 37, 6, None),                      # 4 workgroups x 3 groups, ragged rows
    ([72, 136], 200, 136, wl.LAYER_NORM | wl.PROJECTION, 70, 5, None),      # 5 projection tiles over 4 workgroups
    ([40], 64, 64, wl.LAYER_NORM, 1, 7, None),                              # one workgroup, one row
    ([64], 456, 456, wl.LAYER_NORM, 40, 3, [0, 15, 16, 39]),                # h rows of 512 bytes (k depth class 10)
    ([64], 520, 520, wl.LAYER_NORM, 128, 3, [0, 15, 16, 100, 127]),         # k depth 10 without a projection
    ([64], 1024, 1024, wl.LAYER_NORM, 48, 3, [0, 17, 47]),                  # k depth 16
    ([640, 640], 2048, 640, wl.LAYER_NORM | wl.PROJECTION, 120, 4, [0, 17, 50, 119]),  # the C4 layer, 8 groups of 32
])
def test_rows16_kernel(orc, case):
    """Option "rows16" (on by default): batches of up to 16 * 8 * (32 / workgroups
    per group) rows take the recurrent kernel that works on groups of 16 rows."""
    _rows16(orc, case, 1)


@pytest.mark.parametrize("rows16", [1, 0])
@pytest.mark.parametrize("flags", VARIANTS)
def test_rows16_variants(orc, flags, rows16):
    """Every variant on the persistent path at a small ragged batch, two layers:
    on the 16-row kernel (default) and, with the option off, on the kernel
    with groups of 32 rows."""
    H = 136 if flags & wl.PROJECTION else 200
    _rows16(orc, ([72, H], 200, H, flags, 37, 5, None), rows16)


def test_rows16_c3_layer(orc):
    """The C3 layer (peephole, layer norm, projection: two statistics rounds per
    step) at B = 100 on the 16-row kernel."""
    flags = wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION
    _rows16(orc, ([640], 2048, 640, flags, 100, 4, [0, 15, 16, 63, 99]), 1)


def _rows16(orc, case, rows16):
    import torch

    inputs, N, H, flags, B, T, rows = case
    print(f"rows16={rows16} N={N} H={H} flags={flags} B={B} T={T}", flush=True)
    layers, x = wl.make_custom(inputs, N, H, flags, B, T, seed=N + B, weight_param=0.05 if N < 1024 else 0.03)
    lib_model, y = run_and_compare(orc, layers, x, f"rows16_{N}_{B}", trace=False, rows=rows,
                                   options={"rows16": rows16, "stack": 0})
    lib_model.profile_begin()
    lib_model.forward(torch.zeros((T, B, inputs[0]), dtype=torch.int8, device="cuda"))
    prof = lib_model.profile_end()
    assert prof["recurrent"]["launches"] == len(inputs) and prof["cell"]["launches"] == 0, prof


@pytest.mark.parametrize("stack", [0, 2])
def test_forward_captured_in_a_hip_graph(orc, stack):
    """forward allocates nothing, never synchronizes and launches only kernels, so
    a caller can capture it in a HIP graph: one-step calls with carried state,
    replayed with the program's own synchronization between the replays, give
    what the same calls give when made directly (and what the oracle gives for
    the whole sequence)."""
    import torch

    print(f"graph capture stack={stack}", flush=True)
    flags = wl.LAYER_NORM | wl.PROJECTION
    layers, x = wl.make_custom([72, 136], 200, 136, flags, 20, 6, seed=77, weight_param=0.08)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    lib_model.set_option("stack", stack)  # layer after layer, and all layers in one launch
    T, B, _ = xq.shape
    dims = lib_model.dims()
    want = orc.forward(orc_model, xq)

    def fresh_state():
        hs = torch.cat([torch.full((B * d[2],), lib_model.get_quant(l)["zp_h"], dtype=torch.int8)
                        for l, d in enumerate(dims)]).cuda()
        return hs, torch.zeros(sum(B * d[1] for d in dims), dtype=torch.int16).cuda()

    ws = torch.empty(lib_model.workspace_bytes(1, B), dtype=torch.uint8, device="cuda")
    xin = torch.from_numpy(np.ascontiguousarray(xq[:1])).cuda()
    y = torch.empty((1, B, dims[-1][2]), dtype=torch.int8, device="cuda")
    hs, cs = fresh_state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # first call outside the capture (one-time initialisation of the library)
        lib_model.forward(xin, y=y, workspace=ws, h_state=hs, c_state=cs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lib_model.forward(xin, y=y, workspace=ws, h_state=hs, c_state=cs)
    for rep in range(2):  # the whole sequence twice, from fresh state
        h0, c0 = fresh_state()
        hs.copy_(h0)
        cs.copy_(c0)
        for t in range(T):
            xin.copy_(torch.from_numpy(np.ascontiguousarray(xq[t:t + 1])))
            graph.replay()
            torch.cuda.synchronize()
            assert_equal(f"graph.rep{rep}.y[{t}]", y.cpu().numpy()[0], want[t])
    assert lib_model.device_status() == 0


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(orc, seed):
    """Seeded random layer shapes, variants, batches and lengths on the persistent
    path (whichever recurrent kernel the batch selects), two layers each."""
    rng = np.random.default_rng(1000 + seed)
    flags = int(rng.integers(0, 16))
    N = 8 * int(rng.integers(1, 60))
    H = int(rng.integers(8, N + 1)) if flags & wl.PROJECTION else N
    I = int(rng.integers(1, 200))
    B = int(rng.choice([1, 2, 15, 16, 17, 31, 33, 63, 100]))
    T = int(rng.integers(1, 6))
    print(f"random seed={seed} flags={flags} I={I} N={N} H={H} B={B} T={T}", flush=True)
    layers, x = wl.make_custom([I, H], N, H, flags, B, T, seed=seed + 500, weight_param=0.08)
    run_and_compare(orc, layers, x, f"random{seed}", trace=False, options={"rows16": seed % 3 != 2})


def test_large_input_product_on_the_per_step_path(orc):
    """The general matmul's tile for large products (2048 rows and more, 1024 output columns and more in blocks of
    256: 256 x 256 outputs per workgroup, eight waves): the hoisted W x of the per-step path with T * B = 2100 rows
    (a ragged last row block) by 4 * 320 = 1280 columns, every traced tensor against the oracle."""
    layers, x = wl.make_custom([100], 320, 320, wl.PEEPHOLE, 70, 30, seed=77, weight_param=0.05)
    run_and_compare(orc, layers, x, "tile256", trace=True, options={"path": 1})
