"""The stacked launch (all layers of a stack of equal layers in one kernel, one layer
per XCD, each layer one step behind the one below: the wavefront over layers and
time of Sec. 7's stack) against the CPU oracle, bit for bit, through the C ABI:
outputs and final states of whole sequences, the state of every layer after every
step of one-step calls (the streaming use of Secs. 3.2.2 and 3.2.6), and the
configuration the benchmark shape is built from."""
import numpy as np
import pytest

import lstm_workloads as wl
from parity_util import assert_equal, prepare_both, run_and_compare

pytestmark = pytest.mark.gpu

VARIANTS = [0, wl.LAYER_NORM, wl.PEEPHOLE, wl.PROJECTION, wl.CIFG,
            wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM,
            wl.CIFG | wl.PEEPHOLE | wl.PROJECTION,
            wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.LAYER_NORM | wl.PROJECTION]


def _ran_stacked(lib_model, T, B, I0, layers):
    """One launch of the recurrent class for the whole stack (the launches one after
    the other need one per layer)."""
    import torch

    lib_model.profile_begin()
    lib_model.forward(torch.zeros((T, B, I0), dtype=torch.int8, device="cuda"))
    prof = lib_model.profile_end()
    assert lib_model.device_status() == 0
    return prof["recurrent"]["launches"] == 1 and prof["input_gemm"]["launches"] == 0 and prof["cell"]["launches"] == 0


@pytest.mark.parametrize("flags", VARIANTS)
def test_stack_variants(orc, flags):
    """Three equal layers, every variant, ragged sizes: I = 72, N = 200 (4 workgroups
    per layer, the last with 8 cells), H = 136 with a projection (5 projection tiles
    over 4 workgroups), B = 37 (two row tiles, the second with 5 rows), T = 6."""
    H = 136 if flags & wl.PROJECTION else 200
    print(f"stack variant flags={flags}", flush=True)
    layers, x = wl.make_custom([72, H, H], 200, H, flags, 37, 6, seed=flags + 301, weight_param=0.08)
    lib_model, _ = run_and_compare(orc, layers, x, f"stack{flags}", trace=False, options={"stack": 2})
    assert _ran_stacked(lib_model, 6, 37, 72, layers)


@pytest.mark.parametrize("case", [
    # (inputs, N, H, flags, B, T)
    ([40] + [64] * 7, 64, 64, wl.LAYER_NORM, 1, 9),                                   # 8 layers, one workgroup each, B = 1
    ([256, 512], 512, 512, wl.LAYER_NORM, 16, 12),                                    # the C2 layer, two deep (k depth 20)
    ([100, 320, 320, 320], 1024, 320, wl.LAYER_NORM | wl.PROJECTION, 70, 5),          # 16 workgroups per layer, 3 row tiles
    ([64, 256], 256, 256, wl.CIFG | wl.LAYER_NORM, 100, 4),                           # k depth 8, 4 row tiles
    ([1024, 1024], 1024, 1024, wl.CIFG | wl.LAYER_NORM, 40, 3),                       # the C5 layers (k depth 32)
])
def test_stack_shapes(orc, case):
    inputs, N, H, flags, B, T = case
    print(f"stack shape N={N} H={H} L={len(inputs)} B={B} T={T}", flush=True)
    layers, x = wl.make_custom(inputs, N, H, flags, B, T, seed=N + B + 7, weight_param=0.05 if N < 1024 else 0.03)
    rows = None if B * N * T * len(inputs) < 3e6 else sorted({0, 31, 32, B - 1})
    lib_model, _ = run_and_compare(orc, layers, x, f"stack_{N}_{B}", trace=False, rows=rows, options={"stack": 2})
    assert _ran_stacked(lib_model, T, B, inputs[0], layers)


@pytest.mark.parametrize("flags", [wl.LAYER_NORM | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE])
def test_stack_streaming_every_step_and_layer(orc, flags):
    """One-step calls with carried state on the stacked path: after every call the h
    and c of every layer equal the oracle's traces of that layer at that step."""
    import torch

    print(f"stack streaming flags={flags}", flush=True)
    H = 136 if flags & wl.PROJECTION else 200
    layers, x = wl.make_custom([72, H, H, H], 200, H, flags, 21, 7, seed=flags + 401, weight_param=0.08)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    lib_model.set_option("stack", 2)
    T, B, _ = xq.shape
    dims = lib_model.dims()
    traces = [orc.forward(orc_model, xq, trace_layer=l)[1] for l in range(len(layers))]
    want_y = orc.forward(orc_model, xq)
    hs = torch.cat([torch.full((B * d[2],), lib_model.get_quant(l)["zp_h"], dtype=torch.int8)
                    for l, d in enumerate(dims)]).cuda()
    cs = torch.zeros(sum(B * d[1] for d in dims), dtype=torch.int16).cuda()
    xd = torch.from_numpy(xq).cuda()
    ws = torch.randint(-128, 128, (lib_model.workspace_bytes(1, B),), dtype=torch.int8, device="cuda").view(torch.uint8)
    lib_model.profile_begin()
    for t in range(T):
        y = lib_model.forward(xd[t:t + 1].contiguous(), h_state=hs, c_state=cs, workspace=ws)
        torch.cuda.synchronize()
        assert_equal(f"y[{t}]", y.cpu().numpy()[0], want_y[t])
        h_np, c_np = hs.cpu().numpy(), cs.cpu().numpy()
        ho = co = 0
        for l, (I, N, Hl) in enumerate(dims):
            assert_equal(f"h[{t}] layer {l}", h_np[ho:ho + B * Hl].reshape(B, Hl), traces[l]["h"][t])
            assert_equal(f"c[{t}] layer {l}", c_np[co:co + B * N].reshape(B, N), traces[l]["c"][t])
            ho, co = ho + B * Hl, co + B * N
    prof = lib_model.profile_end()
    assert prof["recurrent"]["launches"] == T and prof["input_gemm"]["launches"] == 0, prof
    assert lib_model.device_status() == 0


@pytest.mark.parametrize("B,T", [(32, 1), (20, 16), (96, 8)])
def test_stack_c4_layers(orc, B, T):
    """The 8-layer stack of the headline configuration on the stacked path: a one-step
    call at B = 32, a short sequence, and three row tiles; sampled rows."""
    print(f"stack C4 B={B} T={T}", flush=True)
    layers, x = wl.make_workload("C4", batch=B, steps=T)
    rows = sorted({0, B // 2, B - 1} | ({31, 32, 64} if B > 64 else set()))
    lib_model, _ = run_and_compare(orc, layers, x, f"stackC4_{B}_{T}", trace=False, rows=rows, options={"stack": 2})
    assert _ran_stacked(lib_model, T, B, 512, layers)


@pytest.mark.parametrize("B,T", [(32, 3000), (70, 700)])
def test_stack_long_sequences_match_the_layer_by_layer_path(orc, B, T):
    """Many hand-offs between XCDs: the 8-layer headline stack over thousands of
    steps on the stacked path gives, bit for bit, what the same library gives layer
    after layer (the path the oracle checks at full size), outputs and final
    states; and the first steps are checked against the oracle directly."""
    import torch

    from paper_2101_05453_amd import binding
    from parity_util import calibrate_on_gpu

    print(f"stack long B={B} T={T}", flush=True)
    layers, x64 = wl.make_workload("C4", batch=B)
    calibrate_on_gpu(layers, x64)
    model = binding.prepare(layers, device=0)
    rng = np.random.Generator(np.random.PCG64(T))
    xq = rng.integers(-128, 128, (T, B, 512), dtype=np.int8)
    xd = torch.from_numpy(xq).cuda()
    outs = {}
    for stack in (0, 2):
        model.set_option("stack", stack)
        hs = torch.zeros(8 * B * 640, dtype=torch.int8, device="cuda")
        cs = torch.zeros(8 * B * 2048, dtype=torch.int16, device="cuda")
        y = model.forward(xd, h_state=hs, c_state=cs)
        torch.cuda.synchronize()
        assert model.device_status() == 0
        outs[stack] = (y.cpu().numpy(), hs.cpu().numpy(), cs.cpu().numpy())
    for name, a, b in zip(("y", "h_state", "c_state"), outs[2], outs[0]):
        assert_equal(f"long.{name}", a, b)
    om = orc.prepare(layers)
    rows = [0, B - 1]
    hs0 = np.zeros(8 * 2 * 640, np.int8)
    cs0 = np.zeros(8 * 2 * 2048, np.int16)
    want = orc.forward(om, np.ascontiguousarray(xq[:12, rows]), h_state=hs0, c_state=cs0)
    assert_equal("long.y vs oracle", outs[2][0][:12, rows], want)


def test_stack_wait_gives_up_and_model_recovers(orc):
    """The bounded waits of the stacked launch: with a barrier that cannot complete
    every workgroup of every layer leaves the kernel -- the layers above give up on
    the flag of the layer below -- the status word says so, and after a reset the
    model computes the right answer again."""
    import torch

    print("stack bounded waits", flush=True)
    layers, x = wl.make_custom([40, 512, 512], 512, 512, wl.LAYER_NORM, 40, 4, seed=33, weight_param=0.05)
    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    lib_model.set_option("stack", 2)
    xd = torch.from_numpy(xq).cuda()
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


def test_stack_falls_back(orc):
    """Layers that differ (or a trace request) run one after the other as before, with
    the option on."""
    layers, x = wl.make_custom([72, 200], 200, 200, wl.LAYER_NORM, 10, 4, seed=9)
    layers2, _ = wl.make_custom([200], 136, 136, wl.LAYER_NORM, 10, 4, seed=10)
    lib_model, _ = run_and_compare(orc, layers + layers2, x, "stack_mixed", trace=True, options={"stack": 2})
    assert not _ran_stacked(lib_model, 4, 10, 72, layers)
