"""Pruned models (Table 1: the 50 %-sparse LSTM and CIFG rows) in 2:4 structured form: the persistent kernel
runs R h on the sparse MFMA from compressed operands.  The integers must be those of the dense arithmetic on
the same (zero-containing) weights, which is what the CPU oracle computes; compared bit for bit through the C
ABI, with the dense kernel run on the same model as a second reference."""
import numpy as np
import pytest

import lstm_workloads as wl
from parity_util import assert_equal, run_and_compare

pytestmark = pytest.mark.gpu

VARIANTS = [0, wl.LAYER_NORM, wl.PEEPHOLE, wl.PROJECTION, wl.CIFG,
            wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION, wl.CIFG | wl.LAYER_NORM,
            wl.CIFG | wl.PEEPHOLE | wl.PROJECTION,
            wl.CIFG | wl.LAYER_NORM | wl.PEEPHOLE | wl.PROJECTION]

# the kernel with groups of 32 rows, one launch per layer (the sparse form belongs to it); sparse = 2: a call in
# which a 2:4 layer would fall back to the dense product fails instead of passing unnoticed
OPTS = {"rows16": 0, "stack": 0, "sparse": 2}


def _dense_again(lib_model, x_shape, y_sparse, seed):
    """The same model and input through the dense product (option sparse = 0) gives the same bytes."""
    import torch

    T, B, I = x_shape
    g = torch.Generator(device="cpu").manual_seed(seed)
    xq = torch.randint(-128, 128, (T, B, I), dtype=torch.int8, generator=g).cuda()
    ys = lib_model.forward(xq).cpu().numpy()
    lib_model.set_option("sparse", 0)
    yd = lib_model.forward(xq).cpu().numpy()
    lib_model.set_option("sparse", 2)
    assert lib_model.device_status() == 0
    assert_equal("sparse against dense kernel", ys, yd)


@pytest.mark.parametrize("flags", VARIANTS)
def test_sparse_variants(orc, flags):
    """Every variant, two layers, ragged sizes (N = 200: the last workgroup of a group has 8 cells; H = 136
    with a projection; B = 37: a group of 32 rows and one of 5), R pruned to 2:4."""
    H = 136 if flags & wl.PROJECTION else 200
    print(f"sparse variant flags={flags}", flush=True)
    layers, x = wl.make_custom([72, H], 200, H, flags, 37, 5, seed=flags + 77, weight_param=0.08)
    wl.prune_2of4(layers)
    lib_model, y = run_and_compare(orc, layers, x, f"sparse{flags}", trace=False, options=OPTS)
    assert lib_model.sparse_layers() == 2
    _dense_again(lib_model, x.shape, y, flags)


@pytest.mark.parametrize("case", [
    # (inputs, N, H, flags, B, T, rows compared with the oracle or None = all)
    ([40], 64, 64, 0, 1, 6, None),                                              # one workgroup per group, k depth 8, B = 1
    ([100], 512, 100, wl.LAYER_NORM | wl.PROJECTION, 70, 4, None),              # H not a multiple of 4 or 64
    ([256, 512], 512, 512, wl.LAYER_NORM, 48, 6, [0, 31, 32, 47]),              # the C2 layer, k depth 20
    ([640, 640], 2048, 640, wl.LAYER_NORM | wl.PROJECTION, 256, 6, "edges"),    # the C4 layer at its batch: all 8 XCDs
    ([1024], 1024, 1024, wl.CIFG | wl.LAYER_NORM, 200, 3, [0, 31, 96, 199]),    # the C5 layer (k depth 32)
])
def test_sparse_shapes(orc, case):
    inputs, N, H, flags, B, T, rows = case
    print(f"sparse shape N={N} H={H} L={len(inputs)} B={B} T={T}", flush=True)
    layers, x = wl.make_custom(inputs, N, H, flags, B, T, seed=N + B + 3, weight_param=0.05 if N < 1024 else 0.03)
    wl.prune_2of4(layers, ("R", "W", "Wproj"))
    if rows == "edges":  # first and last row of every group of 32
        rows = sorted({r for g in range((B + 31) // 32) for r in (32 * g, min(32 * g + 31, B - 1))})
    lib_model, y = run_and_compare(orc, layers, x, f"sparse_{N}_{B}", trace=False, rows=rows, options=OPTS)
    assert lib_model.sparse_layers() == len(inputs)
    _dense_again(lib_model, x.shape, y, N)


def test_sparse_only_where_the_weights_allow(orc):
    """A model with one pruned and one dense layer: the count says so, and both layers give the oracle's
    integers; a single third nonzero in one group of one row makes a layer dense."""
    layers, x = wl.make_custom([72, 200], 200, 200, wl.LAYER_NORM, 40, 4, seed=5, weight_param=0.08)
    wl.prune_2of4(layers[:1])
    lib_model, _ = run_and_compare(orc, layers, x, "sparse_mixed", trace=False, options=OPTS)
    assert lib_model.sparse_layers() == 1
    layers, x = wl.make_custom([72], 200, 200, 0, 8, 3, seed=6, weight_param=0.08)
    wl.prune_2of4(layers)
    R = layers[0].R[2]
    R[17, 40:44] = [0.05, -0.05, 0.05, 0.0]
    lib_model, _ = run_and_compare(orc, layers, x, "sparse_not_quite", trace=False, options=OPTS)
    assert lib_model.sparse_layers() == 0


def test_sparse_required_but_not_possible(orc):
    """Option sparse = 2 where the sparse form does not run (the 16-row kernel takes this batch): the call fails
    with a clean error, and works again with the option at 1."""
    import torch
    from paper_2101_05453_amd import binding

    layers, x = wl.make_custom([72], 200, 200, wl.LAYER_NORM, 8, 3, seed=9, weight_param=0.08)
    wl.prune_2of4(layers)
    lib_model, _ = run_and_compare(orc, layers, x, "sparse_small_batch", trace=False, options={"stack": 0})
    assert lib_model.sparse_layers() == 1
    xq = torch.zeros((3, 8, 72), dtype=torch.int8, device="cuda")
    lib_model.set_option("sparse", 2)
    with pytest.raises(RuntimeError):
        lib_model.forward(xq)
    lib_model.set_option("sparse", 1)
    lib_model.forward(xq)
    torch.cuda.synchronize()
    assert lib_model.device_status() == 0


def test_sparse_with_state_over_calls(orc):
    """A sequence in pieces with carried state: the sparse kernel's state hand-over is the dense kernel's."""
    import torch

    layers, x = wl.make_custom([72, 136], 200, 136, wl.LAYER_NORM | wl.PROJECTION, 33, 9, seed=21, weight_param=0.08)
    wl.prune_2of4(layers)
    lib_model, y = run_and_compare(orc, layers, x, "sparse_whole", trace=False, options=OPTS)
    g = torch.Generator(device="cpu").manual_seed(3)
    xq = torch.randint(-128, 128, (9, 33, 72), dtype=torch.int8, generator=g).cuda()
    dims = lib_model.dims()

    def fresh():
        hs = torch.cat([torch.full((33 * d[2],), lib_model.get_quant(l)["zp_h"], dtype=torch.int8)
                        for l, d in enumerate(dims)]).cuda()
        return hs, torch.zeros(sum(33 * d[1] for d in dims), dtype=torch.int16).cuda()

    hs, cs = fresh()
    whole = lib_model.forward(xq, h_state=hs, c_state=cs).cpu().numpy()
    hs2, cs2 = fresh()
    parts = [lib_model.forward(xq[a:b].contiguous(), h_state=hs2, c_state=cs2).cpu().numpy()
             for a, b in ((0, 1), (1, 5), (5, 9))]
    assert lib_model.device_status() == 0
    assert_equal("pieces.y", np.concatenate(parts), whole)
    assert_equal("pieces.h", hs2.cpu().numpy(), hs.cpu().numpy())
    assert_equal("pieces.c", cs2.cpu().numpy(), cs.cpu().numpy())
