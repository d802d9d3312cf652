"""Shared plumbing of the GPU parity tests: collect statistics with the library's
float run on the GPU (lstm_int_calibrate), prepare both sides from the same float
parameters and statistics, quantize the features with the library (checked against
the oracle's quantizer), run the HIP library and the CPU oracle on the same int8
input, and compare integer tensors element by element."""
import numpy as np

from paper_2101_05453_amd import binding

TRACE_FIELDS = ("tx", "th", "g", "ln", "act", "c", "m", "h")


def calibrate_on_gpu(layers, x, device=0):
    """Fills the statistics of the layer specs from the library's float run over the
    first 16 batch rows of x (Sec. 4); returns x as a float32 device tensor."""
    import torch

    xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda(device)
    binding.calibrate(layers, xd, device=device, max_rows=16)
    return xd


def prepare_both(orc, layers, x, device=0, scale_x=1.0):
    """scale_x: the features fed to the quantizer are x * scale_x (to drive them out of
    the calibrated range)."""
    xd = calibrate_on_gpu(layers, x, device)
    lib_model = binding.prepare(layers, device=device)
    orc_model = orc.prepare(layers)
    if scale_x != 1.0:
        xd = (xd * np.float32(scale_x)).contiguous()
    xq = lib_model.quantize_input(xd).cpu().numpy()
    q0 = orc_model.layer(0)
    assert_equal("quantize_input", xq, orc.quantize_input(xd.cpu().numpy(), q0["s_x"], q0["zp_x"]))
    return lib_model, orc_model, xq


def assert_equal(name, got, want):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape and got.dtype == want.dtype, (name, got.shape, want.shape, got.dtype, want.dtype)
    if not (got == want).all():
        bad = np.argwhere(got != want)
        first = tuple(bad[0])
        raise AssertionError(f"{name}: {len(bad)} of {got.size} differ; first at {first}: "
                             f"gpu={got[first]} oracle={want[first]}")


def compare_traces(name, gpu_tr, orc_tr, flags):
    cifg, ln = bool(flags & 1), bool(flags & 4)
    for f in TRACE_FIELDS:
        g, o = gpu_tr[f].cpu().numpy(), orc_tr[f]
        if f == "ln" and not ln:
            continue
        if cifg and f in ("tx", "th", "g", "ln"):
            g, o = g[:, :, 1:], o[:, :, 1:]  # slot 0 is void under CIFG
        assert_equal(f"{name}.{f}", g, o)


def run_and_compare(orc, layers, x, name, trace=True, rows=None, with_state=True, options=None):
    """Full comparison on small problems (every traced tensor of every layer),
    or on a subset of batch rows (rows=...) for problems the oracle cannot
    finish whole: batch rows never interact, so the oracle runs only those
    rows."""
    import torch

    lib_model, orc_model, xq = prepare_both(orc, layers, x)
    for key, value in (options or {}).items():
        lib_model.set_option(key, value)
    T, B, _ = xq.shape
    dims = lib_model.dims()
    xd = torch.from_numpy(xq).cuda()
    hs = cs = None
    if with_state:
        hs = torch.cat([torch.full((B * d[2],), lib_model.get_quant(l)["zp_h"], dtype=torch.int8)
                        for l, d in enumerate(dims)]).cuda()
        cs = torch.zeros(sum(B * d[1] for d in dims), dtype=torch.int16).cuda()
    # a workspace full of garbage: nothing may depend on what a previous call left behind
    ws = torch.randint(-128, 128, (lib_model.workspace_bytes(T, B),), dtype=torch.int8, device="cuda").view(torch.uint8)
    y = lib_model.forward(xd, h_state=hs, c_state=cs, workspace=ws)
    torch.cuda.synchronize()
    assert lib_model.device_status() == 0, "a wait inside the persistent kernel gave up"
    y = y.cpu().numpy()
    sel = list(range(B)) if rows is None else list(rows)
    xs = np.ascontiguousarray(xq[:, sel])
    Bs = len(sel)
    ohs = np.concatenate([np.full(Bs * d[2], orc_model.layer(l)["zp_h"], np.int8) for l, d in enumerate(dims)])
    ocs = np.zeros(sum(Bs * d[1] for d in dims), np.int16)
    yo = orc.forward(orc_model, xs, h_state=ohs, c_state=ocs)
    assert_equal(f"{name}.y", y[:, sel], yo)
    if with_state:
        hs, cs = hs.cpu().numpy(), cs.cpu().numpy()
        ho = co = hso = cso = 0
        for l, (I, N, H) in enumerate(dims):
            assert_equal(f"{name}.h_state[{l}]", hs[ho:ho + B * H].reshape(B, H)[sel],
                         ohs[hso:hso + Bs * H].reshape(Bs, H))
            assert_equal(f"{name}.c_state[{l}]", cs[co:co + B * N].reshape(B, N)[sel],
                         ocs[cso:cso + Bs * N].reshape(Bs, N))
            ho, co, hso, cso = ho + B * H, co + B * N, hso + Bs * H, cso + Bs * N
    if trace:
        assert rows is None
        for l in range(len(layers)):
            yg, gtr = lib_model.forward(xd, trace_layer=l)
            torch.cuda.synchronize()
            _, otr = orc.forward(orc_model, xq, trace_layer=l)
            compare_traces(f"{name}.L{l}", gtr, otr, layers[l].flags)
            assert_equal(f"{name}.y(traced)", yg.cpu().numpy(), y)
    return lib_model, y
