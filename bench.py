"""Benchmark of the integer LSTM hot path on one MI355X.

A "step" is one lstm_int_forward call: the whole hot path (input GEMM over all
T, then T recurrent steps, for every layer) over one synthetic batch that is
already resident in HBM.  The metric is LSTM cell-steps/s = B*T*L / time.
Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0  # MI355X dense int8 MFMA, TOP/s (published)
PEAK_HBM_GBS = 8000.0  # MI355X HBM3E, GB/s (published)


def algorithmic_work(q, B, T):
    """Per-launch algorithmic int8 ops / bytes of each kernel class for one
    layer (what the operation must move or multiply at the storage types the
    method fixes: int8 weights and activations, int16 gate terms and cell)."""
    I, N, H, G = q["I"], q["N"], q["H"], q["G"]
    proj = bool(q["flags"] & 8)
    return {
        # one launch covers all T*B rows
        "input_gemm": {"ops": 2.0 * T * B * G * N * I, "bytes": G * N * I + T * B * I + 2.0 * T * B * G * N},
        # one launch per step
        "recurrent": {"ops": 2.0 * B * G * N * H, "bytes": G * N * H + B * H + 2.0 * B * G * N},
        "cell": {"ops": 0.0, "bytes": 2.0 * B * G * N * 2 + 4.0 * B * N + B * N},
        "projection": {"ops": 2.0 * B * H * N if proj else 0.0, "bytes": (H * N + B * N + B * H) if proj else 0.0},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (batch rows would shard across GPUs "
                 "with no exchange, but no multi-GPU path is built); use --gpus 1")

    import numpy as np
    import torch

    import lstm_workloads as wl
    from paper_2101_05453_amd import binding, calibration

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    binding.lib()
    cfg = wl.CONFIGS[args.config]
    layers, x = wl.make_workload(args.config)
    calibration.collect_statistics(layers, x)  # statistics from the first 16 rows (Sec. 4)
    model = binding.prepare(layers, device=0)
    L = model.num_layers
    quants = [model.get_quant(l) for l in range(L)]
    xq = calibration.quantize_input(x, quants[0]["s_x"], quants[0]["zp_x"])
    T, B, _ = xq.shape
    xd = torch.from_numpy(xq).cuda()
    y = torch.empty((T, B, quants[-1]["H"]), dtype=torch.int8, device="cuda")
    ws = torch.empty(model.workspace_bytes(T, B), dtype=torch.uint8, device="cuda")

    def step():
        model.forward(xd, y=y, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    cell_steps = B * T * L
    value = cell_steps * args.steps / dt

    # per-kernel device time over the same K steps, HIP events on the launch stream
    model.profile_begin()
    for _ in range(args.steps):
        step()
    prof = model.profile_end()
    work = {k: {"ops": 0.0, "bytes": 0.0, "launches": 0} for k in ("input_gemm", "recurrent", "cell", "projection")}
    for q in quants:
        w = algorithmic_work(q, B, T)
        for k in work:
            n = 1 if k == "input_gemm" else T
            if k == "projection" and not (q["flags"] & 8):
                n = 0
            work[k]["ops"] += w[k]["ops"] * n
            work[k]["bytes"] += w[k]["bytes"] * n
            work[k]["launches"] += n
    kernels = {}
    for k, w in work.items():
        p = prof[k]
        if not p["launches"]:
            continue
        avg_ms = p["total_ms"] / p["launches"]
        ent = {"launches_per_step": w["launches"], "avg_us": avg_ms * 1e3,
               "ms_per_step": p["total_ms"] / args.steps}
        if w["launches"]:
            ent["gbps"] = w["bytes"] / w["launches"] / (avg_ms * 1e-3) / 1e9
            ent["tops"] = w["ops"] / w["launches"] / (avg_ms * 1e-3) / 1e12
        kernels[k] = ent
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    d = kernels[dominant]
    if dominant == "input_gemm":
        roof = {"bound": "mfma", "achieved": d["tops"], "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": d["tops"] / PEAK_INT8_TOPS}
    else:
        roof = {"bound": "hbm", "achieved": d["gbps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": d["gbps"] / PEAK_HBM_GBS}
    roof.update({"kernel": dominant, "avg_launch_us": d["avg_us"], "traffic": None, "kernels": kernels})
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):  # HBM bytes per launch from rocprofv3 --pmc runs (see profiles/)
        rec = json.load(open(tpath)).get(args.config, {}).get(dominant)
        if rec:
            roof["traffic"] = rec["bytes_per_launch"]

    out = {
        "metric": "lstm_cell_steps_per_sec", "value": value, "unit": "cell-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": wl.describe(args.config), "cell_steps_per_step": cell_steps,
                   "batch": B, "seq_len": T, "layers": L},
        "roofline": roof,
    }

    if not args.no_cpu_baseline:
        # the oracle as it stands, on a bounded sample: one batch row per host
        # thread, the first steps of the same workload, all layers
        import oracle

        cores = min(oracle.max_threads(), 16, B)
        Ts = min(T, 16)
        om = oracle.prepare(layers)
        xs = np.ascontiguousarray(xq[:Ts, :cores])
        t0 = time.perf_counter()
        oracle.forward(om, xs, threads=cores)
        dto = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": cores * Ts * L / dto, "unit": "cell-steps/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"first {cores} batch rows x first {Ts} steps x {L} layers of "
                                         f"{args.config}, {dto:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
