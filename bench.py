"""Benchmark of the integer LSTM hot path on one MI355X.

A "step" is one lstm_int_forward call: the whole hot path (input GEMM over all
T, then T recurrent steps, for every layer) over one synthetic batch that is
already resident in HBM.  The metric is LSTM cell-steps/s = B*T*L / time.
Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4] [--batch B] [--seq-len T]

--batch / --seq-len shrink the configuration (its first rows and steps): the streaming and
small-batch regimes of the same stack, which take the stacked launch (one layer per XCD).
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


def algorithmic_work(q, B, T, persistent):
    """Algorithmic int8 ops / bytes of each kernel class for one layer: what the
    operation must move or multiply at the storage types the method fixes (int8
    weights and activations, int16 gate terms and cell state)."""
    I, N, H, G = q["I"], q["N"], q["H"], q["G"]
    proj = bool(q["flags"] & 8)
    Hout = H
    w = {
        # one launch covers all T*B rows
        "input_gemm": {"ops": 2.0 * T * B * G * N * I, "bytes": G * N * I + T * B * I + 2.0 * T * B * G * N,
                       "launches": 1},
    }
    if persistent:
        # one launch runs all T steps; per step: weights once, W x terms, cell
        # state in and out, h in, h out
        weights = G * N * H + (Hout * N if proj else 0)
        step = weights + 2.0 * B * G * N + 4.0 * B * N + B * H + B * Hout
        ops = 2.0 * B * (G * N * H + (Hout * N if proj else 0))
        # bytes_resident: the same step with the weights kept on chip (read from HBM once per launch)
        w["recurrent"] = {"ops": ops * T, "bytes": step * T, "bytes_resident": (step - weights) * T + weights,
                          "launches": 1}
    else:
        w["recurrent"] = {"ops": 2.0 * B * G * N * H * T, "bytes": (G * N * H + B * H + 2.0 * B * G * N) * T,
                          "launches": T}
        w["cell"] = {"ops": 0.0, "bytes": (2.0 * B * G * N * 2 + 4.0 * B * N + B * N) * T, "launches": T}
        if proj:
            w["projection"] = {"ops": 2.0 * B * H * N * T, "bytes": (H * N + B * N + B * H) * T, "launches": T}
    return w


def bench_gru(args, np, torch, wl, binding):
    """One step = one gru_int_forward call on a synthetic batch resident in HBM; checked against the oracle on a
    few rows and steps in the same run.  Roofline of the step kernel: the bytes one step must move with the
    weights re-streamed (3 N^2 int8 weights, int16 W x terms, int16 state in and out, int8 state in and three
    int8 copies out) against its HIP-event time."""
    L, I, N, B, T = (int(v) for v in args.gru.split(","))
    layers, x = wl.make_gru([I] + [N] * (L - 1), N, B, T, seed=0, weight_param=0.03)
    model = binding.gru_prepare(layers, device=0)
    q0 = model.get_quant(0)
    xq = np.clip(np.floor(x.astype(np.float64) / q0["s_x"] + 0.5) + q0["zp_x"], -128, 127).astype(np.int8)
    xd = torch.from_numpy(xq).cuda()
    ws = torch.empty(model.workspace_bytes(T, B), dtype=torch.uint8, device="cuda")
    y = model.forward(xd, workspace=ws)
    for _ in range(args.warmup):
        model.forward(xd, y=y, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        model.forward(xd, y=y, workspace=ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    model.profile_begin()
    for _ in range(args.steps):
        model.forward(xd, y=y, workspace=ws)
    prof = model.profile_end()
    step_us = prof["step"]["total_ms"] / prof["step"]["launches"] * 1e3
    gemm_us = prof["input_gemm"]["total_ms"] / prof["input_gemm"]["launches"] * 1e3
    # which form of the recurrent part the library runs for this shape (include/gru_int.h: gru_int_forward)
    ctiles = (N + 31) // 32
    persistent = ((N + 63) // 64) * 64 <= 1024 and ctiles <= 32 and (B + 31) // 32 <= 8 * (32 // ctiles)
    step_bytes = 3.0 * N * N + 2.0 * B * 3 * N + 4.0 * B * N + B * N + 3.0 * B * N
    gemm_ops = sum(2.0 * T * B * 3 * N * (I if l == 0 else N) for l in range(L)) / L
    out = {"metric": "gru_cell_steps_per_sec", "value": B * T * L / dt, "unit": "cell-steps/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
           "config": {"workload": f"integer GRU: L={L} I={I} N={N} B={B} T={T}", "cell_steps_per_step": B * T * L},
           "roofline": {"bound": "hbm", "achieved": step_bytes / step_us * 1e-3, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": step_bytes / step_us * 1e-3 / PEAK_HBM_GBS,
                        "kernel": "gru_seq_kernel" if persistent else "gru_step_kernel",
                        "path": "persistent: one launch per layer, avg_launch_us is its time per step" if persistent
                        else "one launch per step",
                        "avg_launch_us": step_us, "traffic": None,
                        "kernels": {"input_gemm": {"avg_us": gemm_us, "tops": gemm_ops / gemm_us * 1e-6,
                                                   "frac_mfma": gemm_ops / gemm_us * 1e-6 / PEAK_INT8_TOPS}}}}
    if not args.no_cpu_baseline:
        from oracle import gru as ogru

        rows = sorted(set(int(r) for r in np.linspace(0, B - 1, min(B, 8))))
        Ts = min(T, 16)
        om = ogru.GruModel(layers)
        t0 = time.perf_counter()
        yo, _ = om.forward(xq[:Ts, rows], threads=len(rows))
        ot = time.perf_counter() - t0
        eq = bool((y[:Ts].cpu().numpy()[:, rows] == yo).all())
        out["cpu_baseline"] = {"value": len(rows) * Ts * L / ot, "unit": "cell-steps/s", "cores": len(rows), "kind": "oracle",
                               "sample": f"{len(rows)} rows spread over the batch x first {Ts} steps x {L} layers, {ot:.1f} s"}
        out["parity"] = {"rows": len(rows), "steps": Ts, "layers": L, "equal": eq}
        if not eq:
            print(json.dumps(out))
            sys.exit("bench.py: the GRU output differs from the oracle's")
    print(json.dumps(out))


def sru_float_statistics(layers, x, torch):
    """The calibration run of Sec. 4 for the SRU: the float cell in float64 on the GPU with torch ops (plumbing
    outside the timed region), logging what sru_int_prepare needs: the largest magnitude of state, candidate and
    highway term, and the range of the output, per layer."""
    inp = torch.from_numpy(x).cuda().double()
    for s in layers:
        W = [None if w is None else torch.from_numpy(w).cuda().double() for w in s.W]
        v = [torch.from_numpy(a).cuda().double() for a in s.v]
        b = [torch.from_numpy(a).cuda().double() for a in s.b]
        xc, af, ar = inp @ W[0].T, inp @ W[1].T + b[0], inp @ W[2].T + b[1]
        hw = inp if W[3] is None else inp @ W[3].T
        c = torch.zeros_like(xc[0])
        out = torch.empty_like(xc)
        cmax = max(float(xc.abs().max()), float(hw.abs().max()))
        for t in range(inp.shape[0]):
            f, r = torch.sigmoid(af[t] + v[0] * c), torch.sigmoid(ar[t] + v[1] * c)
            c = f * c + (1 - f) * xc[t]
            out[t] = r * c + (1 - r) * hw[t]
            cmax = max(cmax, float(c.abs().max()))
        s.c_absmax, s.h_min, s.h_max = cmax, min(float(out.min()), 0.0), max(float(out.max()), 0.0)
        inp = out


def bench_sru(args, np, torch, wl, binding):
    """One step = one sru_int_forward call on a synthetic batch resident in HBM; checked against the oracle on a
    few rows in the same run.  Roofline of the scan kernel: the bytes it must stream (the int16 slot terms in, the
    input bytes of a layer whose highway term is its input, the int8 output) against its HIP-event time."""
    L, I, N, B, T = (int(v) for v in args.sru.split(","))
    layers, x = wl.make_sru([I] + [N] * (L - 1), N, B, T, seed=0, weight_param=0.03)
    sru_float_statistics(layers, x, torch)
    model = binding.sru_prepare(layers, device=0)
    q0 = model.get_quant(0)
    xq = np.clip(np.floor(x.astype(np.float64) / q0["s_x"] + 0.5) + q0["zp_x"], -128, 127).astype(np.int8)
    xd = torch.from_numpy(xq).cuda()
    ws = torch.empty(model.workspace_bytes(T, B), dtype=torch.uint8, device="cuda")
    y = model.forward(xd, workspace=ws)
    for _ in range(args.warmup):
        model.forward(xd, y=y, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        model.forward(xd, y=y, workspace=ws)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    model.profile_begin()
    for _ in range(args.steps):
        model.forward(xd, y=y, workspace=ws)
    prof = model.profile_end()
    scan_us = prof["scan"]["total_ms"] / prof["scan"]["launches"] * 1e3
    gemm_us = prof["input_gemm"]["total_ms"] / prof["input_gemm"]["launches"] * 1e3
    G = [4 if s.W[3] is not None else 3 for s in layers]
    scan_bytes = sum(T * B * N * (2.0 * g + 1 + (1 if g == 3 else 0)) for g in G) / L
    gemm_ops = sum(2.0 * T * B * g * N * s.input_size for g, s in zip(G, layers)) / L
    out = {"metric": "sru_cell_steps_per_sec", "value": B * T * L / dt, "unit": "cell-steps/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
           "config": {"workload": f"integer SRU: L={L} I={I} N={N} B={B} T={T}", "cell_steps_per_step": B * T * L},
           "roofline": {"bound": "hbm", "achieved": scan_bytes / scan_us * 1e-3, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": scan_bytes / scan_us * 1e-3 / PEAK_HBM_GBS, "kernel": "sru_scan_kernel",
                        "avg_launch_us": scan_us, "traffic": None,
                        # what actually bounds the scan: its instruction stream.  80 instructions per cell and step
                        # (vector, scalar, LDS and memory instructions of the compiled loops, / 16 cell-steps per
                        # round) against 256 CUs x 64 lanes x 2.4 GHz, one instruction per lane and clock
                        "issue": {"bound": "alu", "achieved": T * B * N * 80.0 / scan_us * 1e-6, "peak": 39.3,
                                  "unit": "T lane-instructions/s", "frac": T * B * N * 80.0 / scan_us * 1e-6 / 39.3},
                        "kernels": {"input_gemm": {"avg_us": gemm_us, "tops": gemm_ops / gemm_us * 1e-6,
                                                   "frac_mfma": gemm_ops / gemm_us * 1e-6 / PEAK_INT8_TOPS}}}}
    if not args.no_cpu_baseline:
        from oracle import sru as osru

        rows = sorted(set(int(r) for r in np.linspace(0, B - 1, min(B, 8))))
        om = osru.SruModel(layers)
        t0 = time.perf_counter()
        yo, _ = om.forward(xq[:, rows], threads=len(rows))
        ot = time.perf_counter() - t0
        eq = bool((y.cpu().numpy()[:, rows] == yo).all())
        out["cpu_baseline"] = {"value": len(rows) * T * L / ot, "unit": "cell-steps/s", "cores": len(rows), "kind": "oracle",
                               "sample": f"{len(rows)} rows spread over the batch x {T} steps x {L} layers, {ot:.1f} s"}
        out["parity"] = {"rows": len(rows), "steps": T, "layers": L, "equal": eq}
        if not eq:
            print(json.dumps(out))
            sys.exit("bench.py: the SRU output differs from the oracle's")
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--batch", type=int, default=0, help="fewer batch rows than the configuration has (its first rows)")
    ap.add_argument("--seq-len", type=int, default=0, help="fewer steps than the configuration has (its first steps)")
    ap.add_argument("--stack", type=int, default=-1, help="option 'stack' of the library (default: the library's own choice)")
    ap.add_argument("--sparse", action="store_true",
                    help="prune the synthetic weights W, R, W_proj to two nonzeros per aligned group of four inputs "
                         "(the structured stand-in for the 50 %% sparse models of Table 1): R h runs on the sparse MFMA")
    ap.add_argument("--phase-timing", action="store_true",
                    help="diagnostics instead of the benchmark: the recurrent kernel's phase timers (workgroup 0), "
                         "microseconds per step and phase, as one JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--path", type=int, default=0, help="0 auto, 1 one launch per operation and step")
    ap.add_argument("--mfma-store-ceiling", action="store_true",
                    help="only measure what the chip sustains for the input GEMM's mix of int8 MFMAs and streaming stores")
    ap.add_argument("--lds-probe", action="store_true",
                    help="only launch the LDS access pattern probes of the matmul kernels' lane -> address maps, for rocprofv3 --pmc")
    ap.add_argument("--gru", default="", metavar="L,I,N,B,T",
                    help="benchmark the integer GRU instead (the cell Sec. 7 names; gru_int_forward): L layers of N cells, "
                         "layer 0 input I, B rows, T steps, e.g. 2,512,2048,256,64; one JSON line")
    ap.add_argument("--sru", default="", metavar="L,I,N,B,T",
                    help="benchmark the integer SRU instead (the other cell Sec. 7 names; sru_int_forward): L layers of N "
                         "cells, layer 0 input I, B rows, T steps, e.g. 4,512,2048,256,64; one JSON line")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of MIB MiB (a known-size reference for rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (batch rows would shard across GPUs "
                 "with no exchange, but no multi-GPU path is built); use --gpus 1")

    import numpy as np
    import torch

    import lstm_workloads as wl
    from paper_2101_05453_amd import binding

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n, "copies": 3}))
        return
    binding.lib()
    if args.sru:
        bench_sru(args, np, torch, wl, binding)
        return
    if args.gru:
        bench_gru(args, np, torch, wl, binding)
        return
    if args.lds_probe:
        rows = []
        for name, mp in (("operand of the 16x16x64 MFMA (row = lane % 16)", 0), ("operand of the 32x32x32 MFMA (row = lane % 32)", 1),
                         ("staging order (four lanes per row)", 2)):
            for stride, swz in ((12, 0), (16, 0), (20, 0), (24, 0), (36, 0), (68, 0), (16, 1), (16, 2)):
                for write in (False, True):
                    binding.lds_probe(mp, stride, swz, write)
                    rows.append({"dispatch": len(rows), "map": name, "stride_words": stride, "swizzle": swz, "write": write})
        print(json.dumps({"lds_probe": rows, "note": "one launch of lds_probe_kernel per row, in this order; run under rocprofv3 "
                          "--pmc SQ_LDS_IDX_ACTIVE SQ_LDS_BANK_CONFLICT: IDX_ACTIVE / 16384 = LDS clocks per wave access of 16 "
                          "bytes per lane (4 for a read and 8 for a write without conflicts); swizzle 1 = piece ^ ((row >> 1) & 3), "
                          "2 = piece ^ ((row >> 2) & 3)"}))
        return
    if args.mfma_store_ceiling:
        rows = [binding.mfma_store_ceiling(s) for s in (0, 1, 2, 4, 8)]
        print(json.dumps({"mfma_store_ceiling": rows, "note": "40 int8 MFMAs (32x32x32) per wave and round on every CU, "
                          "plus stores_per_block KB of streaming stores per wave and round; 4 = the C4 input GEMM's mix"}))
        return
    cfg = wl.CONFIGS[args.config]
    layers, x = wl.make_workload(args.config, batch=args.batch or None, steps=args.seq_len or None)
    if args.sparse:
        wl.prune_2of4(layers, ("W", "R", "Wproj"))
    xf = torch.from_numpy(x).cuda()
    binding.calibrate(layers, xf, device=0, max_rows=16)  # statistics of the float run on the first 16 rows (Sec. 4)
    model = binding.prepare(layers, device=0)
    model.set_option("path", args.path)
    if args.stack >= 0:
        model.set_option("stack", args.stack)
    L = model.num_layers
    quants = [model.get_quant(l) for l in range(L)]
    xd = model.quantize_input(xf)  # features -> int8 codes, resident in HBM before the timed region
    del xf
    T, B, _ = xd.shape
    y = torch.empty((T, B, quants[-1]["H"]), dtype=torch.int8, device="cuda")
    ws = torch.empty(model.workspace_bytes(T, B), dtype=torch.uint8, device="cuda")

    def step():
        model.forward(xd, y=y, workspace=ws)

    if args.phase_timing:
        # phases of the kernel with groups of 32 rows: 0 h tile -> LDS (and W x terms), 1 R h (MFMA), 2 gate sums,
        # 3 publish statistics, 4 wait for them and (mean, sigma), 5 layer norm, sigma/tanh, cell, 6 hidden state,
        # 7 barrier, 8 projection, 9 barrier; 10 = everything before the first step, per launch
        model.set_option("stack", 0)
        step()
        torch.cuda.synchronize()
        model.set_option("phase_timing", 1)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ticks = model.phase_ticks()  # 100 MHz ticks summed over steps, layers and calls
        n = args.steps * T * L
        print(json.dumps({"phase_us_per_step": [round(t / 100.0 / n, 3) for t in ticks[:10]],
                          "step_us": round(sum(ticks[:10]) / 100.0 / n, 3),
                          "prologue_us_per_launch": round(ticks[10] / 100.0 / (args.steps * L), 2),
                          "device_status": model.device_status(), "sparse_layers": model.sparse_layers(),
                          "note": "timers of workgroup 0 only; they cost about 0.3 us per step themselves"}))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if model.device_status() != 0:  # a bounded wait gave up or a group was misplaced: the kernels left early
        sys.exit(f"bench.py: device status {model.device_status()} after the timed loop; the timing is void")
    ms_per_step = dt / args.steps * 1e3
    cell_steps = B * T * L
    value = cell_steps * args.steps / dt

    # per-kernel device time over the same K steps, HIP events on the launch stream
    model.profile_begin()
    for _ in range(args.steps):
        step()
    prof = model.profile_end()
    if model.device_status() != 0:
        sys.exit(f"bench.py: device status {model.device_status()} after the profiled loop; the timing is void")
    persistent = prof["cell"]["launches"] == 0  # the per-step path launches a cell kernel per step
    stacked = persistent and prof["input_gemm"]["launches"] == 0  # all layers in one launch, W x computed per step
    work = {}
    for q in quants:
        for k, v in algorithmic_work(q, B, T, persistent).items():
            e = work.setdefault(k, {"ops": 0.0, "bytes": 0.0, "bytes_resident": 0.0, "launches": 0})
            for f in e:
                e[f] += v.get(f, v["bytes"] if f == "bytes_resident" else 0)
    if stacked:
        # the one kernel does the input GEMM's work too: its ops, its weights once per step, and x; no W x terms
        # go through memory (the 2 B G N bytes per step that the recurrent figure counts for reading them stay in,
        # as the price of comparing both ways against the same figure)
        wi = work.pop("input_gemm")
        work["recurrent"]["ops"] += wi["ops"]
        work["recurrent"]["bytes"] += sum(q["G"] * q["N"] * q["I"] * T + T * B * q["I"] for q in quants)
        work["recurrent"]["bytes_resident"] += sum(T * B * q["I"] for q in quants)
    kernels = {}
    for k, w in work.items():
        p = prof[k]
        if not p["launches"]:
            continue
        per_step_ms = p["total_ms"] / args.steps
        kernels[k] = {"launches_per_step": p["launches"] // args.steps, "avg_us": p["total_ms"] / p["launches"] * 1e3,
                      "ms_per_step": per_step_ms,
                      "gbps": w["bytes"] / (per_step_ms * 1e-3) / 1e9,
                      "tops": w["ops"] / (per_step_ms * 1e-3) / 1e12}
        if k == "recurrent" and persistent:
            # the same launches against the bytes of the variant that keeps the weights on chip
            kernels[k]["gbps_weights_resident"] = w["bytes_resident"] / (per_step_ms * 1e-3) / 1e9
            kernels[k]["frac_hbm_weights_resident"] = kernels[k]["gbps_weights_resident"] / PEAK_HBM_GBS
        if k == "input_gemm":
            # the shape sits near the machine balance (peak ops / peak bytes): both bounds are reported
            kernels[k]["frac_mfma"] = kernels[k]["tops"] / PEAK_INT8_TOPS
            kernels[k]["frac_hbm"] = kernels[k]["gbps"] / PEAK_HBM_GBS
            kernels[k]["ops_per_byte"] = w["ops"] / w["bytes"]
            kernels[k]["machine_balance_ops_per_byte"] = PEAK_INT8_TOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    d = kernels[dominant]
    if dominant == "input_gemm":
        roof = {"bound": "mfma", "achieved": d["tops"], "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": d["tops"] / PEAK_INT8_TOPS}
    else:
        roof = {"bound": "hbm", "achieved": d["gbps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": d["gbps"] / PEAK_HBM_GBS}
    roof.update({"kernel": dominant, "avg_launch_us": d["avg_us"], "traffic": None,
                 "path": "stacked" if stacked else ("persistent" if persistent else "per-step"), "kernels": kernels})
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and not (args.batch or args.seq_len or stacked):  # HBM bytes per launch from rocprofv3 --pmc runs (see profiles/)
        rec = json.load(open(tpath)).get(args.config, {}).get(dominant)
        if rec:
            roof["traffic"] = rec["bytes_per_launch"]

    out = {
        "metric": "lstm_cell_steps_per_sec", "value": value, "unit": "cell-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": wl.describe(args.config) + (f" shrunk to B={B} T={T}" if (args.batch or args.seq_len) else "") +
                               (f" weights pruned 2:4 ({model.sparse_layers()} of {L} layers on the sparse MFMA)" if args.sparse else ""),
                   "cell_steps_per_step": cell_steps,
                   "batch": B, "seq_len": T, "layers": L,
                   "options": "library defaults (plain launch of the recurrent kernel)"},
        "roofline": roof,
    }

    ok = True
    if not args.no_cpu_baseline:
        # the oracle as it stands, on a bounded sample of the same workload: batch rows spread evenly
        # over the batch (so every group of rows of the recurrent kernel is sampled), the first steps,
        # all layers; one row per host thread at a time.  Its output also checks the GPU's.
        import oracle

        xq = xd.cpu().numpy()
        cores = min(oracle.max_threads(), 16, B)
        om = oracle.prepare(layers)
        probe_T = min(T, 4)
        t0 = time.perf_counter()
        oracle.forward(om, np.ascontiguousarray(xq[:probe_T, :cores]), threads=cores)
        rate = cores * probe_T * L / (time.perf_counter() - t0)  # cell-steps/s of the probe
        # about 15 s of work: whole sequences of as many rows as that allows (multiples of the thread count)
        rows = int(max(cores, min(B, (15.0 * rate / (T * L)) // cores * cores)))
        Ts = T if rows * T * L <= 30.0 * rate else max(1, int(15.0 * rate / (rows * L)))
        sel = [(i * B) // rows for i in range(rows)]
        xs = np.ascontiguousarray(xq[:Ts, sel])
        t0 = time.perf_counter()
        yo = oracle.forward(om, xs, threads=cores)
        dto = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": rows * Ts * L / dto, "unit": "cell-steps/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"{rows} batch rows spread evenly over the batch x first {Ts} steps x "
                                         f"{L} layers of {args.config}, {dto:.1f} s"}
        # the output of the last timed call against the oracle's, element by element
        got = y[:Ts].cpu().numpy()[:, sel]
        ok = bool(got.shape == yo.shape and (got == yo).all())
        out["parity"] = {"rows": rows, "steps": Ts, "layers": L, "equal": ok,
                         "mismatches": int((got != yo).sum()) if got.shape == yo.shape else -1}
    print(json.dumps(out), flush=True)
    # release device objects in order before the interpreter tears down
    del xd, y, ws
    model.destroy()
    torch.cuda.synchronize()
    if not ok:
        sys.exit("bench.py: the GPU output differs from the oracle on the sampled rows")


if __name__ == "__main__":
    main()
