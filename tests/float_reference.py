"""TEST INFRASTRUCTURE: a second float LSTM, independent of the library and of the
oracle, used by the CPU tests to fill in calibration statistics and to pin the
oracle's own float LSTM (which in turn checks lstm_int_calibrate on the GPU).

Runs the float LSTM of Sec. 2 (eqs. 1-7) of arXiv 2101.05453 in plain PyTorch
float64 on the CPU over representative inputs and records, at the paper's
"log" nodes (Sec. 4, post-training), min/max of x, h and m, max |c|, and
max |gate sum| per gate when layer norm is on.
"""
import numpy as np
import torch

CIFG, PEEPHOLE, LAYER_NORM, PROJECTION = 1, 2, 4, 8


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)


def _layernorm(v, Lw, b):
    mean = v.mean(dim=1, keepdim=True)
    var = ((v - mean) ** 2).mean(dim=1, keepdim=True)
    sd = var.sqrt()
    xn = torch.where(sd > 0, (v - mean) / torch.where(sd > 0, sd, torch.ones_like(sd)),
                     torch.zeros_like(v))
    return xn * Lw + b


def collect_statistics(layers, x, max_rows=16):
    """Fills x_min..g_absmax of every layer spec in place from a float run over
    the first min(B, max_rows) batch rows of x [T,B,I0]; returns the list of
    per-layer statistics as dicts."""
    x = np.asarray(x, dtype=np.float32)[:, :max_rows]
    T, B, _ = x.shape
    inp = _t(x)
    all_stats = []
    for spec in layers:
        fl = spec.flags
        cifg, ph, ln, proj = bool(fl & CIFG), bool(fl & PEEPHOLE), bool(fl & LAYER_NORM), bool(fl & PROJECTION)
        N, H = spec.num_cells, spec.output_size
        first = 1 if cifg else 0
        W = [None if w is None else _t(w) for w in spec.W]
        R = [None if w is None else _t(w) for w in spec.R]
        bias = [None if w is None else _t(w) for w in spec.b]
        P = [None if w is None else _t(w) for w in spec.P]
        Lw = [None if w is None else _t(w) for w in spec.Lw]
        Wp = None if spec.Wproj is None else _t(spec.Wproj)
        bp = None if spec.bproj is None else _t(spec.bproj)
        # W x for all steps at once
        wx = [None if W[g] is None else inp.reshape(T * B, -1) @ W[g].T for g in range(4)]
        h = torch.zeros(B, H, dtype=torch.float64)
        c = torch.zeros(B, N, dtype=torch.float64)
        out = torch.empty(T, B, H, dtype=torch.float64)
        st = {"x_min": float(inp.min()), "x_max": float(inp.max()), "h_min": np.inf, "h_max": -np.inf,
              "m_min": np.inf, "m_max": -np.inf, "c_absmax": 0.0, "g_absmax": [0.0] * 4}

        def gate(g, t, cell):
            pre = wx[g][t * B:(t + 1) * B] + h @ R[g].T
            if ph and g != 2:
                pre = pre + P[2 if g == 3 else g] * cell
            if ln:
                st["g_absmax"][g] = max(st["g_absmax"][g], float(pre.abs().max()))
                pre = _layernorm(pre, Lw[g], bias[g])
            else:
                pre = pre + bias[g]
            return torch.tanh(pre) if g == 2 else torch.sigmoid(pre)

        for t in range(T):
            f = gate(1, t, c)
            z = gate(2, t, c)
            i = 1.0 - f if cifg else gate(0, t, c)
            c = i * z + f * c
            o = gate(3, t, c)
            m = o * torch.tanh(c)
            h = m @ Wp.T + (bp if bp is not None else 0.0) if proj else m
            out[t] = h
            st["c_absmax"] = max(st["c_absmax"], float(c.abs().max()))
            st["m_min"], st["m_max"] = min(st["m_min"], float(m.min())), max(st["m_max"], float(m.max()))
            st["h_min"], st["h_max"] = min(st["h_min"], float(h.min())), max(st["h_max"], float(h.max()))
        spec.x_min, spec.x_max = st["x_min"], st["x_max"]
        spec.h_min, spec.h_max, spec.m_min, spec.m_max = st["h_min"], st["h_max"], st["m_min"], st["m_max"]
        spec.c_absmax = st["c_absmax"]
        spec.g_absmax = list(st["g_absmax"])
        all_stats.append(st)
        inp = out
    return all_stats
