"""Seeded synthetic LSTM workloads: float parameters and float inputs only.

This module serves both the HIP library's harness and the CPU oracle's tests.
It holds no arithmetic of the method (no quantization, no LSTM evaluation):
it only draws random float tensors of the shapes and distributions of the
five benchmark configurations, which stand in for the private RNN-T speech
models of the paper's Sec. 5 (10 LSTM layers of 2048 units, 8 of them in the
encoder); only the shapes are taken from there.

Recipe (numpy.random.Generator(PCG64)), fixed order:
  layer l draws from PCG64(seed + l):  W_i, W_f, W_z, W_o, R_i..R_o, b_i..b_o,
  P_i, P_f, P_o (peephole only), L_i..L_o (layer norm only), W_proj, b_proj
  (projection only); every tensor that CIFG removes (W_i, R_i, b_i, P_i, L_i)
  is not drawn at all.  The input x draws from PCG64(seed + 100003).
  Everything is float32; N(0, s) means standard deviation s.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

# variant switches (the same bit values as the C ABI's LSTM_INT_* flags)
CIFG = 1
PEEPHOLE = 2
LAYER_NORM = 4
PROJECTION = 8

GATES = ("i", "f", "z", "o")


@dataclass
class LayerSpec:
    """Float parameters of one LSTM layer (Sec. 2, eqs. 1-7) plus the
    statistics a calibration run fills in (Sec. 4)."""

    input_size: int
    num_cells: int
    output_size: int
    flags: int
    W: List[Optional[np.ndarray]] = field(default_factory=lambda: [None] * 4)  # [N, I]
    R: List[Optional[np.ndarray]] = field(default_factory=lambda: [None] * 4)  # [N, H]
    b: List[Optional[np.ndarray]] = field(default_factory=lambda: [None] * 4)  # [N]
    P: List[Optional[np.ndarray]] = field(default_factory=lambda: [None] * 3)  # [N] i,f,o
    Lw: List[Optional[np.ndarray]] = field(default_factory=lambda: [None] * 4)  # [N]
    Wproj: Optional[np.ndarray] = None  # [H, N]
    bproj: Optional[np.ndarray] = None  # [H]
    # calibration statistics (min/max of x, h, m; max|c|; max|gate sum| per gate)
    x_min: float = 0.0
    x_max: float = 0.0
    h_min: float = 0.0
    h_max: float = 0.0
    m_min: float = 0.0
    m_max: float = 0.0
    c_absmax: float = 0.0
    g_absmax: List[float] = field(default_factory=lambda: [0.0] * 4)


@dataclass
class Config:
    name: str
    layer_inputs: List[int]  # input width of each layer
    num_cells: int
    output_size: int
    flags: int
    batch: int
    steps: int
    weight_dist: str  # "uniform" or "normal"
    weight_param: float  # half-width or standard deviation
    input_dist: str  # "normal" or "uniform"
    input_param: float
    seed: int = 0


# The five configurations named by the benchmark definition.
CONFIGS = {
    "C1": Config("C1", [32], 64, 64, 0, 1, 20, "uniform", 0.1, "normal", 1.0),
    "C2": Config("C2", [256], 512, 512, LAYER_NORM, 16, 100, "normal", 0.05, "normal", 1.0),
    "C3": Config("C3", [640], 2048, 640, LAYER_NORM | PEEPHOLE | PROJECTION, 128, 200,
                 "normal", 0.03, "normal", 1.0),
    "C4": Config("C4", [512] + [640] * 7, 2048, 640, LAYER_NORM | PROJECTION, 256, 64,
                 "normal", 0.03, "normal", 1.0),
    "C5": Config("C5", [1024, 1024], 1024, 1024, CIFG | LAYER_NORM, 1024, 32,
                 "normal", 0.04, "uniform", 3.0),
}


def _draw(rng, dist, param, shape):
    if dist == "uniform":
        return rng.uniform(-param, param, size=shape).astype(np.float32)
    if dist == "normal":
        return (rng.standard_normal(size=shape) * param).astype(np.float32)
    raise ValueError(dist)


def make_layer(rng, input_size, num_cells, output_size, flags, weight_dist, weight_param):
    N, I, H = num_cells, input_size, output_size
    first = 1 if flags & CIFG else 0
    spec = LayerSpec(I, N, H, flags)
    for g in range(first, 4):
        spec.W[g] = _draw(rng, weight_dist, weight_param, (N, I))
    for g in range(first, 4):
        spec.R[g] = _draw(rng, weight_dist, weight_param, (N, H))
    for g in range(first, 4):
        spec.b[g] = _draw(rng, "uniform", 0.1, (N,))
    if flags & PEEPHOLE:
        for j in range(first, 3):
            spec.P[j] = _draw(rng, "uniform", 0.1, (N,))
    if flags & LAYER_NORM:
        for g in range(first, 4):
            spec.Lw[g] = rng.uniform(0.5, 1.5, size=(N,)).astype(np.float32)
    if flags & PROJECTION:
        spec.Wproj = _draw(rng, weight_dist, weight_param, (H, N))
        spec.bproj = _draw(rng, "uniform", 0.1, (H,))
    return spec


def make_custom(layer_inputs, num_cells, output_size, flags, batch, steps, seed=0,
                weight_dist="normal", weight_param=0.05, input_dist="normal",
                input_param=1.0):
    """Float layers and the float input x [T, B, I0] for an arbitrary shape."""
    if not (flags & PROJECTION):
        output_size = num_cells
    layers = []
    for l, I in enumerate(layer_inputs):
        rng = np.random.Generator(np.random.PCG64(seed + l))
        layers.append(make_layer(rng, I, num_cells, output_size, flags, weight_dist, weight_param))
    rng = np.random.Generator(np.random.PCG64(seed + 100003))
    x = _draw(rng, input_dist, input_param, (steps, batch, layer_inputs[0]))
    return layers, x


def make_workload(name, batch=None, steps=None, seed=None, num_layers=None):
    """One of C1..C5, optionally with fewer batch rows / steps / layers.

    Reducing the batch keeps the first rows of the full workload's x (the
    tensor is always drawn at full size), so a row subset of the full problem
    is itself a valid smaller problem with identical rows."""
    cfg = CONFIGS[name]
    seed = cfg.seed if seed is None else seed
    inputs = cfg.layer_inputs if num_layers is None else cfg.layer_inputs[:num_layers]
    layers = []
    for l, I in enumerate(inputs):
        rng = np.random.Generator(np.random.PCG64(seed + l))
        layers.append(make_layer(rng, I, cfg.num_cells, cfg.output_size, cfg.flags,
                                 cfg.weight_dist, cfg.weight_param))
    rng = np.random.Generator(np.random.PCG64(seed + 100003))
    x = _draw(rng, cfg.input_dist, cfg.input_param, (cfg.steps, cfg.batch, inputs[0]))
    T = cfg.steps if steps is None else steps
    B = cfg.batch if batch is None else batch
    if T > cfg.steps or B > cfg.batch:
        raise ValueError("steps/batch may only shrink the configuration")
    return layers, np.ascontiguousarray(x[:T, :B])


def prune_2of4(layers, tensors=("R",)):
    """Stand-in for the pruned models of the paper's Table 1 (50 % sparse LSTM and
    CIFG) in structured form: in every aligned group of four consecutive inputs of
    every row of the named weight tensors ("W", "R", "Wproj") the two entries of
    smallest magnitude are set to 0.0 (ties: the lower index goes first).  In place;
    returns layers.  Pure input structure: no arithmetic of the method."""
    def prune(w):
        rows, K = w.shape
        full = (K // 4) * 4
        if full:
            g = w[:, :full].reshape(rows, full // 4, 4)
            order = np.argsort(np.abs(g), axis=2, kind="stable")
            np.put_along_axis(g, order[:, :, :2], np.float32(0.0), axis=2)
            w[:, :full] = g.reshape(rows, full)
        rest = K - full  # a last group of fewer than four inputs keeps at most two
        if rest == 3:
            k = full + np.argmin(np.abs(w[:, full:]), axis=1)
            w[np.arange(rows), k] = 0.0

    for spec in layers:
        for name in tensors:
            if name == "Wproj":
                if spec.Wproj is not None:
                    prune(spec.Wproj)
            else:
                for m in getattr(spec, name):
                    if m is not None:
                        prune(m)
    return layers


@dataclass
class GruLayerSpec:
    """Float parameters of one GRU layer (gate order r, u, n; reset gate applied to the recurrent
    product) and the range of its input."""

    input_size: int
    num_cells: int
    W: List[np.ndarray] = field(default_factory=list)   # 3 x [N, I]
    R: List[np.ndarray] = field(default_factory=list)   # 3 x [N, N]
    bx: List[np.ndarray] = field(default_factory=list)  # 3 x [N]
    bh: List[np.ndarray] = field(default_factory=list)  # 3 x [N]
    x_min: float = 0.0
    x_max: float = 0.0


def make_gru(layer_inputs, num_cells, batch, steps, seed=0, weight_dist="normal", weight_param=0.05,
             input_dist="normal", input_param=1.0):
    """Float GRU layers and the float input x [T, B, I0].  Layer l draws from PCG64(seed + l) in the
    order W_r, W_u, W_n, R_r, R_u, R_n, bx_r..bx_n, bh_r..bh_n (biases U(-0.1, 0.1)); x from
    PCG64(seed + 100003).  The input range of layer 0 is the range of x."""
    layers = []
    for l, I in enumerate(layer_inputs):
        rng = np.random.Generator(np.random.PCG64(seed + l))
        spec = GruLayerSpec(I, num_cells)
        spec.W = [_draw(rng, weight_dist, weight_param, (num_cells, I)) for _ in range(3)]
        spec.R = [_draw(rng, weight_dist, weight_param, (num_cells, num_cells)) for _ in range(3)]
        spec.bx = [_draw(rng, "uniform", 0.1, (num_cells,)) for _ in range(3)]
        spec.bh = [_draw(rng, "uniform", 0.1, (num_cells,)) for _ in range(3)]
        layers.append(spec)
    rng = np.random.Generator(np.random.PCG64(seed + 100003))
    x = _draw(rng, input_dist, input_param, (steps, batch, layer_inputs[0]))
    layers[0].x_min, layers[0].x_max = float(x.min()), float(x.max())
    return layers, x


@dataclass
class SruLayerSpec:
    """Float parameters of one SRU layer (matmul slots c, f, r, s; W[3] is None when the input itself is
    the highway term, which needs input_size = num_cells) and the statistics its quantization needs."""

    input_size: int
    num_cells: int
    W: List[Optional[np.ndarray]] = field(default_factory=list)  # 4 x [N, I], the last may be None
    v: List[np.ndarray] = field(default_factory=list)  # 2 x [N]: v_f, v_r
    b: List[np.ndarray] = field(default_factory=list)  # 2 x [N]: b_f, b_r
    x_min: float = 0.0
    x_max: float = 0.0
    c_absmax: float = 0.0  # largest |c|, |W_c x|, |highway term|
    h_min: float = 0.0
    h_max: float = 0.0


def make_sru(layer_inputs, num_cells, batch, steps, seed=0, weight_dist="normal", weight_param=0.05,
             input_dist="normal", input_param=1.0, highway_matrix=None):
    """Float SRU layers and the float input x [T, B, I0].  Layer l draws from PCG64(seed + l) in the
    order W_c, W_f, W_r, (W_s,) v_f, v_r (U(-1, 1)), b_f, b_r (U(-0.5, 0.5)); x from
    PCG64(seed + 100003).  A layer has W_s when its input size differs from num_cells, or always /
    never with highway_matrix = True / False.  Only the input range of layer 0 is set here: the other
    statistics come from a float run (Sec. 4)."""
    layers = []
    for l, I in enumerate(layer_inputs):
        rng = np.random.Generator(np.random.PCG64(seed + l))
        spec = SruLayerSpec(I, num_cells)
        with_s = (I != num_cells) if highway_matrix is None else highway_matrix
        spec.W = [_draw(rng, weight_dist, weight_param, (num_cells, I)) for _ in range(4 if with_s else 3)]
        if not with_s:
            spec.W.append(None)
        spec.v = [_draw(rng, "uniform", 1.0, (num_cells,)) for _ in range(2)]
        spec.b = [_draw(rng, "uniform", 0.5, (num_cells,)) for _ in range(2)]
        layers.append(spec)
    rng = np.random.Generator(np.random.PCG64(seed + 100003))
    x = _draw(rng, input_dist, input_param, (steps, batch, layer_inputs[0]))
    layers[0].x_min, layers[0].x_max = float(x.min()), float(x.max())
    return layers, x


def describe(name):
    cfg = CONFIGS[name]
    v = [n for bit, n in ((CIFG, "cifg"), (PEEPHOLE, "peephole"), (LAYER_NORM, "layernorm"),
                          (PROJECTION, "projection")) if cfg.flags & bit]
    return (f"{name}: L={len(cfg.layer_inputs)} I={cfg.layer_inputs[0]} N={cfg.num_cells} "
            f"H={cfg.output_size} B={cfg.batch} T={cfg.steps} [{'+'.join(v) or 'basic'}]")
