// Integer-only GRU (include/gru_int.h): the recipe assembled from the building
// blocks of arXiv 2101.05453 (Sec. 7 names the GRU; Secs. 3.2.1, 3.2.2, 3.2.4,
// 3.2.7, 3.2.9 and Sec. 6 supply the blocks), offline phase on the host and
// the online phase as HIP kernels for gfx950.
//
// Online phase per layer:
//   1. tx = sat16(rescale(W x + bx')) for all T*B rows: the library's int8
//      MFMA matmul (kernels.hip), gate-major columns [3N].
//   2. per step ONE kernel, gru_step_kernel: R h8 + bh for the three gates on
//      the 16x16x64 int8 MFMA, each wave a tile of 16 batch rows x 16 cells
//      over the whole depth, with the weights read in operand order (one
//      contiguous KB per wave load).  The MFMA leaves every lane with the
//      three gate accumulators of four cells of one batch row, so the whole
//      elementwise cell (rescale, sigma/tanh tables, reset product, coupled
//      update, the int8 form of the new state) runs in that lane with no
//      exchange of any kind.
// The state is read and written in place (each (row, cell) belongs to one
// lane); the int8 form of step t is read by step t + 1 from the layer's output
// buffer.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/gru_int.h"
#include "kernels.h"
#include "lstm_int_math.h"
#include "model.h"

namespace lstm_int {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr double kInt32MaxD = 2147483647.0;

struct GruLayerHost {
  int32_t I = 0, N = 0, zp_x = 0;
  double s_x = 0, s_W[3] = {0, 0, 0}, s_R[3] = {0, 0, 0};
  int32_t Mx[3] = {0, 0, 0}, ex[3] = {0, 0, 0}, Mh[3] = {0, 0, 0}, eh[3] = {0, 0, 0};
  std::vector<int8_t> Wq, Rq;
  std::vector<int32_t> bxq, bhq, bx_fold;
};

// padded extents of one layer on the device
struct GruDims {
  int Ip, Kp, Ncp, cols_pad;  // input depth / state depth (multiples of 64), cells (multiple of 16), 3N to 128
};
GruDims gru_dims(int I, int N) {
  return GruDims{(I + 63) / 64 * 64, (N + 63) / 64 * 64, (N + 15) / 16 * 16, (3 * N + 127) / 128 * 128};
}

struct GruLayerDev {
  const int8_t *W = nullptr;      // [cols_pad][Ip] gate-major rows, zero beyond the real extents
  const int32_t *bx = nullptr;    // [cols_pad] folded input bias
  const int8_t *Rop = nullptr;    // [Ncp/16][3][Kp/64][64 lanes][16 B]: operand order of the 16x16x64 MFMA
  const int32_t *bh = nullptr;    // [3][Ncp]
};

bool finite_all(const float *a, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!std::isfinite(a[i])) return false;
  return true;
}

// symmetric int8, +-127; scale max|w| / 127 (1 for an all-zero tensor); floor(v / s + 1/2)
double quantize_tensor(const float *src, size_t n, int8_t *dst) {
  double amax = 0.0;
  for (size_t i = 0; i < n; ++i) amax = std::fmax(amax, std::fabs((double)src[i]));
  const double s = amax == 0.0 ? 1.0 : amax / 127.0;
  for (size_t i = 0; i < n; ++i) {
    double r = std::floor((double)src[i] / s + 0.5);
    dst[i] = (int8_t)std::fmin(std::fmax(r, -127.0), 127.0);
  }
  return s;
}

int32_t quantize_bias32(double v, double s) {
  double r = std::floor(v / s + 0.5);
  return (int32_t)std::fmin(std::fmax(r, -kInt32MaxD), kInt32MaxD);
}

int prepare_gru_layer(const gru_int_layer_params &p, bool has_prev, GruLayerHost &q) {
  const int I = p.input_size, N = p.num_cells;
  if (I < 1 || N < 1) return LSTM_INT_E_INVALID_ARG;
  if (I > 32768 || N > 32768) return LSTM_INT_E_UNSUPPORTED;  // accumulation depth, Sec. 3.1.1
  for (int g = 0; g < 3; ++g)
    if (!p.W[g] || !p.R[g] || !p.bx[g] || !p.bh[g]) return LSTM_INT_E_INVALID_ARG;
  q.I = I;
  q.N = N;
  if (has_prev) {  // the int8 form of the state below: scale 2^-7, zero point 0
    q.s_x = std::ldexp(1.0, -7);
    q.zp_x = 0;
  } else {  // asymmetric int8, range widened to 0, nudged zero point (Sec. 3.2.4)
    double lo = p.x_min, hi = p.x_max;
    if (!std::isfinite(lo) || !std::isfinite(hi) || lo > hi) return LSTM_INT_E_BAD_RANGE;
    lo = std::fmin(lo, 0.0);
    hi = std::fmax(hi, 0.0);
    double s = (hi - lo) / 255.0;
    if (s == 0.0) s = 1.0;
    const double z = std::floor(-128.0 - lo / s + 0.5);
    q.s_x = s;
    q.zp_x = (int32_t)std::fmin(std::fmax(z, -128.0), 127.0);
  }
  const double s_h8 = std::ldexp(1.0, -7);
  q.Wq.assign((size_t)3 * N * I, 0);
  q.Rq.assign((size_t)3 * N * N, 0);
  q.bxq.assign((size_t)3 * N, 0);
  q.bhq.assign((size_t)3 * N, 0);
  q.bx_fold.assign((size_t)3 * N, 0);
  for (int g = 0; g < 3; ++g) {
    if (!finite_all(p.W[g], (size_t)N * I) || !finite_all(p.R[g], (size_t)N * N) || !finite_all(p.bx[g], N) ||
        !finite_all(p.bh[g], N))
      return LSTM_INT_E_BAD_RANGE;
    q.s_W[g] = quantize_tensor(p.W[g], (size_t)N * I, q.Wq.data() + (size_t)g * N * I);
    q.s_R[g] = quantize_tensor(p.R[g], (size_t)N * N, q.Rq.data() + (size_t)g * N * N);
    for (int n = 0; n < N; ++n) {  // biases at the scale of their accumulators (Sec. 3.2.4)
      q.bxq[g * N + n] = quantize_bias32(p.bx[g][n], q.s_W[g] * q.s_x);
      q.bhq[g * N + n] = quantize_bias32(p.bh[g][n], q.s_R[g] * s_h8);
    }
    int rc;  // both matmul results go to Q3.12 (Sec. 3.2.4)
    if ((rc = quantize_multiplier(q.s_W[g] * q.s_x * 4096.0, &q.Mx[g], &q.ex[g])) != LSTM_INT_OK) return rc;
    if ((rc = quantize_multiplier(q.s_R[g] * s_h8 * 4096.0, &q.Mh[g], &q.eh[g])) != LSTM_INT_OK) return rc;
    for (int n = 0; n < N; ++n) {  // zero point folded (Sec. 6); accumulators safe for every int8 input
      const int8_t *w = q.Wq.data() + ((size_t)g * N + n) * I;
      int64_t sum = 0, sum_abs = 0;
      for (int k = 0; k < I; ++k) {
        sum += w[k];
        sum_abs += std::abs((int)w[k]);
      }
      const int64_t f = (int64_t)q.bxq[g * N + n] - (int64_t)q.zp_x * sum;
      if (std::llabs(f) + 128 * sum_abs > 2147483647LL) return LSTM_INT_E_UNSUPPORTED;
      q.bx_fold[g * N + n] = (int32_t)f;
      const int8_t *r = q.Rq.data() + ((size_t)g * N + n) * N;
      int64_t rabs = 0;
      for (int k = 0; k < N; ++k) rabs += std::abs((int)r[k]);
      if (std::llabs((int64_t)q.bhq[g * N + n]) + 128 * rabs > 2147483647LL) return LSTM_INT_E_UNSUPPORTED;
    }
  }
  return LSTM_INT_OK;
}

// ---------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------

// the int8 form of a state value: sat8(floor((h16 + 128) / 256))
__device__ __forceinline__ int32_t state_i8(int32_t h16) { return sat8((h16 + 128) >> 8); }

// Start of a layer: the working state (caller's h_state slice or zeros) is used in place; its int8 form
// goes to h8_0 [B][Kp] (pad bytes zero).
__global__ void gru_init_kernel(int16_t *h16, int B, int N, int Kp, int8_t *h8_0, int zero_state) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)B * Kp) return;
  const int b = (int)(i / Kp), k = (int)(i - (int64_t)b * Kp);
  int32_t v = 0;
  if (k < N) {
    if (zero_state)
      h16[(size_t)b * N + k] = 0;
    else
      v = state_i8(h16[(size_t)b * N + k]);
  }
  h8_0[i] = (int8_t)v;
}

struct GruStepArgs {
  int32_t B, N, Ncp, Kp, KS;  // KS = Kp / 64
  const int8_t *h8_prev;      // [B][Kp]
  const int8_t *Rop;
  const int32_t *bh;          // [3][Ncp]
  const int16_t *tx;          // [B][3N] of this step
  int16_t *h16;               // [B][N] in/out
  int8_t *h8_out;             // [B][Kp]
  int8_t *y;                  // [B][N] or NULL
  int32_t Mh[3], rh[3];
  const uint16_t *sig_tab, *tanh_tab;  // [32769] each, Q3.12 inputs
  int16_t *tr_tx, *tr_th, *tr_act, *tr_h16;  // [B][3][N] / [B][N] of this step, or NULL
  int8_t *tr_h8;
};

__global__ __launch_bounds__(256) void gru_step_kernel(GruStepArgs a) {
  const int lane = threadIdx.x & 63;
  const int wave_id = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int ctiles = a.Ncp >> 4;
  const int rt = wave_id / ctiles, ct = wave_id - rt * ctiles;
  if (rt * 16 >= a.B) return;  // uniform per wave; the kernel has no barrier
  const int rowl = lane & 15, q4 = lane >> 4;
  int brow = rt * 16 + rowl;
  const bool row_ok = brow < a.B;
  brow = row_ok ? brow : a.B - 1;  // rows past the batch repeat the last one; never stored

  // R h8 for the three gates: acc[g][v] = sum_k R_g[16 ct + 4 q4 + v][k] h8[brow][k]
  v4i acc[3] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}};
  const int8_t *hp = a.h8_prev + (size_t)brow * a.Kp + (q4 << 4);
  const v4i *wp = reinterpret_cast<const v4i *>(a.Rop) + ((size_t)ct * 3 * a.KS) * 64 + lane;
  const int KS = a.KS;
  constexpr int U = 4;  // k steps whose loads are issued together
  int ks = 0;
  for (; ks + U <= KS; ks += U) {
    v4i hf[U], wf[U][3];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      hf[u] = *reinterpret_cast<const v4i *>(hp + (size_t)(ks + u) * 64);
#pragma unroll
      for (int g = 0; g < 3; ++g) wf[u][g] = wp[((size_t)g * KS + ks + u) * 64];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int g = 0; g < 3; ++g) acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[u][g], hf[u], acc[g], 0, 0, 0);
  }
  for (; ks < KS; ++ks) {
    const v4i hf = *reinterpret_cast<const v4i *>(hp + (size_t)ks * 64);
#pragma unroll
    for (int g = 0; g < 3; ++g) acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wp[((size_t)g * KS + ks) * 64], hf, acc[g], 0, 0, 0);
  }

  // the cell, four cells of one batch row per lane
  const int n0 = ct * 16 + q4 * 4;
  const int N = a.N;
  const size_t row3 = (size_t)brow * 3 * N;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int n = n0 + v;
    if (n >= N || !row_ok) continue;
    int32_t tx[3], th[3];
#pragma unroll
    for (int g = 0; g < 3; ++g) {
      tx[g] = a.tx[row3 + (size_t)g * N + n];
      th[g] = sat16(rescale(acc[g][v] + a.bh[g * a.Ncp + n], a.Mh[g], a.rh[g]));
    }
    const int32_t r = sigmoid_from_table(a.sig_tab, sat16(tx[0] + th[0]));  // Sec. 3.2.1
    const int32_t u = sigmoid_from_table(a.sig_tab, sat16(tx[1] + th[1]));
    const int32_t rn = (r * th[2] + 16384) >> 15;  // Q0.15 x Q3.12 -> Q3.12; |r th| < 2^30
    const int32_t c = tanh_from_table(a.tanh_tab, sat16(tx[2] + rn));
    const int32_t ubar = cifg_input_gate(u);  // 1 - u, Sec. 3.2.9
    const int32_t hold = a.h16[(size_t)brow * N + n];
    const int32_t hn = cell_update32(ubar, c, u, hold, 0);  // Sec. 3.2.7 with both products Q0.30 -> Q0.15
    const int32_t h8 = state_i8(hn);
    a.h16[(size_t)brow * N + n] = (int16_t)hn;
    a.h8_out[(size_t)brow * a.Kp + n] = (int8_t)h8;
    if (a.y) a.y[(size_t)brow * N + n] = (int8_t)h8;
    if (a.tr_tx)
      for (int g = 0; g < 3; ++g) a.tr_tx[row3 + (size_t)g * N + n] = (int16_t)tx[g];
    if (a.tr_th)
      for (int g = 0; g < 3; ++g) a.tr_th[row3 + (size_t)g * N + n] = (int16_t)th[g];
    if (a.tr_act) {
      a.tr_act[row3 + n] = (int16_t)r;
      a.tr_act[row3 + (size_t)N + n] = (int16_t)u;
      a.tr_act[row3 + (size_t)2 * N + n] = (int16_t)c;
    }
    if (a.tr_h16) a.tr_h16[(size_t)brow * N + n] = (int16_t)hn;
    if (a.tr_h8) a.tr_h8[(size_t)brow * N + n] = (int8_t)h8;
  }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

}  // namespace lstm_int

using namespace lstm_int;

struct gru_int_model {
  int device = -1;
  std::vector<GruLayerHost> host;
  std::vector<GruLayerDev> dev;
  uint8_t *arena = nullptr;
  const uint16_t *sig_tab = nullptr, *tanh_tab = nullptr;
};

namespace {

// carve-up of the workspace for (T, B)
struct GruWs {
  size_t xpad, tx, out[2], h8_0, h16, total;
};
GruWs gru_workspace(const gru_int_model *m, int64_t T, int64_t B) {
  GruWs w{};
  size_t off = 0, max_tx = 0, max_out = 0, max_h0 = 0, sum_h16 = 0;
  for (const GruLayerHost &q : m->host) {
    const GruDims d = gru_dims(q.I, q.N);
    max_tx = std::max(max_tx, (size_t)T * B * 3 * q.N * 2);
    max_out = std::max(max_out, (size_t)T * B * d.Kp);
    max_h0 = std::max(max_h0, (size_t)B * d.Kp);
    sum_h16 = std::max(sum_h16, (size_t)B * q.N * 2);
  }
  const GruDims d0 = gru_dims(m->host[0].I, m->host[0].N);
  w.xpad = off; off += align256((size_t)T * B * d0.Ip);
  w.tx = off; off += align256(max_tx);
  w.out[0] = off; off += align256(max_out);
  w.out[1] = off; off += align256(max_out);
  w.h8_0 = off; off += align256(max_h0);
  w.h16 = off; off += align256(sum_h16);
  w.total = off;
  return w;
}

}  // namespace

extern "C" {

int gru_int_prepare(const gru_int_layer_params *layers, int32_t num_layers, int32_t device, gru_int_model **out) {
  if (!layers || !out || num_layers < 1) return LSTM_INT_E_INVALID_ARG;
  *out = nullptr;
  gru_int_model *m = new (std::nothrow) gru_int_model();
  if (!m) return LSTM_INT_E_OUT_OF_MEMORY;
  try {
    m->host.resize(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      if (l > 0 && layers[l].input_size != layers[l - 1].num_cells) {
        delete m;
        return LSTM_INT_E_INVALID_ARG;
      }
      const int rc = prepare_gru_layer(layers[l], l > 0, m->host[l]);
      if (rc != LSTM_INT_OK) {
        delete m;
        return rc;
      }
    }
    m->device = device;
    if (device < 0) {
      *out = m;
      return LSTM_INT_OK;
    }
    // device image: the two Q3.12 tables, then per layer W, bx, R in operand order, bh
    constexpr size_t kTab = 32769;
    std::vector<uint8_t> img;
    auto reserve = [&](size_t bytes) {
      const size_t off = align256(img.size());
      img.resize(off + bytes, 0);
      return off;
    };
    const size_t o_sig = reserve(kTab * 2), o_tanh = reserve(kTab * 2);
    fill_sigmoid_table(3, reinterpret_cast<uint16_t *>(img.data() + o_sig));
    fill_tanh_table(3, reinterpret_cast<uint16_t *>(img.data() + o_tanh));
    struct Off { size_t W, bx, R, bh; };
    std::vector<Off> offs(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      const GruLayerHost &q = m->host[l];
      const int I = q.I, N = q.N;
      const GruDims d = gru_dims(I, N);
      const int KS = d.Kp / 64;
      Off o;
      o.W = reserve((size_t)d.cols_pad * d.Ip);
      o.bx = reserve((size_t)d.cols_pad * 4);
      o.R = reserve((size_t)(d.Ncp / 16) * 3 * KS * 1024);
      o.bh = reserve((size_t)3 * d.Ncp * 4);
      for (int r = 0; r < 3 * N; ++r) std::memcpy(img.data() + o.W + (size_t)r * d.Ip, q.Wq.data() + (size_t)r * I, I);
      std::memcpy(img.data() + o.bx, q.bx_fold.data(), (size_t)3 * N * 4);
      // operand of lane (row = lane % 16, chunk = lane / 16) at k step ks: bytes 64 ks + 16 chunk .. + 15 of weight
      // row 16 ct + row of gate g (zero beyond N in either direction)
      for (int ct = 0; ct < d.Ncp / 16; ++ct)
        for (int g = 0; g < 3; ++g)
          for (int ks = 0; ks < KS; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
              const int n = ct * 16 + (lane & 15), k0 = ks * 64 + (lane >> 4) * 16;
              uint8_t *dst = img.data() + o.R + ((((size_t)ct * 3 + g) * KS + ks) * 64 + lane) * 16;
              if (n < N)
                for (int j = 0; j < 16 && k0 + j < N; ++j) dst[j] = (uint8_t)q.Rq[((size_t)g * N + n) * N + k0 + j];
            }
      for (int g = 0; g < 3; ++g)
        std::memcpy(img.data() + o.bh + (size_t)g * d.Ncp * 4, q.bhq.data() + (size_t)g * N, (size_t)N * 4);
      offs[l] = o;
    }
    if (hipSetDevice(device) != hipSuccess || hipMalloc(reinterpret_cast<void **>(&m->arena), img.size()) != hipSuccess) {
      m->arena = nullptr;
      delete m;
      return LSTM_INT_E_DEVICE;
    }
    if (hipMemcpy(m->arena, img.data(), img.size(), hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipFree(m->arena);
      delete m;
      return LSTM_INT_E_DEVICE;
    }
    m->sig_tab = reinterpret_cast<const uint16_t *>(m->arena + o_sig);
    m->tanh_tab = reinterpret_cast<const uint16_t *>(m->arena + o_tanh);
    m->dev.resize(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      m->dev[l].W = reinterpret_cast<const int8_t *>(m->arena + offs[l].W);
      m->dev[l].bx = reinterpret_cast<const int32_t *>(m->arena + offs[l].bx);
      m->dev[l].Rop = reinterpret_cast<const int8_t *>(m->arena + offs[l].R);
      m->dev[l].bh = reinterpret_cast<const int32_t *>(m->arena + offs[l].bh);
    }
  } catch (const std::bad_alloc &) {
    delete m;
    return LSTM_INT_E_OUT_OF_MEMORY;
  }
  *out = m;
  return LSTM_INT_OK;
}

int gru_int_get_quant(const gru_int_model *m, int32_t layer, gru_int_layer_quant *out) {
  if (!m || !out || layer < 0 || layer >= (int32_t)m->host.size()) return LSTM_INT_E_INVALID_ARG;
  const GruLayerHost &q = m->host[layer];
  out->I = q.I; out->N = q.N; out->zp_x = q.zp_x; out->s_x = q.s_x;
  for (int g = 0; g < 3; ++g) {
    out->s_W[g] = q.s_W[g]; out->s_R[g] = q.s_R[g];
    out->Mx[g] = q.Mx[g]; out->ex[g] = q.ex[g]; out->Mh[g] = q.Mh[g]; out->eh[g] = q.eh[g];
  }
  out->Wq = q.Wq.data(); out->Rq = q.Rq.data();
  out->bxq = q.bxq.data(); out->bhq = q.bhq.data(); out->bx_fold = q.bx_fold.data();
  return LSTM_INT_OK;
}

size_t gru_int_workspace_bytes(const gru_int_model *m, int32_t T, int32_t B) {
  if (!m || T < 0 || B < 0 || m->host.empty()) return 0;
  return gru_workspace(m, T, B).total;
}

int gru_int_forward(const gru_int_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y, int16_t *h_state,
                    void *workspace, size_t workspace_bytes, void *hip_stream, const gru_int_trace *trace) {
  if (!m || T < 0 || B < 0) return LSTM_INT_E_INVALID_ARG;
  if (T == 0 || B == 0) return LSTM_INT_OK;
  if (!x || !y) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  const int L = (int)m->host.size();
  if (trace && (trace->layer < 0 || trace->layer >= L)) return LSTM_INT_E_INVALID_ARG;
  int64_t widest = 0;
  for (const GruLayerHost &q : m->host) widest = std::max<int64_t>(widest, std::max(3 * (int64_t)q.N, (int64_t)gru_dims(q.I, q.N).Ip));
  if ((int64_t)T * B * widest >= ((int64_t)1 << 31)) return LSTM_INT_E_UNSUPPORTED;  // 32-bit row arithmetic of the matmul
  const GruWs w = gru_workspace(m, T, B);
  if (!workspace || workspace_bytes < w.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return LSTM_INT_E_WORKSPACE;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  uint8_t *ws = reinterpret_cast<uint8_t *>(workspace);
  const int64_t TB = (int64_t)T * B;

  const int8_t *in = x;
  int ld_in = m->host[0].I;
  {
    // the matmul reads rows of Ip bytes in 16-byte pieces: a padded copy unless x already has that shape
    const GruDims d0 = gru_dims(m->host[0].I, m->host[0].N);
    if (d0.Ip != m->host[0].I || (reinterpret_cast<uintptr_t>(x) & 15)) {
      int8_t *xp = reinterpret_cast<int8_t *>(ws + w.xpad);
      launch_copy_rows_i8(s, x, m->host[0].I, xp, d0.Ip, (int)TB, m->host[0].I, 0);
      in = xp;
      ld_in = d0.Ip;
    }
  }
  size_t h_off = 0;
  for (int l = 0; l < L; ++l) {
    const GruLayerHost &q = m->host[l];
    const GruLayerDev &dv = m->dev[l];
    const int N = q.N;
    const GruDims d = gru_dims(q.I, N);
    int16_t *tx = reinterpret_cast<int16_t *>(ws + w.tx);
    int8_t *out = reinterpret_cast<int8_t *>(ws + w.out[l & 1]);
    int8_t *h8_0 = reinterpret_cast<int8_t *>(ws + w.h8_0);
    int16_t *h16 = h_state ? h_state + h_off : reinterpret_cast<int16_t *>(ws + w.h16);
    const gru_int_trace *tr = (trace && trace->layer == l) ? trace : nullptr;

    Requant rq{};
    rq.all_hi = 1;
    for (int g = 0; g < 3; ++g) {
      rq.M[g] = q.Mx[g];
      rq.r[g] = 31 - q.ex[g];
      if (rq.r[g] < 33) rq.all_hi = 0;
    }
    rq.M[3] = rq.M[2];
    rq.r[3] = rq.r[2];
    rq.cols_per_gate = N;
    rq.zp = 0;
    launch_gemm_i16(s, in, ld_in, (int)TB, dv.W, d.Ip, 3 * N, dv.bx, rq, tx, 3 * N);

    {
      const int64_t n = (int64_t)B * d.Kp;
      hipLaunchKernelGGL(gru_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, h16, B, N, d.Kp, h8_0,
                         h_state ? 0 : 1);
    }
    GruStepArgs a{};
    a.B = B; a.N = N; a.Ncp = d.Ncp; a.Kp = d.Kp; a.KS = d.Kp / 64;
    a.Rop = dv.Rop; a.bh = dv.bh; a.h16 = h16;
    for (int g = 0; g < 3; ++g) {
      a.Mh[g] = q.Mh[g];
      a.rh[g] = 31 - q.eh[g];
    }
    a.sig_tab = m->sig_tab; a.tanh_tab = m->tanh_tab;
    const int waves = ((B + 15) / 16) * (d.Ncp / 16);
    const dim3 grid((unsigned)((waves + 3) / 4));
    for (int t = 0; t < T; ++t) {
      const size_t tb = (size_t)t * B;
      a.h8_prev = t == 0 ? h8_0 : out + (tb - B) * d.Kp;
      a.tx = tx + tb * 3 * N;
      a.h8_out = out + tb * d.Kp;
      a.y = l == L - 1 ? y + tb * N : nullptr;
      a.tr_tx = tr && tr->tx ? tr->tx + tb * 3 * N : nullptr;
      a.tr_th = tr && tr->th ? tr->th + tb * 3 * N : nullptr;
      a.tr_act = tr && tr->act ? tr->act + tb * 3 * N : nullptr;
      a.tr_h16 = tr && tr->h16 ? tr->h16 + tb * N : nullptr;
      a.tr_h8 = tr && tr->h8 ? tr->h8 + tb * N : nullptr;
      hipLaunchKernelGGL(gru_step_kernel, grid, dim3(256), 0, s, a);
    }
    in = out;
    ld_in = d.Kp;
    h_off += (size_t)B * N;
  }
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

void gru_int_destroy(gru_int_model *m) {
  if (!m) return;
  if (m->arena) {
    (void)hipSetDevice(m->device);
    (void)hipFree(m->arena);
  }
  delete m;
}

}  // extern "C"
