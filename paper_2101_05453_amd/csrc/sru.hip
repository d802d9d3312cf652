// Integer-only SRU (include/sru_int.h): the recipe assembled from the building
// blocks of arXiv 2101.05453 (Sec. 7 names the SRU; Secs. 3.2.1, 3.2.2, 3.2.3,
// 3.2.4, 3.2.7, 3.2.8, 3.2.9 and Sec. 6 supply the blocks), offline phase on the
// host and the online phase as HIP kernels for gfx950.
//
// Online phase per layer, two launches:
//   1. the matmul slots (candidate, forget, reset, highway) of all T*B rows as
//      one int8 MFMA matmul, each slot rescaled to its own int16 format: the
//      register-resident input GEMM of the LSTM path (in_gemm.hip, input depth
//      up to 1024, tile-ordered output) or the general matmul (kernels.hip,
//      row-major output);
//   2. sru_scan_kernel: the recurrence has no matmul, every (row, cell) is a
//      chain of its own through time.  A thread carries four neighbouring cells
//      of one batch row through all T steps with the state in registers; the
//      terms of the next kDepth steps are always in flight, so that the chain
//      waits for arithmetic only.  The kernel is bound by the bytes it streams:
//      four (three) int16 terms in and one int8 out per cell and step.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/sru_int.h"
#include "kernels.h"
#include "lstm_int_math.h"
#include "model.h"
#include "persistent.h"

namespace lstm_int {

namespace {

constexpr double kInt32MaxD = 2147483647.0;

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct SruLayerHost {
  int32_t I = 0, N = 0, G = 0, zp_x = 0, zp_h = 0, m_c = 0;
  double s_x = 0, s_h = 0, s_W[4] = {0, 0, 0, 0}, s_v[2] = {0, 0};
  int32_t Mx[4] = {0, 0, 0, 0}, ex[4] = {0, 0, 0, 0}, Mv[2] = {0, 0}, ev[2] = {0, 0};
  int32_t Ms = 0, es = 0, Mh = 0, eh = 0;
  std::vector<int8_t> Wq;
  std::vector<int16_t> vq;
  std::vector<int32_t> bq, b_fold;
};

// padded extents of one layer on the device
struct SruDims {
  int Ip, Kp, cols_pad;  // input depth and output row length (multiples of 64), G N to 128
};
SruDims sru_dims(int I, int N, int G) {
  return SruDims{(I + 63) / 64 * 64, (N + 63) / 64 * 64, (G * N + 127) / 128 * 128};
}

struct SruLayerDev {
  const int8_t *W = nullptr;     // [cols_pad][Ip] slot-major rows, zero beyond the real extents
  const int32_t *bias = nullptr; // [cols_pad] folded constants
  const int16_t *vq = nullptr;   // [2][N]
  // input depth up to 1024: W once more as the register-resident input GEMM reads it (in_gemm.hip): tiles of 8 cells
  // x 4 slots, row 8 slot + cell % 8, [tile][Ip/32][64 lanes][16 B]
  const int8_t *W2f = nullptr;
  const int32_t *b2 = nullptr;   // [tiles][32]
  int tiles = 0;                 // a multiple of 8 (cells padded to 64)
};

bool finite_all(const float *a, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!std::isfinite(a[i])) return false;
  return true;
}

// symmetric, +-qmax; scale max|w| / qmax (1 for an all-zero tensor); floor(v / s + 1/2)
template <typename T>
double quantize_symmetric(const float *src, size_t n, T *dst, double qmax) {
  double amax = 0.0;
  for (size_t i = 0; i < n; ++i) amax = std::fmax(amax, std::fabs((double)src[i]));
  const double s = amax == 0.0 ? 1.0 : amax / qmax;
  for (size_t i = 0; i < n; ++i) {
    const double r = std::floor((double)src[i] / s + 0.5);
    dst[i] = (T)std::fmin(std::fmax(r, -qmax), qmax);
  }
  return s;
}

// asymmetric int8 over [lo, hi] widened to contain 0, zero point nudged to an integer (Sec. 3.2.4)
int asymmetric8(double lo, double hi, double *s, int32_t *zp) {
  if (!std::isfinite(lo) || !std::isfinite(hi) || lo > hi) return LSTM_INT_E_BAD_RANGE;
  lo = std::fmin(lo, 0.0);
  hi = std::fmax(hi, 0.0);
  double sc = (hi - lo) / 255.0;
  if (sc == 0.0) sc = 1.0;
  *s = sc;
  *zp = (int32_t)std::fmin(std::fmax(std::floor(-128.0 - lo / sc + 0.5), -128.0), 127.0);
  return LSTM_INT_OK;
}

int prepare_sru_layer(const sru_int_layer_params &p, const SruLayerHost *prev, SruLayerHost &q) {
  const int I = p.input_size, N = p.num_cells;
  if (I < 1 || N < 1) return LSTM_INT_E_INVALID_ARG;
  if (I > 32768 || N > 32768) return LSTM_INT_E_UNSUPPORTED;  // accumulation depth, Sec. 3.1.1
  if (!p.W[0] || !p.W[1] || !p.W[2] || !p.v[0] || !p.v[1] || !p.b[0] || !p.b[1]) return LSTM_INT_E_INVALID_ARG;
  const int G = p.W[3] ? 4 : 3;
  if (G == 3 && I != N) return LSTM_INT_E_INVALID_ARG;  // the input itself is the highway term
  q.I = I;
  q.N = N;
  q.G = G;
  int rc;
  if (prev) {  // the output of the layer below
    q.s_x = prev->s_h;
    q.zp_x = prev->zp_h;
  } else if ((rc = asymmetric8(p.x_min, p.x_max, &q.s_x, &q.zp_x)) != LSTM_INT_OK) {
    return rc;
  }
  if ((rc = asymmetric8(p.h_min, p.h_max, &q.s_h, &q.zp_h)) != LSTM_INT_OK) return rc;
  // the state's format: the measured magnitude extended to a power of two (Sec. 3.2.2)
  const double ca = p.c_absmax;
  if (!std::isfinite(ca) || ca < 0.0) return LSTM_INT_E_BAD_RANGE;
  int mc = 0;
  while (mc <= 8 && std::ldexp(1.0, mc) < ca) ++mc;
  if (mc > 8) return LSTM_INT_E_UNSUPPORTED;
  q.m_c = mc;
  const double s_c = std::ldexp(1.0, mc - 15);

  q.Wq.assign((size_t)G * N * I, 0);
  q.vq.assign((size_t)2 * N, 0);
  q.bq.assign((size_t)G * N, 0);
  q.b_fold.assign((size_t)G * N, 0);
  for (int g = 0; g < G; ++g) {
    if (!finite_all(p.W[g], (size_t)N * I)) return LSTM_INT_E_BAD_RANGE;
    q.s_W[g] = quantize_symmetric(p.W[g], (size_t)N * I, q.Wq.data() + (size_t)g * N * I, 127.0);
    const bool gate = g == 1 || g == 2;
    if (gate) {  // biases at the scale of their accumulator (Sec. 3.2.4)
      const float *b = p.b[g - 1];
      if (!finite_all(b, N)) return LSTM_INT_E_BAD_RANGE;
      for (int n = 0; n < N; ++n) {
        const double r = std::floor((double)b[n] / (q.s_W[g] * q.s_x) + 0.5);
        q.bq[g * N + n] = (int32_t)std::fmin(std::fmax(r, -kInt32MaxD), kInt32MaxD);
      }
    }
    // gates to Q3.12, candidate and highway term to the state's format
    const double target = gate ? std::ldexp(1.0, -12) : s_c;
    if ((rc = quantize_multiplier(q.s_W[g] * q.s_x / target, &q.Mx[g], &q.ex[g])) != LSTM_INT_OK) return rc;
    for (int n = 0; n < N; ++n) {  // zero point folded (Sec. 6); accumulators safe for every int8 input
      const int8_t *w = q.Wq.data() + ((size_t)g * N + n) * I;
      int64_t sum = 0, sum_abs = 0;
      for (int k = 0; k < I; ++k) {
        sum += w[k];
        sum_abs += std::abs((int)w[k]);
      }
      const int64_t f = (int64_t)q.bq[g * N + n] - (int64_t)q.zp_x * sum;
      if (std::llabs(f) + 128 * sum_abs > 2147483647LL) return LSTM_INT_E_UNSUPPORTED;
      q.b_fold[g * N + n] = (int32_t)f;
    }
  }
  for (int j = 0; j < 2; ++j) {  // 16-bit recurrent vectors (Sec. 3.2.3); v c goes to Q3.12
    if (!finite_all(p.v[j], N)) return LSTM_INT_E_BAD_RANGE;
    q.s_v[j] = quantize_symmetric(p.v[j], (size_t)N, q.vq.data() + (size_t)j * N, 32767.0);
    if ((rc = quantize_multiplier(q.s_v[j] * s_c * 4096.0, &q.Mv[j], &q.ev[j])) != LSTM_INT_OK) return rc;
  }
  if (G == 3 && (rc = quantize_multiplier(q.s_x / s_c, &q.Ms, &q.es)) != LSTM_INT_OK) return rc;
  return quantize_multiplier(s_c / q.s_h, &q.Mh, &q.eh);
}

// ---------------------------------------------------------------------------
// the scan
// ---------------------------------------------------------------------------

constexpr int kDepth = 4;  // steps whose terms are in flight ahead of the one being computed
constexpr int kSigEntries = 32776;  // the table's 32769 entries, to a multiple of 8
constexpr int kScanBlock = 256;    // threads per workgroup of the scan (each workgroup holds a table: two per compute unit)

struct SruScanArgs {
  int32_t T, B, N, G;
  const int16_t *tx;   // row-major terms [T*B][G*N] (general matmul), or
  const int4 *tx2;     // the register-resident input GEMM's tile order [(t Bp + b) / 32][tile of 8 cells][pair][lane][8]:
                       // lane (row % 32, half) of pair p holds value 4 (slot % 2) + c of slots 2 p, 2 p + 1 for cell
                       // 8 tile + 4 half + c
  int32_t tiles, bp_blocks;  // of tx2: tiles of 8 cells per row block; row blocks per step
  const int8_t *xin;   // layer input [T*B][ld_x]: the highway term of a layer without W_s
  int32_t ld_x, zp_x, zp_h;
  const int16_t *vq;   // [2][N]
  // the four elementwise rescales (x -> highway term, v_f c, v_r c, h16 -> output) in the high-word form: every one of
  // them is followed by a 16-bit clamp or, for the output, by an 8-bit one that the 16-bit clamp cannot change
  // (|zp_h| <= 128)
  RescaleHi ps, pv[2], ph;
  int16_t *c_state;    // [B][N] in/out
  int32_t zero_state;  // start from zeros instead of reading c_state
  int8_t *out;         // [T*B][ld_out] for the next layer's matmul, or NULL
  int32_t ld_out;
  int8_t *y;           // dense [T*B][N], or NULL
  const uint16_t *sig_tab;  // Q3.12
  int16_t *tr_tx, *tr_tv, *tr_act, *tr_c, *tr_h16;  // dumps (row-major form only), each may be NULL
  int8_t *tr_y;
};

// TILE: the terms come in tile order and a wave takes one tile of 8 cells for 32 rows (lane = row % 32 + 32 half):
// its two loads per step are 2 x 1 KB of consecutive memory.  Otherwise (row-major terms) the threads run along the
// cells of a row.  Four cells per thread either way.
// FAST: what the host has checked is compiled in, because a compute unit may hold as little as one wave per SIMD
// here and every instruction of that wave, scalar branches included, is time on the chain from step to step --
// N is a multiple of 4 and y is 4-byte aligned (whole aligned pieces everywhere), no dumps, and the operands of the
// elementwise rescales cannot overflow their left shift (their clamp is dropped).
template <bool TILE, bool FAST>
__global__ __launch_bounds__(kScanBlock) void sru_scan_kernel(SruScanArgs a) {
  constexpr int CPT = 4;             // cells per thread
  constexpr int PRE = FAST ? 1 : 2;  // operand treatment of rescale_sat16_pre
  // the Q3.12 sigma table in LDS: the lookup sits in the chain from one step's state to the next, where a gather
  // from memory costs its full latency every step (measured at 1024 cells, B = 256, T = 64: 117 -> 68 us per layer)
  __shared__ __attribute__((aligned(16))) uint16_t sig_lds[kSigEntries];
  {
    const int4 *src = reinterpret_cast<const int4 *>(a.sig_tab);  // the table's buffer is readable to a multiple of 16 bytes
    int4 *dst = reinterpret_cast<int4 *>(sig_lds);
    for (int i = threadIdx.x; i < kSigEntries / 8; i += kScanBlock) dst[i] = src[i];
    __syncthreads();  // before any thread leaves: every thread of the workgroup gets here
  }
  const int N = a.N;
  int row, n0;
  const int4 *tp = nullptr;
  size_t tp_step = 0;
  if (TILE) {
    const int lane = threadIdx.x & 63;
    const int tiles_used = (N + 7) >> 3;
    const int w = blockIdx.x * (kScanBlock / 64) + (threadIdx.x >> 6);
    const int rbk = w / tiles_used, tile = w - rbk * tiles_used;
    if (rbk >= a.bp_blocks) return;
    row = rbk * 32 + (lane & 31);
    n0 = tile * 8 + 4 * (lane >> 5);
    tp = a.tx2 + ((size_t)rbk * a.tiles + tile) * 128 + lane;
    tp_step = (size_t)a.bp_blocks * a.tiles * 128;
  } else {
    const int N4 = (N + 3) >> 2;
    const int64_t idx = (int64_t)blockIdx.x * kScanBlock + threadIdx.x;
    if (idx >= (int64_t)a.B * N4) return;
    row = (int)(idx / N4);
    n0 = 4 * (int)(idx - (int64_t)row * N4);
  }
  const bool row_ok = row < a.B;
  const int rowc = row_ok ? row : a.B - 1;  // padded rows of the last row block compute on the last row; never stored
  const bool vec = FAST || (N & 3) == 0;    // runs of four cells are whole, aligned pieces
  const bool identity = a.G == 3;

  int32_t cst[CPT], vf[CPT], vr[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int n = n0 + c;
    cst[c] = (n < N && !a.zero_state) ? a.c_state[(size_t)rowc * N + n] : 0;
    vf[c] = n < N ? a.vq[n] : 0;
    vr[c] = n < N ? a.vq[N + n] : 0;
  }

  // the terms of a step as they come from memory
  struct Raw {
    int4 p0, p1;  // tile order: slots (0, 1) and (2, 3); row-major: slots 0..3 as four 8-byte pieces in p0, p1
    int32_t x4;   // the thread's input bytes (identity highway)
  };
  const size_t GN = (size_t)a.G * N;
  auto request = [&](int t) {
    Raw r;
    r.p0 = r.p1 = int4{0, 0, 0, 0};
    r.x4 = 0;
    const size_t tb = (size_t)t * a.B + rowc;
    if (TILE) {
      r.p0 = tp[(size_t)t * tp_step];
      r.p1 = tp[(size_t)t * tp_step + 64];
    } else {
      const int16_t *q = a.tx + tb * GN + n0;
      if (vec) {
        const int2 s0 = *reinterpret_cast<const int2 *>(q), s1 = *reinterpret_cast<const int2 *>(q + N);
        const int2 s2 = *reinterpret_cast<const int2 *>(q + 2 * (size_t)N);
        const int2 s3 = identity ? int2{0, 0} : *reinterpret_cast<const int2 *>(q + 3 * (size_t)N);
        r.p0 = int4{s0.x, s0.y, s1.x, s1.y};
        r.p1 = int4{s2.x, s2.y, s3.x, s3.y};
      } else {
        int32_t e[16];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int c = 0; c < 4; ++c) e[g * 4 + c] = (g < a.G && n0 + c < N) ? q[(size_t)g * N + c] : 0;
        r.p0 = int4{(e[0] & 0xFFFF) | (e[1] << 16), (e[2] & 0xFFFF) | (e[3] << 16), (e[4] & 0xFFFF) | (e[5] << 16),
                    (e[6] & 0xFFFF) | (e[7] << 16)};
        r.p1 = int4{(e[8] & 0xFFFF) | (e[9] << 16), (e[10] & 0xFFFF) | (e[11] << 16), (e[12] & 0xFFFF) | (e[13] << 16),
                    (e[14] & 0xFFFF) | (e[15] << 16)};
      }
    }
    if (identity) {
      const int8_t *xp = a.xin + tb * a.ld_x + n0;
      if (vec) {
        r.x4 = *reinterpret_cast<const int32_t *>(xp);
      } else {
#pragma unroll
        for (int c = 0; c < CPT; ++c) r.x4 |= (n0 + c < N ? (int32_t)(uint8_t)xp[c] : 0) << (8 * c);
      }
    }
    return r;
  };
  auto lo16 = [](int32_t w) { return (int32_t)(int16_t)(w & 0xFFFF); };
  auto hi16 = [](int32_t w) { return w >> 16; };

  auto step = [&](int t, const Raw &r) {
    int32_t tx[4][CPT];  // [slot][cell]
    tx[0][0] = lo16(r.p0.x); tx[0][1] = hi16(r.p0.x); tx[0][2] = lo16(r.p0.y); tx[0][3] = hi16(r.p0.y);
    tx[1][0] = lo16(r.p0.z); tx[1][1] = hi16(r.p0.z); tx[1][2] = lo16(r.p0.w); tx[1][3] = hi16(r.p0.w);
    tx[2][0] = lo16(r.p1.x); tx[2][1] = hi16(r.p1.x); tx[2][2] = lo16(r.p1.y); tx[2][3] = hi16(r.p1.y);
    tx[3][0] = lo16(r.p1.z); tx[3][1] = hi16(r.p1.z); tx[3][2] = lo16(r.p1.w); tx[3][3] = hi16(r.p1.w);
    if (identity) {  // the input itself, brought to the state's format
#pragma unroll
      for (int c = 0; c < CPT; ++c)
        tx[3][c] = rescale_sat16_pre<PRE>((int32_t)(int8_t)((r.x4 >> (8 * c)) & 0xFF) - a.zp_x, a.ps);
    }
    int32_t yv[CPT], hv[CPT], fv[CPT], rv[CPT], tvf[CPT], tvr[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      // both gates read the state before the step (Secs. 3.2.3, 3.2.1)
      // (all products here are of 16-bit values: the 24-bit multiply is exact and runs at full rate)
      tvf[c] = rescale_sat16_pre<PRE>(__mul24(vf[c], cst[c]), a.pv[0]);
      tvr[c] = rescale_sat16_pre<PRE>(__mul24(vr[c], cst[c]), a.pv[1]);
      const int32_t f = sigmoid_from_table(sig_lds, sat16(tx[1][c] + tvf[c]));
      const int32_t g = sigmoid_from_table(sig_lds, sat16(tx[2][c] + tvr[c]));
      const int32_t fbar = 32768 - f < 32767 ? 32768 - f : 32767;  // Sec. 3.2.9
      const int32_t gbar = 32768 - g < 32767 ? 32768 - g : 32767;
      // Sec. 3.2.7: products of a Q0.15 gate and a value in the state's format, each rounded back, saturating sum
      const int32_t cn = sat16(((__mul24(f, cst[c]) + 16384) >> 15) + ((__mul24(fbar, tx[0][c]) + 16384) >> 15));
      const int32_t hn = sat16(((__mul24(g, cn) + 16384) >> 15) + ((__mul24(gbar, tx[3][c]) + 16384) >> 15));
      cst[c] = cn;
      hv[c] = hn;
      fv[c] = f;
      rv[c] = g;
      yv[c] = sat8(rescale_sat16_pre<PRE>(hn, a.ph) + a.zp_h);  // Sec. 3.2.8
    }
    const size_t tb = (size_t)t * a.B + row;
    int32_t packed = 0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) packed |= (int32_t)((uint32_t)(yv[c] & 0xFF) << (8 * c));
    if (FAST) {
      if (row_ok && n0 < N) {  // the only lane-dependent branch of a step
        if (a.out) *reinterpret_cast<int32_t *>(a.out + tb * a.ld_out + n0) = packed;
        if (a.y) *reinterpret_cast<int32_t *>(a.y + tb * N + n0) = packed;
      }
      return;
    }
    if (!row_ok) return;
    auto put = [&](int8_t *o, bool aligned) {
      if (vec && aligned) {
        if (n0 < N) *reinterpret_cast<int32_t *>(o) = packed;
      } else {
#pragma unroll
        for (int c = 0; c < CPT; ++c)
          if (n0 + c < N) o[c] = (int8_t)yv[c];
      }
    };
    if (a.out) put(a.out + tb * a.ld_out + n0, true);
    if (a.y) put(a.y + tb * N + n0, (reinterpret_cast<uintptr_t>(a.y) & 3) == 0);
    if (!TILE) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int n = n0 + c;
        if (n >= N) continue;
        if (a.tr_tx)
#pragma unroll
          for (int g = 0; g < 4; ++g) a.tr_tx[(tb * 4 + g) * N + n] = (int16_t)tx[g][c];
        if (a.tr_tv) {
          a.tr_tv[(tb * 2 + 0) * N + n] = (int16_t)tvf[c];
          a.tr_tv[(tb * 2 + 1) * N + n] = (int16_t)tvr[c];
        }
        if (a.tr_act) {
          a.tr_act[(tb * 2 + 0) * N + n] = (int16_t)fv[c];
          a.tr_act[(tb * 2 + 1) * N + n] = (int16_t)rv[c];
        }
        if (a.tr_c) a.tr_c[tb * N + n] = (int16_t)cst[c];
        if (a.tr_h16) a.tr_h16[tb * N + n] = (int16_t)hv[c];
        if (a.tr_y) a.tr_y[tb * N + n] = (int8_t)yv[c];
      }
    }
  };

  // kDepth steps in flight: named registers, refilled in turn (requests past the end repeat the last step)
  const int T = a.T;
  Raw r0 = request(0), r1 = request(1 < T ? 1 : T - 1), r2 = request(2 < T ? 2 : T - 1), r3 = request(3 < T ? 3 : T - 1);
  static_assert(kDepth == 4, "four named registers sets");
  for (int t = 0; t < T; t += kDepth) {
    step(t, r0);
    r0 = request(t + 4 < T ? t + 4 : T - 1);
    if (t + 1 < T) step(t + 1, r1);
    r1 = request(t + 5 < T ? t + 5 : T - 1);
    if (t + 2 < T) step(t + 2, r2);
    r2 = request(t + 6 < T ? t + 6 : T - 1);
    if (t + 3 < T) step(t + 3, r3);
    r3 = request(t + 7 < T ? t + 7 : T - 1);
  }
  if (row_ok) {
#pragma unroll
    for (int c = 0; c < CPT; ++c)
      if (n0 + c < N) a.c_state[(size_t)row * N + n0 + c] = (int16_t)cst[c];
  }
}

struct SruTimed {
  hipEvent_t start, stop;
  int cls, launches;
};

}  // namespace

}  // namespace lstm_int

using namespace lstm_int;

struct sru_int_model {
  int device = -1;
  bool profiling = false;
  std::vector<SruTimed> timed;
  int register_gemm = 1;
  int num_cus = 0;
  std::vector<SruLayerHost> host;
  std::vector<SruLayerDev> dev;
  uint8_t *arena = nullptr;
  const uint16_t *sig_tab = nullptr;
};

namespace {

struct SruWs {
  size_t xpad, tx, out[2], c, total;
};
SruWs sru_workspace(const sru_int_model *m, int64_t T, int64_t B) {
  SruWs w{};
  size_t off = 0, max_tx = 0, max_out = 0, max_c = 0;
  for (const SruLayerHost &q : m->host) {
    const SruDims d = sru_dims(q.I, q.N, q.G);
    max_tx = std::max(max_tx, (size_t)T * B * q.G * q.N * 2);
    // the same terms in the register-resident input GEMM's tile order: rows padded to 32 per step, cells to 64, 4 slots
    max_tx = std::max(max_tx, (size_t)T * ((B + 31) / 32 * 32) * ((q.N + 63) / 64 * 64) * 4 * 2);
    max_out = std::max(max_out, ((size_t)T * B + 32) * d.Kp);  // 32 rows of slack: that GEMM reads whole blocks of 32 rows
    max_c = std::max(max_c, (size_t)B * q.N * 2);
  }
  const SruDims d0 = sru_dims(m->host[0].I, m->host[0].N, m->host[0].G);
  w.xpad = off; off += align256(((size_t)T * B + 32) * d0.Ip);
  w.tx = off; off += align256(max_tx);
  w.out[0] = off; off += align256(max_out);
  w.out[1] = off; off += align256(max_out);
  w.c = off; off += align256(max_c);
  w.total = off;
  return w;
}

}  // namespace

extern "C" {

int sru_int_prepare(const sru_int_layer_params *layers, int32_t num_layers, int32_t device, sru_int_model **out) {
  if (!layers || !out || num_layers < 1) return LSTM_INT_E_INVALID_ARG;
  *out = nullptr;
  sru_int_model *m = new (std::nothrow) sru_int_model();
  if (!m) return LSTM_INT_E_OUT_OF_MEMORY;
  try {
    m->host.resize(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      if (l > 0 && layers[l].input_size != layers[l - 1].num_cells) {
        delete m;
        return LSTM_INT_E_INVALID_ARG;
      }
      const int rc = prepare_sru_layer(layers[l], l > 0 ? &m->host[l - 1] : nullptr, m->host[l]);
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
    // device image: the Q3.12 sigma table, then per layer W, folded constants, v, and W in the second order
    std::vector<uint8_t> img;
    auto reserve = [&](size_t bytes) {
      const size_t off = align256(img.size());
      img.resize(off + bytes, 0);
      return off;
    };
    const size_t o_sig = reserve((size_t)kSigEntries * 2);
    fill_sigmoid_table(3, reinterpret_cast<uint16_t *>(img.data() + o_sig));
    struct Off { size_t W, bias, vq, W2f, b2; int tiles; };
    std::vector<Off> offs(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      const SruLayerHost &q = m->host[l];
      const int I = q.I, N = q.N, G = q.G;
      const SruDims d = sru_dims(I, N, G);
      Off o{};
      o.W = reserve((size_t)d.cols_pad * d.Ip);
      o.bias = reserve((size_t)d.cols_pad * 4);
      o.vq = reserve((size_t)2 * N * 2);
      if (d.Ip <= 1024) {
        o.tiles = (N + 63) / 64 * 8;
        o.W2f = reserve((size_t)o.tiles * 32 * d.Ip);
        o.b2 = reserve((size_t)o.tiles * 32 * 4);
        for (int g = 0; g < G; ++g)
          for (int n = 0; n < N; ++n) {
            const int tile = n / 8, rho = 8 * g + n % 8;
            const int8_t *w = q.Wq.data() + ((size_t)g * N + n) * I;
            for (int k = 0; k < I; ++k)
              img[o.W2f + ((((size_t)tile * (d.Ip / 32) + k / 32) * 64) + rho + 32 * ((k % 32) / 16)) * 16 + k % 16] = (uint8_t)w[k];
            reinterpret_cast<int32_t *>(img.data() + o.b2)[tile * 32 + rho] = q.b_fold[g * N + n];
          }
      }
      for (int r = 0; r < G * N; ++r) std::memcpy(img.data() + o.W + (size_t)r * d.Ip, q.Wq.data() + (size_t)r * I, I);
      std::memcpy(img.data() + o.bias, q.b_fold.data(), (size_t)G * N * 4);
      std::memcpy(img.data() + o.vq, q.vq.data(), (size_t)2 * N * 2);
      offs[l] = o;
    }
    if (hipSetDevice(device) != hipSuccess || in_gemm_init() != hipSuccess || gemm_init() != hipSuccess ||
        hipMalloc(reinterpret_cast<void **>(&m->arena), img.size()) != hipSuccess) {
      m->arena = nullptr;
      delete m;
      return LSTM_INT_E_DEVICE;
    }
    if (hipMemcpy(m->arena, img.data(), img.size(), hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipFree(m->arena);
      delete m;
      return LSTM_INT_E_DEVICE;
    }
    {
      hipDeviceProp_t prop;
      m->num_cus = hipGetDeviceProperties(&prop, device) == hipSuccess ? prop.multiProcessorCount : 0;
    }
    m->sig_tab = reinterpret_cast<const uint16_t *>(m->arena + o_sig);
    m->dev.resize(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      m->dev[l].W = reinterpret_cast<const int8_t *>(m->arena + offs[l].W);
      m->dev[l].bias = reinterpret_cast<const int32_t *>(m->arena + offs[l].bias);
      m->dev[l].vq = reinterpret_cast<const int16_t *>(m->arena + offs[l].vq);
      if (offs[l].tiles) {
        m->dev[l].W2f = reinterpret_cast<const int8_t *>(m->arena + offs[l].W2f);
        m->dev[l].b2 = reinterpret_cast<const int32_t *>(m->arena + offs[l].b2);
        m->dev[l].tiles = offs[l].tiles;
      }
    }
  } catch (const std::bad_alloc &) {
    delete m;
    return LSTM_INT_E_OUT_OF_MEMORY;
  }
  *out = m;
  return LSTM_INT_OK;
}

int sru_int_get_quant(const sru_int_model *m, int32_t layer, sru_int_layer_quant *out) {
  if (!m || !out || layer < 0 || layer >= (int32_t)m->host.size()) return LSTM_INT_E_INVALID_ARG;
  const SruLayerHost &q = m->host[layer];
  out->I = q.I; out->N = q.N; out->G = q.G;
  out->zp_x = q.zp_x; out->zp_h = q.zp_h; out->m_c = q.m_c;
  out->s_x = q.s_x; out->s_h = q.s_h;
  for (int g = 0; g < 4; ++g) {
    out->s_W[g] = q.s_W[g]; out->Mx[g] = q.Mx[g]; out->ex[g] = q.ex[g];
  }
  for (int j = 0; j < 2; ++j) {
    out->s_v[j] = q.s_v[j]; out->Mv[j] = q.Mv[j]; out->ev[j] = q.ev[j];
  }
  out->Ms = q.Ms; out->es = q.es; out->Mh = q.Mh; out->eh = q.eh;
  out->Wq = q.Wq.data(); out->vq = q.vq.data(); out->bq = q.bq.data(); out->b_fold = q.b_fold.data();
  return LSTM_INT_OK;
}

size_t sru_int_workspace_bytes(const sru_int_model *m, int32_t T, int32_t B) {
  if (!m || T < 0 || B < 0 || m->host.empty()) return 0;
  return sru_workspace(m, T, B).total;
}

int sru_int_forward(const sru_int_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y, int16_t *c_state,
                    void *workspace, size_t workspace_bytes, void *hip_stream, const sru_int_trace *trace) {
  if (!m || T < 0 || B < 0) return LSTM_INT_E_INVALID_ARG;
  if (T == 0 || B == 0) return LSTM_INT_OK;
  if (!x || !y) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  const int L = (int)m->host.size();
  if (trace && (trace->layer < 0 || trace->layer >= L)) return LSTM_INT_E_INVALID_ARG;
  int64_t widest = 0;
  for (const SruLayerHost &q : m->host)
    widest = std::max<int64_t>(widest, std::max(4 * (int64_t)((q.N + 63) / 64 * 64), (int64_t)sru_dims(q.I, q.N, q.G).Ip));
  if ((int64_t)T * ((B + 31) / 32 * 32) * widest >= ((int64_t)1 << 31)) return LSTM_INT_E_UNSUPPORTED;  // 32-bit row arithmetic of the matmuls
  // the scan applies its elementwise rescales in the high-word form, which needs shifts of at least 3: scales below
  // 2^28, which every realistic model has
  for (const SruLayerHost &q : m->host)
    if ((q.G == 3 && 31 - q.es < 3) || 31 - q.ev[0] < 3 || 31 - q.ev[1] < 3 || 31 - q.eh < 3) return LSTM_INT_E_UNSUPPORTED;
  const SruWs w = sru_workspace(m, T, B);
  if (!workspace || workspace_bytes < w.total || (reinterpret_cast<uintptr_t>(workspace) & 255)) return LSTM_INT_E_WORKSPACE;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  uint8_t *ws = reinterpret_cast<uint8_t *>(workspace);
  const int64_t TB = (int64_t)T * B;

  const int8_t *in = x;
  int ld_in = m->host[0].I;
  {
    // the matmuls read rows of Ip bytes in 16-byte pieces, the register-resident one whole blocks of 32 rows: a
    // padded copy (with 32 rows of slack behind it) unless x already has that shape
    const SruDims d0 = sru_dims(m->host[0].I, m->host[0].N, m->host[0].G);
    if (d0.Ip != m->host[0].I || (reinterpret_cast<uintptr_t>(x) & 15) || (B & 31)) {
      int8_t *xp = reinterpret_cast<int8_t *>(ws + w.xpad);
      launch_copy_rows_i8(s, x, m->host[0].I, xp, d0.Ip, (int)TB, m->host[0].I, 0);
      in = xp;
      ld_in = d0.Ip;
    }
  }
  sru_int_model *mm = const_cast<sru_int_model *>(m);  // the profile is bookkeeping beside the model
  auto timed_begin = [&](int cls) {
    if (!m->profiling) return;
    SruTimed e{nullptr, nullptr, cls, 1};
    if (hipEventCreate(&e.start) != hipSuccess || hipEventCreate(&e.stop) != hipSuccess) return;
    (void)hipEventRecord(e.start, s);
    mm->timed.push_back(e);
  };
  auto timed_end = [&]() {
    if (m->profiling && !mm->timed.empty()) (void)hipEventRecord(mm->timed.back().stop, s);
  };
  size_t c_off = 0;
  for (int l = 0; l < L; ++l) {
    const SruLayerHost &q = m->host[l];
    const SruLayerDev &dv = m->dev[l];
    const int N = q.N, G = q.G;
    const SruDims d = sru_dims(q.I, N, G);
    int16_t *tx = reinterpret_cast<int16_t *>(ws + w.tx);
    int8_t *out = reinterpret_cast<int8_t *>(ws + w.out[l & 1]);
    const sru_int_trace *tr = (trace && trace->layer == l) ? trace : nullptr;

    InGemmArgs ga{};
    ga.A = in; ga.a_slack = 1; ga.lda = ld_in; ga.T = T; ga.B = B; ga.Bp = (B + 31) / 32 * 32;
    ga.W2f = dv.W2f; ga.kpad = d.Ip; ga.tiles = dv.tiles; ga.bx2 = dv.b2;
    for (int g = 0; g < 4; ++g) {
      ga.M[g] = g < G ? q.Mx[g] : 1 << 30;  // an empty slot 3 multiplies zeros
      ga.r[g] = g < G ? 31 - q.ex[g] : 33;
    }
    ga.tx2 = reinterpret_cast<int4 *>(ws + w.tx);
    const bool ws_gemm = m->register_gemm && !tr && dv.W2f && m->num_cus == 256 && in_gemm_ws_supported(ga);
    timed_begin(SRU_INT_K_INPUT_GEMM);
    if (ws_gemm) {
      launch_in_gemm_ws(s, ga, m->num_cus);
    } else {
      Requant rq{};
      rq.all_hi = 1;
      for (int g = 0; g < 4; ++g) {
        rq.M[g] = q.Mx[g < G ? g : G - 1];
        rq.r[g] = 31 - q.ex[g < G ? g : G - 1];
        if (rq.r[g] < 33) rq.all_hi = 0;
      }
      rq.cols_per_gate = N;
      rq.zp = 0;
      launch_gemm_i16(s, in, ld_in, (int)TB, dv.W, d.Ip, G * N, dv.bias, rq, tx, G * N);
    }
    timed_end();

    SruScanArgs a{};
    a.T = T; a.B = B; a.N = N; a.G = G;
    a.tx = ws_gemm ? nullptr : tx;
    a.tx2 = ws_gemm ? ga.tx2 : nullptr;
    a.tiles = dv.tiles; a.bp_blocks = ga.Bp / 32;
    a.xin = in; a.ld_x = ld_in; a.zp_x = q.zp_x; a.zp_h = q.zp_h;
    a.vq = dv.vq;
    a.ps = rescale_hi_prepare(G == 3 ? q.Ms : 1 << 30, G == 3 ? 31 - q.es : 33);
    for (int j = 0; j < 2; ++j) a.pv[j] = rescale_hi_prepare(q.Mv[j], 31 - q.ev[j]);
    a.ph = rescale_hi_prepare(q.Mh, 31 - q.eh);
    a.c_state = c_state ? c_state + c_off : reinterpret_cast<int16_t *>(ws + w.c);
    a.zero_state = c_state ? 0 : 1;
    a.out = l == L - 1 ? nullptr : out;
    a.ld_out = d.Kp;
    a.y = l == L - 1 ? y : nullptr;
    a.sig_tab = m->sig_tab;
    if (tr) {
      a.tr_tx = tr->tx; a.tr_tv = tr->tv; a.tr_act = tr->act; a.tr_c = tr->c; a.tr_h16 = tr->h16; a.tr_y = tr->y;
    }
    timed_begin(SRU_INT_K_SCAN);
    constexpr int kWpb = kScanBlock / 64;
    // the specialization that drops the checks the host can make once (see sru_scan_kernel)
    const bool fast = !tr && (N & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 3) == 0 && 31 - q.ev[0] >= 32 &&
                      31 - q.ev[1] >= 32 && 31 - q.eh >= 18 && (G == 4 || 31 - q.es >= 11);
    if (ws_gemm) {
      const dim3 grid((unsigned)(((int64_t)a.bp_blocks * ((N + 7) / 8) + kWpb - 1) / kWpb));
      if (fast)
        hipLaunchKernelGGL((sru_scan_kernel<true, true>), grid, dim3(kScanBlock), 0, s, a);
      else
        hipLaunchKernelGGL((sru_scan_kernel<true, false>), grid, dim3(kScanBlock), 0, s, a);
    } else {
      const dim3 grid((unsigned)(((int64_t)B * ((N + 3) / 4) + kScanBlock - 1) / kScanBlock));
      if (fast)
        hipLaunchKernelGGL((sru_scan_kernel<false, true>), grid, dim3(kScanBlock), 0, s, a);
      else
        hipLaunchKernelGGL((sru_scan_kernel<false, false>), grid, dim3(kScanBlock), 0, s, a);
    }
    timed_end();
    in = out;
    ld_in = d.Kp;
    c_off += (size_t)B * N;
  }
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

int sru_int_set_option(sru_int_model *m, const char *key, int64_t value) {
  if (!m || !key) return LSTM_INT_E_INVALID_ARG;
  if (!strcmp(key, "register_gemm")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->register_gemm = (int)value;
    return LSTM_INT_OK;
  }
  return LSTM_INT_E_INVALID_ARG;
}

int sru_int_profile_begin(sru_int_model *m) {
  if (!m) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  for (SruTimed &e : m->timed) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  m->timed.clear();
  m->profiling = true;
  return LSTM_INT_OK;
}

int sru_int_profile_end(sru_int_model *m, int64_t launches[SRU_INT_K_COUNT], double total_ms[SRU_INT_K_COUNT]) {
  if (!m || !launches || !total_ms) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  m->profiling = false;
  for (int k = 0; k < SRU_INT_K_COUNT; ++k) {
    launches[k] = 0;
    total_ms[k] = 0.0;
  }
  int rc = LSTM_INT_OK;
  if (hipSetDevice(m->device) != hipSuccess) rc = LSTM_INT_E_DEVICE;
  for (SruTimed &e : m->timed) {
    float ms = 0.f;
    if (rc == LSTM_INT_OK && hipEventSynchronize(e.stop) == hipSuccess && hipEventElapsedTime(&ms, e.start, e.stop) == hipSuccess) {
      launches[e.cls] += e.launches;
      total_ms[e.cls] += ms;
    } else {
      rc = LSTM_INT_E_DEVICE;
    }
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  m->timed.clear();
  return rc;
}

void sru_int_destroy(sru_int_model *m) {
  if (!m) return;
  for (SruTimed &e : m->timed) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  if (m->arena) {
    (void)hipSetDevice(m->device);
    (void)hipFree(m->arena);
  }
  delete m;
}

}  // extern "C"
