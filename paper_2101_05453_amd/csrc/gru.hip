// Integer-only GRU (include/gru_int.h): the recipe assembled from the building
// blocks of arXiv 2101.05453 (Sec. 7 names the GRU; Secs. 3.2.1, 3.2.2, 3.2.4,
// 3.2.7, 3.2.9 and Sec. 6 supply the blocks), offline phase on the host and
// the online phase as HIP kernels for gfx950.
//
// Online phase per layer:
//   1. tx = sat16(rescale(W x + bx')) for all T*B rows: the library's int8
//      MFMA matmul (kernels.hip), gate-major columns [3N].
//   2. per step ONE kernel, gru_step_kernel: R h8 + bh for the three gates on
//      the 32x32x32 int8 MFMA, a workgroup per tile of 32 cells x 32 or 64
//      batch rows, depth split over its four waves, weights and state read in
//      operand order (one contiguous KB per wave load, every byte once per
//      workgroup).  The MFMA leaves a lane with the three gate accumulators of
//      the same cells of one batch row, so the whole elementwise cell
//      (rescale, sigma/tanh tables, reset product, coupled update, the int8
//      form of the new state) follows in the same kernel with one LDS
//      reduction and no exchange between workgroups.
//   3. where the layer fits (up to 1024 cells), steps 2 of all T steps as ONE
//      persistent launch, gru_seq_kernel: weights in registers, one barrier
//      per step among the workgroups of an XCD that share 32 batch rows; the
//      input term then comes from the LSTM path's register-resident input GEMM
//      (in_gemm.hip) in its tile order.
// The state is read and written in place (each (row, cell) belongs to one
// thread); its int8 form is written three times: in operand order for the
// next step, row-major for the next layer's matmul, dense for the caller.
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
#include "persistent.h"

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
  int Ip, Kp, Ncp, cols_pad;  // input depth / state depth (multiples of 64), cells (multiple of 32), 3N to 128
};
GruDims gru_dims(int I, int N) {
  return GruDims{(I + 63) / 64 * 64, (N + 63) / 64 * 64, (N + 31) / 32 * 32, (3 * N + 127) / 128 * 128};
}
// bytes of the operand-ordered copy of the int8 state for B rows: whole blocks of 32 rows, an even number of them
size_t hop_bytes(int B, int Kp) { return (size_t)((B + 63) / 64 * 2) * (Kp / 32) * 1024; }

struct GruLayerDev {
  const int8_t *W = nullptr;      // [cols_pad][Ip] gate-major rows, zero beyond the real extents
  const int32_t *bx = nullptr;    // [cols_pad] folded input bias
  const int8_t *Rop = nullptr;    // [Ncp/32][3][Kp/32][64 lanes][16 B]: operand order of the 32x32x32 MFMA
  const int32_t *bh = nullptr;    // [3][Ncp]
  // input depth up to 1024: W once more as the register-resident input GEMM reads it (in_gemm.hip): tiles of 8 cells
  // x 4 gate slots (slot 0 empty, slots 1-3 = r, u, n), row 8 slot + cell % 8, [tile][Ip/32][64 lanes][16 B]
  const int8_t *W2f = nullptr;
  const int32_t *bx2 = nullptr;   // [tiles][32]
  int tiles = 0;                  // a multiple of 8 (cells padded to 64)
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

typedef int v16i __attribute__((ext_vector_type(16)));

// the int8 form of a state value: sat8(floor((h16 + 128) / 256))
__device__ __forceinline__ int32_t state_i8(int32_t h16) { return sat8((h16 + 128) >> 8); }

// Byte offset of state value (row, k) in the operand-ordered copy of h8 that the step kernel reads:
// [row / 32][k / 32][64 lanes][16 B], lane = 32 ((k / 16) % 2) + row % 32 -- the second operand of the
// 32x32x32 int8 MFMA for 32 rows and one 32-deep k step is one contiguous KB.
__host__ __device__ __forceinline__ size_t hop_offset(int row, int k, int KS32) {
  return ((((size_t)(row >> 5) * KS32 + (k >> 5)) * 64 + (((k >> 4) & 1) << 5) + (row & 31)) << 4) + (k & 15);
}

// Start of a layer: the working state (caller's h_state slice or zeros) is used in place; its int8 form
// goes to the operand-ordered buffer hop0 (columns N..Kp-1 zero); sync_vec 16-byte words at sync are cleared.
__global__ void gru_init_kernel(int16_t *h16, int B, int N, int Kp, int8_t *hop0, int zero_state, int4 *sync,
                                int sync_vec) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < sync_vec) sync[i] = int4{0, 0, 0, 0};  // counters and placement words of the persistent kernel
  if (i >= (int64_t)B * Kp) return;
  const int b = (int)(i / Kp), k = (int)(i - (int64_t)b * Kp);
  int32_t v = 0;
  if (k < N) {
    if (zero_state)
      h16[(size_t)b * N + k] = 0;
    else
      v = state_i8(h16[(size_t)b * N + k]);
  }
  hop0[hop_offset(b, k, Kp >> 5)] = (int8_t)v;
}

struct GruStepArgs {
  int32_t B, N, Kp, KS32;     // KS32 = Kp / 32
  int32_t ctiles, rtn;        // tiles of 32 cells; tiles of 32 RB rows
  const int8_t *hop_prev;     // state before the step, operand order
  const int8_t *Rop;          // [ctiles][3][KS32][64 lanes][16 B]
  const int32_t *bh;          // [3][32 ctiles]
  const int16_t *tx;          // [B][3N] of this step, or NULL:
  const int4 *tx2;            // this step's input terms in the input GEMM's tile order [row block][tile of 8 cells][half][lane][8]
  int32_t tiles;              // tiles of 8 cells per row block of tx2
  int16_t *h16;               // [B][N] in/out
  int8_t *hop_out;            // state after the step, operand order
  int8_t *h8_out;             // [B][Kp] row-major (the next layer's matmul input)
  int8_t *y;                  // [B][N] or NULL
  int32_t Mh[3], rh[3];
  const uint16_t *sig_tab, *tanh_tab;  // [32769] each, Q3.12 inputs
  int16_t *tr_tx, *tr_th, *tr_act, *tr_h16;  // [B][3][N] / [B][N] of this step, or NULL
  int8_t *tr_h8;
};

// One step of one layer.  A workgroup owns 32 cells (their r, u, n rows of R: 96 x Kp bytes) and 32 RB batch
// rows (the library launches RB = 1); its four waves split the depth, each running its quarter of the k steps for all RB x 3 tiles of the
// 32x32x32 int8 MFMA with both operands loaded straight into registers in operand order (every byte of the
// weight slice and of the state tile is loaded once per workgroup, a contiguous KB per wave load), and the four
// partial sums meet in LDS.  The MFMA leaves a lane with 16 cells of one batch row, the same cells in each of
// the three gate tiles, so the elementwise cell needs no further exchange.
// Workgroup w takes cell tile (w % 8) + 8 (w / 8 / rtn): the hardware deals consecutive workgroups out to the
// eight XCDs in turn, and every launch here is a multiple of eight workgroups, so an XCD meets the same eighth
// of R at every step of a sequence and keeps it in its L2 (N = 2048: 1.5 MB of 4 MB).  The mapping only places
// the work; results do not depend on where a workgroup runs.
constexpr int kPartTile = 32 * 33;  // one 32 x 32 tile of partial sums in LDS, row stride 33
constexpr int kSeqSigBytes = 65552;  // the sigma table of the persistent kernel in LDS: 32769 entries, to 16 bytes

template <int RB>
__global__ __launch_bounds__(256) void gru_step_kernel(GruStepArgs a) {
  extern __shared__ __attribute__((aligned(16))) int32_t part[];  // [4 waves][RB][3][kPartTile]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, b2 = lane >> 5;
  const int w = blockIdx.x, j = w >> 3;
  const int ct = (w & 7) + 8 * (j / a.rtn), rt = j % a.rtn;
  if (ct >= a.ctiles) return;  // uniform over the workgroup, ahead of every barrier
  const int KS = a.KS32;
  const int rblocks = (a.B + 31) >> 5;  // row blocks that exist in the operand-ordered buffers

  // this thread's share of the elementwise cell, and its W x terms and old state requested now: they come from
  // memory and are not needed before the matmul is done
  const int rsub = threadIdx.x >> 3, cg = threadIdx.x & 7;
  const int N = a.N;
  const int n0 = ct * 32 + 4 * cg;
  const bool vec = (N & 3) == 0;  // runs of four cells are aligned 8-byte pieces of tx and h16
  int rowe[RB];
  int32_t txe[RB][3][4], h16e[RB][4];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    rowe[rb] = (rt * RB + rb) * 32 + rsub;
    const int row = rowe[rb] < a.B ? rowe[rb] : a.B - 1;
    const int16_t *hq = a.h16 + (size_t)row * N + n0;
    if (vec && n0 < N) {
      const short4 h4 = *reinterpret_cast<const short4 *>(hq);
      h16e[rb][0] = h4.x; h16e[rb][1] = h4.y; h16e[rb][2] = h4.z; h16e[rb][3] = h4.w;
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) h16e[rb][c] = n0 + c < N ? hq[c] : 0;
    }
    if (a.tx2) {
      // the input term in the register-resident input GEMM's tile order (this step's row blocks): lane
      // (row % 32, half) of tile n / 8 holds value 4 slot + c for cell 8 (n / 8) + 4 half + c; slots 1-3 = r, u, n
      const int4 *tp = a.tx2 + ((size_t)(rt * RB + rb) * a.tiles + (ct * 4 + (cg >> 1))) * 128 + ((cg & 1) << 5) + rsub;
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        const int slot = g + 1;
        const short4 t4 = *reinterpret_cast<const short4 *>(reinterpret_cast<const int16_t *>(tp + (slot >> 1) * 64) + (slot & 1) * 4);
        txe[rb][g][0] = t4.x; txe[rb][g][1] = t4.y; txe[rb][g][2] = t4.z; txe[rb][g][3] = t4.w;
      }
    } else {
      const int16_t *txp = a.tx + (size_t)row * 3 * N + n0;
      if (vec && n0 < N) {
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          const short4 t4 = *reinterpret_cast<const short4 *>(txp + (size_t)g * N);
          txe[rb][g][0] = t4.x; txe[rb][g][1] = t4.y; txe[rb][g][2] = t4.z; txe[rb][g][3] = t4.w;
        }
      } else {
#pragma unroll
        for (int g = 0; g < 3; ++g)
#pragma unroll
          for (int c = 0; c < 4; ++c) txe[rb][g][c] = n0 + c < N ? txp[(size_t)g * N + c] : 0;
      }
    }
  }

  v16i acc[RB][3];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rb][g][v] = 0;
  const v4i *wp = reinterpret_cast<const v4i *>(a.Rop) + (size_t)ct * 3 * KS * 64 + lane;
  const v4i *hp[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    int blk = rt * RB + rb;
    blk = blk < rblocks ? blk : rblocks - 1;  // a row block past the batch repeats the last one; never stored
    hp[rb] = reinterpret_cast<const v4i *>(a.hop_prev) + (size_t)blk * KS * 64 + lane;
  }
  const int per = (KS + 3) >> 2;
  const int k0 = wave * per, k1 = k0 + per < KS ? k0 + per : KS;
  // U k steps per batch, all their loads in flight together (one wave per SIMD: nothing else hides the
  // latency); steps past the wave's share re-read its last step against zero weights
  constexpr int U = 8;
  for (int ks = k0; ks < k1; ks += U) {
    v4i hf[U][RB], wf[U][3];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kk = ks + u < k1 ? ks + u : k1 - 1;
#pragma unroll
      for (int g = 0; g < 3; ++g) wf[u][g] = wp[((size_t)g * KS + kk) * 64];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) hf[u][rb] = hp[rb][(size_t)kk * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool live = ks + u < k1;
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        const v4i wv = live ? wf[u][g] : v4i{0, 0, 0, 0};
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          acc[rb][g] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv, hf[u][rb], acc[rb][g], 0, 0, 0);
      }
    }
  }
  // partial sums -> LDS as [wave][rb][gate][2 v + b2][33]: result value v of lane (col, b2) is cell
  // 8 (v / 4) + 4 b2 + v % 4 of the tile for batch row col; the odd stride keeps the transposed reads below
  // at two lanes per bank
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) part[((wave * RB + rb) * 3 + g) * kPartTile + (2 * v + b2) * 33 + col] = acc[rb][g][v];
  __syncthreads();

  // The elementwise cell, with the threads laid out along the rows: thread (rsub, cg) takes cells 4 cg .. 4 cg + 3
  // of row rsub in each row block, so that a wave's loads and stores cover runs of 32 consecutive cells of 8 rows
  // (a lane's four cells share the result index v / 4 = cg / 2 and the lane half b2 = cg % 2).
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = rowe[rb];
    const bool row_ok = row < a.B;
    int32_t h84[4], hn4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int n = n0 + c;
      int32_t th[3];
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        const int o = (rb * 3 + g) * kPartTile + (2 * (4 * (cg >> 1) + c) + (cg & 1)) * 33 + rsub;
        const int32_t sum = part[o] + part[o + RB * 3 * kPartTile] + part[o + 2 * RB * 3 * kPartTile] + part[o + 3 * RB * 3 * kPartTile];
        th[g] = sat16(rescale(sum + a.bh[g * 32 * a.ctiles + n], a.Mh[g], a.rh[g]));
      }
      const int32_t r = sigmoid_from_table(a.sig_tab, sat16(txe[rb][0][c] + th[0]));  // Sec. 3.2.1
      const int32_t u = sigmoid_from_table(a.sig_tab, sat16(txe[rb][1][c] + th[1]));
      const int32_t rn = (r * th[2] + 16384) >> 15;  // Q0.15 x Q3.12 -> Q3.12; |r th| < 2^30
      const int32_t cand = tanh_from_table(a.tanh_tab, sat16(txe[rb][2][c] + rn));
      const int32_t ubar = cifg_input_gate(u);  // 1 - u, Sec. 3.2.9
      const int32_t hn = cell_update32(ubar, cand, u, h16e[rb][c], 0);  // Sec. 3.2.7, both products Q0.30 -> Q0.15
      hn4[c] = hn;
      h84[c] = state_i8(hn);
      if (row_ok && n < N) {
        const size_t row3 = (size_t)row * 3 * N;
        if (a.tr_tx)
          for (int g = 0; g < 3; ++g) a.tr_tx[row3 + (size_t)g * N + n] = (int16_t)txe[rb][g][c];
        if (a.tr_th)
          for (int g = 0; g < 3; ++g) a.tr_th[row3 + (size_t)g * N + n] = (int16_t)th[g];
        if (a.tr_act) {
          a.tr_act[row3 + n] = (int16_t)r;
          a.tr_act[row3 + (size_t)N + n] = (int16_t)u;
          a.tr_act[row3 + (size_t)2 * N + n] = (int16_t)cand;
        }
        if (a.tr_h16) a.tr_h16[(size_t)row * N + n] = (int16_t)hn;
        if (a.tr_h8) a.tr_h8[(size_t)row * N + n] = (int8_t)h84[c];
      }
    }
    if (!row_ok || n0 >= N) continue;
    int16_t *hd = a.h16 + (size_t)row * N + n0;
    if (vec) {
      short4 o4;
      o4.x = (short)hn4[0]; o4.y = (short)hn4[1]; o4.z = (short)hn4[2]; o4.w = (short)hn4[3];
      *reinterpret_cast<short4 *>(hd) = o4;
    } else {
      for (int c = 0; c < 4 && n0 + c < N; ++c) hd[c] = (int16_t)hn4[c];
    }
    // the int8 form: operand order for the next step, row-major for the next layer, dense for the caller
    uint32_t pk = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) pk |= (uint32_t)((n0 + c < N ? h84[c] : 0) & 0xFF) << (8 * c);
    *reinterpret_cast<uint32_t *>(a.hop_out + hop_offset(row, n0, KS)) = pk;  // cells past N hold 0 and meet zero weights
    *reinterpret_cast<uint32_t *>(a.h8_out + (size_t)row * a.Kp + n0) = pk;
    if (a.y) {
      int8_t *yd = a.y + (size_t)row * N + n0;
      if (vec && !(reinterpret_cast<uintptr_t>(a.y) & 3))
        *reinterpret_cast<uint32_t *>(yd) = pk;
      else
        for (int c = 0; c < 4 && n0 + c < N; ++c) yd[c] = (int8_t)h84[c];
    }
  }
}

// ---------------------------------------------------------------------------
// Persistent form of the step kernel: one launch runs all T steps of a layer.
// ---------------------------------------------------------------------------
// Wait of one workgroup for the other members of its group (the workgroups that share 32 batch rows), at the end of
// every step: every wave first waits for its own stores, thread 0 adds one to the group's counter and polls it
// (relaxed agent-scope atomics; the members of a group run on one XCD and meet in its L2).  Gives up after
// spin_limit polls or when another workgroup has: the status word becomes 1 and every workgroup leaves the kernel.
__device__ __forceinline__ bool gru_group_sync(unsigned *counter, unsigned &epoch, int GS, int *status, int spin_limit,
                                               int first_sleep, int *lds_flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (GS == 1) return true;
  epoch += (unsigned)GS;
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int i = 0; i < first_sleep; ++i) __builtin_amdgcn_s_sleep(1);  // a poll before the arrivals have landed only delays them
    int budget = spin_limit;
    for (;;) {
      const unsigned c = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((int)(c - epoch) >= 0) break;
      --budget;
      if ((budget & 15) == 0 &&
          (budget <= 0 || __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lds_flag[0] = 0;
        break;
      }
    }
  }
  __syncthreads();
  return lds_flag[0] != 0;
}

struct GruSeqArgs {
  int32_t B, N, Kp, KS32, T;
  int32_t GS, groups;         // workgroups per group (= tiles of 32 cells); groups of 32 batch rows
  const int8_t *hop0;         // state before step 0, operand order
  int8_t *hop_seq;            // [T][row blocks][KS32][64 lanes][16 B]: the state after every step, operand order; the
                              // exchange buffer of the launch, every line written once and never read before that
  size_t hop_step;            // bytes of one step of hop_seq
  const int8_t *Rop;          // [GS][3][KS32][64 lanes][16 B]
  const int32_t *bh;          // [3][32 GS]
  const int16_t *tx;          // [T][B][3N], or NULL:
  const int4 *tx2;            // the input term in the input GEMM's tile order [(t Bp + b) / 32][tile of 8 cells][half][lane][8]
  int32_t tiles, bp_blocks;   // of tx2: tiles of 8 cells per row block; row blocks per step (Bp / 32)
  int16_t *h16;               // [B][N]: read before step 0, written after step T - 1
  int8_t *h8_seq;             // [T][B][Kp] row-major
  int8_t *y;                  // [T][B][N] or NULL
  int32_t Mh[3], rh[3];
  const uint16_t *sig_tab, *tanh_tab;
  unsigned *counters;         // [groups][64], zero at launch
  unsigned long long *tickets;  // [8][32], zero at launch: placement check
  int *status;
  int32_t spin_limit, sync_sleep;
  int32_t extra_arrivals;     // test hook: every barrier waits for this many arrivals more than will come
};

constexpr int kSeqMaxPer = 8;  // k steps per wave: depth up to 4 x 8 x 32 = 1024

// The step kernel's work with the weights kept in registers over the whole sequence: the workgroups that share 32
// batch rows -- one per tile of 32 cells -- form a group on ONE XCD; each keeps its 96 x Kp bytes of R as MFMA
// operands (wave w the k steps of its quarter of the depth: at most 96 registers), its threads' share of the state in
// registers, and per step loads only the int8 state of the group (operand order, one KB per k step, the KB of k step j
// written by member j), runs the matmul and the cell as gru_step_kernel does, publishes its 32 cells of the new state
// and meets the group at one barrier.  A GRU step needs this one exchange (the LSTM with layer norm and projection
// needs three).  Placement: the XCD is read from the XCC_ID register and the place there is w / 8 (the hardware deals
// consecutive workgroups out to the XCDs in turn); every workgroup records its place when it is done and a place taken
// twice or not at all raises the status word (2), as in the LSTM's recurrent kernel.  All workgroups must be resident
// at once (one per compute unit, launched on an otherwise idle stream); if they are not, the bounded waits end the
// kernel with status 1.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gru_seq_kernel(GruSeqArgs a) {
  __shared__ __attribute__((aligned(16))) int32_t part[4 * 3 * kPartTile];
  __shared__ int flag[4];
  // the sigma table (Q3.12, all 32769 entries) in LDS: the reset gate's lookup is the first of two dependent ones on
  // the chain from the matmul to the new state, and from LDS it no longer costs a round trip to the L2
  extern __shared__ __attribute__((aligned(16))) uint16_t sig_lds[];  // kSeqSigBytes, set at launch
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, b2 = lane >> 5;
  const int wg = blockIdx.x;
  const int xcc = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7);  // XCC_ID, bits 3:0
  const int slot = wg >> 3, GS = a.GS;
  auto placement_check = [&]() {
    if (tid == 0) {
      const unsigned places = gridDim.x >> 3;  // at most 32
      const unsigned long long mine = (1ull << 32) + (1ull << (wg >> 3));
      const unsigned long long now =
          __hip_atomic_fetch_add(&a.tickets[xcc * 32], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
      const unsigned count = (unsigned)(now >> 32);
      const unsigned all = places >= 32 ? 0xFFFFFFFFu : (1u << places) - 1;
      if (count > places || (count == places && (unsigned)now != all))
        __hip_atomic_store(a.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  const int group = xcc + 8 * (slot / GS), ct = slot % GS;
  if (group >= a.groups) {  // no rows for this workgroup
    placement_check();
    return;
  }
  const int KS = a.KS32;
  const int per = (KS + 3) >> 2;
  const int k0 = wave * per, k1 = k0 + per < KS ? k0 + per : KS;

  // ---- once: the wave's share of the weights -> registers (k steps past its share hold zeros)
  v4i Wr[3][kSeqMaxPer];
  {
    const v4i *wp = reinterpret_cast<const v4i *>(a.Rop) + (size_t)ct * 3 * KS * 64 + lane;
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int u = 0; u < kSeqMaxPer; ++u) {
        Wr[g][u] = k0 + u < k1 ? wp[((size_t)g * KS + k0 + u) * 64] : v4i{0, 0, 0, 0};
      }
  }
  // this thread's share of the cell: row rsub of the group, cells 4 cg .. 4 cg + 3 of the tile
  const int rsub = tid >> 3, cg = tid & 7;
  const int N = a.N;
  const int n0 = ct * 32 + 4 * cg;
  const int row = group * 32 + rsub;
  const bool row_ok = row < a.B;
  const int rowc = row_ok ? row : a.B - 1;
  const bool vec = (N & 3) == 0;
  int32_t bhe[3][4], h16r[4];
#pragma unroll
  for (int g = 0; g < 3; ++g) {
    const int4 b4 = *reinterpret_cast<const int4 *>(a.bh + g * 32 * GS + n0);
    bhe[g][0] = b4.x; bhe[g][1] = b4.y; bhe[g][2] = b4.z; bhe[g][3] = b4.w;
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) h16r[c] = n0 + c < N ? a.h16[(size_t)rowc * N + n0 + c] : 0;
  {
    const int4 *src = reinterpret_cast<const int4 *>(a.sig_tab);  // readable to a multiple of 16 bytes: the arena goes on
    int4 *dst = reinterpret_cast<int4 *>(sig_lds);
    for (int i = tid; i < kSeqSigBytes / 16; i += 256) dst[i] = src[i];
  }
  if (tid == 0) flag[0] = 1;
  __syncthreads();

  unsigned epoch = 0;
  unsigned *counter = a.counters + group * 64;
  const size_t hop_blk = (size_t)group * KS * 64;  // this group's row block, in 16-byte units
  for (int t = 0; t < a.T; ++t) {
    // W x terms of this thread's cells: from memory, not needed before the matmul is done
    int32_t txe[3][4];
    if (a.tx2) {
      // tile order: lane (row % 32, half b2) of tile n / 8 holds value 4 slot + c for cell 8 (n / 8) + 4 b2 + c, values
      // 0-7 in the first 16 bytes of the lane, 8-15 in the second
      const int4 *tp = a.tx2 + (((size_t)t * a.bp_blocks + group) * a.tiles + (ct * 4 + (cg >> 1))) * 128 + ((cg & 1) << 5) + rsub;
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        const int slot = g + 1;
        const short4 t4 = *reinterpret_cast<const short4 *>(reinterpret_cast<const int16_t *>(tp + (slot >> 1) * 64) + (slot & 1) * 4);
        txe[g][0] = t4.x; txe[g][1] = t4.y; txe[g][2] = t4.z; txe[g][3] = t4.w;
      }
    } else {
      const int16_t *txp = a.tx + ((size_t)t * a.B + rowc) * 3 * N + n0;
      if (vec && n0 < N) {
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          const short4 t4 = *reinterpret_cast<const short4 *>(txp + (size_t)g * N);
          txe[g][0] = t4.x; txe[g][1] = t4.y; txe[g][2] = t4.z; txe[g][3] = t4.w;
        }
      } else {
#pragma unroll
        for (int g = 0; g < 3; ++g)
#pragma unroll
          for (int c = 0; c < 4; ++c) txe[g][c] = n0 + c < N ? txp[(size_t)g * N + c] : 0;
      }
    }
    // ---- R h8: the group's int8 state, the wave's k steps
    const v4i *hp = reinterpret_cast<const v4i *>(t == 0 ? a.hop0 : a.hop_seq + (size_t)(t - 1) * a.hop_step) + hop_blk + lane;
    v4i hf[kSeqMaxPer];
#pragma unroll
    for (int u = 0; u < kSeqMaxPer; ++u)  // k steps past the wave's share meet zero weights: re-read a step that exists
      hf[u] = hp[(size_t)(k0 + u < k1 ? k0 + u : (k0 < KS ? k0 : 0)) * 64];
    v16i acc[3];
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[g][v] = 0;
#pragma unroll
    for (int u = 0; u < kSeqMaxPer; ++u)
#pragma unroll
      for (int g = 0; g < 3; ++g) acc[g] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Wr[g][u], hf[u], acc[g], 0, 0, 0);
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int v = 0; v < 16; ++v) part[(wave * 3 + g) * kPartTile + (2 * v + b2) * 33 + col] = acc[g][v];
    __syncthreads();

    // ---- the cell (as in gru_step_kernel), state in registers
    int32_t h84[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int32_t th[3];
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        const int o = g * kPartTile + (2 * (4 * (cg >> 1) + c) + (cg & 1)) * 33 + rsub;
        const int32_t sum = part[o] + part[o + 3 * kPartTile] + part[o + 6 * kPartTile] + part[o + 9 * kPartTile];
        th[g] = sat16(rescale(sum + bhe[g][c], a.Mh[g], a.rh[g]));
      }
      const int32_t r = sigmoid_from_table(sig_lds, sat16(txe[0][c] + th[0]));
      const int32_t u = sigmoid_from_table(sig_lds, sat16(txe[1][c] + th[1]));
      const int32_t rn = (r * th[2] + 16384) >> 15;
      const int32_t cand = tanh_from_table(a.tanh_tab, sat16(txe[2][c] + rn));
      const int32_t hn = cell_update32(cifg_input_gate(u), cand, u, h16r[c], 0);
      h16r[c] = n0 + c < N ? hn : 0;
      h84[c] = n0 + c < N ? state_i8(hn) : 0;
    }
    if (row_ok && n0 < N) {
      const uint32_t pk = (uint32_t)(h84[0] & 0xFF) | ((uint32_t)(h84[1] & 0xFF) << 8) | ((uint32_t)(h84[2] & 0xFF) << 16) |
                          ((uint32_t)(h84[3] & 0xFF) << 24);
      *reinterpret_cast<uint32_t *>(a.hop_seq + (size_t)t * a.hop_step + hop_offset(row, n0, KS)) = pk;
      *reinterpret_cast<uint32_t *>(a.h8_seq + ((size_t)t * a.B + row) * a.Kp + n0) = pk;
      if (a.y) {
        int8_t *yd = a.y + ((size_t)t * a.B + row) * N + n0;
        if (vec && !(reinterpret_cast<uintptr_t>(a.y) & 3))
          *reinterpret_cast<uint32_t *>(yd) = pk;
        else
          for (int c = 0; c < 4 && n0 + c < N; ++c) yd[c] = (int8_t)h84[c];
      }
    }
    // rows of the block past the batch are never written: their (garbage) state only ever feeds their own results
    if (!gru_group_sync(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, a.sync_sleep, flag)) return;
  }
  if (row_ok)
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (n0 + c < N) a.h16[(size_t)row * N + n0 + c] = (int16_t)h16r[c];
  placement_check();
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

}  // namespace lstm_int

using namespace lstm_int;

struct GruTimed {  // one timed stretch of launches of a forward call made while profiling
  hipEvent_t start, stop;
  int cls, launches;
};

struct gru_int_model {
  int device = -1;
  bool profiling = false;
  std::vector<GruTimed> timed;
  int persistent = 1;   // layers that fit run all their steps in one launch of gru_seq_kernel
  int spin_limit = 1 << 21, sync_sleep = 12;
  int extra_arrivals = 0;  // test hook (option "barrier_never_completes")
  int *status = nullptr;  // device word: nonzero once a wait inside gru_seq_kernel gave up (1) or placement failed (2)
  int num_cus = 0;
  std::vector<GruLayerHost> host;
  std::vector<GruLayerDev> dev;
  uint8_t *arena = nullptr;
  const uint16_t *sig_tab = nullptr, *tanh_tab = nullptr;
};

namespace {

// carve-up of the workspace for (T, B)
constexpr size_t kGruSyncBytes = 256 * 64 * 4;  // group counters [256][64 words]; the placement words lie inside

struct GruWs {
  size_t xpad, tx, out[2], hop[2], h16, sync, hop_seq, total;
};
GruWs gru_workspace(const gru_int_model *m, int64_t T, int64_t B) {
  GruWs w{};
  size_t off = 0, max_tx = 0, max_out = 0, max_hop = 0, sum_h16 = 0;
  for (const GruLayerHost &q : m->host) {
    const GruDims d = gru_dims(q.I, q.N);
    max_tx = std::max(max_tx, (size_t)T * B * 3 * q.N * 2);
    // the same terms in the register-resident input GEMM's tile order: rows padded to 32 per step, cells to 64, 4 gate slots
    max_tx = std::max(max_tx, (size_t)T * ((B + 31) / 32 * 32) * ((q.N + 63) / 64 * 64) * 4 * 2);
    max_out = std::max(max_out, ((size_t)T * B + 32) * d.Kp);  // 32 rows of slack: that GEMM reads whole blocks of 32 rows
    max_hop = std::max(max_hop, hop_bytes((int)B, d.Kp));
    sum_h16 = std::max(sum_h16, (size_t)B * q.N * 2);
  }
  const GruDims d0 = gru_dims(m->host[0].I, m->host[0].N);
  w.xpad = off; off += align256(((size_t)T * B + 32) * d0.Ip);
  w.tx = off; off += align256(max_tx);
  w.out[0] = off; off += align256(max_out);
  w.out[1] = off; off += align256(max_out);
  w.hop[0] = off; off += align256(max_hop);
  w.hop[1] = off; off += align256(max_hop);
  w.h16 = off; off += align256(sum_h16);
  w.sync = off; off += kGruSyncBytes;
  w.hop_seq = off; off += align256(max_hop * (size_t)T);  // the persistent kernel's exchange buffer: one copy per step
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
    const size_t o_sig = reserve(kTab * 2), o_tanh = reserve(kTab * 2), o_status = reserve(256);
    fill_sigmoid_table(3, reinterpret_cast<uint16_t *>(img.data() + o_sig));
    fill_tanh_table(3, reinterpret_cast<uint16_t *>(img.data() + o_tanh));
    struct Off { size_t W, bx, R, bh, W2f, bx2; int tiles; };
    std::vector<Off> offs(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      const GruLayerHost &q = m->host[l];
      const int I = q.I, N = q.N;
      const GruDims d = gru_dims(I, N);
      const int KS = d.Kp / 32;
      Off o;
      o.W = reserve((size_t)d.cols_pad * d.Ip);
      o.bx = reserve((size_t)d.cols_pad * 4);
      o.R = reserve((size_t)(d.Ncp / 32) * 3 * KS * 1024);
      o.bh = reserve((size_t)3 * d.Ncp * 4);
      o.tiles = 0;
      o.W2f = o.bx2 = 0;
      if (d.Ip <= 1024) {
        o.tiles = (N + 63) / 64 * 8;
        o.W2f = reserve((size_t)o.tiles * 32 * d.Ip);
        o.bx2 = reserve((size_t)o.tiles * 32 * 4);
        for (int g = 0; g < 3; ++g)
          for (int n = 0; n < N; ++n) {
            const int tile = n / 8, rho = 8 * (g + 1) + n % 8;
            const int8_t *w = q.Wq.data() + ((size_t)g * N + n) * I;
            for (int k = 0; k < I; ++k)
              img[o.W2f + ((((size_t)tile * (d.Ip / 32) + k / 32) * 64) + rho + 32 * ((k % 32) / 16)) * 16 + k % 16] = (uint8_t)w[k];
            reinterpret_cast<int32_t *>(img.data() + o.bx2)[tile * 32 + rho] = q.bx_fold[g * N + n];
          }
      }
      for (int r = 0; r < 3 * N; ++r) std::memcpy(img.data() + o.W + (size_t)r * d.Ip, q.Wq.data() + (size_t)r * I, I);
      std::memcpy(img.data() + o.bx, q.bx_fold.data(), (size_t)3 * N * 4);
      // first operand of the 32x32x32 MFMA: lane (row = lane % 32, half = lane / 32) holds, for k step ks, bytes
      // 32 ks + 16 half .. + 15 of weight row 32 ct + row of gate g (zero beyond N in either direction)
      for (int ct = 0; ct < d.Ncp / 32; ++ct)
        for (int g = 0; g < 3; ++g)
          for (int ks = 0; ks < KS; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
              const int n = ct * 32 + (lane & 31), k0 = ks * 32 + (lane >> 5) * 16;
              uint8_t *dst = img.data() + o.R + ((((size_t)ct * 3 + g) * KS + ks) * 64 + lane) * 16;
              if (n < N)
                for (int j = 0; j < 16 && k0 + j < N; ++j) dst[j] = (uint8_t)q.Rq[((size_t)g * N + n) * N + k0 + j];
            }
      for (int g = 0; g < 3; ++g)
        std::memcpy(img.data() + o.bh + (size_t)g * d.Ncp * 4, q.bhq.data() + (size_t)g * N, (size_t)N * 4);
      offs[l] = o;
    }
    if (hipSetDevice(device) != hipSuccess || in_gemm_init() != hipSuccess || gemm_init() != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void *>(&gru_seq_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kSeqSigBytes) != hipSuccess ||
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
    m->status = reinterpret_cast<int *>(m->arena + o_status);
    {
      hipDeviceProp_t prop;
      m->num_cus = hipGetDeviceProperties(&prop, device) == hipSuccess ? prop.multiProcessorCount : 0;
    }
    m->sig_tab = reinterpret_cast<const uint16_t *>(m->arena + o_sig);
    m->tanh_tab = reinterpret_cast<const uint16_t *>(m->arena + o_tanh);
    m->dev.resize(num_layers);
    for (int l = 0; l < num_layers; ++l) {
      m->dev[l].W = reinterpret_cast<const int8_t *>(m->arena + offs[l].W);
      m->dev[l].bx = reinterpret_cast<const int32_t *>(m->arena + offs[l].bx);
      m->dev[l].Rop = reinterpret_cast<const int8_t *>(m->arena + offs[l].R);
      m->dev[l].bh = reinterpret_cast<const int32_t *>(m->arena + offs[l].bh);
      if (offs[l].tiles) {
        m->dev[l].W2f = reinterpret_cast<const int8_t *>(m->arena + offs[l].W2f);
        m->dev[l].bx2 = reinterpret_cast<const int32_t *>(m->arena + offs[l].bx2);
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
    // (or, for the input GEMM that reads whole blocks of 32 rows, unless the batch is a multiple of 32: the copy has
    // 32 rows of slack behind it)
    if (d0.Ip != m->host[0].I || (reinterpret_cast<uintptr_t>(x) & 15) || (B & 31)) {
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
    int8_t *hop[2] = {reinterpret_cast<int8_t *>(ws + w.hop[0]), reinterpret_cast<int8_t *>(ws + w.hop[1])};
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
    gru_int_model *mm = const_cast<gru_int_model *>(m);  // the profile is bookkeeping beside the model
    auto timed_begin = [&](int cls, int launches) {
      if (!m->profiling) return;
      GruTimed e{nullptr, nullptr, cls, launches};
      if (hipEventCreate(&e.start) != hipSuccess || hipEventCreate(&e.stop) != hipSuccess) return;
      (void)hipEventRecord(e.start, s);
      mm->timed.push_back(e);
    };
    auto timed_end = [&]() {
      if (m->profiling && !mm->timed.empty()) (void)hipEventRecord(mm->timed.back().stop, s);
    };
    // One launch for all steps (gru_seq_kernel) where the layer fits: depth up to 1024 in registers, one workgroup
    // per tile of 32 cells and group of 32 rows, a group inside one XCD of 32 compute units, all groups resident.
    const int ctiles = d.Ncp / 32;
    const int groups = (B + 31) / 32;
    const bool seq = m->persistent && !tr && m->num_cus == 256 && d.Kp <= 128 * kSeqMaxPer && ctiles <= 32 &&
                     groups <= 8 * (32 / ctiles) && T < (1 << 20);
    // The input term: from the LSTM path's input GEMM where the input depth allows (weights resident in registers, depth
    // up to 1024, output in its tile order, which both recurrent kernels read); else, and with a trace, from the
    // general matmul, row-major.
    InGemmArgs ga{};
    ga.A = in; ga.a_slack = 1; ga.lda = ld_in; ga.T = T; ga.B = B; ga.Bp = (B + 31) / 32 * 32;
    ga.W2f = dv.W2f; ga.kpad = d.Ip; ga.tiles = dv.tiles; ga.bx2 = dv.bx2;
    ga.M[0] = 1 << 30; ga.r[0] = 33;  // the empty gate slot
    for (int g = 0; g < 3; ++g) {
      ga.M[g + 1] = q.Mx[g];
      ga.r[g + 1] = 31 - q.ex[g];
    }
    ga.tx2 = reinterpret_cast<int4 *>(ws + w.tx);
    // (on the launch-per-step path only where the matmul is large: the tile-ordered terms cost the step kernel
    // 0.5 us per step, measured, which 8192 rows and more of a faster matmul pay for)
    const bool ws_gemm = !tr && dv.W2f && m->num_cus == 256 && (seq || TB >= 8192) && in_gemm_ws_supported(ga);
    timed_begin(GRU_INT_K_INPUT_GEMM, 1);
    if (ws_gemm)
      launch_in_gemm_ws(s, ga, m->num_cus);
    else
      launch_gemm_i16(s, in, ld_in, (int)TB, dv.W, d.Ip, 3 * N, dv.bx, rq, tx, 3 * N);
    timed_end();
    {
      const int64_t n = (int64_t)B * d.Kp;  // the state before step 0 goes where step "-1" would have put it
      const int sync_vec = seq ? (int)(kGruSyncBytes / 16) : 0;
      const int64_t work = std::max<int64_t>(n, sync_vec);
      hipLaunchKernelGGL(gru_init_kernel, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, h16, B, N, d.Kp, hop[1],
                         h_state ? 0 : 1, reinterpret_cast<int4 *>(ws + w.sync), sync_vec);
    }
    if (seq) {
      GruSeqArgs q2{};
      q2.B = B; q2.N = N; q2.Kp = d.Kp; q2.KS32 = d.Kp / 32; q2.T = T;
      q2.GS = ctiles; q2.groups = groups;
      q2.hop0 = hop[1];
      q2.hop_seq = reinterpret_cast<int8_t *>(ws + w.hop_seq);
      q2.hop_step = hop_bytes(B, d.Kp);
      q2.Rop = dv.Rop; q2.bh = dv.bh; q2.h16 = h16; q2.h8_seq = out;
      q2.tx = ws_gemm ? nullptr : tx;
      q2.tx2 = ws_gemm ? ga.tx2 : nullptr;
      q2.tiles = dv.tiles; q2.bp_blocks = ga.Bp / 32;
      q2.y = l == L - 1 ? y : nullptr;
      for (int g = 0; g < 3; ++g) {
        q2.Mh[g] = q.Mh[g];
        q2.rh[g] = 31 - q.eh[g];
      }
      q2.sig_tab = m->sig_tab; q2.tanh_tab = m->tanh_tab;
      q2.counters = reinterpret_cast<unsigned *>(ws + w.sync);
      q2.tickets = reinterpret_cast<unsigned long long *>(q2.counters + 2);
      q2.status = m->status;
      q2.spin_limit = m->spin_limit; q2.sync_sleep = m->sync_sleep;
      q2.extra_arrivals = m->extra_arrivals;
      timed_begin(GRU_INT_K_STEP, T);
      hipLaunchKernelGGL(gru_seq_kernel, dim3((unsigned)(8 * ctiles * ((groups + 7) / 8))), dim3(256), kSeqSigBytes, s, q2);
      timed_end();
    } else {
    GruStepArgs a{};
    a.B = B; a.N = N; a.Kp = d.Kp; a.KS32 = d.Kp / 32;
    a.ctiles = d.Ncp / 32;
    a.Rop = dv.Rop; a.bh = dv.bh; a.h16 = h16;
    for (int g = 0; g < 3; ++g) {
      a.Mh[g] = q.Mh[g];
      a.rh[g] = 31 - q.eh[g];
    }
    a.sig_tab = m->sig_tab; a.tanh_tab = m->tanh_tab;
    // 32 rows per workgroup (RB = 1): at large batches two workgroups then share a compute unit and one's cell runs
    // under the other's matmul (measured at N = 2048, B = 256: 12.9 us per step against 13.3 with RB = 2)
    constexpr int rb = 1;
    a.rtn = (B + 32 * rb - 1) / (32 * rb);
    const dim3 grid((unsigned)(8 * a.rtn * ((a.ctiles + 7) / 8)));
    const size_t lds = (size_t)4 * rb * 3 * kPartTile * 4;
    timed_begin(GRU_INT_K_STEP, T);
    for (int t = 0; t < T; ++t) {
      const size_t tb = (size_t)t * B;
      a.hop_prev = hop[(t + 1) & 1];
      a.hop_out = hop[t & 1];
      a.tx = ws_gemm ? nullptr : tx + tb * 3 * N;
      a.tx2 = ws_gemm ? ga.tx2 + (size_t)t * (ga.Bp / 32) * dv.tiles * 128 : nullptr;
      a.tiles = dv.tiles;
      a.h8_out = out + tb * d.Kp;
      a.y = l == L - 1 ? y + tb * N : nullptr;
      a.tr_tx = tr && tr->tx ? tr->tx + tb * 3 * N : nullptr;
      a.tr_th = tr && tr->th ? tr->th + tb * 3 * N : nullptr;
      a.tr_act = tr && tr->act ? tr->act + tb * 3 * N : nullptr;
      a.tr_h16 = tr && tr->h16 ? tr->h16 + tb * N : nullptr;
      a.tr_h8 = tr && tr->h8 ? tr->h8 + tb * N : nullptr;
      hipLaunchKernelGGL(gru_step_kernel<rb>, grid, dim3(256), lds, s, a);
    }
    timed_end();
    }
    in = out;
    ld_in = d.Kp;
    h_off += (size_t)B * N;
  }
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

int gru_int_set_option(gru_int_model *m, const char *key, int64_t value) {
  if (!m || !key) return LSTM_INT_E_INVALID_ARG;
  if (!strcmp(key, "persistent")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->persistent = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "spin_limit")) {
    if (value < 1 || value > (1 << 30)) return LSTM_INT_E_INVALID_ARG;
    m->spin_limit = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "sync_sleep")) {
    if (value < 0 || value > 1024) return LSTM_INT_E_INVALID_ARG;
    m->sync_sleep = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "barrier_never_completes")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->extra_arrivals = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "reset_status")) {
    if (m->device < 0) return LSTM_INT_E_DEVICE;
    const int zero = 0;
    if (hipSetDevice(m->device) != hipSuccess || hipDeviceSynchronize() != hipSuccess ||
        hipMemcpy(m->status, &zero, sizeof(zero), hipMemcpyHostToDevice) != hipSuccess)
      return LSTM_INT_E_DEVICE;
    return LSTM_INT_OK;
  }
  return LSTM_INT_E_INVALID_ARG;
}

int gru_int_device_status(const gru_int_model *m, int32_t *status) {
  if (!m || !status) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  int v = 0;
  if (hipSetDevice(m->device) != hipSuccess || hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(&v, m->status, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess)
    return LSTM_INT_E_DEVICE;
  *status = v;
  return LSTM_INT_OK;
}

int gru_int_profile_begin(gru_int_model *m) {
  if (!m) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  for (GruTimed &e : m->timed) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  m->timed.clear();
  m->profiling = true;
  return LSTM_INT_OK;
}

int gru_int_profile_end(gru_int_model *m, int64_t launches[GRU_INT_K_COUNT], double total_ms[GRU_INT_K_COUNT]) {
  if (!m || !launches || !total_ms) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  m->profiling = false;
  for (int k = 0; k < GRU_INT_K_COUNT; ++k) {
    launches[k] = 0;
    total_ms[k] = 0.0;
  }
  int rc = LSTM_INT_OK;
  if (hipSetDevice(m->device) != hipSuccess) rc = LSTM_INT_E_DEVICE;
  for (GruTimed &e : m->timed) {
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

void gru_int_destroy(gru_int_model *m) {
  if (!m) return;
  for (GruTimed &e : m->timed) {
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
