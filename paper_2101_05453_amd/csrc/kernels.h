// Launch interface of the HIP kernels of liblstm_int (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lstm_int {

// Requantization applied to an int32 accumulator column n:
//   v = acc + bias[n];  gate = number of multiples of cols_per_gate below n;
//   out = sat(rescale(v, M[gate], r[gate])) (+ zp for int8 outputs)
struct Requant {
  int32_t M[4];
  int32_t r[4];  // right shift 31 - e, 1..62
  int32_t cols_per_gate;
  int32_t zp;
  int32_t all_hi;  // every r >= 33: the high-word form of rescale applies
};

// allows the matmul's large tile its 128 KB of LDS; call with the device current before the first launch
hipError_t gemm_init();

// out = requant(A [M, lda] . W^T [ncols, kpad]) as int16 [M, ldc]
//   A: int8 activations, rows readable for kpad bytes (kpad % 64 == 0)
//   W: int8 weights, row-major [ncols_pad, kpad], ncols_pad % 128 == 0,
//      zero beyond the real extents; bias int32 [ncols_pad]
void launch_gemm_i16(hipStream_t s, const int8_t *A, int lda, int M, const int8_t *W, int kpad,
                     int ncols, const int32_t *bias, const Requant &rq, int16_t *out, int ldc);
// same, int8 output with zero point; out2 (may be NULL) receives a copy
void launch_gemm_i8(hipStream_t s, const int8_t *A, int lda, int M, const int8_t *W, int kpad,
                    int ncols, const int32_t *bias, const Requant &rq, int8_t *out, int ldc,
                    int8_t *out2, int ldc2);

// Everything of one step after the two gate matmuls, for every batch row:
// gate sum (Secs. 3.2.4/3.2.5), layer norm (3.2.6), sigma/tanh (3.2.1), CIFG
// (3.2.9), cell update and hidden state (3.2.7).
struct CellArgs {
  int32_t B, N, G, flags, m_c;
  double inv_n;       // 1.0 / N
  const int16_t *tx;  // [B, G*N] of this step
  const int16_t *th;  // [B, G*N]
  int16_t *c;         // [B, N] in/out
  const int16_t *Pq;  // [3, N]
  const int16_t *Lq;  // [4, N]
  const int32_t *qb;  // [4, N]
  int32_t Mc[3], rc[3];
  int32_t Mln[4], rln[4];
  int32_t Mm, rm, zp_m;
  const uint16_t *sig_tab, *tanh_tab, *tanhc_tab;  // [32769] each
  int8_t *m_out;
  int32_t ld_m;  // [B, ld_m]
  int8_t *m_out2;
  int32_t ld_m2;  // optional second copy (NULL to skip)
  // optional dumps of this step, [B,4,N] / [B,N]; NULL to skip
  int16_t *tr_g, *tr_ln, *tr_act, *tr_c;
  int8_t *tr_m;
};
void launch_cell(hipStream_t s, const CellArgs &a);

// dst [rows, ld_dst] <- src [rows, ld_src], first `cols` bytes of each row;
// bytes cols..ld_dst-1 of dst are set to `fill`.
void launch_copy_rows_i8(hipStream_t s, const int8_t *src, int ld_src, int8_t *dst, int ld_dst,
                         int rows, int cols, int fill);
// dst [rows, ld_dst] columns [0, cols) <- src [rows, cols] (dense); other columns of dst are left alone
void launch_place_cols_i8(hipStream_t s, const int8_t *src, int8_t *dst, int ld_dst, int64_t rows, int cols);
// dst [T*B, ld_dst] row (t, b) <- src row (T - 1 - t, b), first cols bytes; `fill` for the rest
void launch_flip_rows_i8(hipStream_t s, const int8_t *src, int ld_src, int8_t *dst, int ld_dst, int T, int B,
                         int cols, int fill);
// dst [rows, ld_dst] <- value for the first cols bytes, `fill` for the rest
void launch_fill_rows_i8(hipStream_t s, int8_t *dst, int ld_dst, int rows, int cols, int value,
                         int fill);
// h0 [rows, ld_h0] <- h_src [rows, ld_src] (first cols bytes; NULL: all zp), padding bytes 0; and
// sync_bytes (a multiple of 16) of zeros at sync;
// and, if c_dst is not NULL, c_dst [rows, c_cols] <- c_src [rows, c_ld_src] -- one launch
void launch_init_layer(hipStream_t s, const int8_t *h_src, int ld_src, int8_t *h0, int ld_h0, int rows, int cols,
                       int zp, void *sync, int64_t sync_bytes, const int8_t *c_src, int c_ld_src, int8_t *c_dst,
                       int c_cols);
void launch_copy_i16(hipStream_t s, const int16_t *src, int16_t *dst, int64_t n);
void launch_fill_i16(hipStream_t s, int16_t *dst, int64_t n, int value);
// q[i] = clamp(floor(x[i] / scale + 1/2) + zp, -128, 127), computed in double (Sec. 3.2.4)
void launch_quantize_input(hipStream_t s, const float *x, int8_t *q, int64_t n, double scale, int zp);
// dump [rows, G*N] (present gates) into [rows, 4, N] gate slots first..3
void launch_scatter_gates(hipStream_t s, const int16_t *src, int16_t *dst, int rows, int G, int N);

}  // namespace lstm_int
