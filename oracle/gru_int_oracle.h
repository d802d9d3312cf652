/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.
 *
 * Plain, slow, scalar CPU statement of an integer-only GRU assembled from the
 * building blocks of "On the quantization of recurrent neural networks"
 * (arXiv 2101.05453).  Sec. 7 of the paper names the GRU as a user of its
 * blocks and gives no recipe for it: PARITY UNPINNED by the paper.  The recipe
 * below is this build's reading; every step cites the block it takes.
 *
 * Float cell (the GRU with the reset gate applied to the recurrent product,
 * gate order r, u, n):
 *   r  = sigma(W_r x + bx_r + R_r h + bh_r)
 *   u  = sigma(W_u x + bx_u + R_u h + bh_u)
 *   n  = tanh (W_n x + bx_n + r . (R_n h + bh_n))
 *   h' = (1 - u) . n + u . h
 *
 * Integer cell:
 *   - x: asymmetric int8 with a nudged zero point (Sec. 3.2.4); W, R: symmetric
 *     int8 per gate tensor, +-127 (Sec. 3.2.4, Table 2); biases int32 at the
 *     scale of their accumulator (Sec. 3.2.4); the zero point of x folded into
 *     the input bias (Sec. 6).
 *   - The state h is recurrent through an elementwise path, like the LSTM's
 *     cell state, and is kept in 16 bits with a power-of-two scale for the same
 *     reason (Sec. 3.2.2): Q0.15, h in [-1, 1) by construction.  As a matmul
 *     operand (and as the layer's output) it is the int8 value
 *     h8 = sat8(rsh_r(h16, 8)): scale 2^-7, zero point 0.
 *   - Both matmul results are rescaled to Q3.12 and saturated to int16, and the
 *     gate sum saturates again (Sec. 3.2.4); sigma and tanh are the 16-bit
 *     functions of Sec. 3.2.1 (Q3.12 in, Q0.15 out).
 *   - r . th_n is a Q0.15 x Q3.12 product brought back to Q3.12 by a rounding
 *     shift of 15 (the elementwise-product rule of Sec. 3.2.7).
 *   - 1 - u is the coupling of Sec. 3.2.9: min(32768 - u, 32767).
 *   - h' = sat16(rsh_r((1-u) n, 15) + rsh_r(u h16, 15)): the cell update of
 *     Sec. 3.2.7 with both products Q0.30 -> Q0.15.
 *
 * Only the tests may use this library.  It shares no code with the HIP
 * library; it calls the primitives of lstm_int_oracle.c (rescale, rounding
 * shift, multiplier quantization, sigma, tanh), which have their own pins.
 */
#ifndef GRU_INT_ORACLE_H
#define GRU_INT_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* gate slots: r (reset), u (update), n (candidate) */
enum { ORC_GRU_R = 0, ORC_GRU_U = 1, ORC_GRU_N = 2 };

typedef struct {
  int32_t input_size, num_cells;
  const float *W[3];  /* [N, I] */
  const float *R[3];  /* [N, N] */
  const float *bx[3]; /* [N] input-side bias */
  const float *bh[3]; /* [N] recurrent-side bias (for n: inside the reset product) */
  float x_min, x_max; /* range of the layer input; ignored for layers > 0 */
} orc_gru_layer_params;

typedef struct {
  int32_t I, N;
  int32_t zp_x;
  double s_x, s_W[3], s_R[3];
  int32_t Mx[3], ex[3]; /* W x + bx -> Q3.12 */
  int32_t Mh[3], eh[3]; /* R h8 + bh -> Q3.12 */
  int8_t *Wq;       /* [3][N][I] */
  int8_t *Rq;       /* [3][N][N] */
  int32_t *bxq;     /* [3][N] at s_W s_x */
  int32_t *bhq;     /* [3][N] at s_R 2^-7 */
  int32_t *bx_fold; /* [3][N] bxq - zp_x sum_k Wq (Sec. 6) */
} orc_gru_layer_quant;

typedef struct {
  int32_t num_layers;
  orc_gru_layer_quant *layers;
} orc_gru_model;

int orc_gru_prepare(const orc_gru_layer_params *layers, int32_t num_layers, orc_gru_model **out);
void orc_gru_destroy(orc_gru_model *m);
const orc_gru_layer_quant *orc_gru_get_layer(const orc_gru_model *m, int32_t layer);

/* optional dumps of one layer; every pointer may be NULL */
typedef struct {
  int32_t layer;
  int16_t *tx;  /* [T,B,3,N] rescaled W x + bx */
  int16_t *th;  /* [T,B,3,N] rescaled R h8 + bh */
  int16_t *act; /* [T,B,3,N] r, u, n in Q0.15 */
  int16_t *h16; /* [T,B,N] state after the step */
  int8_t *h8;   /* [T,B,N] layer output */
} orc_gru_trace;

/* x: [T,B,I0] int8.  y: [T,B,N_last] int8 (scale 2^-7, zero point 0).
 * h_state: int16 Q0.15, layers concatenated, layer l is [B,N_l]; in/out;
 * NULL = zeros.  unfolded != 0 uses sum W (x - zp) + bxq (Sec. 6 identity). */
int orc_gru_forward(const orc_gru_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                    int16_t *h_state, const orc_gru_trace *trace, int unfolded, int threads);

/* the float cell above in double; y: [T,B,N_last] double (may be NULL) */
int orc_gru_float_forward(const orc_gru_layer_params *layers, int32_t num_layers, const float *x,
                          int32_t T, int32_t B, double *y, int threads);

#ifdef __cplusplus
}
#endif
#endif
