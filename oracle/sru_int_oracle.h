/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.
 *
 * Plain, slow, scalar CPU statement of an integer-only SRU (simple recurrent
 * unit) assembled from the building blocks of "On the quantization of
 * recurrent neural networks" (arXiv 2101.05453).  Sec. 7 of the paper names
 * the SRU as a user of its blocks and gives no recipe for it: PARITY UNPINNED
 * by the paper.  The recipe below is this build's reading; every step cites
 * the block it takes.
 *
 * Float cell (no recurrent matmul: the state enters the gates through two
 * weight vectors; slot order c = candidate, f = forget, r = reset, s = highway):
 *   xc = W_c x
 *   f  = sigma(W_f x + v_f . c + b_f)
 *   r  = sigma(W_r x + v_r . c + b_r)          (both gates read the old state)
 *   c' = f . c + (1 - f) . xc
 *   h  = r . c' + (1 - r) . s,   s = W_s x, or s = x when the layer has no W_s
 *                                (then input_size = num_cells)
 *
 * Integer cell:
 *   - x: asymmetric int8 with a nudged zero point (Sec. 3.2.4); every W:
 *     symmetric int8 per tensor, +-127 (Sec. 3.2.4, Table 2); b_f, b_r: int32
 *     at the scale of their accumulator (Sec. 3.2.4); the zero point of x
 *     folded into a per-row constant of every matmul (Sec. 6).
 *   - The state c recurs through an elementwise path and is kept in 16 bits
 *     with a power-of-two scale 2^(m-15), m from a measured magnitude
 *     (Sec. 3.2.2).  The candidate xc and the highway term s are convexly mixed
 *     with it, so they take the same format: c_absmax is the largest magnitude
 *     of c, xc and s seen in calibration.
 *   - W_c x and W_s x are rescaled to the state's format, W_f x + b_f and
 *     W_r x + b_r to Q3.12, all saturated to int16 (Sec. 3.2.4).  Without W_s
 *     the highway term is sat16(rescale(x_q - zp_x, s_x / 2^(m-15))).
 *   - v_f, v_r: symmetric int16, +-32767 (the peephole weights of Sec. 3.2.3);
 *     v . c is rescaled to Q3.12 and saturated, the gate sum saturates again,
 *     sigma is the 16-bit function of Sec. 3.2.1 (Q3.12 in, Q0.15 out).
 *   - 1 - f and 1 - r are the coupling of Sec. 3.2.9: min(32768 - g, 32767).
 *   - c' = sat16(rsh_r(f c, 15) + rsh_r((1-f) xc, 15)) and
 *     h16 = sat16(rsh_r(r c', 15) + rsh_r((1-r) s, 15)): the cell update of
 *     Sec. 3.2.7, both in the state's format.
 *   - The layer output is asymmetric int8 over the measured range of h
 *     (Sec. 3.2.8): y = sat8(rescale(h16, 2^(m-15) / s_h) + zp_h); a stacked
 *     layer reads it with (s_h, zp_h) as its input quantization.
 *
 * Only the tests may use this library.  It shares no code with the HIP
 * library; it calls the primitives of lstm_int_oracle.c (rescale, rounding
 * shift, multiplier quantization, sigma), which have their own pins.
 */
#ifndef SRU_INT_ORACLE_H
#define SRU_INT_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* matmul slots */
enum { ORC_SRU_C = 0, ORC_SRU_F = 1, ORC_SRU_R = 2, ORC_SRU_S = 3 };

typedef struct {
  int32_t input_size, num_cells;
  const float *W[4]; /* [N, I] c, f, r, s; W[3] may be NULL when I = N */
  const float *v[2]; /* [N] v_f, v_r */
  const float *b[2]; /* [N] b_f, b_r */
  float x_min, x_max; /* range of the layer input; ignored for layers > 0 */
  float c_absmax;     /* largest |c|, |W_c x|, |s| */
  float h_min, h_max; /* range of the layer output */
} orc_sru_layer_params;

typedef struct {
  int32_t I, N, G; /* G = 4 with W_s, 3 without */
  int32_t zp_x, zp_h, m_c;
  double s_x, s_h, s_W[4], s_v[2];
  int32_t Mx[4], ex[4]; /* matmul slot -> its int16 format */
  int32_t Mv[2], ev[2]; /* v . c -> Q3.12 */
  int32_t Ms, es;       /* (x_q - zp_x) -> the state's format (no W_s) */
  int32_t Mh, eh;       /* h16 -> output int8 */
  int8_t *Wq;           /* [G][N][I] */
  int16_t *vq;          /* [2][N] */
  int32_t *bq;          /* [G][N] at s_W s_x; zero rows for c and s */
  int32_t *b_fold;      /* [G][N] bq - zp_x sum_k Wq (Sec. 6) */
} orc_sru_layer_quant;

typedef struct {
  int32_t num_layers;
  orc_sru_layer_quant *layers;
} orc_sru_model;

int orc_sru_prepare(const orc_sru_layer_params *layers, int32_t num_layers, orc_sru_model **out);
void orc_sru_destroy(orc_sru_model *m);
const orc_sru_layer_quant *orc_sru_get_layer(const orc_sru_model *m, int32_t layer);

/* optional dumps of one layer; every pointer may be NULL */
typedef struct {
  int32_t layer;
  int16_t *tx;  /* [T,B,4,N] rescaled matmul slots (slot s: the highway term in either form) */
  int16_t *tv;  /* [T,B,2,N] rescaled v . c */
  int16_t *act; /* [T,B,2,N] f, r in Q0.15 */
  int16_t *c;   /* [T,B,N] state after the step */
  int16_t *h16; /* [T,B,N] output before its rescale */
  int8_t *y;    /* [T,B,N] layer output */
} orc_sru_trace;

/* x: [T,B,I0] int8.  y: [T,B,N_last] int8.  c_state: int16, layers
 * concatenated, layer l is [B,N_l]; in/out; NULL = zeros.  unfolded != 0 uses
 * sum W (x - zp) + bq (Sec. 6 identity). */
int orc_sru_forward(const orc_sru_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                    int16_t *c_state, const orc_sru_trace *trace, int unfolded, int threads);

/* what calibration logs per layer (Sec. 4) */
typedef struct {
  double c_absmax, h_min, h_max;
} orc_sru_stats;

/* the float cell above in double; y: [T,B,N_last] double (may be NULL);
 * stats: [num_layers] (may be NULL).  The fields c_absmax, h_min, h_max and
 * x_min, x_max of the parameters are not read. */
int orc_sru_float_forward(const orc_sru_layer_params *layers, int32_t num_layers, const float *x,
                          int32_t T, int32_t B, double *y, orc_sru_stats *stats, int threads);

#ifdef __cplusplus
}
#endif
#endif
