/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.
 *
 * Plain, slow, scalar CPU statement of the integer-only LSTM of
 * "On the quantization of recurrent neural networks" (arXiv 2101.05453):
 * the quantization recipe (Sec. 3, Table 2) and the integer execution of the
 * cell (Sec. 3.2.x, the integer-execution figures), plus the float LSTM of
 * Sec. 2 (eqs. 1-7) that the integer path approximates.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * use this library.  It shares no code with the HIP library: its structs,
 * constants and helpers are its own.
 *
 * Where the paper leaves a detail open (rounding mode, the representation of
 * an effective scale, the sigmoid/tanh algorithm, the sigma = 0 rule of layer
 * norm, ...) the choice made here is stated at the function that makes it.
 * Those choices are "parity unpinned" by the paper: the pins in the CPU test
 * suite fix them only through the error bands and identities the paper and
 * the mathematics give.
 */
#ifndef LSTM_INT_ORACLE_H
#define LSTM_INT_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* variant switches, Sec. 2 (last paragraph) */
#define ORC_CIFG 1u
#define ORC_PEEPHOLE 2u
#define ORC_LAYER_NORM 4u
#define ORC_PROJECTION 8u

/* gate slots, in the order of eqs. (1)-(5): i, f, z, o */
enum { ORC_GI = 0, ORC_GF = 1, ORC_GZ = 2, ORC_GO = 3 };

/* error codes */
enum {
  ORC_OK = 0,
  ORC_INVALID_ARG = -1,
  ORC_UNSUPPORTED = -2,
  ORC_BAD_RANGE = -3,
  ORC_NOMEM = -4
};

/* ------------------------------------------------------------------ */
/* Fixed-point primitives                                              */
/* ------------------------------------------------------------------ */

/* floor((n + floor(d/2)) / d), d > 0: division rounded to nearest, ties up. */
int64_t orc_rhu(int64_t n, int64_t d);
/* floor((a + 2^(k-1)) / 2^k), 1 <= k <= 62: rounding right shift, ties up. */
int64_t orc_rsh_r(int64_t a, int k);
/* rescale of Sec. 3.2.4-3.2.8 with the effective scale M * 2^(e-31):
 * sat32(floor(a*M / 2^(31-e) + 1/2)), a within int32, -31 <= e <= 30. */
int32_t orc_rescale(int64_t a, int32_t M, int e);
/* effective scale s > 0 -> (M, e), s ~= M * 2^(e-31), 2^30 <= M < 2^31.
 * Returns ORC_UNSUPPORTED if e falls outside [-31, 30]. */
int orc_quantize_multiplier(double s, int32_t *M, int *e);
/* floor(sqrt(v)), v >= 0 */
int64_t orc_isqrt(int64_t v);
/* exp(-y / 2^15) as Q0.31, y >= 0 */
int64_t orc_expneg(int64_t y);
/* Sec. 3.2.1: x in Q(m).(15-m) -> Q0.15, output clamped to [0, 32767] /
 * [-32768, 32767]. */
int32_t orc_int_sigmoid(int32_t x, int m);
int32_t orc_int_tanh(int32_t x, int m);
/* Sec. 3.2.6 integer layer norm of one row q[0..n-1]; out in Q3.12. */
int orc_int_layernorm(const int16_t *q, int n, const int16_t *qL,
                      const int32_t *qb, int32_t M_ln, int e_ln, int16_t *out);

/* ------------------------------------------------------------------ */
/* Prepare: float parameters + statistics -> integer model (Table 2)   */
/* ------------------------------------------------------------------ */

typedef struct {
  int32_t input_size, num_cells, output_size;
  uint32_t flags;
  const float *W[4];  /* [N, I]  i,f,z,o ; slot 0 NULL under CIFG */
  const float *R[4];  /* [N, H] */
  const float *b[4];  /* [N] */
  const float *P[3];  /* [N] i,f,o ; PEEPHOLE only */
  const float *Lw[4]; /* [N] ; LAYER_NORM only */
  const float *Wproj; /* [H, N] ; PROJECTION only */
  const float *bproj; /* [H] or NULL */
  float x_min, x_max, h_min, h_max, m_min, m_max;
  float c_absmax;
  float g_absmax[4];
} orc_layer_params;

typedef struct {
  int32_t I, N, H, G; /* G = 4, or 3 under CIFG */
  uint32_t flags;
  int32_t m_c; /* cell state is Q(m_c).(15-m_c) */
  int32_t zp_x, zp_h, zp_m;
  double s_x, s_h, s_m, s_c, s_Wp;
  double s_W[4], s_R[4], s_P[3], s_L[4], s_g[4];
  int32_t Mx[4], ex[4]; /* W x    -> gate scale */
  int32_t Mh[4], eh[4]; /* R h+b  -> gate scale */
  int32_t Mc[3], ec[3]; /* P.c    -> gate scale (i,f,o) */
  int32_t Mln[4], eln[4]; /* layer-norm second stage -> Q3.12 */
  int32_t Mm, em;       /* o.tanh(c) -> m */
  int32_t Mp, ep;       /* projection -> h */
  int8_t *Wq;   /* [4][N][I] */
  int8_t *Rq;   /* [4][N][H] */
  int32_t *qb;  /* [4][N] quantized gate bias */
  int16_t *Pq;  /* [3][N] */
  int16_t *Lq;  /* [4][N] */
  int8_t *Wpq;  /* [H][N] */
  int32_t *qbp; /* [H] */
  int32_t *bx_fold; /* [4][N]  -zp_x * sum_k Wq */
  int32_t *bh_fold; /* [4][N]  (no LN: qb) - zp_h * sum_k Rq */
  int32_t *bp_fold; /* [H]     qbp - zp_m * sum_n Wpq */
} orc_layer_quant;

typedef struct {
  int32_t num_layers;
  orc_layer_quant *layers;
} orc_model;

int orc_prepare(const orc_layer_params *layers, int32_t num_layers,
                orc_model **out);
void orc_destroy(orc_model *m);
const orc_layer_quant *orc_get_layer(const orc_model *m, int32_t layer);

/* ------------------------------------------------------------------ */
/* Integer forward                                                     */
/* ------------------------------------------------------------------ */

/* Optional per-(t, b) dumps of one layer; every pointer may be NULL.
 * Gate-indexed tensors always have 4 slots (i,f,z,o); under CIFG slot 0 of
 * tx/th/g/ln is left untouched and slot 0 of act holds the coupled i. */
typedef struct {
  int32_t layer;
  int16_t *tx;  /* [T,B,4,N] rescaled W x term */
  int16_t *th;  /* [T,B,4,N] rescaled R h (+b) term */
  int16_t *g;   /* [T,B,4,N] gate sum before layer norm / activation */
  int16_t *ln;  /* [T,B,4,N] layer-norm output, Q3.12 (LAYER_NORM only) */
  int16_t *act; /* [T,B,4,N] i,f,z,o after sigmoid/tanh, Q0.15 */
  int16_t *c;   /* [T,B,N] */
  int8_t *m;    /* [T,B,N] */
  int8_t *h;    /* [T,B,H] */
} orc_trace;

/* x: [T,B,I0] int8.  y: [T,B,H_last] int8.
 * h_state: layers concatenated, layer l is [B,H_l]; in/out; NULL = start
 * from real 0 (q = zp_h).  c_state: likewise [B,N_l] int16; NULL = zeros.
 * unfolded != 0 uses sum W (q - zp) + qb instead of the folded biases
 * (Sec. 6: the two are the same integers).
 * threads: OpenMP threads over batch rows (rows are independent). */
int orc_forward(const orc_model *m, const int8_t *x, int32_t T, int32_t B,
                int8_t *y, int8_t *h_state, int16_t *c_state,
                const orc_trace *trace, int unfolded, int threads);

/* ------------------------------------------------------------------ */
/* Float LSTM of Sec. 2 in double, with the "log" nodes of Sec. 4      */
/* ------------------------------------------------------------------ */

typedef struct {
  double x_min, x_max, h_min, h_max, m_min, m_max, c_absmax, g_absmax[4];
} orc_float_stats;

/* x: [T,B,I0] float.  y: [T,B,H_last] double (may be NULL).
 * stats: one entry per layer (may be NULL).  The calibration fields of the
 * layer params are ignored. */
int orc_float_forward(const orc_layer_params *layers, int32_t num_layers,
                      const float *x, int32_t T, int32_t B, double *y,
                      orc_float_stats *stats, int threads);

int orc_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif
