/*
 * sru_int -- integer-only SRU (simple recurrent unit) for AMD MI355X (gfx950),
 * in liblstm_int.so.
 *
 * arXiv 2101.05453, Sec. 7, names the SRU as a cell the paper's design
 * considerations and building blocks apply to, and gives no recipe for it.
 * This is the recipe built here, block by block from the LSTM's:
 *
 * Float cell (no recurrent matmul: the state enters the gates through two weight
 * vectors; matmul slots c = candidate, f = forget, r = reset, s = highway):
 *   xc = W_c x
 *   f  = sigma(W_f x + v_f . c + b_f)
 *   r  = sigma(W_r x + v_r . c + b_r)          (both gates read the old state)
 *   c' = f . c + (1 - f) . xc
 *   h  = r . c' + (1 - r) . s,   s = W_s x, or s = x for a layer without W_s
 *                                (then input_size = num_cells)
 *
 * Integer cell:
 *   x       int8, asymmetric, nudged zero point (Sec. 3.2.4); for layers > 0 the
 *           int8 output of the layer below with its (s_h, zp_h)
 *   W       int8, symmetric per tensor, +-127 (Sec. 3.2.4, Table 2); b_f, b_r int32
 *           at the scale of their accumulator; the zero point of x folded into a
 *           per-row constant of every matmul (Sec. 6)
 *   c       the state, int16 with the power-of-two scale 2^(m-15), m from the
 *           measured magnitude c_absmax of c, xc and s (Sec. 3.2.2): the three are
 *           mixed convexly and share the format
 *   tx_c, tx_s = sat16(rescale(W x + fold)) in the state's format; tx_f, tx_r in
 *           Q3.12 (Sec. 3.2.4); without W_s, tx_s = sat16(rescale(x_q - zp_x))
 *   v_f, v_r int16, symmetric, +-32767 (the peephole weights of Sec. 3.2.3);
 *           tv = sat16(rescale(v_q c)) in Q3.12
 *   f, r    = sigma16(sat16(tx + tv)) in Q0.15 (Sec. 3.2.1)
 *   1 - g   = min(32768 - g, 32767) (the coupling of Sec. 3.2.9)
 *   c'      = sat16(floor((f c + 2^14) / 2^15) + floor(((1-f) tx_c + 2^14) / 2^15))
 *   h16     = sat16(floor((r c' + 2^14) / 2^15) + floor(((1-r) tx_s + 2^14) / 2^15))
 *           (the cell update of Sec. 3.2.7, twice)
 *   y       = sat8(rescale(h16, 2^(m-15) / s_h) + zp_h): asymmetric int8 over the
 *           measured range of h (Sec. 3.2.8)
 *
 * Error codes are those of lstm_int.h.  All tensors are row-major and dense.
 */
#ifndef SRU_INT_H
#define SRU_INT_H

#include <stddef.h>
#include <stdint.h>

#include "lstm_int.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sru_int_model sru_int_model;

/* Float parameters and calibration statistics (Sec. 4) of one layer.  Every
 * pointer is HOST memory, caller-owned, read-only, and may be freed once
 * sru_int_prepare returns.  W[3] may be NULL when input_size = num_cells; the
 * others are non-NULL. */
typedef struct {
  int32_t input_size; /* I */
  int32_t num_cells;  /* N */
  const float *W[4];  /* [N, I] c, f, r, s */
  const float *v[2];  /* [N] v_f, v_r */
  const float *b[2];  /* [N] b_f, b_r */
  float x_min, x_max; /* range of the layer input; ignored for layers > 0 */
  float c_absmax;     /* largest |c|, |W_c x|, |s| */
  float h_min, h_max; /* range of the layer output h */
} sru_int_layer_params;

/* Host views of what prepare derived for one layer, valid until the model is
 * destroyed.  (M, e): effective scale M * 2^(e-31) as in lstm_int_layer_quant. */
typedef struct {
  int32_t I, N, G; /* G = 4 with W_s, 3 without */
  int32_t zp_x, zp_h, m_c;
  double s_x, s_h, s_W[4], s_v[2];
  int32_t Mx[4], ex[4];   /* matmul slot -> its int16 format */
  int32_t Mv[2], ev[2];   /* v c -> Q3.12 */
  int32_t Ms, es;         /* x_q - zp_x -> the state's format (G = 3) */
  int32_t Mh, eh;         /* h16 -> output int8 */
  const int8_t *Wq;       /* [G][N][I] */
  const int16_t *vq;      /* [2][N] */
  const int32_t *bq;      /* [G][N] at s_W s_x; zero for slots c and s */
  const int32_t *b_fold;  /* [G][N] bq - zp_x sum_k Wq (Sec. 6) */
} sru_int_layer_quant;

/* Optional dumps of one layer's intermediate tensors (DEVICE, caller-owned,
 * each may be NULL). */
typedef struct {
  int32_t layer;
  int16_t *tx;  /* [T,B,4,N] slot terms; slot s is the highway term in either form */
  int16_t *tv;  /* [T,B,2,N] */
  int16_t *act; /* [T,B,2,N] f, r in Q0.15 */
  int16_t *c;   /* [T,B,N] state after the step */
  int16_t *h16; /* [T,B,N] */
  int8_t *y;    /* [T,B,N] layer output */
} sru_int_trace;

/*
 * Offline phase: quantizes num_layers stacked layers (layer l + 1 reads layer
 * l's output; its input_size must equal layer l's num_cells) and, for
 * device >= 0, uploads the weights to that HIP device (device = -1: host-only
 * model).  LSTM_INT_E_INVALID_ARG: a missing tensor, no W_s with I != N.
 * LSTM_INT_E_UNSUPPORTED: I or N beyond 2^15 (Sec. 3.1.1), c_absmax beyond 2^8,
 * an effective scale outside [2^-32, 2^30), a folded constant so large that
 * constant + 128 * sum|w| leaves int32.  LSTM_INT_E_BAD_RANGE: min > max, a
 * negative c_absmax, NaN/Inf in a parameter.
 */
int sru_int_prepare(const sru_int_layer_params *layers, int32_t num_layers, int32_t device,
                    sru_int_model **out);

/* Fills *out with views into the model (no copy, no device access). */
int sru_int_get_quant(const sru_int_model *model, int32_t layer, sru_int_layer_quant *out);

/* Device bytes sru_int_forward needs for T steps of B rows (0 on error). */
size_t sru_int_workspace_bytes(const sru_int_model *model, int32_t T, int32_t B);

/*
 * Online phase: T steps over B rows through all layers, integer only.
 *   x        DEVICE int8 [T,B,I0], quantized with layer 0's (s_x, zp_x)
 *   y        DEVICE int8 [T,B,N_last], at the last layer's (s_h, zp_h)
 *   c_state  DEVICE int16, layers concatenated, layer l is [B,N_l] in its own
 *            format; read as the state before step 0 and overwritten with the
 *            state after step T - 1; NULL = start from zeros
 *   workspace DEVICE, >= sru_int_workspace_bytes(model,T,B), 256-byte aligned
 *   hip_stream a hipStream_t (NULL = the default stream)
 *   trace    NULL, or dumps of one layer
 * Per layer two launches: the four (three) matmul slots over all T*B rows as one
 * int8 MFMA matmul -- with the weights resident in registers and a tile-ordered
 * output where the input depth is at most 1024, the device has 256 compute
 * units and no trace of the layer is asked for; the general matmul, row-major,
 * otherwise -- and one scan kernel in which a thread carries four cells of one
 * batch row through all T steps, the terms of the steps ahead already requested.
 * Allocates nothing, never synchronizes the host, launches kernels only.
 * T = 0 or B = 0 is a no-op.  LSTM_INT_E_UNSUPPORTED: T * B * row length beyond
 * 2^31, or an elementwise scale (x to the state's format, v c to Q3.12, h16 to
 * the output) of 2^28 or more.
 */
int sru_int_forward(const sru_int_model *model, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                    int16_t *c_state, void *workspace, size_t workspace_bytes, void *hip_stream,
                    const sru_int_trace *trace);

/* Option "register_gemm": 1 (default) = the register-resident matmul where it
 * applies, 0 = always the general one.  Results never depend on it.  Unknown
 * keys or values give LSTM_INT_E_INVALID_ARG. */
int sru_int_set_option(sru_int_model *model, const char *key, int64_t value);

/*
 * Device time of the forward calls made while profiling is on, measured with
 * HIP events on the stream the kernels run on, per kernel class: the matmul and
 * the scan (one launch each per layer and call).  sru_int_profile_begin resets
 * the record; sru_int_profile_end waits for the recorded work, fills launches[k]
 * and total_ms[k] and destroys the events.  Profiling adds host work to forward
 * and is not meant for calls under graph capture.
 */
#define SRU_INT_K_INPUT_GEMM 0
#define SRU_INT_K_SCAN 1
#define SRU_INT_K_COUNT 2
int sru_int_profile_begin(sru_int_model *model);
int sru_int_profile_end(sru_int_model *model, int64_t launches[SRU_INT_K_COUNT],
                        double total_ms[SRU_INT_K_COUNT]);

void sru_int_destroy(sru_int_model *model);

#ifdef __cplusplus
}
#endif
#endif
