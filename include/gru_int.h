/*
 * gru_int -- integer-only GRU for AMD MI355X (gfx950), in liblstm_int.so.
 *
 * arXiv 2101.05453, Sec. 7, names the GRU as a cell the paper's design
 * considerations and building blocks apply to, and gives no recipe for it.
 * This is the recipe built here, block by block from the LSTM's:
 *
 * Float cell (gate order r = reset, u = update, n = candidate; the reset gate
 * multiplies the recurrent product, so that one recurrent matmul serves all
 * three gates):
 *   r  = sigma(W_r x + bx_r + R_r h + bh_r)
 *   u  = sigma(W_u x + bx_u + R_u h + bh_u)
 *   n  = tanh (W_n x + bx_n + r . (R_n h + bh_n))
 *   h' = (1 - u) . n + u . h
 *
 * Integer cell:
 *   x      int8, asymmetric, nudged zero point (Sec. 3.2.4); for layers > 0 the
 *          int8 form of the state of the layer below
 *   W, R   int8, symmetric per gate tensor, +-127 (Sec. 3.2.4, Table 2)
 *   bx, bh int32 at the scale of the accumulator they join (Sec. 3.2.4); the
 *          zero point of x folded into bx (Sec. 6)
 *   h16    the state, int16 Q0.15: it recurs through an elementwise path like
 *          the LSTM's cell state and is kept in 16 bits with a power-of-two
 *          scale for the same reason (Sec. 3.2.2); |h| < 1 by construction
 *   h8     = sat8(floor((h16 + 128) / 256)): the state as matmul operand and as
 *          layer output, int8 with scale 2^-7 and zero point 0
 *   tx_g   = sat16(rescale(W_g x + bx'_g)), th_g = sat16(rescale(R_g h8 + bh_g)),
 *          both Q3.12 (Sec. 3.2.4)
 *   r, u   = sigma16(sat16(tx + th)) in Q0.15 (Sec. 3.2.1)
 *   n      = tanh16(sat16(tx_n + floor((r th_n + 2^14) / 2^15)))
 *   1 - u  = min(32768 - u, 32767) (the coupling of Sec. 3.2.9)
 *   h16'   = sat16(floor(((1-u) n + 2^14) / 2^15) + floor((u h16 + 2^14) / 2^15))
 *          (the cell update of Sec. 3.2.7)
 * No statistics other than the range of the first layer's input are needed:
 * every other format is fixed.
 *
 * Error codes are those of lstm_int.h.  All tensors are row-major and dense.
 */
#ifndef GRU_INT_H
#define GRU_INT_H

#include <stddef.h>
#include <stdint.h>

#include "lstm_int.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gru_int_model gru_int_model;

/* Float parameters of one layer.  Every pointer is HOST memory, caller-owned,
 * read-only, non-NULL, and may be freed once gru_int_prepare returns. */
typedef struct {
  int32_t input_size; /* I */
  int32_t num_cells;  /* N */
  const float *W[3];  /* [N, I] r, u, n */
  const float *R[3];  /* [N, N] */
  const float *bx[3]; /* [N] input-side bias */
  const float *bh[3]; /* [N] recurrent-side bias; for n inside the reset product */
  float x_min, x_max; /* range of the layer input; ignored for layers > 0 */
} gru_int_layer_params;

/* Host views of what prepare derived for one layer, valid until the model is
 * destroyed.  (M, e): effective scale M * 2^(e-31) as in lstm_int_layer_quant. */
typedef struct {
  int32_t I, N;
  int32_t zp_x;
  double s_x, s_W[3], s_R[3];
  int32_t Mx[3], ex[3];   /* W x + bx -> Q3.12 */
  int32_t Mh[3], eh[3];   /* R h8 + bh -> Q3.12 */
  const int8_t *Wq;       /* [3][N][I] */
  const int8_t *Rq;       /* [3][N][N] */
  const int32_t *bxq;     /* [3][N] at s_W s_x */
  const int32_t *bhq;     /* [3][N] at s_R 2^-7 */
  const int32_t *bx_fold; /* [3][N] bxq - zp_x sum_k Wq (Sec. 6) */
} gru_int_layer_quant;

/* Optional dumps of one layer's intermediate tensors (DEVICE, caller-owned,
 * each may be NULL). */
typedef struct {
  int32_t layer;
  int16_t *tx;  /* [T,B,3,N] */
  int16_t *th;  /* [T,B,3,N] */
  int16_t *act; /* [T,B,3,N] r, u, n in Q0.15 */
  int16_t *h16; /* [T,B,N] state after the step */
  int8_t *h8;   /* [T,B,N] layer output */
} gru_int_trace;

/*
 * Offline phase: quantizes num_layers stacked layers (layer l + 1 reads layer
 * l's h8; its input_size must equal layer l's num_cells) and, for device >= 0,
 * uploads the weights to that HIP device (device = -1: host-only model).
 * LSTM_INT_E_UNSUPPORTED: I or N beyond 2^15 (Sec. 3.1.1), an effective scale
 * outside [2^-32, 2^30), a bias so large that bias + 128 * sum|w| leaves int32.
 * LSTM_INT_E_BAD_RANGE: x_min > x_max, NaN/Inf in a parameter.
 */
int gru_int_prepare(const gru_int_layer_params *layers, int32_t num_layers, int32_t device,
                    gru_int_model **out);

/* Fills *out with views into the model (no copy, no device access). */
int gru_int_get_quant(const gru_int_model *model, int32_t layer, gru_int_layer_quant *out);

/* Device bytes gru_int_forward needs for T steps of B rows (0 on error). */
size_t gru_int_workspace_bytes(const gru_int_model *model, int32_t T, int32_t B);

/*
 * Online phase: T steps over B rows through all layers, integer only.
 *   x        DEVICE int8 [T,B,I0], quantized with layer 0's (s_x, zp_x)
 *   y        DEVICE int8 [T,B,N_last]: h8 of the last layer
 *   h_state  DEVICE int16 Q0.15, layers concatenated, layer l is [B,N_l]; read
 *            as the state before step 0 and overwritten with the state after
 *            step T - 1; NULL = start from zeros
 *   workspace DEVICE, >= gru_int_workspace_bytes(model,T,B), 256-byte aligned
 *   hip_stream a hipStream_t (NULL = the default stream)
 *   trace    NULL, or dumps of one layer
 * Per layer: W x + bx over all T*B rows as one int8 MFMA matmul, then R h8 + bh
 * of the three gates fused with the whole elementwise cell -- as ONE persistent
 * launch for all T steps where the layer fits (N <= 1024, batches of up to
 * 256 * (32 / ceil(N / 32)) rows, no trace of that layer: the recurrent weights
 * stay in registers and the workgroups that share 32 batch rows meet at one
 * barrier per step inside one XCD), else as one launch per step.  Allocates
 * nothing, never synchronizes the host, launches kernels only.
 * The persistent launch needs all its workgroups on the device at once (one
 * per compute unit): nothing else may occupy the device for long while it
 * runs; if that does not hold its bounded waits give up, the call's outputs
 * are not valid and gru_int_device_status reports it.
 * T = 0 or B = 0 is a no-op.
 */
int gru_int_forward(const gru_int_model *model, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                    int16_t *h_state, void *workspace, size_t workspace_bytes, void *hip_stream,
                    const gru_int_trace *trace);

/*
 * Options: "persistent" 1 (default) / 0 = never the one-launch form;
 * "spin_limit" = polls after which a wait inside the persistent kernel gives
 * up; "sync_sleep" = pause before the first poll of a barrier, in units of 64
 * clocks; "barrier_never_completes" 1 = test hook: every barrier waits for an
 * arrival that never comes (keep spin_limit small); "reset_status" clears the
 * status word (synchronizes the device).  Results never depend on the tuning
 * options.  Unknown keys or values give LSTM_INT_E_INVALID_ARG.
 */
int gru_int_set_option(gru_int_model *model, const char *key, int64_t value);

/*
 * Blocking read of the model's device status word: 0 = every persistent launch
 * so far ran to completion; 1 = a wait gave up; 2 = the workgroups of a group
 * were not placed on one XCD; nonzero means the outputs of that call are not
 * valid.  The word is sticky.  Synchronizes the device.
 */
int gru_int_device_status(const gru_int_model *model, int32_t *status);

/*
 * Device time of the forward calls made while profiling is on, measured with
 * HIP events on the stream the kernels run on, per kernel class: the hoisted
 * input matmul (one launch per layer and call) and the recurrent part (the T
 * steps of a layer timed as one stretch -- T launches with their gaps, or the
 * one persistent launch -- and counted as T).  gru_int_profile_begin resets the
 * record; gru_int_profile_end waits for the recorded work, fills launches[k]
 * and total_ms[k] and destroys the events.  Profiling adds host work to
 * forward and is not meant for calls under graph capture.
 */
#define GRU_INT_K_INPUT_GEMM 0
#define GRU_INT_K_STEP 1
#define GRU_INT_K_COUNT 2
int gru_int_profile_begin(gru_int_model *model);
int gru_int_profile_end(gru_int_model *model, int64_t launches[GRU_INT_K_COUNT],
                        double total_ms[GRU_INT_K_COUNT]);

void gru_int_destroy(gru_int_model *model);

#ifdef __cplusplus
}
#endif
#endif
