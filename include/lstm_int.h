/*
 * lstm_int -- integer-only LSTM (arXiv 2101.05453) for AMD MI355X (gfx950).
 *
 * C ABI of the shared library liblstm_int.so.  Two phases, as in the paper:
 *   offline  (Secs. 3.2-3.3, Table 2, Sec. 6): float parameters + collected
 *            statistics -> integer model            -> lstm_int_prepare
 *   online   (Secs. 3.2.4-3.2.9, integer-execution figures): int8 in, int8
 *            out, no floating-point operation on the path -> lstm_int_forward
 *
 * Notation: T timesteps, B batch rows, L layers, I layer input width, N cells,
 * H layer output width (H = N unless PROJECTION), gate order i, f, z, o as in
 * eqs. (1)-(5) of Sec. 2.  All tensors are row-major and dense.
 *
 * Every function returns 0 on success or a negative LSTM_INT_E_* code; no
 * exception crosses this boundary and the library keeps no global state
 * besides the models it hands out.
 */
#ifndef LSTM_INT_H
#define LSTM_INT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Variant switches, Sec. 2 (last paragraph) and the columns of Table 2. */
#define LSTM_INT_CIFG 1u        /* i = 1 - f; the i-gate tensors are absent   */
#define LSTM_INT_PEEPHOLE 2u    /* P . c terms on gates i, f (c^{t-1}), o (c^t) */
#define LSTM_INT_LAYER_NORM 4u  /* norm() . L + b on every gate               */
#define LSTM_INT_PROJECTION 8u  /* h = W_proj m + b_proj                      */

#define LSTM_INT_OK 0
#define LSTM_INT_E_INVALID_ARG (-1)  /* NULL, shape or flag inconsistency       */
#define LSTM_INT_E_UNSUPPORTED (-2)  /* outside the limits stated at prepare    */
#define LSTM_INT_E_BAD_RANGE (-3)    /* min > max, NaN/Inf in a parameter       */
#define LSTM_INT_E_OUT_OF_MEMORY (-4)
#define LSTM_INT_E_DEVICE (-5)       /* HIP error, or host-only model           */
#define LSTM_INT_E_WORKSPACE (-6)    /* workspace too small or misaligned       */

typedef struct lstm_int_model lstm_int_model;

/*
 * Float parameters of one layer (eqs. 1-7) and the statistics of a
 * calibration run (Sec. 4).  Every pointer is HOST memory, caller-owned,
 * read-only, and may be freed once lstm_int_prepare returns.
 * Under CIFG index 0 of W, R, b, P, Lw must be NULL (the dagger rows of
 * Table 2); P only with PEEPHOLE; Lw only with LAYER_NORM; Wproj only with
 * PROJECTION (bproj may be NULL = zeros).
 */
typedef struct {
  int32_t input_size;  /* I */
  int32_t num_cells;   /* N */
  int32_t output_size; /* H; must equal N without PROJECTION */
  uint32_t flags;
  const float *W[4];  /* [N, I] input weights, i,f,z,o */
  const float *R[4];  /* [N, H] recurrent weights */
  const float *b[4];  /* [N] gate bias (applied after norm() with LAYER_NORM) */
  const float *P[3];  /* [N] peephole weights, i,f,o */
  const float *Lw[4]; /* [N] layer-norm weights */
  const float *Wproj; /* [H, N] */
  const float *bproj; /* [H] */
  float x_min, x_max; /* range of the layer input; ignored for layers > 0,  */
                      /* which take the previous layer's h quantization     */
  float h_min, h_max; /* range of the layer output h */
  float m_min, m_max; /* range of the hidden state m (PROJECTION only) */
  float c_absmax;     /* max |c|; extended to a power of two (Sec. 3.2.2) */
  float g_absmax[4];  /* max |W x + R h + P.c| per gate (LAYER_NORM only) */
} lstm_int_layer_params;

/*
 * Host views of everything prepare derived for one layer, valid until the
 * model is destroyed.  Gate-indexed arrays have 4 slots (i,f,z,o); slot 0 is
 * zero under CIFG.  An effective scale s is held as (M, e), s ~= M * 2^(e-31)
 * with 2^30 <= M < 2^31, and applied as
 *   rescale(a) = sat32(floor(a * M / 2^(31-e) + 1/2)).
 */
typedef struct {
  int32_t I, N, H, G; /* G = 4, or 3 under CIFG */
  uint32_t flags;
  int32_t m_c; /* the cell state is Q(m_c).(15 - m_c) */
  int32_t zp_x, zp_h, zp_m; /* real = s * (q - zp) */
  double s_x, s_h, s_m, s_c, s_Wp;
  double s_W[4], s_R[4], s_P[3], s_L[4], s_g[4];
  int32_t Mx[4], ex[4];   /* W x     -> gate scale (Sec. 3.2.4 / 3.2.5) */
  int32_t Mh[4], eh[4];   /* R h + b -> gate scale */
  int32_t Mc[3], ec[3];   /* P . c   -> gate scale; i, f, o */
  int32_t Mln[4], eln[4]; /* layer norm, second stage -> Q3.12 (Sec. 3.2.6) */
  int32_t Mm, em;         /* o . tanh(c) -> m (Sec. 3.2.7) */
  int32_t Mp, ep;         /* projection -> h (Sec. 3.2.8) */
  const int8_t *Wq;       /* [4][N][I] */
  const int8_t *Rq;       /* [4][N][H] */
  const int32_t *qb;      /* [4][N] */
  const int16_t *Pq;      /* [3][N] */
  const int16_t *Lq;      /* [4][N] */
  const int8_t *Wpq;      /* [H][N]; NULL without PROJECTION */
  const int32_t *qbp;     /* [H];    NULL without PROJECTION */
  const int32_t *bx_fold; /* [4][N]  -zp_x * sum_k Wq            (Sec. 6) */
  const int32_t *bh_fold; /* [4][N]  (no LN: qb) - zp_h * sum_k Rq        */
  const int32_t *bp_fold; /* [H]     qbp - zp_m * sum_n Wpq; NULL w/o proj */
} lstm_int_layer_quant;

/*
 * Optional dumps of one layer's intermediate integer tensors, for parity
 * checks.  DEVICE pointers, caller-owned, each may be NULL.  Gate-indexed
 * tensors have 4 slots; under CIFG slot 0 of tx/th/g/ln is not written and
 * slot 0 of act holds the coupled input gate.
 */
typedef struct {
  int32_t layer;
  int16_t *tx;  /* [T,B,4,N] rescaled W x term            */
  int16_t *th;  /* [T,B,4,N] rescaled R h (+ b) term      */
  int16_t *g;   /* [T,B,4,N] gate sum (Secs. 3.2.4/3.2.5) */
  int16_t *ln;  /* [T,B,4,N] layer-norm output, Q3.12     */
  int16_t *act; /* [T,B,4,N] i,f,z,o after sigma/tanh, Q0.15 */
  int16_t *c;   /* [T,B,N] cell state after the step      */
  int8_t *m;    /* [T,B,N] hidden state                    */
  int8_t *h;    /* [T,B,H] layer output                    */
} lstm_int_trace;

/*
 * Offline phase (Table 2; Secs. 3.2.1-3.2.9; Sec. 6).  Quantizes the float
 * parameters of num_layers stacked layers (layer l+1 reads layer l's h with
 * its scale and zero point), derives every effective scale as (M, e), folds
 * the zero points into the biases, and -- for device >= 0 -- uploads the
 * packed weights to that HIP device.  device = -1 builds a host-only model
 * (lstm_int_get_quant works, lstm_int_forward returns LSTM_INT_E_DEVICE).
 * Limits (LSTM_INT_E_UNSUPPORTED): I, N, H <= 2^15 (safe accumulation depth,
 * Sec. 3.1.1); N <= 4096 with LAYER_NORM; c_absmax <= 256; an effective scale
 * outside [2^-32, 2^30); a bias so large that bias + 128 * sum|w| leaves
 * int32.  On success *out owns host and device memory until
 * lstm_int_destroy.
 */
int lstm_int_prepare(const lstm_int_layer_params *layers, int32_t num_layers,
                     int32_t device, lstm_int_model **out);

/*
 * Statistics of a calibration run for one layer (Sec. 4, post-training): the
 * values lstm_int_layer_params carries as x_min .. g_absmax, in double.
 */
typedef struct {
  double x_min, x_max, h_min, h_max, m_min, m_max, c_absmax, g_absmax[4];
} lstm_int_layer_stats;

/*
 * Collects those statistics on the GPU (Sec. 4: the float model runs over
 * representative inputs and ranges are logged at the nodes the execution
 * figures mark "log").  Runs the float LSTM of Sec. 2 -- eqs. (1)-(7) with the
 * variants of `flags`, h^0 = c^0 = 0 -- in double precision over
 * x (DEVICE, float32 [T,B,I0]) for num_layers stacked layers whose float
 * parameters are given as for lstm_int_prepare (HOST; the statistics fields
 * of `layers` are ignored), and writes one lstm_int_layer_stats per layer to
 * stats (HOST, caller-owned): min/max of the layer input, of h and of m,
 * max |c|, and with LAYER_NORM max |W x + R h + P.c| per gate (else 0).
 * y_float (DEVICE, double [T,B,H_last], may be NULL) receives the float
 * output of the last layer.  Offline tooling: allocates and frees device
 * memory, copies the parameters, and returns after the stream has drained.
 * T*B*4*N and T*B*I must stay below 2^31 (LSTM_INT_E_UNSUPPORTED).
 */
int lstm_int_calibrate(const lstm_int_layer_params *layers, int32_t num_layers,
                       int32_t device, const float *x, int32_t T, int32_t B,
                       void *hip_stream, lstm_int_layer_stats *stats,
                       double *y_float);

/* Fills *out with views into the model (no copy, no device access). */
int lstm_int_get_quant(const lstm_int_model *model, int32_t layer,
                       lstm_int_layer_quant *out);

/*
 * The feature quantizer upstream of the first layer (Sec. 3.2.4: asymmetric
 * int8 activations with a nudged zero point): for n float32 values x (DEVICE)
 *   xq[i] = clamp(floor(x[i] / s_x + 1/2) + zp_x, -128, 127)
 * with layer 0's (s_x, zp_x), evaluated in double precision; xq is DEVICE
 * int8 [n], caller-owned.  Asynchronous on hip_stream, allocates nothing.
 * A NaN input gives code 0.
 */
int lstm_int_quantize_input(const lstm_int_model *model, const float *x, int64_t n,
                            int8_t *xq, void *hip_stream);

/* Device bytes lstm_int_forward needs for T steps of B rows (0 on error). */
size_t lstm_int_workspace_bytes(const lstm_int_model *model, int32_t T, int32_t B);

/*
 * Online phase: T steps over B rows through all layers (the time loop and
 * layer stack of Sec. 7 around the cell of Secs. 3.2.4-3.2.9).
 *   x        DEVICE int8 [T,B,I0], quantized with layer 0's (s_x, zp_x)
 *   y        DEVICE int8 [T,B,H_last], with the last layer's (s_h, zp_h)
 *   h_state  DEVICE int8, layers concatenated, layer l is [B,H_l]; read as
 *            h^{-1} and overwritten with h^{T-1}; NULL = start from real 0
 *   c_state  DEVICE int16, likewise [B,N_l]; NULL = zeros
 *   workspace DEVICE, >= lstm_int_workspace_bytes(model,T,B), 256-byte aligned
 *   hip_stream a hipStream_t (NULL = the default stream)
 *   trace    NULL, or dumps of one layer
 * Allocates nothing, never synchronizes the host: all work is enqueued on
 * hip_stream and touches only y, the state buffers, workspace and trace; it
 * launches kernels only (no memset or copy nodes), so a caller may capture it
 * in a HIP graph once one call has run outside a capture (and while no
 * profile is being recorded).
 * T = 0 or B = 0 is a no-op.  Calls sharing a model must not overlap in time
 * unless they use different workspaces and the same stream order.
 */
int lstm_int_forward(const lstm_int_model *model, const int8_t *x, int32_t T,
                     int32_t B, int8_t *y, int8_t *h_state, int16_t *c_state,
                     void *workspace, size_t workspace_bytes, void *hip_stream,
                     const lstm_int_trace *trace);

/*
 * lstm_int_forward for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops with
 * small T and B (one step per call, state carried), harnesses that forbid
 * hipMalloc.  Same arguments, results and rules as lstm_int_forward without a
 * trace, but the workspace is a fixed array of
 * LSTM_INT_STATIC_WORKSPACE_BYTES inside the library's device image (one copy
 * per GPU, held until the process ends; its address on the model's device is
 * looked up when the model is prepared).  The call itself allocates and frees
 * nothing on host or device.
 * LSTM_INT_E_WORKSPACE: lstm_int_workspace_bytes(model, T, B) exceeds
 * LSTM_INT_STATIC_WORKSPACE_BYTES (nothing is enqueued).
 * LSTM_INT_E_INVALID_ARG also while a profile is being recorded.
 * Every call on a GPU, from any model, shares that GPU's array: the call
 * clears what it needs cleared itself and depends on nothing an earlier call
 * left there, but calls that overlap in time on one GPU (different streams or
 * threads) race on it and must be serialized by the caller.
 */
#define LSTM_INT_STATIC_WORKSPACE_BYTES (32u << 20)
int lstm_int_forward_static(const lstm_int_model *model, const int8_t *x, int32_t T,
                            int32_t B, int8_t *y, int8_t *h_state, int16_t *c_state,
                            void *hip_stream);

/*
 * A bidirectional layer (Sec. 7: the bidirectional LSTM is two loops over the
 * same cell, one in each time direction): `fwd` runs from t = 0 up, `bwd` --
 * a model of its own whose option "reverse" is 1 -- from t = T - 1 down, both
 * over the same x, and y (DEVICE int8 [T,B,H_fwd + H_bwd]) receives at every
 * (t, b) the forward stack's output in columns [0, H_fwd) and the backward
 * stack's in [H_fwd, H_fwd + H_bwd), each in its own model's (s_h, zp_h): the
 * concatenation needs no common scale (the paper gives no rule for any other
 * way of joining the two).  Both models must be prepared on the same device
 * with the same input width and input quantization (x_min, x_max of layer 0).
 * State buffers as in lstm_int_forward, per direction, each may be NULL; the
 * backward state enters at t = T - 1 and leaves after t = 0.
 * workspace >= lstm_int_bidirectional_workspace_bytes(fwd, bwd, T, B).
 * The two directions run one after the other on hip_stream.
 * LSTM_INT_E_INVALID_ARG: widths or input quantization differ, fwd has
 * "reverse" set or bwd has not.
 */
size_t lstm_int_bidirectional_workspace_bytes(const lstm_int_model *fwd, const lstm_int_model *bwd,
                                              int32_t T, int32_t B);
int lstm_int_forward_bidirectional(const lstm_int_model *fwd, const lstm_int_model *bwd,
                                   const int8_t *x, int32_t T, int32_t B, int8_t *y,
                                   int8_t *h_state_fwd, int16_t *c_state_fwd,
                                   int8_t *h_state_bwd, int16_t *c_state_bwd,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Options of the online phase.  One selects what is computed:
 *   "reverse": 1 = every layer runs its recursion (eqs. 1-7) from time T - 1
 *           down to 0, i.e. the stack applied to the time-reversed sequence,
 *           outputs and traces stored at their positions in time (the
 *           backward half of a bidirectional layer, Sec. 7); h_state and
 *           c_state then enter at t = T - 1 and leave after t = 0.  Default 0.
 * The others are tuning knobs; results never depend on them.
 *   "path": 0 = choose per layer (default): the persistent recurrent kernel
 *               where the layer shape allows it (N % 8 == 0, N <= 2048,
 *               H <= 1024, no trace of that layer; larger batches and
 *               sequences beyond 2^14 steps run in several launches),
 *               otherwise one launch per operation and step;
 *           1 = always one launch per operation and step;
 *           2 = same as 0.
 *   "stack": models whose layers are all alike (same N, H and variant, each
 *           layer reading the one below; 2 to 8 layers) can run in ONE launch,
 *           layer l on XCD l, each layer one item (step, tile of 32 rows)
 *           behind the layer below -- the stack of Sec. 7 as a wavefront over
 *           layers and time.  Nothing is hoisted then: W x is computed per
 *           item.  0 = never; 1 (default) = where it is expected to be faster
 *           than one layer after the other (small batches: one-step calls,
 *           sequences at up to about 64 rows); 2 = wherever it can run.
 *           Calls with a trace or with "reverse" run layer after layer.
 *   "stack_step_ns", "stack_prefetch_kb", "flag_sleep": knobs of the stacked
 *           launch: expected time of one item (for the choice above), KB of a
 *           layer's W requested ahead of each item, pause between polls of the
 *           layer below's progress flag in units of 64 clocks.
 *   "rows16": 1 (default) = batches of up to 16 * 8 * (32 / ceil(N / 64)) rows
 *           run in a variant of the persistent kernel that works on groups of
 *           16 rows (more compute units busy, half the arithmetic per
 *           workgroup and step); 0 = always groups of 32 or 64 rows.
 *   "cooperative_launch": the persistent kernel needs all its workgroups (one
 *           per compute unit, up to all of them) on the device at once.
 *           0 (default) = plain launch: that holds when nothing else occupies
 *           the device for long -- no second forward call of any model running
 *           concurrently on another stream or from another process; if it does
 *           not hold, the kernel's bounded waits give up and the call ends with
 *           a nonzero device status instead of hanging.  1 = cooperative
 *           launch: the runtime guarantees it, at 16-18 us more per layer and
 *           launch (a third of a one-step call on an 8-layer stack).
 *   "spin_limit": polls after which a wait inside the persistent kernel gives
 *           up (every workgroup then leaves the kernel and the status word of
 *           lstm_int_device_status becomes nonzero).
 *   "barrier_never_completes": 1 = test hook for that path: every barrier
 *           among the workgroups of a group waits for one arrival more than
 *           will come, so the waits give up after spin_limit polls (keep it
 *           small) and the outputs of the call are not valid.  Default 0.
 *   "poll_sleep", "stats_sleep": pause between two polls of a group barrier /
 *           of the layer-norm statistics words inside the persistent kernel,
 *           in units of 64 clocks (0..1024; defaults 0 and 0).
 *   "stats_first_sleep": pause before the first poll of the statistics words
 *           (default 8).
 *   "sync_sleep": pause before the first poll of the barrier at which all
 *           workgroups of a group arrive together (the first polls would find
 *           the count incomplete and delay the arrivals); -1 (default) = 16 for
 *           groups of 16 workgroups and more, else 4.
 *   "idle_sleep", "idle_poll_sleep": the same for the workgroups that have no
 *           projection tile, at the barrier that follows the projection: pause
 *           before their first poll and between polls (defaults 64 and 12).
 *   "sparse": 1 (default) runs the recurrent product of a layer whose quantized
 *           recurrent weights are 2:4 along the contraction (at most two nonzeros
 *           in every aligned group of four h inputs; see lstm_int_sparse_layers)
 *           on the sparse MFMA where the persistent kernel for groups of 32 rows
 *           runs; 0 = always the dense product; 2 = as 1, but a forward call in
 *           which such a layer would run the dense product (batch too small or too
 *           large for that kernel, stacked launch, a trace request) fails with
 *           LSTM_INT_E_UNSUPPORTED instead.  The results are the same integers
 *           either way.
 *   "reset_status": clears the device status word (see lstm_int_device_status)
 *           after a wait gave up; synchronizes the device.
 *   "phase_timing": nonzero makes workgroup 0 of the persistent kernel add the
 *           time it spends in each of its phases to 16 device counters
 *           (diagnostics; read them with lstm_int_phase_ticks).  In a stacked
 *           launch the value is 1 + the layer whose workgroup 0 is timed.
 * Unknown keys or values give LSTM_INT_E_INVALID_ARG.
 */
int lstm_int_set_option(lstm_int_model *model, const char *key, int64_t value);

/*
 * Pruned models (Table 1, the sparse LSTM and sparse CIFG rows): *count receives
 * the number of layers whose quantized recurrent weights R are 2:4 structured
 * -- every row has at most two nonzero weights in each aligned group of four
 * consecutive inputs h[4j .. 4j+3] -- and for which prepare therefore also
 * built the compressed operands of the sparse MFMA (option "sparse").  A zero
 * weight is one whose int8 code is 0; symmetric weight quantization (Table 2)
 * maps a pruned float weight to exactly that.  Host only; no device work.
 */
int lstm_int_sparse_layers(const lstm_int_model *model, int32_t *count);

/*
 * Blocking read of the model's device status word: 0 = every persistent
 * kernel so far ran to completion; nonzero = a wait gave up (1) or the
 * workgroups of a group were not placed on one XCD (2), and the outputs of
 * that call are not valid.  The word is sticky.  Synchronizes the device.
 */
int lstm_int_device_status(const lstm_int_model *model, int32_t *status);

/*
 * Diagnostics: blocking read of the 16 phase counters of "phase_timing", in
 * ticks of the 100 MHz device wall clock, summed over all steps and launches
 * since the option was set.  Phases: 0 load h and W x terms, 1 R h (MFMA),
 * 2 gate sums and statistics, 3 wait, 4 statistics to (mean, sigma),
 * 5 layer norm, sigma/tanh, cell, 6 output gate and hidden state, 7 wait,
 * 8 projection, 9 wait.
 */
int lstm_int_phase_ticks(const lstm_int_model *model, int64_t ticks[16]);

/*
 * Per-kernel device time of the forward calls made while profiling is on,
 * measured with HIP events on the stream the kernels run on.
 * lstm_int_profile_begin resets the counters and makes forward record events
 * (created as the launches need them, any number per call);
 * lstm_int_profile_end synchronizes that stream, fills, per kernel class k
 * (LSTM_INT_K_*), launches[k] and total_ms[k], and destroys the events.
 * Profiling adds host work to forward; throughput is measured with it off.
 */
#define LSTM_INT_K_INPUT_GEMM 0 /* hoisted W x over all T, + rescale        */
#define LSTM_INT_K_RECURRENT 1  /* R h per step (+ fused epilogue if any)   */
#define LSTM_INT_K_CELL 2       /* gate sum, layer norm, activations, cell  */
#define LSTM_INT_K_PROJECTION 3 /* W_proj m + requantization                */
#define LSTM_INT_K_OTHER 4      /* state copies, padding                    */
#define LSTM_INT_K_COUNT 5
int lstm_int_profile_begin(lstm_int_model *model);
int lstm_int_profile_end(lstm_int_model *model, int64_t launches[LSTM_INT_K_COUNT],
                         double total_ms[LSTM_INT_K_COUNT]);

/*
 * Measurement aid for the roofline of the hoisted input GEMM (Sec. 6: the
 * folded-bias matmul W x): runs, on every compute unit, `blocks` rounds of 40
 * int8 MFMAs (32x32x32, operands in registers) followed by stores_per_block
 * (0..8) streaming stores of 1 KB per wave -- 4 is the benchmark layer's mix of
 * matrix work and int16 output -- and reports the sustained TOP/s, the store
 * rate in GB/s and the shader clock in GHz the chip held.  Allocates and frees
 * 256 MiB of device memory; synchronizes.
 */
int lstm_int_mfma_store_ceiling(int32_t device, int32_t stores_per_block, int32_t blocks,
                                double *tops, double *store_gbs, double *clock_ghz);

/*
 * Measurement aid for the LDS layouts of the matmul kernels (the operand tiles
 * of the gate matmuls, Sec. 3.2.4): ONE launch of one workgroup of four waves
 * in which every wave repeats one 16-byte LDS access per lane 4096 times.  What
 * the access costs is read from the hardware counters of that launch (rocprofv3
 * --pmc SQ_LDS_IDX_ACTIVE SQ_LDS_BANK_CONFLICT): IDX_ACTIVE / (4 * 4096) = LDS
 * clocks per wave access.  Rows of `stride_words` 32-bit words; lane -> (row,
 * 16-byte piece) by `map`: 0 = (lane % 16, lane / 16), the operand of the
 * 16x16x64 MFMA; 1 = (lane % 32, lane / 32), of the 32x32x32 MFMA; 2 =
 * (lane / 4, lane % 4), the order in which four lanes fetch a row's 64 bytes;
 * the piece sits at position piece ^ s(row), s by `swizzle`: 0 = none, 1 =
 * (row >> 1) & 3, 2 = (row >> 2) & 3; write != 0 stores instead of loading.
 * Needs stride_words in 4..128 and a multiple of 4.  Synchronizes.
 */
int lstm_int_lds_probe(int32_t device, int32_t map, int32_t stride_words, int32_t swizzle, int32_t write);

void lstm_int_destroy(lstm_int_model *model);

const char *lstm_int_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
