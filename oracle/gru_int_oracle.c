/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.
 *
 * Integer-only GRU from the building blocks of arXiv 2101.05453 (Sec. 7 names
 * the GRU, the recipe is this build's: see gru_int_oracle.h).  Plain scalar C;
 * int64 arithmetic throughout; one batch row at a time.
 */
#include "gru_int_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "lstm_int_oracle.h"

static int64_t clampg(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }
static int64_t sat8g(int64_t v) { return clampg(v, -128, 127); }
static int64_t sat16g(int64_t v) { return clampg(v, -32768, 32767); }

/* float -> integer rounding: floor(v + 1/2) in double, as in the LSTM recipe */
static int64_t round_clamp(double v, double s, int64_t qmax) {
  double r = floor(v / s + 0.5);
  if (r < (double)-qmax) r = (double)-qmax;
  if (r > (double)qmax) r = (double)qmax;
  return (int64_t)r;
}

static int all_finite(const float *a, int64_t n) {
  for (int64_t i = 0; i < n; ++i)
    if (!isfinite(a[i])) return 0;
  return 1;
}

/* symmetric per-tensor scale: max|w| / 127, 1 for an all-zero tensor (Sec. 3.2.4) */
static double tensor_scale(const float *a, int64_t n) {
  double m = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double v = fabs((double)a[i]);
    if (v > m) m = v;
  }
  return m == 0.0 ? 1.0 : m / 127.0;
}

static void free_gru_layer(orc_gru_layer_quant *q) {
  free(q->Wq); free(q->Rq); free(q->bxq); free(q->bhq); free(q->bx_fold);
  memset(q, 0, sizeof(*q));
}

void orc_gru_destroy(orc_gru_model *m) {
  if (!m) return;
  for (int l = 0; l < m->num_layers; ++l) free_gru_layer(&m->layers[l]);
  free(m->layers);
  free(m);
}

const orc_gru_layer_quant *orc_gru_get_layer(const orc_gru_model *m, int32_t layer) {
  if (!m || layer < 0 || layer >= m->num_layers) return NULL;
  return &m->layers[layer];
}

static int prepare_gru_layer(const orc_gru_layer_params *p, int has_prev, orc_gru_layer_quant *q) {
  memset(q, 0, sizeof(*q));
  const int I = p->input_size, N = p->num_cells;
  if (I < 1 || N < 1) return ORC_INVALID_ARG;
  if (I > 32768 || N > 32768) return ORC_UNSUPPORTED; /* accumulation depth, Sec. 3.1.1 */
  for (int g = 0; g < 3; ++g)
    if (!p->W[g] || !p->R[g] || !p->bx[g] || !p->bh[g]) return ORC_INVALID_ARG;
  q->I = I; q->N = N;

  /* layer input: asymmetric int8 with a nudged zero point (Sec. 3.2.4); a
   * stacked layer reads the int8 state of the layer below: scale 2^-7, zero
   * point 0 */
  if (has_prev) {
    q->s_x = ldexp(1.0, -7);
    q->zp_x = 0;
  } else {
    double lo = p->x_min, hi = p->x_max;
    if (!isfinite(lo) || !isfinite(hi) || lo > hi) return ORC_BAD_RANGE;
    if (lo > 0.0) lo = 0.0;
    if (hi < 0.0) hi = 0.0;
    double s = (hi - lo) / 255.0;
    if (s == 0.0) s = 1.0;
    double z = floor(-128.0 - lo / s + 0.5);
    q->s_x = s;
    q->zp_x = (int32_t)clampg((int64_t)z, -128, 127);
  }
  const double s_h8 = ldexp(1.0, -7);

  q->Wq = calloc((size_t)3 * N * I, 1);
  q->Rq = calloc((size_t)3 * N * N, 1);
  q->bxq = calloc((size_t)3 * N, sizeof(int32_t));
  q->bhq = calloc((size_t)3 * N, sizeof(int32_t));
  q->bx_fold = calloc((size_t)3 * N, sizeof(int32_t));
  if (!q->Wq || !q->Rq || !q->bxq || !q->bhq || !q->bx_fold) return ORC_NOMEM;

  for (int g = 0; g < 3; ++g) {
    if (!all_finite(p->W[g], (int64_t)N * I) || !all_finite(p->R[g], (int64_t)N * N) ||
        !all_finite(p->bx[g], N) || !all_finite(p->bh[g], N))
      return ORC_BAD_RANGE;
    q->s_W[g] = tensor_scale(p->W[g], (int64_t)N * I);
    q->s_R[g] = tensor_scale(p->R[g], (int64_t)N * N);
    for (int64_t i = 0; i < (int64_t)N * I; ++i)
      q->Wq[(int64_t)g * N * I + i] = (int8_t)round_clamp(p->W[g][i], q->s_W[g], 127);
    for (int64_t i = 0; i < (int64_t)N * N; ++i)
      q->Rq[(int64_t)g * N * N + i] = (int8_t)round_clamp(p->R[g][i], q->s_R[g], 127);
    /* biases: int32 at the scale of the accumulator they join (Sec. 3.2.4) */
    for (int n = 0; n < N; ++n) {
      q->bxq[g * N + n] = (int32_t)round_clamp(p->bx[g][n], q->s_W[g] * q->s_x, 2147483647LL);
      q->bhq[g * N + n] = (int32_t)round_clamp(p->bh[g][n], q->s_R[g] * s_h8, 2147483647LL);
    }
    /* both matmul results go to Q3.12 (Sec. 3.2.4) */
    int rc;
    if ((rc = orc_quantize_multiplier(q->s_W[g] * q->s_x * 4096.0, &q->Mx[g], &q->ex[g])) != ORC_OK) return rc;
    if ((rc = orc_quantize_multiplier(q->s_R[g] * s_h8 * 4096.0, &q->Mh[g], &q->eh[g])) != ORC_OK) return rc;
    /* zero point of x folded into the input bias (Sec. 6); the accumulators
     * must hold for every int8 input */
    for (int n = 0; n < N; ++n) {
      const int8_t *w = q->Wq + ((int64_t)g * N + n) * I;
      int64_t sum = 0, sum_abs = 0;
      for (int k = 0; k < I; ++k) {
        sum += w[k];
        sum_abs += w[k] < 0 ? -(int64_t)w[k] : (int64_t)w[k];
      }
      int64_t f = (int64_t)q->bxq[g * N + n] - (int64_t)q->zp_x * sum;
      if ((f < 0 ? -f : f) + 128 * sum_abs > 2147483647LL) return ORC_UNSUPPORTED;
      q->bx_fold[g * N + n] = (int32_t)f;
      const int8_t *r = q->Rq + ((int64_t)g * N + n) * N;
      int64_t rabs = 0;
      for (int k = 0; k < N; ++k) rabs += r[k] < 0 ? -(int64_t)r[k] : (int64_t)r[k];
      int64_t bh = q->bhq[g * N + n];
      if ((bh < 0 ? -bh : bh) + 128 * rabs > 2147483647LL) return ORC_UNSUPPORTED;
    }
  }
  return ORC_OK;
}

int orc_gru_prepare(const orc_gru_layer_params *layers, int32_t num_layers, orc_gru_model **out) {
  if (!layers || !out || num_layers < 1) return ORC_INVALID_ARG;
  *out = NULL;
  orc_gru_model *m = calloc(1, sizeof(*m));
  if (!m) return ORC_NOMEM;
  m->layers = calloc((size_t)num_layers, sizeof(orc_gru_layer_quant));
  if (!m->layers) { free(m); return ORC_NOMEM; }
  m->num_layers = num_layers;
  for (int l = 0; l < num_layers; ++l) {
    if (l > 0 && layers[l].input_size != layers[l - 1].num_cells) { orc_gru_destroy(m); return ORC_INVALID_ARG; }
    int rc = prepare_gru_layer(&layers[l], l > 0, &m->layers[l]);
    if (rc != ORC_OK) { orc_gru_destroy(m); return rc; }
  }
  *out = m;
  return ORC_OK;
}

/* the int8 form of the state: matmul operand and layer output */
static int8_t state_to_i8(int16_t h16) { return (int8_t)sat8g(orc_rsh_r(h16, 8)); }

typedef struct {
  int16_t *tx, *th, *act, *h16;
  int8_t *h8;
} gru_row_trace;

/* one step of one batch row: x[I], h16[N] updated in place, h8_prev[N] the
 * int8 form of the state before the step, h8_out[N] after it */
static int gru_step(const orc_gru_layer_quant *q, const int8_t *x, const int8_t *h8_prev, int16_t *h16,
                    int8_t *h8_out, int unfolded, const gru_row_trace *tr, int16_t *tx, int16_t *th,
                    int16_t *act) {
  const int I = q->I, N = q->N;
  for (int g = 0; g < 3; ++g)
    for (int n = 0; n < N; ++n) {
      const int gn = g * N + n;
      const int8_t *w = q->Wq + (int64_t)gn * I, *r = q->Rq + (int64_t)gn * N;
      int64_t accx = 0, acch = 0;
      if (unfolded) {
        for (int k = 0; k < I; ++k) accx += (int64_t)w[k] * ((int64_t)x[k] - q->zp_x);
        accx += q->bxq[gn];
      } else {
        for (int k = 0; k < I; ++k) accx += (int64_t)w[k] * (int64_t)x[k];
        accx += q->bx_fold[gn];
      }
      for (int k = 0; k < N; ++k) acch += (int64_t)r[k] * (int64_t)h8_prev[k];
      acch += q->bhq[gn];
      if (accx != clampg(accx, -2147483647LL - 1, 2147483647LL) ||
          acch != clampg(acch, -2147483647LL - 1, 2147483647LL))
        return ORC_UNSUPPORTED;
      tx[gn] = (int16_t)sat16g(orc_rescale(accx, q->Mx[g], q->ex[g]));
      th[gn] = (int16_t)sat16g(orc_rescale(acch, q->Mh[g], q->eh[g]));
    }
  for (int n = 0; n < N; ++n) {
    /* reset and update gates: Q3.12 sums through the 16-bit sigma (Sec. 3.2.1) */
    const int64_t r = orc_int_sigmoid((int32_t)sat16g((int64_t)tx[n] + th[n]), 3);
    const int64_t u = orc_int_sigmoid((int32_t)sat16g((int64_t)tx[N + n] + th[N + n]), 3);
    /* r . (R_n h + bh_n): Q0.15 x Q3.12 -> Q3.12 */
    const int64_t rn = orc_rsh_r(r * (int64_t)th[2 * N + n], 15);
    const int64_t c = orc_int_tanh((int32_t)sat16g((int64_t)tx[2 * N + n] + rn), 3);
    /* 1 - u by the coupling of Sec. 3.2.9 */
    const int64_t ubar = 32768 - u < 32767 ? 32768 - u : 32767;
    /* state update in the form of Sec. 3.2.7: two Q0.30 products, each
     * rounded to Q0.15, saturating sum */
    const int64_t hn = sat16g(orc_rsh_r(ubar * c, 15) + orc_rsh_r(u * (int64_t)h16[n], 15));
    act[n] = (int16_t)r;
    act[N + n] = (int16_t)u;
    act[2 * N + n] = (int16_t)c;
    h16[n] = (int16_t)hn;
    h8_out[n] = state_to_i8((int16_t)hn);
  }
  if (tr->tx) memcpy(tr->tx, tx, sizeof(int16_t) * 3 * N);
  if (tr->th) memcpy(tr->th, th, sizeof(int16_t) * 3 * N);
  if (tr->act) memcpy(tr->act, act, sizeof(int16_t) * 3 * N);
  if (tr->h16) memcpy(tr->h16, h16, sizeof(int16_t) * N);
  if (tr->h8) memcpy(tr->h8, h8_out, (size_t)N);
  return ORC_OK;
}

int orc_gru_forward(const orc_gru_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                    int16_t *h_state, const orc_gru_trace *trace, int unfolded, int threads) {
  if (!m || !x || !y || T < 0 || B < 0) return ORC_INVALID_ARG;
  if (trace && (trace->layer < 0 || trace->layer >= m->num_layers)) return ORC_INVALID_ARG;
  if (T == 0 || B == 0) return ORC_OK;
  if (threads < 1) threads = 1;
  const int L = m->num_layers;
  int status = ORC_OK;
  const int8_t *in = x;
  int8_t *buf[2] = {NULL, NULL};
  int64_t h_off = 0;
  for (int l = 0; l < L; ++l) {
    const orc_gru_layer_quant *q = &m->layers[l];
    const int I = q->I, N = q->N;
    int8_t *out = y;
    if (l != L - 1) {
      buf[l & 1] = realloc(buf[l & 1], (size_t)T * B * N);
      if (!buf[l & 1]) { status = ORC_NOMEM; break; }
      out = buf[l & 1];
    }
    const orc_gru_trace *tl = (trace && trace->layer == l) ? trace : NULL;
    int16_t *hs = h_state ? h_state + h_off : NULL;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int b = 0; b < B; ++b) {
      int16_t *h16 = malloc(sizeof(int16_t) * (size_t)N * 10 + (size_t)N);
      if (!h16) {
#pragma omp critical
        status = ORC_NOMEM;
        continue;
      }
      int16_t *tx = h16 + N, *th = h16 + 4 * N, *act = h16 + 7 * N;
      int8_t *h8_0 = (int8_t *)(h16 + 10 * N);
      for (int n = 0; n < N; ++n) {
        h16[n] = hs ? hs[(int64_t)b * N + n] : 0;
        h8_0[n] = state_to_i8(h16[n]);
      }
      for (int t = 0; t < T; ++t) {
        const int64_t tb = (int64_t)t * B + b;
        const int8_t *hp = t == 0 ? h8_0 : out + ((int64_t)(t - 1) * B + b) * N;
        gru_row_trace rt;
        memset(&rt, 0, sizeof(rt));
        if (tl) {
          rt.tx = tl->tx ? tl->tx + tb * 3 * N : NULL;
          rt.th = tl->th ? tl->th + tb * 3 * N : NULL;
          rt.act = tl->act ? tl->act + tb * 3 * N : NULL;
          rt.h16 = tl->h16 ? tl->h16 + tb * N : NULL;
          rt.h8 = tl->h8 ? tl->h8 + tb * N : NULL;
        }
        int rc = gru_step(q, in + tb * I, hp, h16, out + tb * N, unfolded, &rt, tx, th, act);
        if (rc != ORC_OK) {
#pragma omp critical
          status = rc;
          break;
        }
      }
      if (hs) memcpy(hs + (int64_t)b * N, h16, sizeof(int16_t) * N);
      free(h16);
    }
    if (status != ORC_OK) break;
    in = out;
    h_off += (int64_t)B * N;
  }
  free(buf[0]);
  free(buf[1]);
  return status;
}

/* ------------------------------------------------------------------ */
/* the float cell, in double                                           */
/* ------------------------------------------------------------------ */

static double sigm(double v) { return 1.0 / (1.0 + exp(-v)); }

int orc_gru_float_forward(const orc_gru_layer_params *layers, int32_t num_layers, const float *x,
                          int32_t T, int32_t B, double *y, int threads) {
  if (!layers || !x || num_layers < 1 || T < 0 || B < 0) return ORC_INVALID_ARG;
  if (T == 0 || B == 0) return ORC_OK;
  if (threads < 1) threads = 1;
  const int64_t TB = (int64_t)T * B;
  double *in = malloc(sizeof(double) * (size_t)TB * layers[0].input_size);
  if (!in) return ORC_NOMEM;
  for (int64_t i = 0; i < TB * layers[0].input_size; ++i) in[i] = x[i];
  int status = ORC_OK;
  for (int l = 0; l < num_layers && status == ORC_OK; ++l) {
    const orc_gru_layer_params *p = &layers[l];
    const int I = p->input_size, N = p->num_cells;
    double *out = malloc(sizeof(double) * (size_t)TB * N);
    if (!out) { status = ORC_NOMEM; break; }
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int b = 0; b < B; ++b) {
      double *h = calloc((size_t)N * 2, sizeof(double));
      if (!h) {
#pragma omp critical
        status = ORC_NOMEM;
        continue;
      }
      double *hn = h + N;
      for (int t = 0; t < T; ++t) {
        const double *xt = in + ((int64_t)t * B + b) * I;
        for (int n = 0; n < N; ++n) {
          double ax[3], ah[3];
          for (int g = 0; g < 3; ++g) {
            double sx = p->bx[g][n], sh = p->bh[g][n];
            const float *w = p->W[g] + (int64_t)n * I, *r = p->R[g] + (int64_t)n * N;
            for (int k = 0; k < I; ++k) sx += (double)w[k] * xt[k];
            for (int k = 0; k < N; ++k) sh += (double)r[k] * h[k];
            ax[g] = sx;
            ah[g] = sh;
          }
          const double rg = sigm(ax[0] + ah[0]), ug = sigm(ax[1] + ah[1]);
          const double cg = tanh(ax[2] + rg * ah[2]);
          hn[n] = (1.0 - ug) * cg + ug * h[n];
        }
        memcpy(h, hn, sizeof(double) * N);
        memcpy(out + ((int64_t)t * B + b) * N, h, sizeof(double) * N);
      }
      free(h);
    }
    free(in);
    in = out;
  }
  if (status == ORC_OK && y) memcpy(y, in, sizeof(double) * (size_t)TB * layers[num_layers - 1].num_cells);
  free(in);
  return status;
}
