/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.
 *
 * Integer-only SRU from the building blocks of arXiv 2101.05453 (Sec. 7 names
 * the SRU, the recipe is this build's: see sru_int_oracle.h).  Plain scalar C;
 * int64 arithmetic throughout; one batch row at a time.
 */
#include "sru_int_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "lstm_int_oracle.h"

static int64_t clamps(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }
static int64_t sat8s(int64_t v) { return clamps(v, -128, 127); }
static int64_t sat16s(int64_t v) { return clamps(v, -32768, 32767); }

/* float -> integer rounding: floor(v / s + 1/2) in double, as in the LSTM recipe */
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

/* symmetric per-tensor scale: max|w| / qmax, 1 for an all-zero tensor (Sec. 3.2.4) */
static double tensor_scale(const float *a, int64_t n, double qmax) {
  double m = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double v = fabs((double)a[i]);
    if (v > m) m = v;
  }
  return m == 0.0 ? 1.0 : m / qmax;
}

/* asymmetric int8 over [lo, hi] extended to contain 0, zero point nudged to an
 * integer (Sec. 3.2.4) */
static int asym8(double lo, double hi, double *s, int32_t *zp) {
  if (!isfinite(lo) || !isfinite(hi) || lo > hi) return ORC_BAD_RANGE;
  if (lo > 0.0) lo = 0.0;
  if (hi < 0.0) hi = 0.0;
  double sc = (hi - lo) / 255.0;
  if (sc == 0.0) sc = 1.0;
  *s = sc;
  *zp = (int32_t)clamps((int64_t)floor(-128.0 - lo / sc + 0.5), -128, 127);
  return ORC_OK;
}

static void free_sru_layer(orc_sru_layer_quant *q) {
  free(q->Wq); free(q->vq); free(q->bq); free(q->b_fold);
  memset(q, 0, sizeof(*q));
}

void orc_sru_destroy(orc_sru_model *m) {
  if (!m) return;
  for (int l = 0; l < m->num_layers; ++l) free_sru_layer(&m->layers[l]);
  free(m->layers);
  free(m);
}

const orc_sru_layer_quant *orc_sru_get_layer(const orc_sru_model *m, int32_t layer) {
  if (!m || layer < 0 || layer >= m->num_layers) return NULL;
  return &m->layers[layer];
}

static int prepare_sru_layer(const orc_sru_layer_params *p, const orc_sru_layer_quant *prev,
                             orc_sru_layer_quant *q) {
  memset(q, 0, sizeof(*q));
  const int I = p->input_size, N = p->num_cells;
  if (I < 1 || N < 1) return ORC_INVALID_ARG;
  if (I > 32768 || N > 32768) return ORC_UNSUPPORTED; /* accumulation depth, Sec. 3.1.1 */
  for (int g = 0; g < 3; ++g)
    if (!p->W[g]) return ORC_INVALID_ARG;
  for (int j = 0; j < 2; ++j)
    if (!p->v[j] || !p->b[j]) return ORC_INVALID_ARG;
  const int G = p->W[3] ? 4 : 3;
  if (G == 3 && I != N) return ORC_INVALID_ARG; /* the input itself is the highway term */
  q->I = I; q->N = N; q->G = G;

  int rc;
  if (prev) { /* a stacked layer reads the output of the layer below */
    q->s_x = prev->s_h;
    q->zp_x = prev->zp_h;
  } else if ((rc = asym8(p->x_min, p->x_max, &q->s_x, &q->zp_x)) != ORC_OK)
    return rc;
  if ((rc = asym8(p->h_min, p->h_max, &q->s_h, &q->zp_h)) != ORC_OK) return rc;

  /* state format: measured magnitude extended to a power of two (Sec. 3.2.2) */
  double ca = p->c_absmax;
  if (!isfinite(ca) || ca < 0.0) return ORC_BAD_RANGE;
  int mc = 0;
  while (mc <= 8 && ldexp(1.0, mc) < ca) ++mc;
  if (mc > 8) return ORC_UNSUPPORTED;
  q->m_c = mc;
  const double s_c = ldexp(1.0, mc - 15);

  q->Wq = calloc((size_t)G * N * I, 1);
  q->vq = calloc((size_t)2 * N, sizeof(int16_t));
  q->bq = calloc((size_t)G * N, sizeof(int32_t));
  q->b_fold = calloc((size_t)G * N, sizeof(int32_t));
  if (!q->Wq || !q->vq || !q->bq || !q->b_fold) return ORC_NOMEM;

  for (int g = 0; g < G; ++g) {
    if (!all_finite(p->W[g], (int64_t)N * I)) return ORC_BAD_RANGE;
    q->s_W[g] = tensor_scale(p->W[g], (int64_t)N * I, 127.0);
    for (int64_t i = 0; i < (int64_t)N * I; ++i)
      q->Wq[(int64_t)g * N * I + i] = (int8_t)round_clamp(p->W[g][i], q->s_W[g], 127);
    const int gate = g == ORC_SRU_F || g == ORC_SRU_R;
    if (gate) { /* biases: int32 at the scale of the accumulator they join (Sec. 3.2.4) */
      const float *b = p->b[g - ORC_SRU_F];
      if (!all_finite(b, N)) return ORC_BAD_RANGE;
      for (int n = 0; n < N; ++n)
        q->bq[g * N + n] = (int32_t)round_clamp(b[n], q->s_W[g] * q->s_x, 2147483647LL);
    }
    /* gates go to Q3.12, candidate and highway term to the state's format */
    const double target = gate ? ldexp(1.0, -12) : s_c;
    if ((rc = orc_quantize_multiplier(q->s_W[g] * q->s_x / target, &q->Mx[g], &q->ex[g])) != ORC_OK) return rc;
    /* zero point of x folded into a per-row constant (Sec. 6); the
     * accumulators must hold for every int8 input */
    for (int n = 0; n < N; ++n) {
      const int8_t *w = q->Wq + ((int64_t)g * N + n) * I;
      int64_t sum = 0, sum_abs = 0;
      for (int k = 0; k < I; ++k) {
        sum += w[k];
        sum_abs += w[k] < 0 ? -(int64_t)w[k] : (int64_t)w[k];
      }
      int64_t f = (int64_t)q->bq[g * N + n] - (int64_t)q->zp_x * sum;
      if ((f < 0 ? -f : f) + 128 * sum_abs > 2147483647LL) return ORC_UNSUPPORTED;
      q->b_fold[g * N + n] = (int32_t)f;
    }
  }
  for (int j = 0; j < 2; ++j) { /* recurrent weight vectors: int16 like peephole weights (Sec. 3.2.3) */
    if (!all_finite(p->v[j], N)) return ORC_BAD_RANGE;
    q->s_v[j] = tensor_scale(p->v[j], N, 32767.0);
    for (int n = 0; n < N; ++n) q->vq[j * N + n] = (int16_t)round_clamp(p->v[j][n], q->s_v[j], 32767);
    if ((rc = orc_quantize_multiplier(q->s_v[j] * s_c * 4096.0, &q->Mv[j], &q->ev[j])) != ORC_OK) return rc;
  }
  if (G == 3 && (rc = orc_quantize_multiplier(q->s_x / s_c, &q->Ms, &q->es)) != ORC_OK) return rc;
  if ((rc = orc_quantize_multiplier(s_c / q->s_h, &q->Mh, &q->eh)) != ORC_OK) return rc;
  return ORC_OK;
}

int orc_sru_prepare(const orc_sru_layer_params *layers, int32_t num_layers, orc_sru_model **out) {
  if (!layers || !out || num_layers < 1) return ORC_INVALID_ARG;
  *out = NULL;
  orc_sru_model *m = calloc(1, sizeof(*m));
  if (!m) return ORC_NOMEM;
  m->layers = calloc((size_t)num_layers, sizeof(orc_sru_layer_quant));
  if (!m->layers) { free(m); return ORC_NOMEM; }
  m->num_layers = num_layers;
  for (int l = 0; l < num_layers; ++l) {
    if (l > 0 && layers[l].input_size != layers[l - 1].num_cells) { orc_sru_destroy(m); return ORC_INVALID_ARG; }
    int rc = prepare_sru_layer(&layers[l], l > 0 ? &m->layers[l - 1] : NULL, &m->layers[l]);
    if (rc != ORC_OK) { orc_sru_destroy(m); return rc; }
  }
  *out = m;
  return ORC_OK;
}

typedef struct {
  int16_t *tx, *tv, *act, *c, *h16;
  int8_t *y;
} sru_row_trace;

/* one step of one batch row: x[I], c[N] updated in place, y[N] written;
 * tx[4N], tv[2N], act[2N], h16[N] are scratch */
static int sru_step(const orc_sru_layer_quant *q, const int8_t *x, int16_t *c, int8_t *y, int unfolded,
                    const sru_row_trace *tr, int16_t *tx, int16_t *tv, int16_t *act, int16_t *h16) {
  const int I = q->I, N = q->N, G = q->G;
  for (int g = 0; g < G; ++g)
    for (int n = 0; n < N; ++n) {
      const int gn = g * N + n;
      const int8_t *w = q->Wq + (int64_t)gn * I;
      int64_t acc = 0;
      if (unfolded) {
        for (int k = 0; k < I; ++k) acc += (int64_t)w[k] * ((int64_t)x[k] - q->zp_x);
        acc += q->bq[gn];
      } else {
        for (int k = 0; k < I; ++k) acc += (int64_t)w[k] * (int64_t)x[k];
        acc += q->b_fold[gn];
      }
      if (acc != clamps(acc, -2147483647LL - 1, 2147483647LL)) return ORC_UNSUPPORTED;
      tx[gn] = (int16_t)sat16s(orc_rescale(acc, q->Mx[g], q->ex[g]));
    }
  if (G == 3) /* the input itself is the highway term, brought to the state's format */
    for (int n = 0; n < N; ++n)
      tx[ORC_SRU_S * N + n] = (int16_t)sat16s(orc_rescale((int64_t)x[n] - q->zp_x, q->Ms, q->es));
  for (int n = 0; n < N; ++n) {
    /* both gates read the state before the step (Sec. 3.2.3 form of v . c) */
    for (int j = 0; j < 2; ++j) {
      tv[j * N + n] = (int16_t)sat16s(orc_rescale((int64_t)q->vq[j * N + n] * c[n], q->Mv[j], q->ev[j]));
      const int64_t sum = sat16s((int64_t)tx[(ORC_SRU_F + j) * N + n] + tv[j * N + n]);
      act[j * N + n] = (int16_t)orc_int_sigmoid((int32_t)sum, 3); /* Sec. 3.2.1 */
    }
    const int64_t f = act[n], r = act[N + n];
    const int64_t fbar = 32768 - f < 32767 ? 32768 - f : 32767; /* Sec. 3.2.9 */
    const int64_t rbar = 32768 - r < 32767 ? 32768 - r : 32767;
    /* Sec. 3.2.7: two Q0.15 x state-format products, each rounded back, saturating sum */
    const int64_t cn = sat16s(orc_rsh_r(f * (int64_t)c[n], 15) + orc_rsh_r(fbar * (int64_t)tx[ORC_SRU_C * N + n], 15));
    const int64_t hn = sat16s(orc_rsh_r(r * cn, 15) + orc_rsh_r(rbar * (int64_t)tx[ORC_SRU_S * N + n], 15));
    c[n] = (int16_t)cn;
    h16[n] = (int16_t)hn;
    y[n] = (int8_t)sat8s((int64_t)orc_rescale(hn, q->Mh, q->eh) + q->zp_h); /* Sec. 3.2.8 */
  }
  if (tr->tx) memcpy(tr->tx, tx, sizeof(int16_t) * 4 * N);
  if (tr->tv) memcpy(tr->tv, tv, sizeof(int16_t) * 2 * N);
  if (tr->act) memcpy(tr->act, act, sizeof(int16_t) * 2 * N);
  if (tr->c) memcpy(tr->c, c, sizeof(int16_t) * N);
  if (tr->h16) memcpy(tr->h16, h16, sizeof(int16_t) * N);
  if (tr->y) memcpy(tr->y, y, (size_t)N);
  return ORC_OK;
}

int orc_sru_forward(const orc_sru_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                    int16_t *c_state, const orc_sru_trace *trace, int unfolded, int threads) {
  if (!m || !x || !y || T < 0 || B < 0) return ORC_INVALID_ARG;
  if (trace && (trace->layer < 0 || trace->layer >= m->num_layers)) return ORC_INVALID_ARG;
  if (T == 0 || B == 0) return ORC_OK;
  if (threads < 1) threads = 1;
  const int L = m->num_layers;
  int status = ORC_OK;
  const int8_t *in = x;
  int8_t *buf[2] = {NULL, NULL};
  int64_t c_off = 0;
  for (int l = 0; l < L; ++l) {
    const orc_sru_layer_quant *q = &m->layers[l];
    const int I = q->I, N = q->N;
    int8_t *out = y;
    if (l != L - 1) {
      buf[l & 1] = realloc(buf[l & 1], (size_t)T * B * N);
      if (!buf[l & 1]) { status = ORC_NOMEM; break; }
      out = buf[l & 1];
    }
    const orc_sru_trace *tl = (trace && trace->layer == l) ? trace : NULL;
    int16_t *cs = c_state ? c_state + c_off : NULL;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int b = 0; b < B; ++b) {
      int16_t *c = calloc((size_t)N * 10, sizeof(int16_t));
      if (!c) {
#pragma omp critical
        status = ORC_NOMEM;
        continue;
      }
      int16_t *tx = c + N, *tv = c + 5 * N, *act = c + 7 * N, *h16 = c + 9 * N;
      if (cs) memcpy(c, cs + (int64_t)b * N, sizeof(int16_t) * N);
      for (int t = 0; t < T; ++t) {
        const int64_t tb = (int64_t)t * B + b;
        sru_row_trace rt;
        memset(&rt, 0, sizeof(rt));
        if (tl) {
          rt.tx = tl->tx ? tl->tx + tb * 4 * N : NULL;
          rt.tv = tl->tv ? tl->tv + tb * 2 * N : NULL;
          rt.act = tl->act ? tl->act + tb * 2 * N : NULL;
          rt.c = tl->c ? tl->c + tb * N : NULL;
          rt.h16 = tl->h16 ? tl->h16 + tb * N : NULL;
          rt.y = tl->y ? tl->y + tb * N : NULL;
        }
        int rc = sru_step(q, in + tb * I, c, out + tb * N, unfolded, &rt, tx, tv, act, h16);
        if (rc != ORC_OK) {
#pragma omp critical
          status = rc;
          break;
        }
      }
      if (cs) memcpy(cs + (int64_t)b * N, c, sizeof(int16_t) * N);
      free(c);
    }
    if (status != ORC_OK) break;
    in = out;
    c_off += (int64_t)B * N;
  }
  free(buf[0]);
  free(buf[1]);
  return status;
}

/* ------------------------------------------------------------------ */
/* the float cell, in double                                           */
/* ------------------------------------------------------------------ */

static double sigm(double v) { return 1.0 / (1.0 + exp(-v)); }

int orc_sru_float_forward(const orc_sru_layer_params *layers, int32_t num_layers, const float *x,
                          int32_t T, int32_t B, double *y, orc_sru_stats *stats, int threads) {
  if (!layers || !x || num_layers < 1 || T < 0 || B < 0) return ORC_INVALID_ARG;
  for (int l = 0; l < num_layers; ++l) {
    const orc_sru_layer_params *p = &layers[l];
    if (!p->W[0] || !p->W[1] || !p->W[2] || !p->v[0] || !p->v[1] || !p->b[0] || !p->b[1]) return ORC_INVALID_ARG;
    if (!p->W[3] && p->input_size != p->num_cells) return ORC_INVALID_ARG;
    if (stats) stats[l].c_absmax = stats[l].h_min = stats[l].h_max = 0.0;
  }
  if (T == 0 || B == 0) return ORC_OK;
  if (threads < 1) threads = 1;
  const int64_t TB = (int64_t)T * B;
  double *in = malloc(sizeof(double) * (size_t)TB * layers[0].input_size);
  if (!in) return ORC_NOMEM;
  for (int64_t i = 0; i < TB * layers[0].input_size; ++i) in[i] = x[i];
  int status = ORC_OK;
  for (int l = 0; l < num_layers && status == ORC_OK; ++l) {
    const orc_sru_layer_params *p = &layers[l];
    const int I = p->input_size, N = p->num_cells;
    double *out = malloc(sizeof(double) * (size_t)TB * N);
    if (!out) { status = ORC_NOMEM; break; }
    double cmax = 0.0, hlo = 0.0, hhi = 0.0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads) reduction(max : cmax, hhi) reduction(min : hlo)
    for (int b = 0; b < B; ++b) {
      double *c = calloc((size_t)N, sizeof(double));
      if (!c) {
#pragma omp critical
        status = ORC_NOMEM;
        continue;
      }
      for (int t = 0; t < T; ++t) {
        const double *xt = in + ((int64_t)t * B + b) * I;
        double *ht = out + ((int64_t)t * B + b) * N;
        for (int n = 0; n < N; ++n) {
          double a[4] = {0.0, p->b[0][n], p->b[1][n], 0.0};
          for (int g = 0; g < (p->W[3] ? 4 : 3); ++g) {
            const float *w = p->W[g] + (int64_t)n * I;
            for (int k = 0; k < I; ++k) a[g] += (double)w[k] * xt[k];
          }
          if (!p->W[3]) a[3] = xt[n];
          const double f = sigm(a[1] + (double)p->v[0][n] * c[n]);
          const double r = sigm(a[2] + (double)p->v[1][n] * c[n]);
          c[n] = f * c[n] + (1.0 - f) * a[0];
          ht[n] = r * c[n] + (1.0 - r) * a[3];
          const double mag = fmax(fabs(c[n]), fmax(fabs(a[0]), fabs(a[3])));
          if (mag > cmax) cmax = mag;
          if (ht[n] < hlo) hlo = ht[n];
          if (ht[n] > hhi) hhi = ht[n];
        }
      }
      free(c);
    }
    if (stats) {
      stats[l].c_absmax = cmax;
      stats[l].h_min = hlo;
      stats[l].h_max = hhi;
    }
    free(in);
    in = out;
  }
  if (status == ORC_OK && y) memcpy(y, in, sizeof(double) * (size_t)TB * layers[num_layers - 1].num_cells);
  free(in);
  return status;
}
