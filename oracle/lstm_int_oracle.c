/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT.  See lstm_int_oracle.h.
 *
 * Every integer step is written as exact arithmetic on int64_t with floor
 * division, in the order the paper's text and integer-execution figures give
 * it: no blocking, no fusion, no reordering.  One batch row at a time; the
 * only parallelism is OpenMP over batch rows, which never interact (eqs. 1-7
 * of Sec. 2 have no cross-row term and layer norm is per row, Sec. 3.2.6).
 */
#include "lstm_int_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ================================================================== */
/* Small helpers                                                       */
/* ================================================================== */

static int64_t floordiv(int64_t n, int64_t d) {
  int64_t q = n / d;
  if ((n % d != 0) && ((n < 0) != (d < 0))) q -= 1;
  return q;
}

static int64_t clamp64(int64_t v, int64_t lo, int64_t hi) {
  return v < lo ? lo : (v > hi ? hi : v);
}

static int64_t sat8(int64_t v) { return clamp64(v, -128, 127); }
static int64_t sat16(int64_t v) { return clamp64(v, -32768, 32767); }
static int64_t sat32(int64_t v) {
  return clamp64(v, -2147483647LL - 1, 2147483647LL);
}

int orc_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ================================================================== */
/* Fixed-point primitives                                              */
/* ================================================================== */

int64_t orc_rhu(int64_t n, int64_t d) { return floordiv(n + d / 2, d); }

int64_t orc_rsh_r(int64_t a, int k) {
  return floordiv(a + ((int64_t)1 << (k - 1)), (int64_t)1 << k);
}

/* The paper only names the operation ("rescale", Sec. 3.2.4); an effective
 * scale is represented here as a 31-bit integer multiplier and a power of
 * two, applied as one exact product and one rounding, ties toward +inf. */
int32_t orc_rescale(int64_t a, int32_t M, int e) {
  int r = 31 - e; /* 1..62 */
  int64_t p = a * (int64_t)M; /* |a| <= 2^31, M < 2^31: |p| <= 2^62 */
  return (int32_t)sat32(floordiv(p + ((int64_t)1 << (r - 1)), (int64_t)1 << r));
}

int orc_quantize_multiplier(double s, int32_t *M, int *e) {
  if (!(s > 0.0) || !isfinite(s)) return ORC_BAD_RANGE;
  int ex = 0;
  double q = frexp(s, &ex); /* s = q * 2^ex, q in [0.5, 1) */
  int64_t m = (int64_t)floor(q * 2147483648.0 + 0.5);
  if (m == 2147483648LL) {
    m = 1073741824LL;
    ex += 1;
  }
  if (ex < -31 || ex > 30) return ORC_UNSUPPORTED;
  *M = (int32_t)m;
  *e = ex;
  return ORC_OK;
}

/* floor(sqrt(v)) by bisection on the defining inequality r^2 <= v. */
int64_t orc_isqrt(int64_t v) {
  if (v <= 0) return 0;
  int64_t lo = 0, hi = 3037000499LL; /* floor(sqrt(2^63-1)) */
  while (lo < hi) {
    int64_t mid = lo + (hi - lo + 1) / 2;
    if (mid * mid <= v) lo = mid; else hi = mid - 1;
  }
  return lo;
}

/* Sec. 3.2.1 fixes the formats of sigma and tanh (16 bit, Q(m).(15-m) in,
 * Q0.15 out, no float, no table) but not an algorithm.  The one used here:
 * exp(-y) for y >= 0 from textbook identities only,
 *   exp(-y) = exp(-rho) * prod_k exp(-2^k)  over the set bits k of y above
 *   1/8, with exp(-rho) on [0, 1/8) by its degree-4 Taylor polynomial,
 * all in Q0.31 with round-half-up products; then
 *   sigma(x) = 1 / (1 + exp(-|x|)),  tanh(x) = (1 - exp(-2|x|)) / (1 + exp(-2|x|))
 * by one rounded division, mirrored for x < 0.
 * EXPC[j+3] = round(exp(-2^j) * 2^31), j = -3..4 (gen_constants.py). */
static const int64_t EXPC[8] = {1895147668LL, 1672461947LL, 1302514674LL,
                                790015084LL,  290630308LL,  39332535LL,
                                720401LL,     242LL};
static const int64_t TAYLOR_C3 = 357913941LL; /* round(2^31 / 6)  */
static const int64_t TAYLOR_C4 = 89478485LL;  /* round(2^31 / 24) */

static int64_t mulr31(int64_t a, int64_t b) {
  return floordiv(a * b + ((int64_t)1 << 30), (int64_t)1 << 31);
}

int64_t orc_expneg(int64_t y) {
  const int64_t one = (int64_t)1 << 31;
  if (y > ((int64_t)1 << 20) - 1) y = ((int64_t)1 << 20) - 1;
  int64_t rho = (y & 0xFFF) << 16; /* fraction below 1/8, as Q0.31 */
  int64_t u = TAYLOR_C3 - mulr31(rho, TAYLOR_C4);
  u = (one >> 1) - mulr31(rho, u);
  u = one - mulr31(rho, u);
  int64_t E = one - mulr31(rho, u);
  for (int k = 12; k <= 19; ++k)
    if ((y >> k) & 1) E = mulr31(E, EXPC[k - 12]);
  return E;
}

int32_t orc_int_sigmoid(int32_t x, int m) {
  const int64_t one = (int64_t)1 << 31;
  int64_t a = x < 0 ? -(int64_t)x : (int64_t)x;
  int64_t E = orc_expneg(a << m);
  int64_t s = orc_rhu((int64_t)1 << 46, one + E);
  if (x < 0) s = 32768 - s;
  return (int32_t)clamp64(s, 0, 32767);
}

int32_t orc_int_tanh(int32_t x, int m) {
  const int64_t one = (int64_t)1 << 31;
  int64_t a = x < 0 ? -(int64_t)x : (int64_t)x;
  int64_t E = orc_expneg(a << (m + 1));
  int64_t t = orc_rhu((one - E) << 15, one + E);
  if (x < 0) t = -t;
  return (int32_t)clamp64(t, -32768, 32767);
}

/* Sec. 3.2.6, the four integer equations after "the integer inference
 * becomes", with s' = 2^-10.  The printed variance has the mean inside the
 * sum; it is read as E[q^2] - mean^2.  The printed q' = (2^10 q - qbar) /
 * sigma has lost the factor 1/s' of its own definition q' = x'/s' two lines
 * above it (qbar and sigma both carry 2^10, so the printed quotient is x'
 * itself, the 2.8-bit value the section sets out to avoid, and the bias scale
 * 2^-10 s_L of Table 2 would not match it); the factor is restored:
 * q' = round(2^10 (2^10 q - qbar) / sigma).  Not fixed by the paper and
 * chosen here: the root is floored, a negative variance (possible only
 * through the rounding of the mean) is taken as 0, sigma = 0 gives q' = 0,
 * q' is not clamped, and the "rescale -> Q3.12" box of the integer-execution
 * figure is applied after the printed division by 2^10 (q'' carries the
 * scale s_L, so the effective scale of that second stage is s_L * 2^12). */
int orc_int_layernorm(const int16_t *q, int n, const int16_t *qL,
                      const int32_t *qb, int32_t M_ln, int e_ln, int16_t *out) {
  if (n < 1 || n > 4096) return ORC_UNSUPPORTED;
  int64_t S1 = 0, S2 = 0;
  for (int i = 0; i < n; ++i) {
    S1 += q[i];
    S2 += (int64_t)q[i] * q[i];
  }
  int64_t mean = orc_rhu(S1 * 1024, n);
  int64_t var = orc_rhu(S2 * 1048576, n) - mean * mean;
  if (var < 0) var = 0;
  int64_t sigma = orc_isqrt(var);
  for (int i = 0; i < n; ++i) {
    int64_t qn = (sigma == 0) ? 0 : orc_rhu(1024 * (1024 * (int64_t)q[i] - mean), sigma);
    int64_t t = qn * qL[i] + qb[i];
    int64_t q2 = sat32(orc_rsh_r(t, 10));
    out[i] = (int16_t)sat16(orc_rescale(q2, M_ln, e_ln));
  }
  return ORC_OK;
}

/* ================================================================== */
/* Prepare (Table 2 and Secs. 3.2.2-3.2.9, Sec. 6)                     */
/* ================================================================== */

/* Float -> integer rounding is floor(v + 1/2) in double everywhere. */
static double round_half_up(double v) { return floor(v + 0.5); }

static int finite_array(const float *a, int64_t n) {
  for (int64_t i = 0; i < n; ++i)
    if (!isfinite(a[i])) return 0;
  return 1;
}

static double max_abs(const float *a, int64_t n) {
  double m = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double v = fabs((double)a[i]);
    if (v > m) m = v;
  }
  return m;
}

/* symmetric: s = max|w| / qmax (s = 1 for an all-zero tensor) */
static double sym_scale(const float *a, int64_t n, double qmax) {
  double m = max_abs(a, n);
  return m == 0.0 ? 1.0 : m / qmax;
}

static int64_t sym_quant(double v, double s, int64_t qmax) {
  double r = round_half_up(v / s);
  if (r < (double)-qmax) r = (double)-qmax;
  if (r > (double)qmax) r = (double)qmax;
  return (int64_t)r;
}

/* asymmetric int8 (Sec. 3.2.4): the range is widened to contain 0, and the
 * zero point is rounded to an integer so that real 0 is a code ("nudged").
 * real = s * (q - zp). */
static int asym_params(double lo_in, double hi_in, double *s, int32_t *zp) {
  if (!isfinite(lo_in) || !isfinite(hi_in) || lo_in > hi_in) return ORC_BAD_RANGE;
  double lo = lo_in < 0.0 ? lo_in : 0.0;
  double hi = hi_in > 0.0 ? hi_in : 0.0;
  double sc = (hi - lo) / 255.0;
  if (sc == 0.0) sc = 1.0;
  double z = round_half_up(-128.0 - lo / sc);
  if (z < -128.0) z = -128.0;
  if (z > 127.0) z = 127.0;
  *s = sc;
  *zp = (int32_t)z;
  return ORC_OK;
}

static void free_layer(orc_layer_quant *q) {
  free(q->Wq); free(q->Rq); free(q->qb); free(q->Pq); free(q->Lq);
  free(q->Wpq); free(q->qbp); free(q->bx_fold); free(q->bh_fold);
  free(q->bp_fold);
  memset(q, 0, sizeof(*q));
}

void orc_destroy(orc_model *m) {
  if (!m) return;
  if (m->layers) {
    for (int l = 0; l < m->num_layers; ++l) free_layer(&m->layers[l]);
    free(m->layers);
  }
  free(m);
}

const orc_layer_quant *orc_get_layer(const orc_model *m, int32_t layer) {
  if (!m || layer < 0 || layer >= m->num_layers) return NULL;
  return &m->layers[layer];
}

/* sum_k w[k], and the worst-case |accumulator| for any int8 input row:
 * |bias| + 128 * sum_k |w[k]| must stay inside int32 (Sec. 3.1.1). */
static int fold_check(const int8_t *w, int K, int64_t zp, int64_t qb,
                      int32_t *folded) {
  int64_t sum = 0, sum_abs = 0;
  for (int k = 0; k < K; ++k) {
    sum += w[k];
    sum_abs += w[k] < 0 ? -(int64_t)w[k] : (int64_t)w[k];
  }
  int64_t f = qb - zp * sum;
  int64_t fa = f < 0 ? -f : f;
  if (fa + 128 * sum_abs > 2147483647LL) return ORC_UNSUPPORTED;
  *folded = (int32_t)f;
  return ORC_OK;
}

static int prepare_layer(const orc_layer_params *p, int has_prev, double prev_s,
                         int32_t prev_zp, orc_layer_quant *q) {
  memset(q, 0, sizeof(*q));
  const uint32_t fl = p->flags;
  const int cifg = (fl & ORC_CIFG) != 0, ph = (fl & ORC_PEEPHOLE) != 0;
  const int ln = (fl & ORC_LAYER_NORM) != 0, proj = (fl & ORC_PROJECTION) != 0;
  if (fl & ~15u) return ORC_INVALID_ARG;
  const int I = p->input_size, N = p->num_cells, H = p->output_size;
  if (I < 1 || N < 1 || H < 1) return ORC_INVALID_ARG;
  if (!proj && H != N) return ORC_INVALID_ARG;
  /* safe accumulation depth of int8 x int8 -> int32, Sec. 3.1.1 */
  if (I > 32768 || H > 32768 || N > 32768) return ORC_UNSUPPORTED;
  if (ln && N > 4096) return ORC_UNSUPPORTED;
  const int g0 = cifg ? 1 : 0;
  for (int g = 0; g < 4; ++g) {
    int present = g >= g0;
    if (present != (p->W[g] != NULL) || present != (p->R[g] != NULL) ||
        present != (p->b[g] != NULL))
      return ORC_INVALID_ARG; /* the dagger rows of Table 2 are void under CIFG */
    if (ln ? present != (p->Lw[g] != NULL) : p->Lw[g] != NULL) return ORC_INVALID_ARG;
  }
  for (int j = 0; j < 3; ++j) {
    int present = ph && !(cifg && j == 0);
    if (present != (p->P[j] != NULL)) return ORC_INVALID_ARG;
  }
  if (proj != (p->Wproj != NULL)) return ORC_INVALID_ARG;
  if (!proj && p->bproj) return ORC_INVALID_ARG;

  q->I = I; q->N = N; q->H = H; q->G = cifg ? 3 : 4; q->flags = fl;

  /* --- activations: x, h, m (Table 2 rows x, h, m) --- */
  int rc;
  if (has_prev) {
    q->s_x = prev_s; /* a stacked layer reads the previous layer's h */
    q->zp_x = prev_zp;
  } else if ((rc = asym_params(p->x_min, p->x_max, &q->s_x, &q->zp_x)) != ORC_OK)
    return rc;
  if ((rc = asym_params(p->h_min, p->h_max, &q->s_h, &q->zp_h)) != ORC_OK) return rc;
  if (proj) {
    if ((rc = asym_params(p->m_min, p->m_max, &q->s_m, &q->zp_m)) != ORC_OK) return rc;
  } else {
    q->s_m = q->s_h; /* h = m without projection */
    q->zp_m = q->zp_h;
  }

  /* --- cell state: measured range extended to a power of two (Sec. 3.2.2) --- */
  double ca = p->c_absmax;
  if (!isfinite(ca) || ca < 0.0) return ORC_BAD_RANGE;
  int mc = 0;
  while (mc <= 8 && ldexp(1.0, mc) < ca) ++mc;
  if (mc > 8) return ORC_UNSUPPORTED;
  q->m_c = mc;
  q->s_c = ldexp(1.0, mc - 15);

  q->Wq = calloc((size_t)4 * N * I, 1);
  q->Rq = calloc((size_t)4 * N * H, 1);
  q->qb = calloc((size_t)4 * N, sizeof(int32_t));
  q->Pq = calloc((size_t)3 * N, sizeof(int16_t));
  q->Lq = calloc((size_t)4 * N, sizeof(int16_t));
  q->bx_fold = calloc((size_t)4 * N, sizeof(int32_t));
  q->bh_fold = calloc((size_t)4 * N, sizeof(int32_t));
  q->Wpq = calloc(proj ? (size_t)H * N : 1, 1);
  q->qbp = calloc(proj ? (size_t)H : 1, sizeof(int32_t));
  q->bp_fold = calloc(proj ? (size_t)H : 1, sizeof(int32_t));
  if (!q->Wq || !q->Rq || !q->qb || !q->Pq || !q->Lq || !q->bx_fold ||
      !q->bh_fold || !q->Wpq || !q->qbp || !q->bp_fold)
    return ORC_NOMEM;

  for (int g = g0; g < 4; ++g) {
    if (!finite_array(p->W[g], (int64_t)N * I) || !finite_array(p->R[g], (int64_t)N * H) ||
        !finite_array(p->b[g], N))
      return ORC_BAD_RANGE;
    /* --- W, R: symmetric int8, +-127 (Sec. 3.2.4) --- */
    q->s_W[g] = sym_scale(p->W[g], (int64_t)N * I, 127.0);
    q->s_R[g] = sym_scale(p->R[g], (int64_t)N * H, 127.0);
    for (int64_t i = 0; i < (int64_t)N * I; ++i)
      q->Wq[(int64_t)g * N * I + i] = (int8_t)sym_quant(p->W[g][i], q->s_W[g], 127);
    for (int64_t i = 0; i < (int64_t)N * H; ++i)
      q->Rq[(int64_t)g * N * H + i] = (int8_t)sym_quant(p->R[g][i], q->s_R[g], 127);

    /* --- gate output scale: Q3.12 (Sec. 3.2.4) or measured (Sec. 3.2.5) --- */
    if (ln) {
      double ga = p->g_absmax[g];
      if (!isfinite(ga) || ga < 0.0) return ORC_BAD_RANGE;
      q->s_g[g] = ga == 0.0 ? 1.0 : ga / 32767.0;
    } else {
      q->s_g[g] = ldexp(1.0, -12);
    }

    /* --- bias: int32 at s_R s_h (Sec. 3.2.4) or 2^-10 s_L (Sec. 3.2.6) --- */
    double s_b;
    if (ln) {
      if (!finite_array(p->Lw[g], N)) return ORC_BAD_RANGE;
      q->s_L[g] = sym_scale(p->Lw[g], N, 32767.0);
      for (int n = 0; n < N; ++n)
        q->Lq[g * N + n] = (int16_t)sym_quant(p->Lw[g][n], q->s_L[g], 32767);
      s_b = ldexp(1.0, -10) * q->s_L[g];
    } else {
      s_b = q->s_R[g] * q->s_h;
    }
    for (int n = 0; n < N; ++n)
      q->qb[g * N + n] = (int32_t)sym_quant(p->b[g][n], s_b, 2147483647LL);

    /* --- effective scales (Secs. 3.2.4, 3.2.5) --- */
    if ((rc = orc_quantize_multiplier(q->s_W[g] * q->s_x / q->s_g[g], &q->Mx[g], &q->ex[g])) != ORC_OK) return rc;
    if ((rc = orc_quantize_multiplier(q->s_R[g] * q->s_h / q->s_g[g], &q->Mh[g], &q->eh[g])) != ORC_OK) return rc;
    if (ln &&
        (rc = orc_quantize_multiplier(q->s_L[g] * 4096.0, &q->Mln[g], &q->eln[g])) != ORC_OK)
      return rc;

    /* --- zero points folded into the biases (Sec. 6) --- */
    for (int n = 0; n < N; ++n) {
      if ((rc = fold_check(q->Wq + ((int64_t)g * N + n) * I, I, q->zp_x, 0,
                           &q->bx_fold[g * N + n])) != ORC_OK) return rc;
      if ((rc = fold_check(q->Rq + ((int64_t)g * N + n) * H, H, q->zp_h,
                           ln ? 0 : q->qb[g * N + n], &q->bh_fold[g * N + n])) != ORC_OK) return rc;
    }
  }

  /* --- peephole: int16 +-32767 (Sec. 3.2.3); gates i, f, o --- */
  if (ph) {
    for (int j = g0; j < 3; ++j) {
      int g = j == 2 ? ORC_GO : j;
      if (!finite_array(p->P[j], N)) return ORC_BAD_RANGE;
      q->s_P[j] = sym_scale(p->P[j], N, 32767.0);
      for (int n = 0; n < N; ++n)
        q->Pq[j * N + n] = (int16_t)sym_quant(p->P[j][n], q->s_P[j], 32767);
      if ((rc = orc_quantize_multiplier(q->s_P[j] * q->s_c / q->s_g[g], &q->Mc[j], &q->ec[j])) != ORC_OK) return rc;
    }
  }

  /* --- hidden state: o.tanh(c) is Q0.30 (Sec. 3.2.7) --- */
  if ((rc = orc_quantize_multiplier(ldexp(1.0, -30) / q->s_m, &q->Mm, &q->em)) != ORC_OK) return rc;

  /* --- projection (Sec. 3.2.8) --- */
  if (proj) {
    if (!finite_array(p->Wproj, (int64_t)H * N)) return ORC_BAD_RANGE;
    if (p->bproj && !finite_array(p->bproj, H)) return ORC_BAD_RANGE;
    q->s_Wp = sym_scale(p->Wproj, (int64_t)H * N, 127.0);
    for (int64_t i = 0; i < (int64_t)H * N; ++i)
      q->Wpq[i] = (int8_t)sym_quant(p->Wproj[i], q->s_Wp, 127);
    double s_b = q->s_Wp * q->s_m;
    for (int j = 0; j < H; ++j) {
      q->qbp[j] = p->bproj ? (int32_t)sym_quant(p->bproj[j], s_b, 2147483647LL) : 0;
      if ((rc = fold_check(q->Wpq + (int64_t)j * N, N, q->zp_m, q->qbp[j], &q->bp_fold[j])) != ORC_OK) return rc;
    }
    if ((rc = orc_quantize_multiplier(q->s_Wp * q->s_m / q->s_h, &q->Mp, &q->ep)) != ORC_OK) return rc;
  }
  return ORC_OK;
}

int orc_prepare(const orc_layer_params *layers, int32_t num_layers, orc_model **out) {
  if (!layers || !out || num_layers < 1) return ORC_INVALID_ARG;
  *out = NULL;
  orc_model *m = calloc(1, sizeof(*m));
  if (!m) return ORC_NOMEM;
  m->layers = calloc((size_t)num_layers, sizeof(orc_layer_quant));
  if (!m->layers) { free(m); return ORC_NOMEM; }
  m->num_layers = num_layers;
  for (int l = 0; l < num_layers; ++l) {
    if (l > 0 && layers[l].input_size != layers[l - 1].output_size) {
      orc_destroy(m);
      return ORC_INVALID_ARG;
    }
    int rc = prepare_layer(&layers[l], l > 0, l > 0 ? m->layers[l - 1].s_h : 0.0,
                           l > 0 ? m->layers[l - 1].zp_h : 0, &m->layers[l]);
    if (rc != ORC_OK) { orc_destroy(m); return rc; }
  }
  *out = m;
  return ORC_OK;
}

/* ================================================================== */
/* Integer forward                                                     */
/* ================================================================== */

/* int8 x int8 accumulation as the plain definition, in int64.  The folded
 * form is sum w*q + b'; the unfolded form is sum w*(q - zp) + b (Sec. 6). */
static int64_t dot_i8(const int8_t *w, const int8_t *a, int K, int64_t zp,
                      int64_t bias, int unfolded) {
  int64_t acc = 0;
  if (unfolded)
    for (int k = 0; k < K; ++k) acc += (int64_t)w[k] * ((int64_t)a[k] - zp);
  else
    for (int k = 0; k < K; ++k) acc += (int64_t)w[k] * (int64_t)a[k];
  return acc + bias;
}

typedef struct {
  int16_t *tx, *th, *g, *ln, *act, *c;
  int8_t *m, *h;
} row_trace; /* pointers already offset to (t, b) */

/* One cell step for one batch row (Secs. 3.2.4-3.2.9).
 * x[I], h_prev[H], c[N] (updated in place), h_out[H].
 * scratch: 4*N int16 for gate sums, 4*N int16 for gate inputs to the
 * activations, N int8 for m. */
static int cell_step(const orc_layer_quant *q, const int8_t *x, const int8_t *h_prev,
                     int16_t *c, int8_t *h_out, int unfolded, const row_trace *tr,
                     int16_t *gsum, int16_t *gin, int16_t *act, int8_t *mq) {
  const int I = q->I, N = q->N, H = q->H;
  const int cifg = (q->flags & ORC_CIFG) != 0, ph = (q->flags & ORC_PEEPHOLE) != 0;
  const int ln = (q->flags & ORC_LAYER_NORM) != 0, proj = (q->flags & ORC_PROJECTION) != 0;
  const int64_t glo = ln ? -32767 : -32768; /* Sec. 3.2.5 vs Sec. 3.2.4 */

  /* gates are taken in the order i, f, z, then the cell, then o: the output
   * gate's peephole reads the new cell state (eq. 5) */
  for (int pass = 0; pass < 2; ++pass) {
    for (int g = cifg ? 1 : 0; g < 4; ++g) {
      if ((pass == 0) != (g != ORC_GO)) continue;
      const int pj = g == ORC_GO ? 2 : g; /* peephole slot; unused for z */
      for (int n = 0; n < N; ++n) {
        const int gn = g * N + n;
        int64_t accx = dot_i8(q->Wq + (int64_t)gn * I, x, I, q->zp_x,
                              unfolded ? 0 : q->bx_fold[gn], unfolded);
        int64_t acch = dot_i8(q->Rq + (int64_t)gn * H, h_prev, H, q->zp_h,
                              unfolded ? (ln ? 0 : q->qb[gn]) : q->bh_fold[gn], unfolded);
        if (accx != sat32(accx) || acch != sat32(acch)) return ORC_UNSUPPORTED;
        int64_t tx = sat16(orc_rescale(accx, q->Mx[g], q->ex[g]));
        int64_t th = sat16(orc_rescale(acch, q->Mh[g], q->eh[g]));
        int64_t tc = 0;
        if (ph && g != ORC_GZ) /* c is c^{t-1} in pass 0 and c^t in pass 1 */
          tc = sat16(orc_rescale((int64_t)q->Pq[pj * N + n] * c[n], q->Mc[pj], q->ec[pj]));
        gsum[gn] = (int16_t)clamp64(tx + th + tc, glo, 32767);
        if (tr->tx) tr->tx[gn] = (int16_t)tx;
        if (tr->th) tr->th[gn] = (int16_t)th;
        if (tr->g) tr->g[gn] = gsum[gn];
      }
      if (ln) {
        int rc = orc_int_layernorm(gsum + g * N, N, q->Lq + g * N, q->qb + g * N,
                                   q->Mln[g], q->eln[g], gin + g * N);
        if (rc != ORC_OK) return rc;
        if (tr->ln) memcpy(tr->ln + g * N, gin + g * N, sizeof(int16_t) * N);
      } else {
        memcpy(gin + g * N, gsum + g * N, sizeof(int16_t) * N);
      }
      for (int n = 0; n < N; ++n) /* Sec. 3.2.1: gate inputs are Q3.12 */
        act[g * N + n] = (int16_t)(g == ORC_GZ ? orc_int_tanh(gin[g * N + n], 3)
                                               : orc_int_sigmoid(gin[g * N + n], 3));
    }
    if (pass == 0) {
      for (int n = 0; n < N; ++n) {
        /* Sec. 3.2.9; the printed max() cannot "fit in int16", min() can */
        if (cifg) act[n] = (int16_t)(32768 - act[N + n] < 32767 ? 32768 - act[N + n] : 32767);
        /* Sec. 3.2.7: Q0.30 -> Q(m_c).(15-m_c) is a shift by 15 + m_c;
         * f.c is Q(m_c).(30-m_c), a shift by 15 */
        int64_t iz = orc_rsh_r((int64_t)act[n] * act[2 * N + n], 15 + q->m_c);
        int64_t fc = orc_rsh_r((int64_t)act[N + n] * c[n], 15);
        c[n] = (int16_t)sat16(iz + fc);
      }
    }
  }
  for (int n = 0; n < N; ++n) {
    /* the cell state goes to tanh in its own format (Sec. 3.2.2) */
    int64_t tc = orc_int_tanh(c[n], q->m_c);
    int64_t prod = (int64_t)act[3 * N + n] * tc; /* Q0.30 */
    mq[n] = (int8_t)sat8((int64_t)orc_rescale(prod, q->Mm, q->em) + q->zp_m);
  }
  if (proj) {
    for (int j = 0; j < H; ++j) {
      int64_t acc = dot_i8(q->Wpq + (int64_t)j * N, mq, N, q->zp_m,
                           unfolded ? q->qbp[j] : q->bp_fold[j], unfolded);
      if (acc != sat32(acc)) return ORC_UNSUPPORTED;
      h_out[j] = (int8_t)sat8((int64_t)orc_rescale(acc, q->Mp, q->ep) + q->zp_h);
    }
  } else {
    memcpy(h_out, mq, (size_t)N);
  }
  if (tr->act) memcpy(tr->act, act, sizeof(int16_t) * 4 * N);
  if (tr->c) memcpy(tr->c, c, sizeof(int16_t) * N);
  if (tr->m) memcpy(tr->m, mq, (size_t)N);
  if (tr->h) memcpy(tr->h, h_out, (size_t)H);
  return ORC_OK;
}

int orc_forward(const orc_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                int8_t *h_state, int16_t *c_state, const orc_trace *trace,
                int unfolded, int threads) {
  if (!m || !x || !y || T < 0 || B < 0) return ORC_INVALID_ARG;
  if (trace && (trace->layer < 0 || trace->layer >= m->num_layers)) return ORC_INVALID_ARG;
  if (T == 0 || B == 0) return ORC_OK;
  if (threads < 1) threads = 1;
  const int L = m->num_layers;
  int status = ORC_OK;
  const int8_t *in = x;
  int8_t *buf[2] = {NULL, NULL};
  int64_t h_off = 0, c_off = 0;
  for (int l = 0; l < L; ++l) {
    const orc_layer_quant *q = &m->layers[l];
    const int I = q->I, N = q->N, H = q->H;
    int8_t *out = y;
    if (l != L - 1) {
      buf[l & 1] = realloc(buf[l & 1], (size_t)T * B * H);
      if (!buf[l & 1]) { status = ORC_NOMEM; break; }
      out = buf[l & 1];
    }
    const orc_trace *tl = (trace && trace->layer == l) ? trace : NULL;
    int8_t *hs = h_state ? h_state + h_off : NULL;
    int16_t *cs = c_state ? c_state + c_off : NULL;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int b = 0; b < B; ++b) {
      int16_t *c = malloc(sizeof(int16_t) * (size_t)N * 13 + (size_t)N + (size_t)H);
      if (!c) {
#pragma omp critical
        status = ORC_NOMEM;
        continue;
      }
      int16_t *gsum = c + N, *gin = c + 5 * N, *act = c + 9 * N;
      int8_t *mq = (int8_t *)(c + 13 * N), *h0 = mq + N;
      memset(act, 0, sizeof(int16_t) * 4 * N);
      /* initial state: real 0, i.e. q = zp_h, and c = 0, unless given */
      for (int j = 0; j < H; ++j) h0[j] = hs ? hs[(int64_t)b * H + j] : (int8_t)q->zp_h;
      for (int n = 0; n < N; ++n) c[n] = cs ? cs[(int64_t)b * N + n] : 0;
      for (int t = 0; t < T; ++t) {
        const int64_t tb = (int64_t)t * B + b;
        const int8_t *hp = t == 0 ? h0 : out + ((int64_t)(t - 1) * B + b) * H;
        row_trace rt;
        memset(&rt, 0, sizeof(rt));
        if (tl) {
          rt.tx = tl->tx ? tl->tx + tb * 4 * N : NULL;
          rt.th = tl->th ? tl->th + tb * 4 * N : NULL;
          rt.g = tl->g ? tl->g + tb * 4 * N : NULL;
          rt.ln = tl->ln ? tl->ln + tb * 4 * N : NULL;
          rt.act = tl->act ? tl->act + tb * 4 * N : NULL;
          rt.c = tl->c ? tl->c + tb * N : NULL;
          rt.m = tl->m ? tl->m + tb * N : NULL;
          rt.h = tl->h ? tl->h + tb * H : NULL;
        }
        int rc = cell_step(q, in + tb * I, hp, c, out + tb * H, unfolded, &rt, gsum,
                           gin, act, mq);
        if (rc != ORC_OK) {
#pragma omp critical
          status = rc;
          break;
        }
      }
      if (hs) memcpy(hs + (int64_t)b * H, out + ((int64_t)(T - 1) * B + b) * H, (size_t)H);
      if (cs) memcpy(cs + (int64_t)b * N, c, sizeof(int16_t) * N);
      free(c);
    }
    if (status != ORC_OK) break;
    in = out;
    h_off += (int64_t)B * H;
    c_off += (int64_t)B * N;
  }
  free(buf[0]);
  free(buf[1]);
  return status;
}

/* ================================================================== */
/* Float LSTM, eqs. (1)-(7) of Sec. 2, in double                        */
/* ================================================================== */

static double sigmoid_d(double v) { return 1.0 / (1.0 + exp(-v)); }

static void stat_minmax(double v, double *lo, double *hi) {
  if (v < *lo) *lo = v;
  if (v > *hi) *hi = v;
}

/* norm() of Sec. 3.2.6: zero mean, unit standard deviation (population
 * variance, no epsilon; a constant row maps to zeros), then * L + b. */
static void layernorm_d(double *v, int n, const float *Lw, const float *b) {
  double mean = 0.0, var = 0.0;
  for (int i = 0; i < n; ++i) mean += v[i];
  mean /= n;
  for (int i = 0; i < n; ++i) var += (v[i] - mean) * (v[i] - mean);
  var /= n;
  double sd = sqrt(var);
  for (int i = 0; i < n; ++i)
    v[i] = (sd > 0.0 ? (v[i] - mean) / sd : 0.0) * (double)Lw[i] + (double)b[i];
}

int orc_float_forward(const orc_layer_params *layers, int32_t num_layers, const float *x,
                      int32_t T, int32_t B, double *y, orc_float_stats *stats,
                      int threads) {
  if (!layers || !x || num_layers < 1 || T < 1 || B < 1) return ORC_INVALID_ARG;
  if (threads < 1) threads = 1;
  int status = ORC_OK;
  double *in = malloc(sizeof(double) * (size_t)T * B * layers[0].input_size);
  if (!in) return ORC_NOMEM;
  for (int64_t i = 0; i < (int64_t)T * B * layers[0].input_size; ++i) in[i] = x[i];
  for (int l = 0; l < num_layers && status == ORC_OK; ++l) {
    const orc_layer_params *p = &layers[l];
    const int I = p->input_size, N = p->num_cells, H = p->output_size;
    const int cifg = (p->flags & ORC_CIFG) != 0, ph = (p->flags & ORC_PEEPHOLE) != 0;
    const int ln = (p->flags & ORC_LAYER_NORM) != 0, proj = (p->flags & ORC_PROJECTION) != 0;
    double *out = malloc(sizeof(double) * (size_t)T * B * H);
    if (!out) { status = ORC_NOMEM; break; }
    orc_float_stats st;
    st.x_min = st.h_min = st.m_min = INFINITY;
    st.x_max = st.h_max = st.m_max = -INFINITY;
    st.c_absmax = 0.0;
    for (int g = 0; g < 4; ++g) st.g_absmax[g] = 0.0;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int b = 0; b < B; ++b) {
      orc_float_stats ls = st;
      double *c = calloc((size_t)N * 6 + H, sizeof(double));
      if (!c) {
#pragma omp critical
        status = ORC_NOMEM;
        continue;
      }
      double *pre = c + N, *mm = c + 5 * N, *h0 = c + 6 * N; /* h0 = zeros */
      for (int t = 0; t < T; ++t) {
        const double *xv = in + ((int64_t)t * B + b) * I;
        const double *hp = t == 0 ? h0 : out + ((int64_t)(t - 1) * B + b) * H;
        double *ho = out + ((int64_t)t * B + b) * H;
        for (int k = 0; k < I; ++k) stat_minmax(xv[k], &ls.x_min, &ls.x_max);
        for (int pass = 0; pass < 2; ++pass) {
          for (int g = cifg ? 1 : 0; g < 4; ++g) {
            if ((pass == 0) != (g != ORC_GO)) continue;
            const int pj = g == ORC_GO ? 2 : g;
            double *pg = pre + g * N;
            for (int n = 0; n < N; ++n) {
              double a = 0.0;
              const float *w = p->W[g] + (int64_t)n * I, *r = p->R[g] + (int64_t)n * H;
              for (int k = 0; k < I; ++k) a += (double)w[k] * xv[k];
              for (int k = 0; k < H; ++k) a += (double)r[k] * hp[k];
              if (ph && g != ORC_GZ) a += (double)p->P[pj][n] * c[n];
              if (!ln) a += (double)p->b[g][n];
              pg[n] = a;
            }
            if (ln) {
              for (int n = 0; n < N; ++n)
                if (fabs(pg[n]) > ls.g_absmax[g]) ls.g_absmax[g] = fabs(pg[n]);
              layernorm_d(pg, N, p->Lw[g], p->b[g]);
            }
            for (int n = 0; n < N; ++n) pg[n] = g == ORC_GZ ? tanh(pg[n]) : sigmoid_d(pg[n]);
          }
          if (pass == 0)
            for (int n = 0; n < N; ++n) {
              double ig = cifg ? 1.0 - pre[N + n] : pre[n];
              c[n] = ig * pre[2 * N + n] + pre[N + n] * c[n];
              if (fabs(c[n]) > ls.c_absmax) ls.c_absmax = fabs(c[n]);
            }
        }
        for (int n = 0; n < N; ++n) {
          mm[n] = pre[3 * N + n] * tanh(c[n]);
          stat_minmax(mm[n], &ls.m_min, &ls.m_max);
        }
        if (proj) {
          for (int j = 0; j < H; ++j) {
            double a = p->bproj ? (double)p->bproj[j] : 0.0;
            const float *w = p->Wproj + (int64_t)j * N;
            for (int n = 0; n < N; ++n) a += (double)w[n] * mm[n];
            ho[j] = a;
          }
        } else {
          memcpy(ho, mm, sizeof(double) * N);
        }
        for (int j = 0; j < H; ++j) stat_minmax(ho[j], &ls.h_min, &ls.h_max);
      }
      free(c);
#pragma omp critical
      {
        stat_minmax(ls.x_min, &st.x_min, &st.x_max); stat_minmax(ls.x_max, &st.x_min, &st.x_max);
        stat_minmax(ls.h_min, &st.h_min, &st.h_max); stat_minmax(ls.h_max, &st.h_min, &st.h_max);
        stat_minmax(ls.m_min, &st.m_min, &st.m_max); stat_minmax(ls.m_max, &st.m_min, &st.m_max);
        if (ls.c_absmax > st.c_absmax) st.c_absmax = ls.c_absmax;
        for (int g = 0; g < 4; ++g)
          if (ls.g_absmax[g] > st.g_absmax[g]) st.g_absmax[g] = ls.g_absmax[g];
      }
    }
    if (stats) stats[l] = st;
    if (y && l == num_layers - 1) memcpy(y, out, sizeof(double) * (size_t)T * B * H);
    free(in);
    in = out;
  }
  free(in);
  return status;
}
