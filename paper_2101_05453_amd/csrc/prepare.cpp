// Offline phase of the integer LSTM (arXiv 2101.05453, Table 2, Secs. 3.2.1-
// 3.2.9 and Sec. 6): float parameters and calibration statistics in, integer
// tensors, zero points, effective scales as (M, e) pairs and folded biases
// out.  Host only; double precision, with every float -> integer rounding
// taken as floor(v + 1/2).
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <limits>

#include "lstm_int_math.h"
#include "model.h"

namespace lstm_int {

namespace {

constexpr double kInt32Max = 2147483647.0;

bool all_finite(const float *a, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!std::isfinite(a[i])) return false;
  return true;
}

// Symmetric quantization of one tensor: scale = max|v| / qmax (1 if the
// tensor is all zero), q = clamp(round(v / scale), -qmax, qmax).
template <typename T>
double quantize_symmetric(const float *src, size_t n, double qmax, T *dst) {
  double amax = 0.0;
  for (size_t i = 0; i < n; ++i) amax = std::fmax(amax, std::fabs((double)src[i]));
  const double scale = amax == 0.0 ? 1.0 : amax / qmax;
  for (size_t i = 0; i < n; ++i) {
    double r = std::floor((double)src[i] / scale + 0.5);
    r = std::fmin(std::fmax(r, -qmax), qmax);
    dst[i] = (T)r;
  }
  return scale;
}

int32_t quantize_bias(double v, double scale) {
  double r = std::floor(v / scale + 0.5);
  r = std::fmin(std::fmax(r, -kInt32Max), kInt32Max);
  return (int32_t)r;
}

// Asymmetric int8 of Sec. 3.2.4: the range is widened to include 0 and the
// zero point rounded to an integer code, so real 0 is exactly representable.
int asymmetric_params(float vmin, float vmax, double *scale, int32_t *zp) {
  if (!std::isfinite(vmin) || !std::isfinite(vmax) || vmin > vmax) return LSTM_INT_E_BAD_RANGE;
  const double lo = std::fmin((double)vmin, 0.0), hi = std::fmax((double)vmax, 0.0);
  double s = (hi - lo) / 255.0;
  if (s == 0.0) s = 1.0;
  double z = std::floor(-128.0 - lo / s + 0.5);
  z = std::fmin(std::fmax(z, -128.0), 127.0);
  *scale = s;
  *zp = (int32_t)z;
  return LSTM_INT_OK;
}

// Sec. 6: sum_k w (a - zp) + b = sum_k w a + (b - zp sum_k w).  The folded
// bias must leave room for the largest accumulation any int8 input can
// produce, |b'| + 128 sum|w| <= 2^31 - 1, so the int32 accumulator is exact.
int fold_zero_point(const int8_t *w, int K, int32_t zp, int32_t bias, int32_t *folded) {
  int64_t sum = 0, mag = 0;
  for (int k = 0; k < K; ++k) {
    sum += w[k];
    mag += std::abs((int)w[k]);
  }
  const int64_t f = (int64_t)bias - (int64_t)zp * sum;
  if (std::llabs(f) + 128 * mag > 2147483647LL) return LSTM_INT_E_UNSUPPORTED;
  *folded = (int32_t)f;
  return LSTM_INT_OK;
}

int prepare_layer(const lstm_int_layer_params &p, const LayerHost *prev, LayerHost &q) {
  if (p.flags & ~15u) return LSTM_INT_E_INVALID_ARG;
  q.flags = p.flags;
  q.I = p.input_size;
  q.N = p.num_cells;
  q.H = p.output_size;
  q.G = q.cifg() ? 3 : 4;
  const int I = q.I, N = q.N, H = q.H;
  if (I < 1 || N < 1 || H < 1) return LSTM_INT_E_INVALID_ARG;
  if (!q.projection() && H != N) return LSTM_INT_E_INVALID_ARG;
  if (I > 32768 || N > 32768 || H > 32768) return LSTM_INT_E_UNSUPPORTED;  // Sec. 3.1.1
  if (q.layer_norm() && N > 4096) return LSTM_INT_E_UNSUPPORTED;
  const int first = q.cifg() ? 1 : 0;

  // which tensors must be present for this variant (Table 2)
  for (int g = 0; g < 4; ++g) {
    const bool want = g >= first;
    if ((p.W[g] != nullptr) != want || (p.R[g] != nullptr) != want || (p.b[g] != nullptr) != want)
      return LSTM_INT_E_INVALID_ARG;
    if ((p.Lw[g] != nullptr) != (want && q.layer_norm())) return LSTM_INT_E_INVALID_ARG;
  }
  for (int j = 0; j < 3; ++j)
    if ((p.P[j] != nullptr) != (q.peephole() && j >= first)) return LSTM_INT_E_INVALID_ARG;
  if ((p.Wproj != nullptr) != q.projection()) return LSTM_INT_E_INVALID_ARG;
  if (p.bproj && !q.projection()) return LSTM_INT_E_INVALID_ARG;

  // activations x, h, m
  int rc;
  if (prev) {
    q.s_x = prev->s_h;
    q.zp_x = prev->zp_h;
  } else if ((rc = asymmetric_params(p.x_min, p.x_max, &q.s_x, &q.zp_x)) != LSTM_INT_OK) {
    return rc;
  }
  if ((rc = asymmetric_params(p.h_min, p.h_max, &q.s_h, &q.zp_h)) != LSTM_INT_OK) return rc;
  if (q.projection()) {
    if ((rc = asymmetric_params(p.m_min, p.m_max, &q.s_m, &q.zp_m)) != LSTM_INT_OK) return rc;
  } else {
    q.s_m = q.s_h;
    q.zp_m = q.zp_h;
  }

  // cell state: power-of-two range, Sec. 3.2.2
  if (!std::isfinite(p.c_absmax) || p.c_absmax < 0.0f) return LSTM_INT_E_BAD_RANGE;
  int m_c = 0;
  for (double pot = 1.0; pot < (double)p.c_absmax; pot *= 2.0) ++m_c;
  if (m_c > 8) return LSTM_INT_E_UNSUPPORTED;
  q.m_c = m_c;
  q.s_c = std::ldexp(1.0, m_c - 15);

  q.Wq.assign((size_t)4 * N * I, 0);
  q.Rq.assign((size_t)4 * N * H, 0);
  q.qb.assign((size_t)4 * N, 0);
  q.Pq.assign((size_t)3 * N, 0);
  q.Lq.assign((size_t)4 * N, 0);
  q.bx_fold.assign((size_t)4 * N, 0);
  q.bh_fold.assign((size_t)4 * N, 0);

  for (int g = first; g < 4; ++g) {
    const size_t nw = (size_t)N * I, nr = (size_t)N * H;
    if (!all_finite(p.W[g], nw) || !all_finite(p.R[g], nr) || !all_finite(p.b[g], N))
      return LSTM_INT_E_BAD_RANGE;
    q.s_W[g] = quantize_symmetric(p.W[g], nw, 127.0, q.Wq.data() + g * nw);
    q.s_R[g] = quantize_symmetric(p.R[g], nr, 127.0, q.Rq.data() + g * nr);

    double bias_scale;
    if (q.layer_norm()) {
      // gate sum at its measured range (Sec. 3.2.5); bias after the norm at
      // 2^-10 s_L (Sec. 3.2.6)
      const float ga = p.g_absmax[g];
      if (!std::isfinite(ga) || ga < 0.0f) return LSTM_INT_E_BAD_RANGE;
      q.s_g[g] = ga == 0.0f ? 1.0 : (double)ga / 32767.0;
      if (!all_finite(p.Lw[g], N)) return LSTM_INT_E_BAD_RANGE;
      q.s_L[g] = quantize_symmetric(p.Lw[g], N, 32767.0, q.Lq.data() + (size_t)g * N);
      bias_scale = std::ldexp(1.0, -10) * q.s_L[g];
    } else {
      q.s_g[g] = std::ldexp(1.0, -12);  // Q3.12, Sec. 3.2.4
      bias_scale = q.s_R[g] * q.s_h;
    }
    for (int n = 0; n < N; ++n) q.qb[(size_t)g * N + n] = quantize_bias(p.b[g][n], bias_scale);

    if ((rc = quantize_multiplier(q.s_W[g] * q.s_x / q.s_g[g], &q.Mx[g], &q.ex[g]))) return rc;
    if ((rc = quantize_multiplier(q.s_R[g] * q.s_h / q.s_g[g], &q.Mh[g], &q.eh[g]))) return rc;
    if (q.layer_norm() &&
        (rc = quantize_multiplier(q.s_L[g] * 4096.0, &q.Mln[g], &q.eln[g])))
      return rc;

    for (int n = 0; n < N; ++n) {
      const size_t row = (size_t)g * N + n;
      if ((rc = fold_zero_point(q.Wq.data() + row * I, I, q.zp_x, 0, &q.bx_fold[row]))) return rc;
      if ((rc = fold_zero_point(q.Rq.data() + row * H, H, q.zp_h,
                                q.layer_norm() ? 0 : q.qb[row], &q.bh_fold[row])))
        return rc;
    }
  }

  if (q.peephole()) {  // Sec. 3.2.3; slots i, f, o act on gates 0, 1, 3
    for (int j = first; j < 3; ++j) {
      const int gate = j == 2 ? 3 : j;
      if (!all_finite(p.P[j], N)) return LSTM_INT_E_BAD_RANGE;
      q.s_P[j] = quantize_symmetric(p.P[j], N, 32767.0, q.Pq.data() + (size_t)j * N);
      if ((rc = quantize_multiplier(q.s_P[j] * q.s_c / q.s_g[gate], &q.Mc[j], &q.ec[j]))) return rc;
    }
  }

  // o . tanh(c) is Q0.30 (Sec. 3.2.7)
  if ((rc = quantize_multiplier(std::ldexp(1.0, -30) / q.s_m, &q.Mm, &q.em))) return rc;

  if (q.projection()) {  // Sec. 3.2.8
    const size_t np = (size_t)H * N;
    if (!all_finite(p.Wproj, np) || (p.bproj && !all_finite(p.bproj, H))) return LSTM_INT_E_BAD_RANGE;
    q.Wpq.assign(np, 0);
    q.qbp.assign(H, 0);
    q.bp_fold.assign(H, 0);
    q.s_Wp = quantize_symmetric(p.Wproj, np, 127.0, q.Wpq.data());
    const double bias_scale = q.s_Wp * q.s_m;
    for (int j = 0; j < H; ++j) {
      if (p.bproj) q.qbp[j] = quantize_bias(p.bproj[j], bias_scale);
      if ((rc = fold_zero_point(q.Wpq.data() + (size_t)j * N, N, q.zp_m, q.qbp[j], &q.bp_fold[j])))
        return rc;
    }
    if ((rc = quantize_multiplier(q.s_Wp * q.s_m / q.s_h, &q.Mp, &q.ep))) return rc;
  }
  return LSTM_INT_OK;
}

}  // namespace

int quantize_multiplier(double s, int32_t *M, int32_t *e) {
  if (!(s > 0.0) || !std::isfinite(s)) return LSTM_INT_E_BAD_RANGE;
  int exponent = 0;
  const double mant = std::frexp(s, &exponent);  // in [0.5, 1)
  int64_t m = (int64_t)std::floor(mant * 2147483648.0 + 0.5);
  if (m == (int64_t)1 << 31) {
    m >>= 1;
    ++exponent;
  }
  if (exponent < -31 || exponent > 30) return LSTM_INT_E_UNSUPPORTED;
  *M = (int32_t)m;
  *e = exponent;
  return LSTM_INT_OK;
}

int prepare_host(const lstm_int_layer_params *layers, int32_t num_layers,
                 std::vector<LayerHost> &out) {
  if (!layers || num_layers < 1) return LSTM_INT_E_INVALID_ARG;
  out.clear();
  out.resize(num_layers);
  for (int l = 0; l < num_layers; ++l) {
    if (l > 0 && layers[l].input_size != layers[l - 1].output_size) return LSTM_INT_E_INVALID_ARG;
    int rc = prepare_layer(layers[l], l ? &out[l - 1] : nullptr, out[l]);
    if (rc != LSTM_INT_OK) return rc;
  }
  return LSTM_INT_OK;
}

// ---------------------------------------------------------------------------
// sigma / tanh tables (Sec. 3.2.1).  exp(-y), y >= 0 with 15 fraction bits, is
// assembled in Q0.31 from exp(-rho) on [0, 1/8) (degree-4 Taylor polynomial in
// Horner form) times the constants exp(-2^j), j = -3..4, for the set bits of
// y; every product is rounded half up to Q0.31.  Then
//   sigma(|x|) = round(2^46 / (2^31 + E)),           E = exp(-|x|)
//   tanh(|x|)  = round(2^15 (2^31 - E) / (2^31 + E)), E = exp(-2|x|)
// kExpPow2[j + 3] = round(exp(-2^j) 2^31).
namespace {
constexpr uint64_t kExpPow2[8] = {1895147668ull, 1672461947ull, 1302514674ull, 790015084ull,
                                  290630308ull,  39332535ull,   720401ull,     242ull};
constexpr uint64_t kOne = 1ull << 31;
constexpr uint64_t kSixth = 357913941ull;        // round(2^31 / 6)
constexpr uint64_t kTwentyFourth = 89478485ull;  // round(2^31 / 24)

// all operands are non-negative here, so unsigned arithmetic is exact
inline uint64_t mul_q31(uint64_t a, uint64_t b) { return (a * b + (1ull << 30)) >> 31; }
inline uint64_t div_round(uint64_t n, uint64_t d) { return (n + d / 2) / d; }
}  // namespace

int64_t exp_neg_q31(int64_t y) {
  uint64_t v = y < 0 ? 0 : (uint64_t)y;
  if (v > (1u << 20) - 1) v = (1u << 20) - 1;
  const uint64_t rho = (v & 0xFFFu) << 16;
  uint64_t acc = kSixth - mul_q31(rho, kTwentyFourth);
  acc = (kOne >> 1) - mul_q31(rho, acc);
  acc = kOne - mul_q31(rho, acc);
  acc = kOne - mul_q31(rho, acc);
  for (int bit = 0; bit < 8; ++bit)
    if (v & (1u << (12 + bit))) acc = mul_q31(acc, kExpPow2[bit]);
  return (int64_t)acc;
}

bool sparse24_row_ok(const int8_t *row, int K) {
  for (int k0 = 0; k0 < K; k0 += 4) {
    int nz = 0;
    for (int k = k0; k < k0 + 4 && k < K; ++k) nz += row[k] != 0;
    if (nz > 2) return false;
  }
  return true;
}

void sparse24_pack_lane(const int8_t *row, int K, int q, int a, int8_t vals[16], uint32_t *index) {
  uint32_t idx = 0;
  for (int j = 0; j < 8; ++j) {
    const int kb = 64 * q + (j < 4 ? 0 : 32) + 16 * a + 4 * (j % 4);
    int pos[2] = {0, 1}, n = 0;
    for (int i = 0; i < 4; ++i)
      if (kb + i < K && row[kb + i] != 0 && n < 2) pos[n++] = i;
    if (n == 1) {  // the second slot takes a neighbouring position, which holds a zero
      if (pos[0] < 3) {
        pos[1] = pos[0] + 1;
      } else {
        pos[1] = 3;
        pos[0] = 2;
      }
    }
    for (int s = 0; s < 2; ++s) {
      const int k = kb + pos[s];
      vals[2 * j + s] = k < K ? row[k] : (int8_t)0;
      idx |= (uint32_t)pos[s] << (4 * j + 2 * s);
    }
  }
  *index = idx;
}

int compress_table_wide(const uint16_t *tab, uint8_t *blob, int *has_tail, int *flat_from) {
  int F = 32768;
  while (F > 0 && tab[F - 1] == tab[32768]) --F;
  *flat_from = F;
  *has_tail = 0;
  for (int sh = 6; sh >= 3; --sh) {
    bool ok = true;
    for (int a = 0; a < 32768 && ok; ++a) {
      const int d = (int)tab[a] - (int)tab[(a >> sh) << sh];
      ok = d >= 0 && d <= 255;
    }
    if (!ok) continue;
    memset(blob, 0, kLutWideBytes);
    uint16_t *base = reinterpret_cast<uint16_t *>(blob + kLutWideBaseOff);
    for (int a = 0; a < 32768; ++a) {
      blob[a] = (uint8_t)(tab[a] - tab[(a >> sh) << sh]);
      if ((a & ((1 << sh) - 1)) == 0) base[a >> sh] = tab[a];
    }
    bool gentle = true;
    for (int a = 16385; a <= 32768 && gentle; ++a) {
      const int step = (int)tab[a] - (int)tab[a - 1];
      gentle = step >= 0 && step <= 1;
    }
    if (gentle) {
      uint16_t *start = reinterpret_cast<uint16_t *>(blob + kLutWideTailOff);
      uint32_t *mask = reinterpret_cast<uint32_t *>(blob + kLutWideTailOff + 1024);
      for (int b = 0; b < 512; ++b) {
        const int a0 = 16384 + 32 * b;
        start[b] = tab[a0];
        uint32_t mk = 0;
        for (int i = 1; i < 32; ++i)
          if (tab[a0 + i] != tab[a0 + i - 1]) mk |= 1u << i;
        mask[b] = mk;
      }
      if (tab[32768] != tab[32767]) mask[511] |= 1u;  // the step to the one entry beyond the last block
      *has_tail = 1;
    }
    return sh;
  }
  return -1;
}

void fill_sigmoid_table(int m, uint16_t *tab) {
  for (int64_t a = 0; a <= 32768; ++a) {
    const uint64_t E = (uint64_t)exp_neg_q31(a << m);
    tab[a] = (uint16_t)div_round(1ull << 46, kOne + E);
  }
}

void fill_tanh_table(int m, uint16_t *tab) {
  for (int64_t a = 0; a <= 32768; ++a) {
    const uint64_t E = (uint64_t)exp_neg_q31(a << (m + 1));
    tab[a] = (uint16_t)div_round((kOne - E) << 15, kOne + E);
  }
}

}  // namespace lstm_int
