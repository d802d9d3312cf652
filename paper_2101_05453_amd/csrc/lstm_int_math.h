// Fixed-point building blocks of the integer LSTM cell, usable from HIP
// device code and from host code (prepare, CPU checks of the device math).
//
// Every function returns the exact integer its definition names; the
// definitions follow arXiv 2101.05453 Secs. 3.2.1-3.2.9.  Where a faster
// evaluation than the plain definition is used (a reciprocal with a fix-up,
// a table), the comment states why the result is the same integer.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define LSTM_HD __host__ __device__ __forceinline__
#else
#define LSTM_HD inline
#endif

namespace lstm_int {

LSTM_HD int32_t clamp_i32(int32_t v, int32_t lo, int32_t hi) {
  return v < lo ? lo : (v > hi ? hi : v);
}
LSTM_HD int32_t sat16(int32_t v) { return clamp_i32(v, -32768, 32767); }
LSTM_HD int32_t sat8(int32_t v) { return clamp_i32(v, -128, 127); }
LSTM_HD int32_t sat32_from64(int64_t v) {
  return v < INT32_MIN ? INT32_MIN : (v > INT32_MAX ? INT32_MAX : (int32_t)v);
}

// rescale of Secs. 3.2.4-3.2.8: an effective scale s ~= M * 2^(e-31),
// 2^30 <= M < 2^31, -31 <= e <= 30, applied with one rounding (ties up):
//   sat32(floor(a * M / 2^r + 1/2)),  r = 31 - e in [1, 62].
// |a * M| <= 2^62 and the rounding term is < 2^62, so int64 holds the sum.
LSTM_HD int32_t rescale(int32_t a, int32_t M, int32_t r) {
  int64_t p = (int64_t)a * (int64_t)M + ((int64_t)1 << (r - 1));
  return sat32_from64(p >> r);
}

// Same value for r >= 33, from the high word of the product only:
// a*M = hi * 2^32 + lo with 0 <= lo < 2^32, and for integers n, d > 0 and a
// fraction 0 <= f < 1, floor((n + f) / d) = floor(n / d); so
// floor((a*M + 2^(r-1)) / 2^r) = floor((hi + 2^(r-33)) / 2^(r-32)).
// The result is below 2^31 in magnitude, no saturation needed.
LSTM_HD int32_t rescale_hi(int32_t a, int32_t M, int32_t r) {
#if defined(__HIP_DEVICE_COMPILE__)
  int32_t hi = __mulhi(a, M);
#else
  int32_t hi = (int32_t)(((int64_t)a * (int64_t)M) >> 32);
#endif
  return (hi + ((int32_t)1 << (r - 33))) >> (r - 32);
}

// floor((a + 2^(k-1)) / 2^k), k >= 1
LSTM_HD int32_t rsh_round(int32_t a, int32_t k) {
  return (int32_t)(((int64_t)a + ((int64_t)1 << (k - 1))) >> k);
}

// floor(sqrt(v)), 0 <= v < 2^52: the double root is within one of the
// answer; the two comparisons settle it exactly.
LSTM_HD int64_t isqrt_u52(int64_t v) {
  if (v <= 0) return 0;
#if defined(__HIP_DEVICE_COMPILE__)
  int64_t r = (int64_t)__dsqrt_rn((double)v);
#else
  int64_t r = (int64_t)__builtin_sqrt((double)v);
#endif
  while (r * r > v) --r;
  while ((r + 1) * (r + 1) <= v) ++r;
  return r;
}

// ---------------------------------------------------------------------------
// Integer layer norm, Sec. 3.2.6 with s' = 2^-10.
// Row statistics from S1 = sum q, S2 = sum q^2 over n <= 4096 int16 values:
//   mean  = floor((S1 * 2^10 + floor(n/2)) / n)
//   var   = max(0, floor((S2 * 2^20 + floor(n/2)) / n) - mean^2)
//   sigma = floor(sqrt(var))
// |mean| <= 2^25, var < 2^50, sigma < 2^25.
struct LnRow {
  int32_t mean;
  int32_t sigma;
  double inv_sigma;  // 1 / sigma rounded to double (unused when sigma == 0)
};

LSTM_HD int64_t floor_div_pos(int64_t a, int64_t d) {  // d > 0
  int64_t q = a / d;
  if (a % d < 0) --q;
  return q;
}

LSTM_HD LnRow ln_row(int64_t S1, int64_t S2, int32_t n) {
  LnRow r;
  int64_t mean = floor_div_pos(S1 * 1024 + (n >> 1), n);
  int64_t var = floor_div_pos(S2 * 1048576 + (n >> 1), n) - mean * mean;
  if (var < 0) var = 0;
  r.mean = (int32_t)mean;
  r.sigma = (int32_t)isqrt_u52(var);
  r.inv_sigma = r.sigma ? 1.0 / (double)r.sigma : 0.0;
  return r;
}

// One element: q' = floor((2^10 (2^10 q - mean) + floor(sigma/2)) / sigma),
// q'' = sat32(floor((q' qL + qb + 2^9) / 2^10)), out = sat16(rescale(q'')).
// The quotient is taken as floor(num * (1/sigma)) in double and corrected by
// the integer remainder: |num| < 2^38 is exact in double and the two
// roundings move the product by less than 2^-14, so the floor is off by at
// most one, which the remainder test repairs.
LSTM_HD int32_t ln_apply(int32_t q, const LnRow &row, int32_t qL, int32_t qb, int32_t M_ln,
                         int32_t r_ln) {
  int64_t qn = 0;
  if (row.sigma != 0) {
    int64_t num = (((int64_t)q << 10) - row.mean) * 1024 + (row.sigma >> 1);
#if defined(__HIP_DEVICE_COMPILE__)
    qn = (int64_t)floor((double)num * row.inv_sigma);
#else
    qn = (int64_t)__builtin_floor((double)num * row.inv_sigma);
#endif
    int64_t rem = num - qn * row.sigma;
    if (rem < 0) {
      --qn;
    } else if (rem >= row.sigma) {
      ++qn;
    }
  }
  int64_t t = qn * (int64_t)qL + (int64_t)qb;
  int32_t q2 = sat32_from64((t + 512) >> 10);
  return sat16(rescale(q2, M_ln, r_ln));
}

// ---------------------------------------------------------------------------
// sigma and tanh, Sec. 3.2.1: int16 in Q(m).(15-m) -> Q0.15.  The device
// reads them from tables indexed by |x| (0..32768) that hold the value before
// mirroring and clamping, 0..32768; ActTables (activations.h) fills them.
//   sigma: x >= 0 -> min(v, 32767);      x < 0 -> 32768 - v
//   tanh:  x >= 0 -> min(v, 32767);      x < 0 -> -v
LSTM_HD int32_t sigmoid_from_table(const uint16_t *tab, int32_t x) {
  int32_t a = x < 0 ? -x : x;
  int32_t v = tab[a];
  return x < 0 ? 32768 - v : (v > 32767 ? 32767 : v);
}
LSTM_HD int32_t tanh_from_table(const uint16_t *tab, int32_t x) {
  int32_t a = x < 0 ? -x : x;
  int32_t v = tab[a];
  return x < 0 ? -v : (v > 32767 ? 32767 : v);
}

// CIFG coupling, Sec. 3.2.9 (the value must fit int16, so the smaller of the
// two): i = min(32768 - f, 32767).
LSTM_HD int32_t cifg_input_gate(int32_t f) {
  int32_t i = 32768 - f;
  return i > 32767 ? 32767 : i;
}

// Cell update, Sec. 3.2.7: i.z is Q0.30 and goes to Q(m_c).(15-m_c) by a
// rounding shift of 15 + m_c; f.c is Q(m_c).(30-m_c), a shift of 15.
LSTM_HD int32_t cell_update(int32_t i, int32_t z, int32_t f, int32_t c, int32_t m_c) {
  return sat16(rsh_round(i * z, 15 + m_c) + rsh_round(f * c, 15));
}

// Hidden state, Sec. 3.2.7: m = sat8(rescale(o . tanh(c), 2^-30 / s_m) + zp_m)
LSTM_HD int32_t hidden_state(int32_t o, int32_t tanh_c, int32_t M_m, int32_t r_m, int32_t zp_m) {
  return sat8(rescale(o * tanh_c, M_m, r_m) + zp_m);
}

}  // namespace lstm_int
