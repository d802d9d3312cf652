// Fixed-point building blocks of the integer LSTM cell, usable from HIP
// device code and from host code (prepare, CPU checks of the device math).
//
// Every function returns the exact integer its definition names; the
// definitions follow arXiv 2101.05453 Secs. 3.2.1-3.2.9.  Where a faster
// evaluation than the plain definition is used (a reciprocal with a fix-up,
// a table), the comment states why the result is the same integer.
#pragma once

#include <math.h>
#include <stdint.h>
#include <string.h>

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

// The same for r >= 32, where the result is below 2^31 in magnitude and needs
// no saturation: one 64-bit multiply-add and one shift.
LSTM_HD int32_t rescale_ge32(int32_t a, int32_t M, int32_t r) {
  return (int32_t)(((int64_t)a * (int64_t)M + ((int64_t)1 << (r - 1))) >> r);
}

// floor((a + 2^(k-1)) / 2^k), k >= 1
LSTM_HD int32_t rsh_round(int32_t a, int32_t k) {
  return (int32_t)(((int64_t)a + ((int64_t)1 << (k - 1))) >> k);
}

// floor(num / d) for |num| < 2^51 and 1 <= d < 2^26, with inv_d = 1.0 / d in
// double.  num is exact in double; the product with the rounded reciprocal is
// off by less than 2^-1 of a unit (relative error 2^-52 on a quotient below
// 2^51), so its floor misses by at most one, and the exact integer remainder
// corrects it.
LSTM_HD int64_t floor_div_recip(int64_t num, int32_t d, double inv_d) {
  int64_t q = (int64_t)floor((double)num * inv_d);
  const int64_t rem = num - q * d;
  if (rem < 0) {
    --q;
  } else if (rem >= d) {
    ++q;
  }
  return q;
}

// floor(sqrt(v)), 0 <= v < 2^52: the double root is within one of the
// answer; the comparisons settle it exactly.
// (r < 2^26, so r * r and v - r * r are exact in double: one fused
// multiply-add gives the remainder, and (r + 1)^2 <= v iff v - r^2 >= 2 r + 1.)
LSTM_HD int64_t isqrt_u52(int64_t v) {
  if (v <= 0) return 0;
  const double dv = (double)v;
  double r = floor(sqrt(dv));
  const double rem = fma(-r, r, dv);
  if (rem < 0.0) {
    r -= 1.0;
  } else if (rem >= 2.0 * r + 1.0) {
    r += 1.0;
  }
  return (int64_t)r;
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

// S2 * 2^20 can reach 2^62, too wide for the reciprocal division; with
// S2 = a n + r (0 <= r < n) the quotient is a 2^20 + floor((r 2^20 + n/2)/n),
// and both divisions have numerators below 2^44.
// For n a power of two both floors are arithmetic right shifts (S2 * 2^20 < 2^62 for n <= 4096).
LSTM_HD LnRow ln_row(int64_t S1, int64_t S2, int32_t n, double inv_n) {
  LnRow r;
  int64_t mean, var;
  if ((n & (n - 1)) == 0) {
    const int sh = __builtin_ctz((unsigned)n);
    mean = (S1 * 1024 + (n >> 1)) >> sh;
    var = (((S2 << 20) + (n >> 1)) >> sh) - mean * mean;
  } else {
    mean = floor_div_recip(S1 * 1024 + (n >> 1), n, inv_n);
    const int64_t a = floor_div_recip(S2, n, inv_n);
    const int64_t low = floor_div_recip(((S2 - a * n) << 20) + (n >> 1), n, inv_n);
    var = (a << 20) + low - mean * mean;
  }
  if (var < 0) var = 0;
  r.mean = (int32_t)mean;
  r.sigma = (int32_t)isqrt_u52(var);
  r.inv_sigma = r.sigma ? 1.0 / (double)r.sigma : 0.0;
  return r;
}

// One element: q' = floor((2^10 (2^10 q - mean) + floor(sigma/2)) / sigma),
// q'' = sat32(floor((q' qL + qb + 2^9) / 2^10)), out = sat16(rescale(q'')).
// All of it in double, every step exact: the numerator is an integer below
// 2^37; its product with the rounded reciprocal is within 2^-15 of the
// quotient, so the floor misses by at most one, and the remainder -- an
// integer below 2^27 in magnitude, which one fused multiply-add returns
// exactly -- corrects it.  |q' qL + qb| < 2^53 and the division by 2^10 is a
// power of two, so the second stage is exact as well.
LSTM_HD int32_t ln_apply(int32_t q, const LnRow &row, int32_t qL, int32_t qb, int32_t M_ln,
                         int32_t r_ln) {
  double qn = 0.0;
  if (row.sigma != 0) {
    const double sg = (double)row.sigma;
    const double num = (double)(q * 1024 - row.mean) * 1024.0 + (double)(row.sigma >> 1);
    qn = floor(num * row.inv_sigma);
    const double rem = fma(-qn, sg, num);
    if (rem < 0.0) {
      qn -= 1.0;
    } else if (rem >= sg) {
      qn += 1.0;
    }
  }
  const double t = fma(qn, (double)qL, (double)qb);
  double q2 = floor((t + 512.0) * (1.0 / 1024.0));
  q2 = q2 < -2147483648.0 ? -2147483648.0 : (q2 > 2147483647.0 ? 2147483647.0 : q2);
  return sat16(rescale((int32_t)q2, M_ln, r_ln));
}

// The same element with everything that does not depend on it prepared ahead.
// Per row:   c0 = -2^10 mean + floor(sigma/2) + 1/2, so that 2^20 q + c0 is the
// numerator plus one half.  The numerator n is an integer, so no multiple of
// sigma lies in (n, n + 1/2]: floor((n + 1/2) / sigma) = floor(n / sigma), and
// (n + 1/2) / sigma stays at least 1/(2 sigma) away from every integer, while
// its product with the rounded reciprocal is off by less than 2^-52 of a
// quotient below 2^37 / sigma, i.e. by less than 2^-15 / sigma.  The floor of
// that product is therefore exact and needs no remainder correction.  A row
// with sigma = 0 has 1/sigma = 0 here, which gives q' = 0 as required.
// Per cell:  qLs = qL / 2^10 and qbs = qb / 2^10 + 2^-11 (both exact), so that
// one fused multiply-add gives (q' qL + qb) / 2^10 + 2^-11 exactly (44 bits).
// That value is a multiple of 2^-10 plus 2^-11, never halfway between two
// integers, and rounding it to the nearest integer is floor((q' qL + qb + 2^9)
// / 2^10).  The rounding is done by adding 1.5 * 2^52, whose sum holds the
// integer in its low mantissa bits; clamping to the int32 range first is the
// same as clamping afterwards because the bounds are integers.
// Stored per row: a = 2^20 / sigma and b = c0 / sigma, so that the quotient estimate is one fused
// multiply-add, q a + b.  Both products are rounded (relative error 2^-53 each, as is the fused
// result), which moves the estimate by less than 3 * 2^-53 * 2^37 / sigma < 2^-14 / sigma, still far
// inside the 1 / (2 sigma) margin above.
struct LnRow2 {
  double a, b;
};
LSTM_HD LnRow2 ln_row2(const LnRow &r) {
  LnRow2 o;
  const double inv = r.sigma ? r.inv_sigma : 0.0;
  o.a = 1048576.0 * inv;
  o.b = ((double)(-(int64_t)r.mean * 1024 + (r.sigma >> 1)) + 0.5) * inv;
  return o;
}
LSTM_HD double ln_weight_scaled(int32_t qL) { return (double)qL * (1.0 / 1024.0); }
LSTM_HD double ln_bias_scaled(int32_t qb) { return (double)qb * (1.0 / 1024.0) + (1.0 / 2048.0); }
// Second-stage rescale constants for a shift r >= 32 (a is below 2^31 in
// magnitude after the shift by k = 33 - r <= 1 only if |a| < 2^30; the
// layer-norm value that is not, saturates the 16-bit result either way, see
// rescale_sat16_pre).
struct RescaleHi {
  int32_t M, add, sh, k;  // k: left shift of the operand; add = 2^(r + k - 33); sh = r + k - 32
};
LSTM_HD RescaleHi rescale_hi_prepare(int32_t M, int32_t r) {
  RescaleHi o;
  o.M = M;
  o.k = r < 33 ? 33 - r : 0;
  o.add = (int32_t)1 << (r + o.k - 33);
  o.sh = r + o.k - 32;
  return o;
}
// sat16(rescale(a, M, r)) for 3 <= r <= 62 from the high word of one 32-bit
// product.  For r >= 33 this is rescale_hi.  For r < 33 the operand is shifted
// left by k = 33 - r first, which is exact if |a| < 2^(31-k); a larger |a| is
// clamped to [-2^(31-k), 2^(31-k) - 1] before, which does not change the saturated result:
// (2^(31-k) - 1) * M / 2^r >= (2^31 - 2^k) 2^30 / 2^33 = 2^28 - 2^(k-3) > 2^15 for k <= 30.
// the operand's clamp and left shift, a no-op when p.k == 0
LSTM_HD int32_t rescale_preshift(int32_t a, const RescaleHi &p) {
  const int32_t lim = (int32_t)(0x7FFFFFFFu >> p.k);
  a = a < lim ? a : lim;
  a = a > -lim - 1 ? a : -lim - 1;
  return (int32_t)((uint32_t)a << p.k);  // two's-complement shift, defined for negative a as well
}
// PRE: 2 = clamp and shift the operand (any operand), 1 = shift only (the caller
// knows that the shifted operand fits 32 bits), 0 = neither (p.k == 0, or done already)
template <int PRE = 2>
LSTM_HD int32_t rescale_sat16_pre(int32_t a, const RescaleHi &p) {
  if (PRE == 2) a = rescale_preshift(a, p);
  if (PRE == 1) a = (int32_t)((uint32_t)a << p.k);
#if defined(__HIP_DEVICE_COMPILE__)
  const int32_t hi = __mulhi(a, p.M);
#else
  const int32_t hi = (int32_t)(((int64_t)a * (int64_t)p.M) >> 32);
#endif
  return sat16((hi + p.add) >> p.sh);
}
LSTM_HD int32_t f64_low_word(double w) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __double2loint(w);
#else
  int64_t bits;
  memcpy(&bits, &w, 8);
  return (int32_t)bits;
#endif
}
// the layer-norm value before its second-stage rescale
LSTM_HD int32_t ln_second_stage(int32_t q, const LnRow2 &row, double qLs, double qbs) {
  const double qn = floor(fma((double)q, row.a, row.b));
  double v = fma(qn, qLs, qbs);
  v = fmin(fmax(v, -2147483648.0), 2147483647.0);
  return f64_low_word(v + 6755399441055744.0);
}
// The same without the clamp, for rows with sigma >= 2^12 (or sigma = 0), which ln_row_is_narrow tells from
// a = 2^20 / sigma <= 2^8: the numerator 2^20 q + c0 is below 2^36 + 2^25 in magnitude (|2^10 q - mean| <= 2^26,
// sigma < 2^25), so |q'| <= 2^24 + 2^13, |q' qL| <= 2^39 + 2^28, and with |qb| <= 2^31 the second-stage value
// (q' qL + qb) / 2^10 stays below 2^30: sat32 never acts.  (sigma = 0: q' = 0 and the value is qb / 2^10.)
LSTM_HD bool ln_row_is_narrow(const LnRow2 &row) { return row.a <= 256.0; }
LSTM_HD int32_t ln_second_stage_narrow(int32_t q, const LnRow2 &row, double qLs, double qbs) {
  const double qn = floor(fma((double)q, row.a, row.b));
  return f64_low_word(fma(qn, qLs, qbs) + 6755399441055744.0);
}
LSTM_HD int32_t ln_apply2(int32_t q, const LnRow2 &row, double qLs, double qbs, const RescaleHi &p) {
  return rescale_sat16_pre(ln_second_stage(q, row, qLs, qbs), p);
}

// Cell update with 32-bit intermediates: |i z| <= 2^30 and the rounding terms
// are below 2^23, so nothing leaves int32.
LSTM_HD int32_t cell_update32(int32_t i, int32_t z, int32_t f, int32_t c, int32_t m_c) {
  const int32_t iz = (i * z + ((int32_t)1 << (14 + m_c))) >> (15 + m_c);
  const int32_t fc = (f * c + 16384) >> 15;
  return sat16(iz + fc);
}

// ---------------------------------------------------------------------------
// sigma and tanh, Sec. 3.2.1: int16 in Q(m).(15-m) -> Q0.15.  The device
// reads them from tables indexed by |x| (0..32768) that hold the value before
// mirroring and clamping, 0..32768 (fill_sigmoid_table / fill_tanh_table).
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

// Compressed forms of such a table for LDS: tab[a] = base[a >> sh] + delta[a] with 8-bit deltas (the tables
// are monotone, so a block of 2^sh entries that rises by at most 255 compresses exactly), and for the flat
// tail a form of its own:
// Entry a of a tail, 16384 <= a <= 32768, from 512 block starts (uint16) and 512 masks (uint32): bit i > 0 of
// a block's mask says that entry i of the block is one above entry i - 1; bit 0 of the LAST block's mask says
// the same of entry 32768 against entry 32767 (|x| = 32768 occurs for x = -32768 only); bit 0 of the other
// masks is clear.
LSTM_HD int32_t lut_tail_value(const uint16_t *starts, const uint32_t *masks, int32_t a) {
  int32_t at = a - 16384;
  const bool beyond = at >= 16384;
  at = beyond ? 16383 : at;
  const uint32_t start = starts[at >> 5];
  const uint32_t mask = masks[at >> 5];
  const uint32_t upto = (2u << (at & 31)) - 2u;  // bits 1..i; i = 31 wraps to all ones but bit 0
#if defined(__HIP_DEVICE_COMPILE__)
  const uint32_t steps = (uint32_t)__popc(mask & upto);
#else
  const uint32_t steps = (uint32_t)__builtin_popcount(mask & upto);
#endif
  return (int32_t)(start + steps + (beyond ? (mask & 1u) : 0u));
}
// Wide form of a compressed table (global memory): the same encoding over ALL 32768 entries, from which a
// kernel copies into LDS as long a prefix (`dom` entries, a multiple of 1024) as its LDS budget allows --
// the longer, the rarer a lookup has to go to the tail.  Layout: 32768 deltas; the bases (32768 >> sh
// uint16, at most 8 KB); 512 tail starts (1 KB) and 512 tail masks (2 KB) for the entries 16384..32767
// (lut_tail_value's form incl. the step to entry 32768, present if the table rises by at most one per entry there).
constexpr int kLutWideBaseOff = 32768, kLutWideTailOff = 32768 + 8192, kLutWideBytes = kLutWideTailOff + 3072;
// bytes of the LDS copy for a prefix of dom entries
LSTM_HD int32_t lut_wide_lds_bytes(int32_t dom, int32_t sh, bool with_tail) {
  return dom + ((((dom >> sh) * 2) + 1023) & ~1023) + (with_tail ? 3072 : 0);
}
// entry a, 16384 <= a <= 32768, from the tail part (`tail` points at the 512 starts, the masks follow
// 1 KB behind)
LSTM_HD int32_t lut_wide_tail(const uint8_t *tail, int32_t a) {
  return lut_tail_value(reinterpret_cast<const uint16_t *>(tail), reinterpret_cast<const uint32_t *>(tail + 1024), a);
}
// host model of a lookup through an LDS copy with prefix dom: |x| = a in 0..32768
LSTM_HD int32_t lut_wide_mag(const uint8_t *blob, int32_t sh, int32_t dom, bool with_tail, int32_t a) {
  if (a >= dom && with_tail) return lut_wide_tail(blob + kLutWideTailOff, a);
  const int32_t ai = a < dom ? a : dom - 1;  // without a tail the table is flat from dom - 1 on
  return (int32_t)reinterpret_cast<const uint16_t *>(blob + kLutWideBaseOff)[ai >> sh] + (int32_t)blob[ai];
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
