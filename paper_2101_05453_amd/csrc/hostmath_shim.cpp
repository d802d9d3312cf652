// Host-only C entry points onto lstm_int_math.h, so that the arithmetic the
// kernels run can be checked exhaustively on a CPU.  Not part of
// liblstm_int.so.
#include "lstm_int_math.h"
#include "model.h"

using namespace lstm_int;

extern "C" {

int32_t hm_rescale(int32_t a, int32_t M, int32_t r) { return rescale(a, M, r); }
int32_t hm_rescale_hi(int32_t a, int32_t M, int32_t r) { return rescale_hi(a, M, r); }
int64_t hm_isqrt(int64_t v) { return isqrt_u52(v); }

// layer norm of one row through ln_row / ln_apply
void hm_layernorm(const int16_t *q, int32_t n, const int16_t *qL, const int32_t *qb, int32_t M,
                  int32_t r, int16_t *out) {
  int64_t s1 = 0, s2 = 0;
  for (int i = 0; i < n; ++i) {
    s1 += q[i];
    s2 += (int64_t)q[i] * q[i];
  }
  const LnRow row = ln_row(s1, s2, n, 1.0 / (double)n);
  for (int i = 0; i < n; ++i) out[i] = (int16_t)ln_apply(q[i], row, qL[i], qb[i], M, r);
}

// the per-row-prepared form used by the persistent kernel (second-stage shift >= 32)
void hm_layernorm2(const int16_t *q, int32_t n, const int16_t *qL, const int32_t *qb, int32_t M,
                   int32_t r, int16_t *out) {
  int64_t s1 = 0, s2 = 0;
  for (int i = 0; i < n; ++i) {
    s1 += q[i];
    s2 += (int64_t)q[i] * q[i];
  }
  const LnRow2 row = ln_row2(ln_row(s1, s2, n, 1.0 / (double)n));
  const RescaleHi p = rescale_hi_prepare(M, r);
  for (int i = 0; i < n; ++i)
    out[i] = ln_row_is_narrow(row)
                 ? (int16_t)rescale_sat16_pre(ln_second_stage_narrow(q[i], row, ln_weight_scaled(qL[i]), ln_bias_scaled(qb[i])), p)
                 : (int16_t)ln_apply2(q[i], row, ln_weight_scaled(qL[i]), ln_bias_scaled(qb[i]), p);
}
// 1 if a row with these statistics takes the second stage without the int32 clamp
int hm_ln_row_is_narrow(const int16_t *q, int32_t n) {
  int64_t s1 = 0, s2 = 0;
  for (int i = 0; i < n; ++i) {
    s1 += q[i];
    s2 += (int64_t)q[i] * q[i];
  }
  return ln_row_is_narrow(ln_row2(ln_row(s1, s2, n, 1.0 / (double)n))) ? 1 : 0;
}
int32_t hm_rescale_sat16_pre(int32_t a, int32_t M, int32_t r) {
  return rescale_sat16_pre(a, rescale_hi_prepare(M, r));
}
int32_t hm_cell_update32(int32_t i, int32_t z, int32_t f, int32_t c, int32_t m_c) {
  return cell_update32(i, z, f, c, m_c);
}

void hm_sigmoid_table(int m, uint16_t *tab) { fill_sigmoid_table(m, tab); }
void hm_tanh_table(int m, uint16_t *tab) { fill_tanh_table(m, tab); }
int32_t hm_sigmoid(const uint16_t *tab, int32_t x) { return sigmoid_from_table(tab, x); }
int32_t hm_tanh(const uint16_t *tab, int32_t x) { return tanh_from_table(tab, x); }
int hm_compress_wide(const uint16_t *tab, uint8_t *blob, int *has_tail, int *flat_from) {
  return compress_table_wide(tab, blob, has_tail, flat_from);
}
int32_t hm_lut_wide_mag(const uint8_t *blob, int sh, int dom, int with_tail, int32_t a) {
  return lut_wide_mag(blob, sh, dom, with_tail != 0, a);
}
int hm_sparse24_row_ok(const int8_t *row, int K) { return sparse24_row_ok(row, K) ? 1 : 0; }
void hm_sparse24_pack_lane(const int8_t *row, int K, int q, int a, int8_t *vals, uint32_t *index) {
  sparse24_pack_lane(row, K, q, a, vals, index);
}
int32_t hm_rescale_ge32(int32_t a, int32_t M, int32_t r) { return rescale_ge32(a, M, r); }
int32_t hm_cifg(int32_t f) { return cifg_input_gate(f); }
int32_t hm_cell_update(int32_t i, int32_t z, int32_t f, int32_t c, int32_t m_c) {
  return cell_update(i, z, f, c, m_c);
}
int32_t hm_hidden(int32_t o, int32_t tc, int32_t M, int32_t r, int32_t zp) {
  return hidden_state(o, tc, M, r, zp);
}

// The library's offline phase on the host (what lstm_int_prepare runs before the upload); *checksum
// receives the sum of every quantized weight, bias and multiplier of every layer, for a cross-check.
int hm_prepare(const lstm_int_layer_params *layers, int32_t num_layers, int64_t *checksum) {
  std::vector<LayerHost> out;
  const int rc = prepare_host(layers, num_layers, out);
  int64_t s = 0;
  for (const LayerHost &h : out) {
    for (int8_t v : h.Wq) s += v;
    for (int8_t v : h.Rq) s += v;
    for (int8_t v : h.Wpq) s += v;
    for (int32_t v : h.qb) s += v;
    for (int32_t v : h.qbp) s += v;
    for (int32_t v : h.bx_fold) s += v;
    for (int32_t v : h.bh_fold) s += v;
    for (int32_t v : h.bp_fold) s += v;
    for (int16_t v : h.Pq) s += v;
    for (int16_t v : h.Lq) s += v;
    for (int g = 0; g < 4; ++g) s += (int64_t)h.Mx[g] + h.ex[g] + h.Mh[g] + h.eh[g] + h.Mln[g] + h.eln[g];
    s += (int64_t)h.Mm + h.em + h.Mp + h.ep + h.zp_x + h.zp_h + h.zp_m + h.m_c;
  }
  if (checksum) *checksum = s;
  return rc;
}
}
