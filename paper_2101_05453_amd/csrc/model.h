// Internal model representation of liblstm_int: host-side quantized tensors
// (what lstm_int_get_quant exposes) and the device-side packed copies.
#pragma once

#include <stdint.h>

#include <vector>

#include "../../include/lstm_int.h"

namespace lstm_int {

// Host-side result of the offline phase for one layer (Table 2).
struct LayerHost {
  int32_t I = 0, N = 0, H = 0, G = 4;
  uint32_t flags = 0;
  int32_t m_c = 0;
  int32_t zp_x = 0, zp_h = 0, zp_m = 0;
  double s_x = 0, s_h = 0, s_m = 0, s_c = 0, s_Wp = 0;
  double s_W[4] = {0, 0, 0, 0}, s_R[4] = {0, 0, 0, 0}, s_P[3] = {0, 0, 0}, s_L[4] = {0, 0, 0, 0},
         s_g[4] = {0, 0, 0, 0};
  int32_t Mx[4] = {0, 0, 0, 0}, ex[4] = {0, 0, 0, 0};
  int32_t Mh[4] = {0, 0, 0, 0}, eh[4] = {0, 0, 0, 0};
  int32_t Mc[3] = {0, 0, 0}, ec[3] = {0, 0, 0};
  int32_t Mln[4] = {0, 0, 0, 0}, eln[4] = {0, 0, 0, 0};
  int32_t Mm = 0, em = 0, Mp = 0, ep = 0;
  std::vector<int8_t> Wq, Rq, Wpq;
  std::vector<int32_t> qb, qbp, bx_fold, bh_fold, bp_fold;
  std::vector<int16_t> Pq, Lq;

  bool cifg() const { return flags & LSTM_INT_CIFG; }
  bool peephole() const { return flags & LSTM_INT_PEEPHOLE; }
  bool layer_norm() const { return flags & LSTM_INT_LAYER_NORM; }
  bool projection() const { return flags & LSTM_INT_PROJECTION; }
};

// Offline phase on the host; returns an LSTM_INT_* code.
int prepare_host(const lstm_int_layer_params *layers, int32_t num_layers,
                 std::vector<LayerHost> &out);

// (M, e) of an effective scale s > 0: s ~= M * 2^(e-31), 2^30 <= M < 2^31.
int quantize_multiplier(double s, int32_t *M, int32_t *e);

// Tables of sigma / tanh before mirroring and clamping: tab[a], a = |x| in
// 0..32768, for inputs in Q(m).(15-m) (Sec. 3.2.1).  Values lie in 0..32768.
void fill_sigmoid_table(int m, uint16_t *tab /*[32769]*/);
void fill_tanh_table(int m, uint16_t *tab /*[32769]*/);
// The wide form (lstm_int_math.h) of a table: returns the block shift (3..6; -1 if none keeps the deltas
// within 8 bits); *has_tail = the tail part is filled (the table rises by at most one per entry from 16384
// on); *flat_from = first index from which on every entry is equal.
int compress_table_wide(const uint16_t *tab, uint8_t *blob /*[kLutWideBytes]*/, int *has_tail, int *flat_from);
// 2:4 structure along k of a weight row (the pruned models of Table 1 in structured form): at most two nonzeros in
// every aligned group of four.
bool sparse24_row_ok(const int8_t *row, int K);
// One lane's operand of the sparse MFMA for k step q (64 deep) of such a row (entries at k >= K count as zero): lane
// half a holds the groups k = 64 q + (j < 4 ? 0 : 32) + 16 a + 4 (j % 4) + 0..3, j = 0..7, as values 2 j, 2 j + 1 (the
// two kept weights in ascending position; zeros fill a group with fewer) and their positions in index bits
// [4 j + 1 : 4 j] and [4 j + 3 : 4 j + 2].
void sparse24_pack_lane(const int8_t *row, int K, int q, int a, int8_t vals[16], uint32_t *index);
// exp(-y / 2^15) in Q0.31, y >= 0 (exposed for host-side checks)
int64_t exp_neg_q31(int64_t y);

}  // namespace lstm_int
