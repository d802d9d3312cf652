// C ABI of liblstm_int (include/lstm_int.h): model lifetime, the upload of the
// packed integer tensors, and the orchestration of the online phase.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.h"
#include "lstm_int_math.h"
#include "model.h"
#include "persistent.h"

using namespace lstm_int;

// Workspace of lstm_int_forward_static: lives in the library's device image, one copy per GPU from the
// moment the image is loaded there until the process ends.  Host code never uses this name as an address
// (on the host it is only a handle for hipGetSymbolAddress); kernels get the per-device pointer below.
static __device__ __align__(256) unsigned char scratch[LSTM_INT_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, looked up once per device

// Looks up (once per device, with that device current) where `scratch` lives on `device`.
int scratch_lookup(int device) {
  if (device < 0 || device >= kMaxDevices) return LSTM_INT_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device]) return LSTM_INT_OK;
  void *ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LSTM_INT_E_DEVICE;
  g_scratch_ptr[device] = ptr;
  return LSTM_INT_OK;
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// A table in the wide compressed form (lstm_int_math.h) and what prepare found out about it.
struct WideTable {
  const uint8_t *blob = nullptr;  // device, [kLutWideBytes]
  int sh = -1;                    // block shift, -1 = does not compress
  int has_tail = 0;               // the tail part (entries 16384..) is filled
  int flat_from = 32768;          // every entry from here on is equal
  // shortest prefix a kernel may keep in LDS (0 = none: the table cannot be used from LDS alone) and whether
  // the tail part has to come with it
  void shortest(int *dom, int *tail) const {
    *dom = 0;
    *tail = 0;
    if (sh < 0) return;
    const int flat_dom = flat_from + 1 <= 32768 ? (flat_from + 1 + 1023) / 1024 * 1024 : 0;  // flat from dom - 1 on
    const int tail_dom = has_tail ? 16384 : 0;
    const int flat_bytes = flat_dom ? lstm_int::lut_wide_lds_bytes(flat_dom, sh, false) : 0;
    const int tail_bytes = tail_dom ? lstm_int::lut_wide_lds_bytes(tail_dom, sh, true) : 0;
    if (flat_dom && (!tail_dom || flat_bytes <= tail_bytes)) {
      *dom = flat_dom;
    } else if (tail_dom) {
      *dom = tail_dom;
      *tail = 1;
    }
  }
};

// Device-side tensors of one layer, all inside the model's single allocation.
struct LayerDev {
  // K extents padded to 64.  Hpad is padded to 128 so that the rows of a step's
  // h never share a 128-byte cache line with another step's (see persistent.hip).
  int Ipad = 0, Hpad = 0, Npad = 0;
  int GN = 0;                        // G * N output columns of the gate matmuls
  int8_t *W = nullptr;               // [pad128(G*N), Ipad]  present gates, gate-major
  int8_t *R = nullptr;               // [pad128(G*N), Hpad]
  int8_t *Wproj = nullptr;           // [pad128(H), Npad]
  int32_t *bx = nullptr, *bh = nullptr, *bp = nullptr;  // folded biases, padded like the rows
  int16_t *Pq = nullptr, *Lq = nullptr;
  int32_t *qb = nullptr;
  const uint16_t *tanhc = nullptr;  // tanh table of the cell format Q(m_c).(15-m_c)
  WideTable wtanhc;  // the same table in the wide form (rec_kernel)
  Requant rq_x, rq_h, rq_p;
  // persistent path (persistent.h): tile-ordered copies; p2 = shape is eligible
  bool p2 = false;
  int GS = 0, ks = 0, Ncp = 0, ptiles = 0, npadp = 0;
  // per gate: bound of |W x + b'x| and |R h + b'h| over all inputs, max over rows of |b'| + 128 sum |w|
  int64_t amax_x[4] = {0, 0, 0, 0}, amax_h[4] = {0, 0, 0, 0};
  int8_t *W2 = nullptr;     // [GS*8][32][Ipad]
  int8_t *W2f = nullptr;    // the same in MFMA operand order [GS*8][Ipad/32][64 lanes][16] (Ipad <= 1024), else NULL
  int32_t *bx2 = nullptr;   // [GS*8][32]
  int4 *R2 = nullptr;       // [GS][4][2][ks][64]
  int4 *R2s = nullptr;      // the same weights in the 2:4 compressed form (persistent.h), or NULL: R is not 2:4
  bool p16 = false;         // the 16-row kernel takes this layer (small batches)
  int ks16 = 0;
  int4 *R2h = nullptr;      // [GS][4][4][ks16][64]
  int32_t *bh4 = nullptr, *qb4 = nullptr;  // [4][Ncp]
  int16_t *Lq4 = nullptr, *Pq3 = nullptr;  // [4][Ncp], [3][Ncp]
  int8_t *Wp2 = nullptr;    // [ptiles][32][npadp]
  int32_t *bp2 = nullptr;   // [ptiles][32]
  // the 32-row kernel's own tiling of W_proj: prow outputs per tile, so that every workgroup of a group has
  // one (H = 640 over 32 workgroups: 20 rows each instead of 20 tiles of 32 over 32 workgroups) and keeps only
  // those rows in LDS; prow = 32 and the arrays above when H needs more tiles than a group has workgroups
  int prow = 32, ptiles3 = 0;
  int8_t *Wp3 = nullptr;    // [ptiles3][32][npadp], rows >= prow of a tile zero
  int32_t *bp3 = nullptr;   // [ptiles3][32]
};

struct Profile {
  bool on = false;
  hipStream_t stream = nullptr;
  std::vector<hipEvent_t> ev;  // pairs (start, stop)
  std::vector<int> cls;
  size_t used = 0;  // pairs in use
  bool failed = false;  // an event could not be created: the times would be incomplete
  void release() {
    for (auto &e : ev)
      if (e) (void)hipEventDestroy(e);
    ev.clear();
    cls.clear();
    used = 0;
  }
};

}  // namespace

struct lstm_int_model {
  int device = -1;
  std::vector<LayerHost> host;
  std::vector<LayerDev> dev;
  void *arena = nullptr;
  const uint16_t *sig3 = nullptr, *tanh3 = nullptr;
  WideTable wsig3, wtanh3;        // the gate tables in the wide form (rec_kernel)
  int *status = nullptr;  // device word raised by the persistent kernel when a wait gives up
  int path = 0;
  int reverse = 0;  // 1: the recursion runs from time T - 1 down to 0
  int cooperative = 0;  // 1: the persistent kernel is launched cooperatively
  int rows16 = 1;       // 1: batches that fit one launch of the 16-row kernel take it
  int sparse = 1;       // 1: layers whose recurrent weights are 2:4 run R h on the sparse MFMA (32-row kernel)
  int stack = 1;        // stacked launch (one layer per XCD): 0 never, 1 where it is expected to be faster, 2 wherever it can run
  int flag_sleep = 2;   // stacked launch: pause between two polls of the layer below's flag, x 64 clocks
  double stack_step_us = 20.5;
  int stack_prefetch_kb = 2048;  // stacked launch: KB of a layer's W asked for ahead of each W x  // expected time of one (step, row tile) item of the stacked launch
  bool stackable = false;            // every layer equal (and eligible): the stacked kernel can run the model
  int stack_ks = 0;
  const StackLayer *stack_layers = nullptr;  // [L] in the arena
  int spin_limit = 1 << 21;
  int poll_sleep = 0, stats_sleep = 0;  // pauses between polls, in units of 64 clocks
  int idle_sleep = 64, idle_poll_sleep = 12;
  int stats_first_sleep = 8;
  int sync_sleep = -1;  // pause before the first poll where all arrive together; -1 = by group size
  int phase_timing = 0;
  int extra_arrivals = 0;  // test hook: group barriers wait for one arrival too many (see RecArgs)
  int num_cus = 256;
  Profile prof;
};

namespace {

struct Workspace {
  size_t tx, out[2], xpad, th, mbuf, c, h0, sync, m2, total;
  size_t tx_bytes, out_bytes, m2_bytes;  // extents of the regions the persistent kernels index
};
constexpr size_t kStatGroupBytes = (size_t)kStatGroupWords * 8;  // statistics words of one group of workgroups
constexpr size_t kSyncBytes = 256 * 64 * 4 + 256 * kStatGroupBytes;  // counters + statistics accumulators
constexpr size_t kStackFlagsOff = 256 * 64 * 4 + 8 * kStatGroupBytes;  // stacked launch: flags behind the counters and the statistics words of its 8 layers

Workspace plan_workspace(const lstm_int_model *m, int64_t T, int64_t B) {
  int maxGN = 0, maxHpad = 0, maxNpad = 0, maxN = 0, maxNpadp = 0;
  for (size_t l = 0; l < m->host.size(); ++l) {
    const LayerHost &h = m->host[l];
    maxGN = std::max(maxGN, h.G * h.N);
    // the persistent path stores 4 gate slots over GS*64 cells, batch padded to 32
    if (!m->dev.empty() && m->dev[l].p2) {
      maxGN = std::max(maxGN, 4 * m->dev[l].Ncp);
      if (h.projection()) maxNpadp = std::max(maxNpadp, m->dev[l].npadp);
    }
    maxHpad = std::max(maxHpad, round_up(h.H, 128));
    maxNpad = std::max(maxNpad, round_up(h.N, 64));
    maxN = std::max(maxN, h.N);
  }
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += align256(bytes);
    return o;
  };
  w.tx_bytes = (size_t)T * ((B + 31) / 32 * 32) * maxGN * 2;
  w.out_bytes = ((size_t)T * B + 32) * maxHpad;
  w.m2_bytes = (size_t)T * round_up(B, 32) * maxNpadp;
  w.tx = take(w.tx_bytes);
  // 32 rows of slack behind the activation buffers: the input GEMM reads whole blocks of 32 rows
  w.out[0] = take(((size_t)T * B + 32) * maxHpad);
  w.out[1] = take(((size_t)T * B + 32) * maxHpad);
  w.xpad = take(((size_t)T * B + 32) * round_up(m->host[0].I, 64));
  w.th = take((size_t)B * maxGN * 2);
  w.mbuf = take((size_t)B * maxNpad);
  w.c = take((size_t)B * maxN * 2);
  w.h0 = take((size_t)B * maxHpad);
  w.sync = take(kSyncBytes);
  w.m2 = take((size_t)T * round_up(B, 32) * maxNpadp);
  w.total = off;
  return w;
}

// Workspace of a stacked launch: the sequential regions are not needed then, so the two layouts overlay.
struct StackPlan {
  size_t out, h0, mbuf, c, xpad, sync, total;
  size_t out_stride, mbuf_stride;
};
StackPlan plan_stack(const lstm_int_model *m, int64_t T, int64_t B) {
  const LayerHost &h = m->host[0];
  const int64_t L = (int64_t)m->host.size(), Hpad = round_up(h.H, 128), Bp = round_up((int)B, 32);
  StackPlan w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += align256(bytes);
    return o;
  };
  w.out_stride = align256(((size_t)T * B + 32) * Hpad);
  w.out = take(w.out_stride * L);
  w.h0 = take((size_t)L * B * Hpad);
  w.mbuf_stride = h.projection() ? align256((size_t)T * Bp * round_up(h.N, 128)) : 0;
  w.mbuf = take(w.mbuf_stride * L);
  w.c = take((size_t)L * B * h.N * 2);
  w.xpad = take(((size_t)T * B + 32) * round_up(h.I, 64));
  w.sync = take(kSyncBytes);
  w.total = off;
  return w;
}

// Whether forward runs T steps of B rows as one stacked launch (a function of the model, its options, T
// and B only: lstm_int_workspace_bytes and lstm_int_forward must agree).
bool stack_chosen(const lstm_int_model *m, int64_t T, int64_t B) {
  if (!m->stackable || m->stack == 0 || m->path == 1 || m->reverse) return false;
  int ks = 0;
  const LayerHost &h = m->host[0];
  const int L = (int)m->host.size();
  if (!stack_supported(h.N, h.H, (int)h.flags, m->dev[0].Ipad, L, (int)T, (int)B, &ks) || ks != m->stack_ks) return false;
  if (kStackFlagsOff + (size_t)L * ((B + 31) / 32) * 128 > kSyncBytes) return false;  // flags behind the statistics words
  if (m->stack == 2) return true;
  // Expected time of the two ways, in microseconds, from the times measured on the 8-layer benchmark stack
  // (N = 2048, H = 640).  One after the other: about 30 us per layer for the input GEMM launch and the weight
  // prologue, and 8.1 us per step up to 128 rows, 11 us per 256 rows beyond.  Stacked: every layer walks its
  // T * tiles items (step, tile of 32 rows) one after the other at about 20.5 us each, one item behind the
  // layer below.
  const double tiles = (double)((B + 31) / 32);
  const double seq = L * (30.0 + T * (B <= 128 ? 8.1 : 11.0 * ((B + 255) / 256)));
  const double stk = 25.0 + (T * tiles + L - 1) * m->stack_step_us;
  return stk < seq;
}

Requant make_requant(const int32_t *M, const int32_t *e, int first, int count, int cols_per_gate,
                     int zp) {
  Requant r;
  r.all_hi = 1;
  for (int g = 0; g < 4; ++g) {
    const int src = first + (g < count ? g : count - 1);
    r.M[g] = M[src];
    r.r[g] = 31 - e[src];
    if (r.r[g] < 33) r.all_hi = 0;
  }
  r.cols_per_gate = cols_per_gate;
  r.zp = zp;
  return r;
}

// Whether everything a launch of a persistent recurrent kernel indexes with these arguments lies inside
// the workspace regions it was given (checked on the host before every launch: an access out of bounds
// on the device can take the whole GPU down).  T_all = steps of the whole call, t0 = first step of this launch.
bool rec_extents_ok(const RecArgs &ra, const Workspace &ws, int T_all, int t0, bool has_proj) {
  const size_t Bp = (size_t)ra.Bp;
  if (ra.Bp % 32 || ra.Bp < ra.B || ra.B < 1 || ra.T < 1 || t0 < 0 || t0 + ra.T > T_all) return false;
  if (ra.groups < 1 || ra.groups > 256 || ra.batch0 < 0 || ra.batch0 >= ra.B) return false;
  // the first row of every group is a real row: later row tiles of a group are skipped or clamped by the kernels
  if ((int64_t)ra.batch0 + (int64_t)(ra.groups - 1) * ra.rows_pg >= ra.B) return false;
  // W x terms: [T_all * Bp / 32][GS * 8 tiles][2][64 lanes] 16-byte pieces
  if ((size_t)T_all * Bp / 32 * (size_t)(ra.GS * 8) * 2 * 64 * 16 > ws.tx_bytes) return false;
  // layer output [T_all, B, Hpad]
  if ((size_t)T_all * ra.B * ra.Hpad > ws.out_bytes) return false;
  // m exchange buffer [T][Bp][npadp] in tiles
  if (has_proj && (size_t)ra.T * Bp * ra.npadp > ws.m2_bytes) return false;
  // counters [groups][64] words and statistics accumulators [groups][4][256] 64-bit words
  if ((size_t)ra.groups * 64 * 4 > (size_t)256 * 64 * 4 || (size_t)ra.groups * kStatGroupBytes > (size_t)256 * kStatGroupBytes)
    return false;
  return true;
}

// Times each launch with a pair of events when profiling is on.
struct Timed {
  Profile &p;
  hipStream_t s;
  bool active;
  Timed(Profile &prof, hipStream_t stream, int cls) : p(prof), s(stream), active(false) {
    if (!p.on) return;
    // events are created as launches need them (any number of launches per call) and freed by profile_end
    if ((p.used + 1) * 2 > p.ev.size()) {
      hipEvent_t e0 = nullptr, e1 = nullptr;
      if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        p.failed = true;
        return;
      }
      p.ev.push_back(e0);
      p.ev.push_back(e1);
      p.cls.push_back(0);
    }
    active = true;
    p.cls[p.used] = cls;
    p.stream = s;
    (void)hipEventRecord(p.ev[2 * p.used], s);
  }
  ~Timed() {
    if (active) {
      (void)hipEventRecord(p.ev[2 * p.used + 1], s);
      ++p.used;
    }
  }
};

// How the one-product rescale must treat an operand bounded by amax in magnitude
// when the shift is r: 0 = as it is (r >= 33), 1 = shifted left by 33 - r (the
// shifted bound still fits 32 bits), 2 = clamped first.
int preshift_mode(int r, int64_t amax) {
  if (r >= 33) return 0;
  const int k = 33 - r;
  return (k < 31 && (amax << k) <= 0x7FFFFFFFll) ? 1 : 2;
}

int upload(lstm_int_model *m) {
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  if (hipDeviceGetAttribute(&m->num_cus, hipDeviceAttributeMultiprocessorCount, m->device) != hipSuccess ||
      m->num_cus < 1)
    return LSTM_INT_E_DEVICE;
  const size_t L = m->host.size();
  m->dev.resize(L);

  // pass 1: sizes; pass 2: fill a host image of the arena, then one copy
  std::vector<uint8_t> image;
  bool need_tanh[9] = {false, false, false, false, false, false, false, false, false};
  for (const LayerHost &h : m->host) need_tanh[h.m_c] = true;
  need_tanh[3] = true;
  size_t tab_off[9], sig_off = 0;
  size_t wide_off[9], wide_sig_off = 0;
  WideTable wide_tab[9], wide_sig;
  for (int pass = 0; pass < 2; ++pass) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
      size_t o = off;
      off += align256(bytes);
      return o;
    };
    sig_off = take(32769 * 2);
    wide_sig_off = take(kLutWideBytes);
    const size_t status_off = take(256);
    if (pass) {
      fill_sigmoid_table(3, reinterpret_cast<uint16_t *>(image.data() + sig_off));
      wide_sig.sh = compress_table_wide(reinterpret_cast<const uint16_t *>(image.data() + sig_off),
                                        image.data() + wide_sig_off, &wide_sig.has_tail, &wide_sig.flat_from);
      wide_sig.blob = static_cast<const uint8_t *>(m->arena) + wide_sig_off;
      m->status = reinterpret_cast<int *>(static_cast<uint8_t *>(m->arena) + status_off);
    }
    for (int mc = 0; mc <= 8; ++mc) {
      if (!need_tanh[mc]) continue;
      tab_off[mc] = take(32769 * 2);
      wide_off[mc] = take(kLutWideBytes);
      if (pass) {
        fill_tanh_table(mc, reinterpret_cast<uint16_t *>(image.data() + tab_off[mc]));
        wide_tab[mc].sh = compress_table_wide(reinterpret_cast<const uint16_t *>(image.data() + tab_off[mc]),
                                              image.data() + wide_off[mc], &wide_tab[mc].has_tail, &wide_tab[mc].flat_from);
        wide_tab[mc].blob = static_cast<const uint8_t *>(m->arena) + wide_off[mc];
      }
    }
    for (size_t l = 0; l < L; ++l) {
      const LayerHost &h = m->host[l];
      LayerDev &d = m->dev[l];
      const int first = 4 - h.G;
      d.Ipad = round_up(h.I, 64);
      d.Hpad = round_up(h.H, 128);
      d.Npad = round_up(h.N, 64);
      d.GN = h.G * h.N;
      const int rows = round_up(d.GN, 128);
      const size_t oW = take((size_t)rows * d.Ipad), oR = take((size_t)rows * d.Hpad);
      const size_t obx = take((size_t)rows * 4), obh = take((size_t)rows * 4);
      const size_t oP = take((size_t)3 * h.N * 2), oL = take((size_t)4 * h.N * 2);
      const size_t oqb = take((size_t)4 * h.N * 4);
      size_t oWp = 0, obp = 0;
      const int prow = round_up(h.H, 128);
      if (h.projection()) {
        oWp = take((size_t)prow * d.Npad);
        obp = take((size_t)prow * 4);
      }
      // tile-ordered copies for the persistent path
      int ks = 0, rt = 0, grp = 0;
      d.p2 = rec_supported(h.N, h.H, (int)h.flags, 32, &ks, &rt, &grp);
      size_t oW2f = 0, oR2h = 0, oR2s = 0;
      bool r_sparse = false;
      int ks16 = 0, grp16 = 0;
      d.p16 = d.p2 && rec16_supported(h.N, h.H, (int)h.flags, 16, &ks16, &grp16);
      size_t oW2 = 0, obx2 = 0, oR2 = 0, obh4 = 0, oqb4 = 0, oLq4 = 0, oPq3 = 0, oWp2 = 0, obp2 = 0, oWp3 = 0, obp3 = 0;
      if (d.p2) {
        d.GS = (h.N + 63) / 64;
        d.ks = ks;
        d.Ncp = d.GS * 64;
        d.ptiles = h.projection() ? (h.H + 31) / 32 : 0;
        d.npadp = round_up(h.N, 128);
        oW2 = take((size_t)d.GS * 8 * 32 * d.Ipad);
        if (d.Ipad <= 1024) oW2f = take((size_t)d.GS * 8 * 32 * d.Ipad);
        obx2 = take((size_t)d.GS * 8 * 32 * 4);
        oR2 = take((size_t)d.GS * 4 * 2 * ks * 64 * 16);
        r_sparse = true;
        for (int g = first; g < 4 && r_sparse; ++g)
          for (int n = 0; n < h.N && r_sparse; ++n)
            r_sparse = sparse24_row_ok(h.Rq.data() + ((size_t)g * h.N + n) * h.H, h.H);
        if (r_sparse) oR2s = take(rec_sparse_bytes(d.GS, ks));
        if (d.p16) {
          d.ks16 = ks16;
          oR2h = take((size_t)d.GS * 4 * 4 * ks16 * 64 * 16);
        }
        obh4 = take((size_t)4 * d.Ncp * 4);
        oqb4 = take((size_t)4 * d.Ncp * 4);
        oLq4 = take((size_t)4 * d.Ncp * 2);
        oPq3 = take((size_t)3 * d.Ncp * 2);
        if (h.projection()) {
          oWp2 = take((size_t)d.ptiles * 32 * d.npadp);
          obp2 = take((size_t)d.ptiles * 32 * 4);
          d.prow = 32;
          d.ptiles3 = d.ptiles;
          if (d.ptiles <= d.GS) {  // at most one 32-row tile per workgroup: spread the outputs evenly instead
            d.prow = round_up((h.H + d.GS - 1) / d.GS, 4);
            d.ptiles3 = (h.H + d.prow - 1) / d.prow;
            oWp3 = take((size_t)d.ptiles3 * 32 * d.npadp);
            obp3 = take((size_t)d.ptiles3 * 32 * 4);
          }
        }
      }
      if (!pass) continue;
      uint8_t *base = image.data();
      if (d.p2) {
        for (int g = first; g < 4; ++g) {
          for (int n = 0; n < h.N; ++n) {
            const size_t src = (size_t)g * h.N + n;
            const size_t trow = (size_t)(n / 8) * 32 + 8 * g + (n % 8);  // tile row rho = 8*gate + cell%8
            int64_t sx = 0, sh = 0;
            for (int k = 0; k < h.I; ++k) sx += std::abs((int)h.Wq[src * h.I + k]);
            for (int k = 0; k < h.H; ++k) sh += std::abs((int)h.Rq[src * h.H + k]);
            d.amax_x[g] = std::max<int64_t>(d.amax_x[g], (int64_t)std::llabs((long long)h.bx_fold[src]) + 128 * sx);
            d.amax_h[g] = std::max<int64_t>(d.amax_h[g], (int64_t)std::llabs((long long)h.bh_fold[src]) + 128 * sh);
            memcpy(base + oW2 + trow * d.Ipad, h.Wq.data() + src * h.I, h.I);
            if (d.Ipad <= 1024) {
              // lane = rho + 32 * (k / 16 % 2) holds bytes k % 16 of k step k / 32
              const int rho = 8 * g + (n % 8);
              for (int k = 0; k < h.I; ++k) {
                const size_t o = ((((size_t)(n / 8) * (d.Ipad / 32) + k / 32) * 64) + rho + 32 * ((k % 32) / 16)) * 16 + k % 16;
                base[oW2f + o] = (uint8_t)h.Wq[src * h.I + k];
              }
            }
            reinterpret_cast<int32_t *>(base + obx2)[trow] = h.bx_fold[src];
            reinterpret_cast<int32_t *>(base + obh4)[(size_t)g * d.Ncp + n] = h.bh_fold[src];
            reinterpret_cast<int32_t *>(base + oqb4)[(size_t)g * d.Ncp + n] = h.qb[src];
            reinterpret_cast<int16_t *>(base + oLq4)[(size_t)g * d.Ncp + n] = h.Lq[src];
            // recurrent weights: [member][wave][tile][ks][lane][16], lane = rho + 32 * (k / 16 % 2)
            const int member = n / 64, wave = (n % 64) / 16, tl = (n % 16) / 8, rho = 8 * g + (n % 8);
            for (int k = 0; k < h.H; ++k) {
              const int kstep = k / 32, lane = rho + 32 * ((k % 32) / 16), byte = k % 16;
              const size_t o = ((((size_t)(member * 4 + wave) * 2 + tl) * ks + kstep) * 64 + lane) * 16 + byte;
              base[oR2 + o] = (uint8_t)h.Rq[src * h.H + k];
            }
            if (r_sparse) {
              const int kw = ks / 2;
              uint8_t *vals = base + oR2s;
              uint32_t *index = reinterpret_cast<uint32_t *>(vals + (size_t)d.GS * 4 * 2 * kw * 64 * 16);
              for (int q = 0; q < kw; ++q)
                for (int a2 = 0; a2 < 2; ++a2) {
                  const size_t slot = (((size_t)(member * 4 + wave) * 2 + tl) * kw + q) * 64 + rho + 32 * a2;
                  sparse24_pack_lane(h.Rq.data() + src * h.H, h.H, q, a2, reinterpret_cast<int8_t *>(vals + slot * 16),
                                     index + slot);
                }
            }
            if (d.p16) {
              // 16-row kernel: [member][wave][tile j][ks16][lane][16]; tile j of a wave holds cell
              // 16 wave + 4 q + j of gate g in row 4 q + g, lane = row + 16 * (k / 16 % 4)
              const int j = n % 4, trow16 = 4 * ((n % 16) / 4) + g;
              for (int k = 0; k < h.H; ++k) {
                const size_t o =
                    ((((size_t)(member * 4 + wave) * 4 + j) * ks16 + k / 64) * 64 + trow16 + 16 * ((k % 64) / 16)) * 16 + k % 16;
                base[oR2h + o] = (uint8_t)h.Rq[src * h.H + k];
              }
            }
          }
        }
        for (int j = first; j < 3; ++j)
          for (int n = 0; n < h.N; ++n)
            reinterpret_cast<int16_t *>(base + oPq3)[(size_t)j * d.Ncp + n] = h.Pq[(size_t)j * h.N + n];
        if (h.projection()) {
          for (int pcol = 0; pcol < h.H; ++pcol) {
            memcpy(base + oWp2 + (size_t)pcol * d.npadp, h.Wpq.data() + (size_t)pcol * h.N, h.N);
            reinterpret_cast<int32_t *>(base + obp2)[pcol] = h.bp_fold[pcol];
            if (d.prow != 32) {
              const size_t row3 = (size_t)(pcol / d.prow) * 32 + pcol % d.prow;
              memcpy(base + oWp3 + row3 * d.npadp, h.Wpq.data() + (size_t)pcol * h.N, h.N);
              reinterpret_cast<int32_t *>(base + obp3)[row3] = h.bp_fold[pcol];
            }
          }
        }
        uint8_t *db = static_cast<uint8_t *>(m->arena);
        d.W2 = reinterpret_cast<int8_t *>(db + oW2);
        d.W2f = d.Ipad <= 1024 ? reinterpret_cast<int8_t *>(db + oW2f) : nullptr;
        d.bx2 = reinterpret_cast<int32_t *>(db + obx2);
        d.R2 = reinterpret_cast<int4 *>(db + oR2);
        d.R2h = d.p16 ? reinterpret_cast<int4 *>(db + oR2h) : nullptr;
        d.R2s = r_sparse ? reinterpret_cast<int4 *>(db + oR2s) : nullptr;
        d.bh4 = reinterpret_cast<int32_t *>(db + obh4);
        d.qb4 = reinterpret_cast<int32_t *>(db + oqb4);
        d.Lq4 = reinterpret_cast<int16_t *>(db + oLq4);
        d.Pq3 = reinterpret_cast<int16_t *>(db + oPq3);
        if (h.projection()) {
          d.Wp2 = reinterpret_cast<int8_t *>(db + oWp2);
          d.bp2 = reinterpret_cast<int32_t *>(db + obp2);
          d.Wp3 = d.prow != 32 ? reinterpret_cast<int8_t *>(db + oWp3) : d.Wp2;
          d.bp3 = d.prow != 32 ? reinterpret_cast<int32_t *>(db + obp3) : d.bp2;
        }
      }
      for (int g = first; g < 4; ++g) {
        for (int n = 0; n < h.N; ++n) {
          const size_t src = (size_t)g * h.N + n, dst = (size_t)(g - first) * h.N + n;
          memcpy(base + oW + dst * d.Ipad, h.Wq.data() + src * h.I, h.I);
          memcpy(base + oR + dst * d.Hpad, h.Rq.data() + src * h.H, h.H);
          reinterpret_cast<int32_t *>(base + obx)[dst] = h.bx_fold[src];
          reinterpret_cast<int32_t *>(base + obh)[dst] = h.bh_fold[src];
        }
      }
      memcpy(base + oP, h.Pq.data(), (size_t)3 * h.N * 2);
      memcpy(base + oL, h.Lq.data(), (size_t)4 * h.N * 2);
      memcpy(base + oqb, h.qb.data(), (size_t)4 * h.N * 4);
      if (h.projection()) {
        for (int j = 0; j < h.H; ++j) {
          memcpy(base + oWp + (size_t)j * d.Npad, h.Wpq.data() + (size_t)j * h.N, h.N);
          reinterpret_cast<int32_t *>(base + obp)[j] = h.bp_fold[j];
        }
      }
      uint8_t *dbase = static_cast<uint8_t *>(m->arena);
      d.W = reinterpret_cast<int8_t *>(dbase + oW);
      d.R = reinterpret_cast<int8_t *>(dbase + oR);
      d.bx = reinterpret_cast<int32_t *>(dbase + obx);
      d.bh = reinterpret_cast<int32_t *>(dbase + obh);
      d.Pq = reinterpret_cast<int16_t *>(dbase + oP);
      d.Lq = reinterpret_cast<int16_t *>(dbase + oL);
      d.qb = reinterpret_cast<int32_t *>(dbase + oqb);
      if (h.projection()) {
        d.Wproj = reinterpret_cast<int8_t *>(dbase + oWp);
        d.bp = reinterpret_cast<int32_t *>(dbase + obp);
      }
      d.tanhc = reinterpret_cast<const uint16_t *>(dbase + tab_off[h.m_c]);
      d.wtanhc = wide_tab[h.m_c];
      d.rq_x = make_requant(h.Mx, h.ex, first, h.G, h.N, 0);
      d.rq_h = make_requant(h.Mh, h.eh, first, h.G, h.N, 0);
      if (h.projection()) d.rq_p = make_requant(&h.Mp, &h.ep, 0, 1, 1 << 28, h.zp_h);
    }
    {  // constants of the stacked kernel, one record per layer (filled when every layer has its tile-ordered copies)
      const size_t oStack = take(L * sizeof(StackLayer));
      if (pass) {
        bool all = true;
        for (size_t l = 0; l < L; ++l) all = all && m->dev[l].p2 && m->dev[l].W2f;
        if (all) {
          StackLayer *recs = reinterpret_cast<StackLayer *>(image.data() + oStack);
          for (size_t l = 0; l < L; ++l) {
            const LayerHost &h = m->host[l];
            const LayerDev &d = m->dev[l];
            StackLayer &r = recs[l];
            memset(&r, 0, sizeof(r));
            r.R2 = d.R2; r.W2f = d.W2f; r.bx2 = d.bx2; r.bh4 = d.bh4; r.Lq4 = d.Lq4; r.qb4 = d.qb4; r.Pq3 = d.Pq3;
            r.Wp2 = d.Wp3; r.bp2 = d.bp3;  // the tiling by rows per workgroup where there is one
            {
              int dom = 0, tail = 0;
              d.wtanhc.shortest(&dom, &tail);
              r.lutc.blob = d.wtanhc.blob; r.lutc.sh = d.wtanhc.sh; r.lutc.dom = dom; r.lutc.tail = tail;
            }
            r.kx = d.Ipad / 32;
            r.pre_x = r.pre_h = 0;
            for (int g = 0; g < 4; ++g) {
              const int sg = g < 4 - h.G ? 4 - h.G : g;  // an absent gate borrows valid numbers; its rows are zero
              r.Mx[g] = h.Mx[sg]; r.rx[g] = 31 - h.ex[sg];
              r.Mh[g] = h.Mh[sg]; r.rh[g] = 31 - h.eh[sg];
              r.Mln[g] = h.Mln[sg]; r.rln[g] = 31 - h.eln[sg];
              r.pre_x = std::max(r.pre_x, preshift_mode(r.rx[g], d.amax_x[sg]));
              r.pre_h = std::max(r.pre_h, preshift_mode(r.rh[g], d.amax_h[sg]));
            }
            for (int j = 0; j < 3; ++j) { r.Mc[j] = h.Mc[j]; r.rc[j] = 31 - h.ec[j]; }
            r.Mm = h.Mm; r.rm = 31 - h.em; r.zp_m = h.zp_m;
            r.Mp = h.Mp; r.rp = 31 - h.ep; r.zp_h = h.zp_h; r.m_c = h.m_c;
          }
          m->stack_layers = reinterpret_cast<const StackLayer *>(static_cast<uint8_t *>(m->arena) + oStack);
        }
      }
    }
    if (!pass) {
      image.assign(off, 0);
      if (hipMalloc(&m->arena, off) != hipSuccess) {
        m->arena = nullptr;
        return LSTM_INT_E_OUT_OF_MEMORY;
      }
    }
  }
  if (hipMemcpy(m->arena, image.data(), image.size(), hipMemcpyHostToDevice) != hipSuccess)
    return LSTM_INT_E_DEVICE;
  const uint8_t *dbase = static_cast<const uint8_t *>(m->arena);
  m->sig3 = reinterpret_cast<const uint16_t *>(dbase + sig_off);
  m->tanh3 = reinterpret_cast<const uint16_t *>(dbase + tab_off[3]);
  m->wsig3 = wide_sig;
  m->wtanh3 = wide_tab[3];
  if (rec_init() != hipSuccess || rec16_init() != hipSuccess || in_gemm_init() != hipSuccess || gemm_init() != hipSuccess || stack_init() != hipSuccess)
    return LSTM_INT_E_DEVICE;
  // The stacked kernel runs models whose layers are all alike (same cells, width and variant; every layer
  // above the first reads the layer below), up to 8 of them, within the shift and table limits of the
  // persistent kernels.
  m->stackable = false;
  if (m->stack_layers && L >= 2 && L <= 8) {
    const LayerHost &h0 = m->host[0];
    bool ok = stack_supported(h0.N, h0.H, (int)h0.flags, m->dev[0].Ipad, (int)L, 1, 1, &m->stack_ks);
    auto shift_ok = [](int r) { return r >= 3 && r <= 62; };
    for (size_t l = 0; l < L && ok; ++l) {
      const LayerHost &h = m->host[l];
      const LayerDev &d = m->dev[l];
      ok = h.N == h0.N && h.H == h0.H && h.flags == h0.flags && (l == 0 || h.I == h0.H) && d.ks == m->stack_ks &&
           shift_ok(31 - h.em) && (!h.projection() || shift_ok(31 - h.ep)) && wide_sig.sh >= 0 && wide_tab[3].sh >= 0 &&
           d.wtanhc.sh >= 0;
      for (int g = 4 - h.G; g < 4 && ok; ++g)
        ok = shift_ok(31 - h.ex[g]) && shift_ok(31 - h.eh[g]) && (!h.layer_norm() || shift_ok(31 - h.eln[g]));
      for (int j = 4 - h.G; j < 3 && ok; ++j) ok = !h.peephole() || shift_ok(31 - h.ec[j]);
    }
    m->stackable = ok;
  }
  return scratch_lookup(m->device);  // the device is current here
}

}  // namespace

extern "C" {

int lstm_int_prepare(const lstm_int_layer_params *layers, int32_t num_layers, int32_t device,
                     lstm_int_model **out) {
  if (!out) return LSTM_INT_E_INVALID_ARG;
  *out = nullptr;
  if (device < -1) return LSTM_INT_E_INVALID_ARG;
  lstm_int_model *m = new (std::nothrow) lstm_int_model();
  if (!m) return LSTM_INT_E_OUT_OF_MEMORY;
  int rc;
  try {
    rc = prepare_host(layers, num_layers, m->host);
    m->device = device;
    if (rc == LSTM_INT_OK && device >= 0) rc = upload(m);
  } catch (const std::bad_alloc &) {
    rc = LSTM_INT_E_OUT_OF_MEMORY;
  }
  if (rc != LSTM_INT_OK) {
    lstm_int_destroy(m);
    return rc;
  }
  *out = m;
  return LSTM_INT_OK;
}

int lstm_int_get_quant(const lstm_int_model *m, int32_t layer, lstm_int_layer_quant *q) {
  if (!m || !q || layer < 0 || layer >= (int32_t)m->host.size()) return LSTM_INT_E_INVALID_ARG;
  const LayerHost &h = m->host[layer];
  memset(q, 0, sizeof(*q));
  q->I = h.I; q->N = h.N; q->H = h.H; q->G = h.G;
  q->flags = h.flags;
  q->m_c = h.m_c;
  q->zp_x = h.zp_x; q->zp_h = h.zp_h; q->zp_m = h.zp_m;
  q->s_x = h.s_x; q->s_h = h.s_h; q->s_m = h.s_m; q->s_c = h.s_c; q->s_Wp = h.s_Wp;
  for (int g = 0; g < 4; ++g) {
    q->s_W[g] = h.s_W[g]; q->s_R[g] = h.s_R[g]; q->s_L[g] = h.s_L[g]; q->s_g[g] = h.s_g[g];
    q->Mx[g] = h.Mx[g]; q->ex[g] = h.ex[g]; q->Mh[g] = h.Mh[g]; q->eh[g] = h.eh[g];
    q->Mln[g] = h.Mln[g]; q->eln[g] = h.eln[g];
  }
  for (int j = 0; j < 3; ++j) {
    q->s_P[j] = h.s_P[j]; q->Mc[j] = h.Mc[j]; q->ec[j] = h.ec[j];
  }
  q->Mm = h.Mm; q->em = h.em; q->Mp = h.Mp; q->ep = h.ep;
  q->Wq = h.Wq.data(); q->Rq = h.Rq.data(); q->qb = h.qb.data();
  q->Pq = h.Pq.data(); q->Lq = h.Lq.data();
  q->bx_fold = h.bx_fold.data(); q->bh_fold = h.bh_fold.data();
  if (h.projection()) {
    q->Wpq = h.Wpq.data(); q->qbp = h.qbp.data(); q->bp_fold = h.bp_fold.data();
  }
  return LSTM_INT_OK;
}

int lstm_int_quantize_input(const lstm_int_model *m, const float *x, int64_t n, int8_t *xq, void *hip_stream) {
  if (!m || n < 0 || m->host.empty()) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  if (n == 0) return LSTM_INT_OK;
  if (!x || !xq) return LSTM_INT_E_INVALID_ARG;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  launch_quantize_input(static_cast<hipStream_t>(hip_stream), x, xq, n, m->host[0].s_x, m->host[0].zp_x);
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

size_t lstm_int_workspace_bytes(const lstm_int_model *m, int32_t T, int32_t B) {
  if (!m || T < 0 || B < 0 || m->host.empty()) return 0;
  if (T == 0 || B == 0) return 256;
  // a call with a trace runs the layers one after the other, so that layout always has to fit
  const size_t seq = plan_workspace(m, T, B).total;
  return m->device >= 0 && stack_chosen(m, T, B) ? std::max(seq, plan_stack(m, T, B).total) : seq;
}

}  // extern "C"

namespace {

// All layers in one launch (stack_kernel.inc.h).  The caller has checked stack_chosen and the workspace size.
int forward_stack(lstm_int_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y, int8_t *h_state,
                  int16_t *c_state, uint8_t *wsb, hipStream_t s) {
  const StackPlan sp = plan_stack(m, T, B);
  const LayerHost &h = m->host[0];
  const LayerDev &d = m->dev[0];
  const int L = (int)m->host.size();
  const int TB = T * B;
  // the first layer reads x in place when its rows are 64-byte multiples and 16-byte aligned
  const int8_t *in = x;
  int ld_in = h.I;
  if ((h.I & 63) || (reinterpret_cast<uintptr_t>(x) & 15)) {
    Timed t(m->prof, s, LSTM_INT_K_OTHER);
    int8_t *xp = reinterpret_cast<int8_t *>(wsb + sp.xpad);
    launch_copy_rows_i8(s, x, h.I, xp, d.Ipad, TB, h.I, 0);
    in = xp;
    ld_in = d.Ipad;
  }
  StackArgs sa;
  memset(&sa, 0, sizeof(sa));
  RecArgs &ra = sa.c;
  ra.T = T; ra.B = B; ra.N = h.N; ra.H = h.H; ra.Hpad = d.Hpad; ra.flags = (int)h.flags; ra.m_c = h.m_c;
  ra.GS = d.GS; ra.groups = L; ra.rows_pg = 32; ra.ks = d.ks; ra.Ncp = d.Ncp; ra.Bp = round_up(B, 32);
  ra.ptiles = d.ptiles3; ra.npadp = d.npadp; ra.prow = d.prow;
  // the tables: the cell-format tanh of every layer at its shortest prefix (a layer whose format is the gates'
  // shares the gate tanh's copy), the two gate tables as long as the LDS left allows
  {
    auto set_lut = [&](int i, const WideTable &w) {
      int dom = 0, tail = 0;
      w.shortest(&dom, &tail);
      ra.lut[i].blob = w.blob; ra.lut[i].sh = w.sh; ra.lut[i].dom = dom; ra.lut[i].tail = tail;
    };
    set_lut(0, m->wsig3);
    set_lut(1, m->wtanh3);
    sa.lutc_lds_bytes = 0;
    for (int l = 0; l < L; ++l) {
      const WideTable &w = m->dev[l].wtanhc;
      if (w.blob == m->wtanh3.blob) continue;
      int dom = 0, tail = 0;
      w.shortest(&dom, &tail);
      sa.lutc_lds_bytes = std::max(sa.lutc_lds_bytes, lut_wide_lds_bytes(dom, w.sh, tail != 0));
    }
  }
  ra.y = y;
  ra.counters = reinterpret_cast<unsigned *>(wsb + sp.sync);
  ra.tickets = m->cooperative ? nullptr : reinterpret_cast<unsigned long long *>(ra.counters + 2);
  ra.acc = reinterpret_cast<unsigned long long *>(wsb + sp.sync + 256 * 64 * 4);
  ra.status = m->status;
  ra.spin_limit = m->spin_limit;
  ra.poll_sleep = m->poll_sleep; ra.stats_sleep = m->stats_sleep; ra.idle_sleep = m->idle_sleep;
  ra.stats_first_sleep = m->stats_first_sleep;
  ra.sync_sleep = m->sync_sleep >= 0 ? m->sync_sleep : (d.GS >= 16 ? 16 : 4);
  ra.idle_poll_sleep = m->idle_poll_sleep;
  ra.ticks = m->phase_timing ? reinterpret_cast<long long *>(m->status + 16) : nullptr;
  ra.extra_arrivals = m->extra_arrivals;
  sa.layers = m->stack_layers;
  sa.L = L;
  sa.row_tiles = (B + 31) / 32;
  sa.x = in; sa.ldx = ld_in; sa.x_shared = 1;
  sa.out_base = reinterpret_cast<int8_t *>(wsb + sp.out); sa.out_stride = sp.out_stride;
  sa.h0_base = reinterpret_cast<const int8_t *>(wsb + sp.h0);
  sa.mbuf_base = reinterpret_cast<int8_t *>(wsb + sp.mbuf); sa.mbuf_stride = sp.mbuf_stride;
  sa.c_base = c_state ? c_state : reinterpret_cast<int16_t *>(wsb + sp.c);
  sa.c_given = c_state != nullptr;
  sa.h_final = h_state;
  const size_t flags_off = kStackFlagsOff;
  sa.flags = reinterpret_cast<unsigned *>(wsb + sp.sync + flags_off);
  sa.flag_sleep = m->flag_sleep;
  sa.tick_layer = std::min(L - 1, std::max(0, m->phase_timing - 1));
  {
    // W of a layer is 4 N Ipad bytes, read by the GS workgroups of one XCD through its 4 MB L2: ask ahead for
    // at most stack_prefetch_kb KB of it per XCD (default 2 MB), spread evenly over the waves
    const int64_t per_wave = (int64_t)m->stack_prefetch_kb * 8 / ((int64_t)d.GS * 4);
    sa.prefetch_lines = (int)std::min<int64_t>(per_wave, 16 * (int64_t)(m->dev[L - 1].Ipad / 32));
  }
  if (stack_lds_bytes(sa) > 160 * 1024) return LSTM_INT_E_UNSUPPORTED;
  {
    // longer prefixes of the gate tables into the LDS that is left, as for the kernels of one layer -- unless a
    // layer shares the gate tanh's copy for its cell format: that copy then stays at the prefix its record names
    bool shares = false;
    for (int l = 0; l < L; ++l) shares = shares || m->dev[l].wtanhc.blob == m->wtanh3.blob;
    bool grew = true;
    while (grew) {
      grew = false;
      for (int i = 0; i < 2; ++i) {
        if (i == 1 && shares) continue;
        const WideTable &w = i == 0 ? m->wsig3 : m->wtanh3;
        const LutWide keep = ra.lut[i];
        if (keep.dom >= 32768 || (!keep.tail && keep.dom - 1 >= w.flat_from)) continue;
        ra.lut[i].dom = keep.dom + 1024;
        ra.lut[i].tail = (ra.lut[i].dom - 1 < w.flat_from) ? 1 : 0;
        if ((ra.lut[i].tail && !w.has_tail) || stack_lds_bytes(sa) > 160 * 1024)
          ra.lut[i] = keep;
        else
          grew = true;
      }
    }
  }
  {
    Timed t(m->prof, s, LSTM_INT_K_OTHER);
    StackInit si;
    memset(&si, 0, sizeof(si));
    si.h_src = h_state; si.h0 = reinterpret_cast<int8_t *>(wsb + sp.h0); si.ld_h0 = d.Hpad; si.rows = B; si.cols = h.H;
    si.L = L;
    for (int l = 0; l < L; ++l) si.zp[l] = m->host[l].zp_h;
    si.sync = reinterpret_cast<int4 *>(wsb + sp.sync);
    si.sync_vec = (long long)((flags_off + (size_t)L * sa.row_tiles * 128 + 15) / 16);
    launch_stack_init(s, si);
  }
  {
    Timed t(m->prof, s, LSTM_INT_K_RECURRENT);
    if (launch_stack(s, sa, m->cooperative != 0) != hipSuccess) return LSTM_INT_E_DEVICE;
  }
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

}  // namespace

extern "C" {

int lstm_int_forward(const lstm_int_model *cm, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                     int8_t *h_state, int16_t *c_state, void *workspace, size_t workspace_bytes,
                     void *hip_stream, const lstm_int_trace *trace) {
  lstm_int_model *m = const_cast<lstm_int_model *>(cm);  // profiling counters only
  if (!m || T < 0 || B < 0) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  if (T == 0 || B == 0) return LSTM_INT_OK;
  if (!x || !y || !workspace) return LSTM_INT_E_INVALID_ARG;
  const int L = (int)m->host.size();
  if (trace && (trace->layer < 0 || trace->layer >= L)) return LSTM_INT_E_INVALID_ARG;
  if ((int64_t)T * B > (int64_t)1 << 30) return LSTM_INT_E_UNSUPPORTED;
  const Workspace ws = plan_workspace(m, T, B);
  if (workspace_bytes < lstm_int_workspace_bytes(m, T, B) || (reinterpret_cast<uintptr_t>(workspace) & 255))
    return LSTM_INT_E_WORKSPACE;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  uint8_t *wsb = static_cast<uint8_t *>(workspace);
  // every layer alike, no dump asked for: all layers in one launch, one layer per XCD, where that is faster
  if (!trace && stack_chosen(m, T, B) && (reinterpret_cast<uintptr_t>(y) & 3) == 0 &&
      (reinterpret_cast<uintptr_t>(h_state) & 3) == 0 && (reinterpret_cast<uintptr_t>(c_state) & 1) == 0) {
    const int rc = forward_stack(m, x, T, B, y, h_state, c_state, wsb, s);
    if (rc != LSTM_INT_E_UNSUPPORTED) return rc;  // the LDS budget did not fit: the layers run one after the other
  }
  int16_t *tx = reinterpret_cast<int16_t *>(wsb + ws.tx);
  int16_t *th = reinterpret_cast<int16_t *>(wsb + ws.th);
  int8_t *mbuf = reinterpret_cast<int8_t *>(wsb + ws.mbuf);
  int16_t *c = reinterpret_cast<int16_t *>(wsb + ws.c);
  int8_t *h0 = reinterpret_cast<int8_t *>(wsb + ws.h0);
  const int TB = T * B;

  // layer 0 reads x in place when its rows are already 64-byte multiples and the batch fills whole
  // blocks of 32 rows (the input GEMM reads whole blocks, up to 31 rows beyond the last real one)
  const int8_t *in = x;
  int ld_in = m->host[0].I;
  // A reverse run is the forward run on the time-flipped sequence: x is flipped on the way in, every
  // buffer between the layers is then indexed by step (step k works at time T - 1 - k), and y (and the
  // traces) are flipped back on the way out.  The kernels know nothing of it.
  const bool rev = m->reverse != 0;
  if ((m->host[0].I & 63) || (reinterpret_cast<uintptr_t>(x) & 15) || (B & 31) || rev) {
    Timed t(m->prof, s, LSTM_INT_K_OTHER);
    int8_t *xp = reinterpret_cast<int8_t *>(wsb + ws.xpad);
    if (rev)
      launch_flip_rows_i8(s, x, m->host[0].I, xp, m->dev[0].Ipad, T, B, m->host[0].I, 0);
    else
      launch_copy_rows_i8(s, x, m->host[0].I, xp, m->dev[0].Ipad, TB, m->host[0].I, 0);
    in = xp;
    ld_in = m->dev[0].Ipad;
  }

  // The final h of a layer on the persistent path goes to the caller's state buffer together with the
  // next such layer's start (one launch less per layer), or at the latest when forward ends.
  struct {
    const int8_t *src = nullptr;
    int ld = 0, cols = 0;
    int8_t *dst = nullptr;
  } pend;
  auto flush_pending = [&]() {
    if (pend.dst) launch_copy_rows_i8(s, pend.src, pend.ld, pend.dst, pend.cols, B, pend.cols, 0);
    pend.dst = nullptr;
  };
  size_t h_off = 0, c_off = 0;
  for (int l = 0; l < L; ++l) {
    const LayerHost &h = m->host[l];
    const LayerDev &d = m->dev[l];
    const bool last = l == L - 1, proj = h.projection();
    const lstm_int_trace *tr = (trace && trace->layer == l) ? trace : nullptr;
    int8_t *out = reinterpret_cast<int8_t *>(wsb + ws.out[l & 1]);
    const size_t step_out = (size_t)B * d.Hpad;

    // persistent path: eligible shape, no dump requested for this layer, batch fits one launch
    int p2_ks = 0, p2_rt = 0, p2_groups = 0;
    bool use_p2 = m->path != 1 && !tr && d.p2 && (reinterpret_cast<uintptr_t>(y) & 3) == 0 &&
                  rec_supported(h.N, h.H, (int)h.flags, B, &p2_ks, &p2_rt, &p2_groups);
    RecArgs ra;
    bool use16 = false;
    if (use_p2) {
      memset(&ra, 0, sizeof(ra));
      ra.T = T; ra.B = B; ra.N = h.N; ra.H = h.H; ra.Hpad = d.Hpad; ra.flags = (int)h.flags; ra.m_c = h.m_c;
      ra.GS = d.GS; ra.groups = p2_groups; ra.rows_pg = 32 * p2_rt; ra.ks = d.ks; ra.Ncp = d.Ncp;
      ra.Bp = round_up(B, 32);
      ra.R2 = d.R2; ra.bh4 = d.bh4; ra.Lq4 = d.Lq4; ra.qb4 = d.qb4; ra.Pq3 = d.Pq3;
      ra.pre_h = 0;
      for (int g = 0; g < 4; ++g) {
        const int sg = g < 4 - h.G ? 4 - h.G : g;  // an absent gate borrows valid numbers; its rows are zero
        ra.Mh[g] = h.Mh[sg]; ra.rh[g] = 31 - h.eh[sg];
        ra.pre_h = std::max(ra.pre_h, preshift_mode(ra.rh[g], d.amax_h[sg]));
        ra.Mln[g] = h.Mln[sg]; ra.rln[g] = 31 - h.eln[sg];
      }
      for (int j = 0; j < 3; ++j) { ra.Mc[j] = h.Mc[j]; ra.rc[j] = 31 - h.ec[j]; }
      ra.Mm = h.Mm; ra.rm = 31 - h.em; ra.zp_m = h.zp_m;
      // the 32-row kernel's tiling of W_proj (the 16-row kernel gets the 32-row tiles back below)
      ra.Wp2 = d.Wp3; ra.bp2 = d.bp3; ra.ptiles = d.ptiles3; ra.prow = d.prow; ra.npadp = d.npadp;
      ra.Mp = h.Mp; ra.rp = 31 - h.ep; ra.zp_h = h.zp_h;
      ra.tx2 = reinterpret_cast<const int4 *>(tx);
      ra.h0 = h0; ra.out = out; ra.y = (last && !rev) ? y : nullptr;
      ra.mbuf = reinterpret_cast<int8_t *>(wsb + ws.m2);
      ra.c_in = c_state ? c_state + c_off : nullptr;
      ra.c_out = c_state ? c_state + c_off : nullptr;
      ra.counters = reinterpret_cast<unsigned *>(wsb + ws.sync);
      // the words share the zeroed counter region: bytes 8..15 of the blocks of groups 0..7 (bytes 0..3
      // are the barrier counter)
      ra.tickets = m->cooperative ? nullptr : reinterpret_cast<unsigned long long *>(ra.counters + 2);
      ra.acc = reinterpret_cast<unsigned long long *>(wsb + ws.sync + 256 * 64 * 4);
      ra.status = m->status;
      ra.spin_limit = m->spin_limit;
      ra.poll_sleep = m->poll_sleep;
      ra.stats_sleep = m->stats_sleep;
      ra.idle_sleep = m->idle_sleep;
      ra.stats_first_sleep = m->stats_first_sleep;
      // the last arrival lands about 0.45 us after a workgroup's own in a group of 32, sooner in small groups
      ra.sync_sleep = m->sync_sleep >= 0 ? m->sync_sleep : (d.GS >= 16 ? 16 : 4);
      ra.idle_poll_sleep = m->idle_poll_sleep;
      ra.ticks = m->phase_timing ? reinterpret_cast<long long *>(m->status + 16) : nullptr;
      ra.extra_arrivals = m->extra_arrivals;
      // the kernel's one-product form of rescale needs shifts in [3, 62]; its tables must compress (lut_ok below)
      auto shift_ok = [](int r) { return r >= 3 && r <= 62; };
      bool ok = shift_ok(ra.rm) && (!proj || shift_ok(ra.rp));
      for (int g = 4 - h.G; g < 4; ++g)
        if (!shift_ok(ra.rh[g]) || (h.layer_norm() && !shift_ok(ra.rln[g]))) ok = false;
      for (int j = 4 - h.G; j < 3; ++j)
        if (h.peephole() && !shift_ok(ra.rc[j])) ok = false;
      // rec_kernel's tables: the shortest prefixes first (the budget test below uses them)
      auto set_lut = [&](int i, const WideTable &w) {
        int dom = 0, tail = 0;
        w.shortest(&dom, &tail);
        ra.lut[i].blob = w.blob; ra.lut[i].sh = w.sh; ra.lut[i].dom = dom; ra.lut[i].tail = tail;
        return dom > 0;
      };
      const bool lut_ok = set_lut(0, m->wsig3) & set_lut(1, m->wtanh3) & set_lut(2, d.wtanhc);
      if (ok && ra.rows_pg == 64 && lut_ok && rec_lds_bytes(ra) > 160 * 1024) {
        // two row tiles per group do not fit the LDS: one tile per group, more launches over the batch
        p2_rt = 1;
        ra.rows_pg = 32;
        p2_groups = std::min(8 * (32 / d.GS), (B + 31) / 32);
        ra.groups = p2_groups;
      }
      if (!ok || !lut_ok || rec_lds_bytes(ra) > 160 * 1024) use_p2 = false;
      // small batches: groups of 16 rows fill more compute units and halve a step's arithmetic
      int k16 = 0, g16 = 0;
      if (use_p2 && m->rows16 && d.p16 && rec16_supported(h.N, h.H, (int)h.flags, B, &k16, &g16)) {
        RecArgs r16 = ra;
        r16.R2h = d.R2h; r16.ks16 = d.ks16; r16.rows_pg = 16; r16.groups = g16;
        r16.Wp2 = d.Wp2; r16.bp2 = d.bp2; r16.ptiles = d.ptiles; r16.prow = 32;
        if (rec16_lds_bytes(r16) <= 160 * 1024) {
          ra = r16;
          p2_groups = g16;
          use16 = true;
        }
      }
      // 2:4 recurrent weights: the 32-row kernel with one row tile per group has a sparse-MFMA form
      if (use_p2 && !use16 && m->sparse && d.R2s && ra.rows_pg == 32) {
        ra.R2 = d.R2s;
        ra.sparse = 1;
      }
    }
    // option "sparse" = 2: a layer with 2:4 recurrent weights must run in the sparse form, or the call fails
    if (m->sparse == 2 && d.R2s && !(use_p2 && ra.sparse)) return LSTM_INT_E_UNSUPPORTED;
    if (use_p2) {
      auto lds_need = [&]() { return use16 ? rec16_lds_bytes(ra) : rec_lds_bytes(ra); };
      // What LDS is left goes to longer prefixes of the two gate tables, 1 KB at a time in turn: a value
      // beyond the prefix costs the whole group a detour (rec_kernel.inc.h, lookup), and with 24576 entries
      // (|x| < 6 in Q3.12) there is about one per million layer-norm outputs instead of one per thousand.
      // A prefix that reaches the table's flat end needs no tail part any more.
      bool grew = true;
      while (grew) {
        grew = false;
        for (int i = 0; i < 2; ++i) {
          const WideTable &w = i == 0 ? m->wsig3 : m->wtanh3;
          LutWide keep = ra.lut[i];
          if (keep.dom >= 32768 || (!keep.tail && keep.dom - 1 >= w.flat_from)) continue;  // nothing left to gain
          ra.lut[i].dom = keep.dom + 1024;
          ra.lut[i].tail = (ra.lut[i].dom - 1 < w.flat_from) ? 1 : 0;
          if (ra.lut[i].tail && !w.has_tail) { ra.lut[i] = keep; continue; }
          if (i == 1 && ra.lut[2].blob == keep.blob) ra.lut[2] = ra.lut[1];  // one copy serves the cell tanh too
          if (lds_need() > 160 * 1024) {
            ra.lut[i] = keep;
            if (i == 1 && ra.lut[2].blob == keep.blob) ra.lut[2] = keep;
          } else {
            grew = true;
          }
        }
      }
    }
    if (use_p2) {
      // bytes of the synchronization region a launch over `groups` groups uses: all counters, and the
      // statistics words of its groups (they follow the counters)
      auto sync_bytes = [](int groups) { return (int64_t)256 * 64 * 4 + (int64_t)groups * (int64_t)kStatGroupBytes; };
      const int launch_rows = p2_groups * ra.rows_pg;
      {
        InGemmArgs ga;
        memset(&ga, 0, sizeof(ga));
        ga.A = in; ga.lda = ld_in; ga.T = T; ga.B = B; ga.Bp = ra.Bp;
        ga.a_slack = in != x;  // the workspace buffers have the slack, the caller's x need not
        ga.W2 = d.W2; ga.W2f = d.W2f; ga.kpad = d.Ipad; ga.tiles = d.GS * 8; ga.bx2 = d.bx2;
        ga.all_hi = 1;
        ga.pre = 0;
        for (int g = 0; g < 4; ++g) {
          const int sg = g < 4 - h.G ? 4 - h.G : g;
          ga.M[g] = h.Mx[sg]; ga.r[g] = 31 - h.ex[sg];
          if (ga.r[g] < 32) ga.all_hi = 0;
          ga.pre = std::max(ga.pre, preshift_mode(ga.r[g], d.amax_x[sg]));
        }
        ga.tx2 = reinterpret_cast<int4 *>(tx);
        // initial h (given, or real 0 = zp_h), the cleared words of the first launch and the previous layer's
        // final h on its way to the state buffer: done by the input GEMM's workgroups ahead of their own
        // work, or by a kernel of their own where the general input GEMM runs
        const int g0 = std::min(p2_groups, (B + ra.rows_pg - 1) / ra.rows_pg);
        const bool ws_gemm = in_gemm_ws_supported(ga);
        if (ws_gemm) {
          ga.has_init = 1;
          ga.init.h_src = h_state ? h_state + h_off : nullptr; ga.init.ld_src = h.H;
          ga.init.h0 = h0; ga.init.ld_h0 = d.Hpad; ga.init.rows = B; ga.init.cols = h.H; ga.init.zp = h.zp_h;
          ga.init.sync = reinterpret_cast<int4 *>(wsb + ws.sync); ga.init.sync_vec = sync_bytes(g0) / 16;
          ga.init.c_src = pend.src; ga.init.c_ld_src = pend.ld; ga.init.c_dst = pend.dst; ga.init.c_cols = pend.cols;
        } else {
          Timed t(m->prof, s, LSTM_INT_K_OTHER);
          launch_init_layer(s, h_state ? h_state + h_off : nullptr, h.H, h0, d.Hpad, B, h.H, h.zp_h, wsb + ws.sync,
                            sync_bytes(g0), pend.src, pend.ld, pend.dst, pend.cols);
        }
        pend.dst = nullptr;
        Timed t(m->prof, s, LSTM_INT_K_INPUT_GEMM);
        if (ws_gemm)
          launch_in_gemm_ws(s, ga, m->num_cus);
        else
          launch_in_gemm(s, ga);
      }
      // One launch takes at most 2^14 steps (the statistics words of the kernel count up over the
      // launch); longer sequences run in pieces, h carried through the layer output and c through a
      // buffer.  Batch rows beyond one launch's groups run in further launches (rows never interact).
      constexpr int kMaxSteps = 1 << 14;
      const int4 *tx2_all = ra.tx2;
      int16_t *c_carry = c_state ? c_state + c_off : c;
      for (int t0 = 0; t0 < T; t0 += kMaxSteps) {
        const int tc = std::min(kMaxSteps, T - t0);
        ra.T = tc;
        ra.tx2 = tx2_all + (size_t)t0 * (ra.Bp / 32) * (d.GS * 8) * 2 * 64;
        ra.h0 = t0 == 0 ? h0 : out + (size_t)(t0 - 1) * step_out;
        ra.out = out + (size_t)t0 * step_out;
        ra.y = (last && !rev) ? y + (size_t)t0 * B * h.H : nullptr;
        ra.c_in = t0 == 0 ? (c_state ? c_state + c_off : nullptr) : c_carry;
        ra.c_out = (c_state || t0 + tc < T) ? c_carry : nullptr;
        for (int b0 = 0; b0 < B; b0 += launch_rows) {
          ra.batch0 = b0;
          ra.groups = std::min(p2_groups, (B - b0 + ra.rows_pg - 1) / ra.rows_pg);
          if (b0 > 0 || t0 > 0) {
            Timed t(m->prof, s, LSTM_INT_K_OTHER);
            launch_fill_i16(s, reinterpret_cast<int16_t *>(wsb + ws.sync), sync_bytes(ra.groups) / 2, 0);
          }
          if (!rec_extents_ok(ra, ws, T, t0, proj)) return LSTM_INT_E_WORKSPACE;
          Timed t(m->prof, s, LSTM_INT_K_RECURRENT);
          const bool coop = m->cooperative != 0;
          if ((use16 ? launch_rec16(s, ra, coop) : launch_rec(s, ra, coop)) != hipSuccess) return LSTM_INT_E_DEVICE;
        }
      }
      {
        Timed t(m->prof, s, LSTM_INT_K_OTHER);
        if (h_state) {
          pend.src = out + (size_t)(T - 1) * step_out;
          pend.ld = d.Hpad;
          pend.dst = h_state + h_off;
          pend.cols = h.H;
        }
        if (last && rev) launch_flip_rows_i8(s, out, d.Hpad, y, h.H, T, B, h.H, 0);
      }
      h_off += (size_t)B * h.H;
      c_off += (size_t)B * h.N;
      in = out;
      ld_in = d.Hpad;
      continue;
    }
    {  // initial state: given, or real 0 (q = zp_h) and c = 0
      Timed t(m->prof, s, LSTM_INT_K_OTHER);
      flush_pending();
      if (h_state)
        launch_copy_rows_i8(s, h_state + h_off, h.H, h0, d.Hpad, B, h.H, 0);
      else
        launch_fill_rows_i8(s, h0, d.Hpad, B, h.H, h.zp_h, 0);
      if (c_state)
        launch_copy_i16(s, c_state + c_off, c, (int64_t)B * h.N);
      else
        launch_fill_i16(s, c, (int64_t)B * h.N, 0);
    }
    {  // W x for every (t, b) at once: it does not depend on t-1 (eqs. 1-5)
      Timed t(m->prof, s, LSTM_INT_K_INPUT_GEMM);
      launch_gemm_i16(s, in, ld_in, TB, d.W, d.Ipad, d.GN, d.bx, d.rq_x, tx, d.GN);
    }
    if (tr && tr->tx) {
      if (rev)  // step k -> time T - 1 - k
        for (int k = 0; k < T; ++k)
          launch_scatter_gates(s, tx + (size_t)k * B * d.GN, tr->tx + (size_t)(T - 1 - k) * B * 4 * h.N, B, h.G, h.N);
      else
        launch_scatter_gates(s, tx, tr->tx, TB, h.G, h.N);
    }

    for (int t = 0; t < T; ++t) {
      const int8_t *hprev = t == 0 ? h0 : out + (size_t)(t - 1) * step_out;
      int8_t *hout = out + (size_t)t * step_out;
      {
        Timed tm(m->prof, s, LSTM_INT_K_RECURRENT);
        launch_gemm_i16(s, hprev, d.Hpad, B, d.R, d.Hpad, d.GN, d.bh, d.rq_h, th, d.GN);
      }
      const int tpos = rev ? T - 1 - t : t;  // position in time of step t, for the traces
      const size_t tg = (size_t)tpos * B * 4 * h.N, tn = (size_t)tpos * B * h.N;
      if (tr && tr->th) launch_scatter_gates(s, th, tr->th + tg, B, h.G, h.N);
      CellArgs a;
      a.B = B; a.N = h.N; a.G = h.G; a.flags = (int32_t)h.flags; a.m_c = h.m_c;
      a.inv_n = 1.0 / (double)h.N;
      a.tx = tx + (size_t)t * B * d.GN;
      a.th = th;
      a.c = c;
      a.Pq = d.Pq; a.Lq = d.Lq; a.qb = d.qb;
      for (int j = 0; j < 3; ++j) { a.Mc[j] = h.Mc[j]; a.rc[j] = 31 - h.ec[j]; }
      for (int g = 0; g < 4; ++g) { a.Mln[g] = h.Mln[g]; a.rln[g] = 31 - h.eln[g]; }
      a.Mm = h.Mm; a.rm = 31 - h.em; a.zp_m = h.zp_m;
      a.sig_tab = m->sig3; a.tanh_tab = m->tanh3; a.tanhc_tab = d.tanhc;
      a.m_out = proj ? mbuf : hout;
      a.ld_m = proj ? d.Npad : d.Hpad;
      a.m_out2 = (!proj && last && !rev) ? y + (size_t)t * B * h.H : nullptr;
      a.ld_m2 = h.H;
      a.tr_g = tr && tr->g ? tr->g + tg : nullptr;
      a.tr_ln = tr && tr->ln ? tr->ln + tg : nullptr;
      a.tr_act = tr && tr->act ? tr->act + tg : nullptr;
      a.tr_c = tr && tr->c ? tr->c + tn : nullptr;
      a.tr_m = tr && tr->m ? tr->m + tn : nullptr;
      {
        Timed tm(m->prof, s, LSTM_INT_K_CELL);
        launch_cell(s, a);
      }
      if (proj) {
        Timed tm(m->prof, s, LSTM_INT_K_PROJECTION);
        launch_gemm_i8(s, mbuf, d.Npad, B, d.Wproj, d.Npad, h.H, d.bp, d.rq_p, hout, d.Hpad,
                       (last && !rev) ? y + (size_t)t * B * h.H : nullptr, h.H);
      }
    }
    {
      Timed t(m->prof, s, LSTM_INT_K_OTHER);
      if (tr && tr->h) {
        if (rev)
          launch_flip_rows_i8(s, out, d.Hpad, tr->h, h.H, T, B, h.H, 0);
        else
          launch_copy_rows_i8(s, out, d.Hpad, tr->h, h.H, TB, h.H, 0);
      }
      if (last && rev) launch_flip_rows_i8(s, out, d.Hpad, y, h.H, T, B, h.H, 0);
      if (h_state)
        launch_copy_rows_i8(s, out + (size_t)(T - 1) * step_out, d.Hpad, h_state + h_off, h.H, B,
                            h.H, 0);
      if (c_state) launch_copy_i16(s, c, c_state + c_off, (int64_t)B * h.N);
    }
    h_off += (size_t)B * h.H;
    c_off += (size_t)B * h.N;
    in = out;
    ld_in = d.Hpad;
  }
  flush_pending();
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

int lstm_int_forward_static(const lstm_int_model *m, const int8_t *x, int32_t T, int32_t B, int8_t *y,
                            int8_t *h_state, int16_t *c_state, void *hip_stream) {
  if (!m || T < 0 || B < 0) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0 || m->device >= kMaxDevices) return LSTM_INT_E_DEVICE;
  if (m->prof.on) return LSTM_INT_E_INVALID_ARG;  // per-kernel timing creates events
  if (T == 0 || B == 0) return LSTM_INT_OK;
  if ((int64_t)T * B > (int64_t)1 << 30) return LSTM_INT_E_UNSUPPORTED;
  if (plan_workspace(m, T, B).total > (size_t)LSTM_INT_STATIC_WORKSPACE_BYTES) return LSTM_INT_E_WORKSPACE;
  void *ws = g_scratch_ptr[m->device];  // set when the model was prepared on this device
  if (!ws) return LSTM_INT_E_DEVICE;
  return lstm_int_forward(m, x, T, B, y, h_state, c_state, ws, LSTM_INT_STATIC_WORKSPACE_BYTES, hip_stream, nullptr);
}

// Workspace of a bidirectional call: the larger of the two directions' own workspaces, then one dense
// [T, B, max(H_fwd, H_bwd)] staging buffer from which each direction's output is placed into its columns of y.
static size_t bidi_stage_offset(const lstm_int_model *f, const lstm_int_model *b, int32_t T, int32_t B) {
  const size_t wf = lstm_int_workspace_bytes(f, T, B), wb = lstm_int_workspace_bytes(b, T, B);
  return ((wf > wb ? wf : wb) + 255) & ~(size_t)255;
}

size_t lstm_int_bidirectional_workspace_bytes(const lstm_int_model *f, const lstm_int_model *b, int32_t T, int32_t B) {
  if (!f || !b || T < 0 || B < 0 || f->host.empty() || b->host.empty()) return 0;
  const int Hm = std::max(f->host.back().H, b->host.back().H);
  return bidi_stage_offset(f, b, T, B) + (((size_t)T * B * Hm + 255) & ~(size_t)255);
}

int lstm_int_forward_bidirectional(const lstm_int_model *f, const lstm_int_model *b, const int8_t *x, int32_t T,
                                   int32_t B, int8_t *y, int8_t *h_state_fwd, int16_t *c_state_fwd,
                                   int8_t *h_state_bwd, int16_t *c_state_bwd, void *workspace, size_t workspace_bytes,
                                   void *hip_stream) {
  if (!f || !b || T < 0 || B < 0 || f->host.empty() || b->host.empty()) return LSTM_INT_E_INVALID_ARG;
  // the two stacks read the same features: same width, same input quantization
  if (f->host[0].I != b->host[0].I || f->host[0].s_x != b->host[0].s_x || f->host[0].zp_x != b->host[0].zp_x)
    return LSTM_INT_E_INVALID_ARG;
  if (f->reverse != 0 || b->reverse != 1) return LSTM_INT_E_INVALID_ARG;
  if (f->device < 0 || f->device != b->device) return LSTM_INT_E_DEVICE;
  if (T == 0 || B == 0) return LSTM_INT_OK;
  if (!x || !y) return LSTM_INT_E_INVALID_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) ||
      workspace_bytes < lstm_int_bidirectional_workspace_bytes(f, b, T, B))
    return LSTM_INT_E_WORKSPACE;
  const int Hf = f->host.back().H, Hb = b->host.back().H;
  const size_t so = bidi_stage_offset(f, b, T, B);
  int8_t *stage = reinterpret_cast<int8_t *>(workspace) + so;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  int rc = lstm_int_forward(f, x, T, B, stage, h_state_fwd, c_state_fwd, workspace, so, hip_stream, nullptr);
  if (rc != LSTM_INT_OK) return rc;
  launch_place_cols_i8(s, stage, y, Hf + Hb, (int64_t)T * B, Hf);
  rc = lstm_int_forward(b, x, T, B, stage, h_state_bwd, c_state_bwd, workspace, so, hip_stream, nullptr);
  if (rc != LSTM_INT_OK) return rc;
  launch_place_cols_i8(s, stage, y + Hf, Hf + Hb, (int64_t)T * B, Hb);
  return hipGetLastError() == hipSuccess ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
}

int lstm_int_set_option(lstm_int_model *m, const char *key, int64_t value) {
  if (!m || !key) return LSTM_INT_E_INVALID_ARG;
  if (!strcmp(key, "path")) {
    if (value < 0 || value > 2) return LSTM_INT_E_INVALID_ARG;
    m->path = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "cooperative_launch")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->cooperative = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "sparse")) {
    if (value < 0 || value > 2) return LSTM_INT_E_INVALID_ARG;
    m->sparse = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "rows16")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->rows16 = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "stack")) {
    if (value < 0 || value > 2) return LSTM_INT_E_INVALID_ARG;
    m->stack = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "stack_prefetch_kb")) {
    if (value < 0 || value > (1 << 20)) return LSTM_INT_E_INVALID_ARG;
    m->stack_prefetch_kb = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "flag_sleep")) {
    if (value < 0 || value > 1024) return LSTM_INT_E_INVALID_ARG;
    m->flag_sleep = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "stack_step_ns")) {  // expected time of one item of the stacked launch, for the choice between the two ways
    if (value < 1 || value > 1000000) return LSTM_INT_E_INVALID_ARG;
    m->stack_step_us = (double)value * 1e-3;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "reverse")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->reverse = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "reset_status")) {  // after a wait gave up: the word is sticky and stops every later kernel
    if (m->device >= 0) {
      if (hipSetDevice(m->device) != hipSuccess || hipDeviceSynchronize() != hipSuccess ||
          hipMemset(m->status, 0, sizeof(int)) != hipSuccess)
        return LSTM_INT_E_DEVICE;
    }
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "phase_timing")) {
    m->phase_timing = (int)std::min<int64_t>(std::max<int64_t>(value, 0), 64);  // stacked launch: 1 + the layer timed (at most the top one)
    if (m->device >= 0 && hipMemset(m->status + 16, 0, 16 * sizeof(long long)) != hipSuccess)
      return LSTM_INT_E_DEVICE;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "poll_sleep") || !strcmp(key, "stats_sleep") || !strcmp(key, "idle_sleep") ||
      !strcmp(key, "idle_poll_sleep") || !strcmp(key, "sync_sleep") || !strcmp(key, "stats_first_sleep")) {
    if (value < (strcmp(key, "sync_sleep") ? 0 : -1) || value > 1024) return LSTM_INT_E_INVALID_ARG;
    int &dst = !strcmp(key, "poll_sleep") ? m->poll_sleep : !strcmp(key, "stats_sleep") ? m->stats_sleep
               : !strcmp(key, "idle_sleep") ? m->idle_sleep
               : !strcmp(key, "sync_sleep") ? m->sync_sleep
               : !strcmp(key, "stats_first_sleep") ? m->stats_first_sleep : m->idle_poll_sleep;
    dst = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "barrier_never_completes")) {
    if (value < 0 || value > 1) return LSTM_INT_E_INVALID_ARG;
    m->extra_arrivals = (int)value;
    return LSTM_INT_OK;
  }
  if (!strcmp(key, "spin_limit")) {
    if (value < 1 || value > (1 << 30)) return LSTM_INT_E_INVALID_ARG;
    m->spin_limit = (int)value;
    return LSTM_INT_OK;
  }
  return LSTM_INT_E_INVALID_ARG;
}

int lstm_int_sparse_layers(const lstm_int_model *m, int32_t *count) {
  if (!m || !count) return LSTM_INT_E_INVALID_ARG;
  int32_t n = 0;
  for (const LayerDev &d : m->dev) n += d.R2s != nullptr;
  *count = n;
  return LSTM_INT_OK;
}

int lstm_int_device_status(const lstm_int_model *m, int32_t *status) {
  if (!m || !status) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  int v = 0;
  if (hipMemcpy(&v, m->status, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return LSTM_INT_E_DEVICE;
  *status = v;
  return LSTM_INT_OK;
}

int lstm_int_phase_ticks(const lstm_int_model *m, int64_t ticks[16]) {
  if (!m || !ticks) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  if (hipMemcpy(ticks, m->status + 16, 16 * sizeof(long long), hipMemcpyDeviceToHost) != hipSuccess)
    return LSTM_INT_E_DEVICE;
  return LSTM_INT_OK;
}

int lstm_int_profile_begin(lstm_int_model *m) {
  if (!m) return LSTM_INT_E_INVALID_ARG;
  if (m->device < 0) return LSTM_INT_E_DEVICE;
  if (hipSetDevice(m->device) != hipSuccess) return LSTM_INT_E_DEVICE;
  Profile &p = m->prof;
  p.release();
  p.failed = false;
  p.on = true;
  return LSTM_INT_OK;
}

int lstm_int_profile_end(lstm_int_model *m, int64_t launches[LSTM_INT_K_COUNT],
                         double total_ms[LSTM_INT_K_COUNT]) {
  if (!m || !launches || !total_ms) return LSTM_INT_E_INVALID_ARG;
  Profile &p = m->prof;
  if (!p.on) return LSTM_INT_E_INVALID_ARG;
  p.on = false;
  for (int k = 0; k < LSTM_INT_K_COUNT; ++k) {
    launches[k] = 0;
    total_ms[k] = 0.0;
  }
  int rc = hipStreamSynchronize(p.stream) == hipSuccess && !p.failed ? LSTM_INT_OK : LSTM_INT_E_DEVICE;
  for (size_t i = 0; i < p.used && rc == LSTM_INT_OK; ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]) != hipSuccess) {
      rc = LSTM_INT_E_DEVICE;
      break;
    }
    launches[p.cls[i]] += 1;
    total_ms[p.cls[i]] += ms;
  }
  p.release();  // no event outlives the measurement
  return rc;
}

void lstm_int_destroy(lstm_int_model *m) {
  if (!m) return;
  if (m->device >= 0) {
    (void)hipSetDevice(m->device);
    m->prof.release();
    if (m->arena) (void)hipFree(m->arena);
  }
  delete m;
}

const char *lstm_int_strerror(int code) {
  switch (code) {
    case LSTM_INT_OK: return "ok";
    case LSTM_INT_E_INVALID_ARG: return "invalid argument";
    case LSTM_INT_E_UNSUPPORTED: return "outside the supported limits";
    case LSTM_INT_E_BAD_RANGE: return "bad range or non-finite parameter";
    case LSTM_INT_E_OUT_OF_MEMORY: return "out of memory";
    case LSTM_INT_E_DEVICE: return "HIP device error or host-only model";
    case LSTM_INT_E_WORKSPACE: return "workspace too small or misaligned";
    default: return "unknown error";
  }
}

}  // extern "C"
