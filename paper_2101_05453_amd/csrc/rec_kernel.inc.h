// Device code of the persistent recurrent kernel (see persistent.hip for the
// design).  Included by the rec_inst_*.hip translation units, which
// instantiate it for their k depth.
#pragma once

#include <type_traits>

#include "lstm_int_math.h"
#include "persistent.h"

namespace lstm_int {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned long long u64;

// ---------------------------------------------------------------------------
// Recurrent kernel
// ---------------------------------------------------------------------------

// Barrier among the GS workgroups of a group.  Every wave first waits for its
// own stores (vmcnt(0)); thread 0 then adds one to the group's counter and
// polls it, pausing poll_sleep x 64 clocks between polls: the polls of all the
// group's workgroups go to one L2 channel, the one that also serves the
// arrivals, and polling at full rate delays those (measured: every poller
// added made the barrier slower).  Gives up after spin_limit polls (or when
// another workgroup gave up), raising the status word so that every workgroup
// leaves the kernel; lds_flag[0] is then 0 for good.
// PENDING: vector memory loads the caller issued after its last store and does
// not need yet (the counter of outstanding operations drains in issue order, so
// waiting until PENDING are left means every store before them is complete).
template <int PENDING = 0>
__device__ __forceinline__ bool group_sync(unsigned *counter, unsigned &epoch, int GS, int *status,
                                           int spin_limit, int first_sleep, int poll_sleep, int *lds_flag) {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
  __syncthreads();
  if (GS == 1) return true;
  epoch += (unsigned)GS;
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // a workgroup that knows the others have work left before they arrive keeps off the counter meanwhile
    for (int i = 0; i < first_sleep; ++i) __builtin_amdgcn_s_sleep(1);
    int budget = spin_limit;
    for (;;) {
      const unsigned c = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((int)(c - epoch) >= 0) break;
      // the status word (another workgroup gave up) is looked at every 16th poll: each look is one more request
      // in the polling thread's queue (measured: 0.3 % of the step)
      --budget;
      if ((budget & 15) == 0 &&
          (budget <= 0 || __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lds_flag[0] = 0;
        break;
      }
      for (int i = 0; i < poll_sleep; ++i) __builtin_amdgcn_s_sleep(1);
    }
  }
  __syncthreads();
  return lds_flag[0] != 0;
}

// Per-layer constants, kept in LDS and read where they are used: as kernel
// arguments they would all be live in scalar registers across the time loop.
struct PrmLds {  // 256 bytes (kPrmLdsBytes in persistent.hip)
  RescaleHi h[4], c[4], ln[4];  // R h terms, peephole terms, layer-norm second stage
  RescaleHi m, p;               // hidden state, projection
  int32_t zp_m, zp_h, m_c, glo;
  int32_t pad[4];
};

static_assert(sizeof(PrmLds) == 256, "rec_lds_bytes assumes 256 bytes");

// Where rec_kernel keeps a table in LDS (byte offsets from the start of the dynamic LDS), for the same
// reason in LDS itself: offD = deltas, offB = bases, offT = tail part (0 = none kept).
struct LutLds {
  int32_t dom, sh, offD, offB, offT, pad[3];
};
static_assert(sizeof(LutLds) == 32, "rec_lds_bytes assumes 3 x 32 bytes");

__device__ __forceinline__ int32_t abs_i32(int32_t v) { return v < 0 ? -v : v; }
// table value t = tab[|x|] -> sigma(x), tanh(x) (Sec. 3.2.1 output clamp)
__device__ __forceinline__ int32_t mirror_sigmoid(int32_t x, int32_t t) {
  return x < 0 ? 32768 - t : (t > 32767 ? 32767 : t);
}
__device__ __forceinline__ int32_t mirror_tanh(int32_t x, int32_t t) {
  return x < 0 ? -t : (t > 32767 ? 32767 : t);
}

// FL: bit 0 CIFG, bit 1 peephole, bit 2 layer norm, bit 3 "no projection" (compile
// time, so that the code carries no tests of them); with bit 3 clear the
// projection is a runtime flag.  SP: the recurrent weights are in the 2:4
// compressed form (persistent.h) and R h runs on the sparse MFMA.
template <int KS, int RT, int FL, bool SP = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void rec_kernel(RecArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const long long t_start = (long long)wall_clock64();
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, b2 = lane >> 5;
  constexpr bool cifg = FL & 1, ph = FL & 2, ln = FL & 4;
  // bit 3: the layer is known to have no projection (measured: dropping the projection code from
  // those kernels gains 1.7 % at C5, while fixing the flag to "on" at compile time loses 5 % at C4)
  const bool proj = !(FL & 8) && (a.flags & 8);
  const int GS = a.GS;

  // Placement: the workgroups of a group share one XCD (one L2).  XCC_ID register (id 20), bits 3:0,
  // is the XCD this workgroup runs on.
  const int wg = blockIdx.x;
  const int xcc = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7);
  const int slot = wg >> 3;
  int xcd = wg & 7;
  if (a.tickets) {
    // Plain launch: the dispatcher deals workgroups out to the XCDs in turn, but starts wherever the
    // kernel before stopped: workgroup w runs on XCD (w + r) % 8 with an r nobody knows beforehand.
    // Each block of 8 consecutive workgroups still covers every XCD once, so (the XCD read from the
    // hardware, w / 8) names a place exactly once -- if the dealing was strict, which every
    // workgroup helps to check when it is done (end of the kernel).
    xcd = xcc;
  } else if (xcc != xcd && GS > 1 && tid == 0) {
    // cooperative launch: workgroup w runs on XCD w % 8
    __hip_atomic_store(a.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // Placement check of a plain launch, made by every workgroup when it is done (not at the start, so
  // that nothing waits for it): one 64-bit word per XCD, low half a sum of 2^(w / 8), high half a count
  // of workgroups.  The workgroup that completes its XCD's count finds every place taken once (the sum
  // is then all ones), or raises the status word; so does one that finds the count exceeded -- and an
  // XCD that got too few leaves another with too many.  (The register is read again: kept from the
  // start it would occupy a register across the time loop.)
  auto placement_check = [&]() {
    if (a.tickets && tid == 0) {
      const int xcc_now = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7);
      const unsigned places = gridDim.x >> 3;  // at most 32
      const u64 mine = ((u64)1 << 32) + ((u64)1 << (wg >> 3));
      const u64 now =
          __hip_atomic_fetch_add(&a.tickets[xcc_now * 32], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
      const unsigned count = (unsigned)(now >> 32);
      const unsigned all = places >= 32 ? 0xFFFFFFFFu : (1u << places) - 1;
      if (count > places || (count == places && (unsigned)now != all))
        __hip_atomic_store(a.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  const int group = xcd + 8 * (slot / GS), member = slot % GS;
  if (group >= a.groups) {  // no rows for this workgroup
    placement_check();
    return;
  }
  constexpr int rows_pg = 32 * RT;
  constexpr int items = RT * 128;  // (rt, gate, row) layer-norm rows of the group
  const int row0 = a.batch0 + group * rows_pg;  // first batch row of the group

  // ---- LDS carve-up (rec_lds_bytes mirrors it)
  constexpr int LS = KS * 32 + 16;  // h tile row stride
  uint8_t *p = lds;
  int8_t *hT = reinterpret_cast<int8_t *>(p);
  int32_t *pred = reinterpret_cast<int32_t *>(p);  // projection partials reuse the h tile between steps
  {
    // whole 1 KB chunks, plus one that takes the loads past the tile (every wave issues the same number)
    const size_t tile_bytes = (((size_t)rows_pg * LS + 1023) / 1024 + 1) * 1024;
    const size_t pred_bytes = proj ? 4 * 16 * 64 * 4 : 0;
    p += tile_bytes > pred_bytes ? tile_bytes : pred_bytes;
  }
  u64 *red = reinterpret_cast<u64 *>(p);                 p += (size_t)items * 8;
  LnRow2 *lnrow = reinterpret_cast<LnRow2 *>(p);         p += (size_t)items * sizeof(LnRow2);
  double *LdL = reinterpret_cast<double *>(p);           p += 4 * 64 * 8;  // layer-norm weights / 2^10 as doubles
  double *bdL = reinterpret_cast<double *>(p);           p += 4 * 64 * 8;  // layer-norm biases / 2^10 + 2^-11 as doubles
  int16_t *PqL = reinterpret_cast<int16_t *>(p);         p += 4 * 64 * 2;  // 3 used
  int32_t *bhL = reinterpret_cast<int32_t *>(p);         p += 4 * 64 * 4;
  PrmLds *prm = reinterpret_cast<PrmLds *>(p);           p += sizeof(PrmLds);
  int *flag = reinterpret_cast<int *>(p);                p += 16;
  u64 *tickL = reinterpret_cast<u64 *>(p);               p += 16 * 8;  // phase timers
  LutLds *lutP = reinterpret_cast<LutLds *>(p);          p += 3 * sizeof(LutLds);
  // compressed sigma / tanh tables (wide form, lstm_int_math.h): deltas of the first dom entries, their
  // bases, and the tail part where one is kept; the cell-format tanh shares the gate one if equal
  const bool share_tanh = a.lut[2].blob == a.lut[1].blob;
  const uint8_t *lutD[3];   // deltas
  const uint16_t *lutB[3];  // bases
  const uint8_t *lutTl[3];  // tail part, or NULL
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    if (i == 2 && share_tanh) {
      lutD[2] = lutD[1]; lutB[2] = lutB[1]; lutTl[2] = lutTl[1];
    } else {
      const int nb = ((((a.lut[i].dom >> a.lut[i].sh) * 2) + 1023) >> 10) << 10;
      lutD[i] = p;                                        p += a.lut[i].dom;
      lutB[i] = reinterpret_cast<const uint16_t *>(p);    p += nb;
      lutTl[i] = a.lut[i].tail ? p : nullptr;             p += a.lut[i].tail ? 3072 : 0;
    }
  }
  int8_t *WpL = reinterpret_cast<int8_t *>(p);
  const int WLS = a.npadp + 16;  // W_proj tile row stride in LDS
  const int my_ptiles = proj ? (a.ptiles > member ? (a.ptiles - member + GS - 1) / GS : 0) : 0;

  // ---- one-time loads: R slice and its biases -> registers, other per-cell
  // parameters, the tables and the W_proj tiles -> LDS
  constexpr int KW = SP ? KS / 2 : KS;  // weight operands per tile: 64-deep k steps in the sparse form
  static_assert(!SP || KS % 2 == 0, "the sparse form takes k in steps of 64");
  v4i Wf[2][KW];
  int Wi[2][SP ? KW : 1];  // sparse form: the index word of each operand
  {
    const int4 *src = a.R2 + ((size_t)(member * 4 + wave) * 2) * KW * 64 + lane;
    const int *isrc = reinterpret_cast<const int *>(a.R2 + (size_t)GS * 4 * 2 * KW * 64) +
                      ((size_t)(member * 4 + wave) * 2) * KW * 64 + lane;
    // all loads of a tile are in flight together before the first is moved to its place
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
      int4 w[KW];
      int wi[KW];
#pragma unroll
      for (int ks = 0; ks < KW; ++ks) {
        w[ks] = src[(size_t)(tl * KW + ks) * 64];
        if (SP) wi[ks] = isrc[(size_t)(tl * KW + ks) * 64];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KW; ++ks) {
        Wf[tl][ks] = v4i{w[ks].x, w[ks].y, w[ks].z, w[ks].w};
        asm volatile("" : "+a"(Wf[tl][ks]));  // resident in accumulation registers for the whole launch
        if (SP) {
          Wi[tl][ks] = wi[ks];
          asm volatile("" : "+v"(Wi[tl][ks]));  // the index operand is read from an ordinary vector register
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const int cell_w = wave * 16 + 4 * b2;  // + tile * 8 + c, within the workgroup's 64 cells
  {
    const int g = tid >> 6, n = tid & 63;  // 256 threads = 4 gates x 64 cells
    const size_t idx = (size_t)g * a.Ncp + member * 64 + n;
    LdL[tid] = ln ? ln_weight_scaled(a.Lq4[idx]) : 0.0;
    bdL[tid] = ln ? ln_bias_scaled(a.qb4[idx]) : 0.0;
    PqL[tid] = (ph && g < 3) ? a.Pq3[idx] : 0;
    bhL[tid] = a.bh4[idx];  // folded recurrent bias, the accumulators' initial value each step
  }
  if (tid < 4) {
    prm->h[tid] = rescale_hi_prepare(a.Mh[tid], a.rh[tid]);
    prm->c[tid] = rescale_hi_prepare(tid < 3 && ph ? a.Mc[tid] : 0, tid < 3 && ph ? a.rc[tid] : 33);
    prm->ln[tid] = rescale_hi_prepare(a.Mln[tid], ln ? a.rln[tid] : 33);
  }
  if (tid < 3) {
    LutLds d;
    d.dom = a.lut[tid].dom; d.sh = a.lut[tid].sh;
    d.offD = (int32_t)(lutD[tid] - lds);
    d.offB = (int32_t)(reinterpret_cast<const uint8_t *>(lutB[tid]) - lds);
    d.offT = lutTl[tid] ? (int32_t)(lutTl[tid] - lds) : 0;
    d.pad[0] = d.pad[1] = d.pad[2] = 0;
    lutP[tid] = d;
  }
  if (tid == 0) {
    prm->m = rescale_hi_prepare(a.Mm, a.rm);
    prm->p = rescale_hi_prepare(proj ? a.Mp : 0, proj ? a.rp : 33);
    prm->zp_m = a.zp_m; prm->zp_h = a.zp_h;
    prm->m_c = a.m_c; prm->glo = ln ? -32767 : -32768;
  }
  for (int i = tid; i < rows_pg * LS / 16; i += 256) reinterpret_cast<int4 *>(hT)[i] = int4{0, 0, 0, 0};
  // tables and W_proj tiles: global -> LDS loads, all in flight together
  {
    auto dma = [&](const void *src, const void *dst) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                       (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };
    // per table: dom / 1024 chunks of deltas, then the chunks of bases, then the 3 chunks of the tail part,
    // which sit in this order in LDS and at fixed offsets in the wide blob
    for (int i = 0; i < (share_tanh ? 2 : 3); ++i) {
      const int nd = a.lut[i].dom >> 10;
      const int nb = (((a.lut[i].dom >> a.lut[i].sh) * 2) + 1023) >> 10;
      const int nt = a.lut[i].tail ? 3 : 0;
      for (int c = wave; c < nd + nb + nt; c += 4) {
        const int so = c < nd ? c * 1024 : (c < nd + nb ? kLutWideBaseOff + (c - nd) * 1024 : kLutWideTailOff + (c - nd - nb) * 1024);
        dma(a.lut[i].blob + so + lane * 16, lutD[i] + c * 1024);
      }
    }
    // the workgroup's tiles pt = 0.. are rows [prow pt, prow pt + prow) of one [rows][WLS] block in LDS (only
    // the prow output rows a tile really has are kept); bytes of the row padding and past the last row read
    // the start of the weights
    const int prow = a.prow;
    const int wp_rows = my_ptiles * prow;
    const int wp_chunks = (wp_rows * WLS + 1023) >> 10;
    for (int c = wave; c < wp_chunks; c += 4) {
      const int o = c * 1024 + lane * 16;
      const int r = o / WLS, col_b = o - r * WLS;
      const int8_t *src = a.Wp2;
      if (r < wp_rows && col_b < a.npadp) {
        const int pt = r / prow;
        src = a.Wp2 + ((size_t)(member + pt * GS) * 32 + (r - pt * prow)) * a.npadp + col_b;
      }
      dma(src, WpL + c * 1024);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  // cell state of this lane's 8 cells x RT row tiles, kept in registers
  int32_t creg[RT][2][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
      const int row = row0 + rt * 32 + col;
      const int n0 = member * 64 + cell_w + tl * 8;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        creg[rt][tl][c] = (a.c_in && row < a.B && n0 + c < a.N) ? a.c_in[(size_t)row * a.N + n0 + c] : 0;
    }

  // h tile staging by global -> LDS loads (no registers in between): wave
  // instruction (wave + 4 j) fills bytes [1024 c, 1024 (c + 1)) of the tile,
  // lane l its 16 bytes at 16 l; the lane's source is wherever that byte range
  // falls in the padded [row][LS] tile (pad bytes and the tail read offset 0
  // and hold garbage that only ever meets zero weights)
  constexpr int TILE_KB = (rows_pg * LS + 1023) / 1024;
  constexpr int NCH = (TILE_KB + 3) / 4;  // chunks per wave
  int hsrc[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int o = (wave + 4 * j) * 1024 + lane * 16;
    const int r = o / LS, c = o - r * LS;
    int row = row0 + r;
    row = row < a.B ? row : a.B - 1;
    hsrc[j] = (r < rows_pg && c < a.Hpad) ? row * a.Hpad + c : 0;
  }

  // projection bias of this thread's four outputs of its first tile
  int32_t bpr[4] = {0, 0, 0, 0};
  if (my_ptiles > 0) {
    const int4 b4 = *reinterpret_cast<const int4 *>(a.bp2 + member * 32 + 8 * (tid >> 6) + 4 * ((tid & 63) >> 5));
    bpr[0] = b4.x; bpr[1] = b4.y; bpr[2] = b4.z; bpr[3] = b4.w;
  }

  if (tid < 16) tickL[tid] = 0;
  if (tid < items) red[tid] = 0;
  if (tid == 0) {
    flag[0] = 1;
    flag[1] = 0;
  }
  __syncthreads();  // LDS contents above are in place before the first step

  unsigned epoch = 0;
  unsigned *counter = a.counters + group * 64;
  u64 *accS = a.acc + (size_t)group * kStatGroupWords;  // [set][round][S1|S2][item]
  int64_t prevS[2][2][2] = {{{0, 0}, {0, 0}}, {{0, 0}, {0, 0}}};  // this thread's item, per round and set: S1, S2
  const double inv_n = 1.0 / (double)a.N;
  const int g_first = cifg ? 1 : 0;
  // uniform: some shift of the layer norm's second stage / of the hidden state's rescale is below 33
  const bool pre_ln = ln && (a.rln[0] < 33 || a.rln[1] < 33 || a.rln[2] < 33 || a.rln[3] < 33);
  const bool pre_m = a.rm < 33;

  // optional phase timing of workgroup 0 (diagnostics): 100 MHz wall clock
  // ticks per phase, summed in LDS (an add that returns nothing, so the timer
  // waits for no memory) and written out after the last step
  long long tick_last = 0;
  const bool timing = a.ticks && wg == 0 && tid == 0;
#define TICK(i)                                                                           \
  do {                                                                                    \
    if (timing) {                                                                         \
      asm volatile("" ::: "memory");                                                      \
      const long long now = (long long)wall_clock64();                                    \
      __hip_atomic_fetch_add(&tickL[i], (u64)(now - tick_last), __ATOMIC_RELAXED,         \
                             __HIP_MEMORY_SCOPE_WORKGROUP);                               \
      tick_last = now;                                                                    \
    }                                                                                     \
  } while (0)
  if (timing) {
    tick_last = t_start;
    __hip_atomic_store(&a.ticks[15], t_start, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  TICK(10);  // everything before the first step

  // the two 16-byte W x pieces of (rt, tile) for step t
  auto tx_ptr = [&](int t, int rt, int tl) -> const int4 * {
    size_t rb = ((size_t)t * a.Bp + row0 + rt * 32) >> 5;
    const size_t rbmax = ((size_t)a.T * a.Bp) >> 5;
    rb = rb < rbmax ? rb : rbmax - 1;
    return a.tx2 + ((rb * (size_t)(GS * 8) + member * 8 + wave * 2 + tl) * 2) * 64 + lane;
  };


  // The W x terms of a step come from memory, not from a cache.  The dense kernel asks for them after the h tile
  // is in LDS: the MFMA phase covers the latency.  The sparse kernel's MFMA phase is too short for that (measured:
  // the gate sums, and then the whole group at the statistics, waited for the slowest workgroup's terms), so it
  // asks for the terms of step t before the last barrier of step t - 1 (those of step 0 ahead of the loop).
  // That is not free -- the polling wave's loads return in issue order, so its polls wait behind its own W x
  // loads -- which is why the dense kernel does not do the same (measured: 1.2 % slower with it).
  constexpr bool TX_AHEAD = SP;
  int4 txv[RT][2][2];
  auto load_tx = [&](int t) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int4 *src = tx_ptr(t, rt, tl);  // clamped to the last row block: step T reads step T - 1's again
        // read once: a streaming load keeps the W x terms from displacing the exchange buffers in L2
        const v4i t0 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(src));
        const v4i t1 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(src + 64));
        txv[rt][tl][0] = int4{t0.x, t0.y, t0.z, t0.w};
        txv[rt][tl][1] = int4{t1.x, t1.y, t1.z, t1.w};
      }
  };
  constexpr int TXLOADS = TX_AHEAD ? RT * 4 : 0;  // vector loads in flight across the step's last barrier
  if (TX_AHEAD && a.T > 0) load_tx(0);

  for (int t = 0; t < a.T; ++t) {
    // ---- h^{t-1} rows of the group -> LDS
    {
      const int8_t *hp = t == 0 ? a.h0 : a.out + (size_t)(t - 1) * a.B * a.Hpad;
#pragma unroll
      for (int j = 0; j < NCH; ++j)  // chunks past the tile land in the spare chunk behind it
        __builtin_amdgcn_global_load_lds(
              (const __attribute__((address_space(1))) void *)(hp + hsrc[j]),
              (__attribute__((address_space(3))) void *)(lds + (wave + 4 * j < TILE_KB ? wave + 4 * j : TILE_KB) * 1024),
              16, 0, 0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    if (!TX_AHEAD) load_tx(t);
    TICK(0);

    // ---- R h on the MFMA: acc[rt][tile][4*gate + c]
    v16i acc[RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rt][tl][v] = bhL[(v >> 2) * 64 + cell_w + tl * 8 + (v & 3)];
    if constexpr (SP) {
      constexpr int DEPTH = 2;  // 64-deep h fragments in flight ahead of the MFMAs
      v8i hf[RT][DEPTH];
      const int8_t *hbase = hT + (size_t)col * LS + (b2 << 5);
      auto frag = [&](int rt, int kq) {
        const v4i lo = *reinterpret_cast<const v4i *>(hbase + (size_t)rt * 32 * LS + kq * 64);
        const v4i hi = *reinterpret_cast<const v4i *>(hbase + (size_t)rt * 32 * LS + kq * 64 + 16);
        return v8i{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      };
#pragma unroll
      for (int kq = 0; kq < DEPTH && kq < KW; ++kq)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) hf[rt][kq] = frag(rt, kq);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kq = 0; kq < KW; ++kq) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
          for (int tl = 0; tl < 2; ++tl)
            acc[rt][tl] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(Wf[tl][kq], hf[rt][kq % DEPTH], acc[rt][tl], Wi[tl][kq], 0, 0);
          if (kq + DEPTH < KW) hf[rt][kq % DEPTH] = frag(rt, kq + DEPTH);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      constexpr int DEPTH = 4;  // h fragments in flight ahead of the MFMAs
      v4i hf[RT][DEPTH];
      const int8_t *hbase = hT + (size_t)col * LS + (b2 << 4);
#pragma unroll
      for (int ks = 0; ks < DEPTH && ks < KS; ++ks)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          hf[rt][ks] = *reinterpret_cast<const v4i *>(hbase + (size_t)rt * 32 * LS + ks * 32);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
          for (int tl = 0; tl < 2; ++tl)
            acc[rt][tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Wf[tl][ks], hf[rt][ks % DEPTH], acc[rt][tl], 0, 0, 0);  // acc starts from the folded bias
          if (ks + DEPTH < KS)
            hf[rt][ks % DEPTH] = *reinterpret_cast<const v4i *>(hbase + (size_t)rt * 32 * LS + (ks + DEPTH) * 32);
        }
        // keep the LDS reads DEPTH iterations ahead of their MFMAs: without
        // this the instruction scheduler sinks each read next to its use
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    TICK(1);

    // ---- gate sums (Secs. 3.2.4/3.2.5) and layer-norm partial statistics.
    // With a peephole the o gate keeps tx + th here and is finished after c^t.
    constexpr int32_t glo = ln ? -32767 : -32768;  // layer norm takes symmetric gate sums
    auto gate_sums = [&](auto pre_tag) {
      constexpr int PRE = decltype(pre_tag)::value;  // operand treatment of the R h rescale (RecArgs::pre_h)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        int32_t s1[4] = {0, 0, 0, 0};
        uint32_t s2[4][2] = {{0, 0}, {0, 0}, {0, 0}, {0, 0}};  // four squares of 16-bit values fit 32 bits
#pragma unroll
        for (int tl = 0; tl < 2; ++tl) {
          const int32_t txw[8] = {txv[rt][tl][0].x, txv[rt][tl][0].y, txv[rt][tl][0].z, txv[rt][tl][0].w,
                                  txv[rt][tl][1].x, txv[rt][tl][1].y, txv[rt][tl][1].z, txv[rt][tl][1].w};
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const RescaleHi pg = prm->h[g];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const int idx = g * 4 + c;
              const int32_t th = rescale_sat16_pre<PRE>(acc[rt][tl][idx], pg);
              const int32_t w = txw[idx >> 1];
              const int32_t tx = (idx & 1) ? (w >> 16) : (int32_t)(int16_t)(w & 0xFFFF);
              int32_t v = tx + th;
              if (ph && g < 2) {
                const int cl = cell_w + tl * 8 + c;
                v += rescale_sat16_pre((int32_t)PqL[g * 64 + cl] * creg[rt][tl][c], prm->c[g]);
              }
              if (!(ph && g == 3)) v = clamp_i32(v, glo, 32767);
              acc[rt][tl][idx] = v;
              s1[g] += v;
              s2[g][tl] += (uint32_t)v * (uint32_t)v;
            }
          }
        }
        if (ln) {
#pragma unroll
          for (int g = 0; g < (ph ? 3 : 4); ++g) {  // with a peephole the o gate follows after c^t
            // the 8 lanes of a row (2 per wave) add into one LDS word: no cross-lane traffic, no wait
            const int64_t pk = ((int64_t)((u64)s2[g][0] + (u64)s2[g][1]) << 24) + s1[g];
            __hip_atomic_fetch_add(&red[(rt * 4 + g) * 32 + col], (u64)pk, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        }
      }
    };
    if (a.pre_h == 0)
      gate_sums(std::integral_constant<int, 0>{});
    else if (a.pre_h == 1)
      gate_sums(std::integral_constant<int, 1>{});
    else
      gate_sums(std::integral_constant<int, 2>{});

    // Layer-norm statistics of a row are summed over the group's workgroups by
    // atomic adds into two 64-bit words per (row, gate), which are never reset:
    // the reader subtracts what it read the step before.  The top byte of each
    // word counts the adds, so the words themselves tell when every workgroup of
    // the group has contributed and no separate barrier is needed.  Value field
    // (56 bits): S1 + 2^22 >= 0 per add, at most 2^23; S2 at most 2^36 per add;
    // with at most 32 adds per step the fields hold more than 2^14 steps.
    constexpr u64 kValMask = ((u64)1 << 56) - 1;
    auto publish_stats = [&](int round, int g_lo, int g_hi) {
      __syncthreads();
      if (tid < items) {
        const int g = (tid >> 5) & 3;
        if (g >= g_lo && g <= g_hi) {
          const int64_t pk = (int64_t)red[tid];
          red[tid] = 0;  // the next adds to this word come after the next barrier
          const int64_t v1 = ((pk + (1 << 23)) & 0xFFFFFF) - (1 << 23);  // signed low 24 bits
          const int64_t v2 = (pk - v1) >> 24;
          u64 *mine = accS + (stat_two_sets(GS) ? (member & 1) : 0) * kStatSetWords;  // this workgroup's set of words
          __hip_atomic_fetch_add(&mine[(round * 2 + 0) * 256 + tid], ((u64)1 << 56) + (u64)(v1 + (1 << 22)),
                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_add(&mine[(round * 2 + 1) * 256 + tid], ((u64)1 << 56) + (u64)v2, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    };
    // false: a wait gave up (status word raised), every thread leaves the kernel
    auto collect_stats = [&](int round, int g_lo, int g_hi) -> bool {
      if (tid < items) {
        const int g = (tid >> 5) & 3;
        if (g >= g_lo && g <= g_hi) {
          // two sets: set 0 holds the adds of the even members, set 1 those of the odd ones
          const bool two = stat_two_sets(GS);
          const unsigned n0 = two ? ((unsigned)GS + 1) >> 1 : (unsigned)GS, n1 = two ? (unsigned)GS >> 1 : 0u;
          const u64 expect0 = (u64)((n0 * (unsigned)(t + 1)) & 0xFFu), expect1 = (u64)((n1 * (unsigned)(t + 1)) & 0xFFu);
          u64 c1[2], c2[2];
          int budget = a.spin_limit;
          // the adds of the other workgroups need this long to land; a poll before that only delays them
          for (int i = 0; i < a.stats_first_sleep; ++i) __builtin_amdgcn_s_sleep(1);
          for (;;) {
            c1[0] = __hip_atomic_load(&accS[(round * 2 + 0) * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c2[0] = __hip_atomic_load(&accS[(round * 2 + 1) * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c1[1] = c2[1] = 0;  // one set: the second set's words are never added to, nor read
            if (two) {
              c1[1] = __hip_atomic_load(&accS[kStatSetWords + (round * 2 + 0) * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              c2[1] = __hip_atomic_load(&accS[kStatSetWords + (round * 2 + 1) * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if ((c1[0] >> 56) == expect0 && (c2[0] >> 56) == expect0 && (c1[1] >> 56) == expect1 && (c2[1] >> 56) == expect1) break;
            --budget;
            if ((budget & 15) == 0 &&
                (budget <= 0 || __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
              __hip_atomic_store(a.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              *flag = 0;
              break;
            }
            for (int i = 0; i < a.stats_sleep; ++i) __builtin_amdgcn_s_sleep(1);
          }
          int64_t S1 = -(int64_t)GS * (1 << 22), S2 = 0;
#pragma unroll
          for (int ss = 0; ss < 2; ++ss) {
            c1[ss] &= kValMask;
            c2[ss] &= kValMask;
            S1 += (int64_t)((c1[ss] - (u64)prevS[round][ss][0]) & kValMask);
            S2 += (int64_t)((c2[ss] - (u64)prevS[round][ss][1]) & kValMask);
            prevS[round][ss][0] = (int64_t)c1[ss];
            prevS[round][ss][1] = (int64_t)c2[ss];
          }
          lnrow[tid] = ln_row2(ln_row(S1, S2, a.N, inv_n));
        }
      }
      __syncthreads();
      return *flag != 0;
    };
    TICK(2);
    if (ln) {
      publish_stats(0, g_first, ph ? 2 : 3);
      TICK(3);
      if (!collect_stats(0, g_first, ph ? 2 : 3)) return;
      TICK(4);
    }

    // ---- layer norm, sigma/tanh, cell update (Secs. 3.2.6, 3.2.1, 3.2.9, 3.2.7),
    // in batches of one weight tile (up to 4 gates x 4 cells of a row).  Every
    // LDS read of a batch is issued before the first use of any of them: the
    // scheduling barriers keep the compiler from sinking each read next to its
    // use, which exposes one LDS round trip per element (measured: more than
    // half of this phase).
    // gates of `gmask` (bit g) of tile (rt, tl): gate sums -> layer norm -> xv[g][c]
    constexpr int LNB = KS >= 32 ? 1 : 2;  // the deepest register-resident R leaves room for less
    auto normalize = [&](int rt, int tl, int gmask, const LnRow2 (&lr)[4], int32_t (&xv)[4][4], bool narrow) {
      if (ln) {
#pragma unroll
        for (int gp = 0; gp < 4; gp += LNB) {  // LNB gates per batch of reads: 8 LNB doubles in flight
          if (!(gmask >> gp & ((1 << LNB) - 1))) continue;
          double wL[LNB][4], wb[LNB][4];
          RescaleHi pl[LNB];
#pragma unroll
          for (int g = gp; g < gp + LNB; ++g)
            if (gmask >> g & 1) {
              pl[g - gp] = prm->ln[g];
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                wL[g - gp][c] = LdL[g * 64 + cell_w + tl * 8 + c];
                wb[g - gp][c] = bdL[g * 64 + cell_w + tl * 8 + c];
              }
            }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int g = gp; g < gp + LNB; ++g)
            if (gmask >> g & 1)
#pragma unroll
              for (int c = 0; c < 4; ++c)
                xv[g][c] = narrow ? ln_second_stage_narrow(acc[rt][tl][g * 4 + c], lr[g], wL[g - gp][c], wb[g - gp][c])
                                  : ln_second_stage(acc[rt][tl][g * 4 + c], lr[g], wL[g - gp][c], wb[g - gp][c]);
          if (pre_ln) {  // some second-stage shift is below 33 (uniform; rare)
#pragma unroll
            for (int g = gp; g < gp + LNB; ++g)
              if (gmask >> g & 1)
#pragma unroll
                for (int c = 0; c < 4; ++c) xv[g][c] = rescale_preshift(xv[g][c], pl[g - gp]);
          }
#pragma unroll
          for (int g = gp; g < gp + LNB; ++g)
            if (gmask >> g & 1)
#pragma unroll
              for (int c = 0; c < 4; ++c) xv[g][c] = rescale_sat16_pre<0>(xv[g][c], pl[g - gp]);
        }
      } else {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if (gmask >> g & 1)
#pragma unroll
            for (int c = 0; c < 4; ++c) xv[g][c] = acc[rt][tl][g * 4 + c];
      }
    };
    // table values of |xv[g][c]| for the gates of gmask; tb[g] = which table (0 sigma, 1 tanh, 2 cell tanh)
    auto lookup = [&](int gmask, const int32_t (&xv)[4][4], const int (&tb)[4], int32_t (&tv)[4][4]) {
      int32_t mag[4][4];
      uint32_t base[4][4], delta[4][4];
      int32_t top[3] = {0, 0, 0};  // largest |x| looked up in each table
      // the tables' places and sizes come from LDS (the same words for every lane)
      LutLds lp[3];
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        bool used = false;
#pragma unroll
        for (int g = 0; g < 4; ++g) used = used || ((gmask >> g & 1) && tb[g] == i);
        if (used) lp[i] = lutP[i];
      }
#pragma unroll
      for (int g = 0; g < 4; ++g)
        if (gmask >> g & 1) {
          const int dom = lp[tb[g]].dom, sh = lp[tb[g]].sh;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            mag[g][c] = abs_i32(xv[g][c]);  // at most 2^15
            top[tb[g]] = top[tb[g]] > mag[g][c] ? top[tb[g]] : mag[g][c];
            const int32_t ai = mag[g][c] < dom ? mag[g][c] : dom - 1;
            base[g][c] = *reinterpret_cast<const uint16_t *>(lds + lp[tb[g]].offB + 2 * (ai >> sh));
            delta[g][c] = lds[lp[tb[g]].offD + ai];
          }
        }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < 4; ++g)
        if (gmask >> g & 1)
#pragma unroll
          for (int c = 0; c < 4; ++c) tv[g][c] = (int32_t)(base[g][c] + delta[g][c]);
      // A value at or beyond the prefix kept in LDS takes its table value from the tail part (a table kept
      // without one is flat from there on, and the clamped index was the lookup).  How often that happens is
      // the launch's choice of prefix: with 16384 entries (|x| < 4 in Q3.12) about one layer-norm output in a
      // thousand, i.e. some lane of most batches -- and the step then waits for the slowest of the group's
      // 128 waves; with 24576 entries it is one in a million.  The tests narrow down from the batch to the
      // gate to the cell.
      bool over = false;
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        bool used = false;
#pragma unroll
        for (int g = 0; g < 4; ++g) used = used || ((gmask >> g & 1) && tb[g] == i);
        if (used) over |= top[i] >= lp[i].dom;
      }
      if (__builtin_amdgcn_ballot_w64(over) != 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if ((gmask >> g & 1) && lp[tb[g]].offT) {
            const int dom = lp[tb[g]].dom;
            const bool og = mag[g][0] >= dom || mag[g][1] >= dom || mag[g][2] >= dom || mag[g][3] >= dom;
            if (__builtin_amdgcn_ballot_w64(og) != 0) {
#pragma unroll
              for (int c = 0; c < 4; ++c)
                if (mag[g][c] >= dom) tv[g][c] = lut_wide_tail(lds + lp[tb[g]].offT, mag[g][c]);
            }
          }
      }
    };
    const int gate_tb[4] = {0, 0, 1, 0};
    constexpr int gates_now = (cifg ? 0 : 1) | 2 | 4 | (ph ? 0 : 8);  // with a peephole the o gate waits for c^t
    int32_t xi[RT][2][4], xf[RT][2][4], xz[RT][2][4], xo[RT][2][4];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      LnRow2 lr[4];
      bool narrow = false;  // uniform: every row of this wave has sigma >= 2^12, the second stage stays within int32
      if (ln) {
        bool wide = false;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          lr[g] = lnrow[(rt * 4 + g) * 32 + col];
          if (gates_now >> g & 1) wide |= !ln_row_is_narrow(lr[g]);
        }
        narrow = __builtin_amdgcn_ballot_w64(wide) == 0;
      }
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        int32_t xv[4][4], tv[4][4];
        if (narrow)
          normalize(rt, tl, gates_now, lr, xv, true);
        else
          normalize(rt, tl, gates_now, lr, xv, false);
        if (KS >= 32) {  // the deepest register-resident R leaves room for two gates' reads at a time
          lookup(gates_now & 3, xv, gate_tb, tv);
          lookup(gates_now & 12, xv, gate_tb, tv);
        } else {
          lookup(gates_now, xv, gate_tb, tv);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          xi[rt][tl][c] = cifg ? 0 : mirror_sigmoid(xv[0][c], tv[0][c]);
          xf[rt][tl][c] = mirror_sigmoid(xv[1][c], tv[1][c]);
          xz[rt][tl][c] = mirror_tanh(xv[2][c], tv[2][c]);
          xo[rt][tl][c] = ph ? 0 : mirror_sigmoid(xv[3][c], tv[3][c]);
        }
      }
    }
    const int32_t m_c = prm->m_c;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      int32_t s1 = 0;
      int64_t s2 = 0;
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int32_t f = xf[rt][tl][c];
          const int32_t i = cifg ? cifg_input_gate(f) : xi[rt][tl][c];
          const int32_t cnew = cell_update32(i, xz[rt][tl][c], f, creg[rt][tl][c], m_c);
          creg[rt][tl][c] = cnew;
          if (ph) {  // finish the o gate sum with P_o . c^t (eq. 5)
            const int cl = cell_w + tl * 8 + c;
            int32_t v = acc[rt][tl][12 + c] +
                        rescale_sat16_pre((int32_t)PqL[2 * 64 + cl] * cnew, prm->c[2]);
            v = clamp_i32(v, glo, 32767);
            acc[rt][tl][12 + c] = v;
            s1 += v;
            s2 += (int64_t)v * v;
          }
        }
      if (ph && ln) {
        const int64_t pk = (s2 << 24) + s1;
        __hip_atomic_fetch_add(&red[(rt * 4 + 3) * 32 + col], (u64)pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
    TICK(5);
    if (ph) {
      if (ln) {
        publish_stats(1, 3, 3);
        if (!collect_stats(1, 3, 3)) return;
      }
    }

    // ---- hidden state (Sec. 3.2.7); m is int8.  tanh of the new cell state in its
    // own format (Sec. 3.2.2), and with a peephole the layer norm and sigma of the o gate
    int32_t tc[RT][2][4];
    {
      const int hid_tb[4] = {2, 2, 0, 0};  // c^t of the two weight tiles, then the o gate sums of the two
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        LnRow2 lr[4];
        if (ph && ln) lr[3] = lnrow[(rt * 4 + 3) * 32 + col];
        // one batch per row tile: c^t of both weight tiles in slots 0 and 1, the o gate sums in 2 and 3
        int32_t xv[4][4], tv[4][4], ov[2][4][4];
#pragma unroll
        for (int tl = 0; tl < 2; ++tl) {
#pragma unroll
          for (int c = 0; c < 4; ++c) xv[tl][c] = creg[rt][tl][c];
          if (ph) {
            normalize(rt, tl, 8, lr, ov[tl], false);
#pragma unroll
            for (int c = 0; c < 4; ++c) xv[2 + tl][c] = ov[tl][3][c];
          }
        }
        lookup(ph ? 15 : 3, xv, hid_tb, tv);
#pragma unroll
        for (int tl = 0; tl < 2; ++tl)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            tc[rt][tl][c] = mirror_tanh(xv[tl][c], tv[tl][c]);
            if (ph) xo[rt][tl][c] = mirror_sigmoid(xv[2 + tl][c], tv[2 + tl][c]);
          }
      }
    }
    // Without a projection m is h and goes to the layer output [T, B, Hpad].  With one it goes to the
    // exchange buffer in the order the projection reads it: [t][row tile][k step][row % 32][32 cells],
    // so that a wave's load of one k step is one contiguous KB of whole cache lines.
    int8_t *mdst = proj ? a.mbuf + (size_t)t * a.Bp * a.npadp : a.out + (size_t)t * a.B * a.Hpad;
    const RescaleHi pm = prm->m;
    const int32_t zp_m = prm->zp_m;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int row = row0 + rt * 32 + col;
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int n0 = member * 64 + cell_w + tl * 8;
        uint32_t pk = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          // sat8 of the sum is unchanged by the 16-bit clamp before it: |zp| <= 128
          int32_t om = xo[rt][tl][c] * tc[rt][tl][c];  // below 2^30 in magnitude
          if (pre_m) om = rescale_preshift(om, pm);
          const int32_t mq = sat8(rescale_sat16_pre<0>(om, pm) + zp_m);
          pk |= (uint32_t)(mq & 0xFF) << (8 * c);
        }
        if (row < a.B && n0 < a.N) {  // N % 8 == 0: the four cells are valid together
          const size_t off = proj ? ((((size_t)(row >> 5) * (a.npadp >> 5) + (n0 >> 5)) * 32 + (row & 31)) * 32 + (n0 & 31))
                                  : (size_t)row * a.Hpad + n0;
          *reinterpret_cast<uint32_t *>(mdst + off) = pk;
          if (!proj && a.y) {
            int8_t *yd = a.y + ((size_t)t * a.B + row) * a.H + n0;  // H = N, a multiple of 4
            __builtin_nontemporal_store(pk, reinterpret_cast<uint32_t *>(yd));  // not read again here
          }
        }
      }
    }
    TICK(6);
    if (proj) {
      if (!group_sync(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, a.sync_sleep, a.poll_sleep, flag)) return;
    } else {
      if (TX_AHEAD) load_tx(t + 1);
      if (!group_sync<TXLOADS>(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, a.sync_sleep, a.poll_sleep, flag)) return;
    }
    TICK(7);

    // ---- projection (Sec. 3.2.8): tile pt of 32 outputs, K = N split over the four waves
    if (proj) {

      const int per_wave = a.npadp >> 7;  // 32-wide k steps per wave, at most 16 (N <= 2048)
      const RescaleHi pp = prm->p;
      const int32_t zp_h = prm->zp_h;
      for (int pt = 0; pt < my_ptiles; ++pt) {
        const int ptile = member + pt * GS;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          // a row tile that starts beyond the batch (second tile of a ragged last group) has no rows in the
          // exchange buffer at all; the test is uniform over the workgroup, so the barriers below stay matched
          if (rt > 0 && row0 + rt * 32 >= a.B) continue;
          // rows of the tile beyond the batch were never written; their results are not stored either
          const int8_t *mrow = a.mbuf + (size_t)t * a.Bp * a.npadp +
                               ((((size_t)((row0 >> 5) + rt) * (a.npadp >> 5) + wave * per_wave) * 32 + col) << 5) +
                               (b2 << 4);
          // operand rows beyond the tile's prow outputs re-read row 0: their results are never stored
          const int8_t *wrow = WpL + ((size_t)pt * a.prow + (col < a.prow ? col : 0)) * WLS + (b2 << 4) + wave * per_wave * 32;
          int4 mv[16];
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            const int kk = k < per_wave ? k : per_wave - 1;  // steps past the end re-read the last one
            mv[k] = *reinterpret_cast<const int4 *>(mrow + kk * 1024);
          }
          v16i pacc;
#pragma unroll
          for (int v = 0; v < 16; ++v) pacc[v] = 0;
          if (per_wave == 16) {  // N = 2048: no padding step, no operand select
#pragma unroll
            for (int k = 0; k < 16; ++k) {
              const v4i wf = *reinterpret_cast<const v4i *>(wrow + k * 32);
              pacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, v4i{mv[k].x, mv[k].y, mv[k].z, mv[k].w}, pacc, 0, 0, 0);
            }
          } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
              const int kk = k < per_wave ? k : per_wave - 1;
              v4i wf = *reinterpret_cast<const v4i *>(wrow + kk * 32);
              if (k >= per_wave) wf = v4i{0, 0, 0, 0};  // ... against zero weights
              pacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, v4i{mv[k].x, mv[k].y, mv[k].z, mv[k].w}, pacc, 0, 0, 0);
            }
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) pred[(wave * 16 + v) * 64 + lane] = pacc[v];
          __syncthreads();
          {
            // thread (q = tid / 64, lane' = tid % 64): outputs 8q + 4*(lane'/32) + 0..3 of row lane' % 32
            const int q = tid >> 6, l2 = tid & 63;
            const int pl = 8 * q + 4 * (l2 >> 5);  // row of the tile; prow is a multiple of 4
            const int p0 = ptile * a.prow + pl;
            const int orow = row0 + rt * 32 + (l2 & 31);
            uint32_t pk = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              const int v = 4 * q + c;
              const int32_t s = pred[(0 * 16 + v) * 64 + l2] + pred[(1 * 16 + v) * 64 + l2] +
                                pred[(2 * 16 + v) * 64 + l2] + pred[(3 * 16 + v) * 64 + l2] +
                                (pt == 0 ? bpr[c] : a.bp2[ptile * 32 + pl + c]);
              const int32_t hq = sat8(rescale_sat16_pre(s, pp) + zp_h);
              pk |= (uint32_t)(hq & 0xFF) << (8 * c);
            }
            if (orow < a.B && p0 < a.H && pl < a.prow) {
              int8_t *od = a.out + ((size_t)t * a.B + orow) * a.Hpad + p0;
              if (p0 + 3 < a.H) {
                *reinterpret_cast<uint32_t *>(od) = pk;
              } else {
                for (int c = 0; c < 4 && p0 + c < a.H; ++c) od[c] = (int8_t)(pk >> (8 * c));
              }
              if (a.y) {
                int8_t *yd = a.y + ((size_t)t * a.B + orow) * a.H + p0;
                for (int c = 0; c < 4 && p0 + c < a.H; ++c) yd[c] = (int8_t)(pk >> (8 * c));
              }
            }
          }
          __syncthreads();
        }
      }
      TICK(8);
      if (TX_AHEAD) load_tx(t + 1);
      if (!group_sync<TXLOADS>(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, my_ptiles == 0 ? a.idle_sleep : 0,
                      my_ptiles == 0 ? a.idle_poll_sleep : a.poll_sleep, flag))
        return;
      TICK(9);
    }
  }
#undef TICK
  if (timing)
    for (int i = 0; i < 11; ++i) a.ticks[i] += (long long)tickL[i];
  if (a.ticks && tid == 0) {
    // spread of the workgroups' lifetimes against workgroup 0's start (maxima over all launches)
    const long long t0 = __hip_atomic_load(&a.ticks[15], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const long long t_end = (long long)wall_clock64();
    if (wg == 0) a.ticks[11] += t_end - t_start;
    __hip_atomic_fetch_max(&a.ticks[12], t_start - t0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_fetch_max(&a.ticks[13], t_end - t0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_fetch_max(&a.ticks[14], t0 - t_start, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  placement_check();
  if (a.c_out) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int row = row0 + rt * 32 + col;
        const int n0 = member * 64 + cell_w + tl * 8;
        if (row < a.B && n0 < a.N)
#pragma unroll
          for (int c = 0; c < 4; ++c) a.c_out[(size_t)row * a.N + n0 + c] = (int16_t)creg[rt][tl][c];
      }
  }
}


typedef void (*rec_fn)(RecArgs);

// sparse-weight kernel for the flags at k depth KS (one row tile per group)
template <int KS>
rec_fn rec_pick_sparse_ks(int fl) {
#define LSTM_REC_CASE(F) \
  if (fl == F) return rec_kernel<KS, 1, F, true>;
  LSTM_REC_CASE(0) LSTM_REC_CASE(1) LSTM_REC_CASE(2) LSTM_REC_CASE(3)
  LSTM_REC_CASE(4) LSTM_REC_CASE(5) LSTM_REC_CASE(6) LSTM_REC_CASE(7)
  LSTM_REC_CASE(8) LSTM_REC_CASE(9) LSTM_REC_CASE(10) LSTM_REC_CASE(11)
  LSTM_REC_CASE(12) LSTM_REC_CASE(13) LSTM_REC_CASE(14) LSTM_REC_CASE(15)
#undef LSTM_REC_CASE
  return nullptr;
}

// kernel for (rt, flags & 7) at k depth KS
template <int KS>
rec_fn rec_pick_ks(int rt, int fl) {
#define LSTM_REC_CASE(R, F) \
  if (rt == R && fl == F) return rec_kernel<KS, R, F>;
  LSTM_REC_CASE(1, 0) LSTM_REC_CASE(1, 1) LSTM_REC_CASE(1, 2) LSTM_REC_CASE(1, 3)
  LSTM_REC_CASE(1, 4) LSTM_REC_CASE(1, 5) LSTM_REC_CASE(1, 6) LSTM_REC_CASE(1, 7)
  LSTM_REC_CASE(1, 8) LSTM_REC_CASE(1, 9) LSTM_REC_CASE(1, 10) LSTM_REC_CASE(1, 11)
  LSTM_REC_CASE(1, 12) LSTM_REC_CASE(1, 13) LSTM_REC_CASE(1, 14) LSTM_REC_CASE(1, 15)
  if (KS < 32) {
    LSTM_REC_CASE(2, 0) LSTM_REC_CASE(2, 1) LSTM_REC_CASE(2, 2) LSTM_REC_CASE(2, 3)
    LSTM_REC_CASE(2, 4) LSTM_REC_CASE(2, 5) LSTM_REC_CASE(2, 6) LSTM_REC_CASE(2, 7)
    LSTM_REC_CASE(2, 8) LSTM_REC_CASE(2, 9) LSTM_REC_CASE(2, 10) LSTM_REC_CASE(2, 11)
    LSTM_REC_CASE(2, 12) LSTM_REC_CASE(2, 13) LSTM_REC_CASE(2, 14) LSTM_REC_CASE(2, 15)
  }
#undef LSTM_REC_CASE
  return nullptr;
}

}  // namespace lstm_int
