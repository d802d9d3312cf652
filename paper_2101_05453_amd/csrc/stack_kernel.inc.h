// Device code of the stacked recurrent kernel: up to 8 equal layers in one
// launch, layer l on XCD l, each layer one step behind the layer below it (the
// stack of Sec. 7 as a wavefront over layers and time).  The per-step
// arithmetic is rec_kernel's (Secs. 3.2.4-3.2.9); what differs:
//   * the W x term of an item (step t, row tile r) is computed here, when the
//     layer's input rows arrive, from weights streamed out of memory as MFMA
//     operands (R stays in registers for the whole launch);
//   * R h^{t-1} runs first and is kept as packed int16 terms, so that the only
//     work between the arrival of the input and the gate sums is W x;
//   * a layer's output rows are stored with agent-scope stores, which write
//     through the XCD's L2, and a flag per (layer, row tile) counts the
//     finished steps; the next layer polls it and reads the rows with loads
//     that bypass its own L2.  Every such line is written once per launch and
//     was never read before, so no cache on the reading side can hold an older
//     copy.
//   * the cell state lives in memory between the items of a row tile.
// Included by the stack_inst_*.hip translation units.
#pragma once

#include <type_traits>

#include "lstm_int_math.h"
#include "persistent.h"
#include "rec_kernel.inc.h"  // group_sync, lut helpers, mirror_*, vector types

namespace lstm_int {

typedef short v2s __attribute__((ext_vector_type(2)));

struct StkPrm {  // per-layer constants in LDS, 320 bytes
  RescaleHi h[4], c[4], ln[4], x[4];
  RescaleHi m, p;
  int32_t zp_m, zp_h, m_c, glo;
  int32_t pad[4];
};
static_assert(sizeof(StkPrm) == 320, "stack_lds_bytes assumes 320 bytes");

// sat16(rescale(.)) of two accumulators, packed low | high; PRE = operand treatment of the rescale
template <int PRE>
__device__ __forceinline__ int32_t stk_requant2(int32_t s0, int32_t s1, const RescaleHi &p) {
  const int32_t v0 = rescale_sat16_pre<PRE>(s0, p), v1 = rescale_sat16_pre<PRE>(s1, p);
  return (v0 & 0xFFFF) | (v1 << 16);
}

// FL as in rec_kernel: bit 0 CIFG, bit 1 peephole, bit 2 layer norm, bit 3 "no projection".
// ONE: the launch has one item per layer (one step, one row tile).
template <int KS, int FL, bool ONE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void stack_kernel(StackArgs sa) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const RecArgs &a = sa.c;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, b2 = lane >> 5;
  constexpr bool cifg = FL & 1, ph = FL & 2, ln = FL & 4;
  constexpr bool proj = !(FL & 8);
  const int GS = a.GS;

  // Placement as in rec_kernel: the XCD comes from the hardware register, the place on it from the
  // workgroup index; here the XCD is the layer.
  const int wg = blockIdx.x;
  const int xcc = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7);
  const int slot = wg >> 3;
  int xcd = wg & 7;
  if (a.tickets) {
    xcd = xcc;
  } else if (xcc != xcd && tid == 0) {
    __hip_atomic_store(a.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
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
  const int layer = xcd, member = slot;  // slot < GS: the launch has GS workgroups per XCD
  if (layer >= sa.L) {
    placement_check();
    return;
  }
  const StackLayer &sl = sa.layers[layer];
  const bool last_layer = layer == sa.L - 1;
  constexpr int items = 128;  // (gate, row) layer-norm rows of a row tile

  // per-layer buffers
  const int8_t *xin = layer == 0 ? sa.x : sa.out_base + (size_t)(layer - 1) * sa.out_stride;
  const int ldx = layer == 0 ? sa.ldx : a.Hpad;
  const bool x_bypass = layer > 0 || !sa.x_shared;  // rows written by another XCD during this launch
  int8_t *out = sa.out_base + (size_t)layer * sa.out_stride;
  const int8_t *h0 = sa.h0_base + (size_t)layer * a.B * a.Hpad;
  int8_t *mbuf = sa.mbuf_base + (size_t)layer * sa.mbuf_stride;
  int16_t *cbuf = sa.c_base + (size_t)layer * a.B * a.N;
  int8_t *yout = last_layer ? a.y : nullptr;
  int8_t *hfin = sa.h_final ? sa.h_final + (size_t)layer * a.B * a.H : nullptr;
  const int kx = sl.kx;

  // ---- LDS carve-up (stack_lds_bytes mirrors it)
  constexpr int LS = KS * 32 + 16;  // tile row stride (h rows and x rows alike)
  uint8_t *p = lds;
  int8_t *hT = reinterpret_cast<int8_t *>(p);
  int32_t *pred = reinterpret_cast<int32_t *>(p);  // projection partials reuse the tile between steps
  {
    const size_t tile_bytes = (((size_t)32 * LS + 1023) / 1024 + 1) * 1024;
    const size_t pred_bytes = proj ? 4 * 16 * 64 * 4 : 0;
    p += tile_bytes > pred_bytes ? tile_bytes : pred_bytes;
  }
  u64 *red = reinterpret_cast<u64 *>(p);                 p += (size_t)items * 8;
  LnRow2 *lnrow = reinterpret_cast<LnRow2 *>(p);         p += (size_t)items * sizeof(LnRow2);
  double *LdL = reinterpret_cast<double *>(p);           p += 4 * 64 * 8;
  double *bdL = reinterpret_cast<double *>(p);           p += 4 * 64 * 8;
  int16_t *PqL = reinterpret_cast<int16_t *>(p);         p += 4 * 64 * 2;
  int32_t *bhL = reinterpret_cast<int32_t *>(p);         p += 4 * 64 * 4;
  int32_t *bxL = reinterpret_cast<int32_t *>(p);         p += 8 * 32 * 4;  // folded input bias, tile row order
  StkPrm *prm = reinterpret_cast<StkPrm *>(p);           p += sizeof(StkPrm);
  int *flag = reinterpret_cast<int *>(p);                p += 16;
  u64 *tickL = reinterpret_cast<u64 *>(p);               p += 12 * 8;  // phase timers
  LutLds *lutP = reinterpret_cast<LutLds *>(p);          p += 3 * sizeof(LutLds);
  // the activation tables as in rec_kernel: prefixes of the wide form; the two gate tables are common to
  // the layers, the cell-format tanh is the layer's own (or the gate tanh's copy when the formats agree)
  const LutWide lw[3] = {a.lut[0], a.lut[1], sl.lutc};
  const bool share_tanh = lw[2].blob == lw[1].blob;
  const uint8_t *lutD[3];
  const uint8_t *lutB[3];
  const uint8_t *lutTl[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    if (i == 2 && share_tanh) {
      lutD[2] = lutD[1]; lutB[2] = lutB[1]; lutTl[2] = lutTl[1];
    } else {
      const int nb = ((((lw[i].dom >> lw[i].sh) * 2) + 1023) >> 10) << 10;
      lutD[i] = p;                            p += lw[i].dom;
      lutB[i] = p;                            p += nb;
      lutTl[i] = lw[i].tail ? p : nullptr;    p += lw[i].tail ? 3072 : 0;
    }
  }
  int8_t *WpL = reinterpret_cast<int8_t *>(p);
  const int WLS = a.npadp + 16;
  const int my_ptiles = proj ? (a.ptiles > member ? (a.ptiles - member + GS - 1) / GS : 0) : 0;

  // ---- one-time loads: R slice -> registers; per-cell parameters, tables, W_proj tiles -> LDS
  v4i Wf[2][KS];
  {
    const int4 *src = sl.R2 + ((size_t)(member * 4 + wave) * 2) * KS * 64 + lane;
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
      int4 w[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) w[ks] = src[(size_t)(tl * KS + ks) * 64];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Wf[tl][ks] = v4i{w[ks].x, w[ks].y, w[ks].z, w[ks].w};
        asm volatile("" : "+a"(Wf[tl][ks]));  // resident in accumulation registers for the whole launch
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const int cell_w = wave * 16 + 4 * b2;  // + tile * 8 + c, within the workgroup's 64 cells
  {
    const int g = tid >> 6, n = tid & 63;
    const size_t idx = (size_t)g * a.Ncp + member * 64 + n;
    LdL[tid] = ln ? ln_weight_scaled(sl.Lq4[idx]) : 0.0;
    bdL[tid] = ln ? ln_bias_scaled(sl.qb4[idx]) : 0.0;
    PqL[tid] = (ph && g < 3) ? sl.Pq3[idx] : 0;
    bhL[tid] = sl.bh4[idx];
    bxL[tid] = sl.bx2[(size_t)member * 256 + tid];  // the workgroup's 8 tiles x 32 rows
  }
  if (tid < 4) {
    prm->h[tid] = rescale_hi_prepare(sl.Mh[tid], sl.rh[tid]);
    prm->x[tid] = rescale_hi_prepare(sl.Mx[tid], sl.rx[tid]);
    prm->c[tid] = rescale_hi_prepare(tid < 3 && ph ? sl.Mc[tid] : 0, tid < 3 && ph ? sl.rc[tid] : 33);
    prm->ln[tid] = rescale_hi_prepare(sl.Mln[tid], ln ? sl.rln[tid] : 33);
  }
  if (tid < 3) {
    LutLds d;
    const LutWide &w = (tid == 2 && share_tanh) ? lw[1] : lw[tid];  // a shared copy has the gate table's prefix
    d.dom = w.dom; d.sh = w.sh;
    d.offD = (int32_t)(lutD[tid] - lds);
    d.offB = (int32_t)(lutB[tid] - lds);
    d.offT = lutTl[tid] ? (int32_t)(lutTl[tid] - lds) : 0;
    d.pad[0] = d.pad[1] = d.pad[2] = 0;
    lutP[tid] = d;
  }
  if (tid == 0) {
    prm->m = rescale_hi_prepare(sl.Mm, sl.rm);
    prm->p = rescale_hi_prepare(proj ? sl.Mp : 0, proj ? sl.rp : 33);
    prm->zp_m = sl.zp_m; prm->zp_h = sl.zp_h;
    prm->m_c = sl.m_c; prm->glo = ln ? -32767 : -32768;
  }
  for (int i = tid; i < 32 * LS / 16; i += 256) reinterpret_cast<int4 *>(hT)[i] = int4{0, 0, 0, 0};
  {
    auto dma = [&](const void *src, const void *dst) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                       (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };
    for (int i = 0; i < (share_tanh ? 2 : 3); ++i) {
      const int nd = lw[i].dom >> 10;
      const int nb = (((lw[i].dom >> lw[i].sh) * 2) + 1023) >> 10;
      const int nt = lw[i].tail ? 3 : 0;
      for (int c = wave; c < nd + nb + nt; c += 4) {
        const int so = c < nd ? c * 1024 : (c < nd + nb ? kLutWideBaseOff + (c - nd) * 1024 : kLutWideTailOff + (c - nd - nb) * 1024);
        dma(lw[i].blob + so + lane * 16, lutD[i] + c * 1024);
      }
    }
    const int prow = a.prow;
    const int wp_rows = my_ptiles * prow;
    const int wp_chunks = (wp_rows * WLS + 1023) >> 10;
    for (int c = wave; c < wp_chunks; c += 4) {
      const int o = c * 1024 + lane * 16;
      const int r = o / WLS, col_b = o - r * WLS;
      const int8_t *src = sl.Wp2;
      if (r < wp_rows && col_b < a.npadp) {
        const int pt = r / prow;
        src = sl.Wp2 + ((size_t)(member + pt * GS) * 32 + (r - pt * prow)) * a.npadp + col_b;
      }
      dma(src, WpL + c * 1024);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }

  constexpr int TILE_KB = (32 * LS + 1023) / 1024;
  constexpr int NCH = (TILE_KB + 3) / 4;  // chunks per wave

  int32_t bpr[4] = {0, 0, 0, 0};
  if (my_ptiles > 0) {
    const int4 b4 = *reinterpret_cast<const int4 *>(sl.bp2 + member * 32 + 8 * (tid >> 6) + 4 * ((tid & 63) >> 5));
    bpr[0] = b4.x; bpr[1] = b4.y; bpr[2] = b4.z; bpr[3] = b4.w;
  }
  if (tid < items) red[tid] = 0;
  if (tid < 12) tickL[tid] = 0;
  if (tid == 0) {
    flag[0] = 1;
    flag[1] = 0;
  }
  __syncthreads();

  // optional phase timing (diagnostics): workgroup 0 of one layer, 100 MHz wall clock ticks per phase
  long long tick_last = 0;
  const bool timing = a.ticks && layer == sa.tick_layer && member == 0 && tid == 0;
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
  if (timing) tick_last = (long long)wall_clock64();

  unsigned epoch = 0;
  unsigned *counter = a.counters + layer * 64;
  u64 *accS = a.acc + (size_t)layer * kStatGroupWords;  // [set][round][S1|S2][item]
  // The layer's counter and statistics words were cleared by another kernel: a first access would fetch
  // them from memory in the middle of the first step.  Adding zero brings them into this XCD's L2 now,
  // while the layers below are still at work.
  if (tid < items) {
#pragma unroll
    for (int ss = 0; ss < 2; ++ss) {
      u64 *w = accS + ss * kStatSetWords;
      __hip_atomic_fetch_add(&w[0 * 256 + tid], (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(&w[1 * 256 + tid], (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ph) {
        __hip_atomic_fetch_add(&w[2 * 256 + tid], (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&w[3 * 256 + tid], (u64)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  if (tid == 0) __hip_atomic_fetch_add(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  int64_t prevS[2][2][2] = {{{0, 0}, {0, 0}}, {{0, 0}, {0, 0}}};  // this thread's item, per round and set: S1, S2
  const double inv_n = 1.0 / (double)a.N;
  const int g_first = cifg ? 1 : 0;
  const bool pre_ln = ln && (sl.rln[0] < 33 || sl.rln[1] < 33 || sl.rln[2] < 33 || sl.rln[3] < 33);
  const bool pre_m = sl.rm < 33;
  constexpr int32_t glo = ln ? -32767 : -32768;
  const int RTILES = sa.row_tiles;
  const int n_items = a.T * RTILES;
  const int pre_h = sl.pre_h, pre_x = sl.pre_x;

  // the tile of 32 rows starting at row0 of a [.., ld] buffer -> LDS; bytes of a row beyond `width`, the
  // row padding and the spare chunk read offset 0 of the buffer (they only ever meet zero weights or are
  // not used); BYPASS = the loads pass the L2 by (rows written by another XCD during this launch)
  auto tile_to_lds = [&](const int8_t *base, int ld, int width, int row0, auto bypass_tag) {
    constexpr int AUX = decltype(bypass_tag)::value ? 16 : 0;  // sc1
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int o = (wave + 4 * j) * 1024 + lane * 16;
      const int r = o / LS, c = o - r * LS;
      int row = row0 + r;
      row = row < a.B ? row : a.B - 1;
      const size_t off = (r < 32 && c < width) ? (size_t)row * ld + c : 0;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void *)(base + off),
          (__attribute__((address_space(3))) void *)(lds + (wave + 4 * j < TILE_KB ? wave + 4 * j : TILE_KB) * 1024), 16,
          0, AUX);
    }
  };

  int32_t creg[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
  for (int it = 0; it < n_items; ++it) {
    const int t = it / RTILES, rtile = it - t * RTILES;
    const int row0 = rtile * 32;
    const int row = row0 + col;

    // ---- cell state of this lane's 8 cells: in registers from step to step when the batch is one row
    // tile, in memory between the items of a row tile otherwise
    if (t == 0 || RTILES > 1) {
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int n0 = member * 64 + cell_w + tl * 8;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          creg[tl][c] = ((t > 0 || sa.c_given) && row < a.B && n0 + c < a.N) ? cbuf[(size_t)row * a.N + n0 + c] : 0;
      }
    }

    // ---- h^{t-1} rows of the tile -> LDS; R h on the MFMA; kept as packed int16 terms
    {
      const int8_t *hp = t == 0 ? h0 : out + (size_t)(t - 1) * a.B * a.Hpad;
      tile_to_lds(hp, a.Hpad, a.Hpad, row0, std::false_type{});
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    TICK(0);
    // The first part of this wave's slice of W (two tiles of kx fragments of 1 KB, contiguous) is asked for
    // ahead of its use, one word per 128-byte line, so that it is on its way into the L2 while R h runs and
    // the input is waited for.  Not all of it: a layer's W can be larger than the XCD's L2, and the last
    // lines would push the first out again before they are used (measured on the 8-layer benchmark stack:
    // about half of W ahead is best, all of it is as slow as none).
    constexpr int NPF = (KS * 16 + 63) / 64;
    unsigned pf[NPF];
    {
      const int8_t *w0 = sl.W2f + ((size_t)(member * 8 + wave * 2) * kx) * 1024;
#pragma unroll
      for (int i = 0; i < NPF; ++i) {
        const int line = lane + 64 * i;
        pf[i] = (line < sa.prefetch_lines && !ONE) ? *reinterpret_cast<const unsigned *>(w0 + (size_t)line * 128) : 0u;
      }
    }
    int32_t thp[2][8];  // [tile][(4 gate + c) / 2]: low half = even index
    {
      v16i acc[2];
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tl][v] = bhL[(v >> 2) * 64 + cell_w + tl * 8 + (v & 3)];
      constexpr int DEPTH = 4;
      v4i hf[DEPTH];
      const int8_t *hbase = hT + (size_t)col * LS + (b2 << 4);
#pragma unroll
      for (int ks = 0; ks < DEPTH && ks < KS; ++ks) hf[ks] = *reinterpret_cast<const v4i *>(hbase + ks * 32);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int tl = 0; tl < 2; ++tl)
          acc[tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Wf[tl][ks], hf[ks % DEPTH], acc[tl], 0, 0, 0);
        if (ks + DEPTH < KS) hf[ks % DEPTH] = *reinterpret_cast<const v4i *>(hbase + (ks + DEPTH) * 32);
        __builtin_amdgcn_sched_barrier(0);
      }
      auto pack = [&](auto pre_tag) {
        constexpr int PRE = decltype(pre_tag)::value;
#pragma unroll
        for (int tl = 0; tl < 2; ++tl)
#pragma unroll
          for (int j = 0; j < 8; ++j)
            thp[tl][j] = stk_requant2<PRE>(acc[tl][2 * j], acc[tl][2 * j + 1], prm->h[(2 * j) >> 2]);
      };
      if (pre_h == 0)
        pack(std::integral_constant<int, 0>{});
      else if (pre_h == 1)
        pack(std::integral_constant<int, 1>{});
      else
        pack(std::integral_constant<int, 2>{});
    }
    // A launch of one item per layer (one step, one row tile -- the streaming call) has no further use for
    // R: W takes its place in the registers while the layers below are still at work, and W x below runs
    // from registers instead of waiting for memory.
    constexpr bool w_resident = ONE;
    if (w_resident) {
      const int8_t *wsrc = sl.W2f + ((size_t)(member * 8 + wave * 2) * kx) * 1024 + (lane << 4);
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        int4 w[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          w[ks] = *reinterpret_cast<const int4 *>(wsrc + ((size_t)tl * kx + (ks < kx ? ks : 0)) * 1024);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          Wf[tl][ks] = v4i{w[ks].x, w[ks].y, w[ks].z, w[ks].w};
          asm volatile("" : "+a"(Wf[tl][ks]));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    TICK(1);

    // ---- W x^t: weights streamed from memory as MFMA operands, DW k steps ahead per tile
    constexpr int DW = 6;
    v4i wq[2][DW];
    const int8_t *wbase = sl.W2f + ((size_t)(member * 8 + wave * 2) * kx) * 1024 + (lane << 4);
    auto wload = [&](int tl, int ks) -> v4i {
      return *reinterpret_cast<const v4i *>(wbase + ((size_t)tl * kx + ks) * 1024);
    };
#pragma unroll
    for (int ks = 0; ks < DW && ks < KS; ++ks)
      if (ks < kx && !w_resident) {
        wq[0][ks] = wload(0, ks);
        wq[1][ks] = wload(1, ks);
      }
    // the input rows: wait until the layer below has finished step t of this row tile
    if (layer > 0) {
      if (tid == 0) {
        const unsigned *f = sa.flags + ((size_t)(layer - 1) * RTILES + rtile) * 32;
        int budget = a.spin_limit;
        for (;;) {
          const unsigned v = __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if ((int)(v - (unsigned)(t + 1)) >= 0) break;
          if (--budget <= 0 || __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
            __hip_atomic_store(a.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            flag[0] = 0;
            break;
          }
          for (int i = 0; i < sa.flag_sleep; ++i) __builtin_amdgcn_s_sleep(1);
        }
      }
    }
    __syncthreads();  // also: every wave has read its h fragments, the tile can be overwritten
    if (flag[0] == 0) return;
    TICK(2);
    {
      const int8_t *xp = xin + (size_t)t * a.B * ldx;
      if (x_bypass)
        tile_to_lds(xp, ldx, kx * 32, row0, std::true_type{});
      else
        tile_to_lds(xp, ldx, kx * 32, row0, std::false_type{});
      // the x chunks are the youngest NCH loads of this wave; the weight loads ahead of them are done then too
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < NPF; ++i) asm volatile("" ::"v"(pf[i]));  // the prefetched words themselves are not used
    }
    __syncthreads();
    TICK(3);
    v16i acc[2];
#pragma unroll
    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tl][v] = bxL[(wave * 2 + tl) * 32 + (v >> 2) * 8 + 4 * b2 + (v & 3)];
    {
      constexpr int DEPTH = 4;
      v4i xf[DEPTH];
      const int8_t *xbase = hT + (size_t)col * LS + (b2 << 4);
#pragma unroll
      for (int ks = 0; ks < DEPTH && ks < KS; ++ks) xf[ks] = *reinterpret_cast<const v4i *>(xbase + ks * 32);
      __builtin_amdgcn_sched_barrier(0);
      if (w_resident) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if (ks < kx) {  // uniform
#pragma unroll
            for (int tl = 0; tl < 2; ++tl)
              acc[tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Wf[tl][ks], xf[ks % DEPTH], acc[tl], 0, 0, 0);
            if (ks + DEPTH < KS) xf[ks % DEPTH] = *reinterpret_cast<const v4i *>(xbase + (ks + DEPTH) * 32);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          if (ks < kx) {  // uniform
#pragma unroll
            for (int tl = 0; tl < 2; ++tl)
              acc[tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wq[tl][ks % DW], xf[ks % DEPTH], acc[tl], 0, 0, 0);
            if (ks + DW < KS && ks + DW < kx) {
              wq[0][ks % DW] = wload(0, ks + DW);
              wq[1][ks % DW] = wload(1, ks + DW);
            }
            if (ks + DEPTH < KS) xf[ks % DEPTH] = *reinterpret_cast<const v4i *>(xbase + (ks + DEPTH) * 32);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }

    TICK(4);
    // ---- gate sums (Secs. 3.2.4/3.2.5) and layer-norm partial statistics
    auto gate_sums = [&](auto pre_tag) {
      constexpr int PRE = decltype(pre_tag)::value;
      int32_t s1[4] = {0, 0, 0, 0};
      uint32_t s2[4][2] = {{0, 0}, {0, 0}, {0, 0}, {0, 0}};
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const RescaleHi pg = prm->x[g];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int idx = g * 4 + c;
            const int32_t tx = rescale_sat16_pre<PRE>(acc[tl][idx], pg);
            const int32_t w = thp[tl][idx >> 1];
            const int32_t th = (idx & 1) ? (w >> 16) : (int32_t)(int16_t)(w & 0xFFFF);
            int32_t v = tx + th;
            if (ph && g < 2) {
              const int cl = cell_w + tl * 8 + c;
              v += rescale_sat16_pre((int32_t)PqL[g * 64 + cl] * creg[tl][c], prm->c[g]);
            }
            if (!(ph && g == 3)) v = clamp_i32(v, glo, 32767);
            acc[tl][idx] = v;
            s1[g] += v;
            s2[g][tl] += (uint32_t)v * (uint32_t)v;
          }
        }
      }
      if (ln) {
#pragma unroll
        for (int g = 0; g < (ph ? 3 : 4); ++g) {
          const int64_t pk = ((int64_t)((u64)s2[g][0] + (u64)s2[g][1]) << 24) + s1[g];
          __hip_atomic_fetch_add(&red[g * 32 + col], (u64)pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
    };
    if (pre_x == 0)
      gate_sums(std::integral_constant<int, 0>{});
    else if (pre_x == 1)
      gate_sums(std::integral_constant<int, 1>{});
    else
      gate_sums(std::integral_constant<int, 2>{});

    // statistics exchange among the layer's workgroups: rec_kernel's words (never reset, the top byte
    // counts the adds); `it` counts the exchanges of this launch
    constexpr u64 kValMask = ((u64)1 << 56) - 1;
    auto publish_stats = [&](int round, int g_lo, int g_hi) {
      __syncthreads();
      if (tid < items) {
        const int g = (tid >> 5) & 3;
        if (g >= g_lo && g <= g_hi) {
          const int64_t pk = (int64_t)red[tid];
          red[tid] = 0;
          const int64_t v1 = ((pk + (1 << 23)) & 0xFFFFFF) - (1 << 23);
          const int64_t v2 = (pk - v1) >> 24;
          u64 *mine = accS + (stat_two_sets(GS) ? (member & 1) : 0) * kStatSetWords;  // this workgroup's set of words
          __hip_atomic_fetch_add(&mine[(round * 2 + 0) * 256 + tid], ((u64)1 << 56) + (u64)(v1 + (1 << 22)),
                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_add(&mine[(round * 2 + 1) * 256 + tid], ((u64)1 << 56) + (u64)v2, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    };
    auto collect_stats = [&](int round, int g_lo, int g_hi) -> bool {
      if (tid < items) {
        const int g = (tid >> 5) & 3;
        if (g >= g_lo && g <= g_hi) {
          // two sets: set 0 holds the adds of the even members, set 1 those of the odd ones
          const bool two = stat_two_sets(GS);
          const unsigned n0 = two ? ((unsigned)GS + 1) >> 1 : (unsigned)GS, n1 = two ? (unsigned)GS >> 1 : 0u;
          const u64 expect0 = (u64)((n0 * (unsigned)(it + 1)) & 0xFFu), expect1 = (u64)((n1 * (unsigned)(it + 1)) & 0xFFu);
          u64 c1[2], c2[2];
          int budget = a.spin_limit;
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
            if (--budget <= 0 || __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
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
    TICK(5);
    if (ln) {
      publish_stats(0, g_first, ph ? 2 : 3);
      if (!collect_stats(0, g_first, ph ? 2 : 3)) return;
    }
    TICK(6);

    // ---- layer norm, sigma/tanh, cell update (Secs. 3.2.6, 3.2.1, 3.2.9, 3.2.7)
    constexpr int LNB = KS >= 32 ? 1 : 2;
    auto normalize = [&](int tl, int gmask, const LnRow2 (&lr)[4], int32_t (&xv)[4][4], bool narrow) {
      if (ln) {
#pragma unroll
        for (int gp = 0; gp < 4; gp += LNB) {
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
                xv[g][c] = narrow ? ln_second_stage_narrow(acc[tl][g * 4 + c], lr[g], wL[g - gp][c], wb[g - gp][c])
                                  : ln_second_stage(acc[tl][g * 4 + c], lr[g], wL[g - gp][c], wb[g - gp][c]);
          if (pre_ln) {
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
            for (int c = 0; c < 4; ++c) xv[g][c] = acc[tl][g * 4 + c];
      }
    };
    // table values of |xv[g][c]| for the gates of gmask; tb[g] = which table (0 sigma, 1 tanh, 2 cell tanh);
    // see rec_kernel's lookup
    auto lookup = [&](int gmask, const int32_t (&xv)[4][4], const int (&tb)[4], int32_t (&tv)[4][4]) {
      int32_t mag[4][4];
      uint32_t base[4][4], delta[4][4];
      int32_t top[3] = {0, 0, 0};  // largest |x| looked up in each table
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
            mag[g][c] = abs_i32(xv[g][c]);
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
    constexpr int gates_now = (cifg ? 0 : 1) | 2 | 4 | (ph ? 0 : 8);
    int32_t xi[2][4], xf_[2][4], xz[2][4], xo[2][4];
    {
      LnRow2 lr[4];
      bool narrow = false;  // uniform: every row of this wave has sigma >= 2^12 (see rec_kernel)
      if (ln) {
        bool wide = false;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          lr[g] = lnrow[g * 32 + col];
          if (gates_now >> g & 1) wide |= !ln_row_is_narrow(lr[g]);
        }
        narrow = __builtin_amdgcn_ballot_w64(wide) == 0;
      }
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        int32_t xv[4][4], tv[4][4];
        if (narrow)
          normalize(tl, gates_now, lr, xv, true);
        else
          normalize(tl, gates_now, lr, xv, false);
        if (KS >= 32) {
          lookup(gates_now & 3, xv, gate_tb, tv);
          lookup(gates_now & 12, xv, gate_tb, tv);
        } else {
          lookup(gates_now, xv, gate_tb, tv);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          xi[tl][c] = cifg ? 0 : mirror_sigmoid(xv[0][c], tv[0][c]);
          xf_[tl][c] = mirror_sigmoid(xv[1][c], tv[1][c]);
          xz[tl][c] = mirror_tanh(xv[2][c], tv[2][c]);
          xo[tl][c] = ph ? 0 : mirror_sigmoid(xv[3][c], tv[3][c]);
        }
      }
    }
    const int32_t m_c = prm->m_c;
    {
      int32_t s1 = 0;
      int64_t s2 = 0;
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int32_t f = xf_[tl][c];
          const int32_t i = cifg ? cifg_input_gate(f) : xi[tl][c];
          const int32_t cnew = cell_update32(i, xz[tl][c], f, creg[tl][c], m_c);
          creg[tl][c] = cnew;
          if (ph) {  // finish the o gate sum with P_o . c^t (eq. 5)
            const int cl = cell_w + tl * 8 + c;
            int32_t v = acc[tl][12 + c] + rescale_sat16_pre((int32_t)PqL[2 * 64 + cl] * cnew, prm->c[2]);
            v = clamp_i32(v, glo, 32767);
            acc[tl][12 + c] = v;
            s1 += v;
            s2 += (int64_t)v * v;
          }
        }
      if (ph && ln) {
        const int64_t pk = (s2 << 24) + s1;
        __hip_atomic_fetch_add(&red[3 * 32 + col], (u64)pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
    // the new cell state goes back to memory: read again by this thread at the tile's next step, or, after
    // the last step, the state the caller gets back
    if (RTILES > 1 || t == a.T - 1) {
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        const int n0 = member * 64 + cell_w + tl * 8;
        if (row < a.B && n0 < a.N)
#pragma unroll
          for (int c = 0; c < 4; ++c) cbuf[(size_t)row * a.N + n0 + c] = (int16_t)creg[tl][c];
      }
    }
    TICK(7);
    if (ph && ln) {
      publish_stats(1, 3, 3);
      if (!collect_stats(1, 3, 3)) return;
    }

    // ---- hidden state (Sec. 3.2.7)
    int32_t tc[2][4];
    {
      const int hid_tb[4] = {2, 2, 0, 0};
      LnRow2 lr[4];
      if (ph && ln) lr[3] = lnrow[3 * 32 + col];
      int32_t xv[4][4], tv[4][4], ov[2][4][4];
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
#pragma unroll
        for (int c = 0; c < 4; ++c) xv[tl][c] = creg[tl][c];
        if (ph) {
          normalize(tl, 8, lr, ov[tl], false);
#pragma unroll
          for (int c = 0; c < 4; ++c) xv[2 + tl][c] = ov[tl][3][c];
        }
      }
      lookup(ph ? 15 : 3, xv, hid_tb, tv);
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          tc[tl][c] = mirror_tanh(xv[tl][c], tv[tl][c]);
          if (ph) xo[tl][c] = mirror_sigmoid(xv[2 + tl][c], tv[2 + tl][c]);
        }
    }
    // Without a projection m is the layer output h: it goes to [T, B, Hpad] with stores that write through
    // the L2 (the next layer's XCD reads it).  With one it goes to the exchange buffer of this XCD.
    int8_t *mdst = proj ? mbuf + (size_t)t * a.Bp * a.npadp : out + (size_t)t * a.B * a.Hpad;
    const RescaleHi pm = prm->m;
    const int32_t zp_m = prm->zp_m;
    const bool final_step = t == a.T - 1;
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
      const int n0 = member * 64 + cell_w + tl * 8;
      uint32_t pk = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int32_t om = xo[tl][c] * tc[tl][c];
        if (pre_m) om = rescale_preshift(om, pm);
        const int32_t mq = sat8(rescale_sat16_pre<0>(om, pm) + zp_m);
        pk |= (uint32_t)(mq & 0xFF) << (8 * c);
      }
      if (row < a.B && n0 < a.N) {
        if (proj) {
          const size_t off = (((size_t)(row >> 5) * (a.npadp >> 5) + (n0 >> 5)) * 32 + (row & 31)) * 32 + (n0 & 31);
          *reinterpret_cast<uint32_t *>(mdst + off) = pk;
        } else {
          __hip_atomic_store(reinterpret_cast<uint32_t *>(mdst + (size_t)row * a.Hpad + n0), pk, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
          if (yout)
            __builtin_nontemporal_store(pk, reinterpret_cast<uint32_t *>(yout + ((size_t)t * a.B + row) * a.H + n0));
          if (final_step && hfin) *reinterpret_cast<uint32_t *>(hfin + (size_t)row * a.H + n0) = pk;
        }
      }
    }
    TICK(8);
    if (!group_sync(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, a.sync_sleep, a.poll_sleep, flag)) return;
    TICK(9);

    // ---- projection (Sec. 3.2.8)
    if (proj) {
      const int per_wave = a.npadp >> 7;
      const RescaleHi pp = prm->p;
      const int32_t zp_h = prm->zp_h;
      for (int pt = 0; pt < my_ptiles; ++pt) {
        const int ptile = member + pt * GS;
        const int8_t *mrow = mbuf + (size_t)t * a.Bp * a.npadp +
                             ((((size_t)(row0 >> 5) * (a.npadp >> 5) + wave * per_wave) * 32 + col) << 5) + (b2 << 4);
        const int8_t *wrow = WpL + ((size_t)pt * a.prow + (col < a.prow ? col : 0)) * WLS + (b2 << 4) + wave * per_wave * 32;
        int4 mv[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          const int kk = k < per_wave ? k : per_wave - 1;
          mv[k] = *reinterpret_cast<const int4 *>(mrow + kk * 1024);
        }
        v16i pacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) pacc[v] = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          const int kk = k < per_wave ? k : per_wave - 1;
          v4i wf = *reinterpret_cast<const v4i *>(wrow + kk * 32);
          if (k >= per_wave) wf = v4i{0, 0, 0, 0};
          pacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, v4i{mv[k].x, mv[k].y, mv[k].z, mv[k].w}, pacc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) pred[(wave * 16 + v) * 64 + lane] = pacc[v];
        __syncthreads();
        {
          const int q = tid >> 6, l2 = tid & 63;
          const int pl = 8 * q + 4 * (l2 >> 5);  // row of the tile; prow is a multiple of 4
          const int p0 = ptile * a.prow + pl;
          const int orow = row0 + (l2 & 31);
          uint32_t pk = 0;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int v = 4 * q + c;
            const int32_t s = pred[(0 * 16 + v) * 64 + l2] + pred[(1 * 16 + v) * 64 + l2] +
                              pred[(2 * 16 + v) * 64 + l2] + pred[(3 * 16 + v) * 64 + l2] +
                              (pt == 0 ? bpr[c] : sl.bp2[ptile * 32 + pl + c]);
            const int32_t hq = sat8(rescale_sat16_pre(s, pp) + zp_h);
            pk |= (uint32_t)(hq & 0xFF) << (8 * c);
          }
          if (orow < a.B && p0 < a.H && pl < a.prow) {
            int8_t *od = out + ((size_t)t * a.B + orow) * a.Hpad + p0;
            if (p0 + 3 < a.H) {
              __hip_atomic_store(reinterpret_cast<uint32_t *>(od), pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
              for (int c = 0; c < 4 && p0 + c < a.H; ++c)
                __hip_atomic_store(od + c, (int8_t)(pk >> (8 * c)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (yout) {
              int8_t *yd = yout + ((size_t)t * a.B + orow) * a.H + p0;
              for (int c = 0; c < 4 && p0 + c < a.H; ++c) yd[c] = (int8_t)(pk >> (8 * c));
            }
            if (final_step && hfin) {
              int8_t *hd = hfin + (size_t)orow * a.H + p0;
              for (int c = 0; c < 4 && p0 + c < a.H; ++c) hd[c] = (int8_t)(pk >> (8 * c));
            }
          }
        }
        __syncthreads();
      }
      TICK(10);
      if (!group_sync(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, my_ptiles == 0 ? a.idle_sleep : 0,
                      my_ptiles == 0 ? a.idle_poll_sleep : a.poll_sleep, flag))
        return;
      TICK(11);
    }
    // every workgroup of the layer is past its stores of step t (and they are acknowledged): tell the
    // layer above
    if (!last_layer && member == 0 && tid == 0)
      __hip_atomic_store(sa.flags + ((size_t)layer * RTILES + rtile) * 32, (unsigned)(t + 1), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  }
#undef TICK
  if (timing)
    for (int i = 0; i < 12; ++i) a.ticks[i] += (long long)tickL[i];
  placement_check();
}

typedef void (*stack_fn)(StackArgs);

}  // namespace lstm_int
