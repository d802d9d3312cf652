// Persistent recurrent kernel for small batches: groups of 16 batch rows on
// the 16x16x64 int8 MFMA (rec_kernel.inc.h has the design; this is the same
// step with half the rows per workgroup, so that 128 rows already fill the
// chip and a workgroup's arithmetic per step is half as long).  FL: bit 0 CIFG,
// bit 1 peephole, bit 2 layer norm; the projection is a runtime flag.
//
// Lane (r = lane % 16, q = lane / 16) of wave w owns batch row r of the group
// and cells 16 w + 4 q + c, c = 0..3, of the workgroup's 64, all four gates:
// weight tile j of the wave holds, in row 4 q' + gate, cell 16 w + 4 q' + j,
// so that result value `gate` of tile j in that lane is (cell 4 q + j, gate).
// The W x terms are read in the layout the input GEMM writes for the 32-row
// kernel (two 16-byte loads per lane and step).
#pragma once

#include "rec_kernel.inc.h"

namespace lstm_int {

// 100 MHz wall clock ticks per phase, summed in LDS by thread 0 of workgroup 0
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

template <int KS16, int FL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void rec16_kernel(RecArgs a) {
  constexpr bool cifg = FL & 1, ph = FL & 2, ln = FL & 4;
  const long long t_start = (long long)wall_clock64();
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, q = lane >> 4;
  const bool proj = a.flags & 8;
  constexpr int g_first = cifg ? 1 : 0;
  const int GS = a.GS;

  // placement, as in rec_kernel
  const int wg = blockIdx.x;
  const int xcc = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7);
  const int slot = wg >> 3;
  int xcd = wg & 7;
  if (a.tickets) {
    xcd = xcc;
  } else if (xcc != xcd && GS > 1 && tid == 0) {
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
  const int group = xcd + 8 * (slot / GS), member = slot % GS;
  if (group >= a.groups) {
    placement_check();
    return;
  }
  constexpr int items = 64;                    // (gate, row) layer-norm rows of the group
  const int row0 = a.batch0 + group * 16;      // first batch row of the group
  const int cellw = wave * 16 + 4 * q;         // + c, within the workgroup's 64 cells

  // ---- LDS carve-up (rec16_lds_bytes mirrors it)
  constexpr int LS = KS16 * 64 + 16;  // h tile row stride: LS / 4 = 4 * odd (mod 64), reads are conflict-free
  constexpr int TILE_KB = (16 * LS + 1023) / 1024;
  uint8_t *p = lds;
  int8_t *hT = reinterpret_cast<int8_t *>(p);
  int32_t *pred = reinterpret_cast<int32_t *>(p);  // projection partials reuse the h tile between steps
  {
    const size_t tile_bytes = (size_t)(TILE_KB + 1) * 1024;  // one spare chunk for the loads past the tile
    const size_t pred_bytes = proj ? 4 * 2 * 4 * 64 * 4 : 0;
    p += tile_bytes > pred_bytes ? tile_bytes : pred_bytes;
  }
  u64 *red = reinterpret_cast<u64 *>(p);                 p += (size_t)items * 8;  // [item] sums
  LnRow2 *lnrow = reinterpret_cast<LnRow2 *>(p);         p += (size_t)items * sizeof(LnRow2);
  double *LdL = reinterpret_cast<double *>(p);           p += 4 * 64 * 8;
  double *bdL = reinterpret_cast<double *>(p);           p += 4 * 64 * 8;
  int32_t *bhL = reinterpret_cast<int32_t *>(p);         p += 4 * 64 * 4;
  int16_t *PqL = reinterpret_cast<int16_t *>(p);         p += 4 * 64 * 2;  // 3 used
  PrmLds *prm = reinterpret_cast<PrmLds *>(p);           p += sizeof(PrmLds);
  int *flag = reinterpret_cast<int *>(p);                p += 16;
  u64 *tickL = reinterpret_cast<u64 *>(p);               p += 16 * 8;  // phase timers
  LutLds *lutP = reinterpret_cast<LutLds *>(p);          p += 3 * sizeof(LutLds);
  // the activation tables as in rec_kernel: prefixes of the wide form, chosen by the launch
  const bool share_tanh = a.lut[2].blob == a.lut[1].blob;
  const uint8_t *lutD[3];
  const uint8_t *lutB[3];
  const uint8_t *lutTl[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    if (i == 2 && share_tanh) {
      lutD[2] = lutD[1]; lutB[2] = lutB[1]; lutTl[2] = lutTl[1];
    } else {
      const int nb = ((((a.lut[i].dom >> a.lut[i].sh) * 2) + 1023) >> 10) << 10;
      lutD[i] = p;                               p += a.lut[i].dom;
      lutB[i] = p;                               p += nb;
      lutTl[i] = a.lut[i].tail ? p : nullptr;    p += a.lut[i].tail ? 3072 : 0;
    }
  }
  int8_t *WpL = reinterpret_cast<int8_t *>(p);
  const int WLS = a.npadp + 16;  // W_proj tile row stride in LDS
  const int my_ptiles = proj ? (a.ptiles > member ? (a.ptiles - member + GS - 1) / GS : 0) : 0;

  // ---- one-time loads: R slice -> registers, per-cell parameters, tables and W_proj tiles -> LDS
  // the loads into LDS go first: they need no registers and are in flight while the R slice arrives
  {
    auto dma = [&](const void *src, const void *dst) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                       (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
    };
    for (int i = 0; i < (share_tanh ? 2 : 3); ++i) {
      const int nd = a.lut[i].dom >> 10;
      const int nb = (((a.lut[i].dom >> a.lut[i].sh) * 2) + 1023) >> 10;
      const int nt = a.lut[i].tail ? 3 : 0;
      for (int c = wave; c < nd + nb + nt; c += 4) {
        const int so = c < nd ? c * 1024 : (c < nd + nb ? kLutWideBaseOff + (c - nd) * 1024 : kLutWideTailOff + (c - nd - nb) * 1024);
        dma(a.lut[i].blob + so + lane * 16, lutD[i] + c * 1024);
      }
    }
    if (tid < 3) {
      LutLds d;
      d.dom = a.lut[tid].dom; d.sh = a.lut[tid].sh;
      d.offD = (int32_t)(lutD[tid] - lds);
      d.offB = (int32_t)(lutB[tid] - lds);
      d.offT = lutTl[tid] ? (int32_t)(lutTl[tid] - lds) : 0;
      d.pad[0] = d.pad[1] = d.pad[2] = 0;
      lutP[tid] = d;
    }
    const int wp_rows = my_ptiles * 32;
    const int wp_chunks = (wp_rows * WLS + 1023) >> 10;
    for (int c = wave; c < wp_chunks; c += 4) {
      const int o = c * 1024 + lane * 16;
      const int rr = o / WLS, col_b = o - rr * WLS;
      const int8_t *src = a.Wp2;
      if (rr < wp_rows && col_b < a.npadp) {
        const int pt = rr >> 5;
        src = a.Wp2 + ((size_t)(member + pt * GS) * 32 + (rr & 31)) * a.npadp + col_b;
      }
      dma(src, WpL + c * 1024);
    }
  }
  v4i Wf[4][KS16];
  {
    const int4 *src = a.R2h + ((size_t)(member * 4 + wave) * 4) * KS16 * 64 + lane;
    // all loads of the slice are issued before the first value is pinned (a pin waits for its load);
    // at the deepest k the staging registers do not hold four tiles, so two at a time
    constexpr int TB = KS16 <= 10 ? 4 : 2;
#pragma unroll
    for (int j0 = 0; j0 < 4; j0 += TB) {
      int4 w[TB][KS16];
#pragma unroll
      for (int j = 0; j < TB; ++j)
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) w[j][ks] = src[(size_t)((j0 + j) * KS16 + ks) * 64];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < TB; ++j)
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
          Wf[j0 + j][ks] = v4i{w[j][ks].x, w[j][ks].y, w[j][ks].z, w[j][ks].w};
          asm volatile("" : "+a"(Wf[j0 + j][ks]));  // resident in accumulation registers for the whole launch
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  {
    const int g = tid >> 6, n = tid & 63;  // 256 threads = 4 gates x 64 cells
    const size_t idx = (size_t)g * a.Ncp + member * 64 + n;
    LdL[tid] = ln_weight_scaled(a.Lq4[idx]);
    bdL[tid] = ln_bias_scaled(a.qb4[idx]);
    bhL[tid] = a.bh4[idx];
    PqL[tid] = (ph && g < 3) ? a.Pq3[idx] : 0;
  }
  if (tid < 4) {
    prm->h[tid] = rescale_hi_prepare(a.Mh[tid], a.rh[tid]);
    prm->c[tid] = rescale_hi_prepare(tid < 3 && ph ? a.Mc[tid] : 0, tid < 3 && ph ? a.rc[tid] : 33);
    prm->ln[tid] = rescale_hi_prepare(a.Mln[tid], a.rln[tid]);
  }
  if (tid == 0) {
    prm->m = rescale_hi_prepare(a.Mm, a.rm);
    prm->p = rescale_hi_prepare(proj ? a.Mp : 0, proj ? a.rp : 33);
    prm->zp_m = a.zp_m; prm->zp_h = a.zp_h;
    prm->m_c = a.m_c; prm->glo = -32767;
  }
  for (int i = tid; i < 16 * LS / 16; i += 256) reinterpret_cast<int4 *>(hT)[i] = int4{0, 0, 0, 0};

  // cell state of this lane's 4 cells of its row, kept in registers
  const int row = row0 + r;
  const int n0 = member * 64 + cellw;
  int32_t creg[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
    creg[c] = (a.c_in && row < a.B && n0 + c < a.N) ? a.c_in[(size_t)row * a.N + n0 + c] : 0;

  // h tile staging: wave instruction (wave + 4 j) fills bytes [1024 c, 1024 (c + 1)) of the tile
  constexpr int NCH = (TILE_KB + 3) / 4;
  int hsrc[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int o = (wave + 4 * j) * 1024 + lane * 16;
    const int rr = o / LS, c = o - rr * LS;
    int rw = row0 + rr;
    rw = rw < a.B ? rw : a.B - 1;
    hsrc[j] = (rr < 16 && c < a.Hpad) ? rw * a.Hpad + c : 0;
  }

  // projection: thread (ct = tid / 64 < 2, lane) finishes outputs 16 ct + 4 q + 0..3 of row r
  int32_t bpr[4] = {0, 0, 0, 0};
  if (my_ptiles > 0 && tid < 128) {
    const int4 b4 = *reinterpret_cast<const int4 *>(a.bp2 + member * 32 + 16 * wave + 4 * q);
    bpr[0] = b4.x; bpr[1] = b4.y; bpr[2] = b4.z; bpr[3] = b4.w;
  }
  if (tid == 0) {
    flag[0] = 1;
    flag[1] = 0;
  }
  if (tid < 16) tickL[tid] = 0;
  if (tid < items) red[tid] = 0;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // tables and W_proj tiles are in LDS
  __syncthreads();

  unsigned epoch = 0;
  unsigned *counter = a.counters + group * 64;
  // one set of words: two sets (as in rec_kernel) made this kernel 2-3 % slower, at 8 and at 32 workgroups per group
  u64 *accS = a.acc + (size_t)group * kStatGroupWords;  // [round][S1|S2][item], item < 64
  int64_t prevS[2][2] = {{0, 0}, {0, 0}};       // this thread's item, per round: S1, S2
  const double inv_n = 1.0 / (double)a.N;
  const bool pre_ln = a.rln[0] < 33 || a.rln[1] < 33 || a.rln[2] < 33 || a.rln[3] < 33;
  const bool pre_m = a.rm < 33;
  constexpr u64 kValMask = ((u64)1 << 56) - 1;

  // optional phase timing of workgroup 0 (diagnostics), phases numbered as in rec_kernel
  long long tick_last = 0;
  const bool timing = a.ticks && wg == 0 && tid == 0;
  if (timing) {
    tick_last = t_start;
    __hip_atomic_store(&a.ticks[15], t_start, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  TICK(10);  // everything before the first step

  // the two 16-byte W x pieces of this lane for step t, read in the layout of the 32-row kernel:
  // cell tile of 8 = 2 wave + q / 2, lane there = row % 32 + 32 * (q % 2)
  v4i txn0, txn1;
  auto tx_request = [&](int t) {
    size_t rb = ((size_t)t * a.Bp + row0) >> 5;
    const size_t rbmax = ((size_t)a.T * a.Bp) >> 5;
    rb = rb < rbmax ? rb : rbmax - 1;
    const int4 *src = a.tx2 + ((rb * (size_t)(GS * 8) + member * 8 + wave * 2 + (q >> 1)) * 2) * 64 +
                      ((row0 + r) & 31) + 32 * (q & 1);
    // read once: streaming loads keep the W x terms from displacing the exchange buffers in L2
    txn0 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(src));
    txn1 = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(src + 64));
  };
  tx_request(0);

  for (int t = 0; t < a.T; ++t) {
    // ---- h^{t-1} rows of the group -> LDS
    {
      const int8_t *hp = t == 0 ? a.h0 : a.out + (size_t)(t - 1) * a.B * a.Hpad;
#pragma unroll
      for (int j = 0; j < NCH; ++j)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(hp + hsrc[j]),
            (__attribute__((address_space(3))) void *)(lds + (wave + 4 * j < TILE_KB ? wave + 4 * j : TILE_KB) * 1024),
            16, 0, 0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    // the W x terms of this step were requested one step ahead (they come from HBM)
    const int32_t txw[8] = {txn0.x, txn0.y, txn0.z, txn0.w, txn1.x, txn1.y, txn1.z, txn1.w};
    TICK(0);

    // ---- R h on the MFMA: acc[j][gate] for cell 4 q + j; each tile's k loop runs to its end
    // before the next tile starts (dependent 16x16x64 MFMAs issue back to back, rotating
    // accumulators do not)
    v4i acc[4];
    RescaleHi ph4[4];  // the R h rescale constants, read here so that the MFMAs cover the LDS round trip
#pragma unroll
    for (int g = 0; g < 4; ++g) ph4[g] = prm->h[g];
    {
      v4i hf[KS16];
      const int8_t *hbase = hT + (size_t)r * LS + (q << 4);
#pragma unroll
      for (int ks = 0; ks < KS16; ++ks) hf[ks] = *reinterpret_cast<const v4i *>(hbase + ks * 64);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[j][g] = bhL[g * 64 + cellw + j];
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks)
          acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(Wf[j][ks], hf[ks], acc[j], 0, 0, 0);
      }
    }

    TICK(1);

    // ---- gate sums (Secs. 3.2.4/3.2.5) and layer-norm partial statistics.
    // With a peephole the o gate keeps tx + th here and is finished after c^t.
    constexpr int32_t glo = ln ? -32767 : -32768;  // layer norm takes symmetric gate sums
    int32_t gs[4][4];  // [gate][cell]
    auto gate_sums = [&](auto pre_tag) {
      constexpr int PRE = decltype(pre_tag)::value;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const RescaleHi pg = ph4[g];
        int32_t s1 = 0;
        uint32_t s2 = 0;  // four squares of 16-bit values fit 32 bits
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int idx = g * 4 + c;
          const int32_t th = rescale_sat16_pre<PRE>(acc[c][g], pg);
          const int32_t w = txw[idx >> 1];
          const int32_t tx = (idx & 1) ? (w >> 16) : (int32_t)(int16_t)(w & 0xFFFF);
          int32_t v = tx + th;
          if (ph && g < 2) v += rescale_sat16_pre((int32_t)PqL[g * 64 + cellw + c] * creg[c], prm->c[g]);
          if (!(ph && g == 3)) v = clamp_i32(v, glo, 32767);
          gs[g][c] = v;
          s1 += v;
          s2 += (uint32_t)v * (uint32_t)v;
        }
        if (ln && !(ph && g == 3)) {
          // the 16 lanes of a row (4 per wave) add into one LDS word: no cross-lane traffic, no wait
          const int64_t pk = ((int64_t)(u64)s2 << 24) + s1;
          __hip_atomic_fetch_add(&red[g * 16 + r], (u64)pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      }
    };
    if (a.pre_h == 0)
      gate_sums(std::integral_constant<int, 0>{});
    else if (a.pre_h == 1)
      gate_sums(std::integral_constant<int, 1>{});
    else
      gate_sums(std::integral_constant<int, 2>{});
    tx_request(t + 1);  // past the last step: the last block again, unused

    // statistics over the group's workgroups: as in rec_kernel (words that are never reset, the top
    // byte counts the adds); item = 16 gate + row
    auto publish_stats = [&](int round, int g_lo, int g_hi) {
      __syncthreads();
      if (tid < items) {
        const int g = tid >> 4;
        if (g >= g_lo && g <= g_hi) {
          const int64_t pk = (int64_t)red[tid];
          red[tid] = 0;  // the next adds to this word come after the next barrier
          const int64_t v1 = ((pk + (1 << 23)) & 0xFFFFFF) - (1 << 23);
          const int64_t v2 = (pk - v1) >> 24;
          __hip_atomic_fetch_add(&accS[(round * 2 + 0) * 256 + tid], ((u64)1 << 56) + (u64)(v1 + (1 << 22)),
                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_add(&accS[(round * 2 + 1) * 256 + tid], ((u64)1 << 56) + (u64)v2, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    };
    // false: a wait gave up (status word raised), every thread leaves the kernel
    auto collect_stats = [&](int round, int g_lo, int g_hi) -> bool {
      if (tid < items) {
        const int g = tid >> 4;
        if (g >= g_lo && g <= g_hi) {
          const u64 expect = (u64)(((unsigned)GS * (unsigned)(t + 1)) & 0xFFu);
          u64 c1, c2;
          int budget = a.spin_limit;
          for (int i = 0; i < a.stats_first_sleep; ++i) __builtin_amdgcn_s_sleep(1);
          for (;;) {
            c1 = __hip_atomic_load(&accS[(round * 2 + 0) * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c2 = __hip_atomic_load(&accS[(round * 2 + 1) * 256 + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((c1 >> 56) == expect && (c2 >> 56) == expect) break;
            if (--budget <= 0 || __hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
              __hip_atomic_store(a.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              *flag = 0;
              break;
            }
            for (int i = 0; i < a.stats_sleep; ++i) __builtin_amdgcn_s_sleep(1);
          }
          c1 &= kValMask;
          c2 &= kValMask;
          const int64_t S1 = (int64_t)((c1 - (u64)prevS[round][0]) & kValMask) - (int64_t)GS * (1 << 22);
          const int64_t S2 = (int64_t)((c2 - (u64)prevS[round][1]) & kValMask);
          prevS[round][0] = (int64_t)c1;
          prevS[round][1] = (int64_t)c2;
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

    // ---- layer norm, sigma/tanh, cell update (Secs. 3.2.6, 3.2.1, 3.2.9, 3.2.7); LDS reads in batches
    // gates of `gmask` (bit g): gate sums -> layer norm -> xv[g][c]
    auto normalize = [&](int gmask, int32_t (&xv)[4][4]) {
      if (ln) {
        LnRow2 lr[4];
        bool wide = false;
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if (gmask >> g & 1) {
            lr[g] = lnrow[g * 16 + r];
            wide |= !ln_row_is_narrow(lr[g]);
          }
        // uniform: every row of this wave has sigma >= 2^12, and the second stage needs no int32 clamp
        const bool narrow = __builtin_amdgcn_ballot_w64(wide) == 0;
        auto second_stage = [&](auto narrow_tag) {
#pragma unroll
        for (int gp = 0; gp < 4; gp += 2) {
          if (!(gmask >> gp & 3)) continue;
          double wL[2][4], wb[2][4];
          RescaleHi pl[2];
#pragma unroll
          for (int g = gp; g < gp + 2; ++g)
            if (gmask >> g & 1) {
              pl[g - gp] = prm->ln[g];
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                wL[g - gp][c] = LdL[g * 64 + cellw + c];
                wb[g - gp][c] = bdL[g * 64 + cellw + c];
              }
            }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int g = gp; g < gp + 2; ++g)
            if (gmask >> g & 1)
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                int32_t v = decltype(narrow_tag)::value ? ln_second_stage_narrow(gs[g][c], lr[g], wL[g - gp][c], wb[g - gp][c])
                                                        : ln_second_stage(gs[g][c], lr[g], wL[g - gp][c], wb[g - gp][c]);
                if (pre_ln) v = rescale_preshift(v, pl[g - gp]);
                xv[g][c] = rescale_sat16_pre<0>(v, pl[g - gp]);
              }
        }
        };
        if (narrow)
          second_stage(std::true_type{});
        else
          second_stage(std::false_type{});
      } else {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          if (gmask >> g & 1)
#pragma unroll
            for (int c = 0; c < 4; ++c) xv[g][c] = gs[g][c];
      }
    };
    // table values of |x[g][c]| for the gates of gmask; tb[g] = which table (0 sigma, 1 tanh, 2 cell tanh);
    // see rec_kernel's lookup
    auto lookup = [&](int gmask, const int32_t (&x)[4][4], const int (&tb)[4], int32_t (&out)[4][4]) {
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
            mag[g][c] = abs_i32(x[g][c]);
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
          for (int c = 0; c < 4; ++c) out[g][c] = (int32_t)(base[g][c] + delta[g][c]);
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
                if (mag[g][c] >= dom) out[g][c] = lut_wide_tail(lds + lp[tb[g]].offT, mag[g][c]);
            }
          }
      }
    };
    constexpr int gates_now = (cifg ? 0 : 1) | 2 | 4 | (ph ? 0 : 8);  // with a peephole the o gate waits for c^t
    int32_t xv[4][4], tv[4][4];
    normalize(gates_now, xv);
    {
      const int gate_tb[4] = {0, 0, 1, 0};
      lookup(gates_now, xv, gate_tb, tv);
    }
    const int32_t m_c = prm->m_c;
    int32_t xo[4];
    int32_t cx[4][4];  // slot 0: the new cell state, for its tanh; slot 3: the o gate with a peephole
    {
      int32_t s1 = 0;
      uint32_t s2 = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int32_t fg = mirror_sigmoid(xv[1][c], tv[1][c]);
        const int32_t ig = cifg ? cifg_input_gate(fg) : mirror_sigmoid(xv[0][c], tv[0][c]);
        const int32_t zg = mirror_tanh(xv[2][c], tv[2][c]);
        xo[c] = ph ? 0 : mirror_sigmoid(xv[3][c], tv[3][c]);
        creg[c] = cell_update32(ig, zg, fg, creg[c], m_c);
        cx[0][c] = creg[c];
        if (ph) {  // finish the o gate sum with P_o . c^t (eq. 5)
          int32_t v = gs[3][c] + rescale_sat16_pre((int32_t)PqL[2 * 64 + cellw + c] * creg[c], prm->c[2]);
          v = clamp_i32(v, glo, 32767);
          gs[3][c] = v;
          s1 += v;
          s2 += (uint32_t)v * (uint32_t)v;
        }
      }
      if (ph && ln) {
        const int64_t pk = ((int64_t)(u64)s2 << 24) + s1;
        __hip_atomic_fetch_add(&red[3 * 16 + r], (u64)pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
    TICK(5);
    // ---- hidden state (Sec. 3.2.7): tanh of the new cell state in its own format (Sec. 3.2.2), and
    // with a peephole the layer norm and sigma of the o gate; the tanh does not wait for the o gate's
    // statistics, so it runs while they travel
    int32_t tcv[4][4];
    const int hid_tb[4] = {2, 2, 2, 0};
    if (ph && ln) {
      publish_stats(1, 3, 3);
      lookup(1, cx, hid_tb, tcv);
      if (!collect_stats(1, 3, 3)) return;
    } else {
      lookup(1, cx, hid_tb, tcv);
    }
    if (ph) {
      int32_t ov[4][4];
      normalize(8, ov);
#pragma unroll
      for (int c = 0; c < 4; ++c) cx[3][c] = ov[3][c];
      lookup(8, cx, hid_tb, tcv);
#pragma unroll
      for (int c = 0; c < 4; ++c) xo[c] = mirror_sigmoid(cx[3][c], tcv[3][c]);
    }
    {
      const RescaleHi pm = prm->m;
      const int32_t zp_m = prm->zp_m;
      uint32_t pk = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int32_t om = xo[c] * mirror_tanh(cx[0][c], tcv[0][c]);
        if (pre_m) om = rescale_preshift(om, pm);
        const int32_t mq = sat8(rescale_sat16_pre<0>(om, pm) + zp_m);
        pk |= (uint32_t)(mq & 0xFF) << (8 * c);
      }
      if (row < a.B && n0 < a.N) {
        if (proj) {
          // exchange buffer [t][row / 16][k step of 64 cells = member][row % 16][64 cells]: a wave's
          // load of one projection k step is one contiguous KB
          int8_t *mdst = a.mbuf + (size_t)t * a.Bp * a.npadp +
                         ((((size_t)(row >> 4) * (a.npadp >> 6) + member) * 16 + (row & 15)) << 6) + cellw;
          *reinterpret_cast<uint32_t *>(mdst) = pk;
        } else {
          *reinterpret_cast<uint32_t *>(a.out + ((size_t)t * a.B + row) * a.Hpad + n0) = pk;
          if (a.y) __builtin_nontemporal_store(pk, reinterpret_cast<uint32_t *>(a.y + ((size_t)t * a.B + row) * a.H + n0));
        }
      }
    }
    TICK(6);
    if (!group_sync(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, a.sync_sleep, a.poll_sleep, flag)) return;
    TICK(7);

    // ---- projection (Sec. 3.2.8): tile pt of 32 outputs as two 16-wide halves, K = N split over the waves
    if (proj) {
      const int ksteps = a.npadp >> 6;
      const int per_wave = (ksteps + 3) >> 2;
      const RescaleHi pp = prm->p;
      const int32_t zp_h = prm->zp_h;
      for (int pt = 0; pt < my_ptiles; ++pt) {
        const int ptile = member + pt * GS;
        v4i pacc[2] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}};
        const int8_t *mbase = a.mbuf + (size_t)t * a.Bp * a.npadp + (((size_t)(row0 >> 4) * ksteps * 16 + r) << 6) + (q << 4);
        const int8_t *wbase = WpL + ((size_t)pt * 32 + r) * WLS + (q << 4);
        // all loads of the wave's k steps first (at most 8: N <= 2048); steps past the end re-read the
        // last one against zero weights
        int4 mv[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          int kk = wave * per_wave + (k < per_wave ? k : per_wave - 1);
          kk = kk < ksteps ? kk : ksteps - 1;
          mv[k] = *reinterpret_cast<const int4 *>(mbase + (size_t)kk * 1024);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          int kk = wave * per_wave + (k < per_wave ? k : per_wave - 1);
          const bool real = k < per_wave && kk < ksteps;
          kk = kk < ksteps ? kk : ksteps - 1;
          const v4i mf = v4i{mv[k].x, mv[k].y, mv[k].z, mv[k].w};
#pragma unroll
          for (int ct = 0; ct < 2; ++ct) {
            v4i wf = *reinterpret_cast<const v4i *>(wbase + (size_t)ct * 16 * WLS + kk * 64);
            if (!real) wf = v4i{0, 0, 0, 0};
            pacc[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, mf, pacc[ct], 0, 0, 0);
          }
        }
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int v = 0; v < 4; ++v) pred[((wave * 2 + ct) * 4 + v) * 64 + lane] = pacc[ct][v];
        __syncthreads();
        if (tid < 128) {
          const int ct = wave;  // threads 0..127: waves 0 and 1
          const int p0 = ptile * 32 + ct * 16 + 4 * q;
          uint32_t pk = 0;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int32_t s = pred[((0 * 2 + ct) * 4 + v) * 64 + lane] + pred[((1 * 2 + ct) * 4 + v) * 64 + lane] +
                              pred[((2 * 2 + ct) * 4 + v) * 64 + lane] + pred[((3 * 2 + ct) * 4 + v) * 64 + lane] +
                              (pt == 0 ? bpr[v] : a.bp2[p0 + v]);
            const int32_t hq = sat8(rescale_sat16_pre(s, pp) + zp_h);
            pk |= (uint32_t)(hq & 0xFF) << (8 * v);
          }
          if (row < a.B && p0 < a.H) {
            int8_t *od = a.out + ((size_t)t * a.B + row) * a.Hpad + p0;
            if (p0 + 3 < a.H) {
              *reinterpret_cast<uint32_t *>(od) = pk;
            } else {
              for (int c = 0; c < 4 && p0 + c < a.H; ++c) od[c] = (int8_t)(pk >> (8 * c));
            }
            if (a.y) {
              int8_t *yd = a.y + ((size_t)t * a.B + row) * a.H + p0;
              for (int c = 0; c < 4 && p0 + c < a.H; ++c) yd[c] = (int8_t)(pk >> (8 * c));
            }
          }
        }
        __syncthreads();
      }
      TICK(8);
      if (!group_sync(counter, epoch, GS + a.extra_arrivals, a.status, a.spin_limit, my_ptiles == 0 ? a.idle_sleep : 0,
                      my_ptiles == 0 ? a.idle_poll_sleep : a.poll_sleep, flag))
        return;
      TICK(9);
    }
  }
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
  if (a.c_out && row < a.B && n0 < a.N) {
#pragma unroll
    for (int c = 0; c < 4; ++c) a.c_out[(size_t)row * a.N + n0 + c] = (int16_t)creg[c];
  }
}

#undef TICK

// kernel for (flags & 7) at k depth KS16
template <int KS16>
rec_fn rec16_pick_ks(int fl) {
  switch (fl & 7) {
    case 0: return rec16_kernel<KS16, 0>;
    case 1: return rec16_kernel<KS16, 1>;
    case 2: return rec16_kernel<KS16, 2>;
    case 3: return rec16_kernel<KS16, 3>;
    case 4: return rec16_kernel<KS16, 4>;
    case 5: return rec16_kernel<KS16, 5>;
    case 6: return rec16_kernel<KS16, 6>;
    default: return rec16_kernel<KS16, 7>;
  }
}

}  // namespace lstm_int
