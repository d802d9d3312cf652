// Input GEMM of the persistent path for gfx950 (MI355X): W x for every (t, b)
// of a layer in one launch (the input contribution has no dependence on the
// recurrence and is hoisted out of the time loop), rescaled to int16
// (Secs. 3.2.4/3.2.5, zero point folded into the bias per Sec. 6) and stored
// in the tile order the recurrent kernel reads (persistent.h).
//
// Weights stay put: a workgroup owns 8 weight tiles (256 weight rows = the 64
// cells of one recurrent-kernel workgroup, 4 gates each), every wave keeps its
// two tiles over the whole k depth in registers as MFMA operands (read from a
// copy of the weights in operand order, 1 KB per wave load), and the workgroup
// streams over blocks of 32 (t, b) rows.  The activation block goes global ->
// LDS without passing through registers, three blocks ahead; the MFMA of block
// i runs interleaved with the requantization and the stores of block i - 1,
// whose results sit in a second set of ordinary vector registers (the file is
// compiled so that MFMA results go there, not to accumulation registers, which
// would cost a copy per value).  Addresses of loads and stores are a scalar
// base per block plus a per-lane offset that never changes.
//
// Work split: workgroup id -> (part of the rows, column block).  The XCD of a
// workgroup is id % 8 and each XCD has its own L2: an XCD works on a group of
// parts and a group of column blocks, so that it reads only that fraction of
// the activations and of the weights (launch_in_gemm_ws).
#include "persistent.h"

#include "lstm_int_math.h"

namespace lstm_int {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef short v2s __attribute__((ext_vector_type(2)));

namespace {

// sat16(rescale(s, M, r)) of two values, packed; PRE = operand treatment (InGemmArgs::pre)
template <int PRE>
__device__ __forceinline__ int32_t requant2(int32_t s0, int32_t s1, const RescaleHi &p0, const RescaleHi &p1) {
  if (PRE == 2) {
    s0 = rescale_preshift(s0, p0);
    s1 = rescale_preshift(s1, p1);
  }
  if (PRE == 1) {
    s0 <<= p0.k;
    s1 <<= p1.k;
  }
  const int32_t v0 = (__mulhi(s0, p0.M) + p0.add) >> p0.sh;
  const int32_t v1 = (__mulhi(s1, p1.M) + p1.add) >> p1.sh;
  // both halves saturate to int16
  const v2s pk = __builtin_amdgcn_cvt_pk_i16(v0, v1);
  return __builtin_bit_cast(int32_t, pk);
}

template <int KS, int PRE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void in_gemm_ws_kernel(InGemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int LS = KS * 32 + 16;                      // activation row stride in LDS
  constexpr int TILE_KB = (32 * LS + 1023) / 1024;      // one block of 32 rows, in 1 KB wave loads
  constexpr int NCH = (TILE_KB + 3) / 4;                // loads per wave (the same for every wave)
  constexpr int BUF = NCH * 4096;                       // one stage; bytes beyond the block are padding
  constexpr int NST = 4;                                // stages: loads run three blocks ahead
  const int tid = threadIdx.x, lane = tid & 63;
  // the chores ahead of the layer's recurrent kernel ride along (one launch less per layer)
  if (a.has_init) layer_init_device(a.init, (long long)blockIdx.x * 256 + tid, (long long)gridDim.x * 256);
  // the wave index as a scalar: tile numbers, LDS stage addresses and store bases stay out of the vector unit
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, b2 = lane >> 5;
  int part, cb;
  if (a.gp) {
    // XCD x = id % 8 works on a.gp-th of the parts and (8 / a.gp)-th of the column blocks
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int pp = a.parts / a.gp, cpx = (a.tiles >> 3) / (8 / a.gp);
    part = (x % a.gp) * pp + j % pp;
    cb = (x / a.gp) * cpx + j / pp;
  } else {
    part = blockIdx.x % a.parts;
    cb = blockIdx.x / a.parts;
  }
  const int nrb = (a.T * a.Bp) >> 5;
  const int per = (nrb + a.parts - 1) / a.parts;
  const int rb0 = part * per;
  const int rb1 = rb0 + per < nrb ? rb0 + per : nrb;
  if (rb0 >= rb1) return;  // the whole workgroup

  // this wave's two weight tiles, all of k, as MFMA operands; the biases; the rescale constants (filled below)
  v4i Wf[2][KS];
  int32_t bias[2][16];
  RescaleHi rs[4];

  // ---- activation block -> LDS: wave load (wave + 4 j) fills bytes
  // [1024 c, 1024 (c + 1)) of the padded [32][LS] block, lane l its 16 bytes at
  // 16 l.  Bytes outside the rows' first kpad bytes (row padding, the tail of
  // the stage) read the start of the buffer; they meet zero weights only.
  // Every wave issues exactly NCH loads per block, so that the number of vector
  // memory operations in flight behind a given block's loads is a constant.
  // The address of a load is a scalar base (the block's first row; rows of
  // consecutive t follow each other in memory) plus a per-lane offset that is
  // the same for every block.  The padded rows of a ragged batch (Bp > B) read
  // the rows that follow in memory -- the first rows of the next t, or, in the
  // last row block, the 31 rows of slack the caller provides behind the buffer;
  // their results are never read back.
  unsigned voff[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int o = (wave + 4 * j) * 1024 + lane * 16;
    const int r = o / LS, c = o - r * LS;
    const bool in = r < 32 && c < a.kpad;  // padding reads (row 0, byte 0) of the block
    voff[j] = in ? (unsigned)(r * a.lda + c) : 0u;  // below 32 * lda + kpad < 2^31
  }
  // the block to be loaded next: its row block, first b, and first row t * B + b
  int st_rb = rb0, st_b, st_row;
  {
    const int t = (rb0 << 5) / a.Bp;
    st_b = (rb0 << 5) - t * a.Bp;
    st_row = t * a.B + st_b;
  }
  const int8_t *st_base = a.A + (size_t)st_row * a.lda;
  auto stage_one = [&](int slot, int j) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(st_base + voff[j]),
                                     (__attribute__((address_space(3))) void *)(lds + slot * BUF + (wave + 4 * j) * 1024),
                                     16, 0, 0);
  };
  auto stage_advance = [&]() {
    if (st_rb + 1 >= rb1) return;  // past the end: the last block again, into a stage nobody reads
    ++st_rb;
    st_b += 32;
    st_row += 32;
    if (st_b >= a.Bp) {
      st_row += a.B - st_b;  // = (t + 1) * B
      st_b = 0;
    }
    st_base = a.A + (size_t)st_row * a.lda;
  };

  // requantize and store the pieces [p_lo, p_hi) of a finished block: piece
  // p = (tile, half, pair) -> two results -> one packed word; four pieces make
  // the 16 bytes of (tile, half).  The accumulators start from the bias.
  int32_t word[4];
  auto pieces = [&](const v16i (&pv)[2], int p_lo, int p_hi, int rb_prev) {
#pragma unroll
    for (int p = p_lo; p < p_hi; ++p) {
      const int tl = p >> 3, half = (p >> 2) & 1, pair = p & 3;
      const int i0 = half * 8 + pair * 2, i1 = i0 + 1;  // = 4 * gate + c
      word[pair] = requant2<PRE>(pv[tl][i0], pv[tl][i1], rs[i0 >> 2], rs[i1 >> 2]);
      if (pair == 3) {
        const int tile = cb * 8 + wave * 2 + tl;
        int4 *dst = a.tx2 + (((size_t)rb_prev * a.tiles + tile) * 2 + half) * 64 + lane;
        // streaming store: 268 MB per C4 layer pass through, nothing of it is read again before the
        // recurrent kernel, and the activation blocks and weights keep their place in L2
        __builtin_nontemporal_store(v4i{word[0], word[1], word[2], word[3]}, reinterpret_cast<v4i *>(dst));
      }
    }
  };

  // One block: 2 * KS MFMAs; under them, in the issue slots they leave free,
  // the loads of the block three ahead and the requantization of the previous
  // block.  Vector memory operations complete in the order issued; a block
  // issues NCH loads and (all but the first) four stores, so at the top of
  // block i everything up to the loads of block i + 1 is complete once at most
  // the operations of block i - 1 -- NCH + 4, or NCH after the first block --
  // are in flight.  Past the barrier that holds for every wave's part of block
  // i + 1, and every wave has finished reading block i - 1, whose stage the
  // loads of block i + 3 overwrite.  The first operands of block i + 1 can
  // therefore be read during the last k steps of block i, ahead of the next
  // barrier: the operand ring runs on across the block boundary, and the first
  // MFMA of a block finds its operand in registers.
  constexpr int DEPTH = 4;
  static_assert(KS % DEPTH == 0, "the operand ring wraps at a block boundary");
  v4i xf[DEPTH];
  auto first_operands = [&](int slot) {
    const uint8_t *xbase = lds + slot * BUF + col * LS + (b2 << 4);
#pragma unroll
    for (int ks = 0; ks < DEPTH && ks < KS; ++ks) xf[ks] = *reinterpret_cast<const v4i *>(xbase + ks * 32);
  };
  auto block = [&](int rb, int slot, v16i (&acc)[2], const v16i (&prev)[2], auto have_prev_tag, auto stores_tag) {
    constexpr bool HAVE = decltype(have_prev_tag)::value;
    if (decltype(stores_tag)::value)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCH + 4) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCH) : "memory");
    // a bare barrier: __syncthreads() would also wait for the stores in flight
    // (its release fence), and nothing here is exchanged through global memory
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const uint8_t *xbase = lds + slot * BUF + col * LS + (b2 << 4);
    const uint8_t *xnext = lds + ((slot + 1) % NST) * BUF + col * LS + (b2 << 4);  // after the last block: never used
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        if (ks == 0) {
          v16i c0;
#pragma unroll
          for (int v = 0; v < 16; ++v) c0[v] = bias[tl][v];
          acc[tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Wf[tl][ks], xf[ks % DEPTH], c0, 0, 0, 0);
        } else {
          acc[tl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(Wf[tl][ks], xf[ks % DEPTH], acc[tl], 0, 0, 0);
        }
      }
      xf[ks % DEPTH] = ks + DEPTH < KS ? *reinterpret_cast<const v4i *>(xbase + (ks + DEPTH) * 32)
                                       : *reinterpret_cast<const v4i *>(xnext + (ks + DEPTH - KS) * 32);
      if (ks < NCH) stage_one((slot + NST - 1) % NST, ks);
      if (HAVE) pieces(prev, ks * 16 / KS, (ks + 1) * 16 / KS, rb - 1);
      // keep the LDS reads DEPTH steps ahead and the other work spread over the k loop
      __builtin_amdgcn_sched_barrier(0);
    }
    // results in ordinary vector registers, where the requantization reads them without a copy
    asm volatile("" : "+v"(acc[0]), "+v"(acc[1]));
    stage_advance();
  };

  static_assert(NCH <= KS, "one load per k step");
  static_assert(NCH + 4 <= 63, "vmcnt field");
  // the first blocks are requested before anything else: their latency covers the weight loads
  for (int i = 0; i < NST - 1; ++i) {
#pragma unroll
    for (int j = 0; j < NCH; ++j) stage_one(i, j);
    stage_advance();
  }

  // ---- the weight tiles
  {
    int4 w[2][KS], bb[2][4];
    auto load_tile = [&](int tl) {
      const int tile = cb * 8 + wave * 2 + tl;
      // operand order: a wave load reads 1 KB in one piece
      const int8_t *wlane = a.W2f + (size_t)tile * 32 * a.kpad + (lane << 4);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        // kpad is a multiple of 64: a 32-byte k step is inside the rows or entirely beyond them
        w[tl][ks] = *reinterpret_cast<const int4 *>(wlane + (ks * 32 < a.kpad ? ks * 1024 : 0));
      // the lane's 16 results of a tile: index 4*gate + c <-> tile row 8*gate + 4*(lane/32) + c
#pragma unroll
      for (int g = 0; g < 4; ++g)
        bb[tl][g] = *reinterpret_cast<const int4 *>(a.bx2 + (size_t)tile * 32 + g * 8 + (b2 << 2));
    };
    auto keep_tile = [&](int tl) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bool in = ks * 32 < a.kpad;
        Wf[tl][ks] = v4i{in ? w[tl][ks].x : 0, in ? w[tl][ks].y : 0, in ? w[tl][ks].z : 0, in ? w[tl][ks].w : 0};
        asm volatile("" : "+a"(Wf[tl][ks]));  // resident in accumulation registers for the whole launch
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bias[tl][g * 4 + 0] = bb[tl][g].x; bias[tl][g * 4 + 1] = bb[tl][g].y;
        bias[tl][g * 4 + 2] = bb[tl][g].z; bias[tl][g * 4 + 3] = bb[tl][g].w;
      }
    };
    // all loads are issued before the first is used, where the registers allow it (2 * KS * 4 of them)
    load_tile(0);
    if (KS <= 20) load_tile(1);
    __builtin_amdgcn_sched_barrier(0);
    keep_tile(0);
    if (KS > 20) {
      load_tile(1);
      __builtin_amdgcn_sched_barrier(0);
    }
    keep_tile(1);
  }
#pragma unroll
  for (int g = 0; g < 4; ++g) rs[g] = a.rs[g];
  // blocks 0 and 1 of the part are loaded before anything else is issued
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCH) : "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  first_operands(0);
  v16i accA[2], accB[2];
  block(rb0, 0, accA, accB, std::false_type{}, std::false_type{});
  int rb = rb0 + 1, slot = 1;
  if (rb < rb1) {
    block(rb, slot, accB, accA, std::true_type{}, std::false_type{});  // the first block stored nothing
    ++rb;
    slot = (slot + 1) % NST;
  }
  // pairs of blocks, so that the two accumulator sets alternate statically
  for (; rb + 1 < rb1; rb += 2, slot = (slot + 2) % NST) {
    block(rb, slot, accA, accB, std::true_type{}, std::true_type{});
    block(rb + 1, (slot + 1) % NST, accB, accA, std::true_type{}, std::true_type{});
  }
  if (rb < rb1) {
    block(rb, slot, accA, accB, std::true_type{}, std::true_type{});
    pieces(accA, 0, 16, rb);
  } else {
    // the last block ran on accB if at least two blocks ran, else on accA
    if (rb1 - rb0 >= 2)
      pieces(accB, 0, 16, rb1 - 1);
    else
      pieces(accA, 0, 16, rb1 - 1);
  }
}

template <int KS>
constexpr unsigned lds_bytes_ks() {  // NST stages of NCH * 4 KB
  return 4u * ((((32 * (KS * 32 + 16) + 1023) / 1024) + 3) / 4) * 4096;
}

template <int KS>
hipError_t init_ks() {
  static_assert(lds_bytes_ks<KS>() <= 160 * 1024, "activation stages exceed LDS");
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(in_gemm_ws_kernel<KS, 0>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes_ks<KS>());
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(in_gemm_ws_kernel<KS, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes_ks<KS>());
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(in_gemm_ws_kernel<KS, 2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes_ks<KS>());
  return e;
}

template <int KS>
void launch_ks(hipStream_t s, const InGemmArgs &a, int grid) {
  if (a.pre == 0)
    hipLaunchKernelGGL((in_gemm_ws_kernel<KS, 0>), dim3(grid), dim3(256), lds_bytes_ks<KS>(), s, a);
  else if (a.pre == 1)
    hipLaunchKernelGGL((in_gemm_ws_kernel<KS, 1>), dim3(grid), dim3(256), lds_bytes_ks<KS>(), s, a);
  else
    hipLaunchKernelGGL((in_gemm_ws_kernel<KS, 2>), dim3(grid), dim3(256), lds_bytes_ks<KS>(), s, a);
}

}  // namespace

hipError_t in_gemm_init() {
  hipError_t e = init_ks<8>();
  if (e == hipSuccess) e = init_ks<16>();
  if (e == hipSuccess) e = init_ks<20>();
  if (e == hipSuccess) e = init_ks<32>();
  return e;
}

bool in_gemm_ws_supported(const InGemmArgs &a) {
  if (a.kpad > 1024 || a.kpad % 64 != 0 || a.tiles % 8 != 0 || !a.W2f) return false;
  if (a.Bp != a.B && !a.a_slack) return false;  // the last row block would read beyond the buffer
  if (32ll * a.lda + a.kpad >= (1ll << 31)) return false;  // 32-bit offsets within a row block
  for (int g = 0; g < 4; ++g)
    if (a.r[g] < 3 || a.r[g] > 62) return false;
  return true;
}

void launch_in_gemm_ws(hipStream_t s, const InGemmArgs &a0, int num_cus) {
  if (a0.T <= 0 || a0.B <= 0) return;
  InGemmArgs a = a0;
  for (int g = 0; g < 4; ++g) {
    a.rs[g] = rescale_hi_prepare(a.M[g], a.r[g]);
    if (a.rs[g].k != 0 && a.pre == 0) a.pre = 2;  // a caller that proved no bound
  }
  const int cbs = a.tiles / 8;
  const int nrb = (a.T * a.Bp) >> 5;
  int parts = num_cus / cbs;
  if (parts < 1) parts = 1;
  if (parts > nrb) parts = nrb;
  a.parts = parts;
  const int grid = parts * cbs;
  // Split over the XCDs (workgroup id % 8; each has its own L2).  With gp part
  // groups an XCD reads 1/gp of the activations and gp/8 of the weights: gp = 8
  // (every XCD reads all weights at once in the prologue, which then takes
  // 8 us of the C4 shape's 80) down to 1 (every XCD reads all activations).
  if (a.gp == 0) a.gp = 2;
  if (grid % 8 != 0 || a.gp < 1 || a.gp > 8 || 8 % a.gp != 0 || parts % a.gp != 0 || cbs % (8 / a.gp) != 0)
    a.gp = 0;  // plain split: part = id % parts
  if (a.kpad <= 256) launch_ks<8>(s, a, grid);
  else if (a.kpad <= 512) launch_ks<16>(s, a, grid);
  else if (a.kpad <= 640) launch_ks<20>(s, a, grid);
  else launch_ks<32>(s, a, grid);
}

}  // namespace lstm_int
