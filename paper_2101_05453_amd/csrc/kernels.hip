// HIP kernels of the integer LSTM cell step for gfx950 (MI355X, wave64).
//
//   gemm_i8_kernel  int8 x int8 -> int32 on the 16x16x64 int8 MFMA, with the
//                   requantization of Secs. 3.2.4-3.2.8 fused into the
//                   epilogue (bias with folded zero point, Sec. 6).  Used for
//                   the input term W x over all T*B rows at once, for the
//                   recurrent term R h of one step, and for the projection.
//   cell_kernel     everything between the gate matmuls and the hidden state
//                   for one batch row per workgroup (layer-norm statistics by
//                   wavefront reductions).
#include "kernels.h"

#include <algorithm>

#include "persistent.h"

#include "lstm_int_math.h"

namespace lstm_int {

typedef int v4i __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// int8 GEMM.  The weight tile is the MFMA's first operand and the activation
// tile its second, so a lane ends up with four consecutive output columns
// (weight rows) of one activation row: D[4*(lane/16)+j][lane%16].
// Both operands are K-contiguous in memory, which is exactly what the MFMA
// wants from each lane (16 consecutive k bytes of one row); the same k
// permutation applies to both, so the dot products do not depend on it.
// ---------------------------------------------------------------------------
// A staged tile in LDS: rows of 64 bytes without padding, the 16-byte piece p of row r at position p ^ ((r >> 1) & 3).
// With this swizzle both accesses are free of bank conflicts -- the operand reads of the 16x16x64 MFMA (row =
// lane % 16, piece = lane / 16: 4 clocks per wave) and the staging stores (row = lane / 4, piece = lane % 4: 8
// clocks, the rate of LDS stores) -- measured with SQ_LDS_BANK_CONFLICT on a probe kernel; rows padded to 80 bytes
// took 8 and 16 clocks, padded to 96 bytes 4 and 16.
constexpr int kLdsRow = 64;
__device__ __forceinline__ int lds_piece(int row, int piece) { return row * kLdsRow + ((piece ^ ((row >> 1) & 3)) << 4); }
// piece c of a staged tile: four neighbouring lanes fetch the 64 bytes of one row, the order the memory system wants
__device__ __forceinline__ int stage_row(int c) { return c >> 2; }
__device__ __forceinline__ int stage_piece(int c) { return c & 3; }

// BM x BN outputs per workgroup of WM x WN waves.  A tile fetches (BM + BN) * 64 bytes per 2 * BM * BN * 64
// operations: 128 operations per byte at 128 x 128 (four waves of 64 x 64, three workgroups per compute unit) and
// 256 at 256 x 256 (eight waves of 128 x 64, one workgroup per compute unit), which large products take
// (16384 x 6144 x 2048: 290 -> 271 us).
// DMA: the operand tiles go from memory straight into LDS (global_load_lds, no registers and no LDS store
// instructions on the way), four k tiles deep, and the operands of tile kt + 1 are read from LDS while tile kt is
// multiplied.
constexpr int kDmaBuffers = 4;
template <int BM, int BN, int WM, int WN, bool OUT8, bool DMA = false>
__global__ __launch_bounds__(WM * WN * 64)
    __attribute__((amdgpu_waves_per_eu(BM == 256 ? 2 : (BM == 128 ? 3 : 1), BM == 256 ? 2 : (BM == 128 ? 3 : 8)))) void gemm_i8_kernel(
    const int8_t *__restrict__ A, int lda, int M, const int8_t *__restrict__ W, int kpad,
    int ncols, const int32_t *__restrict__ bias, Requant rq, void *__restrict__ out, int ldc,
    int8_t *__restrict__ out2, int ldc2, int nrb, int ncb, int xr_n) {
  constexpr int NW = WM * WN, NT = NW * 64;  // waves, threads
  static_assert(NW == 4 || NW == 8, "four or eight waves per workgroup");
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 16, NI = TN / 16;
  static_assert(MI >= 1 && NI >= 1 && TM % 16 == 0 && TN % 16 == 0, "tile shape");
  constexpr int XCH = BM * 4, WCH = BN * 4;  // 16-byte chunks per k-tile
  constexpr int XPT = (XCH + NT - 1) / NT, WPT = (WCH + NT - 1) / NT;

  // operand tiles during the k loop; afterwards (int16 output) each wave's results, kStageRows rows at a time,
  // staged so that the stores cover whole 16-byte pieces of consecutive columns
  constexpr int kStageRow = TN + 8;  // int16 elements; the pad keeps the 8-byte writes off each other's banks
  constexpr int MIG = TM > 64 ? 2 : MI;  // 16-row blocks staged per pass
  constexpr int kStageRows = MIG * 16;
  constexpr int kTileBytes = (BM + BN) * kLdsRow;  // one staged k tile of both operands
  constexpr int kOperandBytes = 2 * kTileBytes;    // two of them: tile kt + 1 is stored while tile kt is multiplied
  constexpr int kStageBytes = OUT8 ? 0 : NW * kStageRows * kStageRow * 2;
  static_assert(!DMA || kDmaBuffers * kTileBytes >= kStageBytes, "the staged results fit the operand buffers");
  __shared__ __attribute__((aligned(16))) int8_t lds_static[DMA ? 16 : (kOperandBytes > kStageBytes ? kOperandBytes : kStageBytes)];
  extern __shared__ __attribute__((aligned(16))) int8_t lds_dynamic[];  // DMA: kDmaBuffers * kTileBytes, set at launch
  int8_t *const lds_buf = DMA ? lds_dynamic : lds_static;
  int8_t *Xs = lds_buf, *Ws = lds_buf + BM * kLdsRow;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  // Workgroup -> tile.  The hardware deals consecutive workgroups out to the eight XCDs in turn, and every XCD has
  // an L2 of its own: XCD x = id % 8 gets the tiles of one cell of an xr_n x (8 / xr_n) split of the tile grid (the
  // host picks the split that moves the fewest bytes: every XCD fetches its rows' activations and its columns'
  // weights once instead of all of both), and walks them in bands of kBand row blocks, the row block running fastest
  // and the column block next, so that the workgroups in flight together share kBand activation tiles.  If the
  // hardware dealt the workgroups differently only the traffic would change: the map is one-to-one whatever runs where.
  constexpr int kBand = 8;
  int rblk, cblk;
  {
    const int id = blockIdx.x, x = id & 7, j = id >> 3;
    const int xc_n = 8 / xr_n, xr = x / xc_n, xc = x - xr * xc_n;
    const int r_lo = xr * nrb / xr_n, r_hi = (xr + 1) * nrb / xr_n;
    const int c_lo = xc * ncb / xc_n, c_hi = (xc + 1) * ncb / xc_n;
    const int nr = r_hi - r_lo, nc = c_hi - c_lo;
    if (j >= nr * nc) return;  // the whole workgroup: the grid is 8 x the largest share
    const int per_band = kBand * nc;
    const int band = j / per_band, in_band = j - band * per_band;
    const int rows_here = nr - band * kBand < kBand ? nr - band * kBand : kBand;
    const int c = in_band / rows_here;
    cblk = c_lo + c;
    rblk = r_lo + band * kBand + (in_band - c * rows_here);
  }
  const int row_base = rblk * BM;  // activation rows
  const int col_base = cblk * BN;  // weight rows = output columns

  v4i acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) acc[ni][mi] = v4i{0, 0, 0, 0};

  const int KT = kpad >> 6;
  if constexpr (DMA) {
    static_assert(NW == 8 && XCH == 1024 && WCH == 1024, "two 1 KB chunks of each operand per wave and k tile");
    // Chunk q of a tile = its rows 16 q .. 16 q + 15 = 1 KB of the unpadded swizzled layout: a wave instruction
    // fills it, lane l with the 16 bytes at position l % 4 of row 16 q + l / 4 -- which, by the swizzle, are piece
    // (l % 4) ^ ((row >> 1) & 3) of that row in memory; the four lanes of a row still fetch its 64 bytes.
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const int8_t *gx0, *gx1, *gw0, *gw1;
    {
      const int ra = 16 * wv + (lane >> 2), rb = ra + 128;
      const int pa = ((lane & 3) ^ ((ra >> 1) & 3)) << 4, pb = ((lane & 3) ^ ((rb >> 1) & 3)) << 4;
      const int xa = row_base + ra < M ? row_base + ra : M - 1;  // rows past the end repeat the last one; never stored
      const int xb = row_base + rb < M ? row_base + rb : M - 1;
      gx0 = A + (size_t)xa * lda + pa;
      gx1 = A + (size_t)xb * lda + pb;
      gw0 = W + (size_t)(col_base + ra) * kpad + pa;
      gw1 = W + (size_t)(col_base + rb) * kpad + pb;
    }
    typedef const __attribute__((address_space(1))) void *gptr;
    typedef __attribute__((address_space(3))) void *lptr;
    // tile kt -> buffer kt % kDmaBuffers; past the last tile the last one again, into a buffer nobody reads, so
    // that every iteration issues the same four loads and the counts below hold to the end
    auto dma = [&](int kt) {
      const int ko = (kt < KT ? kt : KT - 1) << 6;
      int8_t *base = lds_buf + (kt & (kDmaBuffers - 1)) * kTileBytes + wv * 1024;
      __builtin_amdgcn_global_load_lds((gptr)(gx0 + ko), (lptr)base, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr)(gx1 + ko), (lptr)(base + 8192), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr)(gw0 + ko), (lptr)(base + BM * kLdsRow), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((gptr)(gw1 + ko), (lptr)(base + BM * kLdsRow + 8192), 16, 0, 0);
    };
    // every wave's part of the tiles up to the one `left` loads ago has landed, for every wave: vector memory
    // operations complete in the order issued; a bare barrier (__syncthreads() would wait for all of them)
#define GEMM_LANDED(left)                                                \
  do {                                                                   \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(left) : "memory"); \
    __builtin_amdgcn_s_barrier();                                        \
    asm volatile("" ::: "memory");                                       \
  } while (0)
#define GEMM_READ_OPS(xf, wf, kt)                                                                             \
  do {                                                                                                        \
    const int8_t *xs = Xs + ((kt) & (kDmaBuffers - 1)) * kTileBytes, *wsb = Ws + ((kt) & (kDmaBuffers - 1)) * kTileBytes; \
    _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                                                         \
      xf[mi] = *reinterpret_cast<const v4i *>(xs + lds_piece(wm * TM + mi * 16 + (lane & 15), lane >> 4));    \
    _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                                         \
      wf[ni] = *reinterpret_cast<const v4i *>(wsb + lds_piece(wn * TN + ni * 16 + (lane & 15), lane >> 4));   \
  } while (0)
    // Iteration kt: the operands of tile kt are in registers (cur) and tile kt + 1 is complete in LDS.  Tile kt + 3 is
    // requested into the buffer of tile kt - 1 (read two iterations ago, two barriers back), the operands of tile
    // kt + 1 are read (nxt) under the MFMAs of tile kt, and the iteration ends once tile kt + 2 has landed.
#define GEMM_DMA_TILE(xc, wc, xn, wn_, kt)                                                                    \
  do {                                                                                                        \
    dma((kt) + 3);                                                                                            \
    if ((kt) + 1 < KT) GEMM_READ_OPS(xn, wn_, (kt) + 1);                                                      \
    _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                                         \
      _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                                                       \
        acc[ni][mi] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wc[ni], xc[mi], acc[ni][mi], 0, 0, 0);            \
    GEMM_LANDED(4);                                                                                           \
  } while (0)
    v4i xfa[MI], wfa[NI], xfb[MI], wfb[NI];
    dma(0);
    dma(1);
    dma(2);
    GEMM_LANDED(4);  // tiles 0 and 1
    GEMM_READ_OPS(xfa, wfa, 0);
    for (int kt = 0; kt < KT; kt += 2) {
      GEMM_DMA_TILE(xfa, wfa, xfb, wfb, kt);
      if (kt + 1 < KT) GEMM_DMA_TILE(xfb, wfb, xfa, wfa, kt + 1);
    }
    GEMM_LANDED(0);  // the loads past the end too: the buffers are about to hold the staged results
#undef GEMM_DMA_TILE
#undef GEMM_READ_OPS
#undef GEMM_LANDED
  } else {
  // The next k-tile's chunks wait in named registers between their load and their LDS store.  (As arrays filled
  // and drained by helper lambdas they were left in scratch memory in some builds: every chunk then went
  // load -> scratch -> LDS, the loads no longer overlapped the MFMAs, and the kernel ran at half speed.)
  static_assert(XPT <= 2 && WPT <= 2, "at most two chunks per thread and operand");
  // the k tiles kt, kt + 1, kt + 2 on their way from memory to LDS: plain named vector registers
  v4i sa_x0 = {}, sa_x1 = {}, sa_w0 = {}, sa_w1 = {};
  v4i sb_x0 = {}, sb_x1 = {}, sb_w0 = {}, sb_w1 = {};
  v4i sc_x0 = {}, sc_x1 = {}, sc_w0 = {}, sc_w1 = {};
  const int c0 = tid, c1 = tid + NT;
  const int8_t *xsrc0, *xsrc1, *wsrc0, *wsrc1;
  {
    int r0 = row_base + stage_row(c0), r1 = row_base + stage_row(c1);
    r0 = r0 < M ? r0 : M - 1;  // rows past the end repeat the last one; never stored
    r1 = r1 < M ? r1 : M - 1;
    xsrc0 = A + (size_t)r0 * lda + (stage_piece(c0) << 4);
    xsrc1 = A + (size_t)r1 * lda + (stage_piece(c1) << 4);
    wsrc0 = W + (size_t)(col_base + stage_row(c0)) * kpad + (stage_piece(c0) << 4);
    wsrc1 = W + (size_t)(col_base + stage_row(c1)) * kpad + (stage_piece(c1) << 4);
  }
  const bool x0_on = XCH >= NT || c0 < XCH, w0_on = WCH >= NT || c0 < WCH;
  int8_t *const xdst0 = Xs + lds_piece(stage_row(c0), stage_piece(c0));
  int8_t *const xdst1 = Xs + lds_piece(stage_row(c1), stage_piece(c1));
  int8_t *const wdst0 = Ws + lds_piece(stage_row(c0), stage_piece(c0));
  int8_t *const wdst1 = Ws + lds_piece(stage_row(c1), stage_piece(c1));
#define GEMM_LOAD_TILES(st, kt)                                                       \
  do {                                                                               \
    if ((kt) < KT) {                                                                 \
      if (x0_on) st##_x0 = *reinterpret_cast<const v4i *>(xsrc0 + ((kt) << 6));    \
      if (XPT > 1) st##_x1 = *reinterpret_cast<const v4i *>(xsrc1 + ((kt) << 6));  \
      if (w0_on) st##_w0 = *reinterpret_cast<const v4i *>(wsrc0 + ((kt) << 6));    \
      if (WPT > 1) st##_w1 = *reinterpret_cast<const v4i *>(wsrc1 + ((kt) << 6));  \
    }                                                                                \
  } while (0)
#define GEMM_STORE_TILES(st, buf)                                                    \
  do {                                                                               \
    if (x0_on) *reinterpret_cast<v4i *>(xdst0 + (buf) * kTileBytes) = st##_x0;      \
    if (XPT > 1) *reinterpret_cast<v4i *>(xdst1 + (buf) * kTileBytes) = st##_x1;    \
    if (w0_on) *reinterpret_cast<v4i *>(wdst0 + (buf) * kTileBytes) = st##_w0;      \
    if (WPT > 1) *reinterpret_cast<v4i *>(wdst1 + (buf) * kTileBytes) = st##_w1;    \
  } while (0)
  // One k tile: tile kt + 1 goes from its staged registers (nx) into the LDS buffer that tile kt - 1 was read from
  // (every wave is past the barrier that ended kt - 1), the freed registers request tile kt + 4, and tile kt is
  // multiplied out of the other buffer: one barrier per tile, the LDS stores under the MFMAs, global loads three
  // tiles of MFMAs ahead (one tile ahead and two barriers per tile, the loop waited for memory every time round).
#define GEMM_K_TILE(nx, kt)                                                          \
  do {                                                                               \
    if ((kt) + 1 < KT) GEMM_STORE_TILES(nx, ((kt) + 1) & 1);                         \
    GEMM_LOAD_TILES(nx, (kt) + 4);                                                   \
    const int8_t *xs = Xs + ((kt) & 1) * kTileBytes, *wsb = Ws + ((kt) & 1) * kTileBytes; \
    v4i xf[MI], wf[NI];                                                              \
    _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                                \
      xf[mi] = *reinterpret_cast<const v4i *>(xs + lds_piece(wm * TM + mi * 16 + (lane & 15), lane >> 4)); \
    _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                \
      wf[ni] = *reinterpret_cast<const v4i *>(wsb + lds_piece(wn * TN + ni * 16 + (lane & 15), lane >> 4)); \
    _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                \
      _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                              \
        acc[ni][mi] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[ni], xf[mi], acc[ni][mi], 0, 0, 0); \
    __syncthreads();                                                                 \
  } while (0)

  // tile t waits in register set t % 3 (sa, sb, sc)
  GEMM_LOAD_TILES(sa, 0);
  GEMM_LOAD_TILES(sb, 1);
  GEMM_LOAD_TILES(sc, 2);
  GEMM_STORE_TILES(sa, 0);
  __syncthreads();
  GEMM_LOAD_TILES(sa, 3);
  for (int kt = 0; kt < KT; kt += 3) {
    GEMM_K_TILE(sb, kt);
    if (kt + 1 < KT) GEMM_K_TILE(sc, kt + 1);
    if (kt + 2 < KT) GEMM_K_TILE(sa, kt + 2);
  }
#undef GEMM_K_TILE
#undef GEMM_LOAD_TILES
#undef GEMM_STORE_TILES
  }

  // epilogue: + bias, rescale, saturate, store
  const int cpg = rq.cols_per_gate;
  // int16 output with rows of whole 16-byte pieces: through LDS, so that a wave instruction stores 128 consecutive
  // bytes of each of 8 rows (straight from the MFMA layout it is 32 bytes of each of 16 rows, and the memory
  // system wrote several times the output)
  const bool staged = !OUT8 && (ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  int16_t *stage = reinterpret_cast<int16_t *>(lds_buf) + wave * kStageRows * kStageRow;
#pragma unroll
  for (int mg = 0; mg < MI; mg += MIG) {
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int n0 = col_base + wn * TN + ni * 16 + ((lane >> 4) << 2);
      const int4 b4 = *reinterpret_cast<const int4 *>(bias + n0);  // bias is padded like W
      const int32_t bv[4] = {b4.x, b4.y, b4.z, b4.w};
      int32_t Mg[4], rg[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // the column's gate picks its rescale by selects: indexing rq.M / rq.r with a runtime gate would copy the
        // argument struct into scratch memory
        const int n = n0 + j;
        Mg[j] = n >= 3 * cpg ? rq.M[3] : (n >= 2 * cpg ? rq.M[2] : (n >= cpg ? rq.M[1] : rq.M[0]));
        rg[j] = n >= 3 * cpg ? rq.r[3] : (n >= 2 * cpg ? rq.r[2] : (n >= cpg ? rq.r[1] : rq.r[0]));
      }
#pragma unroll
      for (int mi = mg; mi < mg + MIG; ++mi) {
        const int m = row_base + wm * TM + mi * 16 + (lane & 15);
        int32_t v[4];
        if (rq.all_hi) {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = rescale_hi(acc[ni][mi][j] + bv[j], Mg[j], rg[j]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = rescale(acc[ni][mi][j] + bv[j], Mg[j], rg[j]);
        }
        if (m >= M) continue;
        if (OUT8) {
          int8_t *o = reinterpret_cast<int8_t *>(out) + (size_t)m * ldc;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (n0 + j < ncols) {
              const int8_t q = (int8_t)sat8(v[j] + rq.zp);
              o[n0 + j] = q;
              if (out2) out2[(size_t)m * ldc2 + n0 + j] = q;
            }
          }
        } else if (staged) {
          short4 pk;
          pk.x = (short)sat16(v[0]);
          pk.y = (short)sat16(v[1]);
          pk.z = (short)sat16(v[2]);
          pk.w = (short)sat16(v[3]);
          *reinterpret_cast<short4 *>(stage + ((mi - mg) * 16 + (lane & 15)) * kStageRow + ni * 16 + ((lane >> 4) << 2)) = pk;
        } else {
          int16_t *o = reinterpret_cast<int16_t *>(out) + (size_t)m * ldc;
          if (n0 + 3 < ncols && (ldc & 3) == 0) {
            short4 pk;
            pk.x = (short)sat16(v[0]);
            pk.y = (short)sat16(v[1]);
            pk.z = (short)sat16(v[2]);
            pk.w = (short)sat16(v[3]);
            *reinterpret_cast<short4 *>(o + n0) = pk;
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (n0 + j < ncols) o[n0 + j] = (int16_t)sat16(v[j]);
          }
        }
      }
    }
    if (!OUT8 && staged) {
      // a wave reads back only what it wrote itself; LDS serves a wave's requests in order (so the next pass's
      // stores cannot overtake these reads either)
      constexpr int PPR = TN / 8;  // 16-byte pieces per row
#pragma unroll
      for (int i = 0; i < kStageRows * PPR / 64; ++i) {
        const int idx = i * 64 + lane;
        const int r = idx / PPR, pc = idx - r * PPR;
        const int m = row_base + wm * TM + mg * 16 + r;
        const int n = col_base + wn * TN + pc * 8;
        const int4 piece = *reinterpret_cast<const int4 *>(stage + r * kStageRow + pc * 8);
        if (m < M) {
          int16_t *o = reinterpret_cast<int16_t *>(out) + (size_t)m * ldc + n;
          if (n + 7 < ncols) {
            *reinterpret_cast<int4 *>(o) = piece;
          } else {
            const int16_t e[8] = {(int16_t)piece.x, (int16_t)(piece.x >> 16), (int16_t)piece.y, (int16_t)(piece.y >> 16),
                                  (int16_t)piece.z, (int16_t)(piece.z >> 16), (int16_t)piece.w, (int16_t)(piece.w >> 16)};
#pragma unroll
            for (int j = 0; j < 8; ++j)
              if (n + j < ncols) o[j] = e[j];
          }
        }
      }
    }
  }
}

// The split of the tile grid over the XCDs: xr_n row shares x (8 / xr_n) column shares.  Among the splits that keep
// the largest share within 1/8 of an even one, the one for which the XCDs together fetch the fewest bytes.
static int gemm_xcd_rows(int nrb, int ncb, int bm, int bn, int kpad, unsigned *grid) {
  const long long even = ((long long)nrb * ncb + 7) / 8;
  int best = 1;
  long long best_bytes = -1, best_share = 0;
  for (int pass = 0; pass < 2 && best_bytes < 0; ++pass)
    for (int xr = 1; xr <= 8; xr *= 2) {
      const int xc = 8 / xr;
      const long long share = (long long)((nrb + xr - 1) / xr) * ((ncb + xc - 1) / xc);
      if (pass == 0 && share * 8 > even * 9) continue;  // pass 1: nothing is balanced, take the least traffic
      const long long bytes = ((long long)nrb * bm * xc + (long long)ncb * bn * xr) * kpad;
      if (best_bytes < 0 || bytes < best_bytes) best = xr, best_bytes = bytes, best_share = share;
    }
  *grid = (unsigned)(best_share * 8);
  return best;
}

constexpr unsigned kGemmDmaLds = kDmaBuffers * (256 + 256) * kLdsRow;  // 128 KB: beyond the default limit

// once per process and device, before the first launch of the 256 x 256 tile (not from a call under graph capture)
hipError_t gemm_init() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_i8_kernel<256, 256, 2, 4, false, true>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kGemmDmaLds);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_i8_kernel<256, 256, 2, 4, true, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kGemmDmaLds);
  return e;
}

template <bool OUT8>
static void launch_gemm(hipStream_t s, const int8_t *A, int lda, int M, const int8_t *W, int kpad,
                        int ncols, const int32_t *bias, const Requant &rq, void *out, int ldc,
                        int8_t *out2, int ldc2) {
  if (M <= 0 || ncols <= 0) return;
  const int ncols_pad = (ncols + 127) / 128 * 128;
  unsigned grid;
  if (M >= 2048 && ncols_pad >= 1024 && ncols_pad % 256 == 0) {
    const int nrb = (M + 255) / 256, ncb = ncols_pad / 256;
    const int xr = gemm_xcd_rows(nrb, ncb, 256, 256, kpad, &grid);
    hipLaunchKernelGGL((gemm_i8_kernel<256, 256, 2, 4, OUT8, true>), dim3(grid), dim3(512), kGemmDmaLds, s, A, lda, M,
                       W, kpad, ncols, bias, rq, out, ldc, out2, ldc2, nrb, ncb, xr);
  } else if (M > 256) {
    const int nrb = (M + 127) / 128, ncb = ncols_pad / 128;
    const int xr = gemm_xcd_rows(nrb, ncb, 128, 128, kpad, &grid);
    hipLaunchKernelGGL((gemm_i8_kernel<128, 128, 2, 2, OUT8>), dim3(grid), dim3(256), 0, s, A, lda, M, W,
                       kpad, ncols, bias, rq, out, ldc, out2, ldc2, nrb, ncb, xr);
  } else if (M > 32) {
    const int nrb = (M + 63) / 64, ncb = ncols_pad / 64;
    const int xr = gemm_xcd_rows(nrb, ncb, 64, 64, kpad, &grid);
    hipLaunchKernelGGL((gemm_i8_kernel<64, 64, 2, 2, OUT8>), dim3(grid), dim3(256), 0, s, A, lda, M, W,
                       kpad, ncols, bias, rq, out, ldc, out2, ldc2, nrb, ncb, xr);
  } else {
    const int nrb = (M + 31) / 32, ncb = ncols_pad / 128;
    const int xr = gemm_xcd_rows(nrb, ncb, 32, 128, kpad, &grid);
    hipLaunchKernelGGL((gemm_i8_kernel<32, 128, 1, 4, OUT8>), dim3(grid), dim3(256), 0, s, A, lda, M, W,
                       kpad, ncols, bias, rq, out, ldc, out2, ldc2, nrb, ncb, xr);
  }
}

void launch_gemm_i16(hipStream_t s, const int8_t *A, int lda, int M, const int8_t *W, int kpad,
                     int ncols, const int32_t *bias, const Requant &rq, int16_t *out, int ldc) {
  launch_gemm<false>(s, A, lda, M, W, kpad, ncols, bias, rq, out, ldc, nullptr, 0);
}

void launch_gemm_i8(hipStream_t s, const int8_t *A, int lda, int M, const int8_t *W, int kpad,
                    int ncols, const int32_t *bias, const Requant &rq, int8_t *out, int ldc,
                    int8_t *out2, int ldc2) {
  launch_gemm<true>(s, A, lda, M, W, kpad, ncols, bias, rq, out, ldc, out2, ldc2);
}

// ---------------------------------------------------------------------------
// Cell kernel: one workgroup (256 threads) per batch row.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// Sums (s1, s2) over the workgroup; the result is returned to every thread.
__device__ __forceinline__ void block_sum2(int64_t &s1, int64_t &s2, int64_t *red /*[8]*/) {
  s1 = wave_sum_i64(s1);
  s2 = wave_sum_i64(s2);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();  // red may still be read from the previous use
  if (lane == 0) {
    red[wave] = s1;
    red[4 + wave] = s2;
  }
  __syncthreads();
  s1 = red[0] + red[1] + red[2] + red[3];
  s2 = red[4] + red[5] + red[6] + red[7];
}

__global__ __launch_bounds__(256) void cell_kernel(CellArgs a) {
  extern __shared__ __attribute__((aligned(16))) int16_t gs[];  // [4][N] with layer norm
  __shared__ int64_t red[8];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int N = a.N, G = a.G, first = 4 - G;
  const bool cifg = a.flags & 1u, ph = a.flags & 2u, ln = a.flags & 4u;
  const int16_t *tx = a.tx + (size_t)b * G * N;
  const int16_t *th = a.th + (size_t)b * G * N;
  int16_t *c = a.c + (size_t)b * N;
  const int32_t glo = ln ? -32767 : -32768;

  // gate sum of gate slot g at cell n (Secs. 3.2.4 / 3.2.5); cval is the cell
  // state the peephole reads (c^{t-1} for i and f, c^t for o)
  auto gate_sum = [&](int g, int n, int32_t cval) -> int32_t {
    const int col = (g - first) * N + n;
    int32_t v = (int32_t)tx[col] + (int32_t)th[col];
    if (ph && g != 2) {
      const int j = g == 3 ? 2 : g;
      v += sat16(rescale((int32_t)a.Pq[j * N + n] * cval, a.Mc[j], a.rc[j]));
    }
    return clamp_i32(v, glo, 32767);
  };
  auto trace16 = [&](int16_t *base, int g, int n, int32_t v) {
    if (base) base[((size_t)b * 4 + g) * N + n] = (int16_t)v;
  };

  if (!ln) {
    for (int n = tid; n < N; n += 256) {
      const int32_t cold = c[n];
      int32_t act[4];
      for (int g = first; g < 3; ++g) {
        const int32_t v = gate_sum(g, n, cold);
        trace16(a.tr_g, g, n, v);
        act[g] = g == 2 ? tanh_from_table(a.tanh_tab, v) : sigmoid_from_table(a.sig_tab, v);
      }
      if (cifg) act[0] = cifg_input_gate(act[1]);
      const int32_t cnew = cell_update(act[0], act[2], act[1], cold, a.m_c);
      const int32_t vo = gate_sum(3, n, cnew);
      trace16(a.tr_g, 3, n, vo);
      act[3] = sigmoid_from_table(a.sig_tab, vo);
      const int32_t mq = hidden_state(act[3], tanh_from_table(a.tanhc_tab, cnew), a.Mm, a.rm, a.zp_m);
      c[n] = (int16_t)cnew;
      a.m_out[(size_t)b * a.ld_m + n] = (int8_t)mq;
      if (a.m_out2) a.m_out2[(size_t)b * a.ld_m2 + n] = (int8_t)mq;
      for (int g = 0; g < 4; ++g) trace16(a.tr_act, g, n, act[g]);
      if (a.tr_c) a.tr_c[(size_t)b * N + n] = (int16_t)cnew;
      if (a.tr_m) a.tr_m[(size_t)b * N + n] = (int8_t)mq;
    }
    return;
  }

  // ---- layer norm: statistics over the N cells of each gate row (Sec. 3.2.6)
  __shared__ LnRow rows[4];
  const int last_early = ph ? 2 : 3;  // with a peephole, o waits for c^t
  for (int g = first; g <= last_early; ++g) {
    int64_t s1 = 0, s2 = 0;
    for (int n = tid; n < N; n += 256) {
      const int32_t v = gate_sum(g, n, c[n]);
      gs[g * N + n] = (int16_t)v;
      trace16(a.tr_g, g, n, v);
      s1 += v;
      s2 += (int64_t)v * v;
    }
    block_sum2(s1, s2, red);
    if (tid == 0) rows[g] = ln_row(s1, s2, N, a.inv_n);
  }
  __syncthreads();
  auto normed = [&](int g, int n) -> int32_t {
    const int32_t v = ln_apply(gs[g * N + n], rows[g], a.Lq[g * N + n], a.qb[g * N + n], a.Mln[g],
                               a.rln[g]);
    trace16(a.tr_ln, g, n, v);
    return v;
  };
  {
    int64_t s1 = 0, s2 = 0;
    for (int n = tid; n < N; n += 256) {
      int32_t i = 0;
      if (!cifg) i = sigmoid_from_table(a.sig_tab, normed(0, n));
      const int32_t f = sigmoid_from_table(a.sig_tab, normed(1, n));
      const int32_t z = tanh_from_table(a.tanh_tab, normed(2, n));
      if (cifg) i = cifg_input_gate(f);
      const int32_t cnew = cell_update(i, z, f, c[n], a.m_c);
      c[n] = (int16_t)cnew;  // read back below by this same thread only
      trace16(a.tr_act, 0, n, i);
      trace16(a.tr_act, 1, n, f);
      trace16(a.tr_act, 2, n, z);
      if (a.tr_c) a.tr_c[(size_t)b * N + n] = (int16_t)cnew;
      if (ph) {
        const int32_t v = gate_sum(3, n, cnew);
        gs[3 * N + n] = (int16_t)v;
        trace16(a.tr_g, 3, n, v);
        s1 += v;
        s2 += (int64_t)v * v;
      }
    }
    if (ph) {
      block_sum2(s1, s2, red);
      if (tid == 0) rows[3] = ln_row(s1, s2, N, a.inv_n);
      __syncthreads();
    }
  }
  for (int n = tid; n < N; n += 256) {
    const int32_t o = sigmoid_from_table(a.sig_tab, normed(3, n));
    const int32_t mq = hidden_state(o, tanh_from_table(a.tanhc_tab, c[n]), a.Mm, a.rm, a.zp_m);
    a.m_out[(size_t)b * a.ld_m + n] = (int8_t)mq;
    if (a.m_out2) a.m_out2[(size_t)b * a.ld_m2 + n] = (int8_t)mq;
    trace16(a.tr_act, 3, n, o);
    if (a.tr_m) a.tr_m[(size_t)b * N + n] = (int8_t)mq;
  }
}

void launch_cell(hipStream_t s, const CellArgs &a) {
  if (a.B <= 0) return;
  const size_t lds = (a.flags & 4u) ? (size_t)4 * a.N * sizeof(int16_t) : 0;
  hipLaunchKernelGGL(cell_kernel, dim3(a.B), dim3(256), lds, s, a);
}

// ---------------------------------------------------------------------------
// Small data-movement kernels
// ---------------------------------------------------------------------------
__global__ void copy_rows_i8_kernel(const int8_t *src, int ld_src, int8_t *dst, int ld_dst, int rows,
                                    int cols, int value, int fill) {
  const int64_t total = (int64_t)rows * ld_dst;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / ld_dst;
    const int col = (int)(i - r * ld_dst);
    dst[i] = col < cols ? (src ? src[r * ld_src + col] : (int8_t)value) : (int8_t)fill;
  }
}

// dst [rows, ld_dst] columns [0, cols) <- src [rows, cols]; the other columns of dst stay as they are
__global__ void place_cols_i8_kernel(const int8_t *src, int8_t *dst, int ld_dst, int64_t rows, int cols) {
  const int64_t total = rows * cols;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / cols;
    dst[r * ld_dst + (i - r * cols)] = src[i];
  }
}

// dst row (t, b) <- src row (T - 1 - t, b): the time flip at the two ends of a reverse run
__global__ void flip_rows_i8_kernel(const int8_t *src, int ld_src, int8_t *dst, int ld_dst, int T, int B, int cols,
                                    int fill) {
  const int64_t total = (int64_t)T * B * ld_dst;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / ld_dst;
    const int col = (int)(i - r * ld_dst);
    const int64_t t = r / B, b = r - t * B;
    dst[i] = col < cols ? src[((T - 1 - t) * B + b) * ld_src + col] : (int8_t)fill;
  }
}

static int grid_for(int64_t total) {
  int64_t g = (total + 255) / 256;
  return (int)(g < 1 ? 1 : (g > 4096 ? 4096 : g));
}

void launch_copy_rows_i8(hipStream_t s, const int8_t *src, int ld_src, int8_t *dst, int ld_dst,
                         int rows, int cols, int fill) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(copy_rows_i8_kernel, dim3(grid_for((int64_t)rows * ld_dst)), dim3(256), 0, s,
                     src, ld_src, dst, ld_dst, rows, cols, 0, fill);
}

void launch_place_cols_i8(hipStream_t s, const int8_t *src, int8_t *dst, int ld_dst, int64_t rows, int cols) {
  if (rows <= 0 || cols <= 0) return;
  hipLaunchKernelGGL(place_cols_i8_kernel, dim3(grid_for(rows * cols)), dim3(256), 0, s, src, dst, ld_dst, rows, cols);
}

void launch_flip_rows_i8(hipStream_t s, const int8_t *src, int ld_src, int8_t *dst, int ld_dst, int T, int B,
                         int cols, int fill) {
  if (T <= 0 || B <= 0) return;
  hipLaunchKernelGGL(flip_rows_i8_kernel, dim3(grid_for((int64_t)T * B * ld_dst)), dim3(256), 0, s, src, ld_src, dst,
                     ld_dst, T, B, cols, fill);
}

void launch_fill_rows_i8(hipStream_t s, int8_t *dst, int ld_dst, int rows, int cols, int value,
                         int fill) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(copy_rows_i8_kernel, dim3(grid_for((int64_t)rows * ld_dst)), dim3(256), 0, s,
                     (const int8_t *)nullptr, 0, dst, ld_dst, rows, cols, value, fill);
}

// Start of a layer on the persistent path, in one launch: the initial hidden
// state (given rows, or the code of real 0; padding bytes 0), the zeroed
// synchronization words, and -- to save a launch -- a pending copy of rows
// (the previous layer's final h on its way to the caller's state buffer).
// Workgroups [0, zero_blocks) clear, the next h_blocks write h, the rest copy.
__global__ void init_layer_kernel(LayerInit w) {
  layer_init_device(w, blockIdx.x * (long long)blockDim.x + threadIdx.x, (long long)gridDim.x * blockDim.x);
}

void launch_init_layer(hipStream_t s, const int8_t *h_src, int ld_src, int8_t *h0, int ld_h0, int rows, int cols,
                       int zp, void *sync, int64_t sync_bytes, const int8_t *c_src, int c_ld_src, int8_t *c_dst,
                       int c_cols) {
  LayerInit w;
  w.h_src = h_src; w.ld_src = ld_src; w.h0 = h0; w.ld_h0 = ld_h0; w.rows = rows; w.cols = cols; w.zp = zp;
  w.sync = static_cast<int4 *>(sync); w.sync_vec = sync_bytes / 16;  // a multiple of 16 bytes, 16-byte aligned
  w.c_src = c_src; w.c_ld_src = c_ld_src; w.c_dst = c_dst; w.c_cols = c_cols;
  const int64_t most = std::max<int64_t>(std::max<int64_t>(w.sync_vec, (int64_t)rows * ld_h0), c_dst ? (int64_t)rows * c_cols : 0);
  hipLaunchKernelGGL(init_layer_kernel, dim3(grid_for(most)), dim3(256), 0, s, w);
}

__global__ void copy_i16_kernel(const int16_t *src, int16_t *dst, int64_t n, int value) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src ? src[i] : (int16_t)value;
}

void launch_copy_i16(hipStream_t s, const int16_t *src, int16_t *dst, int64_t n) {
  if (n <= 0) return;
  hipLaunchKernelGGL(copy_i16_kernel, dim3(grid_for(n)), dim3(256), 0, s, src, dst, n, 0);
}

void launch_fill_i16(hipStream_t s, int16_t *dst, int64_t n, int value) {
  if (n <= 0) return;
  hipLaunchKernelGGL(copy_i16_kernel, dim3(grid_for(n)), dim3(256), 0, s, (const int16_t *)nullptr,
                     dst, n, value);
}

// Affine quantization of float features to int8 codes (Sec. 3.2.4): q = clamp(floor(v / s + 1/2) + zp),
// in double precision (division and addition are correctly rounded, no contraction).
__global__ void quantize_input_kernel(const float *x, int8_t *q, int64_t n, double s, int zp) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const double v = floor((double)x[i] / s + 0.5) + (double)zp;
    q[i] = v != v ? (int8_t)0 : (int8_t)(v < -128.0 ? -128.0 : (v > 127.0 ? 127.0 : v));
  }
}

void launch_quantize_input(hipStream_t s, const float *x, int8_t *q, int64_t n, double scale, int zp) {
  if (n <= 0) return;
  hipLaunchKernelGGL(quantize_input_kernel, dim3(grid_for(n)), dim3(256), 0, s, x, q, n, scale, zp);
}

__global__ void scatter_gates_kernel(const int16_t *src, int16_t *dst, int rows, int G, int N) {
  const int64_t per_row = (int64_t)G * N, total = rows * per_row;
  const int first = 4 - G;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / per_row;
    const int64_t col = i - r * per_row;  // gi * N + n
    dst[r * 4 * N + (int64_t)first * N + col] = src[i];
  }
}

void launch_scatter_gates(hipStream_t s, const int16_t *src, int16_t *dst, int rows, int G, int N) {
  if (rows <= 0) return;
  hipLaunchKernelGGL(scatter_gates_kernel, dim3(grid_for((int64_t)rows * G * N)), dim3(256), 0, s,
                     src, dst, rows, G, N);
}

}  // namespace lstm_int
