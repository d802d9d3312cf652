// Persistent recurrent path for gfx950 (MI355X).
//
//   in_gemm_kernel   W x for all (t, b) on the 32x32x32 int8 MFMA, rescaled to
//                    int16 (Secs. 3.2.4/3.2.5, zero point folded per Sec. 6)
//                    and stored in the tile order the recurrent kernel reads.
//                    This file holds the general version (any input depth);
//                    in_gemm.hip holds the one used for depths up to 1024.
//   rec_kernel       all T steps of one layer in ONE launch.  A group of GS
//                    workgroups (one per compute unit, all on one XCD, so they
//                    share an L2) owns rows_pg batch rows; each workgroup owns
//                    64 cells and keeps its slice of R in registers as MFMA
//                    operands for the whole sequence, and its slice of W_proj
//                    in LDS.  Per step: R h on the MFMA, gate sums, layer-norm
//                    statistics (summed per workgroup in LDS, then two 64-bit
//                    atomic adds per row and gate into words that also count
//                    their contributions, so readers need no barrier), sigma/tanh,
//                    cell update, hidden state, projection; groups synchronize
//                    through a counter in global memory.  Batch rows never
//                    interact, so groups run independently.
//                    A layer whose recurrent weights are 2:4 sparse has a form
//                    that runs R h on the sparse MFMA (rec_sparse_inst_*.hip).
//   rec16_kernel     the same step on groups of 16 rows (16x16x64 MFMA) for
//                    small batches: rec16_kernel.inc.h, rec16_inst.hip.
//
// Exchange between the workgroups of a group goes through buffers that are
// written once per step, in 128-byte cache lines that nothing has read before
// in the launch, so a compute unit's vector L1 cannot hold a stale copy: a
// step's h rows and m rows are multiples of 128 bytes and 128-byte aligned.
// Stores are complete (vmcnt(0)) before a workgroup arrives at the group
// barrier.
#include "persistent.h"

#include "lstm_int_math.h"

namespace lstm_int {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef unsigned long long u64;

constexpr int kPrmLdsBytes = 256;  // sizeof(PrmLds) in rec_kernel.inc.h

// ---------------------------------------------------------------------------
// Input GEMM: block = 128 (t,b) rows x 4 weight tiles (32 cells), 4 waves 2x2,
// each wave 64 rows x 2 tiles = 2x2 MFMA 32x32 blocks.  Weight tile rows are
// the MFMA's first operand: D[rho][row], rho = 8*gate + 4*(lane/32) + c.
// ---------------------------------------------------------------------------
// A staged k tile in LDS: rows of 64 bytes without padding, the 16-byte piece p of row r at position
// p ^ ((r >> 2) & 3): free of bank conflicts both for the operand reads of the 32x32x32 MFMA (row = lane % 32) and
// for the staging stores (four lanes per row), by the counters of a probe kernel; rows padded to 80 bytes kept the
// reads free and cost the stores twice their time.
__device__ __forceinline__ int in_gemm_piece(int row, int piece) { return row * 64 + ((piece ^ ((row >> 2) & 3)) << 4); }

__global__ __launch_bounds__(256) void in_gemm_kernel(InGemmArgs a) {
  constexpr int kTile = 2 * 128 * 64;  // one staged k tile: 128 activation rows, then 128 weight rows
  __shared__ __attribute__((aligned(16))) int8_t lds[2 * kTile];  // tile kt + 1 is stored while tile kt is multiplied
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row_base = blockIdx.x * 128;  // padded rows m' = t * Bp + b
  const int tile_base = blockIdx.y * 4;
  const int rows_total = a.T * a.Bp;

  // the two activation rows and two weight rows this thread stages per k tile; pointers and the registers the
  // next tiles wait in are named variables of plain vector type on purpose (as small arrays, or as HIP's int4 in a
  // struct, they were left in scratch memory, and the loads then no longer overlapped the MFMAs)
  const int c0 = tid, c1 = tid + 256;
  auto x_row = [&](int c) {
    int m = row_base + (c >> 2);
    m = m < rows_total ? m : rows_total - 1;
    const int t = m / a.Bp;
    int b = m - t * a.Bp;
    b = b < a.B ? b : a.B - 1;  // padded rows repeat the last real one; never read back
    return a.A + ((size_t)t * a.B + b) * a.lda + ((c & 3) << 4);
  };
  const int8_t *const xsrc0 = x_row(c0), *const xsrc1 = x_row(c1);
  const int8_t *const wsrc0 = a.W2 + ((size_t)tile_base * 32 + (c0 >> 2)) * a.kpad + ((c0 & 3) << 4);
  const int8_t *const wsrc1 = a.W2 + ((size_t)tile_base * 32 + (c1 >> 2)) * a.kpad + ((c1 & 3) << 4);
  const int dst0 = in_gemm_piece(c0 >> 2, c0 & 3), dst1 = in_gemm_piece(c1 >> 2, c1 & 3);

  v16i acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  const int KT = a.kpad >> 6;
  // tile t waits in register set t % 3 (sa, sb, sc) between its load and its LDS store
  v4i sa_x0 = {}, sa_x1 = {}, sa_w0 = {}, sa_w1 = {};
  v4i sb_x0 = {}, sb_x1 = {}, sb_w0 = {}, sb_w1 = {};
  v4i sc_x0 = {}, sc_x1 = {}, sc_w0 = {}, sc_w1 = {};
#define IN_GEMM_LOAD(st, kt)                                              \
  do {                                                                    \
    if ((kt) < KT) {                                                      \
      st##_x0 = *reinterpret_cast<const v4i *>(xsrc0 + ((kt) << 6));      \
      st##_x1 = *reinterpret_cast<const v4i *>(xsrc1 + ((kt) << 6));      \
      st##_w0 = *reinterpret_cast<const v4i *>(wsrc0 + ((kt) << 6));      \
      st##_w1 = *reinterpret_cast<const v4i *>(wsrc1 + ((kt) << 6));      \
    }                                                                     \
  } while (0)
#define IN_GEMM_STORE(st, buf)                                            \
  do {                                                                    \
    int8_t *xs_ = lds + (buf) * kTile, *ws_ = xs_ + 128 * 64;             \
    *reinterpret_cast<v4i *>(xs_ + dst0) = st##_x0;                       \
    *reinterpret_cast<v4i *>(xs_ + dst1) = st##_x1;                       \
    *reinterpret_cast<v4i *>(ws_ + dst0) = st##_w0;                       \
    *reinterpret_cast<v4i *>(ws_ + dst1) = st##_w1;                       \
  } while (0)
  // One k tile: tile kt + 1 goes from its registers (nx) into the LDS buffer tile kt - 1 was read from (every wave is
  // past the barrier that ended kt - 1), the freed registers request tile kt + 4, tile kt is multiplied out of the
  // other buffer: one barrier per tile, global loads three tiles ahead.
#define IN_GEMM_K_TILE(nx, kt)                                                                          \
  do {                                                                                                  \
    if ((kt) + 1 < KT) IN_GEMM_STORE(nx, ((kt) + 1) & 1);                                               \
    IN_GEMM_LOAD(nx, (kt) + 4);                                                                         \
    const int8_t *xs = lds + ((kt) & 1) * kTile, *wsb = xs + 128 * 64;                                  \
    _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                  \
      v4i xf[2], wf[2];                                                                                 \
      _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                                   \
        xf[i] = *reinterpret_cast<const v4i *>(xs + in_gemm_piece(wm * 64 + i * 32 + (lane & 31), kk * 2 + (lane >> 5))); \
        wf[i] = *reinterpret_cast<const v4i *>(wsb + in_gemm_piece(wn * 64 + i * 32 + (lane & 31), kk * 2 + (lane >> 5))); \
      }                                                                                                 \
      _Pragma("unroll") for (int ti = 0; ti < 2; ++ti)                                                  \
        _Pragma("unroll") for (int mi = 0; mi < 2; ++mi)                                                \
          acc[ti][mi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[ti], xf[mi], acc[ti][mi], 0, 0, 0);    \
    }                                                                                                   \
    __syncthreads();                                                                                    \
  } while (0)
  IN_GEMM_LOAD(sa, 0);
  IN_GEMM_LOAD(sb, 1);
  IN_GEMM_LOAD(sc, 2);
  IN_GEMM_STORE(sa, 0);
  __syncthreads();
  IN_GEMM_LOAD(sa, 3);
  for (int kt = 0; kt < KT; kt += 3) {
    IN_GEMM_K_TILE(sb, kt);
    if (kt + 1 < KT) IN_GEMM_K_TILE(sc, kt + 1);
    if (kt + 2 < KT) IN_GEMM_K_TILE(sa, kt + 2);
  }
#undef IN_GEMM_K_TILE
#undef IN_GEMM_STORE
#undef IN_GEMM_LOAD

  // epilogue: lane holds gates 0..3 x cells 4*(lane/32)+0..3 of row (lane%32)
#pragma unroll
  for (int ti = 0; ti < 2; ++ti) {
    const int tile = tile_base + wn * 2 + ti;
    int32_t bias[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int4 b4 =
          *reinterpret_cast<const int4 *>(a.bx2 + (size_t)tile * 32 + g * 8 + ((lane >> 5) << 2));
      bias[g * 4 + 0] = b4.x; bias[g * 4 + 1] = b4.y; bias[g * 4 + 2] = b4.z; bias[g * 4 + 3] = b4.w;
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
      const int m0 = row_base + wm * 64 + mi * 32;  // multiple of 32
      if (m0 >= rows_total) continue;
      int4 *dst = a.tx2 + (((size_t)(m0 >> 5) * a.tiles + tile) * 2) * 64 + lane;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        int32_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int idx = half * 8 + e;  // = 4 * gate + c
          const int g = idx >> 2;
          const int32_t s = acc[ti][mi][idx] + bias[idx];
          v[e] = sat16(a.all_hi ? rescale_ge32(s, a.M[g], a.r[g]) : rescale(s, a.M[g], a.r[g]));
        }
        int4 pk;
        pk.x = (v[0] & 0xFFFF) | (v[1] << 16);
        pk.y = (v[2] & 0xFFFF) | (v[3] << 16);
        pk.z = (v[4] & 0xFFFF) | (v[5] << 16);
        pk.w = (v[6] & 0xFFFF) | (v[7] << 16);
        dst[half * 64] = pk;
      }
    }
  }
}

void launch_in_gemm(hipStream_t s, const InGemmArgs &a) {
  if (a.T <= 0 || a.B <= 0) return;
  dim3 grid((a.T * a.Bp + 127) / 128, a.tiles / 4);
  hipLaunchKernelGGL(in_gemm_kernel, grid, dim3(256), 0, s, a);
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static const int kKS[] = {8, 20, 32};

bool rec_supported(int N, int H, int flags, int B, int *ks, int *rt, int *groups) {
  if (N % 8 != 0 || N > 2048 || B < 1) return false;
  if (!(flags & 8) && H != N) return false;
  const int GS = (N + 63) / 64;
  const int need = (((H + 127) / 128) * 128) / 32;  // Hpad / 32
  int k = 0;
  for (int cand : kKS)
    if (!k && cand >= need) k = cand;
  if (!k) return false;
  const int max_groups = 8 * (32 / GS);
  // 64 rows per group when 32 would need more than one launch; the largest
  // register-resident slice (k = 32) leaves no room for the second row tile
  int r = ((B + 31) / 32 > max_groups && k < 32) ? 2 : 1;
  int g = (B + 32 * r - 1) / (32 * r);
  if (g > max_groups) g = max_groups;  // the rest of the batch goes to further launches
  *ks = k;
  *rt = r;
  *groups = g;
  return true;
}

size_t rec_lds_bytes(const RecArgs &a) {
  const int items = (a.rows_pg / 32) * 128;
  const bool proj = a.flags & 8;
  size_t tile = (((size_t)a.rows_pg * (a.ks * 32 + 16) + 1023) / 1024 + 1) * 1024;
  if (proj && tile < 4 * 16 * 64 * 4) tile = 4 * 16 * 64 * 4;
  size_t n = tile + (size_t)items * 8 + (size_t)items * sizeof(LnRow2) + 2 * 4 * 64 * 8 + 4 * 64 * 2 + 4 * 64 * 4 +
             kPrmLdsBytes + 16 + 16 * 8 + 3 * 32 /* LutLds */;
  for (int i = 0; i < 3; ++i)
    if (i < 2 || a.lut[2].blob != a.lut[1].blob) n += (size_t)lut_wide_lds_bytes(a.lut[i].dom, a.lut[i].sh, a.lut[i].tail != 0);
  if (proj) {
    const int per_cu = (a.ptiles + a.GS - 1) / a.GS;
    n += ((size_t)per_cu * a.prow * (a.npadp + 16) + 1023) / 1024 * 1024;  // loaded in whole 1 KB chunks
  }
  return n;
}

typedef void (*rec_fn)(RecArgs);
rec_fn rec_pick_8(int rt, int fl);   // rec_inst_8.hip
rec_fn rec_pick_20(int rt, int fl);  // rec_inst_20.hip
rec_fn rec_pick_32(int rt, int fl);  // rec_inst_32.hip
rec_fn rec_pick_sparse_8(int fl);   // rec_sparse_inst_8.hip
rec_fn rec_pick_sparse_20(int fl);  // rec_sparse_inst_20.hip
rec_fn rec_pick_sparse_32(int fl);  // rec_sparse_inst_32.hip
static rec_fn pick_sparse(int ks, int fl) {
  if (ks == 8) return rec_pick_sparse_8(fl);
  if (ks == 20) return rec_pick_sparse_20(fl);
  if (ks == 32) return rec_pick_sparse_32(fl);
  return nullptr;
}
static rec_fn pick(int ks, int rt, int fl) {
  if (ks == 8) return rec_pick_8(rt, fl);
  if (ks == 20) return rec_pick_20(rt, fl);
  if (ks == 32) return rec_pick_32(rt, fl);
  return nullptr;
}

hipError_t rec_init() {
  for (int ks : kKS)
    for (int rt = 1; rt <= 2; ++rt)
      for (int fl = 0; fl < 16; ++fl) {
        rec_fn fn = pick(ks, rt, fl);
        if (!fn) continue;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
      }
  for (int ks : kKS)
    for (int fl = 0; fl < 16; ++fl) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_sparse(ks, fl)),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

hipError_t launch_rec(hipStream_t s, const RecArgs &a, bool cooperative) {
  const int fl = (a.flags & 7) | ((a.flags & 8) ? 0 : 8);  // bit 3: no projection
  if (a.sparse && a.rows_pg != 32) return hipErrorInvalidValue;
  rec_fn fn = a.sparse ? pick_sparse(a.ks, fl) : pick(a.ks, a.rows_pg / 32, fl);
  if (!fn) return hipErrorInvalidValue;
  const int slots = a.GS * ((a.groups + 7) / 8);
  RecArgs args = a;
  void *params[] = {&args};
  // The kernel needs all its workgroups resident at once (one per compute unit).  A cooperative launch
  // has the runtime guarantee that, at 16-18 us per launch (measured); a plain launch gets it from the
  // in-order stream on a device nothing else occupies.  If the workgroups do not all arrive, the bounded
  // waits give up and raise the status word: an error, not a hang.
  if (cooperative)
    return hipLaunchCooperativeKernel(reinterpret_cast<const void *>(fn), dim3(8 * slots), dim3(256), params,
                                      (unsigned)rec_lds_bytes(a), s);
  return hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(8 * slots), dim3(256), params,
                         (unsigned)rec_lds_bytes(a), s);
}

}  // namespace lstm_int
