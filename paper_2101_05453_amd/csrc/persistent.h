// Launch interface of the persistent recurrent path (gfx950): the input GEMM
// that writes the W x terms in the tile order of the recurrent kernel, and the
// recurrent kernel itself, which runs all T steps of one layer in one launch
// with the recurrent weights resident in registers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lstm_int_math.h"

namespace lstm_int {

// Tile order shared by the two kernels.  Cells are taken in tiles of 8; the 32
// weight rows of a tile are ordered rho = 8*gate + cell_in_tile, which makes a
// 32x32 MFMA leave each lane with all four gates of four cells of one batch
// row.  The W x terms of (t, b) are stored as int16 in
//   tx2[(t*Bp + b) / 32][cell tile][half][lane][8]
// with lane = b % 32 + 32 * ((cell % 8) / 4), half 0 = gates i,f, half 1 =
// gates z,o, and the 8 values = [gate in half][cell % 4].
// What has to be in place before a layer's recurrent kernel starts: the initial h (given, or the zero
// point), cleared synchronization words, and -- to save a launch -- a pending copy of rows (the previous
// layer's final h on its way to the caller's state buffer).  Done by its own small kernel, or by the
// workgroups of the input GEMM ahead of their own work (grid-stride over all threads of the launch).
struct LayerInit {
  const int8_t *h_src;  // [rows, ld_src] or NULL (zero point)
  int ld_src;
  int8_t *h0;           // [rows, ld_h0], columns >= cols zeroed
  int ld_h0, rows, cols, zp;
  int4 *sync;           // sync_vec 16-byte words to clear
  long long sync_vec;
  const int8_t *c_src;  // pending copy [rows, c_cols] from rows of stride c_ld_src, or c_dst == NULL
  int c_ld_src;
  int8_t *c_dst;
  int c_cols;
};
__device__ __forceinline__ void layer_init_device(const LayerInit &w, long long gtid, long long gthreads) {
  for (long long i = gtid; i < w.sync_vec; i += gthreads) w.sync[i] = int4{0, 0, 0, 0};
  const long long total = (long long)w.rows * w.ld_h0;
  for (long long i = gtid; i < total; i += gthreads) {
    const long long r = i / w.ld_h0;
    const int col = (int)(i - r * w.ld_h0);
    w.h0[i] = col < w.cols ? (w.h_src ? w.h_src[r * w.ld_src + col] : (int8_t)w.zp) : (int8_t)0;
  }
  if (w.c_dst) {
    const long long ctotal = (long long)w.rows * w.c_cols;
    for (long long i = gtid; i < ctotal; i += gthreads) {
      const long long r = i / w.c_cols;
      const int col = (int)(i - r * w.c_cols);
      w.c_dst[i] = w.c_src[r * w.c_ld_src + col];
    }
  }
}

struct InGemmArgs {
  const int8_t *A;  // activations [T*B, lda]
  int a_slack;       // the buffer is readable for 31 more rows behind row T*B - 1 (launch_in_gemm_ws needs it
                     // when B is no multiple of 32: the padded rows of the last row block read them)
  int lda, T, B, Bp;
  const int8_t *W2;  // [tiles][32][kpad] tile-ordered weight rows
  const int8_t *W2f; // the same as MFMA operands [tiles][kpad / 32][64 lanes][16]: lane = row + 32 * (k / 16 % 2)
                     // holds bytes k % 16 of k step k / 32 (launch_in_gemm_ws reads this one)
  int kpad, tiles;   // tiles % 4 == 0
  const int32_t *bx2;  // [tiles][32]
  int32_t M[4], r[4], all_hi;
  int4 *tx2;
  // filled by launch_in_gemm_ws
  int pre;            // operand treatment of the rescale: 0 none, 1 left shift, 2 clamp and left shift
  int parts;          // row partitions
  int gp;             // part groups over the 8 XCDs (1, 2, 4 or 8; 0 on entry = chosen by the launch; 0 in the
                      // kernel = workgroup id -> (id % parts, id / parts))
  RescaleHi rs[4];    // per gate, prepared from (M, r)
  int has_init;       // launch_in_gemm_ws only: the workgroups do `init` before their own work
  LayerInit init;
};
// one workgroup per 128 rows x 4 tiles, operands staged per 64-byte k tile
// (any k depth, any shifts)
void launch_in_gemm(hipStream_t s, const InGemmArgs &a);
// weights resident in registers (in_gemm.hip); needs in_gemm_ws_supported(a)
hipError_t in_gemm_init();
bool in_gemm_ws_supported(const InGemmArgs &a);
void launch_in_gemm_ws(hipStream_t s, const InGemmArgs &a, int num_cus);

// One activation table as the persistent kernels keep it in LDS: a prefix of `dom` entries of the table's wide form
// (lstm_int_math.h), and the tail part if lookups at and beyond dom can differ from entry dom - 1.
struct LutWide {
  const uint8_t *blob;  // [kLutWideBytes], global memory
  int32_t sh;           // block shift of the encoding
  int32_t dom;          // entries kept, a multiple of 1024 (the launch chooses it from its LDS budget)
  int32_t tail;         // 1: the tail part is kept (needs dom >= 16384); 0: the table is flat from dom - 1 on
  int32_t pad_;
};

// Layer-norm statistics words of one group of workgroups: [set][round][sum q | sum q^2][item], 64 bits each.  In
// rec_kernel and stack_kernel the group's workgroups add into two sets of words, even members into set 0 and odd
// members into set 1, and every reader adds the two up: half as many atomic adds meet in each cache line (measured at
// 32 workgroups per group: 0.19 us per step; four sets were no better than two, with twice the words to poll).
// Groups of fewer than 16 workgroups keep to one set there (the second set's polls cost more than they save), and
// so does rec16_kernel at any group size.
constexpr int kStatSetWords = 2 * 2 * 256;
constexpr int kStatGroupWords = 2 * kStatSetWords;
__host__ __device__ inline bool stat_two_sets(int GS) { return GS >= 16; }

struct RecArgs {
  int T, B, N, H, Hpad, flags, m_c;
  int GS;         // workgroups (compute units) per group = cells / 64
  int groups;     // groups in this launch, each owns rows_pg batch rows
  int batch0;     // first batch row of this launch
  int rows_pg;    // 32 * RT
  int ks;         // 32-wide k steps held in registers (template KS)
  int Ncp;        // GS * 64
  int Bp;         // B rounded up to 32
  const int4 *R2;      // [GS][4 waves][2 tiles][ks][64 lanes] 16 bytes each (sparse != 0: see rec_sparse_bytes)
  const int4 *R2h;     // 16-row kernel: [GS][4 waves][4 tiles][ks16][64 lanes] 16 bytes each
  int ks16;            // 16-row kernel: 64-wide k steps held in registers
  const int32_t *bh4;  // [4][Ncp]
  const int16_t *Lq4;  // [4][Ncp]
  const int32_t *qb4;  // [4][Ncp]
  const int16_t *Pq3;  // [3][Ncp]
  int32_t Mh[4], rh[4];
  int32_t pre_h;  // operand treatment of the R h rescale: 0 none, 1 left shift, 2 clamp and left shift
  int32_t Mc[3], rc[3];
  int32_t Mln[4], rln[4];
  int32_t Mm, rm, zp_m;
  LutWide lut[3];  // sigma and tanh of the gate format Q3.12, tanh of the cell format (the same blob as the
                   // gate tanh when the formats agree: one copy serves both; the stacked kernel takes the third
                   // from its layer record)
  // projection
  const int8_t *Wp2;   // [ptiles][32][npadp]
  const int32_t *bp2;  // [ptiles][32]
  int ptiles, npadp;
  int prow;            // rec_kernel: output rows per projection tile (4..32, a multiple of 4): tile p holds the
                       // outputs [p * prow, p * prow + prow) in its first prow rows; the other kernels use 32
  int32_t Mp, rp, zp_h;
  // data
  const int4 *tx2;
  const int8_t *h0;  // [B, Hpad]
  int8_t *out;       // [T, B, Hpad]
  int8_t *y;         // [T, B, H] or NULL
  int8_t *mbuf;      // [T][Bp / 32][npadp / 32][32 rows][32 cells] (projection only)
  const int16_t *c_in;  // [B, N] or NULL (zeros)
  int16_t *c_out;       // [B, N] or NULL
  // synchronization scratch, zeroed before the launch
  unsigned *counters;          // [groups][64]
  unsigned long long *tickets; // plain launch: [8 XCDs][32], word 0 of each (zeroed with the counters) sums up
                               // the workgroups that ran there (rec_kernel.inc.h); NULL = cooperative launch
  unsigned long long *acc;     // [groups][kStatGroupWords]
  int *status;                 // [0] != 0: a wait gave up or the placement check failed
  int spin_limit;
  int poll_sleep, stats_sleep;  // pauses between two polls of a barrier / of the statistics words, x 64 clocks
  int stats_first_sleep;  // pause before the first poll of the statistics words
  int sync_sleep;  // pause before the first poll of the barrier at which all workgroups arrive together
  int idle_sleep, idle_poll_sleep;  // workgroups without a projection tile, at the barrier after the projection:
                                    // pause before the first poll, and between polls
  long long *ticks;  // NULL, or [16] phase timers of workgroup 0 (diagnostics)
  int extra_arrivals;  // 0; tests set 1: every group barrier then waits for an arrival that never comes, so that
                       // the bounded waits give up (and every workgroup leaves the kernel) on demand
  int sparse;  // rec_kernel, 32 rows per group: R2 holds the recurrent weights in the 2:4 compressed form below
};

// Recurrent weights with at most two nonzeros in every aligned group of four along k (the pruned models of
// Table 1 in their structured form) as operands of the sparse MFMA v_smfmac_i32_32x32x64_i8, which takes a
// 64-deep k step in the time the dense 32x32x32 instruction takes a 32-deep one:
//   values  [GS][4 waves][2 tiles][ks / 2][64 lanes] 16 bytes,
//   indices [GS][4 waves][2 tiles][ks / 2][64 lanes] 4 bytes, behind all the values.
// Lane = rho + 32 * a (rho = the tile row, as in R2) holds, for k step q, the groups of four
//   k = 64 q + (j < 4 ? 0 : 32) + 16 a + 4 (j % 4) + 0..3,   j = 0..7,
// as value bytes 2 j and 2 j + 1 (the group's two kept weights; a group with fewer nonzeros is filled with
// zeros at other positions) and index bits [4 j + 1 : 4 j], [4 j + 3 : 4 j + 2] (their positions in the group).
// The other operand is dense: lane (row, b) holds k = 64 q + 32 b + 0..31 (layout checked on the device against
// a host product).
inline size_t rec_sparse_bytes(int GS, int ks) { return (size_t)GS * 4 * 2 * (ks / 2) * 64 * (16 + 4); }

// Whether a layer shape can take the persistent path; fills ks and rt.
bool rec_supported(int N, int H, int flags, int B, int *ks, int *rt, int *groups);
// Dynamic LDS bytes of the recurrent kernel for these arguments.
size_t rec_lds_bytes(const RecArgs &a);
// Returns hipSuccess or the launch error.
hipError_t launch_rec(hipStream_t s, const RecArgs &a, bool cooperative);
// One-time per process: raises the kernels' dynamic LDS limits.
hipError_t rec_init();

// The same step for groups of 16 batch rows (rec16_kernel.inc.h): batches of up to 16 * 8 * (32 / GS) rows in
// one launch.  mbuf is
// [T][Bp / 16][npadp / 64][16 rows][64 cells] here.
bool rec16_supported(int N, int H, int flags, int B, int *ks16, int *groups);
size_t rec16_lds_bytes(const RecArgs &a);
hipError_t launch_rec16(hipStream_t s, const RecArgs &a, bool cooperative);
hipError_t rec16_init();

// ---------------------------------------------------------------------------
// Stacked layers in one launch (stack_kernel.inc.h): layer l of a stack of up to 8 equal layers runs on
// XCD l, all at once, each on its own step -- while layer l works on step t, layer l + 1 works on step
// t - 1 (the layers of Sec. 7's stack are loops over the same cell, and step t of layer l + 1 needs only
// step t of layer l).  The batch is walked in row tiles of 32, one (step, tile) item after the other.
// Nothing is hoisted: the W x term of an item is computed when the layer's input for it arrives, with the
// weights W streamed from memory as MFMA operands (R stays resident in registers as in rec_kernel).
// A layer's h rows reach the next XCD through stores that write through the L2 and a flag per
// (layer, row tile) that counts the finished steps.
struct StackLayer {  // constants of one layer, in device memory (uploaded when the model is prepared)
  const int4 *R2;       // as RecArgs
  const int8_t *W2f;    // input weights in MFMA operand order [GS * 8 tiles][kx][64 lanes][16]
  const int32_t *bx2;   // [GS * 8 tiles][32] folded input bias, tile row order
  const int32_t *bh4;
  const int16_t *Lq4;
  const int32_t *qb4;
  const int16_t *Pq3;
  const int8_t *Wp2;
  const int32_t *bp2;
  LutWide lutc;         // tanh of the layer's cell format: wide blob and the prefix its LDS copy keeps
  int32_t kx;           // 32-byte k steps of W x (padded input width / 32), at most the kernel's KS
  int32_t pad0_;
  int32_t Mx[4], rx[4], pre_x;
  int32_t Mh[4], rh[4], pre_h;
  int32_t Mc[3], rc[3];
  int32_t Mln[4], rln[4];
  int32_t Mm, rm, zp_m, Mp, rp, zp_h, m_c;
  int32_t pad1_;
};

struct StackArgs {
  RecArgs c;                 // shape, options and tables common to the layers (per-layer fields unused)
  const StackLayer *layers;  // [L]
  int L;                     // layers in this launch, at most 8
  int row_tiles;             // ceil(B / 32)
  const int8_t *x;           // input of the first layer [T * B, ldx]
  int ldx;
  int x_shared;              // 1: x was written by an earlier launch (plain loads); layers > 0 always read
                             // the previous layer's rows with loads that bypass the L2
  int8_t *out_base;          // layer l writes [T, B, Hpad] at out_base + l * out_stride
  size_t out_stride;
  const int8_t *h0_base;     // initial h of layer l, [B, Hpad], at h0_base + l * B * Hpad
  int8_t *mbuf_base;         // m exchange buffer of layer l at + l * mbuf_stride (projection only)
  size_t mbuf_stride;
  int16_t *c_base;           // running cell state of layer l, [B, N], at + l * B * N (the caller's state
                             // buffer, or workspace)
  int c_given;               // 0: the cell state starts from zero, 1: from c_base
  int8_t *h_final;           // NULL, or the caller's h state: layer l's last h, [B, H], at + l * B * H
  unsigned *flags;           // [L][row_tiles] words 128 bytes apart, zeroed: steps finished
  int lutc_lds_bytes;        // LDS bytes of the largest cell-format tanh copy among the layers (0: all share the
                             // gate tanh table's copy); host side of the LDS budget
  int flag_sleep;            // pause between two polls of a flag, x 64 clocks
  int tick_layer;            // the layer whose workgroup 0 fills the phase timers (diagnostics)
  int prefetch_lines;        // 128-byte lines of a wave's slice of W asked for ahead of W x (at most 16 * kx)
};

struct StackInit {
  const int8_t *h_src;  // NULL, or the caller's h state: layer l is [rows, cols] at + l * rows * cols
  int8_t *h0;           // [L][rows, ld_h0]
  int ld_h0, rows, cols, L;
  int zp[8];            // code of real 0 per layer (h_src == NULL)
  int4 *sync;           // sync_vec 16-byte words to clear
  long long sync_vec;
};
void launch_stack_init(hipStream_t s, const StackInit &w);

// Whether `L` equal layers of this shape can run as a stack launch; ks = the kernel's k depth.
bool stack_supported(int N, int H, int flags, int ipad0, int L, int T, int B, int *ks);
size_t stack_lds_bytes(const StackArgs &a);
hipError_t launch_stack(hipStream_t s, const StackArgs &a, bool cooperative);
hipError_t stack_init();

}  // namespace lstm_int
