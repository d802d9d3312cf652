// Host side of the stacked recurrent kernel (stack_kernel.inc.h): eligibility,
// LDS budget, launch, and the kernel that sets a stack launch up.
#include "persistent.h"

#include "lstm_int_math.h"

namespace lstm_int {

typedef void (*stack_fn)(StackArgs);
stack_fn stack_pick_8(int fl, bool one);   // stack_inst_8.hip
stack_fn stack_pick_20(int fl, bool one);  // stack_inst_20.hip
stack_fn stack_pick_32(int fl, bool one);  // stack_inst_32.hip

static const int kStackKS[] = {8, 20, 32};

// one = the variant for launches of one item per layer (one step, one row tile)
static stack_fn pick(int ks, int fl, bool one) {
  if (ks == 8) return stack_pick_8(fl, one);
  if (ks == 20) return stack_pick_20(fl, one);
  if (ks == 32) return stack_pick_32(fl, one);
  return nullptr;
}

bool stack_supported(int N, int H, int flags, int ipad0, int L, int T, int B, int *ks) {
  if (L < 1 || L > 8 || T < 1 || B < 1) return false;
  if (N % 8 != 0 || N > 2048) return false;
  if (!(flags & 8) && H != N) return false;
  const int hpad = (H + 127) / 128 * 128;
  int k = 0;
  for (int cand : kStackKS)
    if (!k && cand * 32 >= hpad) k = cand;
  if (!k) return false;
  // the input rows of every layer go through the same LDS tile as the h rows
  const int ipad = (H + 63) / 64 * 64;  // layers above the first read the layer below
  if (ipad0 > k * 32 || ipad0 % 64 != 0 || (L > 1 && ipad > k * 32)) return false;
  // the statistics words of the kernel count up over the launch
  const int64_t items = (int64_t)T * ((B + 31) / 32);
  if (items > (1 << 14)) return false;
  *ks = k;
  return true;
}

size_t stack_lds_bytes(const StackArgs &sa) {
  const RecArgs &a = sa.c;
  const int items = 128;
  const bool proj = a.flags & 8;
  size_t tile = (((size_t)32 * (a.ks * 32 + 16) + 1023) / 1024 + 1) * 1024;
  if (proj && tile < 4 * 16 * 64 * 4) tile = 4 * 16 * 64 * 4;
  size_t n = tile + (size_t)items * 8 + (size_t)items * sizeof(LnRow2) + 2 * 4 * 64 * 8 + 4 * 64 * 2 + 4 * 64 * 4 +
             8 * 32 * 4 + 320 /* StkPrm */ + 16 + 12 * 8 + 3 * 32 /* LutLds */;
  for (int i = 0; i < 2; ++i) n += (size_t)lut_wide_lds_bytes(a.lut[i].dom, a.lut[i].sh, a.lut[i].tail != 0);
  n += (size_t)sa.lutc_lds_bytes;  // the largest cell-format copy among the layers
  if (proj) {
    const int per_cu = (a.ptiles + a.GS - 1) / a.GS;
    n += ((size_t)per_cu * a.prow * (a.npadp + 16) + 1023) / 1024 * 1024;
  }
  return n;
}

hipError_t stack_init() {
  for (int ks : kStackKS)
    for (int fl = 0; fl < 32; ++fl) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick(ks, fl & 15, fl >= 16)),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

// Everything a stack launch needs in place: the initial h of every layer ([B, Hpad], given rows or the
// layer's zero point, padding bytes 0) and the zeroed synchronization words and flags.
__global__ void stack_init_kernel(StackInit w) {
  const long long gtid = blockIdx.x * (long long)blockDim.x + threadIdx.x, gthreads = (long long)gridDim.x * blockDim.x;
  for (long long i = gtid; i < w.sync_vec; i += gthreads) w.sync[i] = int4{0, 0, 0, 0};
  const long long per_layer = (long long)w.rows * w.ld_h0, total = per_layer * w.L;
  for (long long i = gtid; i < total; i += gthreads) {
    const int l = (int)(i / per_layer);
    const long long j = i - l * per_layer;
    const long long r = j / w.ld_h0;
    const int col = (int)(j - r * w.ld_h0);
    w.h0[i] = col < w.cols ? (w.h_src ? w.h_src[((long long)l * w.rows + r) * w.cols + col] : (int8_t)w.zp[l]) : (int8_t)0;
  }
}

void launch_stack_init(hipStream_t s, const StackInit &w) {
  const long long most = w.sync_vec > (long long)w.rows * w.ld_h0 * w.L ? w.sync_vec : (long long)w.rows * w.ld_h0 * w.L;
  long long blocks = (most + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(stack_init_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w);
}

hipError_t launch_stack(hipStream_t s, const StackArgs &sa, bool cooperative) {
  const RecArgs &a = sa.c;
  stack_fn fn = pick(a.ks, (a.flags & 7) | ((a.flags & 8) ? 0 : 8), a.T == 1 && sa.row_tiles == 1);
  if (!fn || sa.L < 1 || sa.L > 8) return hipErrorInvalidValue;
  StackArgs args = sa;
  void *params[] = {&args};
  // one workgroup per compute unit, GS per XCD: all of them have to be resident at once (see launch_rec)
  const dim3 grid(8 * a.GS);
  if (cooperative)
    return hipLaunchCooperativeKernel(reinterpret_cast<const void *>(fn), grid, dim3(256), params,
                                      (unsigned)stack_lds_bytes(sa), s);
  return hipLaunchKernel(reinterpret_cast<const void *>(fn), grid, dim3(256), params, (unsigned)stack_lds_bytes(sa), s);
}

}  // namespace lstm_int
