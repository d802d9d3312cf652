// The 16-row recurrent kernel: host side (the instantiations are in rec16_inst_4/10/16.hip).
#include "persistent.h"

#include "lstm_int_math.h"

namespace lstm_int {

static const int kKS16[] = {4, 10, 16};

typedef void (*rec_fn)(RecArgs);
rec_fn rec16_pick_4(int fl);   // rec16_inst_4.hip
rec_fn rec16_pick_10(int fl);  // rec16_inst_10.hip
rec_fn rec16_pick_16(int fl);  // rec16_inst_16.hip
static rec_fn pick16(int ks16, int fl) {
  if (ks16 == 4) return rec16_pick_4(fl);
  if (ks16 == 10) return rec16_pick_10(fl);
  if (ks16 == 16) return rec16_pick_16(fl);
  return nullptr;
}

bool rec16_supported(int N, int H, int flags, int B, int *ks16, int *groups) {
  if (N % 8 != 0 || N > 2048 || B < 1) return false;
  if (!(flags & 8) && H != N) return false;
  const int GS = (N + 63) / 64;
  const int need = (((H + 127) / 128) * 128 + 63) / 64;
  int k = 0;
  for (int cand : kKS16)
    if (!k && cand >= need) k = cand;
  if (!k) return false;
  const int max_groups = 8 * (32 / GS);
  const int g = (B + 15) / 16;
  if (g > max_groups) return false;  // larger batches take the 32-row kernel
  *ks16 = k;
  *groups = g;
  return true;
}

size_t rec16_lds_bytes(const RecArgs &a) {
  const int items = 64;
  const bool proj = a.flags & 8;
  size_t tile = (((size_t)16 * (a.ks16 * 64 + 16) + 1023) / 1024 + 1) * 1024;
  if (proj && tile < 4 * 2 * 4 * 64 * 4) tile = 4 * 2 * 4 * 64 * 4;
  size_t n = tile + (size_t)items * 8 + (size_t)items * sizeof(LnRow2) + 2 * 4 * 64 * 8 + 4 * 64 * 4 + 4 * 64 * 2 +
             256 /* PrmLds */ + 16 + 16 * 8 + 3 * 32 /* LutLds */;
  for (int i = 0; i < 3; ++i)
    if (i < 2 || a.lut[2].blob != a.lut[1].blob) n += (size_t)lut_wide_lds_bytes(a.lut[i].dom, a.lut[i].sh, a.lut[i].tail != 0);
  if (proj) {
    const int per_cu = (a.ptiles + a.GS - 1) / a.GS;
    n += ((size_t)per_cu * 32 * (a.npadp + 16) + 1023) / 1024 * 1024;  // loaded in whole 1 KB chunks
  }
  return n;
}

hipError_t rec16_init() {
  for (int ks : kKS16)
    for (int fl = 0; fl < 8; ++fl) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick16(ks, fl)),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
    }
  return hipSuccess;
}

hipError_t launch_rec16(hipStream_t s, const RecArgs &a, bool cooperative) {
  rec_fn fn = pick16(a.ks16, a.flags & 7);
  if (!fn || !a.R2h) return hipErrorInvalidValue;
  const int slots = a.GS * ((a.groups + 7) / 8);
  RecArgs args = a;
  void *params[] = {&args};
  if (cooperative)
    return hipLaunchCooperativeKernel(reinterpret_cast<const void *>(fn), dim3(8 * slots), dim3(256), params,
                                      (unsigned)rec16_lds_bytes(a), s);
  return hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(8 * slots), dim3(256), params,
                         (unsigned)rec16_lds_bytes(a), s);
}

}  // namespace lstm_int
