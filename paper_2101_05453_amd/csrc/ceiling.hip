// Measurement aids.
// 1. For the input GEMM's roofline: what the chip sustains when every compute unit issues
// int8 MFMAs back to back from registers AND streams results to HBM at a given ratio of bytes per MFMA.
// The hoisted input GEMM (in_gemm.hip) needs 40 MFMAs and 4 KB of int16 output per wave and block of 32
// rows at the benchmark shape, which puts it at the ridge of the int8 MFMA and HBM rooflines; this kernel
// has the same mix with nothing else in it (no operand loads, no LDS), so its rate is the ceiling any
// schedule of that mix can reach at the clock the chip holds under that load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lstm_int.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMfmaPerBlock = 40;  // 2 tiles x 20 k steps: one block of 32 rows at input width 640

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void ceiling_kernel(
    int blocks, int stores_per_block, v4i *out, size_t out_vec, unsigned long long *clocks) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  v4i a = {tid, tid * 3, tid * 5, tid * 7}, b = {tid * 11, tid * 13, tid * 17, tid * 19};
  v16i acc[2];
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[0][v] = acc[1][v] = 0;
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  size_t pos = ((size_t)blockIdx.x * 4 + wave) * 64 * 8 + lane;  // 8 stores of 1 KB per wave and block at most
  const size_t stride = (size_t)gridDim.x * 4 * 64 * 8;
  for (int i = 0; i < blocks; ++i) {
#pragma unroll
    for (int k = 0; k < kMfmaPerBlock / 2; ++k) {
      acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[1], 0, 0, 0);
    }
    for (int s = 0; s < stores_per_block; ++s) {
      size_t p = pos + (size_t)s * 64;
      if (p >= out_vec) p -= out_vec;  // the buffer is at least one round of all workgroups large
      __builtin_nontemporal_store(v4i{a.x + i, b.y + s, i, s}, out + p);
    }
    pos += stride;
    if (pos >= out_vec) pos -= out_vec;
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  if (blockIdx.x == 0 && tid == 0) {
    clocks[0] = c1 - c0;
    clocks[1] = w1 - w0;
  }
  // keep the accumulators alive
  if (acc[0][0] == 0x7fffffff && acc[1][3] == 0x12345) out[0] = v4i{acc[0][1], acc[1][1], 0, 0};
}

// 2. For the LDS layouts of the matmul kernels: what a lane -> address map costs in LDS clocks (bank conflicts), read
// from the hardware counters of the launch.  Every address stays inside the array: row < 32, stride <= 128 words,
// piece < 4.
constexpr int kProbeIters = 4096;
__global__ __launch_bounds__(256) void lds_probe_kernel(int map, int stride_words, int swizzle, int write, int *sink) {
  __shared__ __attribute__((aligned(16))) int lds[4 * 32 * 128];  // 64 KB: four waves x 32 rows x 128 words
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 4 * 32 * 128; i += 256) lds[i] = i;
  __syncthreads();
  int row, piece;
  if (map == 0) {
    row = lane & 15;
    piece = lane >> 4;
  } else if (map == 1) {
    row = lane & 31;
    piece = lane >> 5;
  } else {
    row = lane >> 2;
    piece = lane & 3;
  }
  const int sw = swizzle == 1 ? (row >> 1) & 3 : (swizzle == 2 ? (row >> 2) & 3 : 0);
  v4i *p = reinterpret_cast<v4i *>(lds + wave * 32 * stride_words + row * stride_words + ((piece ^ sw) << 2));
  v4i acc = {0, 0, 0, 0};
  for (int i = 0; i < kProbeIters; ++i) {
    if (write) {
      *p = acc;
      acc.x += i;
      asm volatile("" ::: "memory");
    } else {
      v4i v = *p;
      asm volatile("" : "+v"(v));
      acc += v;
    }
  }
  if (acc.x == 0x7fffffff) sink[threadIdx.x] = acc.y + acc.z + acc.w;
}

}  // namespace

extern "C" int lstm_int_lds_probe(int32_t device, int32_t map, int32_t stride_words, int32_t swizzle, int32_t write) {
  if (device < 0 || map < 0 || map > 2 || swizzle < 0 || swizzle > 2 || stride_words < 4 || stride_words > 128 ||
      (stride_words & 3))
    return LSTM_INT_E_INVALID_ARG;
  if (hipSetDevice(device) != hipSuccess) return LSTM_INT_E_DEVICE;
  int *sink = nullptr;
  int rc = LSTM_INT_E_DEVICE;
  if (hipMalloc(&sink, 256 * sizeof(int)) == hipSuccess) {
    hipLaunchKernelGGL(lds_probe_kernel, dim3(1), dim3(256), 0, nullptr, map, stride_words, swizzle, write, sink);
    if (hipDeviceSynchronize() == hipSuccess) rc = LSTM_INT_OK;
  }
  if (sink) (void)hipFree(sink);
  return rc;
}

extern "C" int lstm_int_mfma_store_ceiling(int32_t device, int32_t stores_per_block, int32_t blocks, double *tops,
                                           double *store_gbs, double *clock_ghz) {
  if (device < 0 || stores_per_block < 0 || stores_per_block > 8 || blocks < 1 || !tops || !store_gbs || !clock_ghz)
    return LSTM_INT_E_INVALID_ARG;
  if (hipSetDevice(device) != hipSuccess) return LSTM_INT_E_DEVICE;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1)
    return LSTM_INT_E_DEVICE;
  const size_t out_bytes = (size_t)256 << 20;  // the benchmark layer's W x terms: 268 MB
  v4i *out = nullptr;
  unsigned long long *clocks = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = LSTM_INT_E_DEVICE;
  if (hipMalloc(&out, out_bytes) == hipSuccess && hipMalloc(&clocks, 16) == hipSuccess &&
      hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
    for (int rep = 0; rep < 2; ++rep) {  // the first launch warms up
      (void)hipEventRecord(e0, nullptr);
      hipLaunchKernelGGL(ceiling_kernel, dim3(cus), dim3(256), 0, nullptr, blocks, stores_per_block, out, out_bytes / 16,
                         clocks);
      (void)hipEventRecord(e1, nullptr);
    }
    float ms = 0.f;
    unsigned long long h[2] = {0, 0};
    if (hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess &&
        hipMemcpy(h, clocks, 16, hipMemcpyDeviceToHost) == hipSuccess && ms > 0.f && h[1] > 0) {
      const double sec = ms * 1e-3;
      *tops = (double)cus * 4 * blocks * kMfmaPerBlock * 65536.0 / sec / 1e12;
      *store_gbs = (double)cus * 4 * blocks * stores_per_block * 1024.0 / sec / 1e9;
      *clock_ghz = (double)h[0] / ((double)h[1] * 10.0);  // shader cycles per 10 ns tick of the wall clock
      rc = LSTM_INT_OK;
    }
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (out) (void)hipFree(out);
  if (clocks) (void)hipFree(clocks);
  return rc;
}
