// On-GPU collection of the statistics lstm_int_prepare needs (Sec. 4,
// post-training: ranges are logged at the nodes the execution figures mark
// "log"): the float LSTM of Sec. 2 (eqs. 1-7, with the CIFG, peephole,
// layer-norm and projection variants) in double precision over representative
// inputs, with min/max of x, h and m, max |c| and, under layer norm, max |gate
// sum| per gate.  Offline tooling like prepare: it allocates device memory,
// synchronizes, and is not on the integer path.
//
// Shape of the computation: per layer one hoisted GEMM W x over all T*B rows,
// then per step a GEMM R h on top of that step's slice, one workgroup per
// batch row for layer norm, activations and the cell update (wavefront
// reductions for the row statistics), and the projection GEMM.  Parameters
// stay float32 in memory (they are float32) and are widened on load; all
// arithmetic and all activations are double.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

#include "../../include/lstm_int.h"

namespace {

constexpr int kCifg = LSTM_INT_CIFG, kPeephole = LSTM_INT_PEEPHOLE, kLayerNorm = LSTM_INT_LAYER_NORM,
              kProjection = LSTM_INT_PROJECTION;

// statistics slots in device memory
enum { S_XMIN, S_XMAX, S_HMIN, S_HMAX, S_MMIN, S_MMAX, S_CABS, S_GABS, S_COUNT = S_GABS + 4 };

__device__ void atomic_min_f64(double *addr, double v) {
  unsigned long long *p = reinterpret_cast<unsigned long long *>(addr);
  unsigned long long old = *p;
  while (v < __longlong_as_double((long long)old)) {
    const unsigned long long seen = atomicCAS(p, old, (unsigned long long)__double_as_longlong(v));
    if (seen == old) break;
    old = seen;
  }
}
__device__ void atomic_max_f64(double *addr, double v) {
  unsigned long long *p = reinterpret_cast<unsigned long long *>(addr);
  unsigned long long old = *p;
  while (v > __longlong_as_double((long long)old)) {
    const unsigned long long seen = atomicCAS(p, old, (unsigned long long)__double_as_longlong(v));
    if (seen == old) break;
    old = seen;
  }
}

// ---- reductions over a workgroup of 256 threads (4 wavefronts of 64)
__device__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ double wave_max(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ double wave_min(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmin(v, __shfl_xor(v, o, 64));
  return v;
}
// every thread gets the result; red: 4 doubles of LDS
template <int OP>  // 0 sum, 1 max, 2 min
__device__ double block_reduce(double v, double *red) {
  v = OP == 0 ? wave_sum(v) : OP == 1 ? wave_max(v) : wave_min(v);
  __syncthreads();  // red may still be read from the previous reduction
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  const double a = red[0], b = red[1], c = red[2], d = red[3];
  return OP == 0 ? (a + b) + (c + d) : OP == 1 ? fmax(fmax(a, b), fmax(c, d)) : fmin(fmin(a, b), fmin(c, d));
}

// x float -> double, and its range
__global__ __launch_bounds__(256) void widen_kernel(const float *x, double *out, int64_t n, double *stats) {
  __shared__ double red[4];
  double lo = INFINITY, hi = -INFINITY;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const double v = x[i];
    out[i] = v;
    lo = fmin(lo, v);
    hi = fmax(hi, v);
  }
  lo = block_reduce<2>(lo, red);
  hi = block_reduce<1>(hi, red);
  if (threadIdx.x == 0) {
    atomic_min_f64(stats + S_XMIN, lo);
    atomic_max_f64(stats + S_XMAX, hi);
  }
}

// range of a double buffer into two statistics slots
__global__ __launch_bounds__(256) void range_kernel(const double *v, int64_t n, double *lo_slot, double *hi_slot) {
  __shared__ double red[4];
  double lo = INFINITY, hi = -INFINITY;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    lo = fmin(lo, v[i]);
    hi = fmax(hi, v[i]);
  }
  lo = block_reduce<2>(lo, red);
  hi = block_reduce<1>(hi, red);
  if (threadIdx.x == 0) {
    atomic_min_f64(lo_slot, lo);
    atomic_max_f64(hi_slot, hi);
  }
}

// C[m][n] = (Cin ? Cin[m][n] : 0) + (bias ? bias[n] : 0) + sum_k A[m][k] * W[n][k]
// A double [M][lda], W float [Nout][K], C double [M][ldc], Cin double [M][ldcin].
// Workgroup = 16 rows x 64 columns, thread = 1 row x 4 columns, k in tiles of 32
// through LDS; the sum over k runs in ascending k within a thread.
__global__ __launch_bounds__(256) void gemm_kernel(const double *A, int lda, const float *W, double *C, int ldc,
                                                   const double *Cin, int ldcin, const float *bias, int M, int Nout,
                                                   int K) {
  __shared__ double As[16][33];
  __shared__ double Ws[64][33];
  const int tid = threadIdx.x, tm = tid >> 4, tn = (tid & 15) << 2;
  const int m0 = blockIdx.x * 16, n0 = blockIdx.y * 64;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (int k0 = 0; k0 < K; k0 += 32) {
    for (int i = tid; i < 16 * 32; i += 256) {
      const int r = i >> 5, k = i & 31;
      As[r][k] = (m0 + r < M && k0 + k < K) ? A[(size_t)(m0 + r) * lda + k0 + k] : 0.0;
    }
    for (int i = tid; i < 64 * 32; i += 256) {
      const int r = i >> 5, k = i & 31;
      Ws[r][k] = (n0 + r < Nout && k0 + k < K) ? (double)W[(size_t)(n0 + r) * K + k0 + k] : 0.0;
    }
    __syncthreads();
#pragma unroll 8
    for (int k = 0; k < 32; ++k) {
      const double a = As[tm][k];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = fma(a, Ws[tn + j][k], acc[j]);
    }
    __syncthreads();
  }
  const int m = m0 + tm;
  if (m >= M) return;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = n0 + tn + j;
    if (n >= Nout) continue;
    double v = acc[j];
    if (Cin) v += Cin[(size_t)m * ldcin + n];
    if (bias) v += (double)bias[n];
    C[(size_t)m * ldc + n] = v;
  }
}

struct CellArgs {
  double *pre;    // [B][4*N] gate sums W x + R h of this step, slot per gate; overwritten
  double *c;      // [B][N] cell state, in/out
  double *m;      // [B][N] hidden state out
  double *h;      // [B][N] also receives m when there is no projection, else NULL
  const float *b[4], *P[3], *Lw[4];
  int N, flags;
  double *stats;
};

__device__ double sigmoid_f64(double v) { return 1.0 / (1.0 + exp(-v)); }

// One workgroup per batch row: eqs. (1)-(6) of Sec. 2 after the matrix
// products.  Gates f, z, i from c^{t-1}; the cell update; gate o from c^t; m.
__global__ __launch_bounds__(256) void cell_kernel(CellArgs a) {
  __shared__ double red[4];
  const int b = blockIdx.x, tid = threadIdx.x, N = a.N;
  const bool cifg = a.flags & kCifg, ph = a.flags & kPeephole, ln = a.flags & kLayerNorm;
  double *pre = a.pre + (size_t)b * 4 * N;
  double *c = a.c + (size_t)b * N;
  // gate g in place: pre[g] <- activation(norm(pre[g] + P . cell) . L + b)
  auto gate = [&](int g) {
    double *pg = pre + (size_t)g * N;
    const float *pw = (ph && g != 2) ? a.P[g == 3 ? 2 : g] : nullptr;
    double amax = 0.0, sum = 0.0;
    for (int n = tid; n < N; n += 256) {
      double v = pg[n];
      if (pw) v += (double)pw[n] * c[n];
      if (!ln) v += (double)a.b[g][n];
      pg[n] = v;
      amax = fmax(amax, fabs(v));
      sum += v;
    }
    if (ln) {
      amax = block_reduce<1>(amax, red);
      if (tid == 0) atomic_max_f64(a.stats + S_GABS + g, amax);
      const double mean = block_reduce<0>(sum, red) / N;
      double sq = 0.0;
      for (int n = tid; n < N; n += 256) {
        const double d = pg[n] - mean;
        sq += d * d;
      }
      const double sd = sqrt(block_reduce<0>(sq, red) / N);
      for (int n = tid; n < N; n += 256) {
        const double xn = sd > 0.0 ? (pg[n] - mean) / sd : 0.0;
        pg[n] = xn * (double)a.Lw[g][n] + (double)a.b[g][n];
      }
    }
    for (int n = tid; n < N; n += 256) pg[n] = g == 2 ? tanh(pg[n]) : sigmoid_f64(pg[n]);
  };
  gate(1);
  gate(2);
  if (!cifg) gate(0);
  double cmax = 0.0;
  for (int n = tid; n < N; n += 256) {
    const double f = pre[N + n];
    const double i = cifg ? 1.0 - f : pre[n];
    const double cn = i * pre[2 * (size_t)N + n] + f * c[n];
    c[n] = cn;
    cmax = fmax(cmax, fabs(cn));
  }
  cmax = block_reduce<1>(cmax, red);  // also orders the writes of c before gate o reads them
  gate(3);
  double lo = INFINITY, hi = -INFINITY;
  for (int n = tid; n < N; n += 256) {
    const double mv = pre[3 * (size_t)N + n] * tanh(c[n]);
    a.m[(size_t)b * N + n] = mv;
    if (a.h) a.h[(size_t)b * N + n] = mv;
    lo = fmin(lo, mv);
    hi = fmax(hi, mv);
  }
  lo = block_reduce<2>(lo, red);
  hi = block_reduce<1>(hi, red);
  if (tid == 0) {
    atomic_max_f64(a.stats + S_CABS, cmax);
    atomic_min_f64(a.stats + S_MMIN, lo);
    atomic_max_f64(a.stats + S_MMAX, hi);
  }
}

struct DevBuf {
  void *p = nullptr;
  DevBuf() = default;
  DevBuf(const DevBuf &) = delete;
  DevBuf &operator=(const DevBuf &) = delete;
  ~DevBuf() {
    if (p) (void)hipFree(p);
  }
  void swap(DevBuf &o) {
    void *t = p;
    p = o.p;
    o.p = t;
  }
  hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 256); }
  template <class T>
  T *as() const {
    return static_cast<T *>(p);
  }
};

void launch_gemm(hipStream_t s, const double *A, int lda, const float *W, double *C, int ldc, const double *Cin,
                 int ldcin, const float *bias, int M, int Nout, int K) {
  dim3 grid((M + 15) / 16, (Nout + 63) / 64);
  hipLaunchKernelGGL(gemm_kernel, grid, dim3(256), 0, s, A, lda, W, C, ldc, Cin, ldcin, bias, M, Nout, K);
}

}  // namespace

extern "C" int lstm_int_calibrate(const lstm_int_layer_params *layers, int32_t num_layers, int32_t device,
                                  const float *x, int32_t T, int32_t B, void *hip_stream,
                                  lstm_int_layer_stats *stats_out, double *y_float) {
  if (!layers || num_layers < 1 || device < 0 || !x || T < 1 || B < 1 || !stats_out) return LSTM_INT_E_INVALID_ARG;
  for (int l = 0; l < num_layers; ++l) {
    const lstm_int_layer_params &p = layers[l];
    const bool cifg = p.flags & kCifg, ph = p.flags & kPeephole, ln = p.flags & kLayerNorm, proj = p.flags & kProjection;
    if (p.input_size < 1 || p.num_cells < 1 || p.output_size < 1 || (p.flags & ~15u)) return LSTM_INT_E_INVALID_ARG;
    if (!proj && p.output_size != p.num_cells) return LSTM_INT_E_INVALID_ARG;
    if (l > 0 && p.input_size != layers[l - 1].output_size) return LSTM_INT_E_INVALID_ARG;
    if ((int64_t)T * B * 4 * p.num_cells >= (1ll << 31) || (int64_t)T * B * p.input_size >= (1ll << 31))
      return LSTM_INT_E_UNSUPPORTED;  // 32-bit row counts times strides in the kernels' index arithmetic
    for (int g = cifg ? 1 : 0; g < 4; ++g) {
      if (!p.W[g] || !p.R[g] || !p.b[g]) return LSTM_INT_E_INVALID_ARG;
      if (ln && !p.Lw[g]) return LSTM_INT_E_INVALID_ARG;
      if (ph && g != 2 && !p.P[g == 3 ? 2 : g]) return LSTM_INT_E_INVALID_ARG;
    }
    if (proj && !p.Wproj) return LSTM_INT_E_INVALID_ARG;
  }
  if (hipSetDevice(device) != hipSuccess) return LSTM_INT_E_DEVICE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t TB = (int64_t)T * B;

  DevBuf in, stats;
  if (in.alloc(sizeof(double) * TB * layers[0].input_size) != hipSuccess) return LSTM_INT_E_OUT_OF_MEMORY;
  if (stats.alloc(sizeof(double) * S_COUNT * num_layers) != hipSuccess) return LSTM_INT_E_OUT_OF_MEMORY;
  {
    std::vector<double> init((size_t)S_COUNT * num_layers, 0.0);
    for (int l = 0; l < num_layers; ++l) {
      double *st = init.data() + (size_t)l * S_COUNT;
      st[S_XMIN] = st[S_HMIN] = st[S_MMIN] = INFINITY;
      st[S_XMAX] = st[S_HMAX] = st[S_MMAX] = -INFINITY;
    }
    if (hipMemcpyAsync(stats.p, init.data(), init.size() * sizeof(double), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
      return LSTM_INT_E_DEVICE;
  }
  const int64_t n_in0 = TB * layers[0].input_size;
  hipLaunchKernelGGL(widen_kernel, dim3((unsigned)std::min<int64_t>((n_in0 + 255) / 256, 1024)), dim3(256), 0, s, x,
                     in.as<double>(), n_in0, stats.as<double>());

  DevBuf prev_out;  // the output of the layer before: the input of the layer at work
  double *cur_in = in.as<double>();
  for (int l = 0; l < num_layers; ++l) {
    const lstm_int_layer_params &p = layers[l];
    const int I = p.input_size, N = p.num_cells, H = p.output_size, first = (p.flags & kCifg) ? 1 : 0;
    const bool ph = p.flags & kPeephole, ln = p.flags & kLayerNorm, proj = p.flags & kProjection;
    double *st = stats.as<double>() + (size_t)l * S_COUNT;

    // parameters -> device; gate matrices concatenated [4][N][.] (slot 0 unused under CIFG)
    DevBuf Wd, Rd, vec, Wpd, wx, pre, c, m, h0;
    DevBuf out;
    const size_t nvec = (size_t)(4 + 3 + 4) * N + H;  // b[4], P[3], Lw[4], bproj
    if (Wd.alloc(sizeof(float) * 4 * N * I) != hipSuccess || Rd.alloc(sizeof(float) * 4 * (size_t)N * H) != hipSuccess ||
        vec.alloc(sizeof(float) * nvec) != hipSuccess || wx.alloc(sizeof(double) * TB * 4 * N) != hipSuccess ||
        pre.alloc(sizeof(double) * B * 4 * (size_t)N) != hipSuccess || c.alloc(sizeof(double) * (size_t)B * N) != hipSuccess ||
        m.alloc(sizeof(double) * (size_t)B * N) != hipSuccess || h0.alloc(sizeof(double) * (size_t)B * H) != hipSuccess ||
        out.alloc(sizeof(double) * TB * H) != hipSuccess || (proj && Wpd.alloc(sizeof(float) * (size_t)H * N) != hipSuccess))
      return LSTM_INT_E_OUT_OF_MEMORY;
    std::vector<float> hv(nvec, 0.0f);
    bool ok = true;
    auto up = [&](void *dst, const void *src, size_t bytes) {
      ok = ok && hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, s) == hipSuccess;
    };
    for (int g = first; g < 4; ++g) {
      up(Wd.as<float>() + (size_t)g * N * I, p.W[g], sizeof(float) * N * I);
      up(Rd.as<float>() + (size_t)g * N * H, p.R[g], sizeof(float) * (size_t)N * H);
      for (int n = 0; n < N; ++n) hv[(size_t)g * N + n] = p.b[g][n];
      if (ln)
        for (int n = 0; n < N; ++n) hv[(size_t)(7 + g) * N + n] = p.Lw[g][n];
    }
    if (ph)
      for (int j = first; j < 3; ++j)
        for (int n = 0; n < N; ++n) hv[(size_t)(4 + j) * N + n] = p.P[j][n];
    if (proj) {
      up(Wpd.p, p.Wproj, sizeof(float) * (size_t)H * N);
      if (p.bproj)
        for (int j = 0; j < H; ++j) hv[(size_t)11 * N + j] = p.bproj[j];
    }
    up(vec.p, hv.data(), sizeof(float) * nvec);
    ok = ok && hipMemsetAsync(c.p, 0, sizeof(double) * (size_t)B * N, s) == hipSuccess;
    ok = ok && hipMemsetAsync(h0.p, 0, sizeof(double) * (size_t)B * H, s) == hipSuccess;
    // the host vectors and the caller's arrays must outlive the copies
    ok = ok && hipStreamSynchronize(s) == hipSuccess;
    if (!ok) return LSTM_INT_E_DEVICE;

    const float *vb = vec.as<float>();
    // W x for all steps (eqs. 1-4, first term), gates first..3 in one product
    launch_gemm(s, cur_in, I, Wd.as<float>() + (size_t)first * N * I, wx.as<double>() + (size_t)first * N, 4 * N,
                nullptr, 0, nullptr, (int)TB, (4 - first) * N, I);
    CellArgs ca;
    ca.pre = pre.as<double>();
    ca.c = c.as<double>();
    ca.m = m.as<double>();
    for (int g = 0; g < 4; ++g) {
      ca.b[g] = vb + (size_t)g * N;
      ca.Lw[g] = vb + (size_t)(7 + g) * N;
    }
    for (int j = 0; j < 3; ++j) ca.P[j] = vb + (size_t)(4 + j) * N;
    ca.N = N;
    ca.flags = (int)p.flags;
    ca.stats = st;
    for (int t = 0; t < T; ++t) {
      const double *hp = t == 0 ? h0.as<double>() : out.as<double>() + (size_t)(t - 1) * B * H;
      double *ho = out.as<double>() + (size_t)t * B * H;
      // + R h^{t-1}
      launch_gemm(s, hp, H, Rd.as<float>() + (size_t)first * N * H, pre.as<double>() + (size_t)first * N, 4 * N,
                  wx.as<double>() + (size_t)t * B * 4 * N + (size_t)first * N, 4 * N, nullptr, B, (4 - first) * N, H);
      ca.h = proj ? nullptr : ho;
      hipLaunchKernelGGL(cell_kernel, dim3(B), dim3(256), 0, s, ca);
      if (proj)  // eq. (7)
        launch_gemm(s, m.as<double>(), N, Wpd.as<float>(), ho, H, nullptr, 0, vb + (size_t)11 * N, B, H, N);
    }
    const int64_t n_out = TB * H;
    hipLaunchKernelGGL(range_kernel, dim3((unsigned)std::min<int64_t>((n_out + 255) / 256, 1024)), dim3(256), 0, s,
                       out.as<double>(), n_out, st + S_HMIN, st + S_HMAX);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return LSTM_INT_E_DEVICE;
    if (l == num_layers - 1 && y_float &&
        hipMemcpy(y_float, out.p, sizeof(double) * n_out, hipMemcpyDeviceToDevice) != hipSuccess)
      return LSTM_INT_E_DEVICE;
    // this layer's output is the next layer's input (the one before it is freed with `out`)
    prev_out.swap(out);
    cur_in = prev_out.as<double>();
  }

  std::vector<double> hs((size_t)S_COUNT * num_layers);
  if (hipMemcpy(hs.data(), stats.p, hs.size() * sizeof(double), hipMemcpyDeviceToHost) != hipSuccess)
    return LSTM_INT_E_DEVICE;
  for (int l = 0; l < num_layers; ++l) {
    const double *st = hs.data() + (size_t)l * S_COUNT;
    lstm_int_layer_stats &o = stats_out[l];
    // the input of layer l > 0 is the output of layer l - 1
    o.x_min = l == 0 ? st[S_XMIN] : hs[(size_t)(l - 1) * S_COUNT + S_HMIN];
    o.x_max = l == 0 ? st[S_XMAX] : hs[(size_t)(l - 1) * S_COUNT + S_HMAX];
    o.h_min = st[S_HMIN];
    o.h_max = st[S_HMAX];
    o.m_min = st[S_MMIN];
    o.m_max = st[S_MMAX];
    o.c_absmax = st[S_CABS];
    for (int g = 0; g < 4; ++g) o.g_absmax[g] = st[S_GABS + g];
  }
  return LSTM_INT_OK;
}
