// Direct convolution kernels: one thread per output element, fp32 accumulation.
// They serve the fp32 problems and every bf16 shape the MFMA path does not take
// (channel counts that are not multiples of 8).  Cross-correlation, zero padding
// (Sec. 3.1); input gradient = adjoint of the forward gather (Sec. 3.2.1).
#include "common.h"

namespace convbn {

namespace {

template <typename T>
__global__ __launch_bounds__(256) void fprop_direct_kernel(const T* __restrict__ x,
                                                           const T* __restrict__ w,
                                                           const float* __restrict__ bias,
                                                           T* __restrict__ z, Geom g) {
  const size_t total = (size_t)g.M * g.Cout;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int co = (int)(idx % g.Cout);
  int m = (int)(idx / g.Cout);
  const int wo = m % g.Wout;
  m /= g.Wout;
  const int ho = m % g.Hout;
  const int n = m / g.Hout;
  float acc = bias ? bias[co] : 0.f;
  for (int i = 0; i < g.kH; ++i) {
    const int h = ho * g.sh + i - g.ph;
    if (h < 0 || h >= g.Hin) continue;
    for (int j = 0; j < g.kW; ++j) {
      const int wi = wo * g.sw + j - g.pw;
      if (wi < 0 || wi >= g.Win) continue;
      const T* xp = x + (((size_t)n * g.Hin + h) * g.Win + wi) * g.Cin;
      const T* wp = w + (((size_t)co * g.kH + i) * g.kW + j) * g.Cin;
      for (int c = 0; c < g.Cin; ++c) acc += to_f32(xp[c]) * to_f32(wp[c]);
    }
  }
  z[idx] = from_f32<T>(acc);
}

// w is [Cin][kH][kW][Cout]
template <typename T>
__global__ __launch_bounds__(256) void dgrad_direct_kernel(const T* __restrict__ dz,
                                                           const T* __restrict__ w,
                                                           const float* __restrict__ bias,
                                                           T* __restrict__ dx, Geom g) {
  const size_t total = (size_t)g.Min * g.Cin;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int ci = (int)(idx % g.Cin);
  int m = (int)(idx / g.Cin);
  const int wi = m % g.Win;
  m /= g.Win;
  const int h = m % g.Hin;
  const int n = m / g.Hin;
  float acc = bias ? bias[ci] : 0.f;
  for (int i = 0; i < g.kH; ++i) {
    const int hz = h + g.ph - i;
    if (hz < 0 || hz % g.sh != 0) continue;
    const int ho = hz / g.sh;
    if (ho >= g.Hout) continue;
    for (int j = 0; j < g.kW; ++j) {
      const int wz = wi + g.pw - j;
      if (wz < 0 || wz % g.sw != 0) continue;
      const int wo = wz / g.sw;
      if (wo >= g.Wout) continue;
      const T* gp = dz + (((size_t)n * g.Hout + ho) * g.Wout + wo) * g.Cout;
      const T* wp = w + (((size_t)ci * g.kH + i) * g.kW + j) * g.Cout;
      for (int c = 0; c < g.Cout; ++c) acc += to_f32(gp[c]) * to_f32(wp[c]);
    }
  }
  dx[idx] = from_f32<T>(acc);
}

// One thread per (co, tap, ci); blockIdx.y selects a slice of output pixels whose
// partial sum goes to part[blockIdx.y][Cout][K].
template <typename T>
__global__ __launch_bounds__(256) void wgrad_direct_kernel(const T* __restrict__ x,
                                                           const T* __restrict__ dz,
                                                           float* __restrict__ part, Geom g,
                                                           int rows_per_split) {
  const size_t P = (size_t)g.Cout * g.K;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= P) return;
  const int ci = (int)(idx % g.Cin);
  int t = (int)(idx / g.Cin);
  const int j = t % g.kW;
  t /= g.kW;
  const int i = t % g.kH;
  const int co = t / g.kH;
  const int m0 = blockIdx.y * rows_per_split;
  const int m1 = min(g.M, m0 + rows_per_split);
  float acc = 0.f;
  for (int m = m0; m < m1; ++m) {
    const int wo = m % g.Wout;
    const int r = m / g.Wout;
    const int ho = r % g.Hout;
    const int n = r / g.Hout;
    const int h = ho * g.sh + i - g.ph;
    const int wi = wo * g.sw + j - g.pw;
    if (h < 0 || h >= g.Hin || wi < 0 || wi >= g.Win) continue;
    acc += to_f32(dz[(size_t)m * g.Cout + co]) *
           to_f32(x[(((size_t)n * g.Hin + h) * g.Win + wi) * g.Cin + ci]);
  }
  part[(size_t)blockIdx.y * P + idx] = acc;
}

}  // namespace

hipError_t launch_fprop_direct(const Geom& g, int dtype, const void* x, const void* w_krsc,
                               const float* bias, void* z, hipStream_t st) {
  const size_t total = (size_t)g.M * g.Cout;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(fprop_direct_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)x,
                       (const bf16_t*)w_krsc, bias, (bf16_t*)z, g);
  else
    hipLaunchKernelGGL(fprop_direct_kernel<float>, grid, dim3(256), 0, st, (const float*)x,
                       (const float*)w_krsc, bias, (float*)z, g);
  return hipGetLastError();
}

hipError_t launch_dgrad_direct(const Geom& g, int dtype, const void* dz, const void* w_crsk,
                               const float* bias, void* dx, hipStream_t st) {
  const size_t total = (size_t)g.Min * g.Cin;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(dgrad_direct_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)dz,
                       (const bf16_t*)w_crsk, bias, (bf16_t*)dx, g);
  else
    hipLaunchKernelGGL(dgrad_direct_kernel<float>, grid, dim3(256), 0, st, (const float*)dz,
                       (const float*)w_crsk, bias, (float*)dx, g);
  return hipGetLastError();
}

int wgrad_direct_splits(const Geom& g) {
  // enough slices to occupy the chip when Cout*K is small, bounded partial storage
  const size_t P = (size_t)g.Cout * g.K;
  int want = (int)((size_t)(256 * 256 * 8) / (P < 1 ? 1 : P));
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  const int maxs = ceil_div(g.M, 64);
  return want < maxs ? want : maxs;
}

hipError_t launch_wgrad_direct(const Geom& g, int dtype, const void* x, const void* dz, float* dwf,
                               hipStream_t st) {
  const size_t P = (size_t)g.Cout * g.K;
  const int ns = wgrad_direct_splits(g);
  const int rps = ceil_div(g.M, ns);
  const dim3 grid((unsigned)((P + 255) / 256), (unsigned)ns);
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(wgrad_direct_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)x,
                       (const bf16_t*)dz, dwf, g, rps);
  else
    hipLaunchKernelGGL(wgrad_direct_kernel<float>, grid, dim3(256), 0, st, (const float*)x,
                       (const float*)dz, dwf, g, rps);
  return hipGetLastError();
}

}  // namespace convbn
