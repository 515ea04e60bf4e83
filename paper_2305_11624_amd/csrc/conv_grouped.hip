// Grouped convolution kernels: the channels are split into `groups` equal parts and an output channel reads
// only the input channels of its own part (the ResNeXt / RegNet style layers among the models of Sec. 4 and
// App. E).  The per-output-channel scale of Sec. 3.3 does not see the grouping -- the weight is a [Cout][kH kW cg]
// matrix (cg = Cin / groups) for the fold and the fold-back exactly as in the dense block -- so only the three
// contractions of Sec. 3.2.1 are written again here:
//   Z[m][o]          = b'[o] + sum_{tap, q < cg} X[m (+) tap][(o / og) cg + q] w'[o][tap][q]
//   dX[m][g cg + q]  = sum_{tap, oo < og} dZ[m (-) tap][g og + oo] w'[g og + oo][tap][q]
//   dw'[o][tap][q]   = sum_m dZ[m][o] X[m (+) tap][(o / og) cg + q]
// Layouts: x [N][H][W][Cin], z [N][Ho][Wo][Cout]; w_krsc [Cout][kH][kW][cg]; w_crsk [cg][kH][kW][Cout].
#include "common.h"

namespace convbn {

namespace {

// ---- any shape, both dtypes: one thread per output element, fp32 accumulation --------------------------
template <typename T>
__global__ __launch_bounds__(256) void g_fprop_direct_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                             const float* __restrict__ bias, T* __restrict__ z, Geom g,
                                                             int cg, int og) {
  const size_t total = (size_t)g.M * g.Cout;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int co = (int)(idx % g.Cout);
  int m = (int)(idx / g.Cout);
  const int wo = m % g.Wout;
  m /= g.Wout;
  const int ho = m % g.Hout;
  const int n = m / g.Hout;
  const int c0 = (co / og) * cg;
  float acc = bias ? bias[co] : 0.f;
  for (int i = 0; i < g.kH; ++i) {
    const int h = ho * g.sh + i - g.ph;
    if (h < 0 || h >= g.Hin) continue;
    for (int j = 0; j < g.kW; ++j) {
      const int wi = wo * g.sw + j - g.pw;
      if (wi < 0 || wi >= g.Win) continue;
      const T* xp = x + (((size_t)n * g.Hin + h) * g.Win + wi) * g.Cin + c0;
      const T* wp = w + (((size_t)co * g.kH + i) * g.kW + j) * cg;
      for (int c = 0; c < cg; ++c) acc += to_f32(xp[c]) * to_f32(wp[c]);
    }
  }
  z[idx] = from_f32<T>(acc);
}

template <typename T>
__global__ __launch_bounds__(256) void g_dgrad_direct_kernel(const T* __restrict__ dz, const T* __restrict__ w,
                                                             T* __restrict__ dx, Geom g, int cg, int og) {
  const size_t total = (size_t)g.Min * g.Cin;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int ci = (int)(idx % g.Cin);
  int m = (int)(idx / g.Cin);
  const int wi = m % g.Win;
  m /= g.Win;
  const int h = m % g.Hin;
  const int n = m / g.Hin;
  const int q = ci % cg, o0 = (ci / cg) * og;
  float acc = 0.f;
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
      const T* gp = dz + (((size_t)n * g.Hout + ho) * g.Wout + wo) * g.Cout + o0;
      const T* wp = w + (((size_t)q * g.kH + i) * g.kW + j) * g.Cout + o0;
      for (int c = 0; c < og; ++c) acc += to_f32(gp[c]) * to_f32(wp[c]);
    }
  }
  dx[idx] = from_f32<T>(acc);
}

// One thread per (co, tap, q); blockIdx.y selects a slice of output pixels whose partial sum goes to
// part[blockIdx.y][Cout][kH kW cg].
template <typename T>
__global__ __launch_bounds__(256) void g_wgrad_direct_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                             float* __restrict__ part, Geom g, int cg, int og,
                                                             int rows_per_split) {
  const size_t P = (size_t)g.Cout * g.kH * g.kW * cg;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= P) return;
  const int q = (int)(idx % cg);
  int t = (int)(idx / cg);
  const int j = t % g.kW;
  t /= g.kW;
  const int i = t % g.kH;
  const int co = t / g.kH;
  const int ci = (co / og) * cg + q;
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
    acc += to_f32(dz[(size_t)m * g.Cout + co]) * to_f32(x[(((size_t)n * g.Hin + h) * g.Win + wi) * g.Cin + ci]);
  }
  part[(size_t)blockIdx.y * P + idx] = acc;
}

int direct_splits(const Geom& g, int cg) {
  // enough slices to occupy the chip when the weight is small, bounded partial storage
  const size_t P = (size_t)g.Cout * g.kH * g.kW * cg;
  int want = (int)((size_t)(256 * 256 * 8) / (P < 1 ? 1 : P));
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  const int maxs = ceil_div(g.M, 64);
  return want < maxs ? want : maxs;
}

}  // namespace

hipError_t launch_g_fprop(const Geom& g, int groups, int dtype, const void* x, const void* w_krsc, const float* bias,
                          void* z, hipStream_t st) {
  const int cg = g.Cin / groups, og = g.Cout / groups;
  const size_t total = (size_t)g.M * g.Cout;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(g_fprop_direct_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)w_krsc,
                       bias, (bf16_t*)z, g, cg, og);
  else
    hipLaunchKernelGGL(g_fprop_direct_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (const float*)w_krsc,
                       bias, (float*)z, g, cg, og);
  return hipGetLastError();
}

hipError_t launch_g_dgrad(const Geom& g, int groups, int dtype, const void* dz, const void* w_crsk, void* dx,
                          hipStream_t st) {
  const int cg = g.Cin / groups, og = g.Cout / groups;
  const size_t total = (size_t)g.Min * g.Cin;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(g_dgrad_direct_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)dz, (const bf16_t*)w_crsk,
                       (bf16_t*)dx, g, cg, og);
  else
    hipLaunchKernelGGL(g_dgrad_direct_kernel<float>, grid, dim3(256), 0, st, (const float*)dz, (const float*)w_crsk,
                       (float*)dx, g, cg, og);
  return hipGetLastError();
}

int g_wgrad_slices(const Geom& g, int groups, int dtype) {
  (void)dtype;
  return direct_splits(g, g.Cin / groups);
}

bool g_wgrad_makes_rsum(const Geom& g, int groups, int dtype) {
  (void)g; (void)groups; (void)dtype;
  return false;
}

hipError_t launch_g_wgrad(const Geom& g, int groups, int dtype, const void* x, const void* dz, float* part,
                          float* r_part, hipStream_t st) {
  (void)r_part;
  const int cg = g.Cin / groups, og = g.Cout / groups;
  const size_t P = (size_t)g.Cout * g.kH * g.kW * cg;
  const int ns = direct_splits(g, cg);
  const int rps = ceil_div(g.M, ns);
  const dim3 grid((unsigned)((P + 255) / 256), (unsigned)ns);
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(g_wgrad_direct_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part,
                       g, cg, og, rps);
  else
    hipLaunchKernelGGL(g_wgrad_direct_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (const float*)dz, part, g,
                       cg, og, rps);
  return hipGetLastError();
}

}  // namespace convbn
