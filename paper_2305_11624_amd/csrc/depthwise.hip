// Depthwise ConvBN block in Tune mode: one filter per channel (groups = channels), BatchNorm folded into
// the filter exactly as for the dense block (Sec. 3.3: the scale is per output channel, so
// w'[c] = s_c w[c], b' = (b - mu) s + beta), backward by Table 2's "Tune" row.
//
// A depthwise convolution has 2 k^2 FLOP per output element against 2-4 bytes of traffic: it is bound by
// memory, not by the matrix cores, so these are plain vector kernels: channels-last tensors, a thread owns
// VEC consecutive channels of one pixel (bf16: 8 channels = one 16-byte access, consecutive threads =
// consecutive channels), the k^2 window positions are re-read through the caches.
//   x, dx [N][H][W][C]   z, dz [N][Ho][Wo][C]   W, dW [C][kH][kW]   folded filter wf [kH kW][C] (tap-major)
#include "common.h"

#include <type_traits>

namespace convbn {

namespace {

template <typename T, int VEC> struct Vec;
template <> struct Vec<float, 1> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[1]) { v[0] = *p; }
  static __device__ __forceinline__ void store(float* p, const float (&v)[1]) { *p = v[0]; }
};
template <> struct Vec<bf16_t, 1> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[1]) { v[0] = (float)*p; }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[1]) { *p = (bf16_t)v[0]; }
};
template <> struct Vec<bf16_t, 8> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    v[0] = bf16_lo(t.x); v[1] = bf16_hi(t.x); v[2] = bf16_lo(t.y); v[3] = bf16_hi(t.y);
    v[4] = bf16_lo(t.z); v[5] = bf16_hi(t.z); v[6] = bf16_lo(t.w); v[7] = bf16_hi(t.w);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                              pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  }
};

// wf[tap][c] = s_c W[c][tap], bfold[c] = (b - mu) s + beta.  gamma == nullptr: s = 1, b' = b.
template <typename T>
__global__ __launch_bounds__(256) void dw_fold_kernel(const T* __restrict__ W, const float* __restrict__ b,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      const float* __restrict__ mean, const float* __restrict__ var,
                                                      float eps, int C, int taps, T* __restrict__ wf,
                                                      float* __restrict__ bfold) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const float s = gamma ? gamma[c] / sqrtf(var[c] + eps) : 1.f;
  if (wf)
    for (int t = 0; t < taps; ++t) wf[(size_t)t * C + c] = from_f32<T>(to_f32(W[(size_t)c * taps + t]) * s);
  if (bfold) bfold[c] = gamma ? ((b ? b[c] : 0.f) - mean[c]) * s + beta[c] : (b ? b[c] : 0.f);
}

// Z[m][c] = b'[c] + sum_tap wf[tap][c] X[window position][c]
template <typename T, int VEC>
__global__ __launch_bounds__(256) void dw_fprop_kernel(const T* __restrict__ x, const T* __restrict__ wf,
                                                       const float* __restrict__ bias, T* __restrict__ z, Geom g) {
  const int cgs = g.Cin / VEC;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)g.M * cgs) return;
  const int c = (int)(idx % cgs) * VEC;
  int m = (int)(idx / cgs);
  const int wo = m % g.Wout;
  m /= g.Wout;
  const int ho = m % g.Hout, n = m / g.Hout;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = bias ? bias[c + e] : 0.f;
  for (int i = 0; i < g.kH; ++i) {
    const int h = ho * g.sh + i - g.ph;
    if ((unsigned)h >= (unsigned)g.Hin) continue;
    for (int j = 0; j < g.kW; ++j) {
      const int w = wo * g.sw + j - g.pw;
      if ((unsigned)w >= (unsigned)g.Win) continue;
      float xv[VEC], wv[VEC];
      Vec<T, VEC>::load(x + (((size_t)n * g.Hin + h) * g.Win + w) * g.Cin + c, xv);
      Vec<T, VEC>::load(wf + (size_t)(i * g.kW + j) * g.Cin + c, wv);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += xv[e] * wv[e];
    }
  }
  Vec<T, VEC>::store(z + idx * VEC, acc);
}

// dX[m'][c] = sum_tap wf[tap][c] dZ[(h + ph - i)/sh, (w + pw - j)/sw][c] over the taps whose quotients are exact
template <typename T, int VEC>
__global__ __launch_bounds__(256) void dw_dgrad_kernel(const T* __restrict__ dz, const T* __restrict__ wf,
                                                       T* __restrict__ dx, Geom g) {
  const int cgs = g.Cin / VEC;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)g.Min * cgs) return;
  const int c = (int)(idx % cgs) * VEC;
  int m = (int)(idx / cgs);
  const int w = m % g.Win;
  m /= g.Win;
  const int h = m % g.Hin, n = m / g.Hin;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  for (int i = 0; i < g.kH; ++i) {
    const int hz = h + g.ph - i;
    if (hz < 0 || hz % g.sh != 0) continue;
    const int ho = hz / g.sh;
    if (ho >= g.Hout) continue;
    for (int j = 0; j < g.kW; ++j) {
      const int wz = w + g.pw - j;
      if (wz < 0 || wz % g.sw != 0) continue;
      const int wo = wz / g.sw;
      if (wo >= g.Wout) continue;
      float gv[VEC], wv[VEC];
      Vec<T, VEC>::load(dz + (((size_t)n * g.Hout + ho) * g.Wout + wo) * g.Cin + c, gv);
      Vec<T, VEC>::load(wf + (size_t)(i * g.kW + j) * g.Cin + c, wv);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += gv[e] * wv[e];
    }
  }
  Vec<T, VEC>::store(dx + idx * VEC, acc);
}

// 3x3 windows, stride S, bf16, C % 8 == 0: a thread owns 8 channels of SEG vertically consecutive outputs of one
// output column.  It first issues every load of the ((SEG-1) S + 3) x 3 input patch those outputs need (kept packed, 16
// bytes each, so all of them are in flight together and the memory latency is paid once per thread), keeps the
// filter (9 x 8 values) in registers, and pays the index arithmetic once per segment: the generic kernel above
// spends its time on integer divisions, on re-reading the filter and on nine dependent trips to memory.
//   out[n][ho][wo][c] = bias[c] + sum_{i,j} wf[tap(i,j)][c] in[n][ho S + i - ph][wo S + j - pw][c]
// FLIP (input gradient of a stride-1 convolution): tap(i,j) is the rotated one, in = dZ, ph = 2 - ph.
constexpr int patch_seg(int S) { return S == 1 ? 4 : 3; }

__device__ __forceinline__ void unpack8(const uint4& t, float (&v)[8]) {
  v[0] = bf16_lo(t.x); v[1] = bf16_hi(t.x); v[2] = bf16_lo(t.y); v[3] = bf16_hi(t.y);
  v[4] = bf16_lo(t.z); v[5] = bf16_hi(t.z); v[6] = bf16_lo(t.w); v[7] = bf16_hi(t.w);
}

template <int S, bool FLIP>
__global__ __launch_bounds__(256) void dw_patch3_kernel(const bf16_t* __restrict__ in, const bf16_t* __restrict__ wf,
                                                      const float* __restrict__ bias, bf16_t* __restrict__ out, int N,
                                                      int Hi, int Wi, int Ho, int Wo, int C, int ph, int pw, int nseg) {
  // the SEG outputs are consecutive along H: consecutive threads are then consecutive (channel group, column)
  // pairs of one row and every load of the wave is one contiguous kilobyte
  constexpr int K = 3, SEG = patch_seg(S), NR = (SEG - 1) * S + K;
  const int cgs = C >> 3;
  const unsigned id = blockIdx.x * 256u + threadIdx.x;
  if (id >= (unsigned)N * nseg * Wo * cgs) return;
  const int cg = id % cgs;
  unsigned t = id / cgs;
  const int wo = t % Wo;
  t /= Wo;
  const int sg = t % nseg, n = t / nseg;
  const int c = cg * 8;
  const int ho0 = sg * SEG;
  // the input patch, then the filter: every load is issued before the first use
  uint4 xr[NR][K];
#pragma unroll
  for (int q = 0; q < NR; ++q) {
    const int h = ho0 * S + q - ph;
    const bool rok = (unsigned)h < (unsigned)Hi;
    const bf16_t* rowp = in + ((size_t)n * Hi + (rok ? h : 0)) * Wi * C + c;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const int w = wo * S + j - pw;
      xr[q][j] = (rok && (unsigned)w < (unsigned)Wi) ? *reinterpret_cast<const uint4*>(rowp + (size_t)w * C)
                                                     : make_uint4(0u, 0u, 0u, 0u);
    }
  }
  float wv[K * K][8], bv[8];
#pragma unroll
  for (int q = 0; q < K * K; ++q) Vec<bf16_t, 8>::load(wf + (size_t)(FLIP ? K * K - 1 - q : q) * C + c, wv[q]);
#pragma unroll
  for (int e = 0; e < 8; ++e) bv[e] = bias ? bias[c + e] : 0.f;
  // every patch element is widened once and multiplied into each output that covers it
  float acc[SEG][8];
#pragma unroll
  for (int o = 0; o < SEG; ++o)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[o][e] = bv[e];
#pragma unroll
  for (int q = 0; q < NR; ++q)
#pragma unroll
    for (int j = 0; j < K; ++j) {
      float xv[8];
      unpack8(xr[q][j], xv);
#pragma unroll
      for (int o = 0; o < SEG; ++o) {
        const int i = q - o * S;
        if (i < 0 || i >= K) continue;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[o][e] += xv[e] * wv[i * K + j][e];
      }
    }
#pragma unroll
  for (int o = 0; o < SEG; ++o)
    if (ho0 + o < Ho) Vec<bf16_t, 8>::store(out + (((size_t)n * Ho + ho0 + o) * Wo + wo) * C + c, acc[o]);
}

// Input gradient of a 3x3 stride-2 depthwise convolution, same idea as the patch kernel: 8 channels of 4
// consecutive dX pixels of one row (first pixel even).  dX[h][w] = sum over the taps (i, j) with h + ph - i and
// w + pw - j even of wf[i][j] dZ[(h + ph - i)/2][(w + pw - j)/2]: at most two dZ rows (which ones depends on the
// parity of h: rows that do not qualify are loaded as zeros) and exactly three dZ columns, the even ones among
// w0 + pw - 2 .. w0 + pw + 3, whose parity pattern is the same for every thread.
__global__ __launch_bounds__(256) void dw_dgrad_s2_patch3_kernel(const bf16_t* __restrict__ dz, const bf16_t* __restrict__ wf,
                                                               bf16_t* __restrict__ dx, int N, int Hin, int Win, int Ho,
                                                               int Wo, int C, int ph, int pw, int nseg) {
  constexpr int K = 3, SEG = 4;
  const int cgs = C >> 3;
  const unsigned id = blockIdx.x * 256u + threadIdx.x;
  if (id >= (unsigned)N * Hin * nseg * cgs) return;
  const int cg = id % cgs;
  unsigned t = id / cgs;
  const int sg = t % nseg;
  t /= nseg;
  const int h = t % Hin, n = t / Hin;
  const int c = cg * 8;
  const int w0 = sg * SEG;
  const int base = w0 + pw - 2;                 // smallest w + pw - j of the segment
  const int par = base & 1;                     // its parity: the same for every thread (w0 is even)
  const int wo_first = (base + par) >> 1;       // first of the three dZ columns (may be negative: zeros)
  uint4 gr[K][3];
#pragma unroll
  for (int i = 0; i < K; ++i) {
    const int hz = h + ph - i;
    const bool rok = hz >= 0 && (hz & 1) == 0 && (hz >> 1) < Ho;
    const bf16_t* rowp = dz + ((size_t)n * Ho + (rok ? hz >> 1 : 0)) * Wo * C + c;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int wo = wo_first + q;
      gr[i][q] = (rok && (unsigned)wo < (unsigned)Wo) ? *reinterpret_cast<const uint4*>(rowp + (size_t)wo * C)
                                                      : make_uint4(0u, 0u, 0u, 0u);
    }
  }
  float wv[K * K][8];
#pragma unroll
  for (int q = 0; q < K * K; ++q) Vec<bf16_t, 8>::load(wf + (size_t)q * C + c, wv[q]);
  bf16_t* orow = dx + ((size_t)n * Hin + h) * Win * C + c;
#pragma unroll
  for (int o = 0; o < SEG; ++o) {
    if (w0 + o >= Win) break;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const int d = o + 2 - j;                  // w + pw - j = base + d
      if ((d & 1) != par) continue;             // odd: this tap does not reach the pixel
      const int q = (d - par) >> 1;             // 0 .. 2 (d = 5 only with par = 1)
#pragma unroll
      for (int i = 0; i < K; ++i) {
        float gv[8];
        unpack8(q == 0 ? gr[i][0] : q == 1 ? gr[i][1] : gr[i][2], gv);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += gv[e] * wv[i * K + j][e];
      }
    }
    Vec<bf16_t, 8>::store(orow + (size_t)(w0 + o) * C, acc);
  }
}

bool patch3_shape(const Geom& g, int dtype) {
  return dtype == CONVBN_BF16 && g.Cin % 8 == 0 && g.kH == 3 && g.kW == 3 && g.sh == g.sw && (g.sh == 1 || g.sh == 2) &&
         (size_t)g.N * (g.Hin > g.Hout ? g.Hin : g.Hout) * ceil_div(g.Win > g.Wout ? g.Win : g.Wout, 3) * (g.Cin / 8) <
             0xffffffffull;
}
template <int S, bool FLIP>
hipError_t launch_patch3(const void* in, const void* wf, const float* bias, void* out, int N, int Hi, int Wi, int Ho,
                       int Wo, int C, int ph, int pw, hipStream_t st) {
  const int nseg = ceil_div(Ho, patch_seg(S));
  const size_t total = (size_t)N * nseg * Wo * (C / 8);
  hipLaunchKernelGGL((dw_patch3_kernel<S, FLIP>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t*)in,
                     (const bf16_t*)wf, bias, (bf16_t*)out, N, Hi, Wi, Ho, Wo, C, ph, pw, nseg);
  return hipGetLastError();
}

// Weight gradient for the shapes of the patch kernel.  An item is SEG vertically consecutive outputs of one column; a
// thread owns 8 channels and every L-th item of its workgroup's slice of the items (L = threads / channel groups
// of the workgroup), loads an item's dZ values and input patch up front and accumulates the 9 x 8 products and
// the channel sums in registers; the L lanes are then summed through LDS.  Outputs as dw_wgrad_kernel.
template <int S>
__global__ __launch_bounds__(256) void dw_wgrad_patch3_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dz,
                                                            float* __restrict__ part, float* __restrict__ r_part, int N,
                                                            int Hi, int Wi, int Ho, int Wo, int C, int ph, int pw,
                                                            int nseg, int cgb, int items_per_slice) {
  constexpr int K = 3, SEG = patch_seg(S), NR = (SEG - 1) * S + K;
  __shared__ float red[256 * 8];
  const int cgs = C >> 3;
  const int L = 256 / cgb;
  const int tx = threadIdx.x % cgb, lane = threadIdx.x / cgb;
  const int cg = blockIdx.x * cgb + tx;
  const bool live = lane < L && cg < cgs;
  const int c = cg * 8;
  const int nitems = N * nseg * Wo;
  const int it0 = blockIdx.y * items_per_slice, it1 = min(nitems, it0 + items_per_slice);
  float acc[K * K][8], racc[8];
#pragma unroll
  for (int q = 0; q < K * K; ++q)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) racc[e] = 0.f;
  if (live)
    for (int it = it0 + lane; it < it1; it += L) {
      const int wo = it % Wo;
      const int t = it / Wo;
      const int sg = t % nseg, n = t / nseg;
      const int ho0 = sg * SEG;
      uint4 gr[SEG], xr[NR][K];
#pragma unroll
      for (int o = 0; o < SEG; ++o)
        gr[o] = ho0 + o < Ho ? *reinterpret_cast<const uint4*>(dz + (((size_t)n * Ho + ho0 + o) * Wo + wo) * C + c)
                             : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int q = 0; q < NR; ++q) {
        const int h = ho0 * S + q - ph;
        const bool rok = (unsigned)h < (unsigned)Hi;
        const bf16_t* rowp = x + ((size_t)n * Hi + (rok ? h : 0)) * Wi * C + c;
#pragma unroll
        for (int jj = 0; jj < K; ++jj) {
          const int w = wo * S + jj - pw;
          xr[q][jj] = (rok && (unsigned)w < (unsigned)Wi) ? *reinterpret_cast<const uint4*>(rowp + (size_t)w * C)
                                                          : make_uint4(0u, 0u, 0u, 0u);
        }
      }
      float gv[SEG][8];
#pragma unroll
      for (int o = 0; o < SEG; ++o) {
        unpack8(gr[o], gv[o]);
#pragma unroll
        for (int e = 0; e < 8; ++e) racc[e] += gv[o][e];
      }
#pragma unroll
      for (int q = 0; q < NR; ++q)
#pragma unroll
        for (int jj = 0; jj < K; ++jj) {
          float xv[8];
          unpack8(xr[q][jj], xv);
#pragma unroll
          for (int o = 0; o < SEG; ++o) {
            const int i = q - o * S;
            if (i < 0 || i >= K) continue;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[i * K + jj][e] += gv[o][e] * xv[e];
          }
        }
    }
  // sum the lanes: one window position at a time (q == 9: the channel sums)
  const int ncol = cgb * 8;
#pragma unroll
  for (int q = 0; q <= K * K; ++q) {
    if (q == K * K && !r_part) continue;
    __syncthreads();
    if (lane < L) {
#pragma unroll
      for (int e = 0; e < 8; ++e) red[lane * ncol + tx * 8 + e] = q < K * K ? acc[q < K * K ? q : 0][e] : racc[e];
    }
    __syncthreads();
    for (int col = threadIdx.x; col < ncol; col += 256) {
      const int cc = blockIdx.x * ncol + col;
      if (cc >= C) continue;
      float v = 0.f;
      for (int l = 0; l < L; ++l) v += red[l * ncol + col];
      if (q < K * K) part[((size_t)blockIdx.y * (K * K) + q) * C + cc] = v;
      else r_part[(size_t)blockIdx.y * C + cc] = v;
    }
  }
}

// workgroup shape of the kernel above: x-blocks, channel groups per block, slices of the items
struct PatchWgPlan { int nxb, cgb, nseg, slices, items_per_slice; };
PatchWgPlan patch_wg_plan(const Geom& g) {
  PatchWgPlan p;
  const int cgs = g.Cin / 8;
  p.nxb = ceil_div(cgs, 64);
  p.cgb = ceil_div(cgs, p.nxb);
  p.nseg = ceil_div(g.Hout, patch_seg(g.sh));
  const int L = 256 / p.cgb;
  const int nitems = g.N * p.nseg * g.Wout;
  int want = ceil_div(256, p.nxb);                       // about one workgroup per CU
  const int maxs = ceil_div(nitems, 2 * L);              // at least two items per thread
  if (want > maxs) want = maxs;
  if (want < 1) want = 1;
  p.items_per_slice = ceil_div(nitems, want);
  p.slices = ceil_div(nitems, p.items_per_slice);
  return p;
}

constexpr int WG_TAPS = 9;     // window positions a weight-gradient workgroup accumulates at once
constexpr int WG_CG = 32;      // channel groups per workgroup (x 8 pixel lanes = 256 threads)

// Partial sums over one slice of the output pixels (blockIdx.y) for WG_TAPS window positions starting at
// tap0 = WG_TAPS blockIdx.z:  part[slice][tap][c] = sum_m dZ[m][c] X[window position of m][c], and (first tap
// chunk only) r_part[slice][c] = sum_m dZ[m][c].  Thread -> channel group tid % 32, pixel lane tid / 32.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void dw_wgrad_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                       float* __restrict__ part, float* __restrict__ r_part, Geom g,
                                                       int px_per_slice) {
  __shared__ float red[8][WG_CG * VEC];
  const int cgs = g.Cin / VEC;
  const int tx = threadIdx.x % WG_CG, ty = threadIdx.x / WG_CG;
  const int cg = blockIdx.x * WG_CG + tx;
  const bool live = cg < cgs;
  const int c = cg * VEC;
  const int taps = g.kH * g.kW, tap0 = blockIdx.z * WG_TAPS;
  const int m0 = blockIdx.y * px_per_slice, m1 = min(g.M, m0 + px_per_slice);
  float acc[WG_TAPS][VEC], racc[VEC];
#pragma unroll
  for (int t = 0; t < WG_TAPS; ++t)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[t][e] = 0.f;
#pragma unroll
  for (int e = 0; e < VEC; ++e) racc[e] = 0.f;
  if (live)
    for (int m = m0 + ty; m < m1; m += 8) {
      const int wo = m % g.Wout;
      const int q = m / g.Wout;
      const int ho = q % g.Hout, n = q / g.Hout;
      float gv[VEC];
      Vec<T, VEC>::load(dz + (size_t)m * g.Cin + c, gv);
#pragma unroll
      for (int e = 0; e < VEC; ++e) racc[e] += gv[e];
#pragma unroll
      for (int t = 0; t < WG_TAPS; ++t) {
        const int tap = tap0 + t;
        if (tap >= taps) break;
        const int i = tap / g.kW, j = tap - i * g.kW;
        const int h = ho * g.sh + i - g.ph, w = wo * g.sw + j - g.pw;
        if ((unsigned)h >= (unsigned)g.Hin || (unsigned)w >= (unsigned)g.Win) continue;
        float xv[VEC];
        Vec<T, VEC>::load(x + (((size_t)n * g.Hin + h) * g.Win + w) * g.Cin + c, xv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[t][e] += gv[e] * xv[e];
      }
    }
  // reduce the eight pixel lanes, one window position at a time (t == WG_TAPS: the channel sums)
  const int ncol = WG_CG * VEC;
#pragma unroll
  for (int t = 0; t <= WG_TAPS; ++t) {
    const int tap = tap0 + t;
    if (t < WG_TAPS && tap >= taps) continue;
    if (t == WG_TAPS && (blockIdx.z != 0 || !r_part)) continue;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[ty][tx * VEC + e] = t < WG_TAPS ? acc[t < WG_TAPS ? t : 0][e] : racc[e];
    __syncthreads();
    for (int col = threadIdx.x; col < ncol; col += 256) {
      const int cc = blockIdx.x * ncol + col;
      if (cc >= g.Cin) continue;
      float v = 0.f;
#pragma unroll
      for (int l = 0; l < 8; ++l) v += red[l][col];
      if (t < WG_TAPS) part[((size_t)blockIdx.y * taps + tap) * g.Cin + cc] = v;
      else r_part[(size_t)blockIdx.y * g.Cin + cc] = v;
    }
  }
}

// sums[row][c] = sum over slices of part[slice][row][c] (rows 0..taps-1) and of r_part[slice][c] (row taps).
// grid (ceil(C/16), taps + 1), thread -> channel tid % 16, slice lane tid / 16
__global__ __launch_bounds__(256) void dw_reduce_kernel(const float* __restrict__ part, const float* __restrict__ r_part,
                                                        int slices, int taps, int C, float* __restrict__ sums) {
  __shared__ float red[16][17];
  const int cl = threadIdx.x & 15, l = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl, row = blockIdx.y;
  float v = 0.f;
  if (c < C && (row < taps || r_part))
    for (int s = l; s < slices; s += 16)
      v += row < taps ? part[((size_t)s * taps + row) * C + c] : r_part[(size_t)s * C + c];
  red[l][cl] = v;
  __syncthreads();
  if (l != 0 || c >= C) return;
  v = 0.f;
#pragma unroll
  for (int k = 0; k < 16; ++k) v += red[k][cl];
  sums[(size_t)row * C + c] = v;
}

// dW[c][tap] = s dw', dgamma = (sum_tap dw' w + r (b - mu)) / sqrt(var + eps), dbeta = r, db = s r.
// gamma == nullptr (Eval path): dW = dw' only.
template <typename T>
__global__ __launch_bounds__(256) void dw_fold_back_kernel(const float* __restrict__ sums, const T* __restrict__ W,
                                                           const float* __restrict__ b, const float* __restrict__ gamma,
                                                           const float* __restrict__ mean, const float* __restrict__ var,
                                                           float eps, int C, int taps, T* __restrict__ dW,
                                                           float* __restrict__ db, float* __restrict__ dgamma,
                                                           float* __restrict__ dbeta) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const float sd = gamma ? sqrtf(var[c] + eps) : 1.f;
  const float s = gamma ? gamma[c] / sd : 1.f;
  float dot = 0.f;
  for (int t = 0; t < taps; ++t) {
    const float dw = sums[(size_t)t * C + c];
    dW[(size_t)c * taps + t] = from_f32<T>(s * dw);
    dot += dw * to_f32(W[(size_t)c * taps + t]);
  }
  if (!gamma) return;
  const float r = sums[(size_t)taps * C + c];
  dgamma[c] = (dot + r * ((b ? b[c] : 0.f) - mean[c])) / sd;
  dbeta[c] = r;
  if (db) db[c] = s * r;
}

bool vec8(const Geom& g, int dtype) { return dtype == CONVBN_BF16 && g.Cin % 8 == 0; }

}  // namespace

hipError_t launch_dw_fold(const Geom& g, int dtype, const void* W, const float* b, const float* gamma,
                          const float* beta, const float* mean, const float* var, void* wf, float* bfold,
                          hipStream_t st) {
  const int C = g.Cin, taps = g.kH * g.kW;
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(dw_fold_kernel<bf16_t>, dim3(ceil_div(C, 256)), dim3(256), 0, st, (const bf16_t*)W, b, gamma,
                       beta, mean, var, g.eps, C, taps, (bf16_t*)wf, bfold);
  else
    hipLaunchKernelGGL(dw_fold_kernel<float>, dim3(ceil_div(C, 256)), dim3(256), 0, st, (const float*)W, b, gamma, beta,
                       mean, var, g.eps, C, taps, (float*)wf, bfold);
  return hipGetLastError();
}

hipError_t launch_dw_fprop(const Geom& g, int dtype, const void* x, const void* wf, const float* bias, void* z,
                           hipStream_t st) {
  if (patch3_shape(g, dtype)) {
    if (g.sh == 1) return launch_patch3<1, false>(x, wf, bias, z, g.N, g.Hin, g.Win, g.Hout, g.Wout, g.Cin, g.ph, g.pw, st);
    return launch_patch3<2, false>(x, wf, bias, z, g.N, g.Hin, g.Win, g.Hout, g.Wout, g.Cin, g.ph, g.pw, st);
  }
  const int vec = vec8(g, dtype) ? 8 : 1;
  const size_t total = (size_t)g.M * (g.Cin / vec);
  const dim3 grid((unsigned)((total + 255) / 256));
  if (vec == 8)
    hipLaunchKernelGGL((dw_fprop_kernel<bf16_t, 8>), grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)wf, bias,
                       (bf16_t*)z, g);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL((dw_fprop_kernel<bf16_t, 1>), grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)wf, bias,
                       (bf16_t*)z, g);
  else
    hipLaunchKernelGGL((dw_fprop_kernel<float, 1>), grid, dim3(256), 0, st, (const float*)x, (const float*)wf, bias,
                       (float*)z, g);
  return hipGetLastError();
}

hipError_t launch_dw_dgrad(const Geom& g, int dtype, const void* dz, const void* wf, void* dx, hipStream_t st) {
  if (patch3_shape(g, dtype) && g.sh == 1 && g.ph <= 2 && g.pw <= 2)   // the same sweep over dZ with the rotated filter
    return launch_patch3<1, true>(dz, wf, nullptr, dx, g.N, g.Hout, g.Wout, g.Hin, g.Win, g.Cin, 2 - g.ph, 2 - g.pw, st);
  if (patch3_shape(g, dtype) && g.sh == 2) {
    const int nseg = ceil_div(g.Win, 4);
    const size_t total = (size_t)g.N * g.Hin * nseg * (g.Cin / 8);
    hipLaunchKernelGGL(dw_dgrad_s2_patch3_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t*)dz,
                       (const bf16_t*)wf, (bf16_t*)dx, g.N, g.Hin, g.Win, g.Hout, g.Wout, g.Cin, g.ph, g.pw, nseg);
    return hipGetLastError();
  }
  const int vec = vec8(g, dtype) ? 8 : 1;
  const size_t total = (size_t)g.Min * (g.Cin / vec);
  const dim3 grid((unsigned)((total + 255) / 256));
  if (vec == 8)
    hipLaunchKernelGGL((dw_dgrad_kernel<bf16_t, 8>), grid, dim3(256), 0, st, (const bf16_t*)dz, (const bf16_t*)wf,
                       (bf16_t*)dx, g);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL((dw_dgrad_kernel<bf16_t, 1>), grid, dim3(256), 0, st, (const bf16_t*)dz, (const bf16_t*)wf,
                       (bf16_t*)dx, g);
  else
    hipLaunchKernelGGL((dw_dgrad_kernel<float, 1>), grid, dim3(256), 0, st, (const float*)dz, (const float*)wf,
                       (float*)dx, g);
  return hipGetLastError();
}

// pixel slices of the weight-gradient reduction: enough workgroups to fill the chip a few times over
int dw_wgrad_slices(const Geom& g, int dtype) {
  if (patch3_shape(g, dtype)) return patch_wg_plan(g).slices;
  const int vec = vec8(g, dtype) ? 8 : 1;
  const int cblocks = ceil_div(g.Cin / vec, WG_CG) * ceil_div(g.kH * g.kW, WG_TAPS);
  int want = ceil_div(1024, cblocks);
  const int maxs = ceil_div(g.M, 64);
  if (want > maxs) want = maxs;
  if (want > 512) want = 512;
  if (want < 1) want = 1;
  return ceil_div(g.M, ceil_div(g.M, want));
}

hipError_t launch_dw_wgrad(const Geom& g, int dtype, const void* x, const void* dz, float* part, float* r_part,
                           hipStream_t st) {
  if (patch3_shape(g, dtype)) {
    const PatchWgPlan p = patch_wg_plan(g);
    const dim3 grid(p.nxb, p.slices);
#define PATCHWG(SV) \
    hipLaunchKernelGGL((dw_wgrad_patch3_kernel<SV>), grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part, \
                       r_part, g.N, g.Hin, g.Win, g.Hout, g.Wout, g.Cin, g.ph, g.pw, p.nseg, p.cgb, p.items_per_slice)
    if (g.sh == 1) PATCHWG(1); else PATCHWG(2);
#undef PATCHWG
    return hipGetLastError();
  }
  const int vec = vec8(g, dtype) ? 8 : 1;
  const int slices = dw_wgrad_slices(g, dtype);
  const int pps = ceil_div(g.M, slices);
  const dim3 grid(ceil_div(g.Cin / vec, WG_CG), slices, ceil_div(g.kH * g.kW, WG_TAPS));
  if (vec == 8)
    hipLaunchKernelGGL((dw_wgrad_kernel<bf16_t, 8>), grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part,
                       r_part, g, pps);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL((dw_wgrad_kernel<bf16_t, 1>), grid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part,
                       r_part, g, pps);
  else
    hipLaunchKernelGGL((dw_wgrad_kernel<float, 1>), grid, dim3(256), 0, st, (const float*)x, (const float*)dz, part,
                       r_part, g, pps);
  return hipGetLastError();
}

hipError_t launch_dw_fold_back(const Geom& g, int dtype, const float* part, const float* r_part, int slices,
                               float* sums, const void* W, const float* b, const float* gamma, const float* mean,
                               const float* var, void* dW, float* db, float* dgamma, float* dbeta, hipStream_t st) {
  const int C = g.Cin, taps = g.kH * g.kW;
  hipLaunchKernelGGL(dw_reduce_kernel, dim3(ceil_div(C, 16), taps + 1), dim3(256), 0, st, part, r_part, slices, taps, C,
                     sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(dw_fold_back_kernel<bf16_t>, dim3(ceil_div(C, 256)), dim3(256), 0, st, sums, (const bf16_t*)W, b,
                       gamma, mean, var, g.eps, C, taps, (bf16_t*)dW, db, dgamma, dbeta);
  else
    hipLaunchKernelGGL(dw_fold_back_kernel<float>, dim3(ceil_div(C, 256)), dim3(256), 0, st, sums, (const float*)W, b,
                       gamma, mean, var, g.eps, C, taps, (float*)dW, db, dgamma, dbeta);
  return hipGetLastError();
}

}  // namespace convbn
