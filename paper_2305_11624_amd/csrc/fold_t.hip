// Fold and fold-back of the TransposedConv-BN block (Sec. 3.2.1: the associative law behind Tune mode
// holds for transposed convolution as well; Sec. 3.3 and Table 2 "Tune" with the per-channel scale on
// the weight's OUTPUT-channel index, which is the innermost one of the transposed block's weight):
//   W      [Ci][taps][Co]     (the channels-last order of the logical [Ci, Co, kH, kW])
//   fold   w_same[ci][tap][co] = s[co] W[ci][tap][co]      read by the backward's input-gradient pass
//          w_swap[co][tap][ci] = s[co] W[ci][tap][co]      read by the forward pass (or [tap][co][ci] where the
//                                                          forward pass is a single product, see conv_pw.hip)
//          b'[co] = (b[co] - mu[co]) s[co] + beta[co]
//   back   dW[ci][tap][co] = s[co] dw'[ci][tap][co],  dgamma[co] = (sum_{ci,tap} dw' W + r (b - mu)) / sqrt(var + eps),
//          dbeta = r, db = s r
// Both are memory-bound passes over the weight; threads run along co, so every access is contiguous.
#include "common.h"

namespace convbn {

namespace {

constexpr int TT = 32;   // tile edge of the ci <-> co transpose

// grid (ceil(Co/TT), ceil(Ci/TT), taps)
template <typename T>
__global__ __launch_bounds__(256) void fold_t_kernel(const T* __restrict__ W, const float* __restrict__ b,
                                                     const float* __restrict__ gamma, const float* __restrict__ beta,
                                                     const float* __restrict__ mean, const float* __restrict__ var,
                                                     float eps, int Ci, int Co, int taps, int tap_major,
                                                     T* __restrict__ w_same, T* __restrict__ w_swap,
                                                     float* __restrict__ bfold) {
  __shared__ float tile[TT][TT + 1];
  const int tx = threadIdx.x % TT, ty = threadIdx.x / TT;   // ty in [0, 8)
  const int co0 = blockIdx.x * TT, ci0 = blockIdx.y * TT, tap = blockIdx.z;
  const int co = co0 + tx;
  // gamma == nullptr (the Eval comparison path): s = 1 and b' = b, i.e. a pure reordering of the weight
  const float s = co < Co ? (gamma ? gamma[co] / sqrtf(var[co] + eps) : 1.f) : 0.f;
  if (bfold && blockIdx.y == 0 && (tap == 0 || tap_major) && ty == 0 && co < Co)
    bfold[(tap_major ? tap * Co : 0) + co] = gamma ? ((b ? b[co] : 0.f) - mean[co]) * s + beta[co] : (b ? b[co] : 0.f);
#pragma unroll
  for (int e = 0; e < TT / 8; ++e) {
    const int ci = ci0 + ty + 8 * e;
    float v = 0.f;
    if (ci < Ci && co < Co) {
      const size_t idx = ((size_t)ci * taps + tap) * Co + co;
      // the scaled weight is rounded once, to the storage type, exactly as it is stored
      const T r = from_f32<T>(to_f32(W[idx]) * s);
      if (w_same) w_same[idx] = r;
      v = to_f32(r);
    }
    tile[ty + 8 * e][tx] = v;
  }
  if (!w_swap) return;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < TT / 8; ++e) {
    const int oc = co0 + ty + 8 * e, ic = ci0 + tx;
    if (oc < Co && ic < Ci)
      w_swap[(tap_major ? (size_t)tap * Co + oc : (size_t)oc * taps + tap) * Ci + ic] = from_f32<T>(tile[tx][ty + 8 * e]);
  }
}

constexpr int FB_ROWS = 8;   // (ci, tap) rows per workgroup of the fold-back

__device__ __forceinline__ void load4(const float* p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load4(const bf16_t* p, float (&v)[4]) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = bf16_lo(t.x); v[1] = bf16_hi(t.x); v[2] = bf16_lo(t.y); v[3] = bf16_hi(t.y);
}
__device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

// Co % 4 == 0.  grid (ceil(Co/256), ceil(rows/FB_ROWS)), rows = Ci*taps.  A wave owns every fourth row of the
// chunk and a lane four consecutive columns, so a wave reads 1 KB of every partial copy per row.
template <typename T>
__global__ __launch_bounds__(256) void fold_back_t_kernel(const float* __restrict__ part, int nsplit,
                                                          const T* __restrict__ W, const float* __restrict__ gamma,
                                                          const float* __restrict__ var, float eps, int rows, int Co,
                                                          T* __restrict__ dW, float* __restrict__ dot_part) {
  __shared__ float red[4][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.x * 256 + lane * 4;
  const int r0 = blockIdx.y * FB_ROWS, r1 = min(rows, r0 + FB_ROWS);
  const size_t P = (size_t)rows * Co;
  float dot[4] = {0.f, 0.f, 0.f, 0.f};
  if (col < Co) {
    float s[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) s[e] = gamma ? gamma[col + e] / sqrtf(var[col + e] + eps) : 1.f;   // null: plain sum
    for (int r = r0 + wave; r < r1; r += 4) {
      const size_t idx = (size_t)r * Co + col;
      float w[4], dw[4] = {0.f, 0.f, 0.f, 0.f};
      load4(W + idx, w);
#pragma unroll 4
      for (int sp = 0; sp < nsplit; ++sp) {
        const float4 t = *reinterpret_cast<const float4*>(part + sp * P + idx);
        dw[0] += t.x; dw[1] += t.y; dw[2] += t.z; dw[3] += t.w;
      }
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) { o[e] = s[e] * dw[e]; dot[e] += dw[e] * w[e]; }
      store4(dW + idx, o);
    }
  }
  if (!dot_part) return;
#pragma unroll
  for (int e = 0; e < 4; ++e) red[wave][lane * 4 + e] = dot[e];
  __syncthreads();
  const int co = blockIdx.x * 256 + threadIdx.x;
  if (co < Co)
    dot_part[(size_t)blockIdx.y * Co + co] = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
}

// Any Co.  grid (ceil(Co/64), ceil(rows/FB_ROWS)).  Thread -> column tid%64, row lane tid/64.
template <typename T>
__global__ __launch_bounds__(256) void fold_back_t_scalar_kernel(const float* __restrict__ part, int nsplit,
                                                                 const T* __restrict__ W,
                                                                 const float* __restrict__ gamma,
                                                                 const float* __restrict__ var, float eps, int rows,
                                                                 int Co, T* __restrict__ dW,
                                                                 float* __restrict__ dot_part) {
  __shared__ float red[4][64];
  const int c = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int co = blockIdx.x * 64 + c;
  const int r0 = blockIdx.y * FB_ROWS, r1 = min(rows, r0 + FB_ROWS);
  const size_t P = (size_t)rows * Co;
  float dot = 0.f;
  if (co < Co) {
    const float s = gamma ? gamma[co] / sqrtf(var[co] + eps) : 1.f;
    for (int r = r0 + rl; r < r1; r += 4) {
      const size_t idx = (size_t)r * Co + co;
      float dw = 0.f;
      for (int sp = 0; sp < nsplit; ++sp) dw += part[sp * P + idx];
      dW[idx] = from_f32<T>(s * dw);
      dot += dw * to_f32(W[idx]);
    }
  }
  if (!dot_part) return;
  red[rl][c] = dot;
  __syncthreads();
  if (rl == 0 && co < Co) dot_part[(size_t)blockIdx.y * Co + co] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
}

// grid ceil(Co/16); thread -> column tid%16, and every sixteenth partial row starting at tid/16
__global__ __launch_bounds__(256) void fold_back_t_finish_kernel(const float* __restrict__ dot_part, int nchunks,
                                                                 const float* __restrict__ r_part, int nrpart,
                                                                 const float* __restrict__ b,
                                                                 const float* __restrict__ gamma,
                                                                 const float* __restrict__ mean,
                                                                 const float* __restrict__ var, float eps, int Co,
                                                                 float* __restrict__ db, float* __restrict__ dgamma,
                                                                 float* __restrict__ dbeta) {
  __shared__ float red[2][16][17];
  const int c = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int co = blockIdx.x * 16 + c;
  float dot = 0.f, r = 0.f;
  if (co < Co) {
    // eight loads in flight per thread: the rows lie Co floats apart, each load is a round trip of its own
    for (int k = g; k < nchunks; k += 16 * 8) {
      float a[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) a[j] = k + 16 * j < nchunks ? dot_part[(size_t)(k + 16 * j) * Co + co] : 0.f;
      dot += ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
    }
    for (int k = g; k < nrpart; k += 16 * 8) {
      float a[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) a[j] = k + 16 * j < nrpart ? r_part[(size_t)(k + 16 * j) * Co + co] : 0.f;
      r += ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
    }
  }
  red[0][g][c] = dot;
  red[1][g][c] = r;
  __syncthreads();
  if (g != 0 || co >= Co) return;
  dot = 0.f; r = 0.f;
#pragma unroll
  for (int k = 0; k < 16; ++k) { dot += red[0][k][c]; r += red[1][k][c]; }
  const float sd = sqrtf(var[co] + eps);
  dgamma[co] = (dot + r * ((b ? b[co] : 0.f) - mean[co])) / sd;
  dbeta[co] = r;
  if (db) db[co] = gamma[co] / sd * r;
}

}  // namespace

hipError_t launch_fold_t(int dtype, int Ci, int Co, int taps, const void* W, const float* b, const float* gamma,
                         const float* beta, const float* mean, const float* var, float eps, int tap_major,
                         void* w_same, void* w_swap, float* bfold, hipStream_t st) {
  const dim3 grid(ceil_div(Co, TT), ceil_div(Ci, TT), taps);
  if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(fold_t_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)W, b, gamma, beta, mean, var, eps,
                       Ci, Co, taps, tap_major, (bf16_t*)w_same, (bf16_t*)w_swap, bfold);
  else
    hipLaunchKernelGGL(fold_t_kernel<float>, grid, dim3(256), 0, st, (const float*)W, b, gamma, beta, mean, var, eps,
                       Ci, Co, taps, tap_major, (float*)w_same, (float*)w_swap, bfold);
  return hipGetLastError();
}

int fold_back_t_chunks(int Ci, int taps) { return ceil_div(Ci * taps, FB_ROWS); }

hipError_t launch_fold_back_t(int dtype, int Ci, int Co, int taps, const float* dwf_part, int nsplit,
                              const float* r_part, int nrpart, const void* W, const float* b, const float* gamma,
                              const float* mean, const float* var, float eps, float* dot_part, void* dW, float* db,
                              float* dgamma, float* dbeta, hipStream_t st) {
  const int rows = Ci * taps, chunks = fold_back_t_chunks(Ci, taps);
  const bool vec = Co % 4 == 0;
  const dim3 grid(ceil_div(Co, vec ? 256 : 64), chunks);
#define FBT(KERNEL, T) \
  hipLaunchKernelGGL(KERNEL<T>, grid, dim3(256), 0, st, dwf_part, nsplit, (const T*)W, gamma, var, eps, rows, Co, \
                     (T*)dW, dot_part)
  if (dtype == CONVBN_BF16) { if (vec) FBT(fold_back_t_kernel, bf16_t); else FBT(fold_back_t_scalar_kernel, bf16_t); }
  else { if (vec) FBT(fold_back_t_kernel, float); else FBT(fold_back_t_scalar_kernel, float); }
#undef FBT
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !gamma) return e;   // no gamma: dW = sum of the partial copies, nothing else
  hipLaunchKernelGGL(fold_back_t_finish_kernel, dim3(ceil_div(Co, 16)), dim3(256), 0, st, dot_part, chunks, r_part,
                     nrpart, b, gamma, mean, var, eps, Co, db, dgamma, dbeta);
  return hipGetLastError();
}

}  // namespace convbn
