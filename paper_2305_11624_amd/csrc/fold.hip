// Memory-bound kernels around the convolution:
//   fold        w' = s w, b' = (b - mu) s + beta            (Sec. 3.3, definitions of w', b')
//   fold-back   dW = s dw', dgamma, dbeta, db               (Table 2, row "Tune")
//   colsum      r_c = sum_{n,h,w} dZ                        (App. B: backward of a broadcast)
//   bn_affine   Z = gamma (Y - mu)/sqrt(var+eps) + beta     (Sec. 3.1; Eval comparison path)
//   bn_bwd      dY = s dZ and the per-channel sums of Table 2, row "Eval"
#include "common.h"

#include <cstring>

namespace convbn {

namespace {

constexpr int FOLD_TCO = 32;  // output channels per tile
constexpr int FOLD_TK = 64;   // reduction-index (tap, ci) entries per tile

// One tile = FOLD_TCO rows of W x FOLD_TK columns.  Rows of W ([Cout][K], K = taps*Cin)
// are read coalesced along K, scaled, written back in the same order (w_krsc) and,
// through an LDS transpose, as [Cin][taps][Cout] (w_crsk) with Cout contiguous.
template <typename T>
__global__ __launch_bounds__(256) void fold_kernel(const T* __restrict__ W, const float* __restrict__ b,
                                                   const float* __restrict__ gamma,
                                                   const float* __restrict__ beta,
                                                   const float* __restrict__ mean,
                                                   const float* __restrict__ var, float eps,
                                                   int identity, int Cout, int K, int Cin, int taps,
                                                   T* __restrict__ w_krsc, T* __restrict__ w_crsk,
                                                   float* __restrict__ bfold) {
  __shared__ T tile[FOLD_TK][FOLD_TCO + 2];
  const int tid = threadIdx.x;
  const int co0 = blockIdx.y * FOLD_TCO;
  const int k0 = blockIdx.x * FOLD_TK;
  // Every load of the kernel (weights, the per-row BN vectors, the inputs of b') is issued before the
  // first use, so the kernel pays one memory round trip, not one per dependent stage.
  const bool do_bias = blockIdx.x == 0 && tid < FOLD_TCO && bfold && co0 + tid < Cout;
  float bg = 1.f, bv = 1.f, bm = 0.f, bb = 0.f, bc = 0.f;
  if (do_bias) {
    const int co = co0 + tid;
    if (!identity) { bg = gamma[co]; bv = var[co]; bm = mean[co]; bb = beta[co]; }
    if (b) bc = b[co];
  }
  // read + scale: a wave reads 64 consecutive columns of one row; rows tid/64 + 4e
  {
    const int kc = tid & 63;
    const int k = k0 + kc;
    T wv[FOLD_TCO / 4];
    float gv[FOLD_TCO / 4], vv[FOLD_TCO / 4];
#pragma unroll
    for (int e = 0; e < FOLD_TCO / 4; ++e) {
      const int co = co0 + (tid >> 6) + 4 * e;
      const bool ok = co < Cout && k < K;
      wv[e] = ok ? W[(size_t)co * K + k] : from_f32<T>(0.f);
      gv[e] = (ok && !identity) ? gamma[co] : 1.f;
      vv[e] = (ok && !identity) ? var[co] : 1.f - eps;
    }
#pragma unroll
    for (int e = 0; e < FOLD_TCO / 4; ++e) {
      const int r = (tid >> 6) + 4 * e;
      const int co = co0 + r;
      const float sc = identity ? 1.f : gv[e] / sqrtf(vv[e] + eps);
      const T v = from_f32<T>(to_f32(wv[e]) * sc);
      if (co < Cout && k < K && w_krsc) w_krsc[(size_t)co * K + k] = v;
      tile[kc][r] = v;
    }
  }
  if (do_bias) {
    const float sc = identity ? 1.f : bg / sqrtf(bv + eps);
    bfold[co0 + tid] = identity ? bc : (bc - bm) * sc + bb;
  }
  if (!w_crsk) return;
  __syncthreads();
  // transposed write: thread -> (k row = tid/4, co cols (tid%4)*8 .. +8)
  {
    const int kr = tid >> 2;
    const int cc = (tid & 3) * 8;
    const int k = k0 + kr;
    if (k < K) {
      const int tap = k / Cin, ci = k - tap * Cin;
      T* dst = w_crsk + ((size_t)ci * taps + tap) * Cout + co0;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (co0 + cc + e < Cout) dst[cc + e] = tile[kr][cc + e];
    }
  }
}

// bf16 fast path (K and Cout multiples of 8): 64 x 64 tiles, every global access is a 16-byte vector --
// rows of W are read and written back eight columns per thread, the transposed copy leaves through an
// LDS tile as rows of 64 consecutive output channels.
struct FoldArgs {
  const bf16_t* W; const float* b; const float* gamma; const float* beta; const float* mean; const float* var;
  bf16_t* w_krsc; bf16_t* w_crsk; float* bfold;
  float eps; int identity, Cout, K, Cin, taps;
};
// One 64 x 64 tile (bx along K, by along Cout) of one block's fold.
__device__ __forceinline__ void fold_tile_bf16x8(const FoldArgs& a, int bx, int by, unsigned short (*tile)[72]) {
  const bf16_t* __restrict__ W = a.W;
  const float* __restrict__ b = a.b; const float* __restrict__ gamma = a.gamma; const float* __restrict__ beta = a.beta;
  const float* __restrict__ mean = a.mean; const float* __restrict__ var = a.var;
  bf16_t* __restrict__ w_krsc = a.w_krsc; bf16_t* __restrict__ w_crsk = a.w_crsk; float* __restrict__ bfold = a.bfold;
  const float eps = a.eps;
  const int identity = a.identity, Cout = a.Cout, K = a.K, Cin = a.Cin, taps = a.taps;
  const int tid = threadIdx.x;
  const int co0 = by * 64;
  const int k0 = bx * 64;
  const bool do_bias = bx == 0 && tid < 64 && bfold && co0 + tid < Cout;
  float bg = 1.f, bv = 1.f, bm = 0.f, bb = 0.f, bc = 0.f;
  if (do_bias) {
    const int co = co0 + tid;
    if (!identity) { bg = gamma[co]; bv = var[co]; bm = mean[co]; bb = beta[co]; }
    if (b) bc = b[co];
  }
  const int kv = (tid & 7) * 8, r = tid >> 3;
  uint4 wv[2];
  float gv[2], vv[2];
  bool ok[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int co = co0 + r + 32 * e;
    ok[e] = co < Cout && k0 + kv < K;
    wv[e] = ok[e] ? *reinterpret_cast<const uint4*>(W + (size_t)co * K + k0 + kv) : make_uint4(0u, 0u, 0u, 0u);
    gv[e] = (ok[e] && !identity) ? gamma[co] : 1.f;
    vv[e] = (ok[e] && !identity) ? var[co] : 1.f - eps;
  }
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const float sc = identity ? 1.f : gv[e] / sqrtf(vv[e] + eps);
    const uint32_t in[4] = {wv[e].x, wv[e].y, wv[e].z, wv[e].w};
    uint32_t out[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[i] = pack_bf16x2(bf16_lo(in[i]) * sc, bf16_hi(in[i]) * sc);
      tile[kv + 2 * i][r + 32 * e] = (unsigned short)(out[i] & 0xffffu);
      tile[kv + 2 * i + 1][r + 32 * e] = (unsigned short)(out[i] >> 16);
    }
    if (ok[e] && w_krsc)
      *reinterpret_cast<uint4*>(w_krsc + (size_t)(co0 + r + 32 * e) * K + k0 + kv) = make_uint4(out[0], out[1], out[2], out[3]);
  }
  if (do_bias) {
    const float sc = identity ? 1.f : bg / sqrtf(bv + eps);
    bfold[co0 + tid] = identity ? bc : (bc - bm) * sc + bb;
  }
  __syncthreads();
  if (!w_crsk) return;
  const int kl = tid >> 2, c16 = (tid & 3) * 16;
  const int k = k0 + kl;
  if (k < K) {
    const int tap = k / Cin, ci = k - tap * Cin;
    bf16_t* dst = w_crsk + ((size_t)ci * taps + tap) * Cout + co0 + c16;
#pragma unroll
    for (int h = 0; h < 2; ++h)
      if (co0 + c16 + 8 * h < Cout)
        *reinterpret_cast<uint4*>(dst + 8 * h) = *reinterpret_cast<const uint4*>(&tile[kl][c16 + 8 * h]);
  }
}

__global__ __launch_bounds__(256) void fold_bf16x8_kernel(FoldArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned short tile[64][72];   // [k][co], 144-byte rows
  fold_tile_bf16x8(a, blockIdx.x, blockIdx.y, tile);
}

// The folds of several blocks in one launch (Sec. 3.3: a training step starts by folding every block's
// BatchNorm into its weights; one launch per block would be bound by the launches, not by memory).
// items[i] covers blocks [first_block, first_block + tiles): tile t of item i is (t % tiles_k, t / tiles_k).
struct FoldGroupItem { FoldArgs a; int first_block, tiles_k; };
__global__ __launch_bounds__(256) void fold_group_kernel(const FoldGroupItem* __restrict__ items, int n) {
  __shared__ __attribute__((aligned(16))) unsigned short tile[64][72];
  int lo = 0, hi = n - 1;   // last item whose first_block <= blockIdx.x
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (items[mid].first_block <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const FoldGroupItem it = items[lo];
  const int t = blockIdx.x - it.first_block;
  fold_tile_bf16x8(it.a, t % it.tiles_k, t / it.tiles_k, tile);
}

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void load4(const float* p, float (&w)[4]) {
  const float4 v = ld4(p);
  w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
}
__device__ __forceinline__ void load4(const bf16_t* p, float (&w)[4]) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
  w[0] = bf16_lo(v.x); w[1] = bf16_hi(v.x); w[2] = bf16_lo(v.y); w[3] = bf16_hi(v.y);
}
__device__ __forceinline__ void store4(float* p, const float (&w)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&w)[4]) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3]));
}

// One block per output channel.  VEC (K % 4 == 0): a thread owns float4 columns of the row.  The
// `nsplit` partial copies of a column lie far apart in memory, so every load is a latency round trip of
// its own.  Short rows (fewer than 256 columns): a thread keeps sixteen copies of one column in
// flight, the copies are divided over as many thread groups as fit the block, and the groups meet in
// LDS.  Long rows: a column per thread, four copies in flight, columns in sequence.  Rows whose length is not a
// multiple of 4: one element per thread; short ones divide the copies over thread groups in the same way.
template <typename T, bool VEC, int NTHR>
__device__ __forceinline__ void fold_back_row(
    const int co, const float* __restrict__ part, int nsplit, const float* __restrict__ r_part, int nrpart,
    const T* __restrict__ W, const float* __restrict__ b, const float* __restrict__ gamma,
    const float* __restrict__ mean, const float* __restrict__ var, float eps, int identity, int Cout,
    int K, T* __restrict__ dW, float* __restrict__ db, float* __restrict__ dgamma,
    float* __restrict__ dbeta) {
  constexpr int NSL = NTHR / 64;
  __shared__ float4 red4[VEC ? NTHR : 1];
  __shared__ float reds[VEC ? 1 : NTHR];
  __shared__ float red[NSL];
  const int tid = threadIdx.x;
  const size_t P = (size_t)Cout * K;
  float s = 1.f, sd = 1.f;
  if (!identity) {
    sd = sqrtf(var[co] + eps);
    s = gamma[co] / sd;
  }
  float dot = 0.f;
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  auto finish = [&](int k4, const float4& v) {   // dW = s dw', <dw', w> of one float4 column
    const float g4[4] = {v.x, v.y, v.z, v.w};
    float w4[4], o4[4];
    load4(W + (size_t)co * K + 4 * k4, w4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      o4[e] = s * g4[e];
      dot += g4[e] * w4[e];
    }
    store4(dW + (size_t)co * K + 4 * k4, o4);
  };
  if (VEC && (K >> 2) >= 256) {
    // long rows: one float4 column per thread at a time, all partial copies summed in registers, no
    // barriers (many such blocks share a CU, which keeps enough loads in flight)
    const int K4 = K >> 2;
    const float* row = part + (size_t)co * K;
    for (int k4 = tid; k4 < K4; k4 += NTHR) {
      float4 v = zero4;
      int sp = 0;
      for (; sp + 3 < nsplit; sp += 4) {
        const float4 a0 = ld4(row + (size_t)sp * P + 4 * k4);
        const float4 a1 = ld4(row + (size_t)(sp + 1) * P + 4 * k4);
        const float4 a2 = ld4(row + (size_t)(sp + 2) * P + 4 * k4);
        const float4 a3 = ld4(row + (size_t)(sp + 3) * P + 4 * k4);
        v.x += (a0.x + a1.x) + (a2.x + a3.x);
        v.y += (a0.y + a1.y) + (a2.y + a3.y);
        v.z += (a0.z + a1.z) + (a2.z + a3.z);
        v.w += (a0.w + a1.w) + (a2.w + a3.w);
      }
      for (; sp < nsplit; ++sp) {
        const float4 a0 = ld4(row + (size_t)sp * P + 4 * k4);
        v.x += a0.x; v.y += a0.y; v.z += a0.z; v.w += a0.w;
      }
      finish(k4, v);
    }
  } else if (VEC) {
    // short rows (fewer than 256 columns): thread -> (column c, group g of the partial copies)
    const int K4 = K >> 2;
    const int G = NTHR / K4;
    const int c = tid % K4, g = tid / K4;
    float4 v = zero4;
    if (g < G) {
      const float* col = part + (size_t)co * K + 4 * c;
      for (int sp0 = g; sp0 < nsplit; sp0 += 16 * G) {
        float4 a[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) a[j] = sp0 + j * G < nsplit ? ld4(col + (size_t)(sp0 + j * G) * P) : zero4;
#pragma unroll
        for (int j = 0; j < 16; j += 4) {
          v.x += (a[j].x + a[j + 1].x) + (a[j + 2].x + a[j + 3].x);
          v.y += (a[j].y + a[j + 1].y) + (a[j + 2].y + a[j + 3].y);
          v.z += (a[j].z + a[j + 1].z) + (a[j + 2].z + a[j + 3].z);
          v.w += (a[j].w + a[j + 1].w) + (a[j + 2].w + a[j + 3].w);
        }
      }
    }
    red4[tid] = v;
    __syncthreads();
    if (g == 0) {
      for (int l = 1; l < G; ++l) {
        const float4 o = red4[l * K4 + c];
        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
      }
      finish(c, v);
    }
  } else if (K * 2 <= NTHR) {
    // short rows whose length is not a multiple of 4 (a first layer: 7 x 7 x 3): thread -> (element k, group g of the
    // partial copies), eight copies in flight per thread, the groups meet in LDS
    const int G = NTHR / K;
    const int k = tid % K, g = tid / K;
    float v = 0.f;
    if (g < G) {
      const float* col = part + (size_t)co * K + k;
      for (int sp0 = g; sp0 < nsplit; sp0 += 8 * G) {
        float a[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = sp0 + j * G < nsplit ? col[(size_t)(sp0 + j * G) * P] : 0.f;
        v += ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
      }
    }
    reds[tid] = v;
    __syncthreads();
    if (g == 0) {
      for (int l = 1; l < G; ++l) v += reds[l * K + k];
      const size_t idx = (size_t)co * K + k;
      dW[idx] = from_f32<T>(s * v);
      dot += v * to_f32(W[idx]);
    }
  } else {
    for (int k = tid; k < K; k += NTHR) {
      const size_t idx = (size_t)co * K + k;
      float v = 0.f;
      int sp = 0;
      for (; sp + 7 < nsplit; sp += 8) {   // eight copies in flight: each load is a round trip of its own
        float a[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = part[(sp + j) * P + idx];
        v += ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
      }
      for (; sp < nsplit; ++sp) v += part[sp * P + idx];
      dW[idx] = from_f32<T>(s * v);
      dot += v * to_f32(W[idx]);
    }
  }
  if (identity) return;
  float r = 0.f;
  for (int q = tid; q < nrpart; q += NTHR) r += r_part[(size_t)q * Cout + co];
  dot = wave_sum(dot);
  r = wave_sum(r);
  __shared__ float redr[NSL];
  if ((tid & 63) == 0) { red[tid >> 6] = dot; redr[tid >> 6] = r; }
  __syncthreads();
  if (tid == 0) {
    dot = 0.f;
    r = 0.f;
    for (int l = 0; l < NSL; ++l) { dot += red[l]; r += redr[l]; }
    const float bc = b ? b[co] : 0.f;
    dbeta[co] = r;
    dgamma[co] = (dot + r * (bc - mean[co])) / sd;
    if (db) db[co] = s * r;
  }
}

template <typename T, bool VEC, int NTHR>
__global__ __launch_bounds__(NTHR) void fold_back_kernel(
    const float* __restrict__ part, int nsplit, const float* __restrict__ r_part, int nrpart,
    const T* __restrict__ W, const float* __restrict__ b, const float* __restrict__ gamma,
    const float* __restrict__ mean, const float* __restrict__ var, float eps, int identity, int Cout,
    int K, T* __restrict__ dW, float* __restrict__ db, float* __restrict__ dgamma,
    float* __restrict__ dbeta) {
  fold_back_row<T, VEC, NTHR>(blockIdx.x, part, nsplit, r_part, nrpart, W, b, gamma, mean, var, eps, identity, Cout, K,
                              dW, db, dgamma, dbeta);
}

// The fold-backs of several blocks in one launch (Table 2 "Tune", last four lines, for every block of a group):
// workgroup w handles output channel w - first_block of the item it falls into.  Same arithmetic, in the same
// order, as the 256-thread single-block kernel.
struct FoldBackGroupItem {
  const float* part; const float* r_part; const bf16_t* W; const float* b; const float* gamma; const float* mean;
  const float* var; bf16_t* dW; float* db; float* dgamma; float* dbeta;
  float eps; int nsplit, nrpart, Cout, K, first_block;
};
__global__ __launch_bounds__(256) void fold_back_group_kernel(const FoldBackGroupItem* __restrict__ items, int n) {
  int lo = 0, hi = n - 1;   // last item whose first_block <= blockIdx.x
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (items[mid].first_block <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const FoldBackGroupItem it = items[lo];
  fold_back_row<bf16_t, true, 256>(blockIdx.x - it.first_block, it.part, it.nsplit, it.r_part, it.nrpart, it.W, it.b,
                                   it.gamma, it.mean, it.var, it.eps, 0, it.Cout, it.K, it.dW, it.db, it.dgamma,
                                   it.dbeta);
}

// Column reductions over a [M][Cout] channels-last tensor.  `cw` threads walk the
// channel dimension (coalesced), 256/cw row lanes stride over this block's rows.
__device__ __forceinline__ int pow2_cw(int Cout) {
  int cw = 1;
  while (cw < Cout && cw < 256) cw <<= 1;
  return cw;
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ dz, int M, int Cout,
                                                     int rows_per_block, float* __restrict__ part) {
  __shared__ float red[256];
  const int cw = pow2_cw(Cout);
  const int lanes = 256 / cw;
  const int tc = threadIdx.x % cw, tr = threadIdx.x / cw;
  const int m0 = blockIdx.x * rows_per_block;
  const int m1 = min(M, m0 + rows_per_block);
  for (int c0 = 0; c0 < Cout; c0 += cw) {
    const int co = c0 + tc;
    float acc = 0.f;
    if (co < Cout)
      for (int m = m0 + tr; m < m1; m += lanes) acc += to_f32(dz[(size_t)m * Cout + co]);
    red[threadIdx.x] = acc;
    __syncthreads();
    if (tr == 0 && co < Cout) {
      for (int l = 1; l < lanes; ++l) acc += red[l * cw + tc];
      part[(size_t)blockIdx.x * Cout + co] = acc;
    }
    __syncthreads();
  }
}

// bf16, Cout % 8 == 0: a thread reads 8 channels (16 bytes) of a row; (Cout/8) threads cover a row,
// the remaining factor of the block strides over rows.  Requires Cout/8 <= 256.
__global__ __launch_bounds__(256) void colsum_bf16x8_kernel(const uint4* __restrict__ dz, int M, int Cout,
                                                            int rows_per_block, float* __restrict__ part) {
  __shared__ float red[256][9];
  const int c8 = Cout >> 3;
  const int lanes = 256 / c8;
  const int tc = threadIdx.x % c8, tr = threadIdx.x / c8;
  const int m0 = blockIdx.x * rows_per_block;
  const int m1 = min(M, m0 + rows_per_block);
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (tr < lanes)
    for (int m = m0 + tr; m < m1; m += lanes) {
      const uint4 v = dz[(size_t)m * c8 + tc];
      a[0] += bf16_lo(v.x); a[1] += bf16_hi(v.x); a[2] += bf16_lo(v.y); a[3] += bf16_hi(v.y);
      a[4] += bf16_lo(v.z); a[5] += bf16_hi(v.z); a[6] += bf16_lo(v.w); a[7] += bf16_hi(v.w);
    }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[threadIdx.x][e] = a[e];
  __syncthreads();
  for (int c = threadIdx.x; c < Cout; c += 256) {
    float acc = 0.f;
    for (int l = 0; l < lanes; ++l) acc += red[l * c8 + (c >> 3)][c & 7];
    part[(size_t)blockIdx.x * Cout + c] = acc;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_affine_fwd_kernel(const T* __restrict__ y,
                                                            const float* __restrict__ gamma,
                                                            const float* __restrict__ beta,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ var, float eps,
                                                            size_t total, int Cout, T* __restrict__ z) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
    const int co = (int)(i % Cout);
    const float ybar = (to_f32(y[i]) - mean[co]) / sqrtf(var[co] + eps);
    z[i] = from_f32<T>(gamma[co] * ybar + beta[co]);
  }
}

// 8 bf16 per thread, Cout % 8 == 0; per-channel scale/shift staged in LDS (2*Cout floats).
__global__ __launch_bounds__(256) void bn_affine_fwd_bf16x8_kernel(
    const uint4* __restrict__ y, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ var, float eps, size_t nvec, int Cout,
    uint4* __restrict__ z, int relu, const uint4* __restrict__ add) {
  extern __shared__ float sm[];
  float* s_s = sm;
  float* s_t = sm + Cout;
  for (int c = threadIdx.x; c < Cout; c += 256) {
    const float s = gamma[c] / sqrtf(var[c] + eps);
    s_s[c] = s;
    s_t[c] = beta[c] - mean[c] * s;
  }
  __syncthreads();
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
    const int co = (int)((i * 8) % Cout);
    const uint4 v = y[i];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int c = co + 2 * e;
      o[e] = pack_bf16x2(bf16_lo(w[e]) * s_s[c] + s_t[c], bf16_hi(w[e]) * s_s[c + 1] + s_t[c + 1]);
    }
    uint4 r = make_uint4(o[0], o[1], o[2], o[3]);
    if (add) r = add8(r, add[i]);   // (an addend and a ReLU behind the block: the descriptor's activation bits)
    z[i] = relu ? relu8(r) : r;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_kernel(const T* __restrict__ dz, const T* __restrict__ y,
                                                     const float* __restrict__ gamma,
                                                     const float* __restrict__ mean,
                                                     const float* __restrict__ var, float eps, int M,
                                                     int Cout, int rows_per_block, T* __restrict__ dy,
                                                     float* __restrict__ part) {
  __shared__ float red0[256];
  __shared__ float red1[256];
  const int cw = pow2_cw(Cout);
  const int lanes = 256 / cw;
  const int tc = threadIdx.x % cw, tr = threadIdx.x / cw;
  const int m0 = blockIdx.x * rows_per_block;
  const int m1 = min(M, m0 + rows_per_block);
  for (int c0 = 0; c0 < Cout; c0 += cw) {
    const int co = c0 + tc;
    float a0 = 0.f, a1 = 0.f;
    if (co < Cout) {
      const float sd = sqrtf(var[co] + eps);
      const float s = gamma[co] / sd, mu = mean[co];
      for (int m = m0 + tr; m < m1; m += lanes) {
        const size_t idx = (size_t)m * Cout + co;
        const float g = to_f32(dz[idx]);
        dy[idx] = from_f32<T>(s * g);
        a0 += g;
        a1 += g * ((to_f32(y[idx]) - mu) / sd);
      }
    }
    red0[threadIdx.x] = a0;
    red1[threadIdx.x] = a1;
    __syncthreads();
    if (tr == 0 && co < Cout) {
      for (int l = 1; l < lanes; ++l) {
        a0 += red0[l * cw + tc];
        a1 += red1[l * cw + tc];
      }
      part[((size_t)blockIdx.x * 2 + 0) * Cout + co] = a0;
      part[((size_t)blockIdx.x * 2 + 1) * Cout + co] = a1;
    }
    __syncthreads();
  }
}

// bf16, Cout % 8 == 0, Cout <= 2048: 16 bytes (8 channels) per thread per row, as colsum_bf16x8_kernel.
__global__ __launch_bounds__(256) void bn_bwd_bf16x8_kernel(const uint4* __restrict__ dz, const uint4* __restrict__ y,
                                                            const float* __restrict__ gamma,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ var, float eps, int M,
                                                            int Cout, int rows_per_block, uint4* __restrict__ dy,
                                                            float* __restrict__ part) {
  __shared__ float red0[256][9];
  __shared__ float red1[256][9];
  const int c8 = Cout >> 3;
  const int lanes = 256 / c8;
  const int tc = threadIdx.x % c8, tr = threadIdx.x / c8;
  const int m0 = blockIdx.x * rows_per_block;
  const int m1 = min(M, m0 + rows_per_block);
  float a0[8], a1[8], sc[8], mu[8], isd[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a0[e] = 0.f; a1[e] = 0.f;
    const int c = min(tc * 8 + e, Cout - 1);
    isd[e] = 1.f / sqrtf(var[c] + eps);
    sc[e] = gamma[c] * isd[e];
    mu[e] = mean[c];
  }
  if (tr < lanes)
    for (int m = m0 + tr; m < m1; m += lanes) {
      const size_t idx = (size_t)m * c8 + tc;
      const uint4 g4 = dz[idx], y4 = y[idx];
      const uint32_t gw[4] = {g4.x, g4.y, g4.z, g4.w}, yw[4] = {y4.x, y4.y, y4.z, y4.w};
      uint32_t ow[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float g0 = bf16_lo(gw[e]), g1 = bf16_hi(gw[e]);
        const float y0 = bf16_lo(yw[e]), y1 = bf16_hi(yw[e]);
        ow[e] = pack_bf16x2(sc[2 * e] * g0, sc[2 * e + 1] * g1);
        a0[2 * e] += g0; a0[2 * e + 1] += g1;
        a1[2 * e] += g0 * ((y0 - mu[2 * e]) * isd[2 * e]);
        a1[2 * e + 1] += g1 * ((y1 - mu[2 * e + 1]) * isd[2 * e + 1]);
      }
      dy[idx] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    }
#pragma unroll
  for (int e = 0; e < 8; ++e) { red0[threadIdx.x][e] = a0[e]; red1[threadIdx.x][e] = a1[e]; }
  __syncthreads();
  for (int c = threadIdx.x; c < Cout; c += 256) {
    float s0 = 0.f, s1 = 0.f;
    for (int l = 0; l < lanes; ++l) {
      s0 += red0[l * c8 + (c >> 3)][c & 7];
      s1 += red1[l * c8 + (c >> 3)][c & 7];
    }
    part[((size_t)blockIdx.x * 2 + 0) * Cout + c] = s0;
    part[((size_t)blockIdx.x * 2 + 1) * Cout + c] = s1;
  }
}

// Sums the per-workgroup partial (dbeta, dgamma) rows: 64 channels per workgroup, 16 waves each take
// every 16th partial row, then a fixed-order reduction through LDS (deterministic).
__global__ __launch_bounds__(1024) void bn_bwd_finalize_kernel(const float* __restrict__ part, int parts,
                                                               const float* __restrict__ gamma,
                                                               const float* __restrict__ var, float eps,
                                                               int Cout, float* __restrict__ dgamma,
                                                               float* __restrict__ dbeta,
                                                               float* __restrict__ db) {
  __shared__ float red[2][16][64];
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int co = blockIdx.x * 64 + lane;
  float a0 = 0.f, a1 = 0.f;
  if (co < Cout) {
#pragma unroll 4
    for (int p = slice; p < parts; p += 16) {
      a0 += part[((size_t)p * 2 + 0) * Cout + co];
      a1 += part[((size_t)p * 2 + 1) * Cout + co];
    }
  }
  red[0][slice][lane] = a0;
  red[1][slice][lane] = a1;
  __syncthreads();
  if (slice != 0 || co >= Cout) return;
  a0 = 0.f; a1 = 0.f;
#pragma unroll
  for (int q = 0; q < 16; ++q) { a0 += red[0][q][lane]; a1 += red[1][q][lane]; }
  dbeta[co] = a0;
  dgamma[co] = a1;
  if (db) db[co] = gamma[co] / sqrtf(var[co] + eps) * a0;
}

template <typename E>
__global__ __launch_bounds__(256) void repitch_kernel(const E* __restrict__ src, E* __restrict__ dst, size_t total,
                                                      size_t inner_in, size_t inner_out) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t row = i / inner_out, c = i - row * inner_out;
    dst[i] = c < inner_in ? src[row * inner_in + c] : E(0);
  }
}

int rows_per_block_for(int M, int parts) { return ceil_div(M, parts); }

}  // namespace

hipError_t launch_repitch(int elem_bytes, size_t rows, size_t inner_in, size_t inner_out, const void* src,
                          void* dst, hipStream_t st) {
  const size_t total = rows * inner_out;
  const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
  if (elem_bytes == 2)
    hipLaunchKernelGGL(repitch_kernel<unsigned short>, dim3(blocks), dim3(256), 0, st, (const unsigned short*)src,
                       (unsigned short*)dst, total, inner_in, inner_out);
  else
    hipLaunchKernelGGL(repitch_kernel<unsigned int>, dim3(blocks), dim3(256), 0, st, (const unsigned int*)src,
                       (unsigned int*)dst, total, inner_in, inner_out);
  return hipGetLastError();
}

hipError_t launch_fold(const Geom& g, int dtype, const void* W, const float* b, const float* gamma,
                       const float* beta, const float* mean, const float* var, int identity,
                       void* w_krsc, void* w_crsk, float* bfold, hipStream_t st) {
  dim3 grid(ceil_div(g.K, FOLD_TK), ceil_div(g.Cout, FOLD_TCO));
  const int taps = g.kH * g.kW;
  if (dtype == CONVBN_BF16 && g.K % 8 == 0 && g.Cout % 8 == 0)
    hipLaunchKernelGGL(fold_bf16x8_kernel, dim3(ceil_div(g.K, 64), ceil_div(g.Cout, 64)), dim3(256), 0, st,
                       FoldArgs{(const bf16_t*)W, b, gamma, beta, mean, var, (bf16_t*)w_krsc, (bf16_t*)w_crsk, bfold,
                                g.eps, identity, g.Cout, g.K, g.Cin, taps});
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(fold_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)W, b, gamma, beta,
                       mean, var, g.eps, identity, g.Cout, g.K, g.Cin, taps, (bf16_t*)w_krsc,
                       (bf16_t*)w_crsk, bfold);
  else
    hipLaunchKernelGGL(fold_kernel<float>, grid, dim3(256), 0, st, (const float*)W, b, gamma, beta,
                       mean, var, g.eps, identity, g.Cout, g.K, g.Cin, taps, (float*)w_krsc,
                       (float*)w_crsk, bfold);
  return hipGetLastError();
}

size_t fold_group_item_bytes() { return sizeof(FoldGroupItem); }

bool fold_group_item(const Geom& g, int dtype, const void* W, const float* b, const float* gamma, const float* beta,
                     const float* mean, const float* var, int identity, void* w_krsc, void* w_crsk, float* bfold,
                     int first_block, void* item_out, int* blocks) {
  if (dtype != CONVBN_BF16 || g.K % 8 != 0 || g.Cout % 8 != 0) return false;
  FoldGroupItem it{};
  it.a = FoldArgs{(const bf16_t*)W, b, gamma, beta, mean, var, (bf16_t*)w_krsc, (bf16_t*)w_crsk, bfold,
                  g.eps, identity, g.Cout, g.K, g.Cin, g.kH * g.kW};
  it.first_block = first_block;
  it.tiles_k = ceil_div(g.K, 64);
  *blocks = it.tiles_k * ceil_div(g.Cout, 64);
  memcpy(item_out, &it, sizeof(it));
  return true;
}

hipError_t launch_fold_group(const void* items_dev, int n, int grid_blocks, hipStream_t st) {
  hipLaunchKernelGGL(fold_group_kernel, dim3(grid_blocks), dim3(256), 0, st, (const FoldGroupItem*)items_dev, n);
  return hipGetLastError();
}

size_t fold_back_group_item_bytes() { return sizeof(FoldBackGroupItem); }

bool fold_back_group_item(const Geom& g, int dtype, const float* dwf_part, int nsplit, const float* r_part, int nrpart,
                          const void* W, const float* b, const float* gamma, const float* mean, const float* var,
                          void* dW, float* db, float* dgamma, float* dbeta, int first_block, void* item_out,
                          int* blocks) {
  if (dtype != CONVBN_BF16 || g.K % 4 != 0) return false;
  FoldBackGroupItem it{dwf_part, r_part, (const bf16_t*)W, b, gamma, mean, var, (bf16_t*)dW, db, dgamma, dbeta,
                       g.eps, nsplit, nrpart, g.Cout, g.K, first_block};
  *blocks = g.Cout;
  memcpy(item_out, &it, sizeof(it));
  return true;
}

hipError_t launch_fold_back_group(const void* items_dev, int n, int grid_blocks, hipStream_t st) {
  hipLaunchKernelGGL(fold_back_group_kernel, dim3(grid_blocks), dim3(256), 0, st, (const FoldBackGroupItem*)items_dev, n);
  return hipGetLastError();
}

hipError_t launch_fold_back(const Geom& g, int dtype, const float* dwf_part, int nsplit,
                            const float* r_part, int nrpart, const void* W, const float* b,
                            const float* gamma, const float* mean, const float* var, int identity,
                            void* dW, float* db, float* dgamma, float* dbeta, hipStream_t st) {
#define FB_LAUNCH(T, VEC, NTHR)                                                                          \
  hipLaunchKernelGGL((fold_back_kernel<T, VEC, NTHR>), dim3(g.Cout), dim3(NTHR), 0, st, dwf_part, nsplit, \
                     r_part, nrpart, (const T*)W, b, gamma, mean, var, g.eps, identity, g.Cout,           \
                     g.K, (T*)dW, db, dgamma, dbeta)
  const bool vec = g.K % 4 == 0;
  // few output channels and many partial copies: a 1024-thread block per channel (16 waves share
  // the copies) keeps enough loads in flight on the few CUs such a grid occupies
  const bool wide = vec && g.Cout <= 128 && nsplit >= 16 && (g.K >> 2) < 256;
  const bool wide_scalar = !vec && g.Cout <= 128 && nsplit >= 16 && g.K * 2 <= 1024;   // (a first layer's 7 x 7 x 3 rows)
  if (dtype == CONVBN_BF16) {
    if (wide) FB_LAUNCH(bf16_t, true, 1024);
    else if (vec) FB_LAUNCH(bf16_t, true, 256);
    else if (wide_scalar) FB_LAUNCH(bf16_t, false, 1024);
    else FB_LAUNCH(bf16_t, false, 256);
  } else {
    if (wide) FB_LAUNCH(float, true, 1024);
    else if (vec) FB_LAUNCH(float, true, 256);
    else if (wide_scalar) FB_LAUNCH(float, false, 1024);
    else FB_LAUNCH(float, false, 256);
  }
#undef FB_LAUNCH
  return hipGetLastError();
}

int colsum_parts(const Geom& g) { return g.M < 256 * 64 ? ceil_div(g.M, 64) : 256; }

hipError_t launch_colsum(const Geom& g, int dtype, const void* dz, float* r_part, hipStream_t st) {
  const int parts = colsum_parts(g);
  const int rpb = rows_per_block_for(g.M, parts);
  if (dtype == CONVBN_BF16 && g.Cout % 8 == 0 && g.Cout <= 2048)
    hipLaunchKernelGGL(colsum_bf16x8_kernel, dim3(parts), dim3(256), 0, st, (const uint4*)dz, g.M, g.Cout,
                       rpb, r_part);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(colsum_kernel<bf16_t>, dim3(parts), dim3(256), 0, st, (const bf16_t*)dz, g.M,
                       g.Cout, rpb, r_part);
  else
    hipLaunchKernelGGL(colsum_kernel<float>, dim3(parts), dim3(256), 0, st, (const float*)dz, g.M,
                       g.Cout, rpb, r_part);
  return hipGetLastError();
}

hipError_t launch_bn_affine_fwd(const Geom& g, int dtype, const void* y, const float* gamma,
                                const float* beta, const float* mean, const float* var, void* z,
                                hipStream_t st) {
  const size_t total = (size_t)g.M * g.Cout;
  if (dtype == CONVBN_BF16 && g.Cout % 8 == 0 && g.Cout <= 4096) {
    const size_t nvec = total / 8;
    const int blocks = (int)min((size_t)2048, (nvec + 255) / 256);
    hipLaunchKernelGGL(bn_affine_fwd_bf16x8_kernel, dim3(blocks), dim3(256), 2 * g.Cout * sizeof(float), st, (const uint4*)y,
                       gamma, beta, mean, var, g.eps, nvec, g.Cout, (uint4*)z, g.post_relu, (const uint4*)g.post_add);
  } else {
    const int blocks = (int)min((size_t)4096, (total + 255) / 256);
    if (dtype == CONVBN_BF16)
      hipLaunchKernelGGL(bn_affine_fwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st,
                         (const bf16_t*)y, gamma, beta, mean, var, g.eps, total, g.Cout, (bf16_t*)z);
    else
      hipLaunchKernelGGL(bn_affine_fwd_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)y,
                         gamma, beta, mean, var, g.eps, total, g.Cout, (float*)z);
    if (g.post_add && hipGetLastError() == hipSuccess) {
      const hipError_t e = launch_eltwise(3 /* a + b */, dtype, z, g.post_add, nullptr, total, st);
      if (e != hipSuccess) return e;
    }
    if (g.post_relu && hipGetLastError() == hipSuccess) return launch_eltwise(0 /* max(a, 0) */, dtype, z, nullptr, nullptr, total, st);
  }
  return hipGetLastError();
}

int bn_bwd_parts(const Geom& g) { return colsum_parts(g); }

hipError_t launch_bn_bwd(const Geom& g, int dtype, const void* dz, const void* y, const float* gamma,
                         const float* mean, const float* var, void* dy, float* part, hipStream_t st) {
  const int parts = bn_bwd_parts(g);
  const int rpb = rows_per_block_for(g.M, parts);
  if (dtype == CONVBN_BF16 && g.Cout % 8 == 0 && g.Cout <= 2048)
    hipLaunchKernelGGL(bn_bwd_bf16x8_kernel, dim3(parts), dim3(256), 0, st, (const uint4*)dz, (const uint4*)y,
                       gamma, mean, var, g.eps, g.M, g.Cout, rpb, (uint4*)dy, part);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(bn_bwd_kernel<bf16_t>, dim3(parts), dim3(256), 0, st, (const bf16_t*)dz,
                       (const bf16_t*)y, gamma, mean, var, g.eps, g.M, g.Cout, rpb, (bf16_t*)dy, part);
  else
    hipLaunchKernelGGL(bn_bwd_kernel<float>, dim3(parts), dim3(256), 0, st, (const float*)dz,
                       (const float*)y, gamma, mean, var, g.eps, g.M, g.Cout, rpb, (float*)dy, part);
  return hipGetLastError();
}

hipError_t launch_bn_bwd_finalize(const Geom& g, const float* part, int parts, const float* gamma,
                                  const float* var, float* dgamma, float* dbeta, float* db,
                                  hipStream_t st) {
  hipLaunchKernelGGL(bn_bwd_finalize_kernel, dim3(ceil_div(g.Cout, 64)), dim3(1024), 0, st, part, parts,
                     gamma, var, g.eps, g.Cout, dgamma, dbeta, db);
  return hipGetLastError();
}

}  // namespace convbn
