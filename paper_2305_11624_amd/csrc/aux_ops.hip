// Glue between ConvBN blocks for the whole-backbone measurement (ResNet-50: ReLU, residual add,
// 3x3/2 max-pool).  The block itself is unaffected by what follows it (Sec. 3.1); these kernels
// only let 53 blocks be chained the way the backbone chains them.  bf16 or fp32, channels-last,
// elementwise and HBM-bound.
#include "common.h"

namespace convbn {

namespace {

template <typename T> struct Vec;
template <> struct Vec<bf16_t> { static constexpr int N = 8; };
template <> struct Vec<float> { static constexpr int N = 4; };

template <typename T> __device__ __forceinline__ void ldv(const T* p, float (&v)[Vec<T>::N]);
template <> __device__ __forceinline__ void ldv<bf16_t>(const bf16_t* p, float (&v)[8]) {
  const uint4 u = *reinterpret_cast<const uint4*>(p);
  v[0] = bf16_lo(u.x); v[1] = bf16_hi(u.x); v[2] = bf16_lo(u.y); v[3] = bf16_hi(u.y);
  v[4] = bf16_lo(u.z); v[5] = bf16_hi(u.z); v[6] = bf16_lo(u.w); v[7] = bf16_hi(u.w);
}
template <> __device__ __forceinline__ void ldv<float>(const float* p, float (&v)[4]) {
  const float4 u = *reinterpret_cast<const float4*>(p);
  v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w;
}
template <typename T> __device__ __forceinline__ void stv(T* p, const float (&v)[Vec<T>::N]);
template <> __device__ __forceinline__ void stv<bf16_t>(bf16_t* p, const float (&v)[8]) {
  *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                            pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
}
template <> __device__ __forceinline__ void stv<float>(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

enum { OP_RELU = 0, OP_RELU_BWD = 1, OP_ADD_RELU = 2, OP_ADD = 3, OP_ADD_RELU_BWD = 4 };

// a (in/out), b (second operand; unused for OP_RELU).  n is a multiple of the vector width.
//   OP_RELU      a = max(a, 0)
//   OP_RELU_BWD  a = b > 0 ? a : 0          (a = gradient, b = the ReLU's output)
//   OP_ADD_RELU  a = max(a + b, 0)
//   OP_ADD       a = a + b
//   OP_ADD_RELU_BWD  a = c > 0 ? a + b : 0  (two gradient branches meet in front of a ReLU whose output is c: the
//                    sum rounded as OP_ADD rounds it, then OP_RELU_BWD, in one pass over the tensors)
template <typename T, int OP>
__global__ __launch_bounds__(256) void eltwise_kernel(T* __restrict__ a, const T* __restrict__ b, const T* __restrict__ c, size_t n) {
  constexpr int V = Vec<T>::N;
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    float x[V], y[V], m[V];
    ldv<T>(a + i * V, x);
    if (OP != OP_RELU) ldv<T>(b + i * V, y);
    if (OP == OP_ADD_RELU_BWD) ldv<T>(c + i * V, m);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      if (OP == OP_RELU) x[e] = fmaxf(x[e], 0.f);
      if (OP == OP_RELU_BWD) x[e] = y[e] > 0.f ? x[e] : 0.f;
      if (OP == OP_ADD_RELU) x[e] = fmaxf(to_f32(from_f32<T>(x[e] + y[e])), 0.f);
      if (OP == OP_ADD) x[e] = x[e] + y[e];
      if (OP == OP_ADD_RELU_BWD) x[e] = m[e] > 0.f ? x[e] + y[e] : 0.f;
    }
    stv<T>(a + i * V, x);
  }
  // the elements past the last whole vector (callers inside the library pass any n)
  for (size_t i = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    float x = to_f32(a[i]);
    const float y = OP != OP_RELU ? to_f32(b[i]) : 0.f;
    if (OP == OP_RELU) x = fmaxf(x, 0.f);
    if (OP == OP_RELU_BWD) x = y > 0.f ? x : 0.f;
    if (OP == OP_ADD_RELU) x = fmaxf(to_f32(from_f32<T>(x + y)), 0.f);
    if (OP == OP_ADD) x = x + y;
    if (OP == OP_ADD_RELU_BWD) x = to_f32(c[i]) > 0.f ? x + y : 0.f;
    a[i] = from_f32<T>(x);
  }
}

// 3x3 window, stride 2, padding 1 max-pool over [N][H][W][C]; idx keeps the winning window
// position (0..8, first maximum in row-major window order) for the backward pass.
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                          unsigned char* __restrict__ idx, int N, int H, int W,
                                                          int C, int Ho, int Wo) {
  const size_t total = (size_t)N * Ho * Wo * C;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int c = (int)(i % C);
    size_t r = i / C;
    const int wo = (int)(r % Wo); r /= Wo;
    const int ho = (int)(r % Ho);
    const int n = (int)(r / Ho);
    float best = -INFINITY;
    int bi = 0;
    for (int di = 0; di < 3; ++di) {
      const int h = ho * 2 + di - 1;
      if (h < 0 || h >= H) continue;
      for (int dj = 0; dj < 3; ++dj) {
        const int w = wo * 2 + dj - 1;
        if (w < 0 || w >= W) continue;
        const float v = to_f32(x[(((size_t)n * H + h) * W + w) * C + c]);
        if (v > best) { best = v; bi = di * 3 + dj; }
      }
    }
    y[i] = from_f32<T>(best);
    idx[i] = (unsigned char)bi;
  }
}

// dx[n,h,w,c] = sum of dy over the (at most four) windows whose recorded winner is (h,w).
template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const T* __restrict__ dy,
                                                          const unsigned char* __restrict__ idx,
                                                          T* __restrict__ dx, int N, int H, int W, int C, int Ho,
                                                          int Wo) {
  const size_t total = (size_t)N * H * W * C;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int c = (int)(i % C);
    size_t r = i / C;
    const int w = (int)(r % W); r /= W;
    const int h = (int)(r % H);
    const int n = (int)(r / H);
    float acc = 0.f;
    // windows ho with ho*2 - 1 <= h <= ho*2 + 1
    for (int ho = (h) / 2; ho <= (h + 1) / 2; ++ho) {
      if (ho < 0 || ho >= Ho) continue;
      const int di = h - (ho * 2 - 1);
      if (di < 0 || di > 2) continue;
      for (int wo = (w) / 2; wo <= (w + 1) / 2; ++wo) {
        if (wo < 0 || wo >= Wo) continue;
        const int dj = w - (wo * 2 - 1);
        if (dj < 0 || dj > 2) continue;
        const size_t o = (((size_t)n * Ho + ho) * Wo + wo) * C + c;
        if (idx[o] == di * 3 + dj) acc += to_f32(dy[o]);
      }
    }
    dx[i] = from_f32<T>(acc);
  }
}

// bf16, C % 8 == 0: a thread owns eight channels of one pixel (16-byte accesses, no 64-bit divisions).
__global__ __launch_bounds__(256) void maxpool_fwd_bf16x8_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y,
                                                                 unsigned char* __restrict__ idx, int N, int H, int W,
                                                                 int C8, int Ho, int Wo) {
  const unsigned total = (unsigned)N * Ho * Wo * C8;
  for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
    const unsigned c8 = i % C8;
    unsigned r = i / C8;
    const int wo = (int)(r % Wo); r /= Wo;
    const int ho = (int)(r % Ho);
    const int n = (int)(r / Ho);
    float best[8];
    int bi[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { best[e] = -INFINITY; bi[e] = 0; }
#pragma unroll
    for (int di = 0; di < 3; ++di) {
      const int h = ho * 2 + di - 1;
      if (h < 0 || h >= H) continue;
#pragma unroll
      for (int dj = 0; dj < 3; ++dj) {
        const int w = wo * 2 + dj - 1;
        if (w < 0 || w >= W) continue;
        const uint4 v = *reinterpret_cast<const uint4*>(x + ((((size_t)n * H + h) * W + w) * C8 + c8) * 8);
        const float f[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                            bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (f[e] > best[e]) { best[e] = f[e]; bi[e] = di * 3 + dj; }
      }
    }
    // the maximum is one of the inputs: packing it back to bf16 is exact
    *reinterpret_cast<uint4*>(y + (size_t)i * 8) =
        make_uint4(pack_bf16x2(best[0], best[1]), pack_bf16x2(best[2], best[3]), pack_bf16x2(best[4], best[5]),
                   pack_bf16x2(best[6], best[7]));
    *reinterpret_cast<uint2*>(idx + (size_t)i * 8) =
        make_uint2((unsigned)bi[0] | (unsigned)bi[1] << 8 | (unsigned)bi[2] << 16 | (unsigned)bi[3] << 24,
                   (unsigned)bi[4] | (unsigned)bi[5] << 8 | (unsigned)bi[6] << 16 | (unsigned)bi[7] << 24);
  }
}

__global__ __launch_bounds__(256) void maxpool_bwd_bf16x8_kernel(const bf16_t* __restrict__ dy,
                                                                 const unsigned char* __restrict__ idx,
                                                                 bf16_t* __restrict__ dx, int N, int H, int W, int C8,
                                                                 int Ho, int Wo) {
  const unsigned total = (unsigned)N * H * W * C8;
  for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
    const unsigned c8 = i % C8;
    unsigned r = i / C8;
    const int w = (int)(r % W); r /= W;
    const int h = (int)(r % H);
    const int n = (int)(r / H);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // windows ho with ho*2 - 1 <= h <= ho*2 + 1
    for (int ho = h / 2; ho <= (h + 1) / 2; ++ho) {
      if (ho >= Ho) continue;
      const int di = h - (ho * 2 - 1);
      for (int wo = w / 2; wo <= (w + 1) / 2; ++wo) {
        if (wo >= Wo) continue;
        const unsigned code = (unsigned)(di * 3 + (w - (wo * 2 - 1)));
        const size_t o = ((((size_t)n * Ho + ho) * Wo + wo) * C8 + c8) * 8;
        const uint2 k = *reinterpret_cast<const uint2*>(idx + o);
        const uint4 v = *reinterpret_cast<const uint4*>(dy + o);
        const float f[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                            bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const unsigned ke = ((e < 4 ? k.x : k.y) >> (8 * (e & 3))) & 0xffu;
          if (ke == code) acc[e] += f[e];
        }
      }
    }
    *reinterpret_cast<uint4*>(dx + (size_t)i * 8) =
        make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]), pack_bf16x2(acc[4], acc[5]),
                   pack_bf16x2(acc[6], acc[7]));
  }
}

int blocks_for(size_t work) {
  const size_t b = (work + 255) / 256;
  return (int)(b < 8192 ? (b ? b : 1) : 8192);
}

}  // namespace

hipError_t launch_eltwise(int op, int dtype, void* a, const void* b, const void* c, size_t n, hipStream_t st) {
#define EL(T, OP) hipLaunchKernelGGL((eltwise_kernel<T, OP>), dim3(blocks_for(n / Vec<T>::N)), dim3(256), 0, st, (T*)a, (const T*)b, (const T*)c, n)
  if (dtype == CONVBN_BF16) {
    if (op == OP_RELU) EL(bf16_t, OP_RELU); else if (op == OP_RELU_BWD) EL(bf16_t, OP_RELU_BWD);
    else if (op == OP_ADD_RELU) EL(bf16_t, OP_ADD_RELU); else if (op == OP_ADD_RELU_BWD) EL(bf16_t, OP_ADD_RELU_BWD); else EL(bf16_t, OP_ADD);
  } else {
    if (op == OP_RELU) EL(float, OP_RELU); else if (op == OP_RELU_BWD) EL(float, OP_RELU_BWD);
    else if (op == OP_ADD_RELU) EL(float, OP_ADD_RELU); else if (op == OP_ADD_RELU_BWD) EL(float, OP_ADD_RELU_BWD); else EL(float, OP_ADD);
  }
#undef EL
  return hipGetLastError();
}

hipError_t launch_maxpool_fwd(int dtype, const void* x, void* y, unsigned char* idx, int N, int H, int W, int C,
                              hipStream_t st) {
  const int Ho = (H + 2 - 3) / 2 + 1, Wo = (W + 2 - 3) / 2 + 1;
  const size_t total = (size_t)N * Ho * Wo * C;
  if (dtype == CONVBN_BF16 && C % 8 == 0 && total / 8 < 0xffffffffull && (size_t)N * H * W * C / 8 < 0xffffffffull)
    hipLaunchKernelGGL(maxpool_fwd_bf16x8_kernel, dim3(blocks_for(total / 8)), dim3(256), 0, st, (const bf16_t*)x,
                       (bf16_t*)y, idx, N, H, W, C / 8, Ho, Wo);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(maxpool_fwd_kernel<bf16_t>, dim3(blocks_for(total)), dim3(256), 0, st, (const bf16_t*)x,
                       (bf16_t*)y, idx, N, H, W, C, Ho, Wo);
  else
    hipLaunchKernelGGL(maxpool_fwd_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, st, (const float*)x,
                       (float*)y, idx, N, H, W, C, Ho, Wo);
  return hipGetLastError();
}

hipError_t launch_maxpool_bwd(int dtype, const void* dy, const unsigned char* idx, void* dx, int N, int H, int W,
                              int C, hipStream_t st) {
  const int Ho = (H + 2 - 3) / 2 + 1, Wo = (W + 2 - 3) / 2 + 1;
  const size_t total = (size_t)N * H * W * C;
  if (dtype == CONVBN_BF16 && C % 8 == 0 && total / 8 < 0xffffffffull)
    hipLaunchKernelGGL(maxpool_bwd_bf16x8_kernel, dim3(blocks_for(total / 8)), dim3(256), 0, st, (const bf16_t*)dy,
                       idx, (bf16_t*)dx, N, H, W, C / 8, Ho, Wo);
  else if (dtype == CONVBN_BF16)
    hipLaunchKernelGGL(maxpool_bwd_kernel<bf16_t>, dim3(blocks_for(total)), dim3(256), 0, st, (const bf16_t*)dy,
                       idx, (bf16_t*)dx, N, H, W, C, Ho, Wo);
  else
    hipLaunchKernelGGL(maxpool_bwd_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, st, (const float*)dy, idx,
                       (float*)dx, N, H, W, C, Ho, Wo);
  return hipGetLastError();
}

}  // namespace convbn
