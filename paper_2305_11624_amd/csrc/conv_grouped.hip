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

// ---- bf16, group widths that are multiples of 8 (24, 48, 64 ...: whatever the matrix-core kernels below do not
// take): vector kernels.  A thread owns one pixel and 8 consecutive output channels (forward) resp. input channels
// (input gradient) of one group; the lanes of a wave are 64 consecutive pixels, so the weight rows they need are the
// same for the whole wave (uniform 16-byte loads) and every 16-byte load of the pixel's own channels feeds 64
// multiply-adds.  (One thread per output element, as in the any-shape kernels above, makes every lane of a wave
// fetch a different weight row: 5.5 ms instead of 0.1 for 2048 channels in 32 groups at 7 x 7.)
struct GvParams {
  const bf16_t* in;     // forward: x; input gradient: dz.  [N][Hi][Wi][Ci]
  const bf16_t* w;      // forward: [Cout][taps][cg]; input gradient: [cg][taps][Cout]
  const float* bias;    // forward only, or null
  bf16_t* out;          // [N][Ho][Wo][Co]
  int N, Hi, Wi, Ci, Ho, Wo, Co, kH, kW, sh, sw, ph, pw;
  int gin, gout;        // channels per group in `in` and in `out`
  int dgrad;            // 0: out pixel (ho, wo) reads in pixel (ho sh + i - ph, ..); 1: out pixel (h, w) reads
                        // in pixel ((h + ph - i) / sh, ..) where the division is exact
  int M;                // N Ho Wo
};

__device__ __forceinline__ void gv_unpack(const uint4& v, float (&f)[8]) {
  f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
  f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

typedef __bf16 gv_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float gv_dot2(unsigned a, unsigned b, float c) {   // c + a.lo b.lo + a.hi b.hi
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gv_bf16x2, a), __builtin_bit_cast(gv_bf16x2, b), c, false);
}

__global__ __launch_bounds__(256) void g_vec_conv_kernel(GvParams p) {
  const int m = blockIdx.x * 256 + threadIdx.x;          // output pixel
  const int oc0 = blockIdx.y * 8;                         // first of the thread's 8 output channels
  const int grp = oc0 / p.gout;
  const int taps = p.kH * p.kW;
  const bool live = m < p.M;
  const int mm = live ? m : 0;
  const int wo = mm % p.Wo;
  const int t1 = mm / p.Wo;
  const int ho = t1 % p.Ho, n = t1 / p.Ho;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = (p.bias && !p.dgrad) ? p.bias[oc0 + e] : 0.f;
  // weight row of output channel oc0 + e at window position t, columns 8 c8 .. 8 c8 + 7 of the group:
  //   forward         w[((oc0 + e) taps + t) gin + 8 c8]
  //   input gradient  w[(((oc0 + e) % gout) taps + t) Ci + grp gin + 8 c8]       (Ci = the block's Cout)
  const size_t wrow = p.dgrad ? (size_t)(oc0 % p.gout) * taps * p.Ci + (size_t)grp * p.gin : (size_t)oc0 * taps * p.gin;
  const size_t wstep_e = p.dgrad ? (size_t)taps * p.Ci : (size_t)taps * p.gin;   // from one output channel to the next
  const size_t wstep_t = p.dgrad ? (size_t)p.Ci : (size_t)p.gin;                 // from one window position to the next
  for (int i = 0; i < p.kH; ++i)
    for (int j = 0; j < p.kW; ++j) {
      int h, w;
      bool ok = live;
      if (!p.dgrad) {
        h = ho * p.sh + i - p.ph; w = wo * p.sw + j - p.pw;
      } else {
        const int hz = ho + p.ph - i, wz = wo + p.pw - j;
        ok = ok && hz >= 0 && wz >= 0 && hz % p.sh == 0 && wz % p.sw == 0;
        h = hz / p.sh; w = wz / p.sw;
      }
      ok = ok && (unsigned)h < (unsigned)p.Hi && (unsigned)w < (unsigned)p.Wi;
      const bf16_t* ip = p.in + (ok ? (((size_t)n * p.Hi + h) * p.Wi + w) * p.Ci + (size_t)grp * p.gin : 0);
      const bf16_t* wp = p.w + wrow + (size_t)(i * p.kW + j) * wstep_t;
      for (int c8 = 0; c8 < p.gin; c8 += 8) {
        uint4 xr = *reinterpret_cast<const uint4*>(ip + c8);
        if (!ok) xr = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          // 8 products per output channel as four packed bf16 dot products accumulated in fp32 (v_dot2c_f32_bf16)
          const uint4 wr = *reinterpret_cast<const uint4*>(wp + e * wstep_e + c8);
          acc[e] = gv_dot2(xr.x, wr.x, acc[e]);
          acc[e] = gv_dot2(xr.y, wr.y, acc[e]);
          acc[e] = gv_dot2(xr.z, wr.z, acc[e]);
          acc[e] = gv_dot2(xr.w, wr.w, acc[e]);
        }
      }
    }
  if (live)
    *reinterpret_cast<uint4*>(p.out + (size_t)m * p.Co + oc0) =
        make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]), pack_bf16x2(acc[4], acc[5]),
                   pack_bf16x2(acc[6], acc[7]));
}

bool gv_supported(const Geom& g, int groups, int dtype) {
  const int cg = g.Cin / groups, og = g.Cout / groups;
  return dtype == CONVBN_BF16 && cg % 8 == 0 && og % 8 == 0;
}
hipError_t gv_launch(const Geom& g, int groups, bool dgrad, const void* in, const void* w, const float* bias, void* out,
                     hipStream_t st) {
  GvParams p{};
  p.in = (const bf16_t*)in; p.w = (const bf16_t*)w; p.bias = bias; p.out = (bf16_t*)out;
  p.N = g.N; p.kH = g.kH; p.kW = g.kW; p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.dgrad = dgrad;
  if (!dgrad) {
    p.Hi = g.Hin; p.Wi = g.Win; p.Ci = g.Cin; p.Ho = g.Hout; p.Wo = g.Wout; p.Co = g.Cout;
    p.gin = g.Cin / groups; p.gout = g.Cout / groups; p.M = g.M;
  } else {
    p.Hi = g.Hout; p.Wi = g.Wout; p.Ci = g.Cout; p.Ho = g.Hin; p.Wo = g.Win; p.Co = g.Cin;
    p.gin = g.Cout / groups; p.gout = g.Cin / groups; p.M = g.Min;
  }
  hipLaunchKernelGGL(g_vec_conv_kernel, dim3(ceil_div(p.M, 256), p.Co / 8), dim3(256), 0, st, p);
  return hipGetLastError();
}

// Weight gradient of the same shapes: a thread owns 8 consecutive input channels q of one (output channel, window
// position) and walks the output rows of its slice (blockIdx.y) with the loops over rows and columns written out, so
// that a pixel costs one 2-byte load of dZ, one 16-byte load of x and 8 multiply-adds, not a chain of divisions.
// part[slice][Cout][taps][cg].
__global__ __launch_bounds__(256) void g_vec_wgrad_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dz,
                                                          float* __restrict__ part, Geom g, int cg, int og,
                                                          int rows_per_slice) {
  const int taps = g.kH * g.kW, q8s = cg / 8;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= g.Cout * taps * q8s) return;
  const int q8 = t % q8s;
  const int t2 = t / q8s;
  const int tap = t2 % taps, o = t2 / taps;
  const int i = tap / g.kW, j = tap - i * g.kW;
  const int c0 = (o / og) * cg + 8 * q8;
  const int rows = g.N * g.Hout;
  const int r0 = blockIdx.y * rows_per_slice, r1 = min(rows, r0 + rows_per_slice);
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int r = r0; r < r1; ++r) {
    const int n = r / g.Hout, ho = r - n * g.Hout;
    const int h = ho * g.sh + i - g.ph;
    if ((unsigned)h >= (unsigned)g.Hin) continue;
    const bf16_t* zp = dz + (size_t)r * g.Wout * g.Cout + o;
    const bf16_t* xp = x + ((size_t)n * g.Hin + h) * g.Win * g.Cin + c0;
    for (int wo = 0; wo < g.Wout; ++wo) {
      const int w = wo * g.sw + j - g.pw;
      if ((unsigned)w >= (unsigned)g.Win) continue;
      const float zv = to_f32(zp[(size_t)wo * g.Cout]);
      float xv[8];
      gv_unpack(*reinterpret_cast<const uint4*>(xp + (size_t)w * g.Cin), xv);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(zv, xv[e], acc[e]);
    }
  }
  float* op = part + ((size_t)blockIdx.y * g.Cout + o) * taps * cg + (size_t)tap * cg + 8 * q8;
  *reinterpret_cast<float4*>(op) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  *reinterpret_cast<float4*>(op + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
}
// The same for the usual small windows (KH x KW known at compile time): a thread owns 8 input channels of one output
// channel for ALL window positions, so a pixel's dZ value and the loop bookkeeping are paid once for KH KW
// 16-byte loads of x and 8 KH KW multiply-adds.
template <int KH, int KW>
__global__ __launch_bounds__(256) void g_vec_wgrad_win_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ dz,
                                                              float* __restrict__ part, Geom g, int cg, int og,
                                                              int rows_per_slice) {
  const int q8s = cg / 8;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= g.Cout * q8s) return;
  const int q8 = t % q8s, o = t / q8s;
  const int c0 = (o / og) * cg + 8 * q8;
  const int rows = g.N * g.Hout;
  const int r0 = blockIdx.y * rows_per_slice, r1 = min(rows, r0 + rows_per_slice);
  float acc[KH * KW][8];
#pragma unroll
  for (int a = 0; a < KH * KW; ++a)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[a][e] = 0.f;
  for (int r = r0; r < r1; ++r) {
    const int n = r / g.Hout, ho = r - n * g.Hout;
    const bf16_t* zp = dz + (size_t)r * g.Wout * g.Cout + o;
    const bf16_t* xn = x + (size_t)n * g.Hin * g.Win * g.Cin + c0;
    for (int wo = 0; wo < g.Wout; ++wo) {
      const float zv = to_f32(zp[(size_t)wo * g.Cout]);
#pragma unroll
      for (int i = 0; i < KH; ++i) {
        const int h = ho * g.sh + i - g.ph;
#pragma unroll
        for (int j = 0; j < KW; ++j) {
          const int w = wo * g.sw + j - g.pw;
          const bool ok = (unsigned)h < (unsigned)g.Hin && (unsigned)w < (unsigned)g.Win;
          const uint4 raw = *reinterpret_cast<const uint4*>(xn + (ok ? ((size_t)h * g.Win + w) * g.Cin : 0));
          float xv[8];
          gv_unpack(ok ? raw : make_uint4(0u, 0u, 0u, 0u), xv);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[i * KW + j][e] = fmaf(zv, xv[e], acc[i * KW + j][e]);
        }
      }
    }
  }
  float* op = part + ((size_t)blockIdx.y * g.Cout + o) * (KH * KW) * cg + 8 * q8;
#pragma unroll
  for (int a = 0; a < KH * KW; ++a) {
    *reinterpret_cast<float4*>(op + (size_t)a * cg) = make_float4(acc[a][0], acc[a][1], acc[a][2], acc[a][3]);
    *reinterpret_cast<float4*>(op + (size_t)a * cg + 4) = make_float4(acc[a][4], acc[a][5], acc[a][6], acc[a][7]);
  }
}
bool gv_wgrad_win(const Geom& g) { return (g.kH == 3 && g.kW == 3) || (g.kH == 1 && g.kW == 1); }
int gv_wgrad_slices(const Geom& g, int groups) {
  const int cg = g.Cin / groups;
  const int wgs = ceil_div(g.Cout * (gv_wgrad_win(g) ? 1 : g.kH * g.kW) * (cg / 8), 256);
  int want = ceil_div(1024, wgs);              // about four workgroups per CU
  // every slice is a full fp32 copy of dw' that the fold-back has to read: at most 96 MB of them, at most 128 (few
  // slices starve the kernel of threads: 3 instead of 16 on 2048 channels at 7 x 7 took 424 instead of 142 us)
  const size_t slice = (size_t)g.Cout * g.kH * g.kW * cg * 4;
  const int cap = (int)((size_t)(96 << 20) / slice) < 128 ? (int)((size_t)(96 << 20) / slice) : 128;
  if (want > cap) want = cap;
  const int rows = g.N * g.Hout;
  if (want > rows) want = rows;
  if (want < 1) want = 1;
  return ceil_div(rows, ceil_div(rows, want));
}

// ---- bf16 MFMA kernels for groups of 4, 8, 16, 32 or 64 channels (cg == og) ---------------------------------
// 32 consecutive channels hold whole groups, so the block is a stack of independent 32 -> 32 channel convolutions
// whose weight is block-diagonal (32 / cg blocks of cg x cg per tap).  One MFMA 32x32x16 takes 32 output channels
// x 32 pixels x 16 input channels of one tap: two per tap and wave.  The products outside the diagonal blocks
// multiply zeros -- with 4 channels per group 7/8 of the matrix work -- which is what keeps the layer on the
// matrix cores at all: the useful work of such a layer (72 FLOP per output element) is too little to hide, and
// the kernel is bound by fetching x, not by the multiplies.
//   * The weight fragments never change for a workgroup's channels: every lane loads its 2 kH kW fragments (the
//     zeros included) from w' once and keeps them in registers.
//   * The pixel operand is read straight from the input patch in LDS (lane = pixel, 16 contiguous bytes = 8
//     channels), tap after tap: no im2col.  A workgroup walks 2-d tiles (TR rows x TC columns of output pixels of
//     one image) for NCH chunks of 32 channels; wave w owns chunk w % NCH and every (4 / NCH)-th group of 32 pixels.
//   * The input gradient of a stride-1 block is the same kernel on dZ with the taps reversed and the weight read
//     in its other order; that of a strided block runs the residue classes of input positions side by side
//     (blockIdx.y), each with the taps that class has and a strided store.
// n / d for 0 <= n < 65536 and 1 <= d < 65536 with m = 2^32 / d + 1 (exact: the error n (m d - 2^32) stays below 2^32)
__device__ __forceinline__ int g_div(int n, unsigned m, int d) { return d == 1 ? n : (int)__umulhi((unsigned)n, m); }
inline unsigned g_magic(int d) { return (unsigned)((1ull << 32) / (unsigned)d + 1); }
// Workgroups that share cache lines and halo rows -- the chunk groups of one tile, the tiles of neighbouring
// workers -- get consecutive logical numbers, and consecutive logical numbers run on the same XCD (the hardware
// deals consecutive workgroup ids round-robin over the 8 XCDs, each with an L2 of its own).
__device__ __forceinline__ int g_logical_block() {
  const int per = gridDim.x >> 3;
  return (gridDim.x & 7) ? (int)blockIdx.x : (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
}

// Small tiles on purpose: a workgroup's phases (fetch, LDS, multiply, store) run one after the other, and what hides
// them is the other workgroup on the same CU and the next tile's fetch -- a workgroup should walk several tiles, and
// the fetch registers stay few.
constexpr int GC_PPT = 6;                  // most 16-byte patch items a thread fetches per tile (16: 1.7x slower, 8: 5 % slower)
constexpr size_t GC_PATCH_MAX = 24 * 1024; // patch bytes (+ 10 KB of output staging)

struct GcParams {
  const bf16_t* in;     // [N][Hi][Wi][C]
  const bf16_t* w;      // mode 0: [C][taps][cg]; mode 1: [cg][taps][C]
  const float* bias;    // [C] or null
  bf16_t* out;          // [N][Ho][Wo][C]
  int N, Hi, Wi, C, Ho, Wo, kH, kW, sh, sw, ph, pw, cg;
  int mode;             // 0 forward, 1 input gradient (taps reversed, ph / pw already those of the reversed window)
  int nch;              // chunks of 32 channels per workgroup (1, 2, 4)
  int TR, TC, ntr, ntc, ntiles;
  int PR, PC, pitch;    // patch rows, columns, bytes per patch pixel (64 nch + 16)
  int nwt;              // groups of 32 pixels per tile
  int ncg, nworkers;    // channel-chunk groups (C / 32 / nch); workgroups per chunk group
  int lcg, lgpp;        // log2 of cg and of the 16-byte granules per patch pixel (4 nch)
  unsigned mTC, mPC;    // g_div multipliers of TC and PC
  int wtaps;            // window positions of the weight tensor; position t of this launch reads its tap tapw[t]
  int tapw[9];          // (forward: t; stride-1 input gradient: reversed), -1: no tap (zeros)
  int OH, OW;           // the output tensor's rows and columns; pixel (r, c) of this launch is its pixel
  int osh, osw, ooh, oow;   // (r osh + ooh, c osw + oow)
  // A strided input gradient runs its residue classes of input positions as blockIdx.y = 0 .. ncls - 1 of one launch:
  // class q has its own padding, extent, output offset and taps (the fields above hold class 0 / the common values).
  int ncls;
  int cph[4], cpw[4], cHo[4], cWo[4], cooh[4], coow[4];
  int ctapw[4][9];
};

// KS: MFMA steps of 16 reduced channels per window position -- 2: the chunk's own 32 channels (groups of 4-32); 4: a
// group of 64 channels = the two chunks of the workgroup (nch = 2), every output chunk reading all 64, nothing masked
template <int TAPS, int KS>
__global__ __launch_bounds__(256) void g_conv_mfma_kernel(GcParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = lane >> 5, px = lane & 31;
  const int lb = g_logical_block();
  const int cgrp = lb % p.ncg, worker = lb / p.ncg;
  const int cls = blockIdx.y;                        // residue class (0 unless a strided input gradient)
  const int ph = p.ncls > 1 ? p.cph[cls] : p.ph, pw = p.ncls > 1 ? p.cpw[cls] : p.pw;
  const int Ho = p.ncls > 1 ? p.cHo[cls] : p.Ho, Wo = p.ncls > 1 ? p.cWo[cls] : p.Wo;
  const int ooh = p.ncls > 1 ? p.cooh[cls] : p.ooh, oow = p.ncls > 1 ? p.coow[cls] : p.oow;
  const int cl = wave % p.nch;                      // this wave's chunk inside the workgroup's channels
  const int chunk = cgrp * p.nch + cl;              // ... and in the tensor
  const int wstep = 4 / p.nch, wfirst = wave / p.nch;
  unsigned char* patch = smem;
  unsigned char* stage = smem + (size_t)p.PR * p.PC * p.pitch + wave * (32 * 80);   // [32 pixels][64 + 16 bytes]

  // ---- patch items of this thread (the same for every tile): 16-byte granule gq of patch pixel (row pr, column pc)
  const int gpp = p.nch * 4;                        // granules per patch pixel
  const int nitems = p.PR * p.PC * gpp;
  int ipr[GC_PPT], ipc[GC_PPT];
#pragma unroll
  for (int k = 0; k < GC_PPT; ++k) {
    const int e = tid + 256 * k;
    const int pix = e >> p.lgpp;
    ipr[k] = g_div(pix, p.mPC, p.PC);
    ipc[k] = (pix - ipr[k] * p.PC) | ((e & (gpp - 1)) << 16);
  }
  uint4 pv[GC_PPT];
  auto fetch = [&](int tile) {
    const int tc = tile % p.ntc;
    const int t2 = tile / p.ntc;
    const int tr = t2 % p.ntr, n = t2 / p.ntr;
    const int h0 = tr * p.TR * p.sh - ph, w0 = tc * p.TC * p.sw - pw;
#pragma unroll
    for (int k = 0; k < GC_PPT; ++k) {
      const int h = h0 + ipr[k], w = w0 + (ipc[k] & 0xffff), gq = ipc[k] >> 16;
      // branch-free: an item outside the image (or past the last tile) loads the tensor's first bytes and drops them
      const bool ok = tid + 256 * k < nitems && tile < p.ntiles && (unsigned)h < (unsigned)p.Hi && (unsigned)w < (unsigned)p.Wi;
      const size_t off = ok ? (((size_t)n * p.Hi + h) * p.Wi + w) * p.C + cgrp * p.nch * 32 + gq * 8 : 0;
      const uint4 v = *reinterpret_cast<const uint4*>(p.in + off);
      pv[k] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int k = 0; k < GC_PPT; ++k)
      if (tid + 256 * k < nitems)
        *reinterpret_cast<uint4*>(patch + (ipr[k] * p.PC + (ipc[k] & 0xffff)) * p.pitch + (ipc[k] >> 16) * 16) = pv[k];
  };

  fetch(worker);   // in flight while the weights arrive

  // ---- weight fragments: row = lane % 32 (output channel; mode 1: input channel), 8 consecutive reduced channels
  bf16x8 wf[TAPS][KS];
  {
    const int row = px, rgrp = row >> p.lcg;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int k0 = ks * 16 + kb * 8;             // first of the 8 reduced channels (local)
        const int tw = p.ncls > 1 ? p.ctapw[cls][t] : p.tapw[t];
        const int twc = tw < 0 ? 0 : tw;                 // (no tap: load tap 0 and drop it)
        const bool lo = tw >= 0 && (KS == 4 || (k0 >> p.lcg) == rgrp), hi = tw >= 0 && (KS == 4 || ((k0 + 4) >> p.lcg) == rgrp);
        // every address below is inside the weight whatever the masks say: load first, zero afterwards, so that
        // all loads of the lane are in flight together
        uint4 v;
        if (KS == 4) {   // groups of 64: rows and columns of the group's 64 x 64 block as they are
          v = p.mode == 0
                  ? *reinterpret_cast<const uint4*>(p.w + ((size_t)(chunk * 32 + row) * p.wtaps + twc) * 64 + k0)
                  : *reinterpret_cast<const uint4*>(p.w + ((size_t)(cl * 32 + row) * p.wtaps + twc) * p.C + cgrp * 64 + k0);
        } else if (p.mode == 0) {
          const bf16_t* wr = p.w + ((size_t)(chunk * 32 + row) * p.wtaps + twc) * p.cg;
          if (p.cg == 4) {
            const uint2 r = *reinterpret_cast<const uint2*>(wr);
            v = make_uint4(r.x, r.y, r.x, r.y);
          } else {
            v = *reinterpret_cast<const uint4*>(wr + (k0 & (p.cg - 1)));
          }
        } else {
          v = *reinterpret_cast<const uint4*>(p.w + ((size_t)(row & (p.cg - 1)) * p.wtaps + twc) * p.C + chunk * 32 + k0);
        }
        v.x = lo ? v.x : 0u; v.y = lo ? v.y : 0u;
        v.z = hi ? v.z : 0u; v.w = hi ? v.w : 0u;
        wf[t][ks] = __builtin_bit_cast(bf16x8, v);
      }
  }
  // bias of the lane's 16 accumulator channels 8 (e / 4) + 4 kb + e % 4
  float bv[16];
#pragma unroll
  for (int e = 0; e < 16; ++e)
    bv[e] = p.bias ? p.bias[chunk * 32 + 8 * (e >> 2) + 4 * kb + (e & 3)] : 0.f;

  for (int tile = worker; tile < p.ntiles; tile += p.nworkers) {
    const int tc = tile % p.ntc;
    const int t2 = tile / p.ntc;
    const int tr = t2 % p.ntr, n = t2 / p.ntr;
    const int r0 = tr * p.TR, c0 = tc * p.TC;
    const int rows = min(p.TR, Ho - r0), cols = min(p.TC, Wo - c0);
    __syncthreads();   // every wave is done with the previous patch
    stash();
    fetch(tile + p.nworkers);
    __syncthreads();   // patch visible
    for (int wt = wfirst; wt < p.nwt; wt += wstep) {
      if (g_div(wt * 32, p.mTC, p.TC) >= rows) break;            // nothing but rows past the image in this and later groups
      const int pl = wt * 32 + px;
      int r = g_div(pl, p.mTC, p.TC), c = pl - r * p.TC;
      if (r >= rows || c >= cols) { r = 0; c = 0; }   // computed and dropped
      const unsigned char* b0 = patch + ((r * p.sh) * p.PC + c * p.sw) * p.pitch + (KS == 4 ? 0 : cl * 64) + kb * 16;
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = bv[e];
#pragma unroll
      for (int t = 0; t < TAPS; ++t) {
        const int i = t / p.kW, j = t - i * p.kW;
        const unsigned char* bp = b0 + (i * p.PC + j) * p.pitch;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 fb = *reinterpret_cast<const bf16x8*>(bp + ks * 32);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[t][ks], fb, acc, 0, 0, 0);
        }
      }
      // ---- the wave's 32 pixels x 32 channels through its own LDS block, so that a store is 16 bytes per lane
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<uint2*>(stage + px * 80 + q * 16 + kb * 8) =
            make_uint2(pack_bf16x2(acc[q * 4 + 0], acc[q * 4 + 1]), pack_bf16x2(acc[q * 4 + 2], acc[q * 4 + 3]));
#pragma unroll
      for (int pass = 0; pass < 2; ++pass) {
        const int sp = pass * 16 + (lane >> 2), gq = lane & 3;
        const uint4 v = *reinterpret_cast<const uint4*>(stage + sp * 80 + gq * 16);
        const int p2 = wt * 32 + sp;
        const int r2 = g_div(p2, p.mTC, p.TC), c2 = p2 - r2 * p.TC;
        if (r2 < rows && c2 < cols)
          *reinterpret_cast<uint4*>(p.out + (((size_t)n * p.OH + (r0 + r2) * p.osh + ooh) * p.OW + (c0 + c2) * p.osw + oow) * p.C +
                                    chunk * 32 + gq * 8) = v;
      }
    }
  }
}

struct GcPlan { bool ok; size_t lds; int grid; };
// in_h / in_w: the tensor the patch is cut from; out_h / out_w: the tensor written
GcPlan gc_plan(int N, int C, int cg, int in_h, int in_w, int out_h, int out_w, int kH, int kW, int sh, int sw, int ph,
               int pw, GcParams* pp) {
  GcPlan pl{false, 0, 0};
  GcParams& p = *pp;
  p = GcParams{};
  if (C % 32 != 0 || (cg != 4 && cg != 8 && cg != 16 && cg != 32 && cg != 64)) return pl;
  const int taps = kH * kW;
  if (taps != 1 && taps != 2 && taps != 3 && taps != 4 && taps != 6 && taps != 9) return pl;
  p.N = N; p.Hi = in_h; p.Wi = in_w; p.C = C; p.Ho = out_h; p.Wo = out_w; p.kH = kH; p.kW = kW;
  p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.cg = cg;
  p.wtaps = taps;
  for (int t = 0; t < taps; ++t) p.tapw[t] = t;
  p.OH = out_h; p.OW = out_w; p.osh = 1; p.osw = 1; p.ooh = 0; p.oow = 0;
  p.ncls = 1;
  const int nchunks = C / 32;
  double best = 0;
  for (int ntc = ceil_div(out_w, 64); ntc <= ceil_div(out_w, 64) + 3 && ntc <= out_w; ++ntc) {
    const int TC = ceil_div(out_w, ntc);
    if (ceil_div(out_w, TC) != ntc) continue;
    const int PC = (TC - 1) * sw + kW;
    for (int nch = 1; nch <= 4; nch *= 2) {
      if (cg == 64 && nch != 2) continue;               // a group of 64 is exactly the two chunks of a workgroup
      if (nchunks % nch != 0) continue;
      const int pitch = 64 * nch + 16;
      for (int TR = 1; TR <= out_h; ++TR) {
        const int PR = (TR - 1) * sh + kH;
        if ((size_t)PR * PC * pitch > GC_PATCH_MAX || PR * PC * nch * 4 > 256 * GC_PPT) break;
        const int ntr = ceil_div(out_h, TR);
        if (ceil_div(out_h, ntr) != TR) continue;         // an evenly split height only
        const int per_round = 4 / nch;
        auto rounds = [&](int rows) { return ceil_div(ceil_div(rows * TC, 32), per_round); };
        const int last = out_h - (ntr - 1) * TR;
        const double work = ((double)(ntr - 1) * rounds(TR) + rounds(last)) * ntc * (nchunks / nch);   // wave rounds per image
        const double fetched = ((double)ntr * PR * ntc * PC) / ((double)out_h * sh * out_w * sw);       // patch pixels / image pixels
        const double score = 1.0 / (work * (1.0 + 0.3 * (fetched - 1.0)));
        if (score >= best) {   // ties: more channels per workgroup (longer contiguous loads)
          best = score;
          p.nch = nch; p.TR = TR; p.ntr = ntr; p.PR = PR; p.pitch = pitch; p.ntc = ntc; p.TC = TC; p.PC = PC;
        }
      }
    }
  }
  if (best == 0) return pl;
  p.lcg = cg == 4 ? 2 : cg == 8 ? 3 : cg == 16 ? 4 : cg == 32 ? 5 : 6;
  p.lgpp = p.nch == 1 ? 2 : p.nch == 2 ? 3 : 4;
  p.mTC = g_magic(p.TC); p.mPC = g_magic(p.PC);
  p.nwt = ceil_div(p.TR * p.TC, 32);
  p.ntiles = N * p.ntr * p.ntc;
  p.ncg = nchunks / p.nch;
  pl.lds = (size_t)p.PR * p.PC * p.pitch + 4 * 32 * 80;
  // two persistent workgroups per CU, each walking several tiles (measured: 1 -> 39, 2 -> 35, 4 -> 41, 8 -> 48 us for
  // fold + forward on 128 channels at 56 x 56: more workgroups start and finish in step and leave a longer tail)
  const int per_cu = (int)(160 * 1024 / pl.lds) < 2 ? 1 : 2;
  int workers = ceil_div(256 * per_cu, p.ncg);
  if (workers > p.ntiles) workers = p.ntiles;
  p.nworkers = workers;
  pl.grid = workers * p.ncg;
  pl.ok = true;
  return pl;
}

GcPlan gc_fprop_plan(const Geom& g, int groups, int dtype, GcParams* p) {
  if (dtype != CONVBN_BF16 || g.Cin != g.Cout || g.sh > 2 || g.sw > 2) return GcPlan{false, 0, 0};
  return gc_plan(g.N, g.Cin, g.Cin / groups, g.Hin, g.Win, g.Hout, g.Wout, g.kH, g.kW, g.sh, g.sw, g.ph, g.pw, p);
}
// stride 1 only: dX is the forward kernel on dZ with the window reversed and padding k - 1 - p
GcPlan gc_dgrad_plan(const Geom& g, int groups, int dtype, GcParams* p) {
  if (dtype != CONVBN_BF16 || g.Cin != g.Cout || g.sh != 1 || g.sw != 1 || g.ph > g.kH - 1 || g.pw > g.kW - 1)
    return GcPlan{false, 0, 0};
  GcPlan pl = gc_plan(g.N, g.Cin, g.Cin / groups, g.Hout, g.Wout, g.Hin, g.Win, g.kH, g.kW, 1, 1, g.kH - 1 - g.ph,
                      g.kW - 1 - g.pw, p);
  if (!pl.ok) return pl;   // (also: tapw has room for the 9 positions a plan accepts, not for any window)
  p->mode = 1;
  for (int t = 0; t < g.kH * g.kW; ++t) p->tapw[t] = g.kH * g.kW - 1 - t;
  return pl;
}
// One dimension of a strided input gradient: the input positions h = s a + q (residue class q) read dZ positions
// a + d - t through window rows i0 + s t (those below k).  With T the largest number of taps of any class, every
// class is a stride-1 window of T positions over dZ with padding T - 1 - d, position i' reading window row
// i0 + s (T - 1 - i') -- or nothing, where that row does not exist.
struct GcClassDim { int i0, d, count; };
GcClassDim gc_class_dim(int q, int s, int pad, int in_size) {
  GcClassDim c;
  c.i0 = (q + pad) % s;
  c.d = (q + pad) / s;
  c.count = in_size > q ? (in_size - q + s - 1) / s : 0;
  return c;
}
int gc_class_taps(int s, int pad, int k) {   // most taps a class has
  int T = 1;
  for (int q = 0; q < s; ++q) {
    const int i0 = (q + pad) % s;
    if (i0 < k && (k - i0 + s - 1) / s > T) T = (k - i0 + s - 1) / s;
  }
  return T;
}
// dX of a strided block: the forward kernel on dZ, one residue class of input positions per blockIdx.y
GcPlan gc_dgrad_strided_plan(const Geom& g, int groups, int dtype, GcParams* p) {
  if (dtype != CONVBN_BF16 || g.Cin != g.Cout || (g.sh == 1 && g.sw == 1) || g.sh > 2 || g.sw > 2) return GcPlan{false, 0, 0};
  const int Th = gc_class_taps(g.sh, g.ph, g.kH), Tw = gc_class_taps(g.sw, g.pw, g.kW);
  GcPlan pl = gc_plan(g.N, g.Cin, g.Cin / groups, g.Hout, g.Wout, ceil_div(g.Hin, g.sh), ceil_div(g.Win, g.sw), Th, Tw, 1, 1,
                      0, 0, p);
  if (!pl.ok) return pl;
  p->mode = 1;
  p->wtaps = g.kH * g.kW;
  p->OH = g.Hin; p->OW = g.Win; p->osh = g.sh; p->osw = g.sw;
  p->ncls = g.sh * g.sw;
  for (int qh = 0; qh < g.sh; ++qh)
    for (int qw = 0; qw < g.sw; ++qw) {
      const int c = qh * g.sw + qw;
      const GcClassDim a = gc_class_dim(qh, g.sh, g.ph, g.Hin), b = gc_class_dim(qw, g.sw, g.pw, g.Win);
      p->cph[c] = Th - 1 - a.d; p->cpw[c] = Tw - 1 - b.d;
      p->cHo[c] = a.count; p->cWo[c] = b.count;
      p->cooh[c] = qh; p->coow[c] = qw;
      for (int i = 0; i < Th; ++i)
        for (int j = 0; j < Tw; ++j) {
          const int wi = a.i0 + g.sh * (Th - 1 - i), wj = b.i0 + g.sw * (Tw - 1 - j);
          p->ctapw[c][i * Tw + j] = (wi < g.kH && wj < g.kW) ? wi * g.kW + wj : -1;
        }
    }
  return pl;
}

hipError_t gc_launch(const GcPlan& pl, const GcParams& p, hipStream_t st) {
#define GCL(T)                                                                                                       \
  do {                                                                                                               \
    if (p.cg == 64) hipLaunchKernelGGL((g_conv_mfma_kernel<T, 4>), dim3(pl.grid, p.ncls), dim3(256), pl.lds, st, p);   \
    else hipLaunchKernelGGL((g_conv_mfma_kernel<T, 2>), dim3(pl.grid, p.ncls), dim3(256), pl.lds, st, p);              \
  } while (0)
  switch (p.kH * p.kW) {
    case 1: GCL(1); break;
    case 2: GCL(2); break;
    case 3: GCL(3); break;
    case 4: GCL(4); break;
    case 6: GCL(6); break;
    default: GCL(9); break;
  }
#undef GCL
  return hipGetLastError();
}

// ---- weight gradient on the same chunks -------------------------------------------------------------------
// dw'[o][tap][q] = sum over pixels of dZ[pixel][o] X[pixel (+) tap][group(o) cg + q] and r[o] = sum dZ (Sec. 3.2.1,
// App. B).  The reduced index is the pixel, so both MFMA operands come from LDS through the transposing load
// (ds_read_tr16_b64: a lane supplies the address of 4 channels of one pixel and receives 4 consecutive pixels of
// one channel): rows = the chunk's 32 input channels at the pixel's window position, columns = its 32 output
// channels, 16 pixels per step, one accumulator tile per tap.  Only the diagonal cg x cg blocks of the 32 x 32
// result are wanted; the rest is computed and dropped.  The waves that share a chunk divide its taps among them
// (every wave walks all pixels of a tile for its own taps, so no sums cross waves); a workgroup keeps its sums in
// registers over all its tiles and writes one fp32 slice of dw' (and of r) at the end.
typedef short gs16x4 __attribute__((ext_vector_type(4)));
typedef short gs16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ gs16x4 g_read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) gs16x4*)(p));
}
__device__ __forceinline__ bf16x8 g_join(gs16x4 a, gs16x4 b) {
  gs16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}

constexpr int GW_PPT = 6;    // most 16-byte patch items a thread fetches per tile
constexpr int GW_ZPT = 4;    // ... and dZ items

struct GwParams {
  const bf16_t* x;      // [N][Hi][Wi][C]
  const bf16_t* dz;     // [N][Ho][Wo][C]
  float* part;          // [nworkers][C][taps cg]
  float* r_part;        // [nworkers][C] or null
  int N, Hi, Wi, C, Ho, Wo, kH, kW, sh, sw, ph, pw, cg;
  int nch, TR, TC, ntr, ntc, ntiles, PR, PC, pitch;
  int npx, nk;          // pixels per tile, 16-pixel steps per tile
  int ncg, nworkers;
  int lcg, lgpp;
  unsigned mTC, mPC;
};

// RB: 32-channel row blocks of the input side per output chunk -- 1: the chunk's own channels (groups of 4-32); 2: a
// group of 64 = both chunks of the workgroup (NCH = 2), all of the 64 x 32 result wanted
template <int TAPS, int NCH, int RB>
__global__ __launch_bounds__(256) void g_wgrad_mfma_kernel(GwParams p) {
  constexpr int NRED = 4 / NCH;                       // waves that share a chunk: they divide its taps among them
  constexpr int TPW = (TAPS + NRED - 1) / NRED;       // taps per wave: wave wq takes taps wq, wq + NRED, ...
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = lane >> 5;
  const int eprime = (lane & 15) >> 2;                           // pixel (of 4) this lane addresses in a transposing read
  const int quad = ((lane >> 4) & 1) * 4 + (lane & 3);           // its 4-channel quad inside the 32-channel chunk
  const int lb = g_logical_block();
  const int cgrp = lb % p.ncg, worker = lb / p.ncg;
  const int cl = wave % NCH, chunk = cgrp * NCH + cl;
  const int wq = wave / NCH;                                      // this wave's place among the waves of its chunk
  const int npx16 = p.nk * 16;
  unsigned char* patch = smem;                                                  // [PR][PC][pitch]
  unsigned char* zt = smem + (size_t)p.PR * p.PC * p.pitch;                     // [npx16][pitch]
  int* poff = reinterpret_cast<int*>(zt + (size_t)npx16 * p.pitch);             // [npx16] window origin of a tile pixel
  for (int e = tid; e < npx16; e += 256) {
    const int r = g_div(e, p.mTC, p.TC), c = e - r * p.TC;
    poff[e] = e < p.npx ? ((r * p.sh) * p.PC + c * p.sw) * p.pitch : 0;
  }

  const int gpp = p.nch * 4;
  const int nitems = p.PR * p.PC * gpp, nz = npx16 * gpp;
  int ipr[GW_PPT], ipc[GW_PPT], zr[GW_ZPT], zc[GW_ZPT];
#pragma unroll
  for (int k = 0; k < GW_PPT; ++k) {
    const int e = tid + 256 * k;
    const int pix = e >> p.lgpp;
    ipr[k] = g_div(pix, p.mPC, p.PC);
    ipc[k] = (pix - ipr[k] * p.PC) | ((e & (gpp - 1)) << 16);
  }
#pragma unroll
  for (int k = 0; k < GW_ZPT; ++k) {
    const int pix = (tid + 256 * k) >> p.lgpp;
    const int r = g_div(pix, p.mTC, p.TC);
    zr[k] = pix < p.npx ? r : (1 << 20);              // never a row of the tile
    zc[k] = pix - r * p.TC;
  }
  const int zgq = tid & (gpp - 1);                          // the granule (8 channels) of every dZ item of this thread
  uint4 pv[GW_PPT], zv[GW_ZPT];
  auto fetch = [&](int tile) {
    const int tc = tile % p.ntc;
    const int t2 = tile / p.ntc;
    const int tr = t2 % p.ntr, n = t2 / p.ntr;
    const int r0 = tr * p.TR, c0 = tc * p.TC;
    const int h0 = r0 * p.sh - p.ph, w0 = c0 * p.sw - p.pw;
#pragma unroll
    for (int k = 0; k < GW_PPT; ++k) {
      const int h = h0 + ipr[k], w = w0 + (ipc[k] & 0xffff), gq = ipc[k] >> 16;
      const bool ok = tid + 256 * k < nitems && tile < p.ntiles && (unsigned)h < (unsigned)p.Hi && (unsigned)w < (unsigned)p.Wi;
      const size_t off = ok ? (((size_t)n * p.Hi + h) * p.Wi + w) * p.C + cgrp * p.nch * 32 + gq * 8 : 0;
      const uint4 v = *reinterpret_cast<const uint4*>(p.x + off);
      pv[k] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
    }
#pragma unroll
    for (int k = 0; k < GW_ZPT; ++k) {
      const bool ok = tid + 256 * k < nz && tile < p.ntiles && r0 + zr[k] < p.Ho && zr[k] < p.TR && c0 + zc[k] < p.Wo;
      const size_t off = ok ? (((size_t)n * p.Ho + r0 + zr[k]) * p.Wo + c0 + zc[k]) * p.C + cgrp * p.nch * 32 + zgq * 8 : 0;
      const uint4 v = *reinterpret_cast<const uint4*>(p.dz + off);
      zv[k] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
    }
  };
  float racc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) racc[j] = 0.f;
  auto stash = [&]() {
#pragma unroll
    for (int k = 0; k < GW_PPT; ++k)
      if (tid + 256 * k < nitems)
        *reinterpret_cast<uint4*>(patch + (ipr[k] * p.PC + (ipc[k] & 0xffff)) * p.pitch + (ipc[k] >> 16) * 16) = pv[k];
#pragma unroll
    for (int k = 0; k < GW_ZPT; ++k)
      if (tid + 256 * k < nz) {
        *reinterpret_cast<uint4*>(zt + ((tid + 256 * k) >> p.lgpp) * p.pitch + zgq * 16) = zv[k];
        racc[0] += bf16_lo(zv[k].x); racc[1] += bf16_hi(zv[k].x); racc[2] += bf16_lo(zv[k].y); racc[3] += bf16_hi(zv[k].y);
        racc[4] += bf16_lo(zv[k].z); racc[5] += bf16_hi(zv[k].z); racc[6] += bf16_lo(zv[k].w); racc[7] += bf16_hi(zv[k].w);
      }
  };

  f32x16 acc[TPW][RB];
  int toff[TPW];                                      // patch offset of the wave's taps
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[u][rb][e] = 0.f;
    const int t = wq + NRED * u;
    const int i = t / p.kW, j = t - i * p.kW;
    toff[u] = (i * p.PC + j) * p.pitch;
  }

  fetch(worker);
  for (int tile = worker; tile < p.ntiles; tile += p.nworkers) {
    __syncthreads();   // the previous tile has been read
    stash();
    fetch(tile + p.nworkers);
    __syncthreads();   // patch, dZ tile (and, first pass, the offset table) visible
    for (int k = 0; k < p.nk; ++k) {
      const int pa = k * 16 + kb * 8 + eprime;        // the lane's pixel in the first transposing read; + 4 in the second
      const unsigned char* za = zt + pa * p.pitch + cl * 64 + quad * 8;
      const bf16x8 zf = g_join(g_read_tr(za), g_read_tr(za + 4 * p.pitch));
      const unsigned char* xa = patch + poff[pa] + (RB == 2 ? 0 : cl * 64) + quad * 8;
      const unsigned char* xb = patch + poff[pa + 4] + (RB == 2 ? 0 : cl * 64) + quad * 8;
#pragma unroll
      for (int u = 0; u < TPW; ++u) {
        if (NRED * (u + 1) <= TAPS || wq + NRED * u < TAPS) {   // (a compile-time yes except for the last of a wave's taps)
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            const bf16x8 xf = g_join(g_read_tr(xa + toff[u] + rb * 64), g_read_tr(xb + toff[u] + rb * 64));
            acc[u][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, zf, acc[u][rb], 0, 0, 0);
          }
        }
      }
    }
  }
  __syncthreads();     // every wave is done with the tiles: LDS is reused for the sums
  float* red = reinterpret_cast<float*>(smem);
  if (p.r_part) {
    // thread -> 8 channels (granule zgq) of every gpp-th item: sum the threads of a granule
#pragma unroll
    for (int j = 0; j < 8; ++j) red[tid * 8 + j] = racc[j];
    __syncthreads();
    if (tid < p.nch * 32) {
      const int gq = tid >> 3, j = tid & 7;
      float v = 0.f;
      for (int t = gq; t < 256; t += gpp) v += red[t * 8 + j];
      p.r_part[(size_t)worker * p.C + cgrp * p.nch * 32 + tid] = v;
    }
    __syncthreads();
  }
  // Accumulator element e of lane l: input channel 8 (e / 4) + 4 (l / 32) + e % 4 (local), output channel l % 32 (local).
  // A run of 4 input channels lies in one group; it is wanted when that is the output channel's group.
  const int co_l = lane & 31;
  const int K = TAPS * p.cg;
  float* orow = p.part + ((size_t)worker * p.C + chunk * 32 + co_l) * K;
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const int t = wq + NRED * u;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int ci0 = 8 * e4 + 4 * kb;
        if (t < TAPS && (RB == 2 || (ci0 >> p.lcg) == (co_l >> p.lcg)))
          *reinterpret_cast<float4*>(orow + t * p.cg + (RB == 2 ? rb * 32 + ci0 : (ci0 & (p.cg - 1)))) =
              make_float4(acc[u][rb][e4 * 4 + 0], acc[u][rb][e4 * 4 + 1], acc[u][rb][e4 * 4 + 2], acc[u][rb][e4 * 4 + 3]);
      }
  }
}

struct GwPlan { bool ok; size_t lds; int grid; };
GwPlan gw_plan(const Geom& g, int groups, int dtype, GwParams* pp) {
  GwPlan pl{false, 0, 0};
  GwParams& p = *pp;
  p = GwParams{};
  const int C = g.Cin, cg = g.Cin / groups, taps = g.kH * g.kW;
  if (dtype != CONVBN_BF16 || g.Cin != g.Cout || g.sh > 2 || g.sw > 2) return pl;
  if (C % 32 != 0 || (cg != 4 && cg != 8 && cg != 16 && cg != 32 && cg != 64) || (taps != 1 && taps != 9)) return pl;
  p.N = g.N; p.Hi = g.Hin; p.Wi = g.Win; p.C = C; p.Ho = g.Hout; p.Wo = g.Wout; p.kH = g.kH; p.kW = g.kW;
  p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.cg = cg;
  const int nchunks = C / 32;
  double best = 0;
  size_t best_lds = 0;
  for (int ntc = ceil_div(g.Wout, 64); ntc <= ceil_div(g.Wout, 64) + 3 && ntc <= g.Wout; ++ntc) {
    const int TC = ceil_div(g.Wout, ntc);
    if (ceil_div(g.Wout, TC) != ntc) continue;
    const int PC = (TC - 1) * g.sw + g.kW;
    // one or two chunks per workgroup: with four, a wave owns all nine taps of its chunk (144 accumulator registers)
    // and the tiles shrink to a handful of pixels -- measured slower on every layer (47 vs 30 us on 256 channels, stride 2)
    for (int nch = 1; nch <= 2; nch *= 2) {
      if (cg == 64 && nch != 2) continue;               // a group of 64 is exactly the two chunks of a workgroup
      if (nchunks % nch != 0) continue;
      const int pitch = 64 * nch + 16, nred = 4 / nch;
      for (int TR = 1; TR <= g.Hout; ++TR) {
        const int PR = (TR - 1) * g.sh + g.kH;
        const int nk = ceil_div(TR * TC, 16);
        size_t lds = (size_t)PR * PC * pitch + (size_t)nk * 16 * pitch + (size_t)nk * 16 * 4;
        if (lds > 36 * 1024 || PR * PC * nch * 4 > 256 * GW_PPT || nk * 16 * nch * 4 > 256 * GW_ZPT) break;
        if (lds < 8192) lds = 8192;                        // the channel sums of dZ meet in the first 8 KB
        if (lds > 64 * 1024) continue;
        const int ntr = ceil_div(g.Hout, TR);
        if (ceil_div(g.Hout, ntr) != TR) continue;
        const double work = (double)ntr * ntc * nk * ceil_div(taps, nred) * (nchunks / nch);   // MFMA steps of the busiest wave
        const double fetched = ((double)ntr * PR * ntc * PC) / ((double)g.Hout * g.sh * g.Wout * g.sw);
        const double score = 1.0 / (work * (1.0 + 0.3 * (fetched - 1.0)));
        if (score >= best) {   // ties: more channels per workgroup (longer contiguous loads)
          best = score; best_lds = lds;
          p.nch = nch; p.TR = TR; p.ntr = ntr; p.PR = PR; p.pitch = pitch; p.nk = nk; p.ntc = ntc; p.TC = TC; p.PC = PC;
        }
      }
    }
  }
  if (best == 0) return pl;
  p.lcg = cg == 4 ? 2 : cg == 8 ? 3 : cg == 16 ? 4 : cg == 32 ? 5 : 6;
  p.lgpp = p.nch == 1 ? 2 : p.nch == 2 ? 3 : 4;
  p.mTC = g_magic(p.TC); p.mPC = g_magic(p.PC);
  p.npx = p.TR * p.TC;
  p.ntiles = g.N * p.ntr * p.ntc;
  p.ncg = nchunks / p.nch;
  // one fp32 slice of dw' per worker: enough workers to fill the chip, not more slices than the fold-back reads cheaply
  const size_t slice = (size_t)C * taps * cg * 4;
  int workers = ceil_div(512, p.ncg);
  const int cap = (int)((size_t)(16 << 20) / slice);
  if (workers > cap) workers = cap;
  if (workers > p.ntiles) workers = p.ntiles;
  if (workers < 1) workers = 1;
  p.nworkers = workers;
  pl.lds = best_lds;
  pl.grid = workers * p.ncg;
  pl.ok = true;
  return pl;
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
  GcParams gp;
  const GcPlan pl = gc_fprop_plan(g, groups, dtype, &gp);
  if (pl.ok) {
    gp.in = (const bf16_t*)x; gp.w = (const bf16_t*)w_krsc; gp.bias = bias; gp.out = (bf16_t*)z;
    return gc_launch(pl, gp, st);
  }
  if (gv_supported(g, groups, dtype)) return gv_launch(g, groups, false, x, w_krsc, bias, z, st);
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
  GcParams gp;
  const GcPlan pl = gc_dgrad_plan(g, groups, dtype, &gp);
  if (pl.ok) {
    gp.in = (const bf16_t*)dz; gp.w = (const bf16_t*)w_crsk; gp.bias = nullptr; gp.out = (bf16_t*)dx;
    return gc_launch(pl, gp, st);
  }
  const GcPlan sp = gc_dgrad_strided_plan(g, groups, dtype, &gp);   // the residue classes of input positions in one launch
  if (sp.ok) {
    gp.in = (const bf16_t*)dz; gp.w = (const bf16_t*)w_crsk; gp.bias = nullptr; gp.out = (bf16_t*)dx;
    return gc_launch(sp, gp, st);
  }
  if (gv_supported(g, groups, dtype)) return gv_launch(g, groups, true, dz, w_crsk, nullptr, dx, st);
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
  GwParams gp;
  if (gw_plan(g, groups, dtype, &gp).ok) return gp.nworkers;
  if (gv_supported(g, groups, dtype)) return gv_wgrad_slices(g, groups);
  return direct_splits(g, g.Cin / groups);
}

bool g_wgrad_makes_rsum(const Geom& g, int groups, int dtype) {
  GwParams gp;
  return gw_plan(g, groups, dtype, &gp).ok;
}

hipError_t launch_g_wgrad(const Geom& g, int groups, int dtype, const void* x, const void* dz, float* part,
                          float* r_part, hipStream_t st) {
  const int cg = g.Cin / groups, og = g.Cout / groups;
  GwParams gp;
  const GwPlan pl = gw_plan(g, groups, dtype, &gp);
  if (pl.ok) {
    gp.x = (const bf16_t*)x; gp.dz = (const bf16_t*)dz; gp.part = part; gp.r_part = r_part;
#define GWL(T, NC, RBV) hipLaunchKernelGGL((g_wgrad_mfma_kernel<T, NC, RBV>), dim3(pl.grid), dim3(256), pl.lds, st, gp)
    if (gp.cg == 64) { if (g.kH * g.kW == 9) GWL(9, 2, 2); else GWL(1, 2, 2); }
    else if (g.kH * g.kW == 9) { if (gp.nch == 1) GWL(9, 1, 1); else GWL(9, 2, 1); }
    else { if (gp.nch == 1) GWL(1, 1, 1); else GWL(1, 2, 1); }
#undef GWL
    return hipGetLastError();
  }
  if (gv_supported(g, groups, dtype)) {
    const int ns = gv_wgrad_slices(g, groups);
    const int rps = ceil_div(g.N * g.Hout, ns);
    if (gv_wgrad_win(g)) {
      const dim3 wgrid(ceil_div(g.Cout * (cg / 8), 256), ns);
      if (g.kH == 3)
        hipLaunchKernelGGL((g_vec_wgrad_win_kernel<3, 3>), wgrid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part,
                           g, cg, og, rps);
      else
        hipLaunchKernelGGL((g_vec_wgrad_win_kernel<1, 1>), wgrid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part,
                           g, cg, og, rps);
      return hipGetLastError();
    }
    const dim3 vgrid(ceil_div(g.Cout * g.kH * g.kW * (cg / 8), 256), ns);
    hipLaunchKernelGGL(g_vec_wgrad_kernel, vgrid, dim3(256), 0, st, (const bf16_t*)x, (const bf16_t*)dz, part, g, cg, og,
                       rps);
    return hipGetLastError();
  }
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
