// bf16 implicit-GEMM convolution on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16,
// fp32 accumulation): forward conv, input gradient and weight gradient of Sec. 3.2.1,
// all three as  D[c][r] = sum_q  Rop[r][q] * Cop[c][q]  with
//
//   pass    r (contiguous in the output)   c                 q (reduced)        output
//   fprop   co                             m=(n,ho,wo)       (tap, ci)          Z[m][co]   (+ bias)
//   dgrad   ci                             m'=(n,h,w)        (tap, co)          dX[m'][ci]
//   wgrad   k=(tap,ci)                     co                m=(n,ho,wo)        dW'[co][k] fp32 partials
//
// Both operands are staged in LDS with the reduced index contiguous, 8 bf16 (16 B)
// per lane per MFMA operand.  fprop/dgrad read activations with the reduced index
// already contiguous in memory (channels-last); wgrad reduces over pixels, which are
// strided in memory, so its loaders transpose 8x8 blocks in registers on the way in.
#include "common.h"

namespace convbn {

namespace {

constexpr int BK = 64;        // reduced-index extent of one LDS stage
constexpr int LDK = BK + 8;   // padded LDS row (144 B): 16-lane b128 reads hit 64 distinct banks

struct IgemmParams {
  const bf16_t* act;   // fprop: x ; dgrad: dz ; wgrad: x
  const bf16_t* wgt;   // fprop: w' [Cout][K] ; dgrad: w'^T [Cin][taps*Cout] ; wgrad: dz
  const float* bias;   // per output row of fprop / dgrad (nullable)
  void* out;
  Geom g;
  int red_per_split;   // wgrad: pixels per blockIdx.y slice (multiple of BK)
};

__device__ __forceinline__ uint4 ldg16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

// ---- operand loaders -------------------------------------------------------------
// Reduced-index-contiguous loaders: thread -> 16-byte chunk (tid%8) of rows tid/8 + 32 p.

// Plain matrix rows [R][K] (the weight operand of fprop and dgrad).
template <int T>
struct PlainRows {
  static constexpr int NREG = T / 32;
  const bf16_t* base;
  int R, K, row0, kc;
  __device__ void init(const IgemmParams& p, int R_, int K_, int tile_row0) {
    base = p.wgt;
    R = R_;
    K = K_;
    kc = (threadIdx.x & 7) * 8;
    row0 = tile_row0 + (threadIdx.x >> 3);
  }
  __device__ void load(int k0, int, uint4 (&v)[NREG]) const {
    const int k = k0 + kc;
#pragma unroll
    for (int p = 0; p < NREG; ++p) {
      const int row = row0 + 32 * p;
      v[p] = (row < R && k < K) ? ldg16(base + (size_t)row * K + k) : zero16();
    }
  }
  __device__ void store(bf16_t* lds, const uint4 (&v)[NREG]) const {
#pragma unroll
    for (int p = 0; p < NREG; ++p)
      *reinterpret_cast<uint4*>(lds + ((threadIdx.x >> 3) + 32 * p) * LDK + kc) = v[p];
  }
};

// fprop activation operand: row m=(n,ho,wo), reduced index (tap, ci) gathered from x.
template <int T>
struct FpropRows {
  static constexpr int NREG = T / 32;
  const bf16_t* x;
  int Cin, Hin, Win, kW, K, kc;
  int hi0[NREG], wi0[NREG], base[NREG];
  __device__ void init(const IgemmParams& p, int tile_row0) {
    const Geom& g = p.g;
    x = p.act;
    Cin = g.Cin; Hin = g.Hin; Win = g.Win; kW = g.kW; K = g.K;
    kc = (threadIdx.x & 7) * 8;
#pragma unroll
    for (int q = 0; q < NREG; ++q) {
      const int m = tile_row0 + (threadIdx.x >> 3) + 32 * q;
      if (m < g.M) {
        const int wo = m % g.Wout;
        const int t = m / g.Wout;
        const int ho = t % g.Hout;
        const int n = t / g.Hout;
        hi0[q] = ho * g.sh - g.ph;
        wi0[q] = wo * g.sw - g.pw;
        base[q] = ((n * Hin + hi0[q]) * Win + wi0[q]) * Cin;
      } else {
        hi0[q] = -(1 << 28);
        wi0[q] = 0;
        base[q] = 0;
      }
    }
  }
  __device__ void load(int k0, int, uint4 (&v)[NREG]) const {
    const int k = k0 + kc;
    const int tap = k / Cin;
    const int ci = k - tap * Cin;
    const int i = tap / kW;
    const int j = tap - i * kW;
    const int koff = (i * Win + j) * Cin + ci;
#pragma unroll
    for (int q = 0; q < NREG; ++q) {
      const bool ok = k < K && (unsigned)(hi0[q] + i) < (unsigned)Hin && (unsigned)(wi0[q] + j) < (unsigned)Win;
      v[q] = ok ? ldg16(x + (base[q] + koff)) : zero16();
    }
  }
  __device__ void store(bf16_t* lds, const uint4 (&v)[NREG]) const {
#pragma unroll
    for (int q = 0; q < NREG; ++q)
      *reinterpret_cast<uint4*>(lds + ((threadIdx.x >> 3) + 32 * q) * LDK + kc) = v[q];
  }
};

// dgrad activation operand: row m'=(n,h,w), reduced index (tap, co) gathered from dz:
// tap (i,j) contributes dz[n,(h+ph-i)/sh,(w+pw-j)/sw,co] when both quotients are exact
// and in range (the adjoint of the forward gather).
template <int T>
struct DgradRows {
  static constexpr int NREG = T / 32;
  const bf16_t* dz;
  int Cout, Hout, Wout, kW, K, sh, sw, kc;
  int hz0[NREG], wz0[NREG], nbase[NREG];
  __device__ void init(const IgemmParams& p, int tile_row0) {
    const Geom& g = p.g;
    dz = p.act;
    Cout = g.Cout; Hout = g.Hout; Wout = g.Wout; kW = g.kW; sh = g.sh; sw = g.sw;
    K = g.kH * g.kW * g.Cout;
    kc = (threadIdx.x & 7) * 8;
#pragma unroll
    for (int q = 0; q < NREG; ++q) {
      const int m = tile_row0 + (threadIdx.x >> 3) + 32 * q;
      if (m < g.Min) {
        const int w = m % g.Win;
        const int t = m / g.Win;
        const int h = t % g.Hin;
        const int n = t / g.Hin;
        hz0[q] = h + g.ph;
        wz0[q] = w + g.pw;
        nbase[q] = n * Hout * Wout * Cout;
      } else {
        hz0[q] = -(1 << 28);
        wz0[q] = 0;
        nbase[q] = 0;
      }
    }
  }
  __device__ void load(int k0, int, uint4 (&v)[NREG]) const {
    const int k = k0 + kc;
    const int tap = k / Cout;
    const int co = k - tap * Cout;
    const int i = tap / kW;
    const int j = tap - i * kW;
#pragma unroll
    for (int q = 0; q < NREG; ++q) {
      const int hz = hz0[q] - i, wz = wz0[q] - j;
      int ho = hz, wo = wz;
      bool ok = k < K && hz >= 0 && wz >= 0;
      if (sh != 1) { ho = hz / sh; ok = ok && (ho * sh == hz); }
      if (sw != 1) { wo = wz / sw; ok = ok && (wo * sw == wz); }
      ok = ok && ho < Hout && wo < Wout;
      v[q] = ok ? ldg16(dz + (nbase[q] + (ho * Wout + wo) * Cout + co)) : zero16();
    }
  }
  __device__ void store(bf16_t* lds, const uint4 (&v)[NREG]) const {
#pragma unroll
    for (int q = 0; q < NREG; ++q)
      *reinterpret_cast<uint4*>(lds + ((threadIdx.x >> 3) + 32 * q) * LDK + kc) = v[q];
  }
};

// 8x8 transpose of bf16 held as 8 x uint4 (in[e] = 8 consecutive row-elements at reduced
// index e)  ->  out[r] = 8 consecutive reduced-index elements of row r.
__device__ __forceinline__ void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
  uint32_t w[8][4];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    w[e][0] = in[e].x; w[e][1] = in[e].y; w[e][2] = in[e].z; w[e][3] = in[e].w;
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    uint32_t o[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t a = w[2 * d][r >> 1], b = w[2 * d + 1][r >> 1];
      o[d] = (r & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
    }
    out[r] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// Transposing loaders (wgrad): the reduced index is the output pixel m; memory is
// contiguous along the row index.  A unit is 8 rows x 8 pixels; thread u < T owns unit
// (row group u % (T/8), pixel group u / (T/8)).
template <int T>
struct WgradDzRows {   // rows = co, from dz[m][Cout]
  static constexpr int NREG = 8;
  const bf16_t* dz;
  int Cout, r0, rg, mg;
  bool active;
  __device__ void init(const IgemmParams& p, int tile_row0) {
    dz = p.wgt;
    Cout = p.g.Cout;
    const int u = threadIdx.x;
    rg = u % (T / 8);
    mg = u / (T / 8);
    r0 = tile_row0 + rg * 8;
    active = u < T && r0 < Cout;
  }
  __device__ void load(int m0, int mend, uint4 (&v)[NREG]) const {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int m = m0 + mg * 8 + e;
      v[e] = (active && m < mend) ? ldg16(dz + ((size_t)m * Cout + r0)) : zero16();
    }
  }
  __device__ void store(bf16_t* lds, const uint4 (&v)[NREG]) const {
    if (threadIdx.x >= T) return;
    uint4 o[8];
    transpose8x8(v, o);
#pragma unroll
    for (int r = 0; r < 8; ++r) *reinterpret_cast<uint4*>(lds + (rg * 8 + r) * LDK + mg * 8) = o[r];
  }
};

template <int T>
struct WgradXRows {   // rows = k=(tap,ci), from x gathered at the pixel's window position
  static constexpr int NREG = 8;
  const bf16_t* x;
  int Cin, Hin, Win, Hout, Wout, sh, sw, rg, mg;
  int di, dj, ci0;     // tap offsets (i - ph, j - pw) and first channel of the row group
  bool active;
  __device__ void init(const IgemmParams& p, int tile_row0) {
    const Geom& g = p.g;
    x = p.act;
    Cin = g.Cin; Hin = g.Hin; Win = g.Win; Hout = g.Hout; Wout = g.Wout; sh = g.sh; sw = g.sw;
    const int u = threadIdx.x;
    rg = u % (T / 8);
    mg = u / (T / 8);
    const int r0 = tile_row0 + rg * 8;
    active = u < T && r0 < g.K;
    const int tap = r0 / Cin;
    ci0 = r0 - tap * Cin;
    const int i = tap / g.kW;
    di = i - g.ph;
    dj = (tap - i * g.kW) - g.pw;
  }
  __device__ void load(int m0, int mend, uint4 (&v)[NREG]) const {
    const int m = m0 + mg * 8;
    int wo = m % Wout;
    const int t = m / Wout;
    int ho = t % Hout;
    int n = t / Hout;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int h = ho * sh + di, w = wo * sw + dj;
      const bool ok = active && (m + e) < mend && (unsigned)h < (unsigned)Hin && (unsigned)w < (unsigned)Win;
      v[e] = ok ? ldg16(x + (((n * Hin + h) * Win + w) * Cin + ci0)) : zero16();
      if (++wo == Wout) {
        wo = 0;
        if (++ho == Hout) { ho = 0; ++n; }
      }
    }
  }
  __device__ void store(bf16_t* lds, const uint4 (&v)[NREG]) const {
    if (threadIdx.x >= T) return;
    uint4 o[8];
    transpose8x8(v, o);
#pragma unroll
    for (int r = 0; r < 8; ++r) *reinterpret_cast<uint4*>(lds + (rg * 8 + r) * LDK + mg * 8) = o[r];
  }
};

enum { PASS_FPROP = 0, PASS_DGRAD = 1, PASS_WGRAD = 2 };

template <int PASS, int T> struct RowLoader;
template <int PASS, int T> struct ColLoader;
template <int T> struct RowLoader<PASS_FPROP, T> : PlainRows<T> {
  __device__ void setup(const IgemmParams& p, int t0) { this->init(p, p.g.Cout, p.g.K, t0); }
};
template <int T> struct ColLoader<PASS_FPROP, T> : FpropRows<T> {
  __device__ void setup(const IgemmParams& p, int t0) { this->init(p, t0); }
};
template <int T> struct RowLoader<PASS_DGRAD, T> : PlainRows<T> {
  __device__ void setup(const IgemmParams& p, int t0) {
    this->init(p, p.g.Cin, p.g.kH * p.g.kW * p.g.Cout, t0);
  }
};
template <int T> struct ColLoader<PASS_DGRAD, T> : DgradRows<T> {
  __device__ void setup(const IgemmParams& p, int t0) { this->init(p, t0); }
};
template <int T> struct RowLoader<PASS_WGRAD, T> : WgradXRows<T> {
  __device__ void setup(const IgemmParams& p, int t0) { this->init(p, t0); }
};
template <int T> struct ColLoader<PASS_WGRAD, T> : WgradDzRows<T> {
  __device__ void setup(const IgemmParams& p, int t0) { this->init(p, t0); }
};

// ---- the kernel ------------------------------------------------------------------
// 256 threads = 4 waves; tile TR (rows) x TC (cols); each wave owns WR x WC as
// (WR/32) x (WC/32) MFMA accumulators.  One LDS stage, next stage prefetched into
// registers while the current one is multiplied.
template <int PASS, int TR, int TC, int WR, int WC>
__global__ __launch_bounds__(256) void igemm_kernel(IgemmParams p) {
  static_assert((TR / WR) * (TC / WC) == 4, "four waves");
  static_assert(PASS != PASS_WGRAD || (TR <= 256 && TC <= 256), "one transposing unit per thread");
  __shared__ __attribute__((aligned(16))) bf16_t ldsR[TR * LDK];
  __shared__ __attribute__((aligned(16))) bf16_t ldsC[TC * LDK];

  const Geom& g = p.g;
  int R, C, red_beg, red_end;
  if (PASS == PASS_FPROP) { R = g.Cout; C = g.M; red_beg = 0; red_end = g.K; }
  else if (PASS == PASS_DGRAD) { R = g.Cin; C = g.Min; red_beg = 0; red_end = g.kH * g.kW * g.Cout; }
  else {
    R = g.K; C = g.Cout;
    red_beg = blockIdx.y * p.red_per_split;
    red_end = min(g.M, red_beg + p.red_per_split);
  }
  const int ntr = (R + TR - 1) / TR;
  const int tile_r0 = (blockIdx.x % ntr) * TR;
  const int tile_c0 = (blockIdx.x / ntr) * TC;

  RowLoader<PASS, TR> rl;
  ColLoader<PASS, TC> cl;
  rl.setup(p, tile_r0);
  cl.setup(p, tile_c0);

  constexpr int NI = WR / 32, NJ = WC / 32;
  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wr0 = (wave % (TR / WR)) * WR;
  const int wc0 = (wave / (TR / WR)) * WC;
  const int frag_off = (lane & 31) * LDK + (lane >> 5) * 8;

  uint4 rv[RowLoader<PASS, TR>::NREG];
  uint4 cv[ColLoader<PASS, TC>::NREG];
  if (red_beg < red_end) {
    rl.load(red_beg, red_end, rv);
    cl.load(red_beg, red_end, cv);
  }
  for (int k0 = red_beg; k0 < red_end; k0 += BK) {
    __syncthreads();
    rl.store(ldsR, rv);
    cl.store(ldsC, cv);
    __syncthreads();
    if (k0 + BK < red_end) {
      rl.load(k0 + BK, red_end, rv);
      cl.load(k0 + BK, red_end, cv);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 a[NI], b[NJ];
#pragma unroll
      for (int i = 0; i < NI; ++i)
        a[i] = *reinterpret_cast<const bf16x8*>(ldsR + (wr0 + i * 32) * LDK + kk * 16 + frag_off);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        b[j] = *reinterpret_cast<const bf16x8*>(ldsC + (wc0 + j * 32) * LDK + kk * 16 + frag_off);
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  // Epilogue.  Accumulator element e of lane l: row 8*(e/4) + 4*(l/32) + e%4, col l%32.
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int col = tile_c0 + wc0 + j * 32 + (lane & 31);
      if (col >= C) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = tile_r0 + wr0 + i * 32 + q * 8 + (lane >> 5) * 4;
        if (row >= R) continue;   // R is a multiple of 8 and row of 4: row+3 < R
        float v0 = acc[i][j][q * 4 + 0], v1 = acc[i][j][q * 4 + 1];
        float v2 = acc[i][j][q * 4 + 2], v3 = acc[i][j][q * 4 + 3];
        if (PASS == PASS_WGRAD) {
          float* o = reinterpret_cast<float*>(p.out) + (size_t)blockIdx.y * ((size_t)C * R) +
                     (size_t)col * R + row;
          *reinterpret_cast<float4*>(o) = make_float4(v0, v1, v2, v3);
        } else {
          if (p.bias) {
            const float4 bb = *reinterpret_cast<const float4*>(p.bias + row);
            v0 += bb.x; v1 += bb.y; v2 += bb.z; v3 += bb.w;
          }
          bf16_t* o = reinterpret_cast<bf16_t*>(p.out) + (size_t)col * R + row;
          *reinterpret_cast<uint2*>(o) = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
        }
      }
    }
}

template <int PASS, int TR, int TC, int WR, int WC>
hipError_t launch_cfg(const IgemmParams& p, int R, int C, int nsplit, hipStream_t st) {
  const int tiles = ceil_div(R, TR) * ceil_div(C, TC);
  hipLaunchKernelGGL((igemm_kernel<PASS, TR, TC, WR, WC>), dim3(tiles, nsplit), dim3(256), 0, st, p);
  return hipGetLastError();
}

template <int PASS>
hipError_t launch_pass(const IgemmParams& p, int R, int C, int nsplit, hipStream_t st) {
  if (PASS == PASS_WGRAD) {
    // rows = taps*Cin (>= 8), cols = Cout
    if (C <= 64) return launch_cfg<PASS, 256, 64, 64, 64>(p, R, C, nsplit, st);
    return launch_cfg<PASS, 128, 128, 64, 64>(p, R, C, nsplit, st);
  }
  if (R <= 64) return launch_cfg<PASS, 64, 256, 64, 64>(p, R, C, nsplit, st);
  return launch_cfg<PASS, 128, 128, 64, 64>(p, R, C, nsplit, st);
}

}  // namespace

bool igemm_supported(const Geom& g, int dtype) {
  return dtype == CONVBN_BF16 && g.Cin % 8 == 0 && g.Cout % 8 == 0;
}

// Number of pixel slices of the weight-gradient reduction: enough blocks to cover the
// chip about twice, each slice a multiple of the LDS stage.
int wgrad_splits(const Geom& g) {
  const int tr = g.Cout <= 64 ? 256 : 128, tc = g.Cout <= 64 ? 64 : 128;
  const int tiles = ceil_div(g.K, tr) * ceil_div(g.Cout, tc);
  int want = ceil_div(512, tiles);
  const int maxs = ceil_div(g.M, 4 * BK);
  if (want > maxs) want = maxs;
  // at most 64 slices, except where so few tiles exist that 64 slices leave CUs idle (a 7x7 stem: 2 tiles)
  const int cap = tiles * 64 >= 256 ? 64 : ceil_div(256, tiles);
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  // make slices multiples of BK and drop empty ones
  const int per = ceil_div(ceil_div(g.M, want), BK) * BK;
  return ceil_div(g.M, per);
}

static int wgrad_red_per_split(const Geom& g, int nsplit) {
  return ceil_div(ceil_div(g.M, nsplit), BK) * BK;
}

hipError_t launch_fprop_igemm(const Geom& g, const void* x, const void* w_krsc, const float* bias,
                              void* z, hipStream_t st) {
  IgemmParams p{(const bf16_t*)x, (const bf16_t*)w_krsc, bias, z, g, 0};
  return launch_pass<PASS_FPROP>(p, g.Cout, g.M, 1, st);
}

hipError_t launch_dgrad_igemm(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                              hipStream_t st) {
  IgemmParams p{(const bf16_t*)dz, (const bf16_t*)w_crsk, bias, dx, g, 0};
  return launch_pass<PASS_DGRAD>(p, g.Cin, g.Min, 1, st);
}

hipError_t launch_wgrad_igemm(const Geom& g, const void* x, const void* dz, float* dwf_part,
                              int nsplit, hipStream_t st) {
  IgemmParams p{(const bf16_t*)x, (const bf16_t*)dz, nullptr, dwf_part, g,
                wgrad_red_per_split(g, nsplit)};
  return launch_pass<PASS_WGRAD>(p, g.K, g.Cout, nsplit, st);
}

}  // namespace convbn
