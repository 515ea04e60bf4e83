// Forward convolution of a network's first layer (Sec. 3.1's Y = w (*) X + b with at most four input
// channels, e.g. the 7x7 / stride-2 stem of a ResNet on RGB images), bf16 MFMA with fp32 accumulation.
//
// With 3 input channels the reduction index (tap, channel) has no 16-byte runs for the generic kernels to
// gather, and padding the channels to 8 makes them multiply and fetch mostly zeros.  Here the pixels are
// widened to 4 channels (8 bytes) on their way into LDS and the reduction index is ordered (window row i, window column
// j padded to 8, channel c padded to 4): the 8 consecutive reduction elements an MFMA lane needs -- two
// window columns x four channels -- are then 16 contiguous bytes of the input row, for every output pixel.
// So no im2col is ever materialised: the operand fragments are read straight from the raw input patch in
// LDS (output pixel wo, window columns j..j+1 -> patch bytes (wo sw + j) 8 ..), consecutive lanes 8 sw bytes
// apart.  The weights (Cout x kH x 8 x 4, zero-padded) stay resident in LDS; a workgroup is persistent and
// walks tiles of 128 consecutive pixels of one output row: patch in (kH rows x (127 sw + 8) pixels), kH x 2
// MFMA k-steps, staged 16-byte stores out.
#include "common.h"

namespace convbn {

namespace {

constexpr int TPX = 128;            // output pixels per tile (32 per wave)
constexpr int KROW = 32;            // reduction elements per window row: 8 columns x 4 channels

struct StemParams {
  const bf16_t* x;      // X3: [N][H][W][3] (W % 4 == 0); else [N][H][W][4]
  const bf16_t* w;      // [Cout][kH][8][4]: the weight zero-padded to 8 window columns and 4 channels
  const float* bias;    // [Cout] or null
  bf16_t* z;            // [N][Ho][Wo][Cout]
  int N, H, W, Cin, Cout, kH, kW, sh, sw, ph, pw, Ho, Wo;
  int ntw, ntiles;      // tiles per output row, tiles in all
  int wpitch;           // LDS bytes per weight row: kH * 64 + 16
  int prow;             // LDS bytes per patch row: ((TPX - 1) sw + 8) * 8
  int pcols;            // pixels per patch row (X3: a multiple of 4, with up to 3 leading pixels of alignment)
};

constexpr int ppt(bool x3) { return x3 ? 3 : 8; }   // most patch items a thread fetches per tile

// NCO: 32-channel fragments per workgroup (Cout = 32 NCO); KH: window rows (0 = run-time, any number); X3: the
// input has 3 channels and is fetched four pixels (24 contiguous bytes) at a time, else 4 channels, one pixel
// (8 bytes) at a time.
template <int NCO, int KH, bool X3>
__global__ __launch_bounds__(256) void stem_fprop_kernel(StemParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* biasl = reinterpret_cast<float*>(smem);                       // [Cout] (first 512 bytes)
  unsigned char* wl = smem + 512;                                      // [Cout][wpitch]
  unsigned char* patch = wl + 32 * NCO * p.wpitch;                     // [kH][prow]; reused to stage the output tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = lane >> 5, px = lane & 31;
  const int kH = KH > 0 ? KH : p.kH;

  // ---- resident weights: rows of the padded [Cout][kH][8][4] block, 16 bytes per load
  const int wrow_g = kH * KROW / 8;   // 16-byte granules per weight row
  for (int e = tid; e < 32 * NCO * wrow_g; e += 256) {
    const int co = e / wrow_g, gq = e - co * wrow_g;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (co < p.Cout) v = *reinterpret_cast<const uint4*>(p.w + ((size_t)co * wrow_g + gq) * 8);
    *reinterpret_cast<uint4*>(wl + co * p.wpitch + gq * 16) = v;
  }
  if (tid < 32 * NCO) biasl[tid] = (p.bias && tid < p.Cout) ? p.bias[tid] : 0.f;

  // patch item e = tid + 256 k of a tile: (row i, pixel -- X3: group of four pixels -- q), the same for every tile
  constexpr int PPT = ppt(X3);
  constexpr int PXI = X3 ? 4 : 1;                 // pixels per item
  constexpr int NLD = X3 ? 3 : 1;                 // 8-byte loads per item
  const int icols = p.pcols / PXI;
  const int npatch = kH * icols;
  int pi[PPT], pq[PPT];
#pragma unroll
  for (int k = 0; k < PPT; ++k) {
    const int e = tid + 256 * k;
    pi[k] = e / icols;
    pq[k] = (e - pi[k] * icols) * PXI;
  }
  // first patch pixel of a tile: wo0 sw - pw, X3: rounded down to a multiple of four pixels
  auto patch_start = [&](int ws) {
    const int wbase = ws * TPX * p.sw - p.pw;
    return X3 ? (wbase >> 2) << 2 : wbase;
  };
  // fetch of a tile's patch into registers (zeros outside the image); the tile after the current one is
  // always in flight while the current one is multiplied
  uint2 pv[PPT][NLD];
  auto fetch = [&](int tile) {
    const int ws = tile % p.ntw;
    const int row = tile / p.ntw;
    const int ho = row % p.Ho, n = row / p.Ho;
    const int wstart = patch_start(ws);
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      const int h = ho * p.sh + pi[k] - p.ph, w = wstart + pq[k];
#pragma unroll
      for (int j = 0; j < NLD; ++j) pv[k][j] = make_uint2(0u, 0u);
      if (tid + 256 * k < npatch && tile < p.ntiles && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W) {
        const uint2* src = reinterpret_cast<const uint2*>(p.x + (((size_t)n * p.H + h) * p.W + w) * (X3 ? 3 : 4));
#pragma unroll
        for (int j = 0; j < NLD; ++j) pv[k][j] = src[j];
      }
    }
  };
  // registers -> LDS, every pixel as 4 channels (X3: the 12 values of four pixels spread over 4 x 8 bytes)
  auto stash = [&]() {
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      if (tid + 256 * k >= npatch) continue;
      unsigned char* dst = patch + pi[k] * p.prow + pq[k] * 8;
      if constexpr (X3) {
        const uint2 a = pv[k][0], b = pv[k][1], c = pv[k][2];
        *reinterpret_cast<uint4*>(dst) = make_uint4(a.x, a.y & 0xffffu, (a.y >> 16) | (b.x << 16), b.x >> 16);
        *reinterpret_cast<uint4*>(dst + 16) = make_uint4(b.y, c.x & 0xffffu, (c.x >> 16) | (c.y << 16), c.y >> 16);
      } else {
        *reinterpret_cast<uint2*>(dst) = pv[k][0];
      }
    }
  };
  fetch(blockIdx.x);

  for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
    const int ws = tile % p.ntw;
    const int row = tile / p.ntw;
    const int ho = row % p.Ho, n = row / p.Ho;
    const int wo0 = ws * TPX;
    __syncthreads();   // the previous tile's staged output has been read
    stash();
    fetch(tile + gridDim.x);
    __syncthreads();   // patch (and, first pass, weights and bias) visible

    f32x16 acc[NCO];
#pragma unroll
    for (int f = 0; f < NCO; ++f)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[f][e] = 0.f;
    // lane's pixel: wo0 + 32 wave + px; its window starts at patch pixel (32 wave + px) sw (+ the alignment pixels)
    const int lead = wo0 * p.sw - p.pw - patch_start(ws);
    const unsigned char* prow0 = patch + ((wave * 32 + px) * p.sw + 2 * kb + lead) * 8;
    const unsigned char* wrow0 = wl + px * p.wpitch + kb * 16;
    auto kstep = [&](int i, int jh) {   // window row i, columns 4 jh .. 4 jh + 3: lanes kb = 0 / 1 take two each
      const unsigned char* bp = prow0 + i * p.prow + jh * 32;
      const uint2 b0 = *reinterpret_cast<const uint2*>(bp);
      const uint2 b1 = *reinterpret_cast<const uint2*>(bp + 8);
      const bf16x8 fb = __builtin_bit_cast(bf16x8, make_uint4(b0.x, b0.y, b1.x, b1.y));
#pragma unroll
      for (int f = 0; f < NCO; ++f) {
        const bf16x8 fa = *reinterpret_cast<const bf16x8*>(wrow0 + f * 32 * p.wpitch + (i * 2 + jh) * 32);
        acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[f], 0, 0, 0);
      }
    };
    if (KH > 0) {
#pragma unroll
      for (int i = 0; i < KH; ++i) { kstep(i, 0); kstep(i, 1); }
    } else {
      for (int i = 0; i < kH; ++i) { kstep(i, 0); kstep(i, 1); }
    }
    __syncthreads();   // every wave is done with the patch: its memory now stages the output tile
    // ---- epilogue: accumulator element e of lane l is channel 8 (e / 4) + 4 (l / 32) + e % 4 of pixel l % 32.
    // Each wave rounds its 32 pixels x Cout channels into its own LDS block ([pixel][Cout], 16-byte granules
    // swizzled by pixel) and reads it back row-wise: every global store is 16 bytes per lane.
    constexpr int ROWB = 32 * NCO * 2;          // bytes per staged pixel row
    constexpr int GR = ROWB / 16;               // 16-byte granules per row
    unsigned char* st = patch + wave * 32 * ROWB;
    const int psw = (px >> 1) & (GR - 1);
#pragma unroll
    for (int f = 0; f < NCO; ++f)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int ch = f * 32 + q * 8 + kb * 4;
        const float4 bb = *reinterpret_cast<const float4*>(biasl + ch);
        const uint2 v = make_uint2(pack_bf16x2(acc[f][q * 4 + 0] + bb.x, acc[f][q * 4 + 1] + bb.y),
                                   pack_bf16x2(acc[f][q * 4 + 2] + bb.z, acc[f][q * 4 + 3] + bb.w));
        *reinterpret_cast<uint2*>(st + px * ROWB + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
      }
    // (a wave reads only what it wrote itself: no workgroup barrier needed, the LDS counter orders it)
    constexpr int RPP = 64 / GR;                // pixel rows covered by one pass of the wave
#pragma unroll
    for (int pass = 0; pass < 32 / RPP; ++pass) {
      const int r = pass * RPP + lane / GR;
      const int g = (lane % GR) ^ ((r >> 1) & (GR - 1));
      const uint4 v = *reinterpret_cast<const uint4*>(st + r * ROWB + ((lane % GR) << 4));
      const int wo = wo0 + wave * 32 + r;
      const int ch = g * 8;
      if (wo < p.Wo && ch < p.Cout)
        *reinterpret_cast<uint4*>(p.z + (((size_t)n * p.Ho + ho) * p.Wo + wo) * p.Cout + ch) = v;
    }
  }
}

// wp[co][i][j][c] (8 columns, 4 channels) = w[co][i][j][c] where it exists, else 0
__global__ __launch_bounds__(256) void stem_pack_weights_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wp,
                                                                int Cout, int kH, int kW, int Cin) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= Cout * kH * KROW) return;
  const int c = e & 3, j = (e >> 2) & 7, t = e >> 5;   // t = co kH + i
  wp[e] = (j < kW && c < Cin) ? w[((size_t)t * kW + j) * Cin + c] : from_f32<bf16_t>(0.f);
}

// ---- weight gradient of a first layer ------------------------------------------------------------------
// dw'[co][i][j][c] = sum over output pixels of dZ[pixel][co] X[pixel's window (i, j)][c]  and  r[co] = sum dZ
// (Sec. 3.2.1, App. B), with the same operand trick as the forward kernel: the reduced index is the pixel, so
// both MFMA operands are read with the transposing LDS load (ds_read_tr16_b64: a lane supplies the address of 8
// bytes -- here one padded input pixel (window column j, 4 channels) resp. 4 output channels of one pixel -- and
// receives 4 consecutive pixels of one row of the operand).  Rows of the left operand are the 32 (j, c) pairs of
// one window row, taken straight from the raw input patch: lane address = patch pixel (pixel sw + j).
// A persistent workgroup walks tiles of 128 pixels of one output row; wave w owns window rows w and w + 4 for
// all output channels and keeps their sums in registers over all its tiles; the partial sums of every workgroup
// go to memory once, as fp32 slices for the fold-back.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ s16x4 read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}
__device__ __forceinline__ bf16x8 join(s16x4 a, s16x4 b) {
  s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}

struct StemWgParams {
  const bf16_t* x;      // X3: [N][H][W][3] (W % 4 == 0); else [N][H][W][4]
  const bf16_t* dz;     // [N][Ho][Wo][Cout]
  float* part;          // [slices][Cout][kH kW Cin]
  float* r_part;        // [slices][Cout] or null
  int N, H, W, Cin, Cout, kH, kW, sh, sw, ph, pw, Ho, Wo;
  int ntw, ntiles, prow, pcols;
  int zpitch;           // LDS bytes per dZ pixel row: 2 Cout + 16
};

template <int NCO, bool X3>
__global__ __launch_bounds__(256) void stem_wgrad_kernel(StemWgParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* patch = smem;                                   // [kH][prow]
  unsigned char* zt = smem + (p.kH * p.prow + 15) / 16 * 16;      // [TPX][zpitch]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = lane >> 5;
  const int eprime = (lane & 15) >> 2;                           // pixel (of 4) this lane addresses in a transposing read
  const int quad = ((lane >> 4) & 1) * 4 + (lane & 3);           // its 8-byte quad inside the 32-row operand block
  constexpr int PPT = ppt(X3), PXI = X3 ? 4 : 1, NLD = X3 ? 3 : 1;
  constexpr int NRW = 2;                                         // window rows per wave: w and w + 4 (kH <= 8)
  constexpr int ZG = 32 * NCO * 2 / 16;                          // 16-byte granules per dZ pixel row
  constexpr int ZPT = TPX * ZG / 256;                            // granules per thread and tile

  const int icols = p.pcols / PXI;
  const int npatch = p.kH * icols;
  int pi[PPT], pq[PPT];
#pragma unroll
  for (int k = 0; k < PPT; ++k) {
    const int e = tid + 256 * k;
    pi[k] = e / icols;
    pq[k] = (e - pi[k] * icols) * PXI;
  }
  auto patch_start = [&](int ws) {
    const int wbase = ws * TPX * p.sw - p.pw;
    return X3 ? (wbase >> 2) << 2 : wbase;
  };
  uint2 pv[PPT][NLD];
  uint4 zv[ZPT];
  auto fetch = [&](int tile) {
    const int ws = tile % p.ntw;
    const int row = tile / p.ntw;
    const int ho = row % p.Ho, n = row / p.Ho;
    const int wstart = patch_start(ws);
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      const int h = ho * p.sh + pi[k] - p.ph, w = wstart + pq[k];
#pragma unroll
      for (int j = 0; j < NLD; ++j) pv[k][j] = make_uint2(0u, 0u);
      if (tid + 256 * k < npatch && tile < p.ntiles && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W) {
        const uint2* src = reinterpret_cast<const uint2*>(p.x + (((size_t)n * p.H + h) * p.W + w) * (X3 ? 3 : 4));
#pragma unroll
        for (int j = 0; j < NLD; ++j) pv[k][j] = src[j];
      }
    }
    // dZ rows of the tile's pixels (zeros past the end of the output row: such pixels then add nothing)
#pragma unroll
    for (int k = 0; k < ZPT; ++k) {
      const int e = tid + 256 * k;
      const int px = e / ZG, gq = e - px * ZG;
      const int wo = ws * TPX + px;
      zv[k] = make_uint4(0u, 0u, 0u, 0u);
      if (tile < p.ntiles && wo < p.Wo && gq * 8 < p.Cout)
        zv[k] = *reinterpret_cast<const uint4*>(p.dz + (((size_t)n * p.Ho + ho) * p.Wo + wo) * p.Cout + gq * 8);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      if (tid + 256 * k >= npatch) continue;
      unsigned char* dst = patch + pi[k] * p.prow + pq[k] * 8;
      if constexpr (X3) {
        const uint2 a = pv[k][0], b = pv[k][1], c = pv[k][2];
        *reinterpret_cast<uint4*>(dst) = make_uint4(a.x, a.y & 0xffffu, (a.y >> 16) | (b.x << 16), b.x >> 16);
        *reinterpret_cast<uint4*>(dst + 16) = make_uint4(b.y, c.x & 0xffffu, (c.x >> 16) | (c.y << 16), c.y >> 16);
      } else {
        *reinterpret_cast<uint2*>(dst) = pv[k][0];
      }
    }
#pragma unroll
    for (int k = 0; k < ZPT; ++k) {
      const int e = tid + 256 * k;
      const int px = e / ZG, gq = e - px * ZG;
      *reinterpret_cast<uint4*>(zt + px * p.zpitch + gq * 16) = zv[k];
    }
  };

  f32x16 acc[NRW][NCO];
#pragma unroll
  for (int t = 0; t < NRW; ++t)
#pragma unroll
    for (int f = 0; f < NCO; ++f)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][f][e] = 0.f;
  // channel sums: thread -> channel tid % Cout' (Cout' = 32 NCO), every (256 / Cout')-th pixel
  constexpr int CW = 32 * NCO, RL = 256 / CW;
  const int rc = tid % CW, rl = tid / CW;
  float racc = 0.f;

  fetch(blockIdx.x);
  for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
    const int ws = tile % p.ntw;
    __syncthreads();   // the previous tile has been read
    stash();
    fetch(tile + gridDim.x);
    __syncthreads();   // patch and dZ tile visible
    const int lead = ws * TPX * p.sw - p.pw - patch_start(ws);
#pragma unroll
    for (int px = rl; px < TPX; px += RL)
      racc += bf16_bits_to_f32(*reinterpret_cast<const unsigned short*>(zt + px * p.zpitch + rc * 2));
    // lane-constant parts of the operand addresses
    const unsigned char* zl = zt + (kb * 8 + eprime) * p.zpitch + (((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2;
    const unsigned char* xl = patch + (((kb * 8 + eprime) * p.sw + quad + lead) * 8);
    for (int k = 0; k < TPX / 16; ++k) {
      bf16x8 zf[NCO];
#pragma unroll
      for (int f = 0; f < NCO; ++f)
        zf[f] = join(read_tr(zl + (k * 16) * p.zpitch + f * 64), read_tr(zl + (k * 16 + 4) * p.zpitch + f * 64));
#pragma unroll
      for (int t = 0; t < NRW; ++t) {
        const int i = wave + 4 * t;
        if (i >= p.kH) break;
        const unsigned char* xr = xl + i * p.prow + (k * 16) * p.sw * 8;
        const bf16x8 xf = join(read_tr(xr), read_tr(xr + 4 * p.sw * 8));
#pragma unroll
        for (int f = 0; f < NCO; ++f) acc[t][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, zf[f], acc[t][f], 0, 0, 0);
      }
    }
  }
  // ---- this workgroup's slice.  Accumulator element e of lane l: operand row 8 (e / 4) + 4 (l / 32) + e % 4 =
  // window column 2 (e / 4) + l / 32, channel e % 4; output channel f 32 + l % 32.
  const int K = p.kH * p.kW * p.Cin;
#pragma unroll
  for (int t = 0; t < NRW; ++t) {
    const int i = wave + 4 * t;
    if (i >= p.kH) break;
#pragma unroll
    for (int f = 0; f < NCO; ++f) {
      const int co = f * 32 + (lane & 31);
      if (co >= p.Cout) continue;
      float* orow = p.part + ((size_t)blockIdx.x * p.Cout + co) * K + (size_t)i * p.kW * p.Cin;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int j = 2 * q + kb;
        if (j >= p.kW) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (c < p.Cin) orow[j * p.Cin + c] = acc[t][f][q * 4 + c];
      }
    }
  }
  if (p.r_part) {
    __syncthreads();   // every wave is done with the tiles: reuse the patch memory
    float* red = reinterpret_cast<float*>(smem);
    red[tid] = racc;
    __syncthreads();
    if (tid < CW && tid < p.Cout) {
      float v = 0.f;
#pragma unroll
      for (int l = 0; l < RL; ++l) v += red[l * CW + tid];
      p.r_part[(size_t)blockIdx.x * p.Cout + tid] = v;
    }
  }
}

struct StemWgPlan { bool ok; bool x3; int nco; size_t lds; int grid; };
StemWgPlan stem_wg_plan(const Geom& g, StemWgParams* pp) {
  StemWgPlan pl{false, false, 0, 0, 0};
  StemWgParams& p = *pp;
  p = StemWgParams{};
  if (g.kH > 8) return pl;   // two window rows per wave
  p.N = g.N; p.H = g.Hin; p.W = g.Win; p.Cin = g.Cin; p.Cout = g.Cout; p.kH = g.kH; p.kW = g.kW;
  p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.Ho = g.Hout; p.Wo = g.Wout;
  p.ntw = ceil_div(g.Wout, TPX);
  p.ntiles = g.N * g.Hout * p.ntw;
  const bool x3 = g.Cin == 3 && g.Win % 4 == 0;
  p.pcols = (TPX - 1) * g.sw + 8;
  if (x3) p.pcols = (p.pcols + 3 + 3) / 4 * 4;
  p.prow = p.pcols * 8;
  pl.nco = ceil_div(g.Cout, 32);
  if (pl.nco != 1 && pl.nco != 2 && pl.nco != 4) return pl;
  if (g.kH * (p.pcols / (x3 ? 4 : 1)) > 256 * ppt(x3)) return pl;
  p.zpitch = 32 * pl.nco * 2 + 16;
  pl.lds = align_up((size_t)g.kH * p.prow, 16) + (size_t)TPX * p.zpitch;
  if (pl.lds < 1024) pl.lds = 1024;   // the channel sums meet in the first KB at the end
  if (pl.lds > 64 * 1024) return pl;
  // two workgroups per CU (a lone one leaves the CU idle while it waits; 65 -> 48 us on the 7x7 stem); every
  // workgroup writes a full fp32 slice of dw', which the fold-back has to sum, so not more
  pl.grid = p.ntiles < 512 ? p.ntiles : 512;
  pl.x3 = x3;
  pl.ok = true;
  return pl;
}

// ---- input gradient of a first layer -------------------------------------------------------------------
// dX[h][w][c] = sum_{i,j,co} dZ[(h + ph - i) / sh][(w + pw - j) / sw][co] w'[co][i][j][c] over the taps for which the
// divisions are exact (Sec. 3.2.1).  With 3 input channels the result has almost no columns for a matrix product, so
// the sh x sw pixels of a block (a, b) = (h / sh, w / sw) and their (padded) 4 channels together form the 16 rows of
// one: every pixel of the block reads the same U x V neighbourhood of dZ -- rows a + Dh - u, columns b + Dw - v --
// only with a different subset of the taps, so   dX[block][(phase, c)] = sum_{u,v,co} Wt[(phase, c)][(u, v, co)]
// dZ[a + Dh - u][b + Dw - v][co],   Wt holding w' where phase (h % sh, w % sw) has a tap at (u, v) and zeros
// elsewhere (49 of 64 positions for 7x7 / stride 2).  That is a stride-1 convolution of dZ with a U x V window whose
// 16 output "channels" are un-shuffled to pixels (depth to space).  MFMA 16x16x32: rows = the 16 (phase, c)
// pairs, columns = 16 blocks, 32 output channels of one (u, v) per step; as in the forward kernel the column
// operand is read straight from the raw dZ patch in LDS (lane = block, 16 contiguous bytes = 8 channels) and the
// packed weight (16 x U V Cout) stays resident in LDS.  A lane ends up with the 4 channels of one dX pixel; the
// tile's pixels are gathered in LDS and leave as whole rows.
typedef float f32x4s __attribute__((ext_vector_type(4)));
constexpr int DG_PPT = 8;      // most 16-byte patch items a thread fetches per tile
constexpr int DG_NBT = 2;      // most 16-block groups a wave multiplies per tile

struct StemDgParams {
  const bf16_t* dz;     // [N][Ho][Wo][Cout]
  const bf16_t* wt;     // [16][U V Cout] packed by stem_dgrad_pack_kernel
  bf16_t* dx;           // [N][H][W][Cin]
  int N, H, W, Cin, Cout, Ho, Wo, sh, sw;
  int U, V, Dh, Dw;     // block (a, b) reads dZ rows a + Dh - u (u < U), columns b + Dw - v (v < V)
  int KT;               // U V Cout
  int TBR, TBC;         // blocks per tile
  int nbr, nbc, ntiles; // tiles per image column / row, tiles in all
  int PR, PC, pitch;    // dZ patch rows (TBR + U - 1), columns (TBC + V - 1), bytes per pixel (2 Cout + 16)
  int wpitch;           // LDS bytes per weight row (2 KT + 16)
  int nbt;              // 16-block groups per tile
  int orow;             // elements per staged dX row: TBC sw Cin
  int fast_store;       // rows leave as 16-byte pieces (all alignments allow it)
  unsigned mTBC, mPC;   // multipliers for n / TBC, n / PC (n < 65536)
};

__device__ __forceinline__ int dg_div(int n, unsigned m, int d) { return d == 1 ? n : (int)__umulhi((unsigned)n, m); }

// UU, VV, KS: the dZ neighbourhood and Cout / 32 at compile time (0: taken from the parameters)
template <int UU, int VV, int KS>
__global__ __launch_bounds__(256) void stem_dgrad_kernel(StemDgParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* wl = smem;                                         // [16][wpitch]
  unsigned char* patch = wl + 16 * p.wpitch;                        // [PR][PC][pitch]
  bf16_t* ost = reinterpret_cast<bf16_t*>(patch + (size_t)p.PR * p.PC * p.pitch);   // [TBR sh][orow]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, kg = lane >> 4;                        // MFMA column (block) / row (phase, c) and 8-channel group

  // ---- resident weight
  const int wgr = p.KT / 8;                                         // 16-byte granules per row
  for (int e = tid; e < 16 * wgr; e += 256) {
    const int r = e / wgr, gq = e - r * wgr;
    *reinterpret_cast<uint4*>(wl + r * p.wpitch + gq * 16) = *reinterpret_cast<const uint4*>(p.wt + (size_t)r * p.KT + gq * 8);
  }
  // ---- patch items of this thread: granule gq (8 channels) of patch pixel (row, column), the same for every tile
  const int gpp = p.Cout / 8;
  const int nitems = p.PR * p.PC * gpp;
  int ipr[DG_PPT], ipc[DG_PPT];
#pragma unroll
  for (int k = 0; k < DG_PPT; ++k) {
    const int e = tid + 256 * k;
    const int pix = e / gpp;
    ipr[k] = dg_div(pix, p.mPC, p.PC);
    ipc[k] = (pix - ipr[k] * p.PC) | ((e - pix * gpp) << 16);
  }
  uint4 pv[DG_PPT];
  auto fetch = [&](int tile) {
    const int tc = tile % p.nbc;
    const int t2 = tile / p.nbc;
    const int tr = t2 % p.nbr, n = t2 / p.nbr;
    // patch row r holds dZ row a0 + Dh - (U - 1) + r, column likewise
    const int h0 = tr * p.TBR + p.Dh - (p.U - 1), w0 = tc * p.TBC + p.Dw - (p.V - 1);
#pragma unroll
    for (int k = 0; k < DG_PPT; ++k) {
      const int h = h0 + ipr[k], w = w0 + (ipc[k] & 0xffff), gq = ipc[k] >> 16;
      const bool ok = tid + 256 * k < nitems && tile < p.ntiles && (unsigned)h < (unsigned)p.Ho && (unsigned)w < (unsigned)p.Wo;
      const size_t off = ok ? (((size_t)n * p.Ho + h) * p.Wo + w) * p.Cout + gq * 8 : 0;
      const uint4 v = *reinterpret_cast<const uint4*>(p.dz + off);
      pv[k] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int k = 0; k < DG_PPT; ++k)
      if (tid + 256 * k < nitems)
        *reinterpret_cast<uint4*>(patch + (ipr[k] * p.PC + (ipc[k] & 0xffff)) * p.pitch + (ipc[k] >> 16) * 16) = pv[k];
  };

  const int nph = p.sh * p.sw;                 // phases: rows 4 phase + c of the product
  const int ksteps = p.Cout / 32;
  fetch(blockIdx.x);
  for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
    const int tc = tile % p.nbc;
    const int t2 = tile / p.nbc;
    const int tr = t2 % p.nbr, n = t2 / p.nbr;
    __syncthreads();   // the previous tile's patch and staged rows have been read
    stash();
    fetch(tile + gridDim.x);
    __syncthreads();   // patch (and, first pass, the weight) visible
    // the wave's block groups: wave, wave + 4 (the lane's block: q = 16 group + col -> row ar, column bc of the tile)
    int ar[DG_NBT], bc[DG_NBT];
    bool live[DG_NBT];
    const unsigned char* bp[DG_NBT];
    f32x4s acc[DG_NBT];
#pragma unroll
    for (int t = 0; t < DG_NBT; ++t) {
      const int q = (wave + 4 * t) * 16 + col;
      live[t] = wave + 4 * t < p.nbt;
      const int a = dg_div(q, p.mTBC, p.TBC);
      ar[t] = a; bc[t] = q - a * p.TBC;
      const bool in = live[t] && a < p.TBR;
      // window origin of the block in the patch: its (u, v) = (0, 0) neighbour is patch pixel (ar + U - 1, bc + V - 1)
      bp[t] = patch + ((in ? a + p.U - 1 : p.U - 1) * p.PC + (in ? bc[t] + p.V - 1 : p.V - 1)) * p.pitch + kg * 16;
      acc[t] = f32x4s{0.f, 0.f, 0.f, 0.f};
    }
    const unsigned char* ap = wl + col * p.wpitch + kg * 16;
    auto step = [&](int u, int v, int ks, int nv, int cout2) {
      const bf16x8 fa = *reinterpret_cast<const bf16x8*>(ap + (u * nv + v) * cout2 + ks * 64);
      const int boff = -(u * p.PC + v) * p.pitch + ks * 64;
#pragma unroll
      for (int t = 0; t < DG_NBT; ++t) {
        const bf16x8 fb = *reinterpret_cast<const bf16x8*>(bp[t] + boff);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc[t], 0, 0, 0);
      }
    };
    if constexpr (UU > 0) {
#pragma unroll
      for (int u = 0; u < UU; ++u)
#pragma unroll
        for (int v = 0; v < VV; ++v)
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) step(u, v, ks, VV, KS * 64);
    } else {
      for (int u = 0; u < p.U; ++u)
        for (int v = 0; v < p.V; ++v)
          for (int ks = 0; ks < ksteps; ++ks) step(u, v, ks, p.V, p.Cout * 2);
    }
    // ---- lane (col, kg): block col of the group, product rows 4 kg .. 4 kg + 3 = phase kg, channels 0..3
#pragma unroll
    for (int t = 0; t < DG_NBT; ++t) {
      if (!live[t] || ar[t] >= p.TBR || kg >= nph) continue;
      const int prow = ar[t] * p.sh + kg / p.sw, pcol = bc[t] * p.sw + kg % p.sw;
      bf16_t* o = ost + (size_t)prow * p.orow + pcol * p.Cin;
      for (int c = 0; c < p.Cin; ++c) o[c] = from_f32<bf16_t>(acc[t][c]);
    }
    __syncthreads();   // the tile's dX pixels are staged
    const int h0 = tr * p.TBR * p.sh, w0 = tc * p.TBC * p.sw;
    const int rows = p.TBR * p.sh;
    if (p.fast_store) {
      const int cpr = p.orow * 2 / 16;                               // 16-byte pieces per staged row
      const int wbytes = p.W * p.Cin * 2, b0 = w0 * p.Cin * 2;
      for (int e = tid; e < rows * cpr; e += 256) {
        const int r = e / cpr, c = e - r * cpr;
        if (h0 + r < p.H && b0 + c * 16 + 16 <= wbytes)
          *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(p.dx) + ((size_t)n * p.H + h0 + r) * wbytes + b0 + c * 16) =
              *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(ost) + (size_t)r * p.orow * 2 + c * 16);
      }
    } else {
      for (int e = tid; e < rows * p.orow; e += 256) {
        const int r = e / p.orow, c = e - r * p.orow;
        if (h0 + r < p.H && w0 * p.Cin + c < p.W * p.Cin)
          p.dx[((size_t)n * p.H + h0 + r) * p.W * p.Cin + w0 * p.Cin + c] = ost[(size_t)r * p.orow + c];
      }
    }
  }
}

// Wt[(phase, c)][(u, v, co)] from w' as [Cin][kH][kW][Cout]: phase (qh, qw) reaches dZ row a + dh(qh) - t through
// window row i0(qh) + sh t, i.e. u = Dh - dh(qh) + t; zeros where a phase has no tap and in the rows of c >= Cin
__global__ __launch_bounds__(256) void stem_dgrad_pack_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt,
                                                              int Cin, int Cout, int kH, int kW, int sh, int sw, int ph,
                                                              int pw, int U, int V, int Dh, int Dw) {
  const int KT = U * V * Cout;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= 16 * KT) return;
  const int r = e / KT, k = e - r * KT;
  const int co = k % Cout, uv = k / Cout, v = uv % V, u = uv / V;
  const int phase = r >> 2, c = r & 3;
  float val = 0.f;
  if (phase < sh * sw && c < Cin) {
    const int qh = phase / sw, qw = phase % sw;
    const int i = (qh + ph) % sh + sh * (u - (Dh - (qh + ph) / sh));
    const int j = (qw + pw) % sw + sw * (v - (Dw - (qw + pw) / sw));
    if (u >= Dh - (qh + ph) / sh && v >= Dw - (qw + pw) / sw && i < kH && j < kW)
      val = to_f32(w[(((size_t)c * kH + i) * kW + j) * Cout + co]);
  }
  wt[e] = from_f32<bf16_t>(val);
}

struct StemDgPlan { bool ok; size_t lds; int grid; };
StemDgPlan stem_dg_plan(const Geom& g, StemDgParams* pp) {
  StemDgPlan pl{false, 0, 0};
  StemDgParams& p = *pp;
  p = StemDgParams{};
  if (g.sh > 2 || g.sw > 2 || g.Cout % 32 != 0 || g.Cout > 128) return pl;
  p.N = g.N; p.H = g.Hin; p.W = g.Win; p.Cin = g.Cin; p.Cout = g.Cout; p.Ho = g.Hout; p.Wo = g.Wout; p.sh = g.sh; p.sw = g.sw;
  // per phase q: first window row i0 = (q + pad) % s, its dZ row offset d = (q + pad) / s, taps T = ceil((k - i0) / s)
  auto span = [](int k, int s, int pad, int* D, int* U) {
    int dmax = 0;
    for (int q = 0; q < s; ++q) dmax = (q + pad) / s > dmax ? (q + pad) / s : dmax;
    int umax = 0;
    for (int q = 0; q < s; ++q) {
      const int i0 = (q + pad) % s;
      if (i0 >= k) continue;
      const int T = (k - i0 + s - 1) / s;
      const int u = dmax - (q + pad) / s + T;
      umax = u > umax ? u : umax;
    }
    *D = dmax; *U = umax;
  };
  span(g.kH, g.sh, g.ph, &p.Dh, &p.U);
  span(g.kW, g.sw, g.pw, &p.Dw, &p.V);
  if (p.U < 1 || p.V < 1) return pl;
  p.KT = p.U * p.V * g.Cout;
  p.wpitch = p.KT * 2 + 16;
  if ((size_t)16 * p.wpitch > 36 * 1024) return pl;
  p.pitch = g.Cout * 2 + 16;
  const int brows = ceil_div(g.Hin, g.sh), bcols = ceil_div(g.Win, g.sw);
  // tiles of 4 block rows x up to 32 block columns, the columns split evenly
  p.nbc = ceil_div(bcols, 32);
  p.TBC = ceil_div(bcols, p.nbc);
  p.TBR = brows < 4 ? brows : 4;
  p.nbr = ceil_div(brows, p.TBR);
  p.PR = p.TBR + p.U - 1; p.PC = p.TBC + p.V - 1;
  p.nbt = ceil_div(p.TBR * p.TBC, 16);
  if (p.nbt > 4 * DG_NBT || p.PR * p.PC * (g.Cout / 8) > 256 * DG_PPT) return pl;
  p.ntiles = g.N * p.nbr * p.nbc;
  p.orow = p.TBC * g.sw * g.Cin;
  p.fast_store = (p.orow * 2) % 16 == 0 && (g.Win * g.Cin * 2) % 16 == 0;
  p.mTBC = (unsigned)((1ull << 32) / (unsigned)p.TBC + 1);
  p.mPC = (unsigned)((1ull << 32) / (unsigned)p.PC + 1);
  pl.lds = (size_t)16 * p.wpitch + (size_t)p.PR * p.PC * p.pitch + align_up((size_t)p.TBR * g.sh * p.orow * 2, 16);
  if (pl.lds > 80 * 1024) return pl;   // two workgroups per CU
  const int per_cu = (int)(160 * 1024 / pl.lds) < 2 ? 1 : 2;
  pl.grid = p.ntiles < 256 * per_cu ? p.ntiles : 256 * per_cu;
  pl.ok = true;
  return pl;
}

bool stem_shape(const Geom& g, int dtype) {
  return dtype == CONVBN_BF16 && g.Cin <= 4 && g.kW <= 8 && g.kH <= 16 && g.Cout % 8 == 0 && g.Cout <= 128 && g.sw <= 4;
}

struct StemPlan { bool ok; bool x3; int nco; size_t lds; int grid; };
StemPlan stem_plan(const Geom& g, StemParams* pp) {
  StemPlan pl{false, false, 0, 0, 0};
  StemParams& p = *pp;
  p = StemParams{};
  p.N = g.N; p.H = g.Hin; p.W = g.Win; p.Cin = g.Cin; p.Cout = g.Cout; p.kH = g.kH; p.kW = g.kW;
  p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.Ho = g.Hout; p.Wo = g.Wout;
  p.ntw = ceil_div(g.Wout, TPX);
  p.ntiles = g.N * g.Hout * p.ntw;
  p.wpitch = g.kH * KROW * 2 + 16;
  const bool x3 = g.Cin == 3 && g.Win % 4 == 0;
  p.pcols = (TPX - 1) * g.sw + 8;
  if (x3) p.pcols = (p.pcols + 3 + 3) / 4 * 4;   // up to 3 leading pixels, whole groups of four
  p.prow = p.pcols * 8;
  pl.nco = ceil_div(g.Cout, 32);
  if (pl.nco != 1 && pl.nco != 2 && pl.nco != 4) return pl;
  if (g.kH * (p.pcols / (x3 ? 4 : 1)) > 256 * ppt(x3)) return pl;   // the patch is fetched in at most ppt() rounds
  const size_t stage = (size_t)4 * 32 * 32 * pl.nco * 2;            // the output tile is staged over the patch
  const size_t patch = (size_t)g.kH * p.prow;
  pl.lds = 512 + (size_t)32 * pl.nco * p.wpitch + (patch > stage ? patch : stage);
  if (pl.lds > 64 * 1024) return pl;   // two or more workgroups per CU hide each other's phases
  const int per_cu = (int)(160 * 1024 / pl.lds) < 4 ? (int)(160 * 1024 / pl.lds) : 4;
  pl.grid = p.ntiles < 256 * per_cu ? p.ntiles : 256 * per_cu;
  pl.x3 = x3;
  pl.ok = true;
  return pl;
}

}  // namespace

// 3-channel inputs whose rows are whole groups of four pixels, and 4-channel inputs, are read as they are; others
// need a copy widened to 4 channels ([N][H][W][4]) of this many bytes (0: none)
size_t stem_input_copy_bytes(const Geom& g) {
  return (g.Cin == 4 || (g.Cin == 3 && g.Win % 4 == 0)) ? 0 : (size_t)g.Min * 4 * 2;
}

bool stem_wgrad_supported(const Geom& g, int dtype) {
  if (!stem_shape(g, dtype)) return false;
  StemWgParams p;
  return stem_wg_plan(g, &p).ok;
}
int stem_wgrad_slices(const Geom& g) {
  StemWgParams p;
  return stem_wg_plan(g, &p).grid;
}
// x as for launch_fprop_stem; part [slices][Cout][K] and r_part [slices][Cout] (nullable): fp32 partial sums
hipError_t launch_wgrad_stem(const Geom& g, const void* x, const void* dz, float* part, float* r_part, hipStream_t st) {
  StemWgParams p;
  const StemWgPlan pl = stem_wg_plan(g, &p);
  if (!pl.ok) return hipErrorInvalidValue;
  p.x = (const bf16_t*)x; p.dz = (const bf16_t*)dz; p.part = part; p.r_part = r_part;
#define STEMWG(NC, X3V) hipLaunchKernelGGL((stem_wgrad_kernel<NC, X3V>), dim3(pl.grid), dim3(256), pl.lds, st, p)
  if (pl.x3) { if (pl.nco == 1) STEMWG(1, true); else if (pl.nco == 2) STEMWG(2, true); else STEMWG(4, true); }
  else { if (pl.nco == 1) STEMWG(1, false); else if (pl.nco == 2) STEMWG(2, false); else STEMWG(4, false); }
#undef STEMWG
  return hipGetLastError();
}

bool stem_dgrad_supported(const Geom& g, int dtype) {
  if (!stem_shape(g, dtype)) return false;
  StemDgParams p;
  return stem_dg_plan(g, &p).ok;
}
size_t stem_dgrad_weight_bytes(const Geom& g) {
  StemDgParams p;
  return stem_dg_plan(g, &p).ok ? (size_t)16 * p.KT * 2 : 0;
}
// w_crsk: w' as [Cin][kH][kW][Cout]; wpack: stem_dgrad_weight_bytes() of scratch
hipError_t launch_dgrad_stem(const Geom& g, const void* dz, const void* w_crsk, void* wpack, void* dx, hipStream_t st) {
  StemDgParams p;
  const StemDgPlan pl = stem_dg_plan(g, &p);
  if (!pl.ok) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_dgrad_pack_kernel, dim3(ceil_div(16 * p.KT, 256)), dim3(256), 0, st, (const bf16_t*)w_crsk,
                     (bf16_t*)wpack, g.Cin, g.Cout, g.kH, g.kW, g.sh, g.sw, g.ph, g.pw, p.U, p.V, p.Dh, p.Dw);
  hipError_t pe = hipGetLastError();
  if (pe != hipSuccess) return pe;
  p.dz = (const bf16_t*)dz; p.wt = (const bf16_t*)wpack; p.dx = (bf16_t*)dx;
#define STEMDG(UUV, VVV, KSV)                                                                                         \
  do {                                                                                                             \
    static LdsLimitOnce lds_once;                                                                                  \
    if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&stem_dgrad_kernel<UUV, VVV, KSV>), \
                                          80 * 1024); e != hipSuccess) return e;                                   \
    hipLaunchKernelGGL((stem_dgrad_kernel<UUV, VVV, KSV>), dim3(pl.grid), dim3(256), pl.lds, st, p);                \
  } while (0)
  if (p.U == 4 && p.V == 4 && g.Cout == 64) STEMDG(4, 4, 2);   // the usual 7x7 / stride-2 stem with 64 channels: unrolled
  else STEMDG(0, 0, 0);
#undef STEMDG
  return hipGetLastError();
}

bool stem_fprop_supported(const Geom& g, int dtype) {
  if (!stem_shape(g, dtype)) return false;
  StemParams p;
  return stem_plan(g, &p).ok;
}

size_t stem_packed_weight_bytes(const Geom& g) { return (size_t)g.Cout * g.kH * KROW * 2; }

// x: the input as it is, or its 4-channel copy where stem_input_copy_bytes() != 0; w: the (folded) weight in its own
// [Cout][kH][kW][Cin] order; wpad: stem_packed_weight_bytes() of scratch for its zero-padded copy
hipError_t launch_fprop_stem(const Geom& g, const void* x, const void* w, void* wpad, const float* bias, void* z,
                             hipStream_t st) {
  StemParams p;
  const StemPlan pl = stem_plan(g, &p);
  if (!pl.ok) return hipErrorInvalidValue;
  const int nel = g.Cout * g.kH * KROW;
  hipLaunchKernelGGL(stem_pack_weights_kernel, dim3(ceil_div(nel, 256)), dim3(256), 0, st, (const bf16_t*)w,
                     (bf16_t*)wpad, g.Cout, g.kH, g.kW, g.Cin);
  hipError_t pe = hipGetLastError();
  if (pe != hipSuccess) return pe;
  p.x = (const bf16_t*)x; p.w = (const bf16_t*)wpad; p.bias = bias; p.z = (bf16_t*)z;
#define STEM(NC, KHV, X3V)                                                                                              \
  do {                                                                                                             \
    static LdsLimitOnce lds_once;                                                                                  \
    if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&stem_fprop_kernel<NC, KHV, X3V>), \
                                          64 * 1024); e != hipSuccess) return e;                                   \
    hipLaunchKernelGGL((stem_fprop_kernel<NC, KHV, X3V>), dim3(pl.grid), dim3(256), pl.lds, st, p);                \
  } while (0)
  if (pl.nco == 2 && g.kH == 7 && pl.x3) STEM(2, 7, true);   // the usual 7x7 RGB stem with 64 channels: rows unrolled
  else if (pl.x3) { if (pl.nco == 1) STEM(1, 0, true); else if (pl.nco == 2) STEM(2, 0, true); else STEM(4, 0, true); }
  else if (pl.nco == 1) STEM(1, 0, false);
  else if (pl.nco == 2) STEM(2, 0, false);
  else STEM(4, 0, false);
#undef STEM
  return hipGetLastError();
}

}  // namespace convbn
