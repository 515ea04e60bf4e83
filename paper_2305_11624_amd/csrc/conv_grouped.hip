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

// ---- bf16 MFMA kernels for groups of 4, 8, 16 or 32 channels (cg == og) ----------------------------------
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
//     in its other order.
constexpr int GC_PPT = 16;                 // most 16-byte patch items a thread fetches per tile
constexpr size_t GC_PATCH_MAX = 52 * 1024; // patch bytes (+ 10 KB of output staging: two workgroups per CU)

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
};

template <int TAPS>
__global__ __launch_bounds__(256) void g_conv_mfma_kernel(GcParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kb = lane >> 5, px = lane & 31;
  const int cgrp = blockIdx.x % p.ncg, worker = blockIdx.x / p.ncg;
  const int cl = wave % p.nch;                      // this wave's chunk inside the workgroup's channels
  const int chunk = cgrp * p.nch + cl;              // ... and in the tensor
  const int wstep = 4 / p.nch, wfirst = wave / p.nch;
  unsigned char* patch = smem;
  unsigned char* stage = smem + (size_t)p.PR * p.PC * p.pitch + wave * (32 * 80);   // [32 pixels][64 + 16 bytes]

  // ---- weight fragments: row = lane % 32 (output channel; mode 1: input channel), 8 consecutive reduced channels
  bf16x8 wf[TAPS][2];
  {
    const int row = px, rgrp = row / p.cg;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int k0 = ks * 16 + kb * 8;             // first of the 8 reduced channels (local)
        const bool lo = k0 / p.cg == rgrp, hi = (k0 + 4) / p.cg == rgrp;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (p.mode == 0) {
          const bf16_t* wr = p.w + ((size_t)(chunk * 32 + row) * TAPS + t) * p.cg;
          if (p.cg == 4) {
            if (lo || hi) {
              const uint2 r = *reinterpret_cast<const uint2*>(wr);
              if (lo) { v.x = r.x; v.y = r.y; } else { v.z = r.x; v.w = r.y; }
            }
          } else if (lo) {
            v = *reinterpret_cast<const uint4*>(wr + (k0 % p.cg));
          }
        } else if (lo || hi) {
          const int tf = TAPS - 1 - t;
          v = *reinterpret_cast<const uint4*>(p.w + ((size_t)(row % p.cg) * TAPS + tf) * p.C + chunk * 32 + k0);
          if (!lo) { v.x = 0u; v.y = 0u; }
          if (!hi) { v.z = 0u; v.w = 0u; }
        }
        wf[t][ks] = __builtin_bit_cast(bf16x8, v);
      }
  }
  // bias of the lane's 16 accumulator channels 8 (e / 4) + 4 kb + e % 4
  float bv[16];
#pragma unroll
  for (int e = 0; e < 16; ++e)
    bv[e] = p.bias ? p.bias[chunk * 32 + 8 * (e >> 2) + 4 * kb + (e & 3)] : 0.f;

  // ---- patch items of this thread (the same for every tile): 16-byte granule gq of patch pixel (row pr, column pc)
  const int gpp = p.nch * 4;                        // granules per patch pixel
  const int nitems = p.PR * p.PC * gpp;
  int ipr[GC_PPT], ipc[GC_PPT];
#pragma unroll
  for (int k = 0; k < GC_PPT; ++k) {
    const int e = tid + 256 * k;
    const int pix = e / gpp;
    ipr[k] = pix / p.PC;
    ipc[k] = (pix - ipr[k] * p.PC) | ((e - pix * gpp) << 16);
  }
  uint4 pv[GC_PPT];
  auto fetch = [&](int tile) {
    const int tc = tile % p.ntc;
    const int t2 = tile / p.ntc;
    const int tr = t2 % p.ntr, n = t2 / p.ntr;
    const int h0 = tr * p.TR * p.sh - p.ph, w0 = tc * p.TC * p.sw - p.pw;
#pragma unroll
    for (int k = 0; k < GC_PPT; ++k) {
      const int h = h0 + ipr[k], w = w0 + (ipc[k] & 0xffff), gq = ipc[k] >> 16;
      pv[k] = make_uint4(0u, 0u, 0u, 0u);
      if (tid + 256 * k < nitems && tile < p.ntiles && (unsigned)h < (unsigned)p.Hi && (unsigned)w < (unsigned)p.Wi)
        pv[k] = *reinterpret_cast<const uint4*>(p.in + (((size_t)n * p.Hi + h) * p.Wi + w) * p.C + cgrp * p.nch * 32 + gq * 8);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int k = 0; k < GC_PPT; ++k)
      if (tid + 256 * k < nitems)
        *reinterpret_cast<uint4*>(patch + (ipr[k] * p.PC + (ipc[k] & 0xffff)) * p.pitch + (ipc[k] >> 16) * 16) = pv[k];
  };

  fetch(worker);
  for (int tile = worker; tile < p.ntiles; tile += p.nworkers) {
    const int tc = tile % p.ntc;
    const int t2 = tile / p.ntc;
    const int tr = t2 % p.ntr, n = t2 / p.ntr;
    const int r0 = tr * p.TR, c0 = tc * p.TC;
    const int rows = min(p.TR, p.Ho - r0), cols = min(p.TC, p.Wo - c0);
    __syncthreads();   // every wave is done with the previous patch
    stash();
    fetch(tile + p.nworkers);
    __syncthreads();   // patch visible
    for (int wt = wfirst; wt < p.nwt; wt += wstep) {
      if ((wt * 32) / p.TC >= rows) break;            // nothing but rows past the image in this and later groups
      const int pl = wt * 32 + px;
      int r = pl / p.TC, c = pl - r * p.TC;
      if (r >= rows || c >= cols) { r = 0; c = 0; }   // computed and dropped
      const unsigned char* b0 = patch + ((r * p.sh) * p.PC + c * p.sw) * p.pitch + cl * 64 + kb * 16;
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = bv[e];
#pragma unroll
      for (int t = 0; t < TAPS; ++t) {
        const int i = t / p.kW, j = t - i * p.kW;
        const unsigned char* bp = b0 + (i * p.PC + j) * p.pitch;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
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
        const int r2 = p2 / p.TC, c2 = p2 - r2 * p.TC;
        if (r2 < rows && c2 < cols)
          *reinterpret_cast<uint4*>(p.out + (((size_t)n * p.Ho + r0 + r2) * p.Wo + c0 + c2) * p.C + chunk * 32 + gq * 8) = v;
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
  if (C % 32 != 0 || (cg != 4 && cg != 8 && cg != 16 && cg != 32)) return pl;
  const int taps = kH * kW;
  if (taps != 1 && taps != 9) return pl;
  p.N = N; p.Hi = in_h; p.Wi = in_w; p.C = C; p.Ho = out_h; p.Wo = out_w; p.kH = kH; p.kW = kW;
  p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.cg = cg;
  p.ntc = ceil_div(out_w, 64);
  p.TC = ceil_div(out_w, p.ntc);
  p.PC = (p.TC - 1) * sw + kW;
  const int nchunks = C / 32;
  double best = 0;
  for (int nch = 1; nch <= 4; nch *= 2) {
    if (nchunks % nch != 0) continue;
    const int pitch = 64 * nch + 16;
    for (int TR = 1; TR <= out_h; ++TR) {
      const int PR = (TR - 1) * sh + kH;
      if ((size_t)PR * p.PC * pitch > GC_PATCH_MAX || PR * p.PC * nch * 4 > 256 * GC_PPT) break;
      const int ntr = ceil_div(out_h, TR);
      if (ceil_div(out_h, ntr) != TR) continue;         // an evenly split height only
      const int per_round = 4 / nch;
      auto rounds = [&](int rows) { return ceil_div(ceil_div(rows * p.TC, 32), per_round); };
      const int last = out_h - (ntr - 1) * TR;
      const double work = ((double)(ntr - 1) * rounds(TR) + rounds(last)) * (nchunks / nch);   // wave rounds per image column
      const double fetched = (double)ntr * PR / ((double)out_h * sh);                          // rows fetched / rows there are
      const double score = 1.0 / (work * (1.0 + 0.3 * (fetched - 1.0)));
      if (score > best) {
        best = score;
        p.nch = nch; p.TR = TR; p.ntr = ntr; p.PR = PR; p.pitch = pitch;
      }
    }
  }
  if (best == 0) return pl;
  p.nwt = ceil_div(p.TR * p.TC, 32);
  p.ntiles = N * p.ntr * p.ntc;
  p.ncg = nchunks / p.nch;
  pl.lds = (size_t)p.PR * p.PC * p.pitch + 4 * 32 * 80;
  const int per_cu = pl.lds > 80 * 1024 ? 1 : pl.lds > 52 * 1024 ? 2 : 3;
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
  p->mode = 1;
  return pl;
}

hipError_t gc_launch(const GcPlan& pl, const GcParams& p, hipStream_t st) {
  if (p.kH * p.kW == 9) hipLaunchKernelGGL(g_conv_mfma_kernel<9>, dim3(pl.grid), dim3(256), pl.lds, st, p);
  else hipLaunchKernelGGL(g_conv_mfma_kernel<1>, dim3(pl.grid), dim3(256), pl.lds, st, p);
  return hipGetLastError();
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
