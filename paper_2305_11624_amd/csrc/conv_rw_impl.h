// bf16 MFMA convolution for shallow 3x3 / stride-1 layers (64 -> 64 channels, large images): the whole weight
// and the whole input window of a workgroup's pixels resident in LDS, no barrier inside the multiply loop.
//
//   forward conv   Z  = w' (*) X + b'     (Sec. 3.1 / 3.3)   act = x,  weights [Cout][taps][Cin]
//   input gradient dX = w'_rot (*) dZ     (Sec. 3.2.1)       act = dz, weights [Cin][taps][Cout], taps reversed
//
// Why a kernel of its own.  With 64 channels on both sides the weight is 72 KB and the layer is a stream of pixels:
// a hundred thousand of them, 128 bytes in and 128 bytes out each, for 4.4 us of matrix work on the whole chip.
// A workgroup that loads a tile, multiplies and stores, in lockstep with every other workgroup, pays the three phases
// one after the other, and the 12.8 MB of output reach memory only after the last multiply.  Here a workgroup (one
// per compute unit) owns L consecutive output pixels, L = M / 256 rounded up: it fetches the nine weight slabs and
// the window rows of its pixels once (about 140 KB of LDS), and after ONE barrier its eight waves run independently:
// every wave takes one or two 32-pixel subtiles (all 64 output channels: two pixel subtiles share the weight
// operands, 4 LDS reads for 4 multiplies), runs the 36 k-steps of the nine taps out of LDS with register
// double-buffering, and stores its pixels as soon as it is done -- waves finish at different times, so stores of one
// overlap the multiplies of another.
//
// Layout in LDS.  Weights: slab t (window position t) = [64 rows][64 channels] bf16, rows 128 bytes apart, the eight
// 16-byte granules of a row permuted by (row / 2) % 8.  Window: pixel p of the window (rows of Wv = Wo + 2 columns,
// zero rows / columns for the padding: copies with an out-of-range offset deliver zeros) at 128 p, granules
// permuted by p % 8.  Both permutations are chosen by the copy (a lane fetches the granule that belongs where it
// writes) and make the 128-bit operand reads of 32 consecutive rows conflict-free without a pad granule, which is
// what lets the weight and a window of more than 600 pixels fit in 160 KB together.
//
// This header holds the kernel's device code and plan (namespace convbn::rw, internal linkage) for the two
// translation units that launch it: on its own (conv_rw.hip) and side by side with the weight gradient of the same
// block in one launch (wgrad_sq.hip).
#pragma once

#include "common.h"

#include <algorithm>
#include <mutex>

namespace convbn {
namespace rw {
namespace {

struct FastDiv {   // exact n / d for 0 <= n < 2^31, without a branch: (hi(n mul) + n add) >> shr
  unsigned mul, shr, add;
  int d;
};

FastDiv make_fastdiv(int d) {
  FastDiv f{0u, 0u, 1u, d};   // d = 1: n itself
  if (d <= 1) return f;
  f.add = 0u;
  unsigned s = 0;
  while ((1ull << (s + 1)) < (unsigned long long)d) ++s;   // 2^s < d <= 2^(s+1)
  f.shr = s;
  f.mul = (unsigned)((((unsigned long long)1 << (32 + s)) + d - 1) / d);
  return f;
}

__device__ __forceinline__ int fdiv(int n, const FastDiv& f) {
  return (int)((__umulhi((unsigned)n, f.mul) + (unsigned)n * f.add) >> f.shr);
}

constexpr int CH = 64;                  // channels, both sides
constexpr int TAPS = 9;
constexpr int NWAVES = 8;
constexpr int WSLAB = CH * CH * 2;      // 8192
constexpr int OFF_W = 512;              // bias and scale first
constexpr int OFF_S = OFF_W + TAPS * WSLAB;        // 1 KB per wave where its surplus copies land
constexpr int OFF_X = OFF_S + NWAVES * 1024;       // window
constexpr int LDS_TOTAL = 160 * 1024;
constexpr int XU = 10;                  // window copies (8 pixels each) per wave
constexpr int MAX_UNITS = (LDS_TOTAL - OFF_X) / 1024;   // 79 -> at most 632 window pixels
constexpr int MAX_L = 512;              // 16 subtiles: two per wave
constexpr unsigned OOB = 0x80000000u;
static_assert(MAX_UNITS <= XU * NWAVES, "every window unit has a wave");

struct RwParams {
  const bf16_t* act;
  const bf16_t* wgt;
  const float* bias;
  BnEpilogue bn;                  // bn.gamma != null: the weight is unfolded, the epilogue applies s and b' (bias unused)
  bf16_t* out;
  int relu;                       // the output leaves as max(., 0)
  const bf16_t* mask;             // not null: laid out like out, the output is zeroed where this is <= 0
  const bf16_t* add;              // not null: laid out like out, added to the (rounded) output before the ReLU and the mask
  unsigned act_bytes, wgt_bytes;
  int N, H, W;
  int act_n_stride, act_h_stride, act_w_stride;   // elements
  int Ho, Wo, M;
  int ph, pw, Hv, Wv;
  int wt0, wt_row, wt_col;        // window position (ti, tj) reads weight tap wt0 + ti wt_row + tj wt_col
  int L;                          // output pixels per workgroup
  int lds_bytes;                  // LDS the largest workgroup touches (host side only)
  FastDiv dHoWo, dWo, dHv, dWv;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
typedef __attribute__((address_space(3))) void* lds_ptr_t;
// 1 KB copy: lane l fetches 16 bytes at byte offset voff (per lane) + soff (wave-uniform) and writes them to
// LDS at lds_wave_base + 16 l.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)voff, (int)soff, 0, 0);
  asm volatile("" ::: "memory");
}

#ifdef RW_TRACE
__device__ unsigned long long rw_trace[1024 * 64];   // [workgroup][wave][8]
#define RW_STAMP(i) do { if ((threadIdx.x & 63) == 0) rw_trace[blockIdx.x * 64 + (threadIdx.x >> 6) * 8 + (i)] = (i) == 7 ? wall_clock64() : clock64(); } while (0)
#else
#define RW_STAMP(i) do {} while (0)
#endif

// One wave's share: NP 32-pixel subtiles (sub[0], sub[1]) x 64 output channels.
template <int NP>
__device__ __forceinline__ void run_wave(const RwParams& p, unsigned char* smem, const int (&sub)[2], int m0, int len,
                                         int v_first, int lane, int wave) {
  const int kb = lane >> 5;
  const int HoWo = p.Ho * p.Wo;
  // window pixel of this lane's output pixel in each subtile (pixel 0 for pixels past the end: read, never stored)
  int wp0[NP];
#pragma unroll
  for (int ps = 0; ps < NP; ++ps) {
    const int pi = sub[ps] * 32 + (lane & 31);
    int pixidx = 0;
    if (pi < len) {
      const int m = m0 + pi;
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      const int ho = fdiv(rem, p.dWo);
      pixidx = (n * p.Hv + ho - v_first) * p.Wv + (rem - ho * p.Wo);
    }
    wp0[ps] = pixidx;
  }
  // weight rows of this lane: row l % 32 of both 32-channel subtiles (their permutation keys are equal)
  const unsigned arow = (unsigned)(OFF_W + (lane & 31) * 128);
  const unsigned am16 = (unsigned)((kb ^ (((lane & 31) >> 1) & 7)) << 4);

  f32x16 acc[2][NP];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int ps = 0; ps < NP; ++ps)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][ps][e] = 0.f;

  bf16x8 fa[2][2], fb[2][NP];
  unsigned xb[NP], xm16[NP];   // of the tap being read: byte address of the lane's window pixel, its granule key
  auto set_tap = [&](int t) {
    const int toff = (t / 3) * p.Wv + (t % 3);
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      const int wp = wp0[ps] + toff;
      xb[ps] = (unsigned)(OFF_X + wp * 128);
      xm16[ps] = (unsigned)((kb ^ (wp & 7)) << 4);
    }
  };
  // operands of k-step kk of tap t: granule 2 kk + kb of a row sits at position (2 kk + kb) ^ key
  auto load_frags = [&](int buf, int t, int kk) {
#pragma unroll
    for (int ps = 0; ps < NP; ++ps)
      fb[buf][ps] = *reinterpret_cast<const bf16x8*>(smem + xb[ps] + (xm16[ps] ^ (unsigned)(kk << 5)));
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fa[buf][i] = *reinterpret_cast<const bf16x8*>(smem + arow + t * WSLAB + i * 4096 + (am16 ^ (unsigned)(kk << 5)));
  };

  set_tap(0);
  load_frags(0, 0, 0);
#pragma unroll
  for (int s = 0; s < TAPS * 4; ++s) {
    const int cur = s & 1;
    if (s + 1 < TAPS * 4) {
      if (((s + 1) & 3) == 0) set_tap((s + 1) >> 2);
      load_frags(cur ^ 1, (s + 1) >> 2, (s + 1) & 3);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int ps = 0; ps < NP; ++ps)
        acc[i][ps] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][ps], acc[i][ps], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }

  RW_STAMP(3);
  // ---- store: bias (and scale), one rounding to bf16.  Accumulator element e of lane l in (i, ps): channel
  // 32 i + 8 (e / 4) + 4 (l / 32) + e % 4, pixel l % 32 of subtile ps -- lanes l and l + 32 hold the two halves of a
  // pixel's 8-channel granule.  Swapping the upper half of one register with the lower half of another gives every
  // lane a whole granule (lanes 0..31: granule 2 j of their pixel, lanes 32..63: granule 2 j + 1), so the stores are
  // 16 bytes per lane, 32 contiguous bytes per pixel, and need no trip through LDS.
  const float* biasl = reinterpret_cast<const float*>(smem);
#pragma unroll
  for (int ps = 0; ps < NP; ++ps) {
    const int pi = sub[ps] * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        unsigned pk[2][2];
#pragma unroll
        for (int qq = 0; qq < 2; ++qq) {
          const int q = 2 * j + qq;
          const int ch = 32 * i + 8 * q + 4 * kb;
          const float4 bb = *reinterpret_cast<const float4*>(biasl + ch);
          const float4 sc = *reinterpret_cast<const float4*>(biasl + CH + ch);
          pk[qq][0] = pack_bf16x2(fmaf(acc[i][ps][4 * q], sc.x, bb.x), fmaf(acc[i][ps][4 * q + 1], sc.y, bb.y));
          pk[qq][1] = pack_bf16x2(fmaf(acc[i][ps][4 * q + 2], sc.z, bb.z), fmaf(acc[i][ps][4 * q + 3], sc.w, bb.w));
        }
        // (a, b) -> (a of lanes 0..31 | b of lanes 0..31,  a of lanes 32..63 | b of lanes 32..63)
        const auto lo = __builtin_amdgcn_permlane32_swap(pk[0][0], pk[1][0], false, false);
        const auto hi = __builtin_amdgcn_permlane32_swap(pk[0][1], pk[1][1], false, false);
        if (pi < len) {
          const size_t o = (size_t)(m0 + pi) * CH + (4 * i + 2 * j + kb) * 8;
          *reinterpret_cast<uint4*>(p.out + o) = post_op8(make_uint4(lo[0], hi[0], lo[1], hi[1]), p.relu, p.mask, p.add, o);
        }
      }
  }
}

// The work of workgroup `block` of `nblocks`; smem: the workgroup's LDS_TOTAL bytes of LDS.
__device__ __forceinline__ void body(const RwParams& p, int block, int nblocks, unsigned char* smem) {
  const int tid = threadIdx.x, lane = tid & 63;
  RW_STAMP(0);
  RW_STAMP(7);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int HoWo = p.Ho * p.Wo;
  const int m0 = block * p.L, len = min(p.L, p.M - m0);
  const int m_last = m0 + len - 1;
  const int n_a = fdiv(m0, p.dHoWo), ho_a = fdiv(m0 - n_a * HoWo, p.dWo);
  const int n_b = fdiv(m_last, p.dHoWo), ho_b = fdiv(m_last - n_b * HoWo, p.dWo);
  const int v_first = n_a * p.Hv + ho_a;
  const int npix = (n_b * p.Hv + ho_b + 3 - v_first) * p.Wv;
  const int nunits = (npix + 7) >> 3;   // <= MAX_UNITS: checked by the host for every workgroup

  const __amdgpu_buffer_rsrc_t act_rsrc = make_rsrc(p.act, p.act_bytes);
  const __amdgpu_buffer_rsrc_t wgt_rsrc = make_rsrc(p.wgt, p.wgt_bytes);

  // weights: slab t, rows 8 wave .. 8 wave + 7 (a lane fetches the granule that belongs at its position)
  {
    const int row = wave * 8 + (lane >> 3);
    const int g = (lane & 7) ^ ((row >> 1) & 7);
    const unsigned voff = (unsigned)((row * (TAPS * CH) + g * 8) * 2);
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
      const int tap = p.wt0 + (t / 3) * p.wt_row + (t % 3) * p.wt_col;
      dma16(wgt_rsrc, voff, (unsigned)(tap * CH * 2), smem + OFF_W + t * WSLAB + wave * 1024);
    }
  }
  // window: unit u = wave + 8 k holds window pixels 8 u .. 8 u + 7; units past the window go to a spare KB of this
  // wave, so that every wave issues the same number of copies
  {
    const int g = (lane & 7) ^ ((lane >> 3) & 7);
#pragma unroll
    for (int k = 0; k < XU; ++k) {
      const int u = wave + NWAVES * k;
      const int pix = u * 8 + (lane >> 3);
      const int slot = fdiv(pix, p.dWv);
      const int w = pix - slot * p.Wv - p.pw;
      const int v = v_first + slot;
      const int n = fdiv(v, p.dHv);
      const int h = v - n * p.Hv - p.ph;
      const bool ok = pix < npix && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W && n < p.N;
      const unsigned voff = ok ? (unsigned)((n * p.act_n_stride + h * p.act_h_stride + w * p.act_w_stride + g * 8) * 2) : OOB;
      dma16(act_rsrc, voff, 0u, u < nunits ? smem + OFF_X + u * 1024 : smem + OFF_S + wave * 1024);
    }
  }

  // bias and scale of the epilogue: Z = s (w (*) X) + b' with s and b' worked out here (Sec. 3.3) when the weight
  // is unfolded
  if (tid < CH) {
    float bias_v = p.bias ? p.bias[tid] : 0.f, scale_v = 1.f;
    if (p.bn.gamma) {
      scale_v = p.bn.gamma[tid] / sqrtf(p.bn.var[tid] + p.bn.eps);
      bias_v = ((p.bn.b ? p.bn.b[tid] : 0.f) - p.bn.mean[tid]) * scale_v + p.bn.beta[tid];
    }
    float* biasl = reinterpret_cast<float*>(smem);
    biasl[tid] = bias_v;
    biasl[CH + tid] = scale_v;
  }
  if (p.bn.gamma && p.bn.w_folded_out) emit_folded_slice(p.bn, p.wgt, block, nblocks);   // while the copies are in flight
  RW_STAMP(1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();   // the one barrier: weights, window, bias and scale are in place for every wave

  // subtiles: with nsub <= 8 wave w takes subtile w; otherwise the first nsub - 8 waves take two each
  RW_STAMP(2);
  const int nsub = (len + 31) >> 5;   // <= 16
  const int extra = nsub > NWAVES ? nsub - NWAVES : 0;
  if (wave < extra) {
    const int sub[2] = {2 * wave, 2 * wave + 1};
    run_wave<2>(p, smem, sub, m0, len, v_first, lane, wave);
  } else {
    const int s = extra + wave;
    if (s < nsub) {
      const int sub[2] = {s, s};
      run_wave<1>(p, smem, sub, m0, len, v_first, lane, wave);
    }
  }
  RW_STAMP(4);
}

// Window pixels workgroup b needs.
int window_pixels(const RwParams& p, int b) {
  const int HoWo = p.Ho * p.Wo;
  const int m0 = b * p.L;
  const int ml = (m0 + p.L < p.M ? m0 + p.L : p.M) - 1;
  const int na = m0 / HoWo, hoa = (m0 - na * HoWo) / p.Wo;
  const int nb = ml / HoWo, hob = (ml - nb * HoWo) / p.Wo;
  return (nb * p.Hv + hob + 3 - (na * p.Hv + hoa)) * p.Wv;
}

// Completes the plan of a problem whose tensors are described in p; false = this kernel does not take it.
bool finish_plan(RwParams& p, int kH, int kW, int C, int R) {
  if (kH != 3 || kW != 3 || C != CH || R != CH) return false;
  if (p.act_bytes >= OOB || p.wgt_bytes >= OOB) return false;
  if (p.M < 64 * 256) return false;   // a stream of pixels long enough to give every compute unit two subtiles
  p.Hv = p.Ho + 2;
  p.Wv = p.Wo + 2;
  // one workgroup per compute unit if its pixels' window fits, else two, three, ... rounds.  The search walks over
  // every workgroup's window; a caller asks for the same problem several times per launch, so the last answer is kept.
  static thread_local struct { int M, Ho, Wo, L, units; } memo = {0, 0, 0, 0, 0};
  if (memo.M != p.M || memo.Ho != p.Ho || memo.Wo != p.Wo) {
    int found = 0, units = 0;
    for (int rounds = 1; rounds <= 8 && !found; ++rounds) {
      p.L = ceil_div(p.M, 256 * rounds);
      if (p.L > MAX_L) continue;
      const int nwg = ceil_div(p.M, p.L);
      int widest = 0;
      for (int b = 0; b < nwg && widest <= MAX_UNITS * 8; ++b) widest = std::max(widest, window_pixels(p, b));
      if (widest <= MAX_UNITS * 8) { found = p.L; units = (widest + 7) / 8; }
    }
    memo = {p.M, p.Ho, p.Wo, found, units};
  }
  if (!memo.L) return false;
  p.L = memo.L;
  p.lds_bytes = OFF_X + memo.units * 1024;
  p.dHoWo = make_fastdiv(p.Ho * p.Wo);
  p.dWo = make_fastdiv(p.Wo);
  p.dHv = make_fastdiv(p.Hv);
  p.dWv = make_fastdiv(p.Wv);
  return true;
}

bool fprop_params(const Geom& g, RwParams* p) {
  RwParams& q = *p;
  q = RwParams{};
  if (g.sh != 1 || g.sw != 1) return false;
  q.N = g.N; q.H = g.Hin; q.W = g.Win; q.Ho = g.Hout; q.Wo = g.Wout; q.M = g.M;
  q.ph = g.ph; q.pw = g.pw;
  q.wt0 = 0; q.wt_row = g.kW; q.wt_col = 1;
  q.act_n_stride = g.Hin * g.Win * g.Cin; q.act_h_stride = g.Win * g.Cin; q.act_w_stride = g.Cin;
  if ((size_t)g.Min * g.Cin * 2 >= OOB || (size_t)g.Cout * g.K * 2 >= OOB) return false;
  q.act_bytes = (unsigned)((size_t)g.Min * g.Cin * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  return finish_plan(q, g.kH, g.kW, g.Cin, g.Cout);
}

bool dgrad_params(const Geom& g, RwParams* p) {
  RwParams& q = *p;
  q = RwParams{};
  if (g.sh != 1 || g.sw != 1) return false;
  if (g.ph > g.kH - 1 || g.pw > g.kW - 1) return false;
  q.N = g.N; q.H = g.Hout; q.W = g.Wout; q.Ho = g.Hin; q.Wo = g.Win; q.M = g.Min;
  q.ph = g.kH - 1 - g.ph; q.pw = g.kW - 1 - g.pw;
  q.wt0 = g.kH * g.kW - 1; q.wt_row = -g.kW; q.wt_col = -1;   // rotated kernel
  q.act_n_stride = g.Hout * g.Wout * g.Cout; q.act_h_stride = g.Wout * g.Cout; q.act_w_stride = g.Cout;
  if ((size_t)g.M * g.Cout * 2 >= OOB || (size_t)g.Cout * g.K * 2 >= OOB) return false;
  q.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  return finish_plan(q, g.kH, g.kW, g.Cout, g.Cin);
}

}  // namespace
}  // namespace rw
}  // namespace convbn
