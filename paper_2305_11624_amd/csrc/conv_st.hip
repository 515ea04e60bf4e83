// bf16 MFMA convolution for deep 3x3 / stride-1 layers (many channels, few pixels) without split sums:
// workgroup tiles of 128 pixels x 64 channels (or 64 x 128) shared by EIGHT waves.
//
//   forward conv   Z  = w' (*) X + b'     (Sec. 3.1 / 3.3)   act = x,  weights [Cout][taps][Cin]
//   input gradient dX = w'_rot (*) dZ     (Sec. 3.2.1)       act = dz, weights [Cin][taps][Cout], taps reversed
//
// Why these shapes.  With a few thousand pixels and 512 channels the output has only about as many 8192-element
// tiles as the chip has compute units, so a tile cannot be larger without splitting the reduction over workgroups
// -- and the fp32 partial sums of such a split were measured to cost more than the larger tile saves.  At this
// size the kernel is bound by how fast a compute unit can pull the folded weight out of the L2 (a 64-channel step
// is 256 cycles of matrix work).  That rate depends on how many waves issue the copies: four waves sustain about
// 30 bytes per clock, eight about 50.  So the tile is shared by eight waves instead of four: every wave issues a
// share of the copies, and the matrix pipe of a SIMD is fed by two waves.  The eight waves are 2 pixel groups
// (half the tile's pixels) x 4 quarters of the reduction: a wave multiplies one of the four 16-channel k-steps of
// every step for all the tile's channels (4 accumulator tiles; 128 x 64: 2 pixel x 2 channel subtiles, 4 operand
// reads for 4 multiplies; 64 x 128: 1 x 4, 5 reads -- with one 32 x 32 tile per wave it would be 2 reads per
// multiply, and the LDS, which serves about one wave-wide read per 5 clocks whatever its width, would be the
// bound), and the four waves of a pixel group add their sums through LDS at the end.  128 x 64 is preferred where
// its window fits: half the weight bytes per step, and a ring deep enough for one barrier per kernel row.
//
// Layout in LDS.  Activations: the window rows the tile's pixels touch, [slot][column][64 channels] with zero
// rows / columns for the padding (out-of-image pixels are copies with an out-of-range buffer offset: zeros),
// rows 144 bytes apart (128 + one pad granule: 16 consecutive rows of a 128-bit operand read fall on distinct
// banks, and a tap is a wave-uniform offset on a per-lane base).  All nine taps of a chunk read the same tile.
// Weights: one [rows][64 channels] slab per (chunk, tap) step in a ring, rows 128 bytes apart with the eight
// granules of a row permuted by (row / 2) % 8 -- chosen by the copy, which picks the granule each lane fetches
// -- so that a slab is exactly eight or sixteen 1 KB copies, one or two per wave and step.
//
// Pipeline.  A step = one tap of one 64-channel chunk = 4 MFMAs per wave; the taps are unrolled; during step s a
// wave issues its share of the slab of step s + DIST and, in the first taps of a chunk, units of the next chunk's
// window tile; operands of step s + 1 are read while step s multiplies.  Barriers open groups of G steps; the
// constants and what they must satisfy are stated at the tile shapes below.
#include "common.h"

#include <mutex>

namespace convbn {

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

constexpr int CB = 64;                  // reduced channels per chunk
constexpr int KK = CB / 16;             // k-steps per step
constexpr int NWAVES = 8;
constexpr int HROW = 144;               // window-tile row pitch: 128 bytes of channels + one pad granule
constexpr int HRPU = 7;                 // whole rows per 1 KB copy (its last lane spills into the next row)
constexpr int HUNIT = HRPU * HROW;      // 1008
constexpr int OFF_W = 1024;             // bias and scale first
constexpr int RED_BYTES = 2 * 4 * 16 * 64 * 16;   // the final reduction: eight waves' accumulators
constexpr unsigned OOB = 0x80000000u;

// The two tile shapes.  Both give a wave four accumulator tiles (a pixel group is half the tile's pixels):
//   64 pixels x 128 channels: 1 pixel x 4 channel subtiles per wave, 16 KB of weights per step, small windows;
//  128 pixels x  64 channels: 2 x 2 subtiles (4 operand reads per 4 multiplies instead of 5), 8 KB of weights per
//                             step and a window tile about twice as large -- fewer bytes per step in all.
//  128 x 64 with a taller window: six window copies per wave (336 window pixels: 128-pixel tiles of 28 x 28 images that
//                             cross an image boundary need up to 300) paid for with a ring of seven slabs
template <int TP_, int TRC_, int HUW_ = 0, int NBUF_ = 0>
struct Shape {
  static constexpr int TP = TP_;                  // output pixels per workgroup
  static constexpr int TRC = TRC_;                // output channels per workgroup
  static constexpr int NPS = TP / 64;             // 32-pixel subtiles per wave
  static constexpr int NCS = TRC / 32;            // 32-channel subtiles per wave
  static constexpr int WPW = TRC / 64;            // weight copies (8 rows each) per wave and step
  static constexpr int HUW = HUW_ ? HUW_ : (TP == 64 ? 3 : 5);    // window-tile copies per wave and chunk
  static constexpr int HUNITS = NWAVES * HUW;     // 24 / 40 -> at most 168 / 280 window pixels per tile
  static constexpr int HBUF = HUNITS * HUNIT + 64;
  static constexpr int WSLAB = TRC * CB * 2;      // 16384 / 8192
  // Steps between workgroup barriers, depth of the weight ring, and how many steps before its own a slab is
  // fetched (L2 latency is several steps long).  A barrier costs about as much as the four multiplies of a step,
  // so the 128 x 64 shape, whose slabs are half as large, spends the LDS it saves on a ring deep enough for one
  // barrier per kernel row: G = 3.  What the schedule needs: at the barrier that opens a group the slabs of its G
  // steps and of the step after are resident (a step reads the operands of the next one), i.e. at most the copies
  // of the DIST - G - 1 latest steps are in flight; a slab's slot was last read in an earlier group:
  // DIST <= NBUF - G + 1; the next chunk's window tile is fetched in the first TAPS + 1 - DIST taps of a chunk.
  static constexpr int G = TP == 64 ? 1 : 3;
  static constexpr int NBUF = NBUF_ ? NBUF_ : (TP == 64 ? 6 : 9);
  static constexpr int DIST = NBUF - G + 1;
  static constexpr int OFF_H = OFF_W + NBUF * WSLAB;
  static constexpr int LDS_BYTES = (OFF_H + 2 * HBUF) > (OFF_W + RED_BYTES) ? (OFF_H + 2 * HBUF) : (OFF_W + RED_BYTES);
  static_assert(NPS * NCS == 4 && TRC <= 128, "four accumulator tiles per wave");
};

struct StParams {
  const bf16_t* act;
  const bf16_t* wgt;
  const float* bias;
  BnEpilogue bn;                  // bn.gamma != null: the weight is unfolded, the epilogue applies s and b' (bias unused)
  bf16_t* out;
  int relu;                       // the output leaves as max(., 0)
  const bf16_t* mask;             // not null: laid out like out, the output is zeroed where this is <= 0
  const bf16_t* add;              // not null: laid out like out, added to the (rounded) output before the ReLU and the mask
  unsigned act_bytes, wgt_bytes;
  int N, H, W, C;
  int act_n_stride, act_h_stride, act_w_stride;   // elements
  int Ho, Wo, R, M;
  int ph, pw, Hv, Wv;
  int wrow;                       // elements per weight row (taps x C)
  int wt0, wt_row, wt_col;        // window position (ti, tj) reads weight tap wt0 + ti wt_row + tj wt_col
  int ntr;                        // channel tiles
  int nchunks;
  int wide;                       // tile shape: 0 = 64 pixels x 128 channels, 1 = 128 x 64, 2 = 128 x 64 with the taller window
  FastDiv dHoWo, dWo, dHv, dWv;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
typedef __attribute__((address_space(3))) void* lds_ptr_t;
// 1 KB copy: lane l fetches 16 bytes at byte offset voff (per lane) + soff (wave-uniform) and writes them to
// LDS at lds_wave_base + 16 l.  The compiler barrier keeps every copy in the stream: the waits count copies.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)voff, (int)soff, 0, 0);
  asm volatile("" ::: "memory");
}
// Workgroup barrier without the memory fence of __syncthreads() (which would drain every outstanding copy).
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
template <int N> __device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// n is a constant once the taps are unrolled: one wait survives
__device__ __forceinline__ void wait_vm_upto(int n) {
  switch (n) {
    case 0: wait_vm<0>(); break; case 1: wait_vm<1>(); break; case 2: wait_vm<2>(); break; case 3: wait_vm<3>(); break;
    case 4: wait_vm<4>(); break; case 5: wait_vm<5>(); break; case 6: wait_vm<6>(); break; case 7: wait_vm<7>(); break;
    case 8: wait_vm<8>(); break; case 9: wait_vm<9>(); break; case 10: wait_vm<10>(); break; case 11: wait_vm<11>(); break;
    case 12: wait_vm<12>(); break; case 13: wait_vm<13>(); break; case 14: wait_vm<14>(); break;
    default: wait_vm<0>(); break;
  }
}

#ifdef ST_TRACE
__device__ unsigned long long st_trace[1024 * 128];
#ifndef ST_TRACE_WAVE
#define ST_TRACE_WAVE 0
#endif
#define STAMP(i) do { if (tid == 64 * ST_TRACE_WAVE && (i) < 128) st_trace[blockIdx.x * 128 + (i)] = clock64(); } while (0)
#else
#define STAMP(i) do {} while (0)
#endif

template <int KH, int KW, class S>
__global__ __launch_bounds__(64 * NWAVES) void conv_st_kernel(StParams p) {
  constexpr int TAPS = KH * KW;
  constexpr int TP = S::TP, TRC = S::TRC, NPS = S::NPS, NCS = S::NCS, WPW = S::WPW, HUW = S::HUW, HBUF = S::HBUF,
                WSLAB = S::WSLAB, OFF_H = S::OFF_H, G = S::G, NBUF = S::NBUF, DIST = S::DIST;
  constexpr int HTAPS = TAPS + 1 - DIST;           // taps of a chunk in which the next window tile is fetched
  constexpr int HPT = (HUW + HTAPS - 1) / HTAPS;   // window units per such tap (the last may get fewer)
  static_assert(TAPS % G == 0 && HTAPS >= 1 && DIST - G - 1 >= 1, "copy schedule");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* biasl = reinterpret_cast<float*>(smem);
  unsigned char* wbuf = smem + OFF_W;
  unsigned char* halo = smem + OFF_H;

  const int tid = threadIdx.x, lane = tid & 63;
  STAMP(0);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wpx = wave & 1, kq = wave >> 1;   // pixel group (half the tile), and which k-step of every step this wave multiplies
  const int ctile = blockIdx.x % p.ntr, ptile = blockIdx.x / p.ntr;
  const int r0 = ctile * TRC;
  const int HoWo = p.Ho * p.Wo;
  const int m0 = ptile * TP, len = min(TP, p.M - m0);
  const int m_last = m0 + len - 1;
  const int n_a = fdiv(m0, p.dHoWo), ho_a = fdiv(m0 - n_a * HoWo, p.dWo);
  const int n_b = fdiv(m_last, p.dHoWo), ho_b = fdiv(m_last - n_b * HoWo, p.dWo);
  const int v_first = n_a * p.Hv + ho_a;
  const int npix = (n_b * p.Hv + ho_b + KH - v_first) * p.Wv;

  const __amdgpu_buffer_rsrc_t act_rsrc = make_rsrc(p.act, p.act_bytes);
  const __amdgpu_buffer_rsrc_t wgt_rsrc = make_rsrc(p.wgt, p.wgt_bytes);
  const int nchunks = p.nchunks;

  float bias_v = (tid < TRC && p.bias) ? p.bias[r0 + tid] : 0.f;
  float scale_v = 1.f;
  if (p.bn.gamma && tid < TRC) {   // Z = s (w (*) X) + b' with s and b' worked out here (Sec. 3.3), no folded weight
    const int ch = r0 + tid;
    scale_v = p.bn.gamma[ch] / sqrtf(p.bn.var[ch] + p.bn.eps);
    bias_v = ((p.bn.b ? p.bn.b[ch] : 0.f) - p.bn.mean[ch]) * scale_v + p.bn.beta[ch];
  }

  // window-tile copies of this wave: unit wave + 8 t, t = 0..3; per-lane byte offsets without the chunk
  unsigned hv[HUW];
  {
    const int lrow = lane == 63 ? 7 : lane / 9;       // lane 63: granule 0 of the next unit's first row
    const int lgran = lane == 63 ? 0 : lane - lrow * 9;
#pragma unroll
    for (int t = 0; t < HUW; ++t) {
      const int pix = (wave + NWAVES * t) * HRPU + lrow;
      const int slot = fdiv(pix, p.dWv);
      const int w = pix - slot * p.Wv - p.pw;
      const int v = v_first + slot;
      const int n = fdiv(v, p.dHv);
      const int h = v - n * p.Hv - p.ph;
      const bool ok = pix < npix && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W && n < p.N && lgran < 8;
      hv[t] = ok ? (unsigned)((n * p.act_n_stride + h * p.act_h_stride + w * p.act_w_stride + lgran * 8) * 2) : OOB;
    }
  }
  // weight copies of this wave: units WPW wave .. of the slab (8 rows each), granules permuted by (row / 2) % 8
  unsigned voff_w[WPW];
#pragma unroll
  for (int j = 0; j < WPW; ++j) {
    const int row = (WPW * wave + j) * 8 + (lane >> 3);
    const int g = (lane & 7) ^ ((row >> 1) & 7);
    voff_w[j] = (unsigned)(((r0 + row) * p.wrow + g * 8) * 2);
  }
  // byte offset of window position t inside the window tile, and of its weights inside a weight row
  int toff[TAPS], wsoff[TAPS];
#pragma unroll
  for (int t = 0; t < TAPS; ++t) {
    const int ti = t / KW, tj = t % KW;
    toff[t] = (ti * p.Wv + tj) * HROW;
    wsoff[t] = (p.wt0 + ti * p.wt_row + tj * p.wt_col) * p.C * 2;
  }

  // LDS byte offsets of this lane's operands
  const int kb = lane >> 5;
  unsigned boff[NPS];
#pragma unroll
  for (int ps = 0; ps < NPS; ++ps) {
    const int pi = wpx * (TP / 2) + ps * 32 + (lane & 31);
    int pixidx = 0;
    if (pi < len) {
      const int m = m0 + pi;
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      const int ho = fdiv(rem, p.dWo);
      pixidx = (n * p.Hv + ho - v_first) * p.Wv + (rem - ho * p.Wo);
    }
    boff[ps] = (unsigned)(pixidx * HROW + kb * 16);
  }
  // weight rows of this lane (row l % 32 of each 32-channel subtile): granule 2 kq + kb sits at
  // position (2 kq + kb) ^ key, key = (row / 2) % 8 -- the same for all its rows, which are 32 apart
  unsigned aoff;
  {
    const int row = lane & 31;
    const int key = (row >> 1) & 7;
    aoff = (unsigned)(row * 128 + ((((2 * kq + kb) ^ key) & 7) << 4));
  }

  // Element offset of the 8 channels this lane stores in epilogue iteration it (wave kq finishes subtile kq: channel
  // subtile kq / NPS, pixel subtile kq % NPS of its pixel group); -1 past the last pixel.
  auto store_off = [&](int it) -> long long {
    const int row = it * 16 + (lane >> 2);
    const int g = (lane & 3) ^ ((row >> 1) & 3);
    const int pi = wpx * (TP / 2) + (kq % NPS) * 32 + row;
    return pi < len ? (long long)((size_t)(m0 + pi) * p.R + r0 + (kq / NPS) * 32 + g * 8) : -1;
  };
  f32x16 acc[4];   // subtile (channel i, pixel ps) at i * NPS + ps
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

  auto issue_weights = [&](int chunk, int t, int slot) {
    const unsigned soff = (unsigned)(wsoff[t] + chunk * (CB * 2));
#pragma unroll
    for (int j = 0; j < WPW; ++j) dma16(wgt_rsrc, voff_w[j], soff, wbuf + slot * WSLAB + (WPW * wave + j) * 1024);
  };
  auto issue_halo = [&](int chunk, int t, int hb) {
    dma16(act_rsrc, hv[t], (unsigned)(chunk * (CB * 2)), halo + hb * HBUF + (wave + NWAVES * t) * HUNIT);
  };

  // window units fetched in tap t of a chunk
  auto halo_units = [&](int t) { return t < HTAPS ? (HUW - t * HPT < HPT ? (HUW - t * HPT > 0 ? HUW - t * HPT : 0) : HPT) : 0; };

  // ---- prologue: the first chunk's window tile and the slabs of steps 0 .. DIST-1 ---------------------
#pragma unroll
  for (int t = 0; t < HUW; ++t) issue_halo(0, t, 0);
#pragma unroll
  for (int s = 0; s < DIST; ++s) issue_weights(0, s, s);

  bf16x8 fa[2][NCS], fb[2][NPS];
  // operands of this wave's k-step of a step: weights from ring slot `slot`, pixels from window tile `hb` at tap offset `to`
  auto load_frags = [&](int buf, int slot, int hb, int to) {
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps)
      fb[buf][ps] = *reinterpret_cast<const bf16x8*>(halo + hb * HBUF + to + kq * 32 + boff[ps]);
#pragma unroll
    for (int i = 0; i < NCS; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(wbuf + slot * WSLAB + aoff + i * 4096);
  };

  if (p.bn.gamma && p.bn.w_folded_out) emit_folded_slice(p.bn, p.wgt, blockIdx.x, gridDim.x);   // while the first copies are in flight
  STAMP(1);
  wait_vm_upto((DIST - G - 1) * WPW);   // as at every later group: the latest DIST - G - 1 slabs may still be on their way
  block_barrier();
  STAMP(2);
  load_frags(0, 0, 0, toff[0]);

  int slot = 0;   // ring slot of the current step
  for (int c = 0; c < nchunks; ++c) {
    const int hb = c & 1;
    const int cnext = min(c + 1, nchunks - 1);   // past the end: the last chunk again (nobody reads it)
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
      // a group opens: the copies that may still be in flight are those of the DIST - G - 1 previous steps (WPW
      // weight units each, + the window units of those taps)
      if (t % G == 0) {
        int inflight = 0;
#pragma unroll
        for (int d = 1; d <= DIST - G - 1; ++d) inflight += WPW + halo_units((t - d + TAPS) % TAPS);
        STAMP(4 + 3 * (c * TAPS + t));
        wait_vm_upto(inflight);
        STAMP(5 + 3 * (c * TAPS + t));
        block_barrier();
        STAMP(6 + 3 * (c * TAPS + t));
      }
      const int t3 = (t + DIST) % TAPS;
      const int c3 = (t + DIST) >= TAPS ? cnext : c;
      const int slot_n = slot + 1 == NBUF ? 0 : slot + 1;
      const int slot_f = slot + DIST >= NBUF ? slot + DIST - NBUF : slot + DIST;
      const int cur = t & 1;
      // the next step's operands (its slab and window tile are resident, see the header) while this step multiplies
      if (t + 1 < TAPS) load_frags(cur ^ 1, slot_n, hb, toff[t + 1]);
      else load_frags(cur ^ 1, slot_n, hb ^ 1, toff[0]);
      __builtin_amdgcn_sched_barrier(0);
#define ST_MMA(j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][(j) / NPS], fb[cur][(j) % NPS], acc[j], 0, 0, 0)
      ST_MMA(0);
      __builtin_amdgcn_sched_barrier(0);
      issue_weights(c3, t3, slot_f);
      __builtin_amdgcn_sched_barrier(0);
      ST_MMA(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < HPT; ++u)
        if (u < halo_units(t)) issue_halo(cnext, t * HPT + u, hb ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      ST_MMA(2);
      ST_MMA(3);
#undef ST_MMA
      __builtin_amdgcn_sched_barrier(0);
      slot = slot_n;
    }
    if (TAPS & 1) {   // an odd number of steps per chunk: the operands fetched last sit in buffer 1, the next chunk starts from 0
#pragma unroll
      for (int ps = 0; ps < NPS; ++ps) fb[0][ps] = fb[1][ps];
#pragma unroll
      for (int i = 0; i < NCS; ++i) fa[0][i] = fa[1][i];
    }
  }
  wait_vm<0>();   // trailing copies must not outlive the workgroup's LDS
  STAMP(125);

  // ---- epilogue: the four waves of a pixel group add their sums, then bias, one rounding to bf16, 16-byte stores ----
  // Accumulator element e of lane l in subtile (i, ps): channel 32 i + 8 (e / 4) + 4 (l / 32) + e % 4, pixel
  // 32 ps + l % 32 of the pixel group.  Every wave leaves its four subtiles in LDS as
  // [pixel group][wave kq][subtile][q][lane] float4; wave kq then sums the four copies of subtile kq, rounds its
  // 32 x 32 block into its own 2 KB of LDS ([pixel][32 ch], granules swizzled by pixel) and reads it back row-wise:
  // four lanes cover one pixel's 64 contiguous bytes.
  if (tid < TRC) { biasl[tid] = bias_v; biasl[TRC + tid] = scale_v; }
  __syncthreads();   // every wave is done with the ring and the window tiles
  {
    float4* red = reinterpret_cast<float4*>(smem + OFF_W);
    float4* mine = red + ((wpx * 4 + kq) * 16) * 64 + lane;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        mine[(i * 4 + q) * 64] = make_float4(acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]);
    __syncthreads();
    float4 sum[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4* src = red + ((wpx * 4) * 16 + kq * 4 + q) * 64 + lane;
      const float4 c0 = src[0], c1 = src[16 * 64], c2 = src[2 * 16 * 64], c3 = src[3 * 16 * 64];
      sum[q] = make_float4((c0.x + c1.x) + (c2.x + c3.x), (c0.y + c1.y) + (c2.y + c3.y), (c0.z + c1.z) + (c2.z + c3.z),
                           (c0.w + c1.w) + (c2.w + c3.w));
    }
    __syncthreads();   // all copies read: their space holds the staging blocks next
    unsigned char* stage = smem + OFF_W + wave * 2048;
    const int px = lane & 31;
    const int psw = (px >> 1) & 3;
    const int ci = kq / NPS, pss = kq % NPS;   // the subtile this wave finishes
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int ch = q * 8 + kb * 4;
      const float4 bb = *reinterpret_cast<const float4*>(biasl + ci * 32 + ch);
      const float4 sc = *reinterpret_cast<const float4*>(biasl + TRC + ci * 32 + ch);
      const uint2 v = make_uint2(pack_bf16x2(fmaf(sum[q].x, sc.x, bb.x), fmaf(sum[q].y, sc.y, bb.y)),
                                 pack_bf16x2(fmaf(sum[q].z, sc.z, bb.z), fmaf(sum[q].w, sc.w, bb.w)));
      *reinterpret_cast<uint2*>(stage + px * 64 + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int row = it * 16 + (lane >> 2);
      const uint4 v = *reinterpret_cast<const uint4*>(stage + row * 64 + ((lane & 3) << 4));
      (void)pss;
      const long long o = store_off(it);
      if (o >= 0) *reinterpret_cast<uint4*>(p.out + o) = post_op8(v, p.relu, p.mask, p.add, (size_t)o);
    }
  }
  STAMP(126);
}

// Largest number of window-tile pixels any TP-pixel tile needs.
int max_window_pixels(const StParams& p, int kH, int TP) {
  const int HoWo = p.Ho * p.Wo;
  int a = HoWo, b = TP;
  while (b) { const int t = a % b; a = b; b = t; }
  const int period = HoWo / a;   // tile starts repeat modulo the image size after `period` tiles
  int best = 0;
  for (int m0 = 0, t = 0; m0 < p.M && t <= period; m0 += TP, ++t) {
    const int ml = (m0 + TP < p.M ? m0 + TP : p.M) - 1;
    const int na = m0 / HoWo, hoa = (m0 - na * HoWo) / p.Wo;
    const int nb = ml / HoWo, hob = (ml - nb * HoWo) / p.Wo;
    const int ns = nb * p.Hv + hob + kH - (na * p.Hv + hoa);
    if (ns > best) best = ns;
  }
  return best * p.Wv;
}

// Completes the plan of a problem whose tensors are described in p; false = this kernel does not take it.
using Narrow = Shape<64, 128>;
using Wide = Shape<128, 64>;
using Tall = Shape<128, 64, 6, 7>;

template <class S>
bool shape_fits(const StParams& p, int kH) {
  if (p.R % S::TRC) return false;
  if (max_window_pixels(p, kH, S::TP) > S::HUNITS * HRPU) return false;
  // small tiles are for problems that would not fill the chip with larger ones
  const long long tiles = (long long)ceil_div(p.M, S::TP) * (p.R / S::TRC);
  return tiles >= 96 && tiles <= 640;
}

bool finish_plan(StParams& p, int kH, int kW) {
  if (kH != 3 || kW != 3) return false;
  if (p.C % CB) return false;
  if (p.act_bytes >= OOB || p.wgt_bytes >= OOB) return false;
  p.Hv = p.Ho - 1 + kH;
  p.Wv = p.Wo - 1 + kW;
  const bool wide_ok = shape_fits<Wide>(p, kH), narrow_ok = shape_fits<Narrow>(p, kH);
  const bool tall_ok = !wide_ok && shape_fits<Tall>(p, kH);
#if defined(ST_FORCE_NARROW)
  p.wide = 0;
  if (!narrow_ok) return false;
#else
  if (!wide_ok && !narrow_ok && !tall_ok) return false;
  p.wide = wide_ok ? 1 : (narrow_ok ? 0 : 2);
#endif
  p.dHoWo = make_fastdiv(p.Ho * p.Wo);
  p.dWo = make_fastdiv(p.Wo);
  p.dHv = make_fastdiv(p.Hv);
  p.dWv = make_fastdiv(p.Wv);
  p.ntr = p.R / (p.wide ? Wide::TRC : Narrow::TRC);   // (Tall has Wide's channel tile)
  p.nchunks = p.C / CB;
  return true;
}

bool fprop_params(const Geom& g, StParams* p) {
  StParams& q = *p;
  q = StParams{};
  if (g.sh != 1 || g.sw != 1) return false;
  q.N = g.N; q.C = g.Cin; q.H = g.Hin; q.W = g.Win; q.Ho = g.Hout; q.Wo = g.Wout; q.R = g.Cout; q.M = g.M;
  q.ph = g.ph; q.pw = g.pw;
  q.wt0 = 0; q.wt_row = g.kW; q.wt_col = 1;
  q.wrow = g.kH * g.kW * g.Cin;
  q.act_n_stride = g.Hin * g.Win * g.Cin; q.act_h_stride = g.Win * g.Cin; q.act_w_stride = g.Cin;
  if ((size_t)g.Min * g.Cin * 2 >= OOB || (size_t)g.Cout * g.K * 2 >= OOB) return false;
  q.act_bytes = (unsigned)((size_t)g.Min * g.Cin * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  return finish_plan(q, g.kH, g.kW);
}

bool dgrad_params(const Geom& g, StParams* p) {
  StParams& q = *p;
  q = StParams{};
  if (g.sh != 1 || g.sw != 1) return false;
  if (g.ph > g.kH - 1 || g.pw > g.kW - 1) return false;
  q.N = g.N; q.C = g.Cout; q.H = g.Hout; q.W = g.Wout; q.Ho = g.Hin; q.Wo = g.Win; q.R = g.Cin; q.M = g.Min;
  q.ph = g.kH - 1 - g.ph; q.pw = g.kW - 1 - g.pw;
  q.wt0 = g.kH * g.kW - 1; q.wt_row = -g.kW; q.wt_col = -1;   // rotated kernel
  q.wrow = g.kH * g.kW * g.Cout;
  q.act_n_stride = g.Hout * g.Wout * g.Cout; q.act_h_stride = g.Wout * g.Cout; q.act_w_stride = g.Cout;
  if ((size_t)g.M * g.Cout * 2 >= OOB || (size_t)g.Cout * g.K * 2 >= OOB) return false;
  q.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  return finish_plan(q, g.kH, g.kW);
}

template <class S>
hipError_t launch_shape(const StParams& p, hipStream_t st) {
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_st_kernel<3, 3, S>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS_BYTES);
  });
  if (attr_err != hipSuccess) return attr_err;
  const int tiles = ceil_div(p.M, S::TP) * p.ntr;
  hipLaunchKernelGGL((conv_st_kernel<3, 3, S>), dim3(tiles), dim3(64 * NWAVES), S::LDS_BYTES, st, p);
  return hipGetLastError();
}

hipError_t launch(const StParams& p, hipStream_t st) {
  return p.wide == 1 ? launch_shape<Wide>(p, st) : (p.wide == 2 ? launch_shape<Tall>(p, st) : launch_shape<Narrow>(p, st));
}

}  // namespace

bool st_fprop_supported(const Geom& g, int dtype) {
  StParams p;
  return dtype == CONVBN_BF16 && fprop_params(g, &p);
}
bool st_dgrad_supported(const Geom& g, int dtype) {
  StParams p;
  return dtype == CONVBN_BF16 && dgrad_params(g, &p);
}
hipError_t launch_fprop_st(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z,
                           hipStream_t st, const BnEpilogue* bn) {
  StParams p;
  if (!fprop_params(g, &p)) return hipErrorInvalidValue;
  if (bn) p.bn = *bn;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_krsc; p.bias = bias; p.out = (bf16_t*)z;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  return launch(p, st);
}
hipError_t launch_dgrad_st(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                           hipStream_t st) {
  StParams p;
  if (!dgrad_params(g, &p)) return hipErrorInvalidValue;
  p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = bias; p.out = (bf16_t*)dx;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  return launch(p, st);
}

}  // namespace convbn

#ifdef ST_TRACE
extern "C" int convbn_debug_read_st_trace(unsigned long long* host, size_t n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(convbn::st_trace), n * sizeof(unsigned long long));
}
#endif
