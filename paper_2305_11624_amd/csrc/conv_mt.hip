// bf16 MFMA convolution for deep layers (3x3 windows, stride 1, many channels, few pixels): large
// 256-pixel x 128-channel workgroup tiles with the reduced channels split over several workgroups.
//
//   forward conv   Z  = w' (*) X + b'     (Sec. 3.1 / 3.3)   act = x,  weights [Cout][taps][Cin]
//   input gradient dX = w'_rot (*) dZ     (Sec. 3.2.1)       act = dz, weights [Cin][taps][Cout], taps reversed
//
// Why this shape.  A compute unit receives at most 64 bytes per clock from the L2, and the folded weight is
// what a deep layer streams: a workgroup that owns TP pixels x TRC channels fetches TRC rows of weights per
// reduction step but (thanks to the window tile below) only ~TP/4 rows of activations, for TP TRC / 32 cycles
// of matrix work.  With 64 x 128 tiles the copies alone need the full 64 B/clk; 256 x 128 needs 24.  Tiles of
// that size are fewer than the chip has compute units, so the reduction (channel chunks of 32) is divided over
// gridDim.y workgroups; each writes its fp32 accumulators as they sit in registers (1 KB per store
// instruction), and the workgroup that arrives last at the tile's counter sums the copies in a fixed order,
// adds the bias and stores the bf16 result -- one launch, deterministic sums.
//
// Layout in LDS.  Activations: the window rows the tile's pixels touch, as [slot][column][32 channels] with
// zero rows / columns for the padding (copies of out-of-image pixels use an out-of-range buffer offset, which
// the hardware turns into zeros); rows are 80 bytes apart (64 + one pad granule), so 16 consecutive rows of a
// 128-bit operand read fall on distinct banks and a tap is a wave-uniform offset added to a per-lane base.
// All nine taps of a chunk read the same tile: an input element is fetched once per chunk, not once per tap.
// Weights: one [128 rows][32 channels] slab per (chunk, tap) step in a ring of four, rows 64 bytes apart with
// the four 16-byte granules of a row permuted by (row / 4) % 4 (the copy chooses which granule each lane
// fetches), which also spreads 16 consecutive rows over all banks and makes a slab exactly eight 1 KB copies:
// one per wave and step.
//
// Pipeline.  Eight waves = 4 pixel groups x 2 channel groups, each wave 64 pixels x 64 channels (2 x 2 MFMA
// tiles, 32x32x16).  A step = one tap of one chunk = 2 k-steps x 4 MFMAs per wave.  The taps are unrolled, so
// everything about a step except its ring slot is known at compile time.  During step s every wave issues its
// 1 KB of the slab of step s + 3 and, in the first five taps of a chunk, one unit of the next chunk's window
// tile.  Copies complete in issue order: "at most the copies of step s - 1 outstanding" at the barrier of step s
// means the slab of step s + 1 and -- at a chunk's last tap -- the next window tile are resident, which is what
// the operand prefetch of the step's last k-step reads.
#include "common.h"

#include <atomic>
#include <chrono>
#include <mutex>

namespace convbn {

namespace {

struct FastDiv {   // exact n / d for 0 <= n < 2^31
  unsigned mul, shr;
  int d;
};

FastDiv make_fastdiv(int d) {
  FastDiv f{0u, 0u, d};
  if (d <= 1) return f;
  unsigned s = 0;
  while ((1ull << (s + 1)) < (unsigned long long)d) ++s;   // 2^s < d <= 2^(s+1)
  f.shr = s;
  f.mul = (unsigned)((((unsigned long long)1 << (32 + s)) + d - 1) / d);
  return f;
}

__device__ __forceinline__ int fdiv(int n, const FastDiv& f) {
  return f.d == 1 ? n : (int)(__umulhi((unsigned)n, f.mul) >> f.shr);
}

constexpr int TP = 256;                 // output pixels per workgroup
constexpr int TRC = 128;                // output channels per workgroup
constexpr int CB = 32;                  // reduced channels per chunk
constexpr int NWAVES = 8;
constexpr int HROW = 80;                // window-tile row pitch: 64 bytes of channels + one pad granule
constexpr int HRPU = 12;                // whole rows per 1 KB copy (its last four lanes spill into the next row)
constexpr int HUNIT = HRPU * HROW;      // 960
constexpr int HUW = 5;                  // window-tile copies per wave and chunk
constexpr int HUNITS = NWAVES * HUW;    // 40 -> at most 480 window pixels per tile
constexpr int HBUF = HUNITS * HUNIT + 64;
constexpr int WSLAB = TRC * CB * 2;     // 8192
constexpr int NBUF = 4;
constexpr int DIST = NBUF - 1;
constexpr int OFF_W = 1024;             // bias first
constexpr int OFF_H = OFF_W + NBUF * WSLAB;
constexpr int LDS_BYTES = OFF_H + 2 * HBUF;
constexpr int DUMP_FLOATS = TP * TRC;   // one workgroup's accumulators
constexpr unsigned OOB = 0x80000000u;

struct MtParams {
  const bf16_t* act;
  const bf16_t* wgt;
  const float* bias;
  bf16_t* out;
  float* part;                    // [tile][split][wave][64 registers][lane] fp32 accumulator dumps
  unsigned long long* counters;   // [tile]: (launch tag << 8) | arrivals
  unsigned long long tag;
  unsigned act_bytes, wgt_bytes;
  int N, H, W, C;
  int act_n_stride, act_h_stride, act_w_stride;   // elements
  int Ho, Wo, R, M;
  int ph, pw, Hv, Wv;
  int wrow;                       // elements per weight row (taps x C)
  int wt0, wt_row, wt_col;        // window position (ti, tj) reads weight tap wt0 + ti wt_row + tj wt_col
  int ntr;                        // channel tiles
  int nchunks, chunks_per_split, ksplit;
  int allow_split;                // split sums cost a trip through memory: measured slower than the smaller tiles of the general kernel
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

// Accumulator dumps cross workgroups that may run on different XCDs, whose L2 caches are not coherent with
// each other.  Instead of fences (an L2 write-back of everything the XCD holds, and an invalidate on the other
// side), the dumps are written and read with device-scope accesses: the store writes through to memory, the
// load misses any stale line.  Completion is what the vmcnt wait before the arrival count establishes.
__device__ __forceinline__ void store_device_scope(float* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void load_device_scope(f32x4& v, const float* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
}

template <int KH, int KW>
__global__ __launch_bounds__(64 * NWAVES) void conv_mt_kernel(MtParams p) {
  constexpr int TAPS = KH * KW;
  static_assert(TAPS >= HUW + 1 && TAPS >= DIST, "the copy schedule assumes a window of at least six taps");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* biasl = reinterpret_cast<float*>(smem);
  unsigned char* wbuf = smem + OFF_W;
  unsigned char* halo = smem + OFF_H;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wpx = wave & 3, wch = wave >> 2;
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
  const int cbeg = blockIdx.y * p.chunks_per_split;
  const int cend = min(p.nchunks, cbeg + p.chunks_per_split);
  const int nloc = cend - cbeg;

  float bias_v = (tid < TRC && p.bias) ? p.bias[r0 + tid] : 0.f;

  // window-tile copies of this wave: unit wave + 8 t, t = 0..4; per-lane byte offsets without the chunk
  unsigned hv[HUW];
  {
    const int lrow = lane / 5, lgran = lane - lrow * 5;   // lanes 60..63: row 12 = the next unit's first row
#pragma unroll
    for (int t = 0; t < HUW; ++t) {
      const int pix = (wave + NWAVES * t) * HRPU + lrow;
      const int slot = fdiv(pix, p.dWv);
      const int w = pix - slot * p.Wv - p.pw;
      const int v = v_first + slot;
      const int n = fdiv(v, p.dHv);
      const int h = v - n * p.Hv - p.ph;
      const bool ok = pix < npix && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W && n < p.N && lgran < 4;
      hv[t] = ok ? (unsigned)((n * p.act_n_stride + h * p.act_h_stride + w * p.act_w_stride + lgran * 8) * 2) : OOB;
    }
  }
  // weight copy of this wave: rows 16 wave .. 16 wave + 15 of the slab, granules permuted by (row / 4) % 4
  unsigned voff_w;
  {
    const int row = wave * 16 + (lane >> 2);
    const int g = (lane & 3) ^ ((row >> 2) & 3);
    voff_w = (unsigned)(((r0 + row) * p.wrow + g * 8) * 2);
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
  unsigned boff[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int pi = wpx * 64 + j * 32 + (lane & 31);
    int pixidx = 0;
    if (pi < len) {
      const int m = m0 + pi;
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      const int ho = fdiv(rem, p.dWo);
      pixidx = (n * p.Hv + ho - v_first) * p.Wv + (rem - ho * p.Wo);
    }
    boff[j] = (unsigned)(pixidx * HROW + kb * 16);
  }
  const unsigned aoff = (unsigned)((wch * 64 + (lane & 31)) * 64 + ((kb ^ (((lane & 31) >> 2) & 3)) << 4));

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  auto issue_weights = [&](int chunk, int t, int slot) {
    dma16(wgt_rsrc, voff_w, (unsigned)(wsoff[t] + chunk * (CB * 2)), wbuf + slot * WSLAB + wave * 1024);
  };
  auto issue_halo = [&](int chunk, int t, int hb) {
    dma16(act_rsrc, hv[t], (unsigned)(chunk * (CB * 2)), halo + hb * HBUF + (wave + NWAVES * t) * HUNIT);
  };

  // ---- prologue: the first chunk's window tile and the slabs of steps 0 .. DIST-1 ---------------------
#pragma unroll
  for (int t = 0; t < HUW; ++t) issue_halo(cbeg, t, 0);
#pragma unroll
  for (int s = 0; s < DIST; ++s) issue_weights(cbeg, s, s);

  bf16x8 fa[2][2], fb[2][2];
  // operands of k-step kk: weights from ring slot `slot`, pixels from window tile `hb` at tap offset `to`
  auto load_frags = [&](int buf, int slot, int hb, int to, int kk) {
    const unsigned char* a = wbuf + slot * WSLAB + (kk ? (aoff ^ 32u) : aoff);
    const unsigned char* b = halo + hb * HBUF + to + kk * 32;
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(a + i * 2048);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[buf][j] = *reinterpret_cast<const bf16x8*>(b + boff[j]);
  };

  wait_vm<0>();
  block_barrier();
  load_frags(0, 0, 0, toff[0], 0);

  int slot = 0;   // ring slot of the current step
  for (int lc = 0; lc < nloc; ++lc) {
    const int hb = lc & 1;
    const int cnext = min(cbeg + lc + 1, cend - 1);   // past the end: the last chunk again (nobody reads it)
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
      // copies that may still be in flight: those of the previous step
      if (t == 0 || t > HUW) wait_vm<1>(); else wait_vm<2>();
      block_barrier();
      const int t3 = (t + DIST) % TAPS;
      const int c3 = (t + DIST) >= TAPS ? cnext : cbeg + lc;
      const int slot_n = (slot + 1) & (NBUF - 1);
      const int slot_f = (slot + DIST) & (NBUF - 1);

      load_frags(1, slot, hb, toff[t], 1);
      __builtin_amdgcn_sched_barrier(0);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][0], fb[0][0], acc[0][0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      issue_weights(c3, t3, slot_f);
      if (t < HUW) issue_halo(cnext, t, hb ^ 1);
      __builtin_amdgcn_sched_barrier(0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][1], fb[0][0], acc[1][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][0], fb[0][1], acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][1], fb[0][1], acc[1][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      // the next step's first operands (its slab and window tile are resident, see the header)
      if (t + 1 < TAPS) load_frags(0, slot_n, hb, toff[t + 1], 0);
      else load_frags(0, slot_n, hb ^ 1, toff[0], 0);
      __builtin_amdgcn_sched_barrier(0);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][0], fb[1][0], acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][1], fb[1][0], acc[1][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][0], fb[1][1], acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][1], fb[1][1], acc[1][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      slot = slot_n;
    }
  }
  wait_vm<0>();   // trailing copies must not outlive the workgroup's LDS

  // ---- split sums: dump the accumulators; the last workgroup of the tile sums all dumps in split order ----
  // Accumulator element e of lane l in MFMA tile (i, j): channel 32 i + 8 (e / 4) + 4 (l / 32) + e % 4 of the
  // wave's 64, pixel 32 j + l % 32 of the wave's 64.
  if (p.ksplit > 1) {
    float* dump = p.part + ((size_t)blockIdx.x * p.ksplit) * DUMP_FLOATS + (size_t)wave * (64 * 64) + lane * 4;
    {
      float* mine = dump + (size_t)blockIdx.y * DUMP_FLOATS;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
            store_device_scope(mine + ((i * 2 + j) * 4 + q) * 256, v);
          }
    }
    wait_vm<0>();      // this thread's dump has reached memory ...
    __syncthreads();   // ... and so has every other thread's, before the arrival is counted
    int* flag = reinterpret_cast<int*>(smem + OFF_W);
    if (tid == 0) {
      unsigned long long* c = p.counters + blockIdx.x;
      unsigned long long old = __hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned long long cnt;
      for (;;) {   // a word that does not carry this launch's tag is stale: count from zero
        cnt = (old >> 8) == p.tag ? (old & 255ull) : 0ull;
        const unsigned long long want = (p.tag << 8) | (cnt + 1);
        if (__hip_atomic_compare_exchange_strong(c, &old, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
          break;
      }
      *flag = (int)cnt == p.ksplit - 1;
      // the last arrival leaves the count at zero under the same tag: a replay of a captured launch (same
      // arguments, same tag) starts from zero again
      if (*flag) __hip_atomic_store(c, p.tag << 8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!*flag) return;
    // the last workgroup of the tile: all dumps are in memory; sum them in split order (deterministic)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int s = 0; s < p.ksplit; ++s) {
      const float* src = dump + (size_t)s * DUMP_FLOATS;
      f32x4 v[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) load_device_scope(v[k], src + k * 256);
      wait_vm<0>();
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        asm volatile("" : "+v"(v[k]));   // the loads above are invisible to the compiler: order the uses after the wait
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[k >> 3][(k >> 2) & 1][(k & 3) * 4 + e] += v[k][e];
      }
    }
  }
  // ---- epilogue: bias, one rounding to bf16, 16-byte stores ------------------------------------------------
  // Each wave rounds a 32-pixel x 64-channel block into its own 4 KB of LDS ([pixel][64 ch], granules swizzled
  // by pixel) and reads it back row-wise: eight lanes cover one pixel's 128 contiguous bytes.
  if (tid < TRC) biasl[tid] = bias_v;
  __syncthreads();
  {
    unsigned char* stage = smem + OFF_W + wave * 4096;
    const int px = lane & 31;
    const int psw = (px >> 1) & 7;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ch = i * 32 + q * 8 + kb * 4;
          const float4 bb = *reinterpret_cast<const float4*>(biasl + wch * 64 + ch);
          const uint2 v = make_uint2(pack_bf16x2(acc[i][j][q * 4 + 0] + bb.x, acc[i][j][q * 4 + 1] + bb.y),
                                     pack_bf16x2(acc[i][j][q * 4 + 2] + bb.z, acc[i][j][q * 4 + 3] + bb.w));
          *reinterpret_cast<uint2*>(stage + px * 128 + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
        }
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int row = it * 8 + (lane >> 3);
        const int g = (lane & 7) ^ ((row >> 1) & 7);
        const uint4 v = *reinterpret_cast<const uint4*>(stage + row * 128 + ((lane & 7) << 4));
        const int pi = wpx * 64 + j * 32 + row;
        if (pi < len) *reinterpret_cast<uint4*>(p.out + (size_t)(m0 + pi) * p.R + r0 + wch * 64 + g * 8) = v;
      }
    }
  }
}

// Largest number of window-tile pixels any TP-pixel tile needs.
int max_window_pixels(const MtParams& p, int kH) {
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
bool finish_plan(MtParams& p, int kH, int kW) {
  if (kH != 3 || kW != 3) return false;
  if (p.C % CB || p.R % TRC || p.C < 128) return false;
  if (p.act_bytes >= OOB || p.wgt_bytes >= OOB) return false;
  p.Hv = p.Ho - 1 + kH;
  p.Wv = p.Wo - 1 + kW;
  if (max_window_pixels(p, kH) > HUNITS * HRPU) return false;
  p.dHoWo = make_fastdiv(p.Ho * p.Wo);
  p.dWo = make_fastdiv(p.Wo);
  p.dHv = make_fastdiv(p.Hv);
  p.dWv = make_fastdiv(p.Wv);
  p.ntr = p.R / TRC;
  p.nchunks = p.C / CB;
  const long long tiles = (long long)ceil_div(p.M, TP) * p.ntr;
  // split the chunks over as many workgroups as still fit the chip in one round (at least two chunks each)
  int ks = 1;
  while (ks * 2 <= 8 && tiles * ks * 2 <= 256 && p.nchunks % (ks * 2) == 0 && p.nchunks / (ks * 2) >= 2) ks *= 2;
  if (tiles * ks < 128) return false;   // too few workgroups either way: the smaller tiles of the general kernel do better
  if (ks > 1 && !p.allow_split) return false;
  p.ksplit = ks;
  p.chunks_per_split = p.nchunks / ks;
  return true;
}

bool fprop_params(const Geom& g, MtParams* p) {
  MtParams& q = *p;
  q = MtParams{};
  if (g.sh != 1 || g.sw != 1) return false;
  q.N = g.N; q.C = g.Cin; q.H = g.Hin; q.W = g.Win; q.Ho = g.Hout; q.Wo = g.Wout; q.R = g.Cout; q.M = g.M;
  q.ph = g.ph; q.pw = g.pw;
  q.wt0 = 0; q.wt_row = g.kW; q.wt_col = 1;
  q.wrow = g.kH * g.kW * g.Cin;
  q.act_n_stride = g.Hin * g.Win * g.Cin; q.act_h_stride = g.Win * g.Cin; q.act_w_stride = g.Cin;
  q.act_bytes = (unsigned)((size_t)g.Min * g.Cin * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  if ((size_t)g.Min * g.Cin * 2 >= OOB || (size_t)g.Cout * g.K * 2 >= OOB) return false;
  return finish_plan(q, g.kH, g.kW);
}

bool dgrad_params(const Geom& g, MtParams* p) {
  MtParams& q = *p;
  q = MtParams{};
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
  // the window must cover exactly the dZ grid: Hout - 1 + kH = Hin + 2 (kH - 1 - ph) holds for stride 1
  return finish_plan(q, g.kH, g.kW);
}

size_t scratch_bytes(const MtParams& p) {
  if (p.ksplit == 1) return 0;
  const size_t tiles = (size_t)ceil_div(p.M, TP) * p.ntr;
  return align_up(tiles * 8, 256) + tiles * p.ksplit * DUMP_FLOATS * 4;
}

// Tag of a launch: distinguishes this launch's arrival counts from whatever the workspace held before.
unsigned long long next_tag() {
  static std::atomic<unsigned long long> tag{
      (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() * 0x9E3779B97F4A7C15ull};
  return tag.fetch_add(1, std::memory_order_relaxed) & ((1ull << 56) - 1);
}

hipError_t launch(MtParams& p, float* scratch, hipStream_t st) {
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_mt_kernel<3, 3>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  });
  if (attr_err != hipSuccess) return attr_err;
  const int tiles = ceil_div(p.M, TP) * p.ntr;
  if (p.ksplit > 1) {
    if (!scratch) return hipErrorInvalidValue;
    p.counters = reinterpret_cast<unsigned long long*>(scratch);
    p.part = reinterpret_cast<float*>(reinterpret_cast<char*>(scratch) + align_up((size_t)tiles * 8, 256));
    p.tag = next_tag();
  }
  hipLaunchKernelGGL((conv_mt_kernel<3, 3>), dim3(tiles, p.ksplit), dim3(64 * NWAVES), LDS_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace

bool mt_fprop_supported(const Geom& g, int dtype) {
  MtParams p;
  return dtype == CONVBN_BF16 && fprop_params(g, &p);
}
bool mt_dgrad_supported(const Geom& g, int dtype) {
  MtParams p;
  return dtype == CONVBN_BF16 && dgrad_params(g, &p);
}
size_t mt_fprop_scratch_bytes(const Geom& g) {
  MtParams p;
  return fprop_params(g, &p) ? scratch_bytes(p) : 0;
}
size_t mt_dgrad_scratch_bytes(const Geom& g) {
  MtParams p;
  return dgrad_params(g, &p) ? scratch_bytes(p) : 0;
}
hipError_t launch_fprop_mt(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z,
                           float* scratch, hipStream_t st) {
  MtParams p;
  if (!fprop_params(g, &p)) return hipErrorInvalidValue;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_krsc; p.bias = bias; p.out = (bf16_t*)z;
  return launch(p, scratch, st);
}
hipError_t launch_dgrad_mt(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                           float* scratch, hipStream_t st) {
  MtParams p;
  if (!dgrad_params(g, &p)) return hipErrorInvalidValue;
  p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = bias; p.out = (bf16_t*)dx;
  return launch(p, scratch, st);
}

}  // namespace convbn
