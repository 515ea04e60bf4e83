// bf16 MFMA convolution with the input window tile resident in LDS.
//
// A workgroup owns TP consecutive output pixels (in (n,ho,wo) order) x TRC output channels.
// All input rows those pixels touch are copied once into LDS as [slot][column][channel chunk]
// (zero rows/columns stand in for the padding), then every tap (i,j) of the kernel window is
// one MFMA sweep over the SAME LDS tile at a wave-uniform offset of (i*Wv + j) pixels: each
// input element is fetched from memory once per workgroup instead of once per tap.  The weight
// tile of the current (tap, channel chunk) streams through a double-buffered LDS stage.
//
// Global -> LDS copies are buffer loads that write LDS directly (16 bytes per lane, lane l of a
// wave lands at base + 16 l); out-of-range lanes are given an offset beyond the buffer and
// deliver zeros, which is how padding is materialised without branches.  LDS rows are unpadded;
// the 16-byte granule g of row r is stored at granule g ^ swz(r) so that the 16-lane groups of
// a 128-bit LDS read fall on distinct banks.
//
//   forward conv   Z  = w' (*) X + b'        (Sec. 3.1 / 3.3)    act = x,  weights [Cout][taps][Cin]
//   input gradient dX = w'_rot (*) dZ        (Sec. 3.2.1), stride 1: the same sweep over dz with
//                  the taps reversed and padding k-1-p,          weights [Cin][taps][Cout]
#include "common.h"

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

struct TileParams {
  const bf16_t* act;     // activations, channels-last, explicit strides (elements)
  const bf16_t* wgt;     // [R][taps][C]
  const float* bias;     // [R] or null
  bf16_t* out;           // [M][R]
  unsigned act_bytes, wgt_bytes;
  int N, H, W, C;        // activation grid the window slides over
  int act_n_stride, act_h_stride, act_w_stride;
  int Ho, Wo, R;
  int kH, kW, sh, sw, ph, pw;
  int flip;              // weight tap order reversed
  int M;                 // N*Ho*Wo
  int Hv, Wv;            // rows / columns of one image's (virtually padded) window footprint
  int ntr;               // channel tiles
  int nhb, hps, spread;  // activation tile ring depth, copy slices per step, steps a prefetch spans
  int ksplit, chunks_per_split;   // channel chunks are divided over gridDim.y workgroups
  float* part;           // [ksplit][M][R] fp32 partial outputs when ksplit > 1
  int halo_stride;       // bytes per activation tile buffer
  FastDiv dHoWo, dWo, dHv, dWv;
};

constexpr unsigned OOB = 0x80000000u;   // beyond any buffer: the load returns zeros

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_off, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)byte_off, 0, 0, 0);
}

constexpr int DIST = 3;   // steps between issuing a copy and consuming it
constexpr int NBUF = 4;   // weight ring (DIST + 1)

// Workgroup barrier without the memory fence of __syncthreads(): the fence would drain every
// outstanding copy (vmcnt(0)) and serialise the pipeline.  Ordering of the copies is handled by
// the explicit vmcnt waits; LDS reads are ordered by their own data dependences.
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int N> __device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Waits until at most 2*(wpw + hps) of this wave's copies are outstanding.
template <int WPW> __device__ __forceinline__ void wait_two_steps(int hps) {
  switch (hps) {
    case 0: wait_vm<2 * WPW>(); break;
    case 1: wait_vm<2 * (WPW + 1)>(); break;
    case 2: wait_vm<2 * (WPW + 2)>(); break;
    case 4: wait_vm<2 * (WPW + 4)>(); break;
    default: wait_vm<2 * (WPW + 8)>(); break;
  }
}

// PSUB: 32-pixel subtiles per wave (tile = 128*PSUB pixels); NCH: 32-channel subtiles (TRC = 32 NCH);
// CB: channels per LDS chunk.
//
// Pipeline.  A "step" is one tap of one channel chunk.  Every step each wave issues exactly
// hps + WPW copies: hps 1 KB slices of a future chunk's activation tile (or dummies into a scratch
// KB when there is nothing to fetch) and the weight tile of step it+DIST.  Copies complete in issue
// order, so "at most 2 steps' worth outstanding" means everything issued DIST steps ago has landed.
// The activation tile ring has nhb buffers: 1 (single chunk), 2 (next chunk fetched during the
// first `spread` steps of the current one) or 4 (1x1 windows: one step per chunk, fetched DIST
// chunks ahead).
template <int NW, int PSUB, int NCH, int CB>
__global__ __launch_bounds__(64 * NW) void conv_tile_kernel(TileParams p) {
  constexpr int TP = 32 * NW * PSUB;
  constexpr int TRC = NCH * 32;
  constexpr int GPR = CB / 8;            // 16-byte granules per LDS row
  constexpr int RPU = 64 / GPR;          // rows filled by one wave-wide 1 KB copy
  constexpr int ROWB = CB * 2;           // bytes per LDS row
  constexpr int SWZ_SHIFT = (CB == 64) ? 1 : 2;   // rows per 256-byte bank cycle = 2 or 4
  constexpr int WUNITS = TRC / RPU;      // 1 KB copies per weight tile
  constexpr int WPW = (WUNITS + NW - 1) / NW;  // per wave (waves beyond WUNITS issue dummies)
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* biasl = reinterpret_cast<float*>(smem);               // [TRC] bias of this channel tile (first KB)
  unsigned char* wbuf = smem + 1024;                           // [NBUF][TRC][CB] bf16
  unsigned char* scratch = wbuf + NBUF * TRC * ROWB;           // 1 KB target of the dummy copies (zeros only)
  unsigned char* halo = scratch + 1024;                        // [nhb][halo_stride]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ctile = blockIdx.x % p.ntr, ptile = blockIdx.x / p.ntr;
  const int r0 = ctile * TRC;
  const int m0 = ptile * TP;
  const int m_last = min(p.M, m0 + TP) - 1;
  const int HoWo = p.Ho * p.Wo;
  const int n_a = fdiv(m0, p.dHoWo), ho_a = fdiv(m0 - n_a * HoWo, p.dWo);
  const int n_b = fdiv(m_last, p.dHoWo), ho_b = fdiv(m_last - n_b * HoWo, p.dWo);
  const int v_first = n_a * p.Hv + ho_a * p.sh;
  const int nslots = n_b * p.Hv + ho_b * p.sh + p.kH - v_first;
  const int npix = nslots * p.Wv;
  const int hunits = (npix + RPU - 1) / RPU;

  const __amdgpu_buffer_rsrc_t act_rsrc = make_rsrc(p.act, p.act_bytes);
  const __amdgpu_buffer_rsrc_t wgt_rsrc = make_rsrc(p.wgt, p.wgt_bytes);
  const int taps = p.kH * p.kW;
  const int cbeg = blockIdx.y * p.chunks_per_split;                       // first channel chunk of this workgroup
  const int nchunks = min((p.C + CB - 1) / CB, cbeg + p.chunks_per_split);  // one past its last chunk
  if (tid < TRC) biasl[tid] = (p.bias && r0 + tid < p.R) ? p.bias[r0 + tid] : 0.f;   // read after many barriers

  // this lane's place inside every 1 KB copy unit
  const int urow = lane / GPR;
  const int ugran = lane % GPR;

  // weight tile of step `step` (chunk, tap) -> ring slot step % NBUF
  auto issue_weights = [&](int chunk, int tap, int step) {
    const int tw = p.flip ? taps - 1 - tap : tap;
    unsigned char* dst = wbuf + (step % NBUF) * (TRC * ROWB);
#pragma unroll
    for (int j = 0; j < WPW; ++j) {
      const int u = wave + NW * j;
      const int row = u * RPU + urow;
      const int g = ugran ^ ((row >> SWZ_SHIFT) & (GPR - 1));
      const int ch = chunk * CB + g * 8;
      unsigned off = (unsigned)((((r0 + row) * taps + tw) * p.C + ch) * 2);
      if (u >= WUNITS || chunk >= nchunks || r0 + row >= p.R || ch >= p.C) off = OOB;
      dma16(wgt_rsrc, off, u < WUNITS ? dst + u * 1024 : scratch);
    }
  };
  // unit u of the activation tile of `chunk` (a dummy if there is no such unit)
  auto issue_halo_unit = [&](int chunk, int u) {
    const int pix = u * RPU + urow;
    const int g = ugran ^ ((pix >> SWZ_SHIFT) & (GPR - 1));
    const int slot = fdiv(pix, p.dWv);
    const int w = pix - slot * p.Wv - p.pw;
    const int v = v_first + slot;
    const int n = fdiv(v, p.dHv);
    const int h = v - n * p.Hv - p.ph;
    const int ch = chunk * CB + g * 8;
    unsigned off = (unsigned)((n * p.act_n_stride + h * p.act_h_stride + w * p.act_w_stride + ch) * 2);
    const bool real = u < hunits && chunk < nchunks;
    const bool ok = real && pix < npix && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W &&
                    n < p.N && ch < p.C;
    if (!ok) off = OOB;
    dma16(act_rsrc, off, real ? halo + (chunk % p.nhb) * p.halo_stride + u * 1024 : scratch);
  };

  // LDS pixel row of this lane's output pixels (tap (0,0))
  int pixidx[PSUB];
#pragma unroll
  for (int t = 0; t < PSUB; ++t) {
    const int m = m0 + wave * (32 * PSUB) + t * 32 + (lane & 31);
    pixidx[t] = 0;
    if (m < p.M) {
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      const int ho = fdiv(rem, p.dWo);
      const int wo = rem - ho * p.Wo;
      pixidx[t] = (n * p.Hv + ho * p.sh - v_first) * p.Wv + wo * p.sw;
    }
  }
  const int kb = lane >> 5;
  // weight operand: byte offset of granule (2 kk + kb) of row (lane%32) for each kk
  int woff[CB / 16];
  {
    const int row = lane & 31;   // 32 | subtile stride, so the swizzle term depends on the lane only
#pragma unroll
    for (int kk = 0; kk < CB / 16; ++kk)
      woff[kk] = row * ROWB + (((2 * kk + kb) ^ ((row >> SWZ_SHIFT) & (GPR - 1))) * 16);
  }

  f32x16 acc[PSUB][NCH];
#pragma unroll
  for (int t = 0; t < PSUB; ++t)
#pragma unroll
    for (int r = 0; r < NCH; ++r)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][r][e] = 0.f;

  // ---- prologue: the copies steps -DIST .. -1 would have issued --------------------------------
  if (p.nhb == 4) {
    for (int s = 0; s < DIST; ++s) {
      for (int j = 0; j < p.hps; ++j) issue_halo_unit(cbeg + s, wave + NW * j);
      issue_weights(cbeg + s, 0, s);
    }
  } else {
    for (int u = wave; u < hunits; u += NW) issue_halo_unit(cbeg, u);
    for (int s = 0; s < DIST; ++s) {
      if (s > 0)
        for (int j = 0; j < p.hps; ++j) issue_halo_unit(nchunks, 0);   // dummies keep the count uniform
      const int c = s / taps;
      issue_weights(cbeg + c, s - c * taps, s);
    }
  }

  // position of the weight prefetch (step it + DIST)
  int pc = cbeg + DIST / taps, pt = DIST % taps;
  int it = 0;
  for (int c = cbeg; c < nchunks; ++c) {
    int tap = 0;
    const unsigned char* hb = halo + (c % p.nhb) * p.halo_stride;
    for (int ti = 0; ti < p.kH; ++ti) {
      for (int tj = 0; tj < p.kW; ++tj, ++tap, ++it) {
        wait_two_steps<WPW>(p.hps);
        block_barrier();   // this step's tiles have landed for every wave; last step's reads are done
        // activation slices of the chunk nhb-1 ahead, then the weights DIST steps ahead
        for (int j = 0; j < p.hps; ++j) {
          const bool live = tap < p.spread;
          issue_halo_unit(live ? c + p.nhb - 1 : nchunks, wave + NW * (tap * p.hps + j));
        }
        issue_weights(pc, pt, it + DIST);
        if (++pt == taps) { pt = 0; ++pc; }

        const int tapidx = ti * p.Wv + tj;
        const unsigned char* wb = wbuf + (it % NBUF) * (TRC * ROWB);
        int prow[PSUB], pswz[PSUB];
#pragma unroll
        for (int t = 0; t < PSUB; ++t) {
          const int r = pixidx[t] + tapidx;
          prow[t] = r * ROWB;
          pswz[t] = (r >> SWZ_SHIFT) & (GPR - 1);
        }
#pragma unroll
        for (int kk = 0; kk < CB / 16; ++kk) {
          bf16x8 a[NCH], b[PSUB];
#pragma unroll
          for (int t = 0; t < PSUB; ++t)
            b[t] = *reinterpret_cast<const bf16x8*>(hb + prow[t] + (((2 * kk + kb) ^ pswz[t]) * 16));
#pragma unroll
          for (int r = 0; r < NCH; ++r)
            a[r] = *reinterpret_cast<const bf16x8*>(wb + r * 32 * ROWB + woff[kk]);
#pragma unroll
          for (int t = 0; t < PSUB; ++t)
#pragma unroll
            for (int r = 0; r < NCH; ++r)
              acc[t][r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r], b[t], acc[t][r], 0, 0, 0);
        }
      }
    }
  }
  wait_vm<0>();   // trailing dummy copies must not outlive the workgroup's LDS

  // ---- epilogue -------------------------------------------------------------------------------
  // Accumulator element e of lane l: channel 8*(e/4) + 4*(l/32) + e%4, pixel l%32.  Each wave
  // rounds a 32-pixel x 64-channel block to bf16 into its own 4 KB of LDS ([pixel][64 ch], granules
  // swizzled by pixel), then reads it back row-wise so that every global store is 16 bytes per lane
  // and eight lanes cover one pixel's 128 contiguous bytes.
  if (p.ksplit > 1) {
    // fp32 partial sums of this workgroup's channel chunks; bias and rounding happen in the reduction
#pragma unroll
    for (int t = 0; t < PSUB; ++t) {
      const int m = m0 + wave * (32 * PSUB) + t * 32 + (lane & 31);
      if (m >= p.M) continue;
      float* orow = p.part + ((size_t)blockIdx.y * p.M + m) * p.R;
#pragma unroll
      for (int r = 0; r < NCH; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = r0 + r * 32 + q * 8 + kb * 4;
          if (row < p.R)
            *reinterpret_cast<float4*>(orow + row) = make_float4(acc[t][r][q * 4 + 0], acc[t][r][q * 4 + 1],
                                                                 acc[t][r][q * 4 + 2], acc[t][r][q * 4 + 3]);
        }
    }
    return;
  }
  block_barrier();   // every wave's copies have landed and every wave is done with the ring
  {
    unsigned char* stage = smem + 1024 + wave * 4096;   // behind the bias, over the (now idle) ring and tiles
    const int px = lane & 31;
    const int psw = (px >> 1) & 7;
#pragma unroll
    for (int t = 0; t < PSUB; ++t) {
      const int mbase = m0 + wave * (32 * PSUB) + t * 32;
#pragma unroll
      for (int rp = 0; rp < NCH / 2; ++rp) {
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2) {
          const int r = 2 * rp + r2;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int ch = r2 * 32 + q * 8 + kb * 4;          // channel inside this 64-channel block
            const float4 bb = *reinterpret_cast<const float4*>(biasl + r * 32 + q * 8 + kb * 4);
            const uint2 v = make_uint2(pack_bf16x2(acc[t][r][q * 4 + 0] + bb.x, acc[t][r][q * 4 + 1] + bb.y),
                                       pack_bf16x2(acc[t][r][q * 4 + 2] + bb.z, acc[t][r][q * 4 + 3] + bb.w));
            *reinterpret_cast<uint2*>(stage + px * 128 + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = i * 8 + (lane >> 3);
          const int g = (lane & 7) ^ ((row >> 1) & 7);
          const uint4 v = *reinterpret_cast<const uint4*>(stage + row * 128 + ((lane & 7) << 4));
          const int m = mbase + row;
          const int ch = r0 + rp * 64 + g * 8;
          if (m < p.M && ch < p.R) *reinterpret_cast<uint4*>(p.out + (size_t)m * p.R + ch) = v;
        }
      }
    }
  }
}

// out[m][r] = bf16( sum_s part[s][m][r] + bias[r] ), eight channels per thread (R % 8 == 0).
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int ksplit,
                                                              size_t MR, int R, const float* __restrict__ bias,
                                                              bf16_t* __restrict__ out) {
  const size_t nvec = MR >> 3;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) {
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int sp = 0; sp < ksplit; ++sp) {
      const float4 u = *reinterpret_cast<const float4*>(part + sp * MR + i * 8);
      const float4 v = *reinterpret_cast<const float4*>(part + sp * MR + i * 8 + 4);
      a[0] += u.x; a[1] += u.y; a[2] += u.z; a[3] += u.w;
      a[4] += v.x; a[5] += v.y; a[6] += v.z; a[7] += v.w;
    }
    if (bias) {
      const int r = (int)((i * 8) % R);
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] += bias[r + e];
    }
    *reinterpret_cast<uint4*>(out + i * 8) = make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]),
                                                        pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7]));
  }
}

// Largest number of LDS row slots any TP-pixel tile needs.
int max_slots(const TileParams& p, int TP) {
  const int HoWo = p.Ho * p.Wo;
  int a = HoWo, b = TP;
  while (b) { const int t = a % b; a = b; b = t; }
  const int period = HoWo / a;   // tile starts repeat modulo the image size after `period` tiles
  int best = 0;
  for (int m0 = 0, t = 0; m0 < p.M && t <= period; m0 += TP, ++t) {
    const int ml = (m0 + TP < p.M ? m0 + TP : p.M) - 1;
    const int na = m0 / HoWo, hoa = (m0 - na * HoWo) / p.Wo;
    const int nb = ml / HoWo, hob = (ml - nb * HoWo) / p.Wo;
    const int ns = nb * p.Hv + hob * p.sh + p.kH - (na * p.Hv + hoa * p.sh);
    if (ns > best) best = ns;
  }
  return best;
}

struct TilePlan { bool ok; int nw, psub, nch, cb; size_t lds; };

// fp32 partial-output bytes a problem needs (0 when the channel chunks are not split).
size_t partial_bytes(const TileParams& p) {
  return p.ksplit > 1 ? (size_t)p.ksplit * p.M * p.R * 4 : 0;
}

constexpr size_t LDS_LIMIT = 160 * 1024;
constexpr size_t LDS_USABLE = LDS_LIMIT - 1024;
constexpr size_t LDS_TWO_PER_CU = 80 * 1024;   // two workgroups of up to this size share one CU

// Fills nhb / hps / spread / halo_stride for (psub, nch, cb); returns the LDS bytes (0 = impossible).
size_t plan_lds(TileParams& p, int nw, int psub, int nch, int cb) {
  const int taps = p.kH * p.kW;
  if (p.C % cb) return 0;
  // split the channel chunks over several workgroups when the pixel x channel tiling alone
  // leaves most of the chip idle
  const int all_chunks = p.C / cb;
  const long long blocks = (long long)ceil_div(p.M, 32 * nw * psub) * ceil_div(p.R, nch * 32);
  int ks = 1;
  if (blocks < 200 && all_chunks >= 4) {
    ks = (int)((400 + blocks - 1) / blocks);
    if (ks > all_chunks / 2) ks = all_chunks / 2;
    if (ks > 8) ks = 8;
  }
  p.chunks_per_split = ceil_div(all_chunks, ks);
  p.ksplit = ceil_div(all_chunks, p.chunks_per_split);
  const int nchunks = p.chunks_per_split;
  const size_t rowb = (size_t)cb * 2;
  const int rpu = (int)(1024 / rowb);
  const int slots = max_slots(p, 32 * nw * psub);
  const int hunits = ceil_div(slots * p.Wv, rpu);
  const int per_wave = ceil_div(hunits, nw);
  int nhb, spread, need;
  if (nchunks == 1) { nhb = 1; spread = 0; need = 0; }
  else if (taps == 1) { nhb = 4; spread = 1; need = per_wave; }
  else if (taps > DIST) { nhb = 2; spread = taps - DIST; need = ceil_div(per_wave, spread); }
  else return 0;
  int hps = 0;
  if (need > 0) { hps = 1; while (hps < need) hps *= 2; }
  if (hps > 8) return 0;
  if (hps == 0) spread = 0;
  p.nhb = nhb; p.hps = hps; p.spread = spread;
  p.halo_stride = hunits * 1024;
  const size_t lds = (size_t)NBUF * nch * 32 * rowb + 2 * 1024 + (size_t)nhb * p.halo_stride;
  const size_t stage = 1024 + (size_t)nw * 4096;   // the epilogue stages 4 KB per wave behind the bias
  return lds < stage ? stage : lds;
}

TilePlan make_plan(TileParams& p) {
  TilePlan pl{false, 0, 0, 0, 0, 0};
  if (p.C % 8 || p.R % 8) return pl;
  if (p.act_bytes >= OOB || p.wgt_bytes >= OOB) return pl;   // byte offsets must stay below the zero-fill offset
  p.dHoWo = make_fastdiv(p.Ho * p.Wo);
  p.dWo = make_fastdiv(p.Wo);
  p.dHv = make_fastdiv(p.Hv);
  p.dWv = make_fastdiv(p.Wv);
  pl.nch = p.R > 64 ? 4 : 2;
  // 256-pixel tiles run by eight waves when that still yields ~1.5 workgroups per CU, else
  // 128-pixel tiles run by four; one 32-pixel subtile per wave either way
  const long long blocks256 = (long long)ceil_div(p.M, 256) * ceil_div(p.R, pl.nch * 32);
  pl.nw = (blocks256 >= 384 || p.M >= 4096) ? 8 : 4;
  pl.psub = 1;
  // 64-channel chunks when two workgroups still share one CU's LDS, else 32-channel chunks
  TileParams q = p;
  size_t lds = p.C > 32 ? plan_lds(q, pl.nw, pl.psub, pl.nch, 64) : 0;
  pl.cb = 64;
  if (lds == 0 || lds > LDS_TWO_PER_CU) {
    TileParams q32 = p;
    const size_t lds32 = plan_lds(q32, pl.nw, pl.psub, pl.nch, 32);
    if (lds32 != 0 && (lds == 0 || lds32 <= LDS_TWO_PER_CU || lds > LDS_USABLE)) { q = q32; lds = lds32; pl.cb = 32; }
  }
  if (lds == 0 || lds > LDS_USABLE) return pl;
  p = q;
  pl.lds = lds;
  p.ntr = ceil_div(p.R, pl.nch * 32);
  pl.ok = true;
  return pl;
}

template <int NW, int PSUB, int NCH, int CB>
hipError_t launch_inst(const TileParams& p, const TilePlan& pl, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_tile_kernel<NW, PSUB, NCH, CB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_USABLE);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int ptiles = ceil_div(p.M, 32 * NW * PSUB);
  hipLaunchKernelGGL((conv_tile_kernel<NW, PSUB, NCH, CB>), dim3(p.ntr * ptiles, p.ksplit), dim3(64 * NW), pl.lds, st, p);
  hipError_t le = hipGetLastError();
  if (le != hipSuccess || p.ksplit == 1) return le;
  const size_t MR = (size_t)p.M * p.R;
  const int rblocks = (int)(((MR >> 3) + 255) / 256 < 2048 ? ((MR >> 3) + 255) / 256 : 2048);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(rblocks), dim3(256), 0, st, p.part, p.ksplit, MR, p.R, p.bias, p.out);
  return hipGetLastError();
}

hipError_t launch_plan(const TileParams& p, const TilePlan& pl, hipStream_t st) {
#define CASE(NWV, PS, NC, CBV) \
  if (pl.nw == NWV && pl.psub == PS && pl.nch == NC && pl.cb == CBV) return launch_inst<NWV, PS, NC, CBV>(p, pl, st);
  CASE(4, 1, 2, 32) CASE(4, 1, 2, 64) CASE(4, 1, 4, 32) CASE(4, 1, 4, 64)
  CASE(8, 1, 2, 32) CASE(8, 1, 2, 64) CASE(8, 1, 4, 32) CASE(8, 1, 4, 64)
  CASE(4, 2, 2, 32) CASE(4, 2, 2, 64) CASE(4, 2, 4, 32) CASE(4, 2, 4, 64)
#undef CASE
  return hipErrorInvalidValue;
}

bool fprop_params(const Geom& g, TileParams* p) {
  TileParams& q = *p;
  q = TileParams{};
  q.N = g.N; q.C = g.Cin; q.Ho = g.Hout; q.Wo = g.Wout; q.R = g.Cout; q.M = g.M;
  q.kH = g.kH; q.kW = g.kW; q.flip = 0;
  if (g.kH == 1 && g.kW == 1 && g.ph == 0 && g.pw == 0) {
    // a 1x1 window with stride s reads the s-subsampled grid: slide with stride 1 over that grid
    q.H = g.Hout; q.W = g.Wout; q.sh = 1; q.sw = 1; q.ph = 0; q.pw = 0;
    q.act_h_stride = g.sh * g.Win * g.Cin;
    q.act_w_stride = g.sw * g.Cin;
  } else {
    q.H = g.Hin; q.W = g.Win; q.sh = g.sh; q.sw = g.sw; q.ph = g.ph; q.pw = g.pw;
    q.act_h_stride = g.Win * g.Cin;
    q.act_w_stride = g.Cin;
  }
  q.act_n_stride = g.Hin * g.Win * g.Cin;
  q.act_bytes = (unsigned)((size_t)g.N * g.Hin * g.Win * g.Cin * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  q.Hv = (q.Ho - 1) * q.sh + q.kH;
  q.Wv = (q.Wo - 1) * q.sw + q.kW;
  return true;
}

bool dgrad_params(const Geom& g, TileParams* p) {
  if (g.sh != 1 || g.sw != 1) return false;
  if (g.ph > g.kH - 1 || g.pw > g.kW - 1) return false;
  TileParams& q = *p;
  q = TileParams{};
  q.N = g.N; q.C = g.Cout; q.H = g.Hout; q.W = g.Wout;
  q.Ho = g.Hin; q.Wo = g.Win; q.R = g.Cin; q.M = g.Min;
  q.kH = g.kH; q.kW = g.kW; q.sh = 1; q.sw = 1;
  q.ph = g.kH - 1 - g.ph; q.pw = g.kW - 1 - g.pw; q.flip = 1;
  q.act_n_stride = g.Hout * g.Wout * g.Cout;
  q.act_h_stride = g.Wout * g.Cout;
  q.act_w_stride = g.Cout;
  q.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  q.Hv = (q.Ho - 1) + q.kH;
  q.Wv = (q.Wo - 1) + q.kW;
  return true;
}

}  // namespace

bool tile_fprop_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  TileParams p;
  return fprop_params(g, &p) && make_plan(p).ok;
}

bool tile_dgrad_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  TileParams p;
  return dgrad_params(g, &p) && make_plan(p).ok;
}

size_t tile_fprop_partial_bytes(const Geom& g) {
  TileParams p;
  if (!fprop_params(g, &p) || !make_plan(p).ok) return 0;
  return partial_bytes(p);
}

size_t tile_dgrad_partial_bytes(const Geom& g) {
  TileParams p;
  if (!dgrad_params(g, &p) || !make_plan(p).ok) return 0;
  return partial_bytes(p);
}

hipError_t launch_fprop_tile(const Geom& g, const void* x, const void* w_krsc, const float* bias,
                             void* z, float* partials, hipStream_t st) {
  TileParams p;
  fprop_params(g, &p);
  const TilePlan pl = make_plan(p);
  if (p.ksplit > 1 && !partials) return hipErrorInvalidValue;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_krsc; p.bias = bias; p.out = (bf16_t*)z;
  p.part = partials;
  return launch_plan(p, pl, st);
}

hipError_t launch_dgrad_tile(const Geom& g, const void* dz, const void* w_crsk, void* dx,
                             float* partials, hipStream_t st) {
  TileParams p;
  dgrad_params(g, &p);
  const TilePlan pl = make_plan(p);
  if (p.ksplit > 1 && !partials) return hipErrorInvalidValue;
  p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = nullptr; p.out = (bf16_t*)dx;
  p.part = partials;
  return launch_plan(p, pl, st);
}

}  // namespace convbn
