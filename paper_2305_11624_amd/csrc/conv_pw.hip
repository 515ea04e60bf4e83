// Pointwise (1x1, stride 1, unpadded) bf16 convolution as a persistent,
// weight-stationary streaming product
//     out[m][r] = sum_c act[m][c] wgt[r][c] (+ bias[r]),     m over all N*H*W pixels:
//   forward conv   Z  = w' (*) X + b'   (Sec. 3.1 / 3.3)   act = x,   wgt = w' as [Cout][Cin]
//   input gradient dX = w'_rot (*) dZ   (Sec. 3.2.1)       act = dz,  wgt = w' as [Cin][Cout]
//
// (Shapes the tiled product of conv_gm.hip takes -- most layers of a ResNet-50, and every strided pointwise layer -- are
// handed on to it by the launch functions at the end of this file; this kernel keeps the rest.)
//
// Most of these layers move many MB of activations for a few GFLOP: they are bound by memory (or by the
// global->LDS copy path), and a kernel that hands every pixel tile to a workgroup of its own pays that workgroup's
// start-up (weights, tables, first copies in flight) and drain (stores) once per tile, with the memory
// idle in between.  Here a workgroup keeps its [TRC][C] block of the weights in LDS for its whole life
// and walks over pixel tiles g, g + G, g + 2G, ...: [TP pixels][CB channels] activation slabs stream
// through a ring of LDS slots (direct global->LDS copies, DIST steps ahead, across tile boundaries), and
// a finished output tile is rounded, staged through LDS and stored from inside the loop while the
// copies of the following tiles are already in flight.
//
// LDS rows carry one 16-byte pad granule (see conv_tile.hip: 128-bit operand reads of 16 consecutive rows
// then fall on distinct banks), so a 1 KB copy covers RPU whole rows; every wave issues the same number
// of copies per step (a surplus copy repeats another unit), which makes "at most n copies outstanding"
// mean "everything issued DIST-1 or more steps ago has landed".  The stores of the epilogue share the
// counter with the copies; they can only make such a wait longer, never shorter.
#include "common.h"

#include <type_traits>

namespace convbn {

namespace {

struct PwDiv { unsigned mul, shr; int d; };   // exact n / d for 0 <= n < 2^31
PwDiv make_div(int d) {
  PwDiv f{0u, 0u, d};
  if (d <= 1) return f;
  unsigned sh = 0;
  while ((1ull << (sh + 1)) < (unsigned long long)d) ++sh;   // 2^sh < d <= 2^(sh+1)
  f.shr = sh;
  f.mul = (unsigned)((((unsigned long long)1 << (32 + sh)) + d - 1) / d);
  return f;
}
__device__ __forceinline__ int pdiv(int n, const PwDiv& f) {
  return f.d == 1 ? n : (int)(__umulhi((unsigned)n, f.mul) >> f.shr);
}

struct PwParams {
  const bf16_t* act;     // [M][C]
  const bf16_t* wgt;     // [R][C]
  const float* bias;     // [R] or null
  BnEpilogue bn;         // bn.gamma != null: the weight is unfolded, the epilogue applies s and b' (bias unused)
  bf16_t* out;           // [M][R]
  int relu;              // the output leaves as max(., 0)
  const bf16_t* mask;    // not null: [M][R], the output is zeroed where this is <= 0
  const bf16_t* add;     // not null: [M][R], added to the (rounded) output before the ReLU and the mask
  unsigned act_bytes, wgt_bytes;
  int M, C, R;
  int ntr;               // channel tiles
  int groups;            // workgroups per channel tile; group g owns pixel tiles g, g + groups, ...
  int ntiles, nchunks;
  int wpitch;            // LDS bytes per weight row: 2 C + 16
  int wtile_bytes;       // TRC rows of wpitch bytes, rounded up to whole 1 KB copies
  // Depth-to-space output (d2s_co > 0): the R channels are (tap, co) pairs, tap = (a, b) of a kh x kw window, and
  // channel block tap of pixel (n, h, w) is stored at pixel (n, h kh + a, w kw + b) of an [N][H kh][W kw][co] tensor --
  // a transposed convolution whose stride equals its window (Sec. 3.2.1) is exactly this product.
  int d2s_co, d2s_kh, d2s_kw, d2s_H, d2s_W;
  PwDiv d_co, d_kw, d_HW, d_W;
};

constexpr unsigned OOB = 0x80000000u;   // beyond any buffer: the load returns zeros

typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
// 1 KB copy: lane l fetches 16 bytes at voff (per lane) + soff (wave-uniform) and writes them to LDS at
// lds_wave_base + 16 l.  The compiler barrier keeps every copy in the instruction stream (the waits count
// copies; two copies to the same LDS range would otherwise be merged).
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)voff, (int)soff, 0, 0);
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void block_barrier() {   // no memory fence: that would drain the copies
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
template <int N> __device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int NW, int CB> struct PwCfg {
  static constexpr int TP = 32 * NW;           // pixels per tile (one 32-pixel group per wave)
  static constexpr int GPR = CB / 8;
  static constexpr int LPR = GPR + 1;
  static constexpr int RPU = 64 / LPR;         // rows per 1 KB copy: 7 (CB 64) / 12 (CB 32)
  static constexpr int ROWP = LPR * 16;        // 144 / 80 bytes
  static constexpr int UNITB = RPU * ROWP;
  static constexpr int KK = CB / 16;
  static constexpr int NBUF = CB == 64 ? 4 : 5;
  static constexpr int DIST = NBUF - 1;
  static constexpr int AUNITS = (TP + RPU - 1) / RPU;
  static constexpr int APW = (AUNITS + NW - 1) / NW;   // copies per wave and step
  static constexpr int SLOT = AUNITS * UNITB + 64;
};

// SC: unfolded weight, BatchNorm scale and folded bias applied by the epilogue (an instantiation of its own).
template <int NW, int NCH, int CB, bool SC = false>
__global__ __launch_bounds__(64 * NW) void conv_pw_kernel(PwParams p) {
  using Cfg = PwCfg<NW, CB>;
  constexpr int TP = Cfg::TP, TRC = 32 * NCH, GPR = Cfg::GPR, LPR = Cfg::LPR, RPU = Cfg::RPU, ROWP = Cfg::ROWP;
  constexpr int UNITB = Cfg::UNITB, KK = Cfg::KK, NBUF = Cfg::NBUF, DIST = Cfg::DIST;
  constexpr int AUNITS = Cfg::AUNITS, APW = Cfg::APW, SLOT = Cfg::SLOT;
  static_assert(NCH % 2 == 0 && AUNITS < 2 * NW * APW && NW * APW < 2 * AUNITS, "tile shape");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* biasl = reinterpret_cast<float*>(smem);              // [TRC]
  unsigned char* stage = smem + 1024;                         // [NW][4 KB] output staging, one per wave
  unsigned char* wtile = stage + NW * 4096;                   // [TRC][wpitch] weights, resident
  unsigned char* ring = wtile + p.wtile_bytes;                // [NBUF][SLOT] activation slabs

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ctile = blockIdx.x % p.ntr, grp = blockIdx.x / p.ntr;
  const int r0 = ctile * TRC;
  const int my_tiles = (p.ntiles - grp + p.groups - 1) / p.groups;
  const int nsteps = my_tiles * p.nchunks;
  const int tile_stride = p.groups * TP;                      // pixels between two tiles of this workgroup
  const __amdgpu_buffer_rsrc_t act_rsrc = make_rsrc(p.act, p.act_bytes);
  const __amdgpu_buffer_rsrc_t wgt_rsrc = make_rsrc(p.wgt, p.wgt_bytes);

  if (tid < TRC) {
    float bias_v = (p.bias && r0 + tid < p.R) ? p.bias[r0 + tid] : 0.f, scale_v = 1.f;
    if (SC && r0 + tid < p.R) {
      const int ch = r0 + tid;
      scale_v = p.bn.gamma[ch] / sqrtf(p.bn.var[ch] + p.bn.eps);
      bias_v = ((p.bn.b ? p.bn.b[ch] : 0.f) - p.bn.mean[ch]) * scale_v + p.bn.beta[ch];
    }
    biasl[tid] = bias_v;
    if (SC) biasl[128 + tid] = scale_v;   // scales behind the (at most 128) biases
  }

  // ---- the weight block: LDS byte o of the tile is row o / wpitch, byte o % wpitch (the last 16: pad)
  for (int u = wave; u * 1024 < p.wtile_bytes; u += NW) {
    const int o = u * 1024 + lane * 16;
    const int row = o / p.wpitch, col = o - row * p.wpitch;
    const bool ok = row < TRC && r0 + row < p.R && col < 2 * p.C;
    dma16(wgt_rsrc, ok ? (unsigned)((r0 + row) * p.C * 2 + col) : OOB, 0u, wtile + u * 1024);
  }

  // ---- this wave's activation copies of a step: unit u covers tile rows u RPU .. (its last lanes the head
  // of the following row, which the next unit writes again with the same values)
  const int lrow = lane / LPR, lgran = lane - lrow * LPR;
  unsigned voff_a[APW];
  int row_a[APW], au_off[APW];
#pragma unroll
  for (int j = 0; j < APW; ++j) {
    int u = wave + NW * j;
    u = u < AUNITS ? u : u - AUNITS;
    const int row = u * RPU + lrow;
    const bool ok = row < TP && lgran < GPR;
    voff_a[j] = ok ? (unsigned)((row * p.C + lgran * 8) * 2) : OOB;
    row_a[j] = ok ? row : 0x7fffffff;
    au_off[j] = u * UNITB;
  }
  // copy position (the step DIST ahead of the one being multiplied; at the end it stays on the last step,
  // whose slab it fetches again into a slot nobody reads any more)
  int ct = 0, cc = 0, cm0 = grp * TP;
  auto issue_copy = [&](int j, int slot_off) {
    const int lim = p.M - cm0;                                // rows of the tile that exist
    const unsigned soff = (unsigned)((cm0 * p.C + cc * CB) * 2);
    dma16(act_rsrc, row_a[j] < lim ? voff_a[j] : OOB, soff, ring + slot_off + au_off[j]);
  };
  auto advance_copy = [&]() {
    const bool last = ct == my_tiles - 1 && cc == p.nchunks - 1;
    const bool wrap = cc + 1 == p.nchunks;
    if (!last) {
      cc = wrap ? 0 : cc + 1;
      ct += wrap ? 1 : 0;
      cm0 += wrap ? tile_stride : 0;
    }
  };
#pragma unroll
  for (int s = 0; s < DIST; ++s) {
#pragma unroll
    for (int j = 0; j < APW; ++j) issue_copy(j, s * SLOT);
    advance_copy();
  }

  // ---- operand addresses: this wave multiplies pixels 32 wave .. of the tile with all TRC channels
  const int kb = lane >> 5;
  const unsigned boff = (unsigned)((wave * 32 + (lane & 31)) * ROWP + kb * 16);
  const unsigned char* const wlane = wtile + (lane & 31) * p.wpitch + kb * 16;
  const int wsub = 32 * p.wpitch;                              // bytes between two 32-channel subtiles

  f32x16 acc[NCH];
#pragma unroll
  for (int r = 0; r < NCH; ++r)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[r][e] = 0.f;

  bf16x8 fa[2][NCH], fb[2];
  auto load_frags = [&](int buf, int slot_off, int coff, int kk) {
    fb[buf] = *reinterpret_cast<const bf16x8*>(ring + slot_off + boff + kk * 32);
#pragma unroll
    for (int r = 0; r < NCH; ++r) fa[buf][r] = *reinterpret_cast<const bf16x8*>(wlane + r * wsub + coff + kk * 32);
  };

  int c = 0, m0 = grp * TP;                                    // chunk and first pixel of the current step

  // Where this lane's 16 bytes of epilogue store (rp, i) go: element offset into out, or -1 past the tensor.  Row
  // i * 8 + lane / 8 of the wave's 32 pixels, granule (lane % 8) ^ swizzle of the 64-channel pair rp.
  auto out_off = [&](int rp, int i, int m_first) -> long long {
    const int row = i * 8 + (lane >> 3);
    const int g = (lane & 7) ^ ((row >> 1) & 7);
    const int pi = wave * 32 + row;
    const int ch = r0 + rp * 64 + g * 8;
    if (pi >= min(TP, p.M - m_first) || ch >= p.R) return -1;
    size_t o = (size_t)(m_first + pi) * p.R + ch;
    if (p.d2s_co > 0) {
      const int tap = pdiv(r0 + rp * 64, p.d_co);          // the whole 64-channel block is one tap's
      const int ta = pdiv(tap, p.d_kw), tb = tap - ta * p.d2s_kw;
      const int m = m_first + pi;
      const int n = pdiv(m, p.d_HW), rem = m - n * (p.d2s_H * p.d2s_W);
      const int h = pdiv(rem, p.d_W), w = rem - h * p.d2s_W;
      o = (((size_t)n * (p.d2s_H * p.d2s_kh) + h * p.d2s_kh + ta) * (p.d2s_W * p.d2s_kw) + w * p.d2s_kw + tb) *
              p.d2s_co + (ch - tap * p.d2s_co);
    }
    return (long long)o;
  };
  // The addend and the mask of a tile's outputs are requested when the tile's last chunk begins, a step before
  // the epilogue needs them: loads return in order, so a load issued in the epilogue itself would wait for every
  // copy of the following steps that is already in flight -- the ring would drain once per tile.
  const bool has_post = p.add != nullptr || p.mask != nullptr;
  uint4 addv[NCH / 2][4], maskv[NCH / 2][4];
  wait_vm<(DIST - 1) * APW>();   // the weights and the slab of step 0 have landed
  __syncthreads();               // (the bias too)
  load_frags(0, 0, 0, 0);

  auto step = [&](auto slot) {
    constexpr int S = decltype(slot)::value;
    constexpr int SN = (S + 1) % NBUF, SF = (S + NBUF - 1) % NBUF;
    const bool tile_end = c + 1 == p.nchunks;
    const int nc = tile_end ? 0 : c + 1;
    wait_vm<(DIST - 2) * APW>();
    block_barrier();   // the next step's slab is resident for every wave; the previous step's slot is free
    if (tile_end && has_post) {
#pragma unroll
      for (int rp = 0; rp < NCH / 2; ++rp)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const long long o = out_off(rp, i, m0);
          addv[rp][i] = (p.add && o >= 0) ? *reinterpret_cast<const uint4*>(p.add + o) : make_uint4(0u, 0u, 0u, 0u);
          maskv[rp][i] = (p.mask && o >= 0) ? *reinterpret_cast<const uint4*>(p.mask + o) : make_uint4(0u, 0u, 0u, 0u);
        }
    }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) load_frags((kk + 1) & 1, S * SLOT, c * CB * 2, kk + 1);
      else load_frags((kk + 1) & 1, SN * SLOT, nc * CB * 2, 0);
      __builtin_amdgcn_sched_barrier(0);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][0], fb[kk & 1], acc[0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = (kk * APW) / KK; j < ((kk + 1) * APW) / KK; ++j) issue_copy(j, SF * SLOT);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 1; r < NCH; ++r)
        acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][r], fb[kk & 1], acc[r], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    advance_copy();
    if (tile_end) {
      // Output tile: accumulator element e of lane l is channel 8 (e / 4) + 4 (l / 32) + e % 4, pixel l % 32.
      // Each wave rounds 32 pixels x 64 channels to bf16 into its 4 KB of LDS ([pixel][64 ch], granules
      // swizzled by pixel) and reads them back row-wise: every store is 16 bytes per lane, eight lanes
      // cover one pixel's 128 contiguous bytes.
      unsigned char* const st = stage + wave * 4096;
      const int px = lane & 31, psw = (px >> 1) & 7;
#pragma unroll
      for (int rp = 0; rp < NCH / 2; ++rp) {
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2) {
          const int r = 2 * rp + r2;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int ch = r2 * 32 + q * 8 + kb * 4;
            const float4 bb = *reinterpret_cast<const float4*>(biasl + r * 32 + q * 8 + kb * 4);
            uint2 v;
            if constexpr (SC) {   // unfolded weight: the BatchNorm scale is applied here
              const float4 sc = *reinterpret_cast<const float4*>(biasl + 128 + r * 32 + q * 8 + kb * 4);
              v = make_uint2(pack_bf16x2(fmaf(acc[r][q * 4 + 0], sc.x, bb.x), fmaf(acc[r][q * 4 + 1], sc.y, bb.y)),
                             pack_bf16x2(fmaf(acc[r][q * 4 + 2], sc.z, bb.z), fmaf(acc[r][q * 4 + 3], sc.w, bb.w)));
            } else {
              v = make_uint2(pack_bf16x2(acc[r][q * 4 + 0] + bb.x, acc[r][q * 4 + 1] + bb.y),
                             pack_bf16x2(acc[r][q * 4 + 2] + bb.z, acc[r][q * 4 + 3] + bb.w));
            }
            *reinterpret_cast<uint2*>(st + px * 128 + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[r][q * 4 + e] = 0.f;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = i * 8 + (lane >> 3);
          uint4 v = *reinterpret_cast<const uint4*>(st + row * 128 + ((lane & 7) << 4));
          const long long o = out_off(rp, i, m0);
          if (p.add) v = add8(v, addv[rp][i]);
          if (p.relu) v = relu8(v);
          if (p.mask) v = mask8(v, maskv[rp][i]);
          if (o >= 0) *reinterpret_cast<uint4*>(p.out + o) = v;
        }
      }
      m0 += tile_stride;
    }
    c = nc;
  };
  for (int left = nsteps;;) {
    step(std::integral_constant<int, 0>{}); if (--left == 0) break;
    step(std::integral_constant<int, 1>{}); if (--left == 0) break;
    step(std::integral_constant<int, 2>{}); if (--left == 0) break;
    step(std::integral_constant<int, 3>{}); if (--left == 0) break;
    if constexpr (NBUF == 5) { step(std::integral_constant<int, 4>{}); if (--left == 0) break; }
  }
  wait_vm<0>();   // trailing copies must not outlive the workgroup's LDS
}

constexpr size_t LDS_USABLE = 159 * 1024;
constexpr int MIN_WORK = 128;   // (pixel tiles x channel tiles) below which the per-tile kernels are used

struct PwPlan { bool ok; int nch, cb; size_t lds; };

template <int NW, int CB> size_t plan_cfg(PwParams& p, int nch) {
  using Cfg = PwCfg<NW, CB>;
  if (p.C % CB) return 0;
  const int TRC = 32 * nch;
  p.wpitch = 2 * p.C + 16;
  p.wtile_bytes = (int)align_up((size_t)TRC * p.wpitch, 1024);
  p.nchunks = p.C / CB;
  p.ntiles = ceil_div(p.M, Cfg::TP);
  p.ntr = ceil_div(p.R, TRC);
  // about one workgroup per CU, every workgroup the same number of tiles where that is possible
  int groups = 256 / p.ntr;
  if (groups < 1) groups = 1;
  const int per_group = ceil_div(p.ntiles, groups);
  p.groups = ceil_div(p.ntiles, per_group);
  return 1024 + (size_t)NW * 4096 + p.wtile_bytes + (size_t)Cfg::NBUF * Cfg::SLOT;
}

PwPlan make_plan(PwParams& p) {
  PwPlan pl{false, 0, 0, 0};
  if (p.C % 16 || p.R % 8) return pl;
  if ((size_t)p.M * p.C * 2 >= OOB || (size_t)p.M * p.R * 2 >= OOB || (size_t)p.R * p.C * 2 >= OOB) return pl;
  // 128 output channels per workgroup where the weight block then still fits next to the ring, else 64
  for (int nch : {p.R > 64 ? 4 : 2, 2})
    for (int cb : {64, 32}) {
      PwParams q = p;
      const size_t lds = cb == 64 ? plan_cfg<4, 64>(q, nch) : plan_cfg<4, 32>(q, nch);
      if (lds == 0 || lds > LDS_USABLE || q.ntiles * q.ntr < MIN_WORK) continue;
      // the narrower block doubles the passes over the activations: measured to pay only with many tiles
      if (nch == 2 && p.R > 64 && q.ntiles < MIN_WORK) continue;
      p = q;
      pl.nch = nch; pl.cb = cb; pl.lds = lds; pl.ok = true;
      return pl;
    }
  return pl;
}

template <int NW, int NCH, int CB, bool SC = false>
hipError_t launch_inst(const PwParams& p, const PwPlan& pl, hipStream_t st) {
  static LdsLimitOnce lds_once;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&conv_pw_kernel<NW, NCH, CB, SC>),
                                        (int)LDS_USABLE); e != hipSuccess) return e;
  hipLaunchKernelGGL((conv_pw_kernel<NW, NCH, CB, SC>), dim3(p.ntr * p.groups), dim3(64 * NW), pl.lds, st, p);
  return hipGetLastError();
}

hipError_t launch_plan(const PwParams& p, const PwPlan& pl, hipStream_t st) {
  if (p.bn.gamma) {   // the ablation is built for 64-channel chunks
    if (pl.nch == 2 && pl.cb == 64) return launch_inst<4, 2, 64, true>(p, pl, st);
    if (pl.nch == 4 && pl.cb == 64) return launch_inst<4, 4, 64, true>(p, pl, st);
    return hipErrorInvalidValue;
  }
  if (pl.nch == 2 && pl.cb == 64) return launch_inst<4, 2, 64>(p, pl, st);
  if (pl.nch == 2 && pl.cb == 32) return launch_inst<4, 2, 32>(p, pl, st);
  if (pl.nch == 4 && pl.cb == 64) return launch_inst<4, 4, 64>(p, pl, st);
  if (pl.nch == 4 && pl.cb == 32) return launch_inst<4, 4, 32>(p, pl, st);
  return hipErrorInvalidValue;
}

bool pointwise(const Geom& g) {
  return g.kH == 1 && g.kW == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0;
}
// a downsampling shortcut: 1x1 window, a stride, no padding -- the product over the output pixels, whose input rows
// (forward) or output rows (input gradient) are every stride-th pixel
bool strided_pointwise(const Geom& g) {
  return g.kH == 1 && g.kW == 1 && (g.sh > 1 || g.sw > 1) && g.ph == 0 && g.pw == 0 && g.Cin % 8 == 0 && g.Cout % 8 == 0;
}
GmStride stride_of(const Geom& g, int scatter) {
  return GmStride{scatter, g.N, g.Hout, g.Wout, g.Hin, g.Win, g.sh, g.sw};
}
bool strided_fits(const Geom& g) { return (size_t)g.Min * g.Cin * 2 < OOB && (size_t)g.M * g.Cout * 2 < OOB; }
PwParams fprop_params(const Geom& g) {
  PwParams p{};
  p.M = g.M; p.C = g.Cin; p.R = g.Cout;
  p.act_bytes = (unsigned)((size_t)g.M * g.Cin * 2);
  p.wgt_bytes = (unsigned)((size_t)g.Cout * g.Cin * 2);
  return p;
}
PwParams dgrad_params(const Geom& g) {
  PwParams p{};
  p.M = g.M; p.C = g.Cout; p.R = g.Cin;
  p.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  p.wgt_bytes = (unsigned)((size_t)g.Cout * g.Cin * 2);
  return p;
}

// forward of a transposed convolution whose stride equals its window (no padding): g is the convolution it is
// the adjoint of, so the product runs over g's OUTPUT pixels with g.Cout reduced and taps x g.Cin produced channels
bool d2s_shape(const Geom& g) {
  return g.kH == g.sh && g.kW == g.sw && g.ph == 0 && g.pw == 0 && g.kH * g.kW > 1 && g.Cin % 64 == 0 &&
         g.Hin == g.Hout * g.kH && g.Win == g.Wout * g.kW;
}
PwParams d2s_params(const Geom& g) {
  PwParams p{};
  p.M = g.M; p.C = g.Cout; p.R = g.kH * g.kW * g.Cin;
  p.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  p.wgt_bytes = (unsigned)((size_t)p.R * g.Cout * 2);
  p.d2s_co = g.Cin; p.d2s_kh = g.kH; p.d2s_kw = g.kW; p.d2s_H = g.Hout; p.d2s_W = g.Wout;
  p.d_co = make_div(g.Cin); p.d_kw = make_div(g.kW); p.d_HW = make_div(g.Hout * g.Wout); p.d_W = make_div(g.Wout);
  return p;
}

}  // namespace

bool pw_tconv_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16 || !d2s_shape(g)) return false;
  PwParams p = d2s_params(g);
  return make_plan(p).ok;
}
hipError_t launch_tconv_pw(const Geom& g, const void* x, const void* w_tap_major, const float* bias_per_tap, void* z,
                           hipStream_t st) {
  PwParams p = d2s_params(g);
  const PwPlan pl = make_plan(p);
  if (!pl.ok) return hipErrorInvalidValue;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_tap_major; p.bias = bias_per_tap; p.out = (bf16_t*)z;
  return launch_plan(p, pl, st);
}

bool pw_fprop_scaled_supported(const Geom& g, int dtype) {
  if (dtype == CONVBN_BF16 && strided_pointwise(g)) return strided_fits(g) && gm_supported(g.M, g.Cin, g.Cout);
  if (dtype != CONVBN_BF16 || !pointwise(g)) return false;
  if (gm_supported(g.M, g.Cin, g.Cout)) return true;
  PwParams p = fprop_params(g);
  const PwPlan pl = make_plan(p);
  return pl.ok && pl.cb == 64;
}
bool pw_fprop_supported(const Geom& g, int dtype) {
  if (dtype == CONVBN_BF16 && strided_pointwise(g)) return strided_fits(g) && gm_supported(g.M, g.Cin, g.Cout);
  if (dtype != CONVBN_BF16 || !pointwise(g)) return false;
  if (gm_supported(g.M, g.Cin, g.Cout)) return true;
  PwParams p = fprop_params(g);
  return make_plan(p).ok;
}
bool pw_dgrad_supported(const Geom& g, int dtype) {
  if (dtype == CONVBN_BF16 && strided_pointwise(g)) return strided_fits(g) && gm_supported(g.M, g.Cout, g.Cin);
  if (dtype != CONVBN_BF16 || !pointwise(g)) return false;
  if (gm_supported(g.M, g.Cout, g.Cin)) return true;
  PwParams p = dgrad_params(g);
  return make_plan(p).ok;
}
hipError_t launch_fprop_pw(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z,
                           hipStream_t st, const BnEpilogue* bn) {
  if (strided_pointwise(g)) {
    const GmStride sd = stride_of(g, 0);
    return launch_gm(g.M, g.Cin, g.Cout, x, w_krsc, bias, bn, z, g.post_relu, g.post_mask, g.post_add, st, &sd);
  }
  if (gm_supported(g.M, g.Cin, g.Cout))   // the middle stages: one output tile per workgroup
    return launch_gm(g.M, g.Cin, g.Cout, x, w_krsc, bias, bn, z, g.post_relu, g.post_mask, g.post_add, st);
  PwParams p = fprop_params(g);
  const PwPlan pl = make_plan(p);
  if (!pl.ok) return hipErrorInvalidValue;
  if (bn) p.bn = *bn;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_krsc; p.bias = bias; p.out = (bf16_t*)z;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  return launch_plan(p, pl, st);
}
hipError_t launch_dgrad_pw(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                           hipStream_t st) {
  if (strided_pointwise(g)) {
    // the pixels no output pixel reads hold the bias alone (an input gradient has none: zeros): those rows everywhere
    // first, then the product lands on every stride-th pixel; a post-operation covers all of dx, as passes of its own
    const size_t n = (size_t)g.Min * g.Cin;
    if (hipError_t e = launch_gm_fill(dx, (size_t)g.Min, g.Cin, bias, st); e != hipSuccess) return e;
    const GmStride sd = stride_of(g, 1);
    hipError_t e = launch_gm(g.M, g.Cout, g.Cin, dz, w_crsk, bias, nullptr, dx, 0, nullptr, nullptr, st, &sd);
    if (e == hipSuccess && g.post_add) e = launch_eltwise(3 /* a + b */, CONVBN_BF16, dx, g.post_add, nullptr, n, st);
    if (e == hipSuccess && g.post_relu) e = launch_eltwise(0, CONVBN_BF16, dx, nullptr, nullptr, n, st);
    if (e == hipSuccess && g.post_mask) e = launch_eltwise(1, CONVBN_BF16, dx, g.post_mask, nullptr, n, st);
    return e;
  }
  if (gm_supported(g.M, g.Cout, g.Cin))
    return launch_gm(g.M, g.Cout, g.Cin, dz, w_crsk, bias, nullptr, dx, g.post_relu, g.post_mask, g.post_add, st);
  PwParams p = dgrad_params(g);
  const PwPlan pl = make_plan(p);
  if (!pl.ok) return hipErrorInvalidValue;
  p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = bias; p.out = (bf16_t*)dx;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  return launch_plan(p, pl, st);
}

}  // namespace convbn
