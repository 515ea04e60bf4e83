// bf16 convolution as a tiled matrix product without a window tile in LDS
//     out[m][r] = sum_{tap, c} act[row(m, tap)][c] wgt[r][tap][c] (+ bias[r]),     m over the output pixels:
//   forward conv   Z  = w' (*) X + b'   (Sec. 3.1 / 3.3)   act = x,   wgt = w' as [Cout][taps][Cin]
//   input gradient dX = w'_rot (*) dZ   (Sec. 3.2.1)       act = dz,  wgt = w' as [Cin][taps][Cout]
// for pointwise (1x1) layers with or without a stride, and -- window mode -- for strided 3x3 layers, forward and the
// residue classes of the input gradient.
//
// One output tile per workgroup, as large as still fills the chip: 256 (or 128) pixels x 128 channels, shared by
// EIGHT waves as 4 (2) pixel groups x 2 channel groups, so that a wave owns 64 x 64 (32 x 64) outputs and reads four
// (three) operand fragments for four (two) multiplies, and the matrix pipe of every SIMD is fed by two waves.  Channel
// counts that are no multiple of 128 get 128 x 64 tiles, and so do layers with too few 128 x 128 tiles for the chip.
//
// Pipeline.  The reduction runs over 64-channel chunks (window mode: over the taps, chunks innermost).  A chunk of
// the activation tile and of the weight tile is copied global -> LDS directly (1 KB per instruction: 8 rows x 128
// bytes) into one of three stages, two chunks ahead; every wave issues the same number of copies per chunk, so "at
// most that many copies outstanding" means the current chunk has landed; one barrier per chunk.  LDS rows are 128
// bytes, unpadded: the copy permutes the eight 16-byte granules of row r by (r / 2) % 8 (it chooses which granule
// each lane fetches), so that the 128-bit operand reads of 16 consecutive rows fall on distinct banks.  The copies of
// a chunk are issued between its multiplies; operands are double-buffered in registers one 16-channel step ahead.
// A copy's per-lane byte offset is free, which is all a stride needs: a strided pointwise layer gathers every
// stride-th pixel's row (forward) or scatters its output rows (input gradient); in window mode the offset of a row
// is recomputed per tap from the output pixel's window origin, rows outside the image being zero-fill copies.
//
// Layers that are bound by their stores rather than by the product (64 or 128 reduced channels over tens of
// thousands of pixels) run a variant with all their one or two chunks resident: no ring, about 70 registers, 33 or
// 65 KB of LDS -- several workgroups share a compute unit, and one's stores overlap another's loads.
#include "common.h"

namespace convbn {

namespace {

constexpr int NWAVES = 8;
constexpr int CB = 64;                 // reduced channels per chunk
constexpr int KK = CB / 16;
constexpr int NSTAGE = 3;
constexpr unsigned OOB = 0x80000000u;  // beyond any buffer: the load returns zeros

struct GmParams {
  const bf16_t* act;     // [M][C]
  const bf16_t* wgt;     // [R][C]
  const float* bias;     // [R] or null
  BnEpilogue bn;         // bn.gamma != null: the weight is unfolded, the epilogue applies s and b' (bias unused)
  bf16_t* out;           // [M][R]
  int relu;
  const bf16_t* mask;    // not null: [M][R], the output is zeroed where this is <= 0
  const bf16_t* add;     // not null: [M][R], added to the (rounded) output before the ReLU and the mask
  unsigned act_bytes, wgt_bytes;
  int M, C, R;
  int ntr;               // channel tiles
  int nchunks;
  // A pointwise layer with a stride (a downsampling shortcut) is the same product over the output pixels, whose rows
  // of the strided tensor are not consecutive: row m = (n, ho, wo) of the dense side is pixel (n, ho sh, wo sw) of an
  // [N][Hs][Ws] tensor.  gather: the activation rows are taken from there (forward); scatter: the output rows go there
  // (input gradient; the other pixels of dx are zero and are filled by the caller).
  int gather, scatter;
  int Ho, Wo, Hs, Ws, sh, sw;
  // Window mode (template flag CONV): a kH x kW window slides with stride (csh, csw) and padding (cph, cpw) over an
  // [N][aH][aW] activation grid; output pixel m = (n, ho, wo) of an [N][oHo][oWo] grid.  Every tap is a step of its own
  // in the reduction, its activation rows gathered per output pixel (zeros outside the grid): no window tile in LDS,
  // the taps re-read their rows through the L2 -- for strided layers, whose windows hardly overlap.
  GmConv cv;
};

// pixel index in the strided tensor of row m of the dense side
__device__ __forceinline__ size_t strided_row(const GmParams& p, int m) {
  const int hw = p.Ho * p.Wo;
  const int n = m / hw, rem = m - n * hw;
  const int ho = rem / p.Wo, wo = rem - ho * p.Wo;
  return ((size_t)n * p.Hs + (size_t)ho * p.sh) * p.Ws + (size_t)wo * p.sw;
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
// 1 KB copy: lane l fetches 16 bytes at voff (per lane, range-checked) + soff (wave-uniform) and writes them to LDS
// at lds_wave_base + 16 l.  The compiler barrier keeps every copy in the instruction stream: the waits count copies.
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

// TM: pixels per workgroup (256: a wave owns 2 x 2 subtiles of 32 x 32; 128: 1 x 2).
// RES > 0: the reduction is RES chunks in all (64 or 128 channels), each with a stage of its own and requested at the
// start: no ring, few registers -- what such a layer needs is several workgroups per compute unit, so that one's
// stores and another's loads overlap.
// TN: output channels per workgroup (128; 64 for layers whose channel count is no multiple of 128 -- the two channel
// groups of waves then own 32 channels each).
template <int TM, int RES = 0, int TN = 128>
struct GmCfg {
  static constexpr bool ONE = RES > 0;
  static constexpr int CW = TN / 2;                     // channels per wave
  static constexpr int NPS = TM / 128;                  // 32-pixel subtiles per wave
  static constexpr int NCS = CW / 32;                   // 32-channel subtiles per wave
  static constexpr int AUW = TM / 8 / NWAVES;           // activation copies (8 rows each) per wave and chunk
  static constexpr int WUW = TN / 8 / NWAVES;           // weight copies per wave and chunk
  static constexpr int CPW = AUW + WUW;
  static constexpr int STAGE = (TM + TN) * 128;
  static constexpr int OFF_BIAS = (RES ? RES : NSTAGE) * STAGE;   // [TN] bias, [TN] scale
  static constexpr int LDS_BYTES = OFF_BIAS + 2 * TN * 4;
  static_assert(NWAVES * 32 * CW * 2 <= STAGE, "the epilogue stages every wave's outputs (32 pixels at a time) in the first stage");
};

template <int TM, int RES = 0, int TN = 128, bool CONV = false>
__global__ __launch_bounds__(64 * NWAVES) void conv_gm_kernel(GmParams p) {
  static_assert(!CONV || RES == 0, "window mode runs on the ring");
  using Cfg = GmCfg<TM, RES, TN>;
  constexpr bool ONE = Cfg::ONE;
  constexpr int CW = Cfg::CW;
  constexpr int GR = CW / 8;          // 16-byte granules of a wave's staged output row
  constexpr int RPI = 64 / GR;        // rows one store instruction covers
  constexpr int ITS = 32 / RPI;       // store instructions per 32-pixel subtile
  constexpr int NPS = Cfg::NPS, NCS = Cfg::NCS, AUW = Cfg::AUW, WUW = Cfg::WUW, CPW = Cfg::CPW, STAGE = Cfg::STAGE;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* biasl = reinterpret_cast<float*>(smem + Cfg::OFF_BIAS);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;      // pixel group, channel group
  // Workgroups are handed to the eight XCDs in turn (id % 8), and each XCD has its own L2: the channel tiles of one
  // pixel tile read the same activation rows and should share one.  Pixel tiles go in groups of eight, one per XCD;
  // the k-th workgroup of an XCD (k = id / 8) is channel tile k % ntr of the XCD's (k / ntr)-th pixel tile.
  const int kx = (int)blockIdx.x >> 3;
  const int ctile = kx % p.ntr, ptile = (kx / p.ntr) * 8 + ((int)blockIdx.x & 7);
  if (ptile * TM >= p.M) return;   // (the last group of eight may be short)
  const int r0 = ctile * TN, m0 = ptile * TM;
  const __amdgpu_buffer_rsrc_t act_rsrc = make_rsrc(p.act, p.act_bytes);
  const __amdgpu_buffer_rsrc_t wgt_rsrc = make_rsrc(p.wgt, p.wgt_bytes);

  if (tid < TN) {
    const int ch = r0 + tid;
    float bias_v = p.bias ? p.bias[ch] : 0.f, scale_v = 1.f;
    if (p.bn.gamma) {   // Z = s (w (*) X) + b' (Sec. 3.3), s and b' worked out here
      scale_v = p.bn.gamma[ch] / sqrtf(p.bn.var[ch] + p.bn.eps);
      bias_v = ((p.bn.b ? p.bn.b[ch] : 0.f) - p.bn.mean[ch]) * scale_v + p.bn.beta[ch];
    }
    biasl[tid] = bias_v;
    biasl[TN + tid] = scale_v;
  }

  // ---- copies of this wave: unit u covers rows 8 u .. 8 u + 7 of its tile; lane l writes LDS granule l % 8 of row
  // 8 u + l / 8 and fetches the granule that belongs there, (l % 8) ^ key(row), key = (row / 2) % 8
  const int crow = lane >> 3, cpos = lane & 7;
  unsigned voff_a[AUW], voff_w[WUW];
  int cv_h[AUW], cv_w[AUW];   // window mode: the row's window origin (h, w of tap (0, 0)); voff_a holds its image and granule
#pragma unroll
  for (int j = 0; j < AUW; ++j) {
    const int row = (wave + NWAVES * j) * 8 + crow;
    const int g = cpos ^ ((row >> 1) & 7);
    if constexpr (CONV) {
      const int m = min(m0 + row, p.M - 1);
      const int hw = p.cv.oHo * p.cv.oWo;
      const int n = m / hw, rem = m - n * hw;
      const int ho = rem / p.cv.oWo, wo = rem - ho * p.cv.oWo;
      cv_h[j] = m0 + row < p.M ? ho * p.cv.csh - p.cv.cph : -(1 << 20);   // rows past the last pixel: never inside the grid
      cv_w[j] = wo * p.cv.csw - p.cv.cpw;
      voff_a[j] = (unsigned)((n * p.cv.a_n + g * 8) * 2);
    } else {
      const size_t arow = (p.gather && m0 + row < p.M) ? strided_row(p, m0 + row) : (size_t)(m0 + row);
      voff_a[j] = m0 + row < p.M ? (unsigned)((arow * p.C + g * 8) * 2) : OOB;   // rows past the last pixel: zeros
      cv_h[j] = cv_w[j] = 0;
    }
  }
#pragma unroll
  for (int j = 0; j < WUW; ++j) {
    const int row = (wave + NWAVES * j) * 8 + crow;
    const int g = cpos ^ ((row >> 1) & 7);
    voff_w[j] = (unsigned)(((size_t)(r0 + row) * (CONV ? p.cv.wrow : p.C) + g * 8) * 2);
  }
  // copy i (0 .. CPW-1) of a reduction step: chunk `chunk` of (window mode) tap (ti, tj)
  auto issue_copy = [&](int i, int chunk, int ti, int tj, unsigned char* stage) {
    const unsigned soff = (unsigned)(chunk * (CB * 2));
    if (i < AUW) {
      const int ii = i < AUW ? i : 0;
      unsigned voff = voff_a[ii];
      if constexpr (CONV) {
        const int h = cv_h[ii] + ti, w = cv_w[ii] + tj;
        const bool ok = (unsigned)h < (unsigned)p.cv.aH && (unsigned)w < (unsigned)p.cv.aW;
        voff = ok ? voff + (unsigned)((h * p.cv.a_h + w * p.cv.a_w) * 2) : OOB;
      }
      dma16(act_rsrc, voff, soff, stage + (wave + NWAVES * i) * 1024);
    } else {
      const int jj = i - AUW < WUW ? i - AUW : 0;
      const unsigned wsoff = CONV ? (unsigned)((p.cv.wt0 + ti * p.cv.wt_row + tj * p.cv.wt_col) * p.C * 2) + soff : soff;
      dma16(wgt_rsrc, voff_w[jj], wsoff, stage + TM * 128 + (wave + NWAVES * (i - AUW)) * 1024);
    }
  };

  // ---- operand addresses: row l % 32 of a subtile, granule 2 kk + l / 32 of the chunk, which sits at position
  // (2 kk + kb) ^ key = (2 kk) ^ (kb ^ key); key depends on l % 32 only (subtiles start at multiples of 32 rows)
  const int kb = lane >> 5;
  const int rl = lane & 31;
  const unsigned lane_off = (unsigned)(rl * 128 + (((kb ^ ((rl >> 1) & 7)) & 7) << 4));
  unsigned boff[NPS], aoff[NCS];
#pragma unroll
  for (int ps = 0; ps < NPS; ++ps) boff[ps] = (unsigned)((wm * (32 * NPS) + ps * 32) * 128) + lane_off;
#pragma unroll
  for (int i = 0; i < NCS; ++i) aoff[i] = (unsigned)(TM * 128 + (wn * CW + i * 32) * 128) + lane_off;

  f32x16 acc[NCS][NPS];
#pragma unroll
  for (int i = 0; i < NCS; ++i)
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][ps][e] = 0.f;

  bf16x8 fa[2][NCS], fb[2][NPS];
  auto load_frags = [&](int buf, const unsigned char* stage, int kk) {
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps) fb[buf][ps] = *reinterpret_cast<const bf16x8*>(stage + (boff[ps] ^ (unsigned)(kk << 5)));
#pragma unroll
    for (int i = 0; i < NCS; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(stage + (aoff[i] ^ (unsigned)(kk << 5)));
  };

  // ---- the addend and the mask of this lane's outputs (see the epilogue for the lane -> output map) are requested
  // before the first copy, so that they arrive while the product runs instead of holding up every store
  auto out_off = [&](int ps, int it) -> long long {
    const int row = it * RPI + lane / GR;
    const int g = (lane % GR) ^ ((row >> 1) & (GR - 1));
    const int m = m0 + wm * (32 * NPS) + ps * 32 + row;
    if (m >= p.M) return -1;
    if constexpr (CONV) {
      if (p.cv.out_strided) {
        const int hw = p.cv.oHo * p.cv.oWo;
        const int n = m / hw, rem = m - n * hw;
        const int ho = rem / p.cv.oWo, wo = rem - ho * p.cv.oWo;
        return (long long)p.cv.out_base + (long long)n * p.cv.out_n + (long long)ho * p.cv.out_h + (long long)wo * p.cv.out_w +
               r0 + wn * CW + g * 8;
      }
    }
    const size_t orow = p.scatter ? strided_row(p, m) : (size_t)m;
    return (long long)(orow * p.R + r0 + wn * CW + g * 8);
  };
  uint4 addv[NPS][ITS], maskv[NPS][ITS];
  if (!ONE && (p.add || p.mask)) {
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps)
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const long long o = out_off(ps, it);
        addv[ps][it] = (p.add && o >= 0) ? *reinterpret_cast<const uint4*>(p.add + o) : make_uint4(0u, 0u, 0u, 0u);
        maskv[ps][it] = (p.mask && o >= 0) ? *reinterpret_cast<const uint4*>(p.mask + o) : make_uint4(0u, 0u, 0u, 0u);
      }
    asm volatile("" ::: "memory");
  }

  // ---- prologue: chunks 0 and 1 (a chunk past the end is the last one again, into a stage nobody reads)
  // (window mode: a step is (tap, chunk), chunks innermost; p.nchunks counts the steps and cpt the chunks per tap)
  const int nchunks = p.nchunks;
  const int cpt = CONV ? p.C / CB : nchunks;
  int f_c = 0, f_i = 0, f_j = 0;   // the step whose copies are issued next: chunk and tap
  auto advance_fill = [&]() {       // ... the one after it (the last step stays)
    if constexpr (CONV) {
      if (f_c + 1 < cpt) ++f_c;
      else if (f_j + 1 < p.cv.kW) { f_c = 0; ++f_j; }
      else if (f_i + 1 < p.cv.kH) { f_c = 0; f_j = 0; ++f_i; }
    } else {
      if (f_c + 1 < nchunks) ++f_c;
    }
  };
#pragma unroll
  for (int i = 0; i < CPW; ++i) issue_copy(i, f_c, f_i, f_j, smem);
  advance_fill();
  if constexpr (RES != 1) {
#pragma unroll
    for (int i = 0; i < CPW; ++i) issue_copy(i, f_c, f_i, f_j, smem + STAGE);
  }
  advance_fill();

  int st_cur = 0;   // stage of the current chunk
  for (int c = 0; c < nchunks; ++c) {
    if (ONE && c == RES - 1) wait_vm<0>();   // (all chunks resident: the last one has nothing behind it)
    else wait_vm<CPW>();    // this chunk has landed (the next one's copies may be in flight) ...
    block_barrier();   // ... for every wave, and everybody is done with the stage refilled below
    const unsigned char* const stage = smem + st_cur * STAGE;
    const int st_fill = st_cur >= 1 ? st_cur - 1 : NSTAGE - 1;   // (c + 2) % 3
    unsigned char* const fill = smem + st_fill * STAGE;
    load_frags(0, stage, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int cur = kk & 1;
      if (kk + 1 < KK) load_frags(cur ^ 1, stage, kk + 1);
      __builtin_amdgcn_sched_barrier(0);
      // the copies of the chunk two ahead, spread over the multiplies of this one
      constexpr int PER = (CPW + KK - 1) / KK;
      int issued = 0;
#pragma unroll
      for (int i = 0; i < NCS; ++i)
#pragma unroll
        for (int ps = 0; ps < NPS; ++ps) {
          acc[i][ps] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][ps], acc[i][ps], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (!ONE && issued < PER && kk * PER + issued < CPW) {
            issue_copy(kk * PER + issued, f_c, f_i, f_j, fill);
            ++issued;
            __builtin_amdgcn_sched_barrier(0);
          }
        }
#pragma unroll
      for (; issued < PER; ++issued)
        if (!ONE && kk * PER + issued < CPW) issue_copy(kk * PER + issued, f_c, f_i, f_j, fill);
      __builtin_amdgcn_sched_barrier(0);
    }
    st_cur = st_cur + 1 == NSTAGE ? 0 : st_cur + 1;
    advance_fill();
  }
  wait_vm<0>();      // trailing copies must not outlive the loop: the ring becomes the staging space
  __syncthreads();   // (and the bias is visible)

  // ---- epilogue.  Accumulator element e of lane l in subtile (i, ps): channel 32 i + 8 (e / 4) + 4 (l / 32) + e % 4,
  // pixel 32 ps + l % 32 of the wave's block.  Per 32-pixel subtile the wave rounds 32 pixels x CW channels to bf16
  // into its own 64 CW bytes ([pixel][CW ch], granules swizzled by pixel) and reads them back row-wise: every store is 16
  // bytes per lane, GR lanes cover one pixel's CW contiguous channels.
  unsigned char* const st = smem + wave * (32 * CW * 2);
  const int px = lane & 31, psw = (px >> 1) & (GR - 1);
#pragma unroll
  for (int ps = 0; ps < NPS; ++ps) {
#pragma unroll
    for (int i = 0; i < NCS; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int ch = i * 32 + q * 8 + kb * 4;
        const float4 bb = *reinterpret_cast<const float4*>(biasl + wn * CW + ch);
        const float4 sc = *reinterpret_cast<const float4*>(biasl + TN + wn * CW + ch);
        const uint2 v = make_uint2(pack_bf16x2(fmaf(acc[i][ps][q * 4 + 0], sc.x, bb.x), fmaf(acc[i][ps][q * 4 + 1], sc.y, bb.y)),
                                   pack_bf16x2(fmaf(acc[i][ps][q * 4 + 2], sc.z, bb.z), fmaf(acc[i][ps][q * 4 + 3], sc.w, bb.w)));
        *reinterpret_cast<uint2*>(st + px * (CW * 2) + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
      }
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      const int row = it * RPI + lane / GR;
      uint4 v = *reinterpret_cast<const uint4*>(st + row * (CW * 2) + ((lane % GR) << 4));
      const long long o = out_off(ps, it);
      if constexpr (ONE) {
        if (o >= 0) *reinterpret_cast<uint4*>(p.out + o) = post_op8(v, p.relu, p.mask, p.add, (size_t)o);
      } else {
        if (p.add) v = add8(v, addv[ps][it]);
        if (p.relu) v = relu8(v);
        if (p.mask) v = mask8(v, maskv[ps][it]);
        if (o >= 0) *reinterpret_cast<uint4*>(p.out + o) = v;
      }
    }
  }
}

constexpr int MIN_TILES = 160;       // fewer 256-pixel tiles leave too many compute units without one: 128-pixel tiles then,
constexpr int MIN_TILES_SMALL = 96;  // down to this many (measured against the split-sum plans of the LDS-tile kernel:
                                     // 1024 -> 256 at 14 x 14, 98 tiles, 10.8 against 12.0 us)
constexpr int MAX_PIXELS = 32768;    // longer pixel ranges with short reductions stream through the weight-stationary kernel

struct GmPlan { int tm, res, tn; };   // tm == 0: not taken

GmPlan choose_plan(int M, int C, int R) {
  GmPlan none{0, 0, 0};
  if (M < 1 || C < CB || C % CB || R % 64) return none;
  if ((size_t)M * C * 2 >= OOB || (size_t)M * R * 2 >= OOB || (size_t)R * C * 2 >= OOB) return none;
  const int tn = R % 128 == 0 ? 128 : 64;
  const int ntr = R / tn;
  const long long t128 = (long long)ceil_div(M, 128) * ntr, t256 = (long long)ceil_div(M, 256) * ntr;
  // short reductions over many tiles: every chunk resident, several workgroups per compute unit
  if ((C == CB || C == 2 * CB) && t128 >= 3 * MIN_TILES) return GmPlan{128, C / CB, tn};
  if (tn == 64) return t128 >= MIN_TILES_SMALL ? GmPlan{128, 0, 64} : none;
  // (measured on the 56 x 56 stage: with 256 reduced channels the tile beats the streaming kernel, 21.9 against 26.1 us
  // for 256 -> 128; with 64 or 128 both are bound by their stores and take the same time)
  if (M > MAX_PIXELS && C < 256) return none;
  if (t256 >= MIN_TILES) return GmPlan{256, 0, 128};
  // too few 128 x 128 tiles for the chip: twice as many of half the channels (measured: 1024 -> 256 at 14 x 14, 98 tiles,
  // 10.4 -> 9.0 us; 2048 -> 512 at 7 x 7, 52 tiles, 16.8 us on the split-sum tile kernel -> 12.6)
  if (t128 < MIN_TILES && 2 * t128 >= MIN_TILES_SMALL) return GmPlan{128, 0, 64};
  if (t128 >= MIN_TILES_SMALL) return GmPlan{128, 0, 128};
  return none;
}

template <int TM, int RES, int TN>
hipError_t launch_inst(const GmParams& p, hipStream_t st) {
  static LdsLimitOnce lds_once;
  constexpr int lds = GmCfg<TM, RES, TN>::LDS_BYTES;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&conv_gm_kernel<TM, RES, TN>), lds);
      e != hipSuccess) return e;
  hipLaunchKernelGGL((conv_gm_kernel<TM, RES, TN>), dim3(ceil_div(ceil_div(p.M, TM), 8) * 8 * p.ntr), dim3(64 * NWAVES), lds, st, p);
  return hipGetLastError();
}

template <int TM, int TN>
hipError_t launch_conv_inst(const GmParams& p, hipStream_t st) {
  static LdsLimitOnce lds_once;
  constexpr int lds = GmCfg<TM, 0, TN>::LDS_BYTES;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&conv_gm_kernel<TM, 0, TN, true>), lds);
      e != hipSuccess) return e;
  hipLaunchKernelGGL((conv_gm_kernel<TM, 0, TN, true>), dim3(ceil_div(ceil_div(p.M, TM), 8) * 8 * p.ntr), dim3(64 * NWAVES), lds, st, p);
  return hipGetLastError();
}

// tile of the window mode: tm = 0: not taken
GmPlan conv_tile_plan(int M, int C, int R, const GmConv& cv) {
  GmPlan none{0, 0, 0};
  if (M < 1 || C % CB || R % 128 || cv.kH < 1 || cv.kW < 1 || cv.kH * cv.kW > 16) return none;
  const long long t256 = (long long)ceil_div(M, 256) * (R / 128), t128 = (long long)ceil_div(M, 128) * (R / 128);
  if (t256 >= MIN_TILES) return GmPlan{256, 0, 128};
  // (as in the plain mode; 3x3 / 2 layers: 512 channels to 7 x 7, 52 tiles, forward 30.8 -> 27.9 us; 256 channels to 14 x 14,
  // 98 tiles, forward 19.5 -> 17.9, input gradient 33.4 -> 28.8)
  if (t128 < MIN_TILES && 2 * t128 >= MIN_TILES_SMALL) return GmPlan{128, 0, 64};
  if (t128 >= MIN_TILES_SMALL) return GmPlan{128, 0, 128};
  return none;
}

}  // namespace

bool gm_conv_supported(int M, int C, int R, const GmConv& cv) { return conv_tile_plan(M, C, R, cv).tm != 0; }

hipError_t launch_gm_conv(int M, int C, int R, const GmConv& cv, const void* act, unsigned act_bytes, const void* wgt,
                          unsigned wgt_bytes, const float* bias, void* out, int relu, const void* mask, const void* add,
                          hipStream_t st) {
  const GmPlan pl = conv_tile_plan(M, C, R, cv);
  const int tm = pl.tm;
  if (tm == 0 || act_bytes >= OOB || wgt_bytes >= OOB) return hipErrorInvalidValue;
  GmParams p{};
  p.M = M; p.C = C; p.R = R;
  p.act_bytes = act_bytes; p.wgt_bytes = wgt_bytes;
  p.ntr = R / pl.tn;
  p.nchunks = cv.kH * cv.kW * (C / CB);   // steps: (tap, chunk)
  p.cv = cv;
  p.act = (const bf16_t*)act; p.wgt = (const bf16_t*)wgt; p.bias = bias; p.out = (bf16_t*)out;
  p.relu = relu; p.mask = (const bf16_t*)mask; p.add = (const bf16_t*)add;
  if (pl.tn == 64) return launch_conv_inst<128, 64>(p, st);
  return tm == 256 ? launch_conv_inst<256, 128>(p, st) : launch_conv_inst<128, 128>(p, st);
}

bool gm_supported(int M, int C, int R) { return choose_plan(M, C, R).tm != 0; }

// every row of a [rows][R] bf16 tensor <- bias (zeros if null); R is a multiple of 8
__global__ __launch_bounds__(256) void gm_fill_kernel(uint4* __restrict__ p, size_t n16, int R8, const float* __restrict__ bias) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (bias) {
      const float* b = bias + (i % (size_t)R8) * 8;
      v = make_uint4(pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3]), pack_bf16x2(b[4], b[5]), pack_bf16x2(b[6], b[7]));
    }
    p[i] = v;
  }
}

hipError_t launch_gm_fill(void* p, size_t rows, int R, const float* bias, hipStream_t st) {
  const size_t n16 = rows * (size_t)R / 8;
  const int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
  hipLaunchKernelGGL(gm_fill_kernel, dim3(blocks < 1 ? 1 : blocks), dim3(256), 0, st, (uint4*)p, n16, R / 8, bias);
  return hipGetLastError();
}

hipError_t launch_gm(int M, int C, int R, const void* act, const void* wgt, const float* bias, const BnEpilogue* bn,
                     void* out, int relu, const void* mask, const void* add, hipStream_t st, const GmStride* sd) {
  const GmPlan pl = choose_plan(M, C, R);
  if (pl.tm == 0) return hipErrorInvalidValue;
  GmParams p{};
  p.M = M; p.C = C; p.R = R;
  p.act_bytes = (unsigned)((size_t)M * C * 2);
  if (sd) {
    const size_t strided_pixels = (size_t)sd->N * sd->Hs * sd->Ws;
    if (strided_pixels * (size_t)(sd->scatter ? R : C) * 2 >= OOB) return hipErrorInvalidValue;
    p.gather = !sd->scatter; p.scatter = sd->scatter;
    p.Ho = sd->Ho; p.Wo = sd->Wo; p.Hs = sd->Hs; p.Ws = sd->Ws; p.sh = sd->sh; p.sw = sd->sw;
    if (p.gather) p.act_bytes = (unsigned)(strided_pixels * C * 2);
    if (p.scatter && (mask || add || relu)) return hipErrorInvalidValue;   // the caller applies them to all of dx
  }
  p.wgt_bytes = (unsigned)((size_t)R * C * 2);
  p.ntr = R / pl.tn;
  p.nchunks = C / CB;
  p.act = (const bf16_t*)act; p.wgt = (const bf16_t*)wgt; p.bias = bias; p.out = (bf16_t*)out;
  if (bn) p.bn = *bn;
  p.relu = relu; p.mask = (const bf16_t*)mask; p.add = (const bf16_t*)add;
#define GM_CASE(TM_, RES_, TN_) if (pl.tm == TM_ && pl.res == RES_ && pl.tn == TN_) return launch_inst<TM_, RES_, TN_>(p, st);
  GM_CASE(256, 0, 128) GM_CASE(128, 0, 128) GM_CASE(128, 1, 128) GM_CASE(128, 2, 128)
  GM_CASE(128, 0, 64) GM_CASE(128, 1, 64) GM_CASE(128, 2, 64)
#undef GM_CASE
  return hipErrorInvalidValue;
}

}  // namespace convbn
