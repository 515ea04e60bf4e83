// bf16 MFMA convolution with the input window tile resident in LDS.
//
// A workgroup owns TP consecutive output pixels (in (n,ho,wo) order) x TRC output channels.
// All input rows those pixels touch are copied once into LDS as [slot][column][channel chunk]
// (zero rows/columns stand in for the padding), then every tap (i,j) of the kernel window is
// one MFMA sweep over the SAME LDS tile at a wave-uniform offset of (i*Wv + j) pixels: each
// input element is fetched from memory once per workgroup instead of once per tap.  The weight
// slab of every (tap, channel chunk) step streams through an LDS ring.
//
// Global -> LDS copies are buffer loads that write LDS directly (16 bytes per lane, lane l of a
// wave lands at base + 16 l); a lane given an offset beyond the buffer delivers zeros, which is
// how padding is materialised without branches.  LDS rows are padded by one 16-byte granule
// (row pitch 144 or 80 bytes) so that the 128-bit MFMA operand reads of 16 consecutive rows fall
// on distinct banks; the operand addresses then are "lane base + wave-uniform step offset +
// immediate", i.e. one vector add per step.  A 1 KB copy therefore covers RPU whole padded rows
// (7 or 12) and its last lanes the head of the following row, which the next copy writes again
// with the same values.
//
// Everything a copy needs per lane (row validity, padding, tails) is folded once into a per-lane
// byte offset; a step only adds a wave-uniform scalar offset (tap, channel chunk) to it.
//
//   forward conv   Z  = w' (*) X + b'        (Sec. 3.1 / 3.3)    act = x,  weights [Cout][taps][Cin]
//   input gradient dX = w'_rot (*) dZ        (Sec. 3.2.1), stride 1: the same sweep over dz with
//                  the taps reversed and padding k-1-p,          weights [Cin][taps][Cout];
//                  strided: one such sweep per residue class of input positions (see
//                  dgrad_class_params), written to that class's positions of dX
#include "common.h"

#include <type_traits>

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
  BnEpilogue bn;         // bn.gamma != null: the weight is unfolded, the epilogue applies s and b' (bias unused)
  bf16_t* out;           // [M][R]
  int relu;              // the output leaves as max(., 0)
  const bf16_t* mask;    // not null: laid out like out, the output is zeroed where this is <= 0
  const bf16_t* add;     // not null: laid out like out, added to the (rounded) output before the ReLU and the mask
  unsigned act_bytes, wgt_bytes;
  int N, H, W, C;        // activation grid the window slides over
  int act_n_stride, act_h_stride, act_w_stride;
  int Ho, Wo, R;
  int kH, kW, sh, sw, ph, pw;
  int wrow;              // elements per output-channel row of the weight tensor (its taps x C)
  // window position (ti, tj) reads tap wt0 + ti wt_row + tj wt_col of the weight tensor (forward: the same
  // position; input gradient: the rotated one; strided input gradient: every stride-th tap, rotated)
  int wt0, wt_row, wt_col;
  int no_split;          // the output is strided: no split sums (their reduction assumes a dense output)
  int out_strided;       // output pixel (n, ho, wo) lives at out_base + n out_n + ho out_h + wo out_w (elements)
  int out_base, out_n, out_h, out_w;
  int M;                 // N*Ho*Wo
  int Hv, Wv;            // rows / columns of one image's (virtually padded) window footprint
  int ntr;               // channel tiles
  int nhb, hps, spread;  // activation tile ring depth, copy units per wave and step, steps a prefetch spans
  int min_hps;           // host side: the planner picks at least this many copy units per wave and step
  int ksplit, chunks_per_split;   // channel chunks are divided over gridDim.y workgroups
  float* part;           // [ksplit][M][R] fp32 partial outputs when ksplit > 1
  int halo_stride;       // bytes per activation tile buffer
  int tab_off;           // byte offset of the per-lane copy-offset table in LDS (multi-chunk only)
  int tab_rows;          // live table rows per wave (spread * copies per step)
  int ucap;              // copy units per activation tile buffer; unit ucap is a spare KB that takes the surplus copies
  int tile_rows;         // > 0: a pixel tile is this many whole output rows of one image (else TP consecutive pixels)
  int tiles_per_image;
  FastDiv dTpi;
  FastDiv dHoWo, dWo, dHv, dWv;
};

constexpr unsigned OOB = 0x80000000u;   // beyond any buffer: the load returns zeros

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// 1 KB copy: lane l fetches 16 bytes at byte offset voff (per lane) + soff (wave-uniform) of the
// buffer and writes them to LDS at lds_wave_base + 16 l.
// The compiler barrier keeps every copy in the instruction stream: the waits below count copies, and
// two copies into the same LDS range (the dummies) would otherwise be merged as a dead store.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)voff, (int)soff, 0, 0);
  asm volatile("" ::: "memory");
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would drain every
// outstanding copy (vmcnt(0)) and serialise the pipeline.  Ordering of the copies is handled by
// the explicit vmcnt waits; LDS reads are ordered by their own data dependences.
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int N> __device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Compile-time layout of one instantiation (shared by the kernel and the host planner).
template <int NCH, int CB> struct TileCfg {
  static constexpr int TRC = NCH * 32;         // output channels per workgroup
  static constexpr int GPR = CB / 8;           // data granules (16 B) per LDS row
  static constexpr int LPR = GPR + 1;          // lanes per row: data granules + one pad granule
  static constexpr int RPU = 64 / LPR;         // whole rows per 1 KB copy: 7 (CB 64) / 12 (CB 32)
  static constexpr int ROWP = LPR * 16;        // row pitch: 144 / 80 bytes
  static constexpr int UNITB = RPU * ROWP;     // LDS bytes between consecutive copies: 1008 / 960
  static constexpr int KK = CB / 16;           // MFMA k-steps per channel chunk
  static constexpr int NBUF = CB == 64 ? 4 : 5;   // weight ring slots
  static constexpr int DIST = NBUF - 1;        // steps between issuing a copy and its step
  static constexpr int WUNITS = (TRC + RPU - 1) / RPU;
  static constexpr int WSLAB = WUNITS * UNITB + 64;   // + room for the last copy's spill lanes
};

// NW waves as NW/NWC pixel groups x NWC channel groups, each wave owning 32 pixels x 32 NCH/NWC of
// the workgroup's TRC = 32 NCH channels; CB channels per LDS chunk; HPS
// activation copies per wave and step (0: the channels of this workgroup are a single chunk, whose
// activation tile is fetched once up front).
//
// Pipeline.  A "step" is one tap of one channel chunk (KK x NCH MFMAs per wave).  Every step each
// wave issues exactly HPS + WPW copies: HPS 1 KB units of a future chunk's activation tile (zero-fill
// copies into a spare KB when there is nothing to fetch) and its share of the weight slab of step
// it+DIST.  Copies complete in issue order, so "at most DIST-2 steps' worth outstanding" means that
// everything issued DIST-1 or more steps ago has landed, i.e. the data of steps <= it+1.  The MFMA
// operands are double-buffered in registers one k-step ahead; only the last k-step of a step reads
// the next step's LDS data, which is why step it+1 must be resident at the barrier of step it and
// why the slab written during step it is the one of step it-1 (= it+DIST modulo the ring).
// The activation tile has nhb buffers: 1 (single chunk) or a ring -- the tile of chunk c + nhb - 1 is
// fetched during the first `spread` steps of chunk c and has to land DIST - 1 steps before its first
// step, so spread <= (nhb - 1) taps - DIST + 1: two buffers for windows of at least DIST taps, more
// for fewer (1x1 windows: NBUF buffers, one step per chunk).
// The step loop is branch-free apart from its back edge: all per-step decisions are scalar selects,
// and the per-lane copy offsets of the activation tile come from a table in LDS built once per
// workgroup (row k of wave w = copy unit w + NW k; rows past the tile hold the zero-fill offset).
// SC: the weight is unfolded and the epilogue applies the BatchNorm scale and folded bias it works out itself (an
// instantiation of its own, so the default kernels carry none of it).
#ifdef TILE_TRACE
__device__ unsigned long long tile_trace[1024 * 32];
#ifndef TILE_TRACE_WAVE
#define TILE_TRACE_WAVE 0
#endif
#define STAMP(i) do { if (threadIdx.x == 64 * TILE_TRACE_WAVE) { tile_trace[bx * 32 + (i)] = clock64(); tile_trace[bx * 32 + 16 + (i)] = wall_clock64(); } } while (0)
#else
#define STAMP(i) do {} while (0)
#endif

// The work of workgroup (bx, by) of a launch of gx x (splits) workgroups; smem: the workgroup's LDS.
template <int NW, int NWC, int NCH, int CB, int HPS, bool SC = false>
__device__ __forceinline__ void tile_body(const TileParams& p, int bx, int by, int gx, unsigned char* smem) {
  STAMP(0);
  using Cfg = TileCfg<NCH, CB>;
  constexpr int NWP = NW / NWC;            // waves along the pixels
  constexpr int NCW = NCH / NWC;           // 32-channel subtiles per wave
  static_assert(NW % NWC == 0 && NCH % NWC == 0 && NCW % 2 == 0, "channel groups must split the tile evenly");
  constexpr int TP = 32 * NWP;
  constexpr int TRC = Cfg::TRC, GPR = Cfg::GPR, LPR = Cfg::LPR, RPU = Cfg::RPU, ROWP = Cfg::ROWP;
  constexpr int UNITB = Cfg::UNITB, KK = Cfg::KK, NBUF = Cfg::NBUF, DIST = Cfg::DIST;
  constexpr int WUNITS = Cfg::WUNITS, WSLAB = Cfg::WSLAB;
  constexpr int WPW = (WUNITS + NW - 1) / NW;  // weight copies per wave and step (surplus ones are dummies)
  constexpr bool MULTI = HPS > 0;
  constexpr int CPS = HPS + WPW;               // copies per wave and step
  float* biasl = reinterpret_cast<float*>(smem);               // [TRC] bias of this channel tile (first KB)
  unsigned char* wbuf = smem + 1024;                           // [NBUF] weight slabs
  unsigned char* scratch = wbuf + NBUF * WSLAB;                // 1 KB target of the dummy copies (zeros only)
  unsigned char* halo = scratch + 1024;                        // [nhb][halo_stride]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wp = wave % NWP;               // pixel group and channel group of this wave
  const int cw0 = (wave / NWP) * NCW;      // its first 32-channel subtile
  const int ctile = bx % p.ntr, ptile = bx / p.ntr;
  const int r0 = ctile * TRC;
  const int HoWo = p.Ho * p.Wo;
  // pixels [m0, m0 + len) of this tile: TP consecutive pixels, or whole rows of one image
  int m0 = ptile * TP, len = min(TP, p.M - m0);
  if (p.tile_rows > 0) {
    const int n = fdiv(ptile, p.dTpi);
    const int row0 = (ptile - n * p.tiles_per_image) * p.tile_rows;
    m0 = n * HoWo + row0 * p.Wo;
    len = min(p.tile_rows, p.Ho - row0) * p.Wo;
  }
  const int m_last = m0 + len - 1;
  const int n_a = fdiv(m0, p.dHoWo), ho_a = fdiv(m0 - n_a * HoWo, p.dWo);
  const int n_b = fdiv(m_last, p.dHoWo), ho_b = fdiv(m_last - n_b * HoWo, p.dWo);
  const int v_first = n_a * p.Hv + ho_a * p.sh;
  const int nslots = n_b * p.Hv + ho_b * p.sh + p.kH - v_first;
  const int npix = nslots * p.Wv;
  const int hunits = (npix + RPU - 1) / RPU;

  const __amdgpu_buffer_rsrc_t act_rsrc = make_rsrc(p.act, p.act_bytes);
  const __amdgpu_buffer_rsrc_t wgt_rsrc = make_rsrc(p.wgt, p.wgt_bytes);
  const int taps = p.kH * p.kW;
  const int cbeg = by * p.chunks_per_split;                       // first channel chunk of this workgroup
  const int nchunks = min(p.C / CB, cbeg + p.chunks_per_split);           // one past its last chunk
  const int nsteps = (nchunks - cbeg) * taps;
  // bias of this channel tile: fetched now, parked in LDS after the main loop (nothing waits for it)
  float bias_v = (tid < TRC && p.bias && r0 + tid < p.R) ? p.bias[r0 + tid] : 0.f;
  float scale_v = 1.f;
  if (SC && tid < TRC && r0 + tid < p.R) {
    const int ch = r0 + tid;
    scale_v = p.bn.gamma[ch] / sqrtf(p.bn.var[ch] + p.bn.eps);
    bias_v = ((p.bn.b ? p.bn.b[ch] : 0.f) - p.bn.mean[ch]) * scale_v + p.bn.beta[ch];
  }

  // this lane's place inside every 1 KB copy: row lrow (RPU = the spill row) and granule lgran (GPR = pad)
  const int lrow = lane / LPR;
  const int lgran = lane - lrow * LPR;

  // the weight copies this wave issues every step: per-lane byte offsets (the step's part is added as a
  // scalar) and LDS offsets inside a slab.  A surplus copy repeats unit u - WUNITS (same bytes, same place).
  unsigned voff_w[WPW];
  int wu_off[WPW];
#pragma unroll
  for (int j = 0; j < WPW; ++j) {
    int u = wave + NW * j;
    u = u < WUNITS ? u : u - WUNITS;
    const int row = u * RPU + lrow;
    const bool ok = row < TRC && r0 + row < p.R && lgran < GPR;
    voff_w[j] = ok ? (unsigned)(((r0 + row) * p.wrow + lgran * 8) * 2) : OOB;
    wu_off[j] = u * UNITB;
  }
  // byte offset (without the channel chunk) of this lane's 16 bytes of copy unit u of the activation tile
  auto halo_voff = [&](int u) -> unsigned {
    const int pix = u * RPU + lrow;
    const int slot = fdiv(pix, p.dWv);
    const int w = pix - slot * p.Wv - p.pw;
    const int v = v_first + slot;
    const int n = fdiv(v, p.dHv);
    const int h = v - n * p.Hv - p.ph;
    const bool ok = u < hunits && pix < npix && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W &&
                    n < p.N && lgran < GPR;
    return ok ? (unsigned)((n * p.act_n_stride + h * p.act_h_stride + w * p.act_w_stride + lgran * 8) * 2) : OOB;
  };
  // this wave's share of the weight slab of (chunk, tap) -> ring slot at byte offset slot_off
  auto issue_weights = [&](int chunk, int wtap, int slot_off) {
    const unsigned soff = (unsigned)((wtap * p.C + chunk * CB) * 2);
    unsigned char* dst = wbuf + slot_off;
#pragma unroll
    for (int j = 0; j < WPW; ++j) dma16(wgt_rsrc, voff_w[j], soff, dst + wu_off[j]);
  };

  // LDS byte offsets of this lane's MFMA operands: pixel row (tap (0,0)) and weight row, k-half kb
  const int kb = lane >> 5;
  unsigned boff;
  {
    const int pi = wp * 32 + (lane & 31);
    const int m = m0 + pi;
    int pixidx = 0;
    if (pi < len) {
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      const int ho = fdiv(rem, p.dWo);
      const int wo = rem - ho * p.Wo;
      pixidx = (n * p.Hv + ho * p.sh - v_first) * p.Wv + wo * p.sw;
    }
    boff = (unsigned)(pixidx * ROWP + kb * 16);
  }
  const unsigned aoff = (unsigned)((cw0 * 32 + (lane & 31)) * ROWP + kb * 16);

  f32x16 acc[NCW];
#pragma unroll
  for (int r = 0; r < NCW; ++r)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[r][e] = 0.f;

  // ---- prologue: the copies steps -DIST .. -1 would have issued --------------------------------
  // table row k of this wave: [(k NW + wave) 64 + lane]; rows tab_rows .. tab_rows+HPS-1 are all zero-fill
  unsigned* const tab_lane = reinterpret_cast<unsigned*>(smem + p.tab_off) + wave * 64 + lane;
  constexpr int TROW = NW * 64;   // table entries per row
  if (MULTI) {
    for (int k = 0; k < p.tab_rows + HPS; ++k) tab_lane[k * TROW] = k < p.tab_rows ? halo_voff(wave + NW * k) : OOB;
  }
  if (MULTI && taps == 1) {
    // 1x1 window, several chunks: the chunk of step s goes to ring buffer s
    for (int s = 0; s < DIST; ++s) {
      const int cs = min(cbeg + s, nchunks - 1);
#pragma unroll
      for (int j = 0; j < HPS; ++j) {
        const int u = wave + NW * j;
        dma16(act_rsrc, tab_lane[j * TROW], (unsigned)(cs * CB * 2), u < hunits ? halo + s * p.halo_stride + u * UNITB : scratch);
      }
      issue_weights(cs, p.wt0, s * WSLAB);
    }
  } else {
    // the tiles of the first nhb - 1 chunks (one unless the window has fewer taps than the pipeline is deep)
    for (int hb = 0; hb < (MULTI ? p.nhb - 1 : 1); ++hb)
      for (int u = wave; u < hunits; u += NW)
        dma16(act_rsrc, halo_voff(u), (unsigned)(min(cbeg + hb, nchunks - 1) * CB * 2),
              halo + hb * p.halo_stride + u * UNITB);
    for (int s = 0; s < DIST; ++s) {
      if (s > 0) {
#pragma unroll
        for (int j = 0; j < HPS; ++j) dma16(act_rsrc, OOB, 0u, scratch);   // dummies keep the count uniform
      }
      const int cs = s / taps, ti = (s - cs * taps) / p.kW, tj = s - cs * taps - ti * p.kW;
      issue_weights(min(cbeg + cs, nchunks - 1), p.wt0 + ti * p.wt_row + tj * p.wt_col, s * WSLAB);
    }
  }

  // Per-tap tables, lane t = window position t (at most 64 taps): byte offset of the tap inside the
  // activation tile and byte offset of its weights inside a weight row.  A step reads its entries with one
  // lane-select each instead of tracking rows and columns in scalar registers: with one or two waves per
  // SIMD the scalar bookkeeping of a step, not the matrix pipe, is what bounds the loop.
  int vt_toff, vt_wt;
  {
    const int t = lane < taps ? lane : 0;
    const int ti = t / p.kW, tj = t - ti * p.kW;
    vt_toff = (ti * p.Wv + tj) * ROWP;
    vt_wt = (p.wt0 + ti * p.wt_row + tj * p.wt_col) * p.C * 2;
  }
  // Wave-uniform bookkeeping.  A position is (window position, chunk, offset of the chunk's activation tile
  // buffer, offset of the buffer being refilled = the previous chunk's).  The weight ring needs no state: the
  // loop is unrolled NBUF times, so every step knows its slab at compile time.  Everything a step needs
  // from the scalar unit -- its operand offsets and the descriptors of its copies -- is computed during
  // the PREVIOUS step, in the shadow of that step's multiplies.
  struct Pos { int tap, c, hoff, foff; };
  const int hlimit = p.nhb * p.halo_stride;
  auto advance = [&](const Pos& q) {
    const bool e = q.tap + 1 == taps;
    const int h = q.hoff + (e ? p.halo_stride : 0);
    return Pos{e ? 0 : q.tap + 1, q.c + (e ? 1 : 0), h == hlimit ? 0 : h, e ? q.hoff : q.foff};
  };
  auto bstep_of = [&](const Pos& q) { return q.hoff + __builtin_amdgcn_readlane(vt_toff, q.tap); };
  // copies of one step: HPS activation units of the chunk nhb-1 ahead (per-lane offsets from the LDS table,
  // zero-fill rows when there is nothing to fetch) and the weight slab of the step DIST ahead
  struct Copies { unsigned hv[HPS > 0 ? HPS : 1]; int ku; unsigned hsoff; int hbase; unsigned wsoff; };
  auto act_copies = [&](const Pos& q, Copies& d) {
    if (MULTI) {
      const bool hlive = q.tap < p.spread && q.c + p.nhb - 1 < nchunks;
      const int krow = hlive ? q.tap * HPS : p.tab_rows;
      const unsigned* trow = tab_lane + krow * TROW;
#pragma unroll
      for (int j = 0; j < HPS; ++j) d.hv[j] = trow[j * TROW];
      d.ku = wave + NW * krow;
      d.hsoff = (unsigned)((q.c + p.nhb - 1) * CB * 2);
      d.hbase = q.foff;
    }
  };
  int pc = cbeg + DIST / taps, pt = DIST % taps;   // copy position: step it + DIST (past the end it re-fetches
  auto wgt_copies = [&](Copies& d) {               // the last chunk, which nobody reads)
    d.wsoff = (unsigned)__builtin_amdgcn_readfirstlane(__builtin_amdgcn_readlane(vt_wt, pt) + min(pc, nchunks - 1) * (CB * 2));
    const bool pwrap = pt + 1 == taps;
    pt = pwrap ? 0 : pt + 1;
    pc += pwrap ? 1 : 0;
  };

  Pos P{0, cbeg, 0, (p.nhb - 1) * p.halo_stride};
  Pos Pn = advance(P);
  int bstep = 0, nbstep = bstep_of(Pn);           // offsets of the current / next step's pixel rows
  Copies cp;
  act_copies(P, cp);
  wgt_copies(cp);
  unsigned char* const wlane = wbuf + aoff;

  bf16x8 fa[2][NCW], fb[2];
  auto load_frags = [&](int buf, const unsigned char* a, int bs, int kk) {
    fb[buf] = *reinterpret_cast<const bf16x8*>(halo + boff + bs + kk * 32);
#pragma unroll
    for (int r = 0; r < NCW; ++r) fa[buf][r] = *reinterpret_cast<const bf16x8*>(a + r * 32 * ROWP + kk * 32);
  };

  if (SC && p.bn.w_folded_out) emit_folded_slice(p.bn, p.wgt, bx, gx);   // while the first copies are in flight
  STAMP(1);
  wait_vm<(DIST - 1) * (WPW + HPS)>();   // the activation tile of the first chunk and the slab of step 0 have landed
  block_barrier();
  STAMP(2);
  load_frags(0, wlane, bstep, 0);

  auto step = [&](auto slot) {
    constexpr int S = decltype(slot)::value;            // ring slot of this step's slab
    constexpr int SN = (S + 1) % NBUF;                  // ... of the next step's
    constexpr int SF = (S + NBUF - 1) % NBUF;           // ... of the one refilled now (step it + DIST)
    wait_vm<(DIST - 2) * (WPW + HPS)>();
    block_barrier();   // the next step's data is resident for every wave; the previous step's slab is free

    // Copies are issued between the multiplies: a wave stalls on every copy it hands to the memory pipe,
    // and the matrix pipe keeps working through those stalls only if it has been fed first.  Units past
    // the tile go to the spare KB behind it (unit ucap), so no copy needs a branch or a select.
    auto issue_copy = [&](int idx) {   // copy idx of this step: HPS activation units, then WPW weight units
      if (idx < HPS) {
        dma16(act_rsrc, cp.hv[idx < HPS ? idx : 0], cp.hsoff, halo + cp.hbase + min(cp.ku + NW * idx, p.ucap) * UNITB);
      } else {
        const int j = idx - HPS < WPW ? idx - HPS : 0;
        dma16(wgt_rsrc, voff_w[j], cp.wsoff, wbuf + SF * WSLAB + wu_off[j]);
      }
    };
    // KK k-steps: operands of k-step kk+1 (or of the next step's first) load while kk multiplies.  The
    // scheduling barriers pin the order written here: operand reads of the following k-step, one multiply,
    // this k-step's share of the copies, the remaining multiplies, a share of the next step's bookkeeping.
    Pos P2 = Pn;
    int n2bstep = 0;
    Copies ncp = cp;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) load_frags((kk + 1) & 1, wlane + S * WSLAB, bstep, kk + 1);
      else load_frags((kk + 1) & 1, wlane + SN * WSLAB, nbstep, 0);
      __builtin_amdgcn_sched_barrier(0);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][0], fb[kk & 1], acc[0], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int idx = (kk * CPS) / KK; idx < ((kk + 1) * CPS) / KK; ++idx) issue_copy(idx);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 1; r < NCW; ++r)
        acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][r], fb[kk & 1], acc[r], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (kk == 0) { P2 = advance(Pn); n2bstep = bstep_of(P2); }
      if (kk == (KK > 2 ? 1 : 0)) act_copies(Pn, ncp);
      if (kk == KK - 1) wgt_copies(ncp);
      __builtin_amdgcn_sched_barrier(0);
    }
    P = Pn; Pn = P2;
    bstep = nbstep; nbstep = n2bstep;
    cp = ncp;
  };
  // Element offset of the channel block a lane stores for epilogue iteration (rp, i): pixel 32 wp + 8 i + lane / 8,
  // channels r0 + (cw0 / 2 + rp) 64 + 8 g; -1 where nothing is stored.
  auto store_off = [&](int rp, int i) -> long long {
    const int row = i * 8 + (lane >> 3);
    const int g = (lane & 7) ^ ((row >> 1) & 7);
    const int pi = wp * 32 + row;
    const int ch = r0 + (cw0 / 2 + rp) * 64 + g * 8;
    if (pi >= len || ch >= p.R) return -1;
    size_t o = (size_t)(m0 + pi) * p.R;
    if (p.out_strided) {
      const int m = m0 + pi;
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      const int ho = fdiv(rem, p.dWo);
      o = (size_t)p.out_base + (size_t)n * p.out_n + (size_t)ho * p.out_h + (size_t)(rem - ho * p.Wo) * p.out_w;
    }
    return (long long)(o + ch);
  };
  for (int left = nsteps;;) {
    step(std::integral_constant<int, 0>{}); if (--left == 0) break;
    step(std::integral_constant<int, 1>{}); if (--left == 0) break;
    step(std::integral_constant<int, 2>{}); if (--left == 0) break;
    step(std::integral_constant<int, 3>{}); if (--left == 0) break;
    if constexpr (NBUF == 5) { step(std::integral_constant<int, 4>{}); if (--left == 0) break; }
  }
  wait_vm<0>();   // trailing copies must not outlive the workgroup's LDS
  STAMP(3);

  // ---- epilogue -------------------------------------------------------------------------------
  // Accumulator element e of lane l: channel 8*(e/4) + 4*(l/32) + e%4, pixel l%32.  Each wave
  // rounds a 32-pixel x 64-channel block to bf16 into its own 4 KB of LDS ([pixel][64 ch], granules
  // swizzled by pixel), then reads it back row-wise so that every global store is 16 bytes per lane
  // and eight lanes cover one pixel's 128 contiguous bytes.
  if (p.ksplit > 1) {
    // fp32 partial sums of this workgroup's channel chunks; bias and rounding happen in the reduction
    const int pi = wp * 32 + (lane & 31);
    if (pi < len) {
      float* orow = p.part + ((size_t)by * p.M + m0 + pi) * p.R;
#pragma unroll
      for (int r = 0; r < NCW; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = r0 + (cw0 + r) * 32 + q * 8 + kb * 4;
          if (row < p.R)
            *reinterpret_cast<float4*>(orow + row) = make_float4(acc[r][q * 4 + 0], acc[r][q * 4 + 1],
                                                                 acc[r][q * 4 + 2], acc[r][q * 4 + 3]);
        }
    }
    return;
  }
  if (tid < TRC) { biasl[tid] = bias_v; if (SC) biasl[128 + tid] = scale_v; }   // scales behind the (at most 128) biases
  __syncthreads();   // every wave's copies have landed, every wave is done with the ring, the bias is visible
  {
    unsigned char* stage = smem + 1024 + wave * 4096;   // behind the bias, over the (now idle) ring and tiles
    const int px = lane & 31;
    const int psw = (px >> 1) & 7;
    const int pbase = wp * 32;
#pragma unroll
    for (int rp = 0; rp < NCW / 2; ++rp) {
#pragma unroll
      for (int r2 = 0; r2 < 2; ++r2) {
        const int r = 2 * rp + r2;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ch = r2 * 32 + q * 8 + kb * 4;          // channel inside this 64-channel block
          const float4 bb = *reinterpret_cast<const float4*>(biasl + (cw0 + r) * 32 + q * 8 + kb * 4);
          uint2 v;
          if constexpr (SC) {   // unfolded weight: the BatchNorm scale is applied here
            const float4 sc = *reinterpret_cast<const float4*>(biasl + 128 + (cw0 + r) * 32 + q * 8 + kb * 4);
            v = make_uint2(pack_bf16x2(fmaf(acc[r][q * 4 + 0], sc.x, bb.x), fmaf(acc[r][q * 4 + 1], sc.y, bb.y)),
                           pack_bf16x2(fmaf(acc[r][q * 4 + 2], sc.z, bb.z), fmaf(acc[r][q * 4 + 3], sc.w, bb.w)));
          } else {
            v = make_uint2(pack_bf16x2(acc[r][q * 4 + 0] + bb.x, acc[r][q * 4 + 1] + bb.y),
                           pack_bf16x2(acc[r][q * 4 + 2] + bb.z, acc[r][q * 4 + 3] + bb.w));
          }
          *reinterpret_cast<uint2*>(stage + px * 128 + (((ch >> 3) ^ psw) << 4) + ((ch & 7) << 1)) = v;
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = i * 8 + (lane >> 3);
        const int g = (lane & 7) ^ ((row >> 1) & 7);
        const uint4 v = *reinterpret_cast<const uint4*>(stage + row * 128 + ((lane & 7) << 4));
        (void)g; (void)pbase;
        const long long o = store_off(rp, i);
        if (o >= 0) *reinterpret_cast<uint4*>(p.out + o) = post_op8(v, p.relu, p.mask, p.add, (size_t)o);
      }
    }
  }
  STAMP(4);
}

template <int NW, int NWC, int NCH, int CB, int HPS, bool SC = false>
__global__ __launch_bounds__(64 * NW) void conv_tile_kernel(TileParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  tile_body<NW, NWC, NCH, CB, HPS, SC>(p, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.x, smem);
}

// Several problems of one kernel shape in ONE launch (the residue classes of a strided input gradient: each alone
// leaves most of the chip idle, and launches of one stream do not overlap): the workgroups of problem c are
// [first[c], first[c + 1]).  No split sums.
struct TileMulti {
  TileParams p[4];
  int first[5];
  int n;
};
template <int NW, int NWC, int NCH, int CB, int HPS>
__global__ __launch_bounds__(64 * NW) void conv_tile_multi_kernel(TileMulti m) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int b = (int)blockIdx.x;
  int c = 0;
  while (c + 1 < m.n && b >= m.first[c + 1]) ++c;
  c = __builtin_amdgcn_readfirstlane(c);
  tile_body<NW, NWC, NCH, CB, HPS, false>(m.p[c], b - m.first[c], 0, m.first[c + 1] - m.first[c], smem);
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

struct TilePlan { bool ok; int nw, nwc, nch, cb, hps; size_t lds; };

// fp32 partial-output bytes a problem needs (0 when the channel chunks are not split).
size_t partial_bytes(const TileParams& p) {
  return p.ksplit > 1 ? (size_t)p.ksplit * p.M * p.R * 4 : 0;
}

constexpr size_t LDS_LIMIT = 160 * 1024;
constexpr size_t LDS_USABLE = LDS_LIMIT - 1024;

// Fills ksplit / nhb / hps / spread / halo_stride / tab_off / tab_rows for (nw, nch, cb); returns the
// LDS bytes (0 = this configuration cannot run the problem).
template <int NCH, int CB>
size_t plan_lds_cfg(TileParams& p, int nw, int nwc, bool rows) {
  using Cfg = TileCfg<NCH, CB>;
  const int taps = p.kH * p.kW;
  if (p.C % CB) return 0;
  // split the channel chunks over several workgroups when the pixel x channel tiling alone
  // leaves most of the chip idle
  const int all_chunks = p.C / CB;
  const int TPx = 32 * (nw / nwc);
  p.tile_rows = 0;
  p.tiles_per_image = 0;
  if (rows) {
    // whole-row tiles: only where they fill most of the tile's lanes
    if (p.Wo > TPx) return 0;
    const int tr = TPx / p.Wo < p.Ho ? TPx / p.Wo : p.Ho;
    if ((long long)p.M * 100 < (long long)85 * p.N * ceil_div(p.Ho, tr) * TPx) return 0;
    p.tile_rows = tr;
    p.tiles_per_image = ceil_div(p.Ho, tr);
    p.dTpi = make_fastdiv(p.tiles_per_image);
  }
  const long long ptiles = rows ? (long long)p.N * p.tiles_per_image : ceil_div(p.M, TPx);
  const long long blocks = ptiles * ceil_div(p.R, Cfg::TRC);
  int ks = 1;
  if (blocks < 160 && all_chunks >= 4 && !p.no_split) {
    ks = (int)((200 + blocks - 1) / blocks);
    if (ks > all_chunks / 2) ks = all_chunks / 2;
    if (ks > 8) ks = 8;
  }
  p.chunks_per_split = ceil_div(all_chunks, ks);
  p.ksplit = ceil_div(all_chunks, p.chunks_per_split);
  const int nchunks = p.chunks_per_split;
  const int slots = rows ? (p.tile_rows - 1) * p.sh + p.kH : max_slots(p, TPx);
  const int hunits = ceil_div(slots * p.Wv, Cfg::RPU);
  const int per_wave = ceil_div(hunits, nw);
  int nhb, spread, hps;
  if (nchunks == 1) { nhb = 1; spread = 0; hps = 0; }
  else {
    // 1x1 windows with several chunks: the generic implicit-GEMM kernel is only faster for mid-sized pixel
    // counts with many more output than input channels (many channel tiles re-reading a short reduction)
    if (taps == 1 && p.M > 2048 && p.M <= 8192 && p.R >= 2 * p.C) return 0;
    // copies per wave and step (the kernel is instantiated for 1, 2, 3, 4, 6, 8), spread over as few
    // steps as the pipeline leaves between two chunks
    nhb = 2;
    while ((nhb - 1) * taps - Cfg::DIST + 1 < 1) ++nhb;
    const int room = (nhb - 1) * taps - Cfg::DIST + 1;
    const int max_spread = room < taps ? room : taps;
    static const int hps_values[] = {1, 2, 3, 4, 6, 8};
    hps = 0;
    for (int v : hps_values)
      if (v >= p.min_hps && ceil_div(per_wave, v) <= max_spread) { hps = v; break; }
    if (hps == 0) return 0;
    spread = ceil_div(per_wave, hps);
  }
  p.nhb = nhb; p.hps = hps; p.spread = spread;
  p.tab_rows = spread * hps;
  p.ucap = hunits;
  p.halo_stride = (hunits + (nchunks > 1 ? 1 : 0)) * Cfg::UNITB + 64;
  size_t lds = 1024 + (size_t)Cfg::NBUF * Cfg::WSLAB + 1024 + (size_t)nhb * p.halo_stride;
  p.tab_off = (int)lds;
  if (nhb > 1) lds += (size_t)(p.tab_rows + hps) * nw * 256;
  const size_t stage = 1024 + (size_t)nw * 4096;   // the epilogue stages 4 KB per wave behind the bias
  return lds < stage ? stage : lds;
}

size_t plan_lds(TileParams& p, int nw, int nwc, int nch, int cb, bool rows) {
  if (nwc > 1 && nch != 4) return 0;   // channel groups need two 32-channel subtiles per wave
  if (nch == 2) return cb == 64 ? plan_lds_cfg<2, 64>(p, nw, nwc, rows) : plan_lds_cfg<2, 32>(p, nw, nwc, rows);
  return cb == 64 ? plan_lds_cfg<4, 64>(p, nw, nwc, rows) : plan_lds_cfg<4, 32>(p, nw, nwc, rows);
}

TilePlan make_plan(TileParams& p) {
  TilePlan pl{false, 0, 0, 0, 0, 0, 0};
  if (p.C % 8 || p.R % 8) return pl;
  if (p.act_bytes >= OOB || p.wgt_bytes >= OOB) return pl;   // byte offsets must stay below the zero-fill offset
  p.dHoWo = make_fastdiv(p.Ho * p.Wo);
  p.dWo = make_fastdiv(p.Wo);
  p.dHv = make_fastdiv(p.Hv);
  p.dWv = make_fastdiv(p.Wv);
  pl.nch = p.R > 64 ? 4 : 2;
  // Candidate shapes (waves, channel groups, channels per chunk):
  //   (8,1): 256 pixels, eight waves -- two per SIMD hide each other's scalar work; many pixels.
  //   (16,1): 512 pixels, whole-row tiles only.
  //   (4,1): 128 pixels, four waves.
  //   (4,2): 64 pixels, the four waves split the 128 channels two ways -- a small pixel tile that still
  //          gives every wave a 32 x 64 block; deep reductions over few pixels (no split sums up to
  //          ~3000 pixels), and the stride-2 3x3 layers whose window tiles would not fit otherwise.
  // First choice: whole-row tiles where they apply (wide images: a smaller activation tile for the
  // same pixels).  Then the first candidate that fills the chip (>= 160 workgroups) without splitting
  // the channel chunks -- split sums cost an fp32 round trip through memory and a second kernel.
  // Else the first that fits, largest tile first for many pixels, smallest first for few.
  // 64-channel chunks wherever the LDS allows.
  struct Cand { int nw, nwc, cb; };
  static const Cand many[] = {{8, 1, 64}, {8, 1, 32}, {4, 1, 64}, {4, 1, 32}, {4, 2, 64}, {4, 2, 32}};
  static const Cand few[] = {{4, 2, 64}, {4, 2, 32}, {4, 1, 64}, {4, 1, 32}, {8, 1, 64}, {8, 1, 32}};
  constexpr int NCAND = 6;
  {
    // Whole-row tiles of 8 or 16 waves.  Workgroups of this size run one per CU, in rounds; a round costs a
    // fixed start-up and drain (the tile's copies and stores go at memory speed with the matrix pipe idle)
    // plus its steps, which take twice as long with four waves per SIMD as with two -- so the larger tile
    // wins where it saves rounds (N = 32, 56 x 56: 224 workgroups in one round instead of 448 in two).
    TileParams best{};
    size_t best_lds = 0;
    long long best_cost = 0;
    int best_nw = 0;
    for (int nw : {8, 16}) {
      TileParams q = p;
      if (nw == 16 && pl.nch != 2) continue;   // sixteen waves are built for 64 output channels per workgroup
      const size_t lds = p.C >= 64 ? plan_lds(q, nw, 1, pl.nch, 64, true) : 0;
      const long long wgs = (long long)q.N * q.tiles_per_image * ceil_div(q.R, pl.nch * 32);
      if (lds == 0 || lds > LDS_USABLE || q.ksplit != 1 || wgs < 160) continue;
      const long long steps = (long long)p.kH * p.kW * (p.C / 64);
      const long long cost = ceil_div((int)wgs, 256) * (8000 + steps * 260 * (nw / 4));
      if (best_nw == 0 || cost < best_cost) { best = q; best_lds = lds; best_cost = cost; best_nw = nw; }
    }
    if (best_nw != 0) {
      p = best;
      pl.nw = best_nw; pl.nwc = 1; pl.cb = 64; pl.lds = best_lds; pl.hps = p.hps;
      p.ntr = ceil_div(p.R, pl.nch * 32);
      pl.ok = true;
      return pl;
    }
  }
  const long long blocks256 = (long long)ceil_div(p.M, 256) * ceil_div(p.R, pl.nch * 32);
  const Cand* fallback = (blocks256 >= 384 || p.M >= 4096) ? many : few;
  for (int pass = 0; pass < 2; ++pass) {
    const Cand* cands = pass == 0 ? many : fallback;
    for (int i = 0; i < NCAND; ++i) {
      const Cand& cd = cands[i];
      if (p.C < cd.cb) continue;
      TileParams q = p;
      const size_t lds = plan_lds(q, cd.nw, cd.nwc, pl.nch, cd.cb, false);
      if (lds == 0 || lds > LDS_USABLE) continue;
      if (pass == 0) {
        const long long blocks = (long long)ceil_div(q.M, 32 * (cd.nw / cd.nwc)) * ceil_div(q.R, pl.nch * 32);
        if (q.ksplit != 1 || blocks < 160) continue;
      }
      p = q;
      pl.nw = cd.nw; pl.nwc = cd.nwc; pl.cb = cd.cb; pl.lds = lds; pl.hps = p.hps;
      p.ntr = ceil_div(p.R, pl.nch * 32);
      pl.ok = true;
      return pl;
    }
  }
  return pl;
}

template <int NW, int NWC, int NCH, int CB, int HPS, bool SC = false>
hipError_t launch_inst(const TileParams& p, const TilePlan& pl, hipStream_t st) {
  static LdsLimitOnce lds_once;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&conv_tile_kernel<NW, NWC, NCH, CB, HPS, SC>),
                                        (int)LDS_USABLE); e != hipSuccess) return e;
  const int ptiles = p.tile_rows > 0 ? p.N * p.tiles_per_image : ceil_div(p.M, 32 * (NW / NWC));
  hipLaunchKernelGGL((conv_tile_kernel<NW, NWC, NCH, CB, HPS, SC>), dim3(p.ntr * ptiles, p.ksplit), dim3(64 * NW), pl.lds, st,
                     p);
  hipError_t le = hipGetLastError();
  if (le != hipSuccess || p.ksplit == 1) return le;
  const size_t MR = (size_t)p.M * p.R;
  const int rblocks = (int)(((MR >> 3) + 255) / 256 < 2048 ? ((MR >> 3) + 255) / 256 : 2048);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(rblocks), dim3(256), 0, st, p.part, p.ksplit, MR, p.R, p.bias, p.out);
  le = hipGetLastError();
  // split sums: the reduction wrote the output, ReLU and mask follow as passes of their own
  if (le == hipSuccess && p.add) le = launch_eltwise(3 /* a + b */, CONVBN_BF16, p.out, p.add, nullptr, MR, st);
  if (le == hipSuccess && p.relu) le = launch_eltwise(0, CONVBN_BF16, p.out, nullptr, nullptr, MR, st);
  if (le == hipSuccess && p.mask) le = launch_eltwise(1, CONVBN_BF16, p.out, p.mask, nullptr, MR, st);
  return le;
}

// The scale-in-the-epilogue ablation is built for the plans of the 3x3 benchmark shapes only.
bool scaled_plan(const TilePlan& pl) {
  return (pl.nw == 16 && pl.nwc == 1 && pl.nch == 2 && pl.cb == 64 && pl.hps == 0) ||
         (pl.nw == 8 && pl.nwc == 1 && pl.nch == 2 && pl.cb == 64 && pl.hps == 0) ||
         (pl.nw == 4 && pl.nwc == 2 && pl.nch == 4 && pl.cb == 64 && pl.hps == 1);
}

hipError_t launch_plan(const TileParams& p, const TilePlan& pl, hipStream_t st) {
  if (p.bn.gamma) {
    if (pl.nw == 16 && pl.hps == 0) return launch_inst<16, 1, 2, 64, 0, true>(p, pl, st);
    if (pl.nw == 8 && pl.hps == 0) return launch_inst<8, 1, 2, 64, 0, true>(p, pl, st);
    return launch_inst<4, 2, 4, 64, 1, true>(p, pl, st);
  }
#define CASE(NWV, WC, NC, CBV, H) \
  if (pl.nw == NWV && pl.nwc == WC && pl.nch == NC && pl.cb == CBV && pl.hps == H) \
    return launch_inst<NWV, WC, NC, CBV, H>(p, pl, st);
#define CASES(NWV, WC, NC, CBV) \
  CASE(NWV, WC, NC, CBV, 0) CASE(NWV, WC, NC, CBV, 1) CASE(NWV, WC, NC, CBV, 2) CASE(NWV, WC, NC, CBV, 3) \
  CASE(NWV, WC, NC, CBV, 4) CASE(NWV, WC, NC, CBV, 6) CASE(NWV, WC, NC, CBV, 8)
  CASES(4, 1, 2, 32) CASES(4, 1, 2, 64) CASES(4, 1, 4, 32) CASES(4, 1, 4, 64)
  CASES(8, 1, 2, 32) CASES(8, 1, 2, 64) CASES(8, 1, 4, 32) CASES(8, 1, 4, 64)
  CASES(4, 2, 4, 32) CASES(4, 2, 4, 64) CASES(16, 1, 2, 64)
#undef CASES
#undef CASE
  return hipErrorInvalidValue;
}

template <int NW, int NWC, int NCH, int CB, int HPS>
hipError_t launch_multi_inst(const TileMulti& m, size_t lds, hipStream_t st) {
  static LdsLimitOnce lds_once;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&conv_tile_multi_kernel<NW, NWC, NCH, CB, HPS>),
                                        (int)LDS_USABLE); e != hipSuccess) return e;
  hipLaunchKernelGGL((conv_tile_multi_kernel<NW, NWC, NCH, CB, HPS>), dim3(m.first[m.n]), dim3(64 * NW), lds, st, m);
  return hipGetLastError();
}
// the kernel shapes the strided 3x3 layers of a ResNet ask for; anything else runs class by class
bool multi_shape(const TilePlan& pl) {
  return (pl.nw == 4 && pl.nwc == 2 && pl.nch == 4 && pl.cb == 64 && (pl.hps == 2 || pl.hps == 3)) ||
         (pl.nw == 4 && pl.nwc == 1 && pl.nch == 4 && pl.cb == 32 && (pl.hps == 4 || pl.hps == 6));
}
hipError_t launch_multi(const TileMulti& m, const TilePlan& pl, size_t lds, hipStream_t st) {
  if (pl.cb == 64 && pl.hps == 2) return launch_multi_inst<4, 2, 4, 64, 2>(m, lds, st);
  if (pl.cb == 64 && pl.hps == 3) return launch_multi_inst<4, 2, 4, 64, 3>(m, lds, st);
  if (pl.cb == 32 && pl.hps == 4) return launch_multi_inst<4, 1, 4, 32, 4>(m, lds, st);
  if (pl.cb == 32 && pl.hps == 6) return launch_multi_inst<4, 1, 4, 32, 6>(m, lds, st);
  return hipErrorInvalidValue;
}

// A 1x1 window with stride 1 and no padding is a plain matrix product over all N*H*W pixels: present
// the activations as one image of M rows and one column, so a pixel tile is exactly its own rows.
void flatten_pointwise(TileParams& q, int M, int C) {
  q.N = 1; q.H = M; q.W = 1; q.Ho = M; q.Wo = 1;
  q.act_n_stride = 0; q.act_h_stride = C; q.act_w_stride = 0;
  q.sh = q.sw = 1; q.ph = q.pw = 0;
  q.Hv = M; q.Wv = 1;
}

bool fprop_params(const Geom& g, TileParams* p) {
  TileParams& q = *p;
  q = TileParams{};
  q.N = g.N; q.C = g.Cin; q.Ho = g.Hout; q.Wo = g.Wout; q.R = g.Cout; q.M = g.M;
  q.kH = g.kH; q.kW = g.kW;
  if (g.kH * g.kW > 64) return false;   // the kernel keeps one table entry per tap in a lane
  q.wt0 = 0; q.wt_row = g.kW; q.wt_col = 1;
  q.wrow = g.kH * g.kW * q.C;
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
  if (g.kH == 1 && g.kW == 1 && g.ph == 0 && g.pw == 0 && g.sh == 1 && g.sw == 1) flatten_pointwise(q, g.M, g.Cin);
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
  q.ph = g.kH - 1 - g.ph; q.pw = g.kW - 1 - g.pw;
  if (g.kH * g.kW > 64) return false;
  q.wt0 = g.kH * g.kW - 1; q.wt_row = -g.kW; q.wt_col = -1;   // rotated kernel
  q.wrow = g.kH * g.kW * q.C;
  q.act_n_stride = g.Hout * g.Wout * g.Cout;
  q.act_h_stride = g.Wout * g.Cout;
  q.act_w_stride = g.Cout;
  q.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  q.Hv = (q.Ho - 1) + q.kH;
  q.Wv = (q.Wo - 1) + q.kW;
  if (g.kH == 1 && g.kW == 1 && g.ph == 0 && g.pw == 0) flatten_pointwise(q, g.Min, g.Cout);
  return true;
}

// Input gradient of a strided convolution, one residue class of input positions at a time
// (Sec. 3.2.1: dX = w'_rot (*) dZ): the positions h = sh hq + a, w = sw wq + b only receive the taps
// i = i0 + sh ti, j = j0 + sw tj with i0 = (a + ph) mod sh, j0 = (b + pw) mod sw, and
//   dX[n, h, w] = sum_{ti,tj} w'[i, j] . dZ[n, hq + dh0 - ti, wq + dw0 - tj],   dh0 = (a + ph - i0) / sh,
// which is a stride-1 sweep over dZ with a (kh x kw) window, padding (kh-1-dh0, kw-1-dw0) and the taps
// taken in reverse -- no multiplications with the zeros a dilated dZ would contain.  The result is
// written to the class's positions of dX.
enum ClassKind { CLASS_RUN, CLASS_NO_PIXELS, CLASS_ZERO, CLASS_UNSUPPORTED };
ClassKind dgrad_class_params(const Geom& g, int a, int b, TileParams* p) {
  const int Hq = a < g.Hin ? (g.Hin - a + g.sh - 1) / g.sh : 0;
  const int Wq = b < g.Win ? (g.Win - b + g.sw - 1) / g.sw : 0;
  if (Hq == 0 || Wq == 0) return CLASS_NO_PIXELS;
  const int i0 = (a + g.ph) % g.sh, j0 = (b + g.pw) % g.sw;
  const int kh = i0 < g.kH ? (g.kH - i0 + g.sh - 1) / g.sh : 0;
  const int kw = j0 < g.kW ? (g.kW - j0 + g.sw - 1) / g.sw : 0;
  if (kh == 0 || kw == 0) return CLASS_ZERO;   // no tap reaches these positions
  const int dh0 = (a + g.ph - i0) / g.sh, dw0 = (b + g.pw - j0) / g.sw;
  if (kh - 1 - dh0 < 0 || kw - 1 - dw0 < 0 || kh * kw > 64) return CLASS_UNSUPPORTED;
  TileParams& q = *p;
  q = TileParams{};
  q.N = g.N; q.C = g.Cout; q.H = g.Hout; q.W = g.Wout;
  q.Ho = Hq; q.Wo = Wq; q.R = g.Cin; q.M = g.N * Hq * Wq;
  q.kH = kh; q.kW = kw; q.sh = 1; q.sw = 1;
  q.ph = kh - 1 - dh0; q.pw = kw - 1 - dw0;
  q.wt0 = (i0 + g.sh * (kh - 1)) * g.kW + j0 + g.sw * (kw - 1);
  q.wt_row = -g.sh * g.kW; q.wt_col = -g.sw;
  q.act_n_stride = g.Hout * g.Wout * g.Cout;
  q.act_h_stride = g.Wout * g.Cout;
  q.act_w_stride = g.Cout;
  q.act_bytes = (unsigned)((size_t)g.M * g.Cout * 2);
  q.wgt_bytes = (unsigned)((size_t)g.Cout * g.K * 2);
  q.Hv = (q.Ho - 1) + q.kH;
  q.Wv = (q.Wo - 1) + q.kW;
  q.wrow = g.kH * g.kW * g.Cout;
  q.no_split = 1;
  q.out_strided = 1;
  q.out_base = (a * g.Win + b) * g.Cin;
  q.out_n = g.Hin * g.Win * g.Cin;
  q.out_h = g.sh * g.Win * g.Cin;
  q.out_w = g.sw * g.Cin;
  return CLASS_RUN;
}

// The same problem for the tiled product's window mode (conv_gm.hip), which takes strided windows: they hardly overlap,
// so a window tile in LDS buys little and costs the chunk width (32-channel chunks here against 64 there).
GmConv gm_conv_of(const TileParams& q) {
  GmConv c{};
  c.kH = q.kH; c.kW = q.kW; c.cph = q.ph; c.cpw = q.pw; c.csh = q.sh; c.csw = q.sw; c.aH = q.H; c.aW = q.W;
  c.a_n = q.act_n_stride; c.a_h = q.act_h_stride; c.a_w = q.act_w_stride;
  c.oHo = q.Ho; c.oWo = q.Wo;
  c.wt0 = q.wt0; c.wt_row = q.wt_row; c.wt_col = q.wt_col; c.wrow = q.wrow;
  c.out_strided = q.out_strided; c.out_base = q.out_base; c.out_n = q.out_n; c.out_h = q.out_h; c.out_w = q.out_w;
  return c;
}

// Every pixel row of out ([pixels][R] bf16, R % 8 == 0) := bf16(bias) (zeros without a bias).
__global__ __launch_bounds__(256) void fill_rows_kernel(uint4* __restrict__ out, size_t n16, int R,
                                                        const float* __restrict__ bias) {
  const int r8 = R >> 3;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (bias) {
      const float* bb = bias + (size_t)(i % r8) * 8;
      v = make_uint4(pack_bf16x2(bb[0], bb[1]), pack_bf16x2(bb[2], bb[3]), pack_bf16x2(bb[4], bb[5]),
                     pack_bf16x2(bb[6], bb[7]));
    }
    out[i] = v;
  }
}

}  // namespace

bool tile_fprop_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  TileParams p;
  if (!fprop_params(g, &p)) return false;
  if ((g.sh > 1 || g.sw > 1) && g.kH * g.kW > 1 && p.C % 8 == 0 && p.act_bytes < OOB && p.wgt_bytes < OOB &&
      (size_t)p.M * p.R * 2 < OOB && gm_conv_supported(p.M, p.C, p.R, gm_conv_of(p)))
    return true;   // the tiled product's window mode takes it
  return make_plan(p).ok;
}

bool tile_dgrad_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  TileParams p;
  if (g.sh == 1 && g.sw == 1) return dgrad_params(g, &p) && make_plan(p).ok;
  if ((size_t)g.Min * g.Cin * 2 >= OOB || g.Cin % 8) return false;
  for (int a = 0; a < g.sh; ++a)
    for (int b = 0; b < g.sw; ++b) {
      const ClassKind k = dgrad_class_params(g, a, b, &p);
      if (k == CLASS_RUN && p.act_bytes < OOB && p.wgt_bytes < OOB && gm_conv_supported(p.M, p.C, p.R, gm_conv_of(p))) continue;
      if (k == CLASS_UNSUPPORTED || (k == CLASS_RUN && !make_plan(p).ok)) return false;
    }
  return true;
}

bool tile_fprop_scaled_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  TileParams p;
  if (!fprop_params(g, &p)) return false;
  const TilePlan pl = make_plan(p);
  return pl.ok && p.ksplit == 1 && scaled_plan(pl);
}

size_t tile_fprop_partial_bytes(const Geom& g) {
  TileParams p;
  if (!fprop_params(g, &p) || !make_plan(p).ok) return 0;
  return partial_bytes(p);
}

size_t tile_dgrad_partial_bytes(const Geom& g) {
  TileParams p;
  if (g.sh != 1 || g.sw != 1) return 0;   // the residue-class launches do not split their sums
  if (!dgrad_params(g, &p) || !make_plan(p).ok) return 0;
  return partial_bytes(p);
}

hipError_t launch_fprop_tile(const Geom& g, const void* x, const void* w_krsc, const float* bias,
                             void* z, float* partials, hipStream_t st, const BnEpilogue* bn) {
  TileParams p;
  fprop_params(g, &p);
  if (!bn && (g.sh > 1 || g.sw > 1) && g.kH * g.kW > 1) {
    const GmConv cv = gm_conv_of(p);
    if (gm_conv_supported(p.M, p.C, p.R, cv))
      return launch_gm_conv(p.M, p.C, p.R, cv, x, p.act_bytes, w_krsc, p.wgt_bytes, bias, z, g.post_relu, g.post_mask,
                            g.post_add, st);
  }
  const TilePlan pl = make_plan(p);
  if (p.ksplit > 1 && (!partials || bn)) return hipErrorInvalidValue;   // split sums add the bias in their reduction
  if (bn && !scaled_plan(pl)) return hipErrorInvalidValue;
  if (bn) p.bn = *bn;
  p.act = (const bf16_t*)x; p.wgt = (const bf16_t*)w_krsc; p.bias = bias; p.out = (bf16_t*)z;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  p.part = partials;
  return launch_plan(p, pl, st);
}

hipError_t launch_dgrad_tile(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                             float* partials, hipStream_t st) {
  TileParams p;
  if (g.sh != 1 || g.sw != 1) {
    bool zero_first = false;
    for (int a = 0; a < g.sh; ++a)
      for (int b = 0; b < g.sw; ++b) zero_first |= dgrad_class_params(g, a, b, &p) == CLASS_ZERO;
    // an addend also reaches the positions no tap does: then the whole post-operation follows as passes of its own
    const bool defer = zero_first && g.post_add != nullptr;
    if (zero_first) {   // positions no tap reaches hold the bias alone: fill dX once, the other classes overwrite theirs
      const size_t n16 = (size_t)g.Min * g.Cin * 2 / 16;
      const int blocks = (int)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
      hipLaunchKernelGGL(fill_rows_kernel, dim3(blocks), dim3(256), 0, st, (uint4*)dx, n16, g.Cin, bias);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    // all classes as one launch where they share a kernel shape (the one that needs the most copy units per step
    // sets it for all), at most four of them, none with split sums
    {
      TileMulti m{};
      TilePlan pls[4];
      int n = 0, hps = 0;
      bool same = true;
      for (int a = 0; a < g.sh && same; ++a)
        for (int b = 0; b < g.sw && same; ++b) {
          TileParams q;
          if (dgrad_class_params(g, a, b, &q) != CLASS_RUN) continue;
          if (n == 4) { same = false; break; }
          pls[n] = make_plan(q);
          same = pls[n].ok && q.ksplit == 1 && multi_shape(pls[n]) &&
                 (n == 0 || (pls[n].nw == pls[0].nw && pls[n].nwc == pls[0].nwc && pls[n].nch == pls[0].nch && pls[n].cb == pls[0].cb));
          if (pls[n].hps > hps) hps = pls[n].hps;
          ++n;
        }
      if (same && n >= 2) {
        size_t lds = 0;
        n = 0;
        for (int a = 0; a < g.sh && same; ++a)
          for (int b = 0; b < g.sw && same; ++b) {
            TileParams& q = m.p[n];
            if (dgrad_class_params(g, a, b, &q) != CLASS_RUN) continue;
            q.min_hps = hps;
            const TilePlan pl = make_plan(q);
            same = pl.ok && q.ksplit == 1 && pl.hps == hps && pl.nw == pls[0].nw && pl.nwc == pls[0].nwc &&
                   pl.nch == pls[0].nch && pl.cb == pls[0].cb;
            if (!same) break;
            q.act = (const bf16_t*)dz; q.wgt = (const bf16_t*)w_crsk; q.bias = bias; q.out = (bf16_t*)dx;
            q.relu = g.post_relu; q.mask = (const bf16_t*)g.post_mask; q.add = (const bf16_t*)g.post_add;
            if (defer) { q.relu = 0; q.mask = nullptr; q.add = nullptr; }
            q.part = nullptr;
            const int ptiles = q.tile_rows > 0 ? q.N * q.tiles_per_image : ceil_div(q.M, 32 * (pl.nw / pl.nwc));
            m.first[n + 1] = m.first[n] + q.ntr * ptiles;
            if (pl.lds > lds) lds = pl.lds;
            pls[n] = pl;
            ++n;
          }
        // (measured: it pays for the deep layer, whose classes are long reductions over few pixels -- 512 channels,
        // 14 x 14, 100 workgroups per class: 48.5 -> 33.5 us; with 256 channels at 28 x 28, 98 workgroups per class,
        // the classes are bound by their traffic and one launch takes 42.9 against 40.4 us)
        if (same && m.first[n] <= 448 && g.Cout >= 512) {
          m.n = n;
          hipError_t e = launch_multi(m, pls[0], lds, st);
          if (e != hipSuccess) return e;
          goto classes_done;
        }
      }
    }
    for (int a = 0; a < g.sh; ++a)
      for (int b = 0; b < g.sw; ++b) {
        if (dgrad_class_params(g, a, b, &p) != CLASS_RUN) continue;
        {
          const GmConv cv = gm_conv_of(p);
          if (gm_conv_supported(p.M, p.C, p.R, cv)) {
            hipError_t e = launch_gm_conv(p.M, p.C, p.R, cv, dz, p.act_bytes, w_crsk, p.wgt_bytes, bias, dx,
                                          defer ? 0 : g.post_relu, defer ? nullptr : g.post_mask,
                                          defer ? nullptr : g.post_add, st);
            if (e != hipSuccess) return e;
            continue;
          }
        }
        const TilePlan pl = make_plan(p);
        if (!pl.ok) return hipErrorInvalidValue;
        p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = bias; p.out = (bf16_t*)dx;
        p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
        if (defer) { p.relu = 0; p.mask = nullptr; p.add = nullptr; }
        p.part = nullptr;
        hipError_t e = launch_plan(p, pl, st);
        if (e != hipSuccess) return e;
      }
  classes_done:
    if (defer) {
      const size_t n = (size_t)g.Min * g.Cin;
      hipError_t e = launch_eltwise(3 /* a + b */, CONVBN_BF16, dx, g.post_add, nullptr, n, st);
      if (e == hipSuccess && g.post_relu) e = launch_eltwise(0, CONVBN_BF16, dx, nullptr, nullptr, n, st);
      if (e == hipSuccess && g.post_mask) e = launch_eltwise(1, CONVBN_BF16, dx, g.post_mask, nullptr, n, st);
      return e;
    }
    return hipSuccess;
  }
  dgrad_params(g, &p);
  const TilePlan pl = make_plan(p);
  if (p.ksplit > 1 && !partials) return hipErrorInvalidValue;
  p.act = (const bf16_t*)dz; p.wgt = (const bf16_t*)w_crsk; p.bias = bias; p.out = (bf16_t*)dx;
  p.relu = g.post_relu; p.mask = (const bf16_t*)g.post_mask; p.add = (const bf16_t*)g.post_add;
  p.part = partials;
  return launch_plan(p, pl, st);
}

}  // namespace convbn

#ifdef TILE_TRACE
extern "C" int convbn_debug_read_tile_trace(unsigned long long* host, size_t n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(convbn::tile_trace), n * sizeof(unsigned long long));
}
#endif
