// bf16 MFMA weight gradient  dw'[co][tap][ci] = sum_m dZ[m][co] * Xpad[m (+) tap][ci]
// (Sec. 3.2.1: dJ/dw = dJ/dY (.) X) together with the per-channel sum r_c = sum_m dZ[m][co]
// (App. B), both as fp32 partial sums over slices ("splits") of the output pixels.
//
// A workgroup owns a (CO_T x CI_T) channel tile, a group of TPB taps and one pixel split, and
// walks the split in tiles of 128 output pixels.  Per tile the dZ rows and the input-window rows
// those pixels touch are copied into LDS in their natural [pixel][channel] order (direct
// global->LDS buffer loads, zero-filled outside the tensors), double-buffered so the next tile
// streams in while the current one is multiplied.  The reduced index of this GEMM is the pixel,
// which is the strided direction of that layout, so the MFMA operands are read with the
// transposing LDS load (ds_read_b64_tr_b16: a 16-lane group turns a 4-pixel x 16-channel block
// into "lane = channel, 4 pixels per lane").  Every tap reuses the same LDS tile at a
// wave-uniform pixel offset.
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

constexpr int TP = 128;          // output pixels per tile
constexpr int ROWB = 144;        // LDS row: 64 channels of bf16 + one 16-byte pad granule
constexpr int UNITB = 7 * ROWB;  // bytes one wave-wide copy advances: 7 rows (its 64th lane lands on
                                 // the first granule of row 8, where it repeats the next copy's data)
constexpr int ZTILE = TP * ROWB + 1024;   // dZ tile: 128 rows, rounded up to whole copies + slack
constexpr unsigned OOB = 0x80000000u;

struct WgParams {
  const bf16_t* x;
  const bf16_t* dz;
  float* part;       // [nsplit][Co][taps][Cin]
  float* r_part;     // [nsplit][Co]
  unsigned x_bytes, dz_bytes;
  int N, H, W, Cin;                      // input grid the window slides over
  int x_n_stride, x_h_stride, x_w_stride;
  int Ho, Wo, Co;
  int kH, kW, sh, sw, ph, pw;
  int M, Hv, Wv;
  int nci, nco, ntg;                     // channel tiles, tap groups
  int ntiles, tiles_per_split;           // 128-pixel tiles
  int tpi;                               // tiles per image (tiles never straddle images), 0 = tiles are
                                         // consecutive 128-pixel runs of the whole batch
  int halo_sub_bytes;                    // bytes of one 64-channel window tile
  int buf_bytes;                         // bytes of one stage (window tiles + dZ tiles + pixel table)
  FastDiv dHoWo, dWo, dHv, dWv, dkW;
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_off, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)byte_off, 0, 0, 0);
}
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void wait_all_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// LDS rows are 144 bytes apart (no swizzle): 16 consecutive rows read 128 bits each, or 4
// consecutive rows read 32 bytes each, hit 64 distinct banks, and every address is affine in the row.
typedef int i32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned lds_off(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const void*)p;
}
// Transposing LDS read issued outside the compiler's memory model (see the main loop).
__device__ __forceinline__ void tr_read(i32x2& dst, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(dst) : "v"(addr));
}
template <int OFF> __device__ __forceinline__ void tr_read_imm(i32x2& dst, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int N> __device__ __forceinline__ void wait_lgkm() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
// Orders every later use of `v` after the preceding asm statements (the wait above).
__device__ __forceinline__ void pin(i32x2& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin1(int& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin1f(float& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ bf16x8 join2(i32x2 a, i32x2 b) {
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  i32x4 v = {a[0], a[1], b[0], b[1]};
  return __builtin_bit_cast(bf16x8, v);
}

// Transposing read: this lane supplies the address of (its pixel, its channel quad); it receives
// 4 consecutive pixels of one channel.
__device__ __forceinline__ s16x4 read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}
__device__ __forceinline__ bf16x8 join(s16x4 a, s16x4 b) {
  s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// TPB taps per workgroup.  Waves 0..3 form a 2x2 grid over the channel tile, each owning NA
// co-subtiles x NB ci-subtiles (32 channels each); with NT > 1 further groups of four waves take
// the following taps, so eight or twelve waves share one LDS tile, hold more accumulators and -- what
// matters most -- each hand the memory pipe fewer of the tile's copies.
// A single tap (1x1 windows) with NT = 2: the second group takes the upper half of every tile's pixels
// instead and the two groups add their accumulators through LDS at the end -- what eight waves buy
// there is the copies: each wave hands the memory pipe half as many.
template <int TPB, int NA, int NB, int NT>
__global__ __launch_bounds__(256 * NT) void wgrad_tile_kernel(WgParams p) {
  constexpr int NWAVES = 4 * NT;
  constexpr int TH = (TPB + NT - 1) / NT;    // taps per wave
  constexpr bool KSPLIT = TPB == 1 && NT == 2;   // one tap, two wave groups: they split the tile's pixels
  constexpr int KS = KSPLIT ? TP / 32 : TP / 16;  // 16-pixel steps per wave and tile
  constexpr int CO_T = 64 * NA, CI_T = 64 * NB;
  constexpr int NZS = NA, NXS = NB;          // 64-channel LDS sub-tiles of dZ / of the window
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int bx = blockIdx.x;
  const int tg = bx % p.ntg; bx /= p.ntg;
  const int cit = bx % p.nci;
  const int cot = bx / p.nci;
  const int split = blockIdx.y;
  const int ci0 = cit * CI_T, co0 = cot * CO_T;
  const int taps = p.kH * p.kW;
  const int HoWo = p.Ho * p.Wo;
  const int tile_beg = split * p.tiles_per_split;
  const int tile_end = min(p.ntiles, tile_beg + p.tiles_per_split);

  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t z_rsrc = make_rsrc(p.dz, p.dz_bytes);

  // layout of one stage
  auto xs_base = [&](int buf, int sub) { return smem + buf * p.buf_bytes + sub * p.halo_sub_bytes; };
  auto zs_base = [&](int buf, int sub) { return smem + buf * p.buf_bytes + NXS * p.halo_sub_bytes + sub * ZTILE; };
  auto pt_base = [&](int buf) {
    return reinterpret_cast<int*>(smem + buf * p.buf_bytes + NXS * p.halo_sub_bytes + NZS * ZTILE);
  };

  // place of this lane in a wave-wide copy: 7 rows x 9 granules (granule 8 = pad), lane 63 = row 7 granule 0
  const int urow = lane == 63 ? 7 : (lane * 57) >> 9;
  const int ugran = lane == 63 ? 0 : lane - urow * 9;

  // Placement of a pixel tile: its pixel range and the window rows it touches (wave-uniform).
  constexpr int ZQ = ((TP + 6) / 7 + NWAVES - 1) / NWAVES;   // dZ copy slots per wave (19 copies in all)
  struct TileGeo { int m0, m_end, v_first, npix, hunits, nq; };
  auto tile_geo = [&](int tile) {
    TileGeo t;
    t.m0 = tile * TP;
    t.m_end = min(p.M, tile * TP + TP);
    if (p.tpi > 0) {
      const int n = tile / p.tpi;
      t.m0 = n * HoWo + (tile - n * p.tpi) * TP;
      t.m_end = min(t.m0 + TP, (n + 1) * HoWo);
    }
    const int m_last = t.m_end - 1;
    const int n_a = fdiv(t.m0, p.dHoWo), ho_a = fdiv(t.m0 - n_a * HoWo, p.dWo);
    const int n_b = fdiv(m_last, p.dHoWo), ho_b = fdiv(m_last - n_b * HoWo, p.dWo);
    t.v_first = n_a * p.Hv + ho_a * p.sh;
    const int nslots = n_b * p.Hv + ho_b * p.sh + p.kH - t.v_first;
    t.npix = nslots * p.Wv;
    t.hunits = (t.npix + 6) / 7;
    t.nq = ZQ + (t.hunits + NWAVES - 1) / NWAVES;   // copy slots per wave: dZ rows, then window rows
    return t;
  };
  // Copy slots [q_beg, q_end) of this wave for tile `t` into stage `buf`; slot 0 also writes the
  // pixel table.  Slots 0..ZQ-1 are dZ rows (copy u = wave + NWAVES q of 19, all sub-tiles), slot
  // ZQ + j is window copy u = wave + NWAVES j.
  auto issue_slots = [&](const TileGeo& t, int buf, int q_beg, int q_end) {
    for (int q = q_beg; q < q_end; ++q) {
      if (q < ZQ) {
        const int u = wave + NWAVES * q;
        const int row = u * 7 + urow;
        if (u < (TP + 6) / 7) {
#pragma unroll
          for (int sub = 0; sub < NZS; ++sub) {
            const int ch = co0 + sub * 64 + (ugran << 3);
            unsigned off = (unsigned)(((t.m0 + row) * p.Co + ch) * 2);
            if (row >= TP || t.m0 + row >= t.m_end || ugran == 8 || ch >= p.Co) off = OOB;
            dma16(z_rsrc, off, zs_base(buf, sub) + u * UNITB);
          }
        }
      } else {
        const int u = wave + NWAVES * (q - ZQ);
        if (u < t.hunits) {
          const int pix = u * 7 + urow;
          const int slot = fdiv(pix, p.dWv);
          const int w = pix - slot * p.Wv - p.pw;
          const int v = t.v_first + slot;
          const int n = fdiv(v, p.dHv);
          const int h = v - n * p.Hv - p.ph;
          const bool ok = pix < t.npix && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W && n < p.N;
          const int base = n * p.x_n_stride + h * p.x_h_stride + w * p.x_w_stride;
#pragma unroll
          for (int sub = 0; sub < NXS; ++sub) {
            const int ch = ci0 + sub * 64 + (ugran << 3);
            unsigned off = (unsigned)((base + ch) * 2);
            if (!ok || ugran == 8 || ch >= p.Cin) off = OOB;
            dma16(x_rsrc, off, xs_base(buf, sub) + u * UNITB);
          }
        }
      }
    }
    if (q_beg == 0 && tid < TP) {
      // pixel table: window-tile row of tap (0,0) for each of the 128 output pixels
      const int m = t.m0 + tid;
      int idx = 0;
      if (m < t.m_end) {
        const int n = fdiv(m, p.dHoWo);
        const int rem = m - n * HoWo;
        const int ho = fdiv(rem, p.dWo);
        const int wo = rem - ho * p.Wo;
        idx = (n * p.Hv + ho * p.sh - t.v_first) * p.Wv + wo * p.sw;
      }
      pt_base(buf)[tid] = idx;
    }
  };

  // taps of this group, as pixel offsets into the window tile
  const int th = wave >> 2;                    // which half of the tap group (or of the pixels) this wave multiplies
  const int kbeg = KSPLIT ? th * KS : 0;       // its first 16-pixel step of a tile
  int tapno[TH], tapoff[TH];
#pragma unroll
  for (int t = 0; t < TH; ++t) {
    const int tl = KSPLIT ? t : th * TH + t;   // tap inside the group
    const int tap = tg * TPB + tl;
    const int i = fdiv(tap, p.dkW);
    const bool live = tl < TPB && tap < taps;
    tapno[t] = live ? tap : -1;                // surplus taps recompute tap 0 and are never stored
    tapoff[t] = live ? (i * p.Wv + (tap - i * p.kW)) * ROWB : 0;
  }

  // wave -> subtiles: ci across wave&1, co across (wave>>1)&1
  const int wci = (wave & 1) * NB, wco = ((wave >> 1) & 1) * NA;   // first 32-channel subtile index
  const int kb = lane >> 5;
  const int eprime = (lane & 15) >> 2;         // pixel (of 4) this lane addresses in a transposing read
  const int chq = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;   // channel quad inside the 32-channel subtile

  f32x16 acc[TH][NB][NA];
#pragma unroll
  for (int t = 0; t < TH; ++t)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][b][a][e] = 0.f;

  const bool do_r = (cit == 0 && tg == 0 && p.r_part != nullptr);
  float racc[NZS][8];
#pragma unroll
  for (int s = 0; s < NZS; ++s)
#pragma unroll
    for (int e = 0; e < 8; ++e) racc[s][e] = 0.f;

  // Operand fragments of one 16-pixel step, split in two groups so that one group is always in
  // flight while the other is multiplied (the LDS counter holds at most 15 outstanding reads):
  //   group 0: the dZ fragments and the first H0 window fragments, group 1: the rest.
  // The transposing reads are issued as inline asm (the compiler would otherwise fence every
  // LDS read against the in-flight global->LDS copies of the NEXT tile) and are ordered against
  // their MFMAs by explicit lgkmcnt waits plus register dependences.
  constexpr int NF = TH * NB;                   // window fragments per step (tap-major)
  constexpr int H0 = (NF + 1) / 2;
  constexpr int N0 = 2 * (NA + H0), N1 = 2 * (NF - H0);
  static_assert(N0 <= 15 && N1 <= 15, "groups must fit the LDS counter");
  i32x2 fz[2][NA][2];
  i32x2 fx[2][NF][2];

  if (tile_beg < tile_end) {
    const TileGeo t0 = tile_geo(tile_beg);
    issue_slots(t0, 0, 0, t0.nq);
  }
  for (int tile = tile_beg; tile < tile_end; ++tile) {
    const int buf = (tile - tile_beg) & 1;
    wait_all_copies();
    __syncthreads();   // tile landed for every wave, pixel table visible, previous tile's reads done

    // byte offset of this lane's window-tile rows (tap (0,0)) for its two pixels of every step,
    // read before the next copies start
    int ptv[KS][2];
    {
      const int* ptab = pt_base(buf);
#pragma unroll
      for (int k = 0; k < KS; ++k) {
        ptv[k][0] = ptab[(kbeg + k) * 16 + kb * 8 + eprime] * ROWB;
        ptv[k][1] = ptab[(kbeg + k) * 16 + kb * 8 + eprime + 4] * ROWB;
      }
    }
    if (do_r && tid < 256) {
      // column sums of the dZ tile: thread -> granule tid%8, pixels tid/8 + 32 j
#pragma unroll
      for (int s2 = 0; s2 < NZS; ++s2)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int px = (tid >> 3) + 32 * j;
          const uint4 v = *reinterpret_cast<const uint4*>(zs_base(buf, s2) + px * ROWB + ((tid & 7) << 4));
          racc[s2][0] += bf16_lo(v.x); racc[s2][1] += bf16_hi(v.x);
          racc[s2][2] += bf16_lo(v.y); racc[s2][3] += bf16_hi(v.y);
          racc[s2][4] += bf16_lo(v.z); racc[s2][5] += bf16_hi(v.z);
          racc[s2][6] += bf16_lo(v.w); racc[s2][7] += bf16_hi(v.w);
        }
    }
    // settle every compiler-tracked LDS read here, so that no compiler-inserted wait lands inside
    // the hand-counted pipeline below
#pragma unroll
    for (int k = 0; k < KS; ++k) { pin1(ptv[k][0]); pin1(ptv[k][1]); }
#pragma unroll
    for (int s2 = 0; s2 < NZS; ++s2)
#pragma unroll
      for (int e = 0; e < 8; ++e) pin1f(racc[s2][e]);
    // next tile's copies: issued in one go (issuing them in slices between the MFMA groups was
    // measured slower: the copies are bandwidth-limited and block at issue either way)
    if (tile + 1 < tile_end) {
      const TileGeo tn = tile_geo(tile + 1);
      issue_slots(tn, buf ^ 1, 0, tn.nq);
    }

    // lane-constant parts of the operand addresses
    const unsigned zlane = lds_off(zs_base(buf, 0)) + (kbeg * 16 + kb * 8 + eprime) * ROWB + chq * 2;
    const unsigned xlane = lds_off(xs_base(buf, 0)) + chq * 2;

    auto issue_g0 = [&](int k, int set) {
#pragma unroll
      for (int a2 = 0; a2 < NA; ++a2) {
        const int sub = (wco + a2) >> 1;
#pragma unroll
        for (int h = 0; h < 2; ++h)
          tr_read(fz[set][a2][h], zlane + sub * ZTILE + ((wco + a2) & 1) * 64 + (k * 16 + 4 * h) * ROWB);
      }
#pragma unroll
      for (int f = 0; f < H0; ++f) {
        const int t = f / NB, b2 = f % NB;
        const int sub = (wci + b2) >> 1;
#pragma unroll
        for (int h = 0; h < 2; ++h)
          tr_read(fx[set][f][h], xlane + ptv[k][h] + (tapoff[t] + sub * p.halo_sub_bytes + ((wci + b2) & 1) * 64));
      }
    };
    auto issue_g1 = [&](int k, int set) {
#pragma unroll
      for (int f = H0; f < NF; ++f) {
        const int t = f / NB, b2 = f % NB;
        const int sub = (wci + b2) >> 1;
#pragma unroll
        for (int h = 0; h < 2; ++h)
          tr_read(fx[set][f][h], xlane + ptv[k][h] + (tapoff[t] + sub * p.halo_sub_bytes + ((wci + b2) & 1) * 64));
      }
    };
    auto mma = [&](int set, int f_beg, int f_end) {
#pragma unroll
      for (int a2 = 0; a2 < NA; ++a2) { pin(fz[set][a2][0]); pin(fz[set][a2][1]); }
#pragma unroll
      for (int f = f_beg; f < f_end; ++f) {
        pin(fx[set][f][0]); pin(fx[set][f][1]);
        const int t = f / NB, b2 = f % NB;
        const bf16x8 xf = join2(fx[set][f][0], fx[set][f][1]);
#pragma unroll
        for (int a2 = 0; a2 < NA; ++a2)
          acc[t][b2][a2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, join2(fz[set][a2][0], fz[set][a2][1]),
                                                                 acc[t][b2][a2], 0, 0, 0);
      }
    };

    issue_g0(0, 0);
    issue_g1(0, 0);
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      const int set = k & 1;
      wait_lgkm<N1>();                       // group 0 of step k is in (the youngest N1 reads are group 1)
      mma(set, 0, H0);
      if (k + 1 < KS) { issue_g0(k + 1, set ^ 1); wait_lgkm<N0>(); }
      else wait_lgkm<0>();                   // group 1 of step k is in
      mma(set, H0, NF);
      if (k + 1 < KS) issue_g1(k + 1, set ^ 1);
    }
  }

  if (KSPLIT) {
    // the upper-half group hands its sums to the lower-half group through LDS (stage 0 is free now)
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem) + (wave & 3) * (NA * NB * 16 * 64) + lane;
    if (th == 1) {
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int e = 0; e < 16; ++e) red[((b * NA + a) * 16 + e) * 64] = acc[0][b][a][e];
    }
    __syncthreads();
    if (th == 0) {
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[0][b][a][e] += red[((b * NA + a) * 16 + e) * 64];
    }
  }
  // ---- epilogue: partial dw' ------------------------------------------------------------------
  // accumulator element e of lane l: ci row 8*(e/4) + 4*(l/32) + e%4, co column l%32
#pragma unroll
  for (int t = 0; t < TH; ++t) {
    const int tap = tapno[t];
    if (tap < 0 || (KSPLIT && th != 0)) continue;
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      const int co = co0 + (wco + a) * 32 + (lane & 31);
      if (co >= p.Co) continue;
      float* orow = p.part + (((size_t)split * p.Co + co) * taps + tap) * p.Cin;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ci = ci0 + (wci + b) * 32 + q * 8 + kb * 4;
          if (ci >= p.Cin) continue;
          *reinterpret_cast<float4*>(orow + ci) = make_float4(acc[t][b][a][q * 4 + 0], acc[t][b][a][q * 4 + 1],
                                                              acc[t][b][a][q * 4 + 2], acc[t][b][a][q * 4 + 3]);
        }
    }
  }
  if (do_r) {
    __syncthreads();   // all waves are done with the stages: reuse stage 0 as reduction scratch
    float* red = reinterpret_cast<float*>(smem);   // [32 pixel lanes][64 NZS channels]
#pragma unroll
    for (int s = 0; s < NZS; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (tid < 256) red[(tid >> 3) * (64 * NZS) + s * 64 + (tid & 7) * 8 + e] = racc[s][e];
    __syncthreads();
    for (int c = tid; c < 64 * NZS; c += 256 * NT) {
      float v = 0.f;
      for (int l = 0; l < 32; ++l) v += red[l * (64 * NZS) + c];
      if (co0 + c < p.Co) p.r_part[(size_t)split * p.Co + co0 + c] = v;
    }
  }
}

constexpr size_t LDS_USABLE = 159 * 1024;

int max_slots(const WgParams& p) {
  const int HoWo = p.Ho * p.Wo;
  int best = 0;
  if (p.tpi > 0) {   // the same tile pattern in every image
    for (int j = 0; j < p.tpi; ++j) {
      const int a = j * TP, b = (a + TP < HoWo ? a + TP : HoWo) - 1;
      const int ns = (b / p.Wo) * p.sh + p.kH - (a / p.Wo) * p.sh;
      if (ns > best) best = ns;
    }
    return best;
  }
  int a = HoWo, b = TP;
  while (b) { const int t = a % b; a = b; b = t; }
  const int period = HoWo / a;
  for (int m0 = 0, t = 0; m0 < p.M && t <= period; m0 += TP, ++t) {
    const int ml = (m0 + TP < p.M ? m0 + TP : p.M) - 1;
    const int na = m0 / HoWo, hoa = (m0 - na * HoWo) / p.Wo;
    const int nb = ml / HoWo, hob = (ml - nb * HoWo) / p.Wo;
    const int ns = nb * p.Hv + hob * p.sh + p.kH - (na * p.Hv + hoa * p.sh);
    if (ns > best) best = ns;
  }
  return best;
}

struct WgPlan { bool ok; int tpb, na, nb, nt, nsplit; size_t lds; };

bool base_params(const Geom& g_in, WgParams* p) {
  WgParams& q = *p;
  q = WgParams{};
  // A 1x1 / stride-1 / unpadded layer is a product over pixels, whatever the image shape: presented as images of one
  // row of TP pixels, a tile's window rows are exactly its own pixels (as rows of a 56-wide image a 128-pixel tile
  // would fetch four of them, 224 pixels).
  Geom g = g_in;
  if (g.kH == 1 && g.kW == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 && g.M % TP == 0) {
    g.N = g.M / TP; g.Hin = g.Hout = 1; g.Win = g.Wout = TP;
  }
  q.N = g.N; q.Cin = g.Cin; q.Ho = g.Hout; q.Wo = g.Wout; q.Co = g.Cout; q.M = g.M;
  q.kH = g.kH; q.kW = g.kW;
  if (g.kH == 1 && g.kW == 1 && g.ph == 0 && g.pw == 0) {
    q.H = g.Hout; q.W = g.Wout; q.sh = 1; q.sw = 1; q.ph = 0; q.pw = 0;
    q.x_h_stride = g.sh * g.Win * g.Cin;
    q.x_w_stride = g.sw * g.Cin;
  } else {
    q.H = g.Hin; q.W = g.Win; q.sh = g.sh; q.sw = g.sw; q.ph = g.ph; q.pw = g.pw;
    q.x_h_stride = g.Win * g.Cin;
    q.x_w_stride = g.Cin;
  }
  q.x_n_stride = g.Hin * g.Win * g.Cin;
  const size_t xb = (size_t)g.N * g.Hin * g.Win * g.Cin * 2, zb = (size_t)g.M * g.Cout * 2;
  if (xb >= OOB || zb >= OOB) return false;
  q.x_bytes = (unsigned)xb;
  q.dz_bytes = (unsigned)zb;
  q.Hv = (q.Ho - 1) * q.sh + q.kH;
  q.Wv = (q.Wo - 1) * q.sw + q.kW;
  q.dHoWo = make_fastdiv(q.Ho * q.Wo);
  q.dWo = make_fastdiv(q.Wo);
  q.dHv = make_fastdiv(q.Hv);
  q.dWv = make_fastdiv(q.Wv);
  q.dkW = make_fastdiv(q.kW);
  // images of at least two tiles get their own tiles (fewer window rows per tile at image borders)
  q.tpi = q.Ho * q.Wo >= 2 * TP ? ceil_div(q.Ho * q.Wo, TP) : 0;
  q.ntiles = q.tpi > 0 ? q.N * q.tpi : ceil_div(q.M, TP);
  return true;
}

WgPlan make_plan(const Geom& g, WgParams* pp) {
  WgPlan pl{false, 0, 0, 0, 1, 0, 0};
  if (g.Cin % 8 || g.Cout % 8) return pl;
  WgParams& p = *pp;
  if (!base_params(g, &p)) return pl;
  const int taps = g.kH * g.kW;
  // accumulator shape by window size and channel counts
  if (taps == 1) { pl.tpb = 1; pl.na = g.Cout > 64 ? 2 : 1; pl.nb = g.Cin > 64 ? 2 : 1; pl.nt = 2; }   // eight waves: two pixel halves
  else if (taps <= 3) { pl.tpb = 3; pl.na = g.Cout > 64 ? 2 : 1; pl.nb = 1; pl.nt = 1; }
  else { pl.tpb = 9; pl.na = g.Cout > 64 ? 2 : 1; pl.nb = 1; pl.nt = 3; }   // twelve waves: 3 + 3 + 3 taps
  // every pixel split writes a full fp32 copy of dw': keep that traffic near the size of the inputs
  const size_t copy_bytes = (size_t)g.Cout * g.K * 4;
  const size_t in_bytes = ((size_t)g.M * g.Cout + (size_t)g.N * g.Hin * g.Win * g.Cin) * 2;
  const int cap = (int)((3 * in_bytes + 24 * 1024 * 1024) / copy_bytes);
  // 128 output channels per workgroup only if the splits that cap allows still fill the chip
  if (pl.na == 2 && (long long)ceil_div(g.Cin, 64 * pl.nb) * ceil_div(g.Cout, 128) * ceil_div(taps, pl.tpb) *
                            (cap < 1 ? 1 : cap) < 256)
    pl.na = 1;
  const int slots = max_slots(p);
  const int hunits = ceil_div(slots * p.Wv, 7);
  p.halo_sub_bytes = (int)align_up((size_t)hunits * UNITB + 16, 1024);
  // shrink the channel tile until two stages fit the LDS
  for (;;) {
    p.buf_bytes = pl.nb * p.halo_sub_bytes + pl.na * ZTILE + 1024;
    pl.lds = 2 * (size_t)p.buf_bytes;
    if (pl.lds <= LDS_USABLE) break;
    if (pl.nb > 1) pl.nb = 1;
    else if (pl.na > 1) pl.na = 1;
    else return pl;
  }
  p.nci = ceil_div(g.Cin, 64 * pl.nb);
  p.ntg = ceil_div(taps, pl.tpb);
  p.nco = ceil_div(g.Cout, 64 * pl.na);
  // pixel splits: about one workgroup per CU (a workgroup fills a CU's LDS), at least 2 tiles each
  const int base_blocks = p.nci * p.nco * p.ntg;
  int want = 256 / base_blocks;
  if (want > cap) want = cap;
  const int max_split = ceil_div(p.ntiles, 2);
  if (want > max_split) want = max_split;
  if (want < 1) want = 1;
  p.tiles_per_split = ceil_div(p.ntiles, want);
  pl.nsplit = ceil_div(p.ntiles, p.tiles_per_split);
  pl.ok = true;
  return pl;
}

template <int TPB, int NA, int NB, int NT>
hipError_t launch_inst(const WgParams& p, const WgPlan& pl, hipStream_t st) {
  static LdsLimitOnce lds_once;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&wgrad_tile_kernel<TPB, NA, NB, NT>),
                                        (int)LDS_USABLE); e != hipSuccess) return e;
  hipLaunchKernelGGL((wgrad_tile_kernel<TPB, NA, NB, NT>), dim3(p.nci * p.nco * p.ntg, pl.nsplit), dim3(256 * NT), pl.lds,
                     st, p);
  return hipGetLastError();
}

}  // namespace

bool wgrad_tile_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  WgParams p;
  return make_plan(g, &p).ok;
}

int wgrad_tile_splits(const Geom& g) {
  WgParams p;
  return make_plan(g, &p).nsplit;
}

hipError_t launch_wgrad_tile(const Geom& g, const void* x, const void* dz, float* dwf_part, float* r_part,
                             hipStream_t st) {
  WgParams p;
  const WgPlan pl = make_plan(g, &p);
  p.x = (const bf16_t*)x; p.dz = (const bf16_t*)dz; p.part = dwf_part; p.r_part = r_part;
#define CASE(T, A, B, W) \
  if (pl.tpb == T && pl.na == A && pl.nb == B && pl.nt == W) return launch_inst<T, A, B, W>(p, pl, st);
  CASE(9, 1, 1, 3) CASE(9, 2, 1, 3) CASE(3, 1, 1, 1) CASE(3, 2, 1, 1)
  CASE(1, 2, 2, 2) CASE(1, 1, 2, 2) CASE(1, 2, 1, 2) CASE(1, 1, 1, 2)
#undef CASE
  return hipErrorInvalidValue;
}

}  // namespace convbn
