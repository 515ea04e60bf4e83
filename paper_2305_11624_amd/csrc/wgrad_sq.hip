// bf16 MFMA weight gradient of a 3x3 window, one 32 x 32 channel pair per workgroup with all nine taps:
//   dw'[co][tap][ci] = sum_m dZ[m][co] * Xpad[m (+) tap][ci]      (Sec. 3.2.1: dJ/dw = dJ/dY (.) X)
//   r[co]            = sum_m dZ[m][co]                            (App. B)
//
// Why this shape.  Every workgroup that shares the chip adds one fp32 copy of its outputs to what the
// fold-back has to read again, so the copies must be small: a workgroup owns 32 output x 32 input channels
// x 9 taps = 9216 outputs (36 KB).  Deep layers (512 x 512 channels: 256 channel pairs) then need no pixel
// split at all -- one copy of dw', written once -- and wide-image layers (64 x 64 channels: 4 pairs) split
// the pixels 60-fold for 9 MB of copies where 64 x 64 x 9 tiles wrote 30.  The nine taps share one window
// tile of X in LDS, so a workgroup fetches a pixel of X once, not nine times; what a compute unit pulls from
// the L2 stays near 25 bytes per clock.
//
// A workgroup walks its pixels in tiles of 128 KS.  Per tile the dZ rows and the window rows of X those
// pixels touch are copied global -> LDS in their natural [pixel][32 channels] order (64-byte rows, 1 KB per
// copy instruction, zero fill outside the tensors through an out-of-range buffer offset), double-buffered.
// The reduced index is the pixel -- the strided direction of that layout -- so the MFMA operands are read
// with the transposing LDS load (ds_read_b64_tr_b16: a 16-lane group turns 4 pixels x 16 channels into
// "lane = channel, 4 pixels"); four consecutive 64-byte rows are 256 contiguous bytes, one access per bank.
// The eight waves split each tile's pixels (16 KS each), every wave holds all nine accumulator tiles, and
// the waves add their sums through LDS at the end.
#include "common.h"
#include "conv_rw_impl.h"   // the input gradient that can share a launch with this kernel

#include <atomic>
#include <chrono>
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

constexpr int NWAVES = 8;
constexpr int TAPS = 9;
constexpr int MAXXU = 6;                 // window copies per wave and tile, at most
constexpr int ROWB = 64;                 // LDS row: 32 channels of bf16, no padding
constexpr int RED_BYTES = 4 * TAPS * 16 * 64 * 4;   // four waves' accumulators (147456): the final reduction
constexpr unsigned OOB = 0x80000000u;
constexpr size_t LDS_USABLE = 159 * 1024;

struct SqParams {
  const bf16_t* x;
  const bf16_t* dz;
  float* part;       // [nsplit][Co][taps][Cin]
  float* r_part;     // [nsplit][Co] or null
  // Fused fold-back (Table 2 "Tune", last four lines), one pixel split only: dW = s dw' is stored instead of the
  // fp32 copy, the workgroups of an output-channel tile leave their partial <dw', w> (and r) in tagged slots
  // [nci + 1][Co]; the one that finds all of them in place finishes dgamma, dbeta, db for the tile's 32 channels.
  const bf16_t* wgt;   // the unfolded weight; null: not fused
  bf16_t* dW;
  bf16_t* w_t;         // optional: w' = s w is left here as [Cin][taps][Cout], for the input gradient that follows
  const float* gamma; const float* mean; const float* var; const float* b;
  float* db; float* dgamma; float* dbeta;
  uint4* slots;              // {value, tag low, tag high, 0}
  unsigned long long tag;    // of this launch, never 0
  float eps;
  unsigned x_bytes, dz_bytes;
  int N, H, W, Cin;
  int x_n_stride, x_h_stride, x_w_stride;
  int Ho, Wo, Co;
  int kW, sh, sw, ph, pw;
  int M, Hv, Wv;
  int nci, nco;
  int bc, bi, nbci, blocks_per_split, nblocks;   // workgroup -> (channel pair, split) mapping, see the kernel
  int ntiles, tiles_per_split;
  int hunits;         // 1 KB units of a stage's window tile
  int stage_bytes;    // dZ tile + window tile
  // A tile is TILE consecutive output pixels = step_n images + step_h rows + step_w pixels; what that step adds to a
  // pixel's byte offset among the window rows of the whole tensor, and what the carries out of the column and the row add
  int step_h, step_w, step_off, carry_w_off, carry_h_off;
  int max_pixel_off;  // largest offset (inside a stage's window tile) a pixel of the tile can have
  FastDiv dHoWo, dWo, dHv, dWv;
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef int i32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
// 1 KB copy: lane l fetches 16 bytes at byte offset voff (per lane) + soff (wave-uniform; not part of the range
// check) and writes them to LDS at lds_wave_base + 16 l.  The compiler barrier keeps every copy in the stream:
// the waits count copies.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, void* lds_wave_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)lds_wave_base, 16, (int)voff, (int)soff, 0, 0);
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void wait_all_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ unsigned lds_off(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const void*)p;
}
// Transposing LDS reads issued as inline asm with hand-counted waits: the compiler would otherwise hold
// every LDS read until the global -> LDS copies of the NEXT tile have landed.
__device__ __forceinline__ void tr_read(i32x2& dst, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(dst) : "v"(addr));
}
// ... at a compile-time byte offset from the address (the instruction's offset field): the taps of a kernel row and
// the 16-pixel steps of a tile cost no address arithmetic
template <int OFF> __device__ __forceinline__ void tr_read_at(i32x2& dst, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int N> __device__ __forceinline__ void wait_lgkm() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void pin(i32x2& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin1(int& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void pin1f(float& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ bf16x8 join2(i32x2 a, i32x2 b) {
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  i32x4 v = {a[0], a[1], b[0], b[1]};
  return __builtin_bit_cast(bf16x8, v);
}

// Values that cross workgroups (which may run on XCDs whose L2 caches are not coherent with each other) are
// written through to memory and read past any stale line with device-scope accesses.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_device_scope16(uint4* p, uint4 v) {
  const u32x4 r = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(r) : "memory");
}
__device__ __forceinline__ uint4 load_device_scope16(const uint4* p) {
  u32x4 r;
  asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(r) : "v"(p) : "memory");
  return make_uint4(r.x, r.y, r.z, r.w);
}
// A slot of the exchange between workgroups: a value and the tag of the launch that wrote it, in one store.
__device__ __forceinline__ void store_slot(uint4* p, float v, unsigned long long tag) {
  store_device_scope16(p, make_uint4(__float_as_uint(v), (unsigned)tag, (unsigned)(tag >> 32), 0u));
}

// Number of transposing reads issued up to and including those of multiply slot s (slot = 9 k + tap): two per
// slot, plus two for the dZ fragment of every 16-pixel step begun so far.
constexpr int reads_through(int s) { return 2 * (s + 1) + 2 * (s / TAPS + 1); }

#ifdef SQ_TRACE
__device__ unsigned long long sq_trace[512 * 64];
#ifndef SQ_TRACE_WAVE
#define SQ_TRACE_WAVE 0
#endif
#define STAMP(i) do { if (tid == 64 * SQ_TRACE_WAVE && (i) < 64) sq_trace[block * 64 + (i)] = clock64(); } while (0)
#else
#define STAMP(i) do {} while (0)
#endif

// KS: 16-pixel steps per wave and tile (tile = 128 KS pixels).  NCPY: copies per wave and tile (KS dZ units + the
// window units wave, wave + 8, ...; units past a tile's window rows are zero-fill copies, so the count is fixed).
// The work of workgroup `block`; smem: the workgroup's LDS.
template <int KS, int NCPY>
__device__ __forceinline__ void sq_body(const SqParams& p, int block, unsigned char* smem) {
  constexpr int TILE = 128 * KS;
  constexpr int ZT = TILE * ROWB;          // dZ tile bytes
  constexpr int NS = TAPS * KS;            // multiplies per wave and tile
  constexpr int NXU = NCPY - KS;           // window units per wave
  constexpr int AHEAD = 4;                 // operands are read this many multiplies ahead
  constexpr int NSTAGE = 3;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  STAMP(0);
  // Workgroup -> work.  Workgroups are handed to the eight XCDs in turn (id % 8), and each XCD has its own L2:
  // the workgroups of one XCD should read the same slices of X and dZ.  The work is cut into blocks of bc x bi
  // channel pairs of one pixel split (pairs that share dZ slices along one side and X slices along the other);
  // block j goes to XCD j % 8, whose k-th workgroup (k = id / 8) takes pair k % (bc bi) of its (k / (bc bi))-th block.
  const int bsize = p.bc * p.bi;
  const int k_x = block >> 3;
  const int blk = (k_x / bsize) * 8 + (block & 7);
  if (blk >= p.nblocks) return;
  const int w_b = k_x % bsize;
  const int split = blk / p.blocks_per_split;
  const int jb = blk - split * p.blocks_per_split;
  const int cot = (jb / p.nbci) * p.bc + w_b % p.bc;
  const int cit = (jb % p.nbci) * p.bi + w_b / p.bc;
  const int ci0 = cit * 32, co0 = cot * 32;
  const int HoWo = p.Ho * p.Wo;
  const int tile_beg = split * p.tiles_per_split;
  const int tile_end = min(p.ntiles, tile_beg + p.tiles_per_split);

  const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.x, p.x_bytes);
  const __amdgpu_buffer_rsrc_t z_rsrc = make_rsrc(p.dz, p.dz_bytes);

  // place of this lane in a 1 KB copy: 16 rows x 4 granules
  const int urow = lane >> 2, ugran = lane & 3;
  // Everything a copy or an operand read needs per lane is kept as running state that a step to the next tile
  // updates with additions, compares and selects: the loop is bound by the instructions a wave issues between
  // its multiplies, and a division or a 32-bit multiply per address costs several multiplies' worth of issue slots.
  //
  // dZ copies: per-lane byte offset inside a tile; the tile's first row is added per copy (the range check of the
  // copy covers only the per-lane offset: rows past the last pixel then lie past the buffer and arrive as zeros)
  unsigned zoff[KS];
#pragma unroll
  for (int j = 0; j < KS; ++j) zoff[j] = (unsigned)((((wave + NWAVES * j) * 16 + urow) * p.Co + co0 + ugran * 8) * 2);
  const unsigned ztile_bytes = (unsigned)(TILE * 2) * (unsigned)p.Co;
  // first window row of a tile (wave-uniform)
  auto tile_vfirst = [&](int tile) {
    const int m0 = tile * TILE;
    const int n_a = fdiv(m0, p.dHoWo);
    return n_a * p.Hv + fdiv(m0 - n_a * HoWo, p.dWo) * p.sh;
  };
  // window copies: unit u = wave + 8 j covers window pixels 16 u .. of the tile; this lane's pixel is column w of
  // window row vfirst + slot.  State: the row's place hv inside its image's Hv window rows and the byte offset xo
  // of the lane's 16 bytes (meaningless while the row is padding).  A step of dv = dn Hv + dh window rows adds
  // xstep = dn (image) + dh (row) bytes, and one image less Hv rows where hv wraps.
  const int ns_b = p.x_n_stride * 2, hs_b = p.x_h_stride * 2;
  const int wrap_b = ns_b - p.Hv * hs_b;
  int xhv[NXU];
  unsigned xo[NXU];
  bool xcol_ok[NXU];
  const int vf_beg = tile_vfirst(tile_beg);
#pragma unroll
  for (int j = 0; j < NXU; ++j) {
    const int pix = (wave + NWAVES * j) * 16 + urow;
    const int slot = fdiv(pix, p.dWv);
    const int w = pix - slot * p.Wv - p.pw;
    xcol_ok[j] = (unsigned)w < (unsigned)p.W;
    const int v = vf_beg + slot;
    const int n = fdiv(v, p.dHv);
    xhv[j] = v - n * p.Hv;
    xo[j] = (unsigned)(n * ns_b + (xhv[j] - p.ph) * hs_b + (w * p.x_w_stride + ci0 + ugran * 8) * 2);
  }
  // the stage holds exactly p.hunits window units: the waves whose last unit lies past them issue one copy less
  const bool has_last = wave + NWAVES * (NXU - 1) < p.hunits;
  // the step from one tile's first window row to the next one's, split on the scalar unit
  int x_dh = 0, x_step = 0;
  auto set_step = [&](int dv) {
    const int dn = fdiv(dv, p.dHv);
    x_dh = dv - dn * p.Hv;
    x_step = dn * ns_b + x_dh * hs_b;
  };
  auto advance_window = [&](int j) {
    int hv = xhv[j] + x_dh;
    const bool wr = hv >= p.Hv;
    xhv[j] = wr ? hv - p.Hv : hv;
    xo[j] += (unsigned)(x_step + (wr ? wrap_b : 0));
  };
  // Copy i of a tile into `stage` (a zero-fill copy if the tile does not exist: the count stays fixed).  ztile: byte
  // offset of the tile's first dZ row, past any buffer for a tile that does not exist.  The window state must have
  // been advanced to the tile.
  auto issue_copy = [&](int i, unsigned ztile, bool live, unsigned char* stage) {
    if (i < KS) {
      const int ii = i < KS ? i : 0;
      dma16(z_rsrc, zoff[ii] + ztile, 0u, stage + (wave + NWAVES * ii) * 1024);
    } else {
      const int j = i - KS < NXU ? i - KS : 0;
      if (j == NXU - 1 && !has_last) return;   // wave-uniform: this wave's last unit lies past the window tile
      const bool ok = live && xcol_ok[j] && (unsigned)(xhv[j] - p.ph) < (unsigned)p.H;   // rows past the last image lie past the buffer
      dma16(x_rsrc, ok ? xo[j] : OOB, 0u, stage + ZT + (wave + NWAVES * j) * 1024);
    }
  };

  // Operand reads.  Output pixel m = (n, ho, wo) reads window row n Hv + ho sh, column wo sw (+ tap): state per
  // pixel this lane addresses (two per 16-pixel step) is (wo, ho) and the byte offset pg of that place among the
  // window rows of the whole tensor; inside a tile's window tile the offset is pg - (first window row) Wv ROWB.
  const int kb = lane >> 5;
  const int eprime = (lane & 15) >> 2;                        // pixel (of 4) this lane addresses in a transposing read
  const int chq = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;    // channel quad inside the 32 channels
  const int pbase = wave * (16 * KS);                          // this wave's first pixel of a tile
  const int plane = pbase + kb * 8 + eprime;                   // ... and this lane's first pixel of a 16-pixel step
  const int row_b = p.Wv * ROWB;                               // one window row
  int pwo[KS][2], pho[KS][2], pg[KS][2];
#pragma unroll
  for (int k = 0; k < KS; ++k)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int m = tile_beg * TILE + plane + k * 16 + 4 * h;   // (past the last pixel: an image that does not exist)
      const int n = fdiv(m, p.dHoWo);
      const int rem = m - n * HoWo;
      pho[k][h] = fdiv(rem, p.dWo);
      pwo[k][h] = rem - pho[k][h] * p.Wo;
      pg[k][h] = ((n * p.Hv + pho[k][h] * p.sh) * p.Wv + pwo[k][h] * p.sw) * ROWB;
    }
  auto advance_pixel = [&](int k, int h) {
    int wo = pwo[k][h] + p.step_w;
    const bool cw = wo >= p.Wo;
    pwo[k][h] = cw ? wo - p.Wo : wo;
    int ho = pho[k][h] + p.step_h + (cw ? 1 : 0);
    const bool ch = ho >= p.Ho;
    pho[k][h] = ch ? ho - p.Ho : ho;
    pg[k][h] += p.step_off + (cw ? p.carry_w_off : 0) + (ch ? p.carry_h_off : 0);
  };
  // offset inside the window tile of a tile whose first window row is vfirst; pixels past the last one (their dZ
  // rows are zeros) are held inside the tile so that they read numbers, not whatever else the LDS holds
  auto pixel_rel = [&](int k, int h, int vfirst) { return min(pg[k][h] - vfirst * row_b, p.max_pixel_off); };

  f32x16 acc[TAPS];
#pragma unroll
  for (int t = 0; t < TAPS; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  const bool do_r = (cit == 0 && p.r_part != nullptr);
  float racc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) racc[e] = 0.f;

  // ---- prologue: the copies of the first two tiles, the pixel offsets of the first ----------------------------
  int vf_cur = vf_beg, vf_next = 0;
  int ptv[KS][2];
#pragma unroll
  for (int k = 0; k < KS; ++k)
#pragma unroll
    for (int h = 0; h < 2; ++h) ptv[k][h] = pixel_rel(k, h, vf_beg);
  {
    const bool live0 = tile_beg < tile_end;
#pragma unroll
    for (int i = 0; i < NCPY; ++i) issue_copy(i, live0 ? (unsigned)tile_beg * ztile_bytes : OOB, live0, smem);
    const bool live1 = tile_beg + 1 < tile_end;
    vf_next = live1 ? tile_vfirst(tile_beg + 1) : vf_beg;
    set_step(vf_next - vf_beg);
#pragma unroll
    for (int j = 0; j < NXU; ++j) advance_window(j);
#pragma unroll
    for (int i = 0; i < NCPY; ++i) issue_copy(i, live1 ? (unsigned)(tile_beg + 1) * ztile_bytes : OOB, live1, smem + p.stage_bytes);
  }

  const unsigned zlane0 = lds_off(smem) + plane * ROWB + chq * 2;
  const unsigned xlane0 = lds_off(smem) + ZT + chq * 2;
  int stage_off = 0;                        // byte offset of the current tile's stage
  STAMP(1);
  for (int tile = tile_beg; tile < tile_end; ++tile) {
    STAMP(20 + 2 * (tile - tile_beg) < 58 ? 20 + 2 * (tile - tile_beg) : 63);
    // this tile has landed; the next one's copies may be in flight
    if (has_last) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCPY) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NCPY - 1) : "memory");
    STAMP(21 + 2 * (tile - tile_beg) < 59 ? 21 + 2 * (tile - tile_beg) : 63);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();          // ... for every wave; everybody is done with the stage refilled below
    asm volatile("" ::: "memory");
    STAMP(2 + 2 * (tile - tile_beg));
    unsigned char* const zs = smem + stage_off;
    int fill_off = stage_off + 2 * p.stage_bytes;
    if (fill_off >= NSTAGE * p.stage_bytes) fill_off -= NSTAGE * p.stage_bytes;
    unsigned char* const fill = smem + fill_off;
    const int tile_f = tile + 2;
    const bool live_f = tile_f < tile_end;
    const int vf_fill = live_f ? tile_vfirst(tile_f) : vf_next;
    set_step(vf_fill - vf_next);            // the window state stands at tile + 1
    const unsigned ztile_f = live_f ? (unsigned)tile_f * ztile_bytes : OOB;

    if (do_r) {
      // column sums of the dZ tile: thread -> granule tid % 4, pixels tid / 4 + 128 j.  Read through inline asm
      // like the operands: a compiler-visible LDS read would first drain the copies in flight.
      typedef int i32x4 __attribute__((ext_vector_type(4)));
      i32x4 rv[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j)
        asm volatile("ds_read_b128 %0, %1" : "=v"(rv[j]) : "v"(lds_off(zs) + ((tid >> 2) + 128 * j) * ROWB + ((tid & 3) << 4)));
      wait_lgkm<0>();
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        asm volatile("" : "+v"(rv[j]));
        racc[0] += bf16_lo((unsigned)rv[j][0]); racc[1] += bf16_hi((unsigned)rv[j][0]);
        racc[2] += bf16_lo((unsigned)rv[j][1]); racc[3] += bf16_hi((unsigned)rv[j][1]);
        racc[4] += bf16_lo((unsigned)rv[j][2]); racc[5] += bf16_hi((unsigned)rv[j][2]);
        racc[6] += bf16_lo((unsigned)rv[j][3]); racc[7] += bf16_hi((unsigned)rv[j][3]);
      }
    }

    // Read addresses of this tile: one register per (16-pixel step, half, kernel row); the tap's column and the dZ
    // rows of a step are compile-time offsets of the read.
    const unsigned zlane = zlane0 + (unsigned)stage_off;
    const unsigned xlane = xlane0 + (unsigned)stage_off;
    unsigned rb[KS][2][3];
#pragma unroll
    for (int k = 0; k < KS; ++k)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        rb[k][h][0] = xlane + (unsigned)ptv[k][h];
        rb[k][h][1] = rb[k][h][0] + (unsigned)row_b;
        rb[k][h][2] = rb[k][h][1] + (unsigned)row_b;
      }
    // Operands are read AHEAD multiplies before their multiply: fx ring slot s % (AHEAD + 1); the dZ fragment of a
    // 16-pixel step goes just before the window fragment of its first tap.
    i32x2 fz[2][2];
    i32x2 fx[AHEAD + 1][2];
    int pnext[KS][2];
    auto read_z = [&](i32x2& dst, int k, int h) {
      switch (k * 2 + h) {
        case 0: tr_read_at<0>(dst, zlane); break;
        case 1: tr_read_at<4 * ROWB>(dst, zlane); break;
        case 2: tr_read_at<16 * ROWB>(dst, zlane); break;
        default: tr_read_at<20 * ROWB>(dst, zlane); break;
      }
    };
    auto read_x = [&](i32x2& dst, unsigned base, int col) {
      switch (col) {
        case 0: tr_read_at<0>(dst, base); break;
        case 1: tr_read_at<ROWB>(dst, base); break;
        default: tr_read_at<2 * ROWB>(dst, base); break;
      }
    };
    auto issue_reads = [&](int s) {
      const int k = s / TAPS, f = s % TAPS;
      if (f == 0) {
#pragma unroll
        for (int h = 0; h < 2; ++h) read_z(fz[k & 1][h], k, h);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) read_x(fx[s % (AHEAD + 1)][h], rb[k][h][f / 3], f % 3);
    };
#pragma unroll
    for (int s = 0; s < AHEAD; ++s) issue_reads(s);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int k = s / TAPS, f = s % TAPS;
      constexpr int last = NS - 1;
      if (s + AHEAD < NS) issue_reads(s + AHEAD);
      // everything issued after the reads of slot s may still be in flight
      switch (reads_through(s + AHEAD < last ? s + AHEAD : last) - reads_through(s)) {
        case 0: wait_lgkm<0>(); break;
        case 2: wait_lgkm<2>(); break;
        case 4: wait_lgkm<4>(); break;
        case 6: wait_lgkm<6>(); break;
        case 8: wait_lgkm<8>(); break;
        default: wait_lgkm<10>(); break;
      }
      pin(fz[k & 1][0]); pin(fz[k & 1][1]); pin(fx[s % (AHEAD + 1)][0]); pin(fx[s % (AHEAD + 1)][1]);
      acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(join2(fx[s % (AHEAD + 1)][0], fx[s % (AHEAD + 1)][1]),
                                                       join2(fz[k & 1][0], fz[k & 1][1]), acc[f], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      // in the shadow of the multiply: one copy of the tile two ahead (its window state stepped first), then the
      // pixel offsets of the next tile
      if (s < NCPY) {
        if (s >= KS && s - KS < NXU) advance_window(s - KS);
        issue_copy(s, ztile_f, live_f, fill);
      }
      if (s >= NS - 2 * KS) {
        const int e = s - (NS - 2 * KS);
        advance_pixel(e >> 1, e & 1);
        pnext[e >> 1][e & 1] = pixel_rel(e >> 1, e & 1, vf_next);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    STAMP(3 + 2 * (tile - tile_beg));
#pragma unroll
    for (int k = 0; k < KS; ++k) { ptv[k][0] = pnext[k][0]; ptv[k][1] = pnext[k][1]; }
    vf_cur = vf_next; vf_next = vf_fill;
    stage_off += p.stage_bytes;
    if (stage_off >= NSTAGE * p.stage_bytes) stage_off = 0;
  }
  (void)vf_cur;

  // ---- the eight waves add their accumulators through LDS ---------------------------------------------
  // [copy][tap][e][lane] floats; waves 4..7 hand theirs to waves 0..3, then those four copies are summed by all.
  STAMP(60);
  wait_all_copies();
  __syncthreads();
  // Fused fold-back: what the epilogue needs from memory (this wave's 32 x 32 blocks of w, four lanes per 64-byte
  // row, and the channel scale) is requested now and arrives while the accumulators are summed.
  const bool fused = p.wgt != nullptr;
  const int co_l = lane & 31;
  uint4 wpa0 = make_uint4(0u, 0u, 0u, 0u), wpb0 = wpa0, wpa1 = wpa0, wpb1 = wpa0;   // (tap wave | wave + 8) x (rows 0..15 | 16..31)
  float gam = 1.f, vr = 1.f;
  if (fused) {
    gam = p.gamma[co0 + co_l];
    vr = p.var[co0 + co_l];
    auto w_block = [&](int tap, int it) {
      return *reinterpret_cast<const uint4*>(p.wgt + ((size_t)(co0 + it * 16 + (lane >> 2)) * TAPS + tap) * p.Cin + ci0 + (lane & 3) * 8);
    };
    wpa0 = w_block(wave, 0); wpb0 = w_block(wave, 1);
    if (wave + NWAVES < TAPS) { wpa1 = w_block(wave + NWAVES, 0); wpb1 = w_block(wave + NWAVES, 1); }
  }
  // copies as [copy][tap][q][lane] float4 (q = accumulator elements 4 q .. 4 q + 3): every access is 16 bytes per
  // lane, consecutive lanes consecutive banks
  float4* red = reinterpret_cast<float4*>(smem);
  constexpr int COPY4 = TAPS * 4 * 64;   // float4 per copy
  if (wave >= 4) {
    float4* mine = red + (size_t)(wave - 4) * COPY4 + lane;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        mine[(t * 4 + q) * 64] = make_float4(acc[t][4 * q], acc[t][4 * q + 1], acc[t][4 * q + 2], acc[t][4 * q + 3]);
  }
  __syncthreads();
  if (wave < 4) {
    float4* mine = red + (size_t)wave * COPY4 + lane;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 o = mine[(t * 4 + q) * 64];
        mine[(t * 4 + q) * 64] = make_float4(o.x + acc[t][4 * q], o.y + acc[t][4 * q + 1], o.z + acc[t][4 * q + 2],
                                             o.w + acc[t][4 * q + 3]);
      }
  }
  // channel sums of dZ: a thread holds 8 channels (granule tid % 4) of its pixel rows; add the 16 lanes of a wave
  // that share a granule, then the eight waves through LDS (behind the accumulator copies)
  float* rred = reinterpret_cast<float*>(smem + RED_BYTES);
  if (do_r) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = racc[e];
#pragma unroll
      for (int off = 4; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
      if (lane < 4) rred[wave * 32 + lane * 8 + e] = v;
    }
  }
  __syncthreads();
  // Accumulator element e of lane l: ci row 8 (e / 4) + 4 (l / 32) + e % 4, co column l % 32.  Wave w sums the
  // four copies of taps w and w + 8 in the accumulators' own [e][lane] order (consecutive lanes, consecutive
  // banks) and stores 4 input channels per lane and instruction.
  STAMP(61);
  float dot = 0.f;
  const float scale = fused ? gam / sqrtf(vr + p.eps) : 1.f;
  auto finish_tap = [&](int tap, const uint4& wpa, const uint4& wpb) {
    const float4* src = red + (size_t)tap * (4 * 64) + lane;
    const size_t o = (((size_t)split * p.Co + co0 + co_l) * TAPS + tap) * p.Cin + ci0 + 4 * kb;
    float v[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 c0 = src[q * 64], c1 = src[q * 64 + COPY4], c2 = src[q * 64 + 2 * COPY4], c3 = src[q * 64 + 3 * COPY4];
      v[q][0] = (c0.x + c1.x) + (c2.x + c3.x); v[q][1] = (c0.y + c1.y) + (c2.y + c3.y);
      v[q][2] = (c0.z + c1.z) + (c2.z + c3.z); v[q][3] = (c0.w + c1.w) + (c2.w + c3.w);
    }
    if (!fused) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(p.part + o + 8 * q) = make_float4(v[q][0], v[q][1], v[q][2], v[q][3]);
      return;
    }
    // Fused fold-back.  In the accumulators a lane holds 4 input channels of one output channel: stores and loads
    // of that shape would touch memory in 8-byte pieces.  The 32 x 32 block of w and of dW for this tap therefore
    // passes through LDS (the space of this tap's first accumulator copy, which only this wave uses): global
    // accesses are 16 bytes per lane, four lanes per 64-byte row of the block.
    unsigned char* wtile = reinterpret_cast<unsigned char*>(red + (size_t)tap * (4 * 64));   // [32 co][32 ci] bf16
    unsigned char* otile = wtile + 2048;
    *reinterpret_cast<uint4*>(wtile + (lane >> 2) * 64 + (lane & 3) * 16) = wpa;
    *reinterpret_cast<uint4*>(wtile + (16 + (lane >> 2)) * 64 + (lane & 3) * 16) = wpb;
    // w' of this block in the transposed order: [32 ci][32 co], in the space of this tap's second accumulator copy
    unsigned short* ttile = reinterpret_cast<unsigned short*>(red + COPY4 + (size_t)tap * (4 * 64));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint2 w = *reinterpret_cast<const uint2*>(wtile + co_l * 64 + (8 * q + 4 * kb) * 2);
      dot += v[q][0] * bf16_lo(w.x) + v[q][1] * bf16_hi(w.x) + v[q][2] * bf16_lo(w.y) + v[q][3] * bf16_hi(w.y);
      *reinterpret_cast<uint2*>(otile + co_l * 64 + (8 * q + 4 * kb) * 2) =
          make_uint2(pack_bf16x2(scale * v[q][0], scale * v[q][1]), pack_bf16x2(scale * v[q][2], scale * v[q][3]));
      if (p.w_t) {   // the same product and rounding as the fold kernel's
        const unsigned a = pack_bf16x2(bf16_lo(w.x) * scale, bf16_hi(w.x) * scale);
        const unsigned b = pack_bf16x2(bf16_lo(w.y) * scale, bf16_hi(w.y) * scale);
        unsigned short* col = ttile + (8 * q + 4 * kb) * 32 + co_l;
        col[0] = (unsigned short)a; col[32] = (unsigned short)(a >> 16);
        col[64] = (unsigned short)b; col[96] = (unsigned short)(b >> 16);
      }
    }
    if (p.w_t) {
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int ci = it * 16 + (lane >> 2), g = lane & 3;
        *reinterpret_cast<uint4*>(p.w_t + ((size_t)(ci0 + ci) * TAPS + tap) * p.Co + co0 + g * 8) =
            *reinterpret_cast<const uint4*>(ttile + ci * 32 + g * 8);
      }
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int co = it * 16 + (lane >> 2), g = lane & 3;
      *reinterpret_cast<uint4*>(p.dW + ((size_t)(co0 + co) * TAPS + tap) * p.Cin + ci0 + g * 8) =
          *reinterpret_cast<const uint4*>(otile + co * 64 + g * 16);
    }
  };
  finish_tap(wave, wpa0, wpb0);
  if (wave + NWAVES < TAPS) finish_tap(wave + NWAVES, wpa1, wpb1);
  if (do_r && tid < 32) {
    float v = 0.f;
    for (int w = 0; w < NWAVES; ++w) v += rred[w * 32 + tid];
    if (fused) store_slot(p.slots + (size_t)p.nci * p.Co + co0 + tid, v, p.tag);   // r: the row behind the nci rows
    else p.r_part[(size_t)split * p.Co + co0 + tid] = v;
  }
  STAMP(62);
  if (!fused) return;
  // <dw', w> of this workgroup's channel pair: the two lane halves of a wave, then the eight waves
  dot += __shfl_xor(dot, 32, 64);
  float* dred = rred + NWAVES * 32;
  if (lane < 32) dred[wave * 32 + lane] = dot;
  __syncthreads();
  if (tid < 32) {
    float v = 0.f;
    for (int w = 0; w < NWAVES; ++w) v += dred[w * 32 + tid];
    store_slot(p.slots + (size_t)cit * p.Co + co0 + tid, v, p.tag);
  }
  STAMP(50);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's slots have reached memory ...
  __syncthreads();                                    // ... and every other thread's, before anyone looks
  STAMP(51);
  // Which workgroup of this output-channel tile finishes last is found without a shared counter (an atomic at
  // device scope is a round trip to memory, and a compare-and-swap loop over 16 workgroups that end together takes
  // many): a slot carries its value and this launch's tag in one 16-byte store, every workgroup stores its own
  // slots first and then reads all nci + 1 rows of the tile, a thread per slot.  Whoever finds every tag in place
  // has all the values in hand and finishes the tile; the workgroup whose stores landed last always does, and if
  // two do they write the same numbers.  Finishers clear the slots, so a replay of a captured launch (same tag)
  // finds none of them valid.
  float mine = 0.f, rmine = 0.f;
  int ok = 1;
  for (int i = tid >> 5; i <= p.nci; i += NWAVES * 2) {
    const uint4 sl = load_device_scope16(p.slots + (size_t)i * p.Co + co0 + (tid & 31));
    ok &= (((unsigned long long)sl.z << 32) | sl.y) == p.tag;
    if (i < p.nci) mine += __uint_as_float(sl.x); else rmine = __uint_as_float(sl.x);
  }
  STAMP(52);
  if (!__syncthreads_and(ok)) return;
  for (int i = tid >> 5; i <= p.nci; i += NWAVES * 2)
    store_device_scope16(p.slots + (size_t)i * p.Co + co0 + (tid & 31), make_uint4(0u, 0u, 0u, 0u));
  rred[tid] = mine;
  if ((p.nci >> 4 << 4) + (tid >> 5) == p.nci) rred[NWAVES * 64 + (tid & 31)] = rmine;   // the thread that read row nci
  __syncthreads();
  STAMP(53);
  if (tid >= 32) return;
  // dgamma = (<dw', w> + r (b - mu)) / sqrt(var + eps), dbeta = r, db = s r
  const int ch = co0 + tid;
  float d = 0.f;
  for (int i = 0; i < NWAVES * 2; ++i) d += rred[i * 32 + tid];
  const float r = rred[NWAVES * 64 + tid];
  const float sd = sqrtf(p.var[ch] + p.eps);
  const float bb = p.b ? p.b[ch] : 0.f;
  p.dgamma[ch] = (d + r * (bb - p.mean[ch])) / sd;
  p.dbeta[ch] = r;
  if (p.db) p.db[ch] = p.gamma[ch] / sd * r;
}

template <int KS, int NCPY>
__global__ __launch_bounds__(64 * NWAVES) void wgrad_sq_kernel(SqParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  sq_body<KS, NCPY>(p, blockIdx.x, smem);
}

// Weight gradient and input gradient of one block in ONE launch: the two passes are independent (both read dZ), each
// fills the chip with one workgroup per compute unit and a tail of its own, and two launches cannot overlap.  As one
// grid the first nsq workgroups are the weight gradient's, the rest the input gradient's (conv_rw_impl.h): compute
// units that finish -- or never had -- a workgroup of the first take workgroups of the second, and the phases in
// which all workgroups of one pass load or drain at once are filled by the other's multiplies.
template <int KS, int NCPY>
__global__ __launch_bounds__(64 * NWAVES) void wgrad_dgrad_pair_kernel(SqParams ps, rw::RwParams pr, int nsq) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  if ((int)blockIdx.x < nsq) sq_body<KS, NCPY>(ps, blockIdx.x, smem);
  else rw::body(pr, (int)blockIdx.x - nsq, (int)gridDim.x - nsq, smem);
}

// Largest number of window-tile pixels any tile of `tile` consecutive output pixels needs.
int max_window_pixels(const SqParams& p, int tile) {
  const int HoWo = p.Ho * p.Wo;
  int a = HoWo, b = tile;
  while (b) { const int t = a % b; a = b; b = t; }
  const int period = HoWo / a;
  int best = 0;
  for (int m0 = 0, t = 0; m0 < p.M && t <= period; m0 += tile, ++t) {
    const int ml = (m0 + tile < p.M ? m0 + tile : p.M) - 1;
    const int na = m0 / HoWo, hoa = (m0 - na * HoWo) / p.Wo;
    const int nb = ml / HoWo, hob = (ml - nb * HoWo) / p.Wo;
    const int ns = nb * p.Hv + hob * p.sh + 3 - (na * p.Hv + hoa * p.sh);
    if (ns > best) best = ns;
  }
  return best * p.Wv;
}

struct SqPlan { bool ok; int ks, ncpy, nsplit; size_t lds; };

SqPlan make_plan(const Geom& g, SqParams* pp) {
  SqPlan pl{false, 0, 0, 0, 0};
  SqParams& p = *pp;
  p = SqParams{};
  if (g.kH != 3 || g.kW != 3) return pl;
  if (g.Cin % 32 || g.Cout % 32) return pl;
  const size_t xb = (size_t)g.Min * g.Cin * 2, zb = (size_t)g.M * g.Cout * 2;
  if (xb >= OOB || zb >= OOB) return pl;
  p.N = g.N; p.Cin = g.Cin; p.Ho = g.Hout; p.Wo = g.Wout; p.Co = g.Cout; p.M = g.M;
  p.kW = g.kW; p.H = g.Hin; p.W = g.Win; p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
  p.x_n_stride = g.Hin * g.Win * g.Cin; p.x_h_stride = g.Win * g.Cin; p.x_w_stride = g.Cin;
  p.x_bytes = (unsigned)xb; p.dz_bytes = (unsigned)zb;
  p.Hv = (p.Ho - 1) * p.sh + 3;
  p.Wv = (p.Wo - 1) * p.sw + 3;
  // byte offsets among the window rows of the whole tensor (and two images past it) are kept in 32 bits
  if ((long long)(p.N + 2) * p.Hv * p.Wv * ROWB >= (long long)OOB) return pl;
  p.dHoWo = make_fastdiv(p.Ho * p.Wo);
  p.dWo = make_fastdiv(p.Wo);
  p.dHv = make_fastdiv(p.Hv);
  p.dWv = make_fastdiv(p.Wv);
  p.nci = g.Cin / 32;
  p.nco = g.Cout / 32;
  // 256-pixel tiles where three stages fit the LDS and a wave carries their window copies, else 128
  for (int ks = 2; ks >= 1; --ks) {
    const int tile = 128 * ks;
    const int hunits = ceil_div(max_window_pixels(p, tile), 16);
    const int nxu = ceil_div(hunits, NWAVES);
    const int stage = tile * ROWB + hunits * 1024;
    size_t lds = 3 * (size_t)stage;
    if (lds < (size_t)RED_BYTES + 4096) lds = (size_t)RED_BYTES + 4096;   // the final reduction: four accumulator copies + channel sums, dot products, flag
    if (lds > LDS_USABLE || nxu > MAXXU) continue;
    pl.ks = ks; pl.ncpy = ks + nxu; pl.lds = lds;
    p.hunits = hunits; p.stage_bytes = stage;
    p.ntiles = ceil_div(g.M, tile);
    const int rem = tile % (p.Ho * p.Wo);
    p.step_h = rem / p.Wo;
    p.step_w = rem % p.Wo;
    p.step_off = (((tile / (p.Ho * p.Wo)) * p.Hv + p.step_h * p.sh) * p.Wv + p.step_w * p.sw) * ROWB;
    p.carry_w_off = (p.sh * p.Wv - p.Wo * p.sw) * ROWB;
    p.carry_h_off = (p.Hv - p.Ho * p.sh) * p.Wv * ROWB;
    p.max_pixel_off = hunits * 1024 - (2 * p.Wv + 3) * ROWB;
    break;
  }
  if (pl.ks == 0) return pl;
  // pixel splits: about one workgroup per compute unit
  const int pairs = p.nci * p.nco;
  int want = pairs >= 192 ? 1 : (256 + pairs / 2) / pairs;
  if (want > p.ntiles) want = p.ntiles;
  if (want < 1) want = 1;
  p.tiles_per_split = ceil_div(p.ntiles, want);
  pl.nsplit = ceil_div(p.ntiles, p.tiles_per_split);
  // blocks of up to 4 x 8 channel pairs that go to one XCD together
  p.bi = p.nci % 8 == 0 ? 8 : (p.nci <= 8 ? p.nci : 1);
  p.bc = p.bi == 1 ? 1 : (p.nco % 4 == 0 ? 4 : (p.nco <= 4 ? p.nco : 1));
  p.nbci = p.nci / p.bi;
  p.blocks_per_split = p.nbci * (p.nco / p.bc);
  p.nblocks = p.blocks_per_split * pl.nsplit;
  pl.ok = true;
  return pl;
}

template <int KS, int NCPY>
hipError_t launch_inst(const SqParams& p, const SqPlan& pl, hipStream_t st) {
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_sq_kernel<KS, NCPY>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_USABLE);
  });
  if (attr_err != hipSuccess) return attr_err;
  const int grid = 8 * ceil_div(p.nblocks, 8) * p.bc * p.bi;
  hipLaunchKernelGGL((wgrad_sq_kernel<KS, NCPY>), dim3(grid), dim3(64 * NWAVES), pl.lds, st, p);
  return hipGetLastError();
}

template <int KS, int NCPY>
hipError_t launch_pair_inst(const SqParams& ps, const SqPlan& pl, const rw::RwParams& pr, hipStream_t st) {
  static LdsLimitOnce lds_once;
  if (hipError_t e = set_lds_limit_once(lds_once, reinterpret_cast<const void*>(&wgrad_dgrad_pair_kernel<KS, NCPY>),
                                        (int)LDS_USABLE); e != hipSuccess) return e;
  const int nsq = 8 * ceil_div(ps.nblocks, 8) * ps.bc * ps.bi;
  const int nrw = ceil_div(pr.M, pr.L);
  const size_t lds = pl.lds > (size_t)pr.lds_bytes ? pl.lds : (size_t)pr.lds_bytes;   // <= LDS_USABLE: checked by the caller
  hipLaunchKernelGGL((wgrad_dgrad_pair_kernel<KS, NCPY>), dim3(nsq + nrw), dim3(64 * NWAVES), lds, st, ps, pr, nsq);
  return hipGetLastError();
}

unsigned long long next_tag() {
  static std::atomic<unsigned long long> tag{
      (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count() * 0x9E3779B97F4A7C15ull};
  const unsigned long long t = tag.fetch_add(1, std::memory_order_relaxed);
  return t ? t : tag.fetch_add(1, std::memory_order_relaxed);   // 0 marks a cleared slot
}

hipError_t dispatch(const SqParams& p, const SqPlan& pl, hipStream_t st) {
#define CASE(K, X) if (pl.ks == K && pl.ncpy == K + X) return launch_inst<K, K + X>(p, pl, st);
  CASE(2, 1) CASE(2, 2) CASE(2, 3) CASE(2, 4) CASE(2, 5) CASE(2, 6)
  CASE(1, 1) CASE(1, 2) CASE(1, 3) CASE(1, 4) CASE(1, 5) CASE(1, 6)
#undef CASE
  return hipErrorInvalidValue;
}

}  // namespace

bool wgrad_sq_fused_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  SqParams p;
  const SqPlan pl = make_plan(g, &p);
  return pl.ok && pl.nsplit == 1;
}

size_t wgrad_sq_fused_scratch_bytes(const Geom& g) {
  return (size_t)(g.Cin / 32 + 1) * g.Cout * sizeof(uint4);
}

hipError_t launch_wgrad_sq_fused(const Geom& g, const void* x, const void* dz, const void* W, const float* b,
                                 const float* gamma, const float* mean, const float* var, void* dW, float* db,
                                 float* dgamma, float* dbeta, void* scratch, void* w_folded_out, hipStream_t st) {
  SqParams p;
  const SqPlan pl = make_plan(g, &p);
  if (!pl.ok || pl.nsplit != 1 || !scratch) return hipErrorInvalidValue;
  p.x = (const bf16_t*)x; p.dz = (const bf16_t*)dz; p.part = nullptr;
  p.r_part = reinterpret_cast<float*>(scratch);   // only its non-NULL-ness matters here: the channel sums are wanted
  p.wgt = (const bf16_t*)W; p.dW = (bf16_t*)dW; p.w_t = (bf16_t*)w_folded_out; p.gamma = gamma; p.mean = mean; p.var = var; p.b = b;
  p.db = db; p.dgamma = dgamma; p.dbeta = dbeta; p.eps = g.eps;
  p.slots = reinterpret_cast<uint4*>(scratch);   // workspace pieces are 256-byte aligned
  p.tag = next_tag();
  return dispatch(p, pl, st);
}

// One launch for the input gradient (resident-weight kernel) and the weight gradient (fp32 copies for the fold-back)
// of a block: where both kernels take the problem and the weight gradient runs on 256-pixel tiles.
bool wgrad_dgrad_pair_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  SqParams ps;
  rw::RwParams pr;
  const SqPlan pl = make_plan(g, &ps);
  // (the weight-gradient kernel keeps a KB of LDS of its own, so the pair has LDS_USABLE, not all 160 KB, for either body)
  return pl.ok && pl.ks == 2 && rw::dgrad_params(g, &pr) && (size_t)pr.lds_bytes <= LDS_USABLE;
}

hipError_t launch_wgrad_dgrad_pair(const Geom& g, const void* x, const void* dz, const void* w_crsk, void* dx,
                                   float* dwf_part, float* r_part, hipStream_t st) {
  SqParams ps;
  rw::RwParams pr;
  const SqPlan pl = make_plan(g, &ps);
  if (!pl.ok || pl.ks != 2 || !rw::dgrad_params(g, &pr) || (size_t)pr.lds_bytes > LDS_USABLE) return hipErrorInvalidValue;
  ps.x = (const bf16_t*)x; ps.dz = (const bf16_t*)dz; ps.part = dwf_part; ps.r_part = r_part;
  pr.act = (const bf16_t*)dz; pr.wgt = (const bf16_t*)w_crsk; pr.bias = nullptr; pr.out = (bf16_t*)dx;
  pr.relu = g.post_relu; pr.mask = (const bf16_t*)g.post_mask; pr.add = (const bf16_t*)g.post_add;
#define CASE(X) if (pl.ncpy == 2 + X) return launch_pair_inst<2, 2 + X>(ps, pl, pr, st);
  CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6)
#undef CASE
  return hipErrorInvalidValue;
}

bool wgrad_sq_supported(const Geom& g, int dtype) {
  if (dtype != CONVBN_BF16) return false;
  SqParams p;
  return make_plan(g, &p).ok;
}

int wgrad_sq_splits(const Geom& g) {
  SqParams p;
  return make_plan(g, &p).nsplit;
}

hipError_t launch_wgrad_sq(const Geom& g, const void* x, const void* dz, float* dwf_part, float* r_part,
                           hipStream_t st) {
  SqParams p;
  const SqPlan pl = make_plan(g, &p);
  if (!pl.ok) return hipErrorInvalidValue;
  p.x = (const bf16_t*)x; p.dz = (const bf16_t*)dz; p.part = dwf_part; p.r_part = r_part;
  return dispatch(p, pl, st);
}

}  // namespace convbn

#ifdef SQ_TRACE
extern "C" int convbn_debug_read_sq_trace(unsigned long long* host, size_t n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(convbn::sq_trace), n * sizeof(unsigned long long));
}
#endif
