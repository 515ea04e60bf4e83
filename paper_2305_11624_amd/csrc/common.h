// Shared device helpers and the internal launch interface of libconvbn (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>
#include <stdint.h>

#include "../../include/convbn.h"

namespace convbn {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs; NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  bf16_t h = (bf16_t)f;
  return (uint32_t)__builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Geometry of one block, with the derived sizes the kernels index with.
struct Geom {
  int N, Cin, Hin, Win, Cout, kH, kW, sh, sw, ph, pw, Hout, Wout;
  int M;      // N*Hout*Wout   (output pixels)
  int Min;    // N*Hin*Win     (input pixels)
  int K;      // kH*kW*Cin     (reduction length of the forward conv)
  float eps;
  int act;    // the descriptor's CONVBN_ACT_* bits
  // What the convolution launched with this Geom does to its output on the way out (set per call by the host side,
  // not part of the problem): `post_add` (a tensor laid out like the output, or null) is added first, then ReLU, and /
  // or zero where `post_mask` (a tensor laid out like the output) is <= 0.
  int post_relu;
  const void* post_mask;
  const void* post_add;
  const void* add_out;   // the descriptor's addends (CONVBN_ACT_ADD_OUT / _IN), null where the bit is not set
  const void* add_in;
};

// The same on 8 packed bf16 values: max(., 0), and zero where the 8 packed bf16 values of m4 are <= 0.
__device__ __forceinline__ uint4 relu8(uint4 v) {
  unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned neg = ((w[i] >> 15) & 0x00010001u) * 0xffffu;   // 0xffff in every half whose sign bit is set
    w[i] &= ~neg;
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ uint4 mask8(uint4 v, uint4 m4) {
  unsigned w[4] = {v.x, v.y, v.z, v.w};
  const unsigned m[4] = {m4.x, m4.y, m4.z, m4.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned lo = __uint_as_float(m[i] << 16) > 0.f ? 0x0000ffffu : 0u;
    const unsigned hi = __uint_as_float(m[i] & 0xffff0000u) > 0.f ? 0xffff0000u : 0u;
    w[i] &= lo | hi;
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}
// v + a on 8 packed bf16 values each, added in fp32 and rounded once: what the element-wise sum of the two rounded
// tensors gives.
__device__ __forceinline__ uint4 add8(uint4 v, uint4 a4) {
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
  const unsigned a[4] = {a4.x, a4.y, a4.z, a4.w};
  unsigned r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    r[i] = pack_bf16x2(__uint_as_float(w[i] << 16) + __uint_as_float(a[i] << 16),
                       __uint_as_float(w[i] & 0xffff0000u) + __uint_as_float(a[i] & 0xffff0000u));
  return make_uint4(r[0], r[1], r[2], r[3]);
}
// ... about to be stored at element offset o of the output, the addend and the mask read on the spot.  (Requesting the mask values
// before the multiplies was measured on all four kernels that use this and changed nothing: what the mask costs them
// is its bytes, not the wait.)
__device__ __forceinline__ uint4 post_op8(uint4 v, int relu, const bf16_t* mask, const bf16_t* add, size_t o) {
  if (add) v = add8(v, *reinterpret_cast<const uint4*>(add + o));
  if (relu) v = relu8(v);
  if (mask) v = mask8(v, *reinterpret_cast<const uint4*>(mask + o));
  return v;
}

// Per-channel epilogue of a forward convolution that is given the UNFOLDED weight: Z = s (w (*) X) + b' with
// s = gamma / sqrt(var + eps) and b' = (b - mu) s + beta worked out by the kernel itself -- the same forward
// result as folding the weight first (Sec. 3.3), without materialising w'.  gamma == nullptr: not used.
struct BnEpilogue {
  const float* gamma;
  const float* beta;
  const float* mean;
  const float* var;
  const float* b;   // convolution bias or nullptr
  float eps;
  // Optional: the launch also leaves w' = s w as [Cin][taps][Cout] -- what Tune mode keeps for backward (Sec. 3.4.2)
  // -- every workgroup writing one slice of it, so that a forward pass that keeps w' is still a single launch.
  void* w_folded_out;
  int taps, Cin, Cout;
};

// Slice `wg` of `nwg` of w' = bf16(float(w) s), written in [Cin][taps][Cout] order (w is [Cout][taps][Cin]); the same
// values, bit for bit, as the fold kernel's.  Called by all threads of a workgroup.
__device__ __forceinline__ void emit_folded_slice(const BnEpilogue& bn, const bf16_t* __restrict__ w, int wg, int nwg) {
  bf16_t* out = static_cast<bf16_t*>(bn.w_folded_out);
  const int P = bn.Cout * bn.taps * bn.Cin;
  const int per = (P + nwg - 1) / nwg;
  const int end = min(P, (wg + 1) * per);
  for (int j = wg * per + (int)threadIdx.x; j < end; j += (int)blockDim.x) {
    const int co = j % bn.Cout;
    const int rest = j / bn.Cout;
    const int tap = rest % bn.taps, ci = rest / bn.taps;
    const float s = bn.gamma[co] / sqrtf(bn.var[co] + bn.eps);
    out[j] = (bf16_t)((float)w[((size_t)co * bn.taps + tap) * bn.Cin + ci] * s);
  }
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Raises a kernel's dynamic-LDS limit once per process -- also when several host threads launch it for the first
// time together -- and remembers the outcome.
struct LdsLimitOnce {
  std::once_flag once;
  hipError_t err = hipSuccess;
};
inline hipError_t set_lds_limit_once(LdsLimitOnce& s, const void* kernel, int bytes) {
  std::call_once(s.once, [&] { s.err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
  return s.err;
}
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- launchers (each enqueues on `st`, returns the hipError of the launch) ----

// fold.hip
// w_krsc / w_crsk / bfold may each be NULL (skipped).  identity != 0: s = 1, b' = b.
hipError_t launch_fold(const Geom& g, int dtype, const void* W, const float* b, const float* gamma,
                       const float* beta, const float* mean, const float* var, int identity,
                       void* w_krsc, void* w_crsk, float* bfold, hipStream_t st);
// Grouped fold: fold_group_item() writes one table entry (fold_group_item_bytes() bytes, host memory) for a
// bf16 block with K and Cout multiples of 8 (false otherwise) and returns its number of workgroups;
// launch_fold_group() runs a table that has been copied to device memory.
size_t fold_group_item_bytes();
bool fold_group_item(const Geom& g, int dtype, const void* W, const float* b, const float* gamma, const float* beta,
                     const float* mean, const float* var, int identity, void* w_krsc, void* w_crsk, float* bfold,
                     int first_block, void* item_out, int* blocks);
hipError_t launch_fold_group(const void* items_dev, int n, int grid_blocks, hipStream_t st);
// Sums `nsplit` fp32 partial copies of dJ/dw' ([nsplit][Cout][K]) and `nrpart` partial
// row-sum vectors ([nrpart][Cout]); writes dW, db, dgamma, dbeta (Table 2 "Tune").
// identity != 0 (Eval path): dW = sum of partials only, other outputs untouched.
hipError_t launch_fold_back(const Geom& g, int dtype, const float* dwf_part, int nsplit,
                            const float* r_part, int nrpart, const void* W, const float* b,
                            const float* gamma, const float* mean, const float* var, int identity,
                            void* dW, float* db, float* dgamma, float* dbeta, hipStream_t st);
// Grouped fold-back: fold_back_group_item() writes one table entry (host memory) for a bf16 block whose K is a
// multiple of 4 (false otherwise) and returns its number of workgroups; launch_fold_back_group() runs a table
// that has been copied to device memory.
size_t fold_back_group_item_bytes();
bool fold_back_group_item(const Geom& g, int dtype, const float* dwf_part, int nsplit, const float* r_part, int nrpart,
                          const void* W, const float* b, const float* gamma, const float* mean, const float* var,
                          void* dW, float* db, float* dgamma, float* dbeta, int first_block, void* item_out,
                          int* blocks);
hipError_t launch_fold_back_group(const void* items_dev, int n, int grid_blocks, hipStream_t st);
// fold_t.hip : fold / fold-back of the transposed block, weight [Ci][taps][Co] with the scale on co.
// w_same ([Ci][taps][Co]), w_swap ([Co][taps][Ci]) and bfold may each be NULL (skipped).  tap_major != 0:
// w_swap is [taps][Co][Ci] and bfold [taps][Co] (b' repeated for every tap) instead.  gamma == NULL: s = 1, b' = b.
hipError_t launch_fold_t(int dtype, int Ci, int Co, int taps, const void* W, const float* b, const float* gamma,
                         const float* beta, const float* mean, const float* var, float eps, int tap_major,
                         void* w_same, void* w_swap, float* bfold, hipStream_t st);
int fold_back_t_chunks(int Ci, int taps);   // rows of dot_part ([chunks][Co] fp32 scratch)
// gamma == NULL (Eval path): dW = sum of the partial copies only; dot_part and the other outputs are not touched.
hipError_t launch_fold_back_t(int dtype, int Ci, int Co, int taps, const float* dwf_part, int nsplit,
                              const float* r_part, int nrpart, const void* W, const float* b, const float* gamma,
                              const float* mean, const float* var, float eps, float* dot_part, void* dW, float* db,
                              float* dgamma, float* dbeta, hipStream_t st);
int colsum_parts(const Geom& g);
hipError_t launch_colsum(const Geom& g, int dtype, const void* dz, float* r_part, hipStream_t st);
hipError_t launch_bn_affine_fwd(const Geom& g, int dtype, const void* y, const float* gamma,
                                const float* beta, const float* mean, const float* var, void* z,
                                hipStream_t st);
int bn_bwd_parts(const Geom& g);
hipError_t launch_bn_bwd(const Geom& g, int dtype, const void* dz, const void* y, const float* gamma,
                         const float* mean, const float* var, void* dy, float* part /*[parts][2][Cout]*/,
                         hipStream_t st);
hipError_t launch_bn_bwd_finalize(const Geom& g, const float* part, int parts, const float* gamma,
                                  const float* var, float* dgamma, float* dbeta, float* db,
                                  hipStream_t st);

// Copies a [rows][inner_in] matrix of `elem_bytes`-wide elements (2 or 4) into [rows][inner_out]:
// the first min(inner_in, inner_out) elements of every row, zeros behind them (fold.hip).
hipError_t launch_repitch(int elem_bytes, size_t rows, size_t inner_in, size_t inner_out, const void* src,
                          void* dst, hipStream_t st);

// aux_ops.hip : glue between blocks for the whole-backbone measurement
//   op: 0 relu (a), 1 relu backward (a = b > 0 ? a : 0), 2 a = relu(a + b), 3 a += b;  n % 8 == 0
hipError_t launch_eltwise(int op, int dtype, void* a, const void* b, const void* c, size_t n, hipStream_t st);
hipError_t launch_maxpool_fwd(int dtype, const void* x, void* y, unsigned char* idx, int N, int H, int W, int C,
                              hipStream_t st);
hipError_t launch_maxpool_bwd(int dtype, const void* dy, const unsigned char* idx, void* dx, int N, int H, int W,
                              int C, hipStream_t st);

// depthwise.hip : the depthwise block (groups = channels; g.Cin == g.Cout), plain vector kernels.
// wf is the folded filter in tap-major order [kH kW][C]; gamma == NULL means s = 1 (Eval comparison path).
hipError_t launch_dw_fold(const Geom& g, int dtype, const void* W, const float* b, const float* gamma,
                          const float* beta, const float* mean, const float* var, void* wf, float* bfold,
                          hipStream_t st);
hipError_t launch_dw_fprop(const Geom& g, int dtype, const void* x, const void* wf, const float* bias, void* z,
                           hipStream_t st);
hipError_t launch_dw_dgrad(const Geom& g, int dtype, const void* dz, const void* wf, void* dx, hipStream_t st);
int dw_wgrad_slices(const Geom& g, int dtype);
// part [slices][taps][C], r_part [slices][C] (nullable), sums [(taps + 1)][C]: fp32 scratch
hipError_t launch_dw_wgrad(const Geom& g, int dtype, const void* x, const void* dz, float* part, float* r_part,
                           hipStream_t st);
hipError_t launch_dw_fold_back(const Geom& g, int dtype, const float* part, const float* r_part, int slices,
                               float* sums, const void* W, const float* b, const float* gamma, const float* mean,
                               const float* var, void* dW, float* db, float* dgamma, float* dbeta, hipStream_t st);

// conv_grouped.hip : the three contractions of a grouped block (groups divides g.Cin and g.Cout; cg = Cin / groups).
// w_krsc is [Cout][kH][kW][cg], w_crsk [cg][kH][kW][Cout]; part [slices][Cout][kH kW cg] fp32.  Where
// g_wgrad_makes_rsum() the weight-gradient launch also writes r_part [slices][Cout] (else it ignores it).
hipError_t launch_g_fprop(const Geom& g, int groups, int dtype, const void* x, const void* w_krsc, const float* bias,
                          void* z, hipStream_t st);
hipError_t launch_g_dgrad(const Geom& g, int groups, int dtype, const void* dz, const void* w_crsk, void* dx,
                          hipStream_t st);
int g_wgrad_slices(const Geom& g, int groups, int dtype);
bool g_wgrad_makes_rsum(const Geom& g, int groups, int dtype);
hipError_t launch_g_wgrad(const Geom& g, int groups, int dtype, const void* x, const void* dz, float* part,
                          float* r_part, hipStream_t st);

// conv_direct.hip : one thread per output element, fp32 accumulation (any shape, both dtypes)
hipError_t launch_fprop_direct(const Geom& g, int dtype, const void* x, const void* w_krsc,
                               const float* bias, void* z, hipStream_t st);
hipError_t launch_dgrad_direct(const Geom& g, int dtype, const void* dz, const void* w_crsk,
                               const float* bias /*[Cin] or null*/, void* dx, hipStream_t st);
int wgrad_direct_splits(const Geom& g);
hipError_t launch_wgrad_direct(const Geom& g, int dtype, const void* x, const void* dz,
                               float* dwf_part /*[splits][Cout][K]*/, hipStream_t st);

// conv_stem.hip : forward convolution of a first layer (at most 4 input channels), bf16 MFMA, operands read
// straight from the raw input patch.  w is the weight as [Cout][kH][kW][Cin].
bool stem_fprop_supported(const Geom& g, int dtype);
bool stem_wgrad_supported(const Geom& g, int dtype);
int stem_wgrad_slices(const Geom& g);             // fp32 partial copies of dw' (and of r) the kernel writes
hipError_t launch_wgrad_stem(const Geom& g, const void* x, const void* dz, float* part, float* r_part, hipStream_t st);
bool stem_dgrad_supported(const Geom& g, int dtype);
size_t stem_dgrad_weight_bytes(const Geom& g);    // scratch for the input gradient's packed weight
hipError_t launch_dgrad_stem(const Geom& g, const void* dz, const void* w_crsk, void* wpack, void* dx, hipStream_t st);
size_t stem_packed_weight_bytes(const Geom& g);   // scratch for the weight padded to 8 window columns x 4 channels
size_t stem_input_copy_bytes(const Geom& g);      // scratch for a 4-channel copy of the input (0: read as it is)
hipError_t launch_fprop_stem(const Geom& g, const void* x, const void* w, void* wpad, const float* bias, void* z,
                             hipStream_t st);

// conv_igemm.hip : bf16 MFMA implicit GEMM
bool igemm_supported(const Geom& g, int dtype);
int wgrad_splits(const Geom& g);
hipError_t launch_fprop_igemm(const Geom& g, const void* x, const void* w_krsc, const float* bias,
                              void* z, hipStream_t st);
hipError_t launch_dgrad_igemm(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                              hipStream_t st);
hipError_t launch_wgrad_igemm(const Geom& g, const void* x, const void* dz, float* dwf_part,
                              int nsplit, hipStream_t st);

// conv_tile.hip : bf16 MFMA convolution with the input window tile resident in LDS
// (every input element is fetched once per block and reused by all taps).
// conv_pw.hip: persistent weight-stationary kernel for 1x1 / stride-1 convolutions over long pixel ranges
// the tiled matrix product that takes the pointwise layers of the middle stages (conv_gm.hip); reached through the
// pw_* calls below
bool gm_supported(int M, int C, int R);
// sd != null: a strided pointwise layer -- the M rows are the pixels of the dense side [N][Ho][Wo], and the rows of the
// activations (scatter == 0) or of the output (scatter == 1; no post-operation then) are pixel (n, ho sh, wo sw) of an
// [N][Hs][Ws] tensor.
struct GmStride { int scatter, N, Ho, Wo, Hs, Ws, sh, sw; };
// Window mode of the same kernel (no window tile in LDS: every tap gathers its rows; for strided layers).  A kH x kW
// window slides with stride (csh, csw) and padding (cph, cpw) over an [N][aH][aW] activation grid with element strides
// a_n, a_h, a_w; output pixel (n, ho, wo) of an [N][oHo][oWo] grid is stored at element out_base + n out_n + ho out_h +
// wo out_w (out_strided) or at row m of a dense [M][R] tensor; window position (ti, tj) multiplies with tap
// wt0 + ti wt_row + tj wt_col of the weight tensor, whose rows (one per output channel) have wrow elements.
struct GmConv {
  int kH, kW, cph, cpw, csh, csw, aH, aW;
  int a_n, a_h, a_w;
  int oHo, oWo;
  int wt0, wt_row, wt_col, wrow;
  int out_strided, out_base, out_n, out_h, out_w;
};
bool gm_conv_supported(int M, int C, int R, const GmConv& cv);
hipError_t launch_gm_conv(int M, int C, int R, const GmConv& cv, const void* act, unsigned act_bytes, const void* wgt,
                          unsigned wgt_bytes, const float* bias, void* out, int relu, const void* mask, const void* add,
                          hipStream_t st);
hipError_t launch_gm(int M, int C, int R, const void* act, const void* wgt, const float* bias, const BnEpilogue* bn,
                     void* out, int relu, const void* mask, const void* add, hipStream_t st, const GmStride* sd = nullptr);
hipError_t launch_gm_fill(void* p, size_t rows, int R, const float* bias, hipStream_t st);   // rows of bias (null: zeros), R % 8 == 0
bool pw_fprop_supported(const Geom& g, int dtype);
bool pw_fprop_scaled_supported(const Geom& g, int dtype);     // ... with a BnEpilogue
bool pw_dgrad_supported(const Geom& g, int dtype);
hipError_t launch_fprop_pw(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z,
                           hipStream_t st, const BnEpilogue* bn = nullptr);
hipError_t launch_dgrad_pw(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                           hipStream_t st);
// Forward of a transposed convolution whose stride equals its window (no padding), as one product with a
// depth-to-space store; g is the convolution the block is the adjoint of.  w_tap_major is [taps][g.Cin][g.Cout]
// (rows (tap, co)), bias_per_tap [taps][g.Cin] (the folded bias repeated per tap).
bool pw_tconv_supported(const Geom& g, int dtype);
hipError_t launch_tconv_pw(const Geom& g, const void* x, const void* w_tap_major, const float* bias_per_tap, void* z,
                           hipStream_t st);

// conv_st.hip : 3x3 / stride-1 convolutions of deep layers on 64-pixel x 128-channel tiles shared by eight waves
// (no split sums, no scratch).
bool st_fprop_supported(const Geom& g, int dtype);
bool st_dgrad_supported(const Geom& g, int dtype);
// bn != nullptr: w_krsc is the UNFOLDED weight and the epilogue applies the BatchNorm scale and folded bias itself
hipError_t launch_fprop_st(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z, hipStream_t st,
                           const BnEpilogue* bn = nullptr);
hipError_t launch_dgrad_st(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx, hipStream_t st);

// conv_rw.hip : 3x3 / stride-1 convolutions of shallow layers (64 -> 64 channels, long pixel streams): weight and
// window resident in LDS, one barrier per workgroup (no scratch).
bool rw_fprop_supported(const Geom& g, int dtype);
bool rw_dgrad_supported(const Geom& g, int dtype);
// bn != nullptr: w_krsc is the UNFOLDED weight and the epilogue applies the BatchNorm scale and folded bias itself
hipError_t launch_fprop_rw(const Geom& g, const void* x, const void* w_krsc, const float* bias, void* z, hipStream_t st,
                           const BnEpilogue* bn = nullptr);
hipError_t launch_dgrad_rw(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx, hipStream_t st);

bool tile_fprop_supported(const Geom& g, int dtype);
bool tile_fprop_scaled_supported(const Geom& g, int dtype);   // ... with a BnEpilogue
bool tile_dgrad_supported(const Geom& g, int dtype);
// Some problems split the reduced channels over several workgroups and need fp32 partial-output
// storage of this many bytes (0 otherwise), passed as `partials`.
size_t tile_fprop_partial_bytes(const Geom& g);
size_t tile_dgrad_partial_bytes(const Geom& g);
hipError_t launch_fprop_tile(const Geom& g, const void* x, const void* w_krsc, const float* bias,
                             void* z, float* partials, hipStream_t st, const BnEpilogue* bn = nullptr);
// The input-gradient launchers take an optional per-input-channel bias: a transposed convolution's forward
// pass is this kernel (Sec. 3.2.1), and its folded bias b' is added here.
hipError_t launch_dgrad_tile(const Geom& g, const void* dz, const void* w_crsk, const float* bias, void* dx,
                             float* partials, hipStream_t st);

// wgrad_tile.hip : bf16 MFMA weight gradient with LDS-resident pixel tiles; also produces the
// per-channel sums r (one partial per split) when r_part != nullptr.
bool wgrad_tile_supported(const Geom& g, int dtype);
int wgrad_tile_splits(const Geom& g);
hipError_t launch_wgrad_tile(const Geom& g, const void* x, const void* dz, float* dwf_part, float* r_part,
                             hipStream_t st);

// wgrad_sq.hip : bf16 MFMA weight gradient of 3x3 windows (any stride), one 32 x 32 channel pair x 9 taps per
// workgroup; same outputs as launch_wgrad_tile (fp32 dw' copies [splits][Cout][taps][Cin], r_part [splits][Cout]).
bool wgrad_sq_supported(const Geom& g, int dtype);
int wgrad_sq_splits(const Geom& g);
hipError_t launch_wgrad_sq(const Geom& g, const void* x, const void* dz, float* dwf_part, float* r_part,
                           hipStream_t st);
// Input gradient and weight gradient (fp32 copies as launch_wgrad_sq writes them) of a block in one launch, where the
// resident-weight convolution takes the input gradient.
bool wgrad_dgrad_pair_supported(const Geom& g, int dtype);
hipError_t launch_wgrad_dgrad_pair(const Geom& g, const void* x, const void* dz, const void* w_crsk, void* dx,
                                   float* dwf_part, float* r_part, hipStream_t st);
// Weight gradient and fold-back in one launch, for problems whose pixels need no split (deep layers): writes dW,
// dgamma, dbeta and (b given) db directly; no fp32 copy of dw' is stored.  scratch: wgrad_sq_fused_scratch_bytes().
// w_folded_out (optional): the launch also leaves w' = s w there as [Cin][taps][Cout], for an input gradient that
// runs after it.
bool wgrad_sq_fused_supported(const Geom& g, int dtype);
size_t wgrad_sq_fused_scratch_bytes(const Geom& g);
hipError_t launch_wgrad_sq_fused(const Geom& g, const void* x, const void* dz, const void* W, const float* b,
                                 const float* gamma, const float* mean, const float* var, void* dW, float* db,
                                 float* dgamma, float* dbeta, void* scratch, void* w_folded_out, hipStream_t st);

}  // namespace convbn
