// C ABI of libconvbn: argument validation, workspace carving and the launch sequences
// of the Tune-mode block (Sec. 3.3-3.4, Table 2 "Tune") and of the Eval-mode comparison
// block (Sec. 3.1, Table 2 "Eval").  Host code only enqueues; nothing here synchronises.
#include <stdarg.h>
#include <stdio.h>

#include <mutex>

#include "common.h"

using namespace convbn;

namespace {

thread_local char g_err[256] = "no error";

convbn_status fail(convbn_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int out_size(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

struct WgradWay;
WgradWay wgrad_way(const Geom& g, int dtype);
bool needs_cin_pad(const Geom& g, int dtype);
Geom padded_geom(const Geom& g);
long long widest_partial_elems(const Geom& g, int dtype);

// Fills `g`; returns CONVBN_OK or the reason the descriptor is not usable.
convbn_status make_geom(const convbn_desc* d, Geom* g) {
  if (!d) return fail(CONVBN_ERR_NULL, "descriptor is NULL");
  if (d->N < 1 || d->Cin < 1 || d->Hin < 1 || d->Win < 1 || d->Cout < 1 || d->kH < 1 || d->kW < 1)
    return fail(CONVBN_ERR_SHAPE, "non-positive dimension in descriptor");
  if (d->stride_h < 1 || d->stride_w < 1) return fail(CONVBN_ERR_SHAPE, "stride must be >= 1");
  if (d->pad_h < 0 || d->pad_w < 0) return fail(CONVBN_ERR_SHAPE, "padding must be >= 0");
  if (d->Hin + 2 * d->pad_h < d->kH || d->Win + 2 * d->pad_w < d->kW)
    return fail(CONVBN_ERR_SHAPE, "kernel larger than the padded input (empty output)");
  if (d->dtype != CONVBN_F32 && d->dtype != CONVBN_BF16)
    return fail(CONVBN_ERR_UNSUPPORTED, "dtype %d is not CONVBN_F32 or CONVBN_BF16", d->dtype);
  if (d->layout != CONVBN_LAYOUT_NHWC)
    return fail(CONVBN_ERR_UNSUPPORTED, "layout %d: only CONVBN_LAYOUT_NHWC is supported", d->layout);
  if (!(d->eps >= 0.f)) return fail(CONVBN_ERR_SHAPE, "eps must be >= 0");
  if (d->act < 0 || d->act > (CONVBN_ACT_RELU_OUT | CONVBN_ACT_RELU_IN | CONVBN_ACT_ADD_OUT | CONVBN_ACT_ADD_IN))
    return fail(CONVBN_ERR_UNSUPPORTED, "act %d: unknown activation bits", d->act);
  if (((d->act & CONVBN_ACT_ADD_OUT) && !d->add_out) || ((d->act & CONVBN_ACT_ADD_IN) && !d->add_in))
    return fail(CONVBN_ERR_NULL, "act %d asks for an addend that the descriptor does not give", d->act);
  g->act = d->act; g->post_relu = 0; g->post_mask = nullptr; g->post_add = nullptr;
  g->add_out = (d->act & CONVBN_ACT_ADD_OUT) ? d->add_out : nullptr;
  g->add_in = (d->act & CONVBN_ACT_ADD_IN) ? d->add_in : nullptr;
  g->N = d->N; g->Cin = d->Cin; g->Hin = d->Hin; g->Win = d->Win;
  g->Cout = d->Cout; g->kH = d->kH; g->kW = d->kW;
  g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
  g->Hout = out_size(d->Hin, d->kH, d->stride_h, d->pad_h);
  g->Wout = out_size(d->Win, d->kW, d->stride_w, d->pad_w);
  g->eps = d->eps;
  const long long lim = 0x7fffffffLL;
  const long long ax = (long long)d->N * d->Hin * d->Win * d->Cin;
  const long long az = (long long)d->N * g->Hout * g->Wout * d->Cout;
  const long long pp = (long long)d->Cout * d->kH * d->kW * d->Cin;
  if (ax > lim || az > lim || pp > lim)
    return fail(CONVBN_ERR_UNSUPPORTED, "a tensor has more than 2^31-1 elements");
  g->M = d->N * g->Hout * g->Wout;
  g->Min = d->N * d->Hin * d->Win;
  g->K = d->kH * d->kW * d->Cin;
  // the kernels index the fp32 partial copies of split sums with 32 bits as well
  if (widest_partial_elems(*g, d->dtype) > lim)
    return fail(CONVBN_ERR_UNSUPPORTED, "a buffer of partial sums would have more than 2^31-1 elements");
  return CONVBN_OK;
}

size_t esize(int dtype) { return dtype == CONVBN_BF16 ? 2 : 4; }

// How the weight-gradient step of a problem runs: number of fp32 partial copies of dw', number of
// partial r vectors, and whether the weight-gradient kernel produces r itself.
// bf16 problems whose input-channel count is not a multiple of 8 (a network's first layer: 3
// channels) run the MFMA kernels on copies padded with zero channels; the copies live in scratch.
bool needs_cin_pad(const Geom& g, int dtype) {
  return dtype == CONVBN_BF16 && g.Cin % 8 != 0 && g.Cout % 8 == 0;
}
Geom padded_geom(const Geom& g) {
  Geom q = g;
  q.Cin = (g.Cin + 7) / 8 * 8;
  q.K = g.kH * g.kW * q.Cin;
  return q;
}

struct WgradWay { int nsplit; int nrpart; bool fused_r; bool sq = false; };
WgradWay wgrad_way(const Geom& g0, int dtype) {
  if (needs_cin_pad(g0, dtype) && stem_wgrad_supported(g0, dtype)) {   // a first layer: its own kernel
    const int s = stem_wgrad_slices(g0);
    return {s, s, true};
  }
  const Geom g = needs_cin_pad(g0, dtype) ? padded_geom(g0) : g0;
  if (wgrad_sq_supported(g, dtype)) {
    const int s = wgrad_sq_splits(g);
    return {s, s, true, true};
  }
  if (wgrad_tile_supported(g, dtype)) {
    const int s = wgrad_tile_splits(g);
    return {s, s, true};
  }
  return {igemm_supported(g, dtype) ? wgrad_splits(g) : wgrad_direct_splits(g), colsum_parts(g), false};
}
int nsplit_for(const Geom& g, int dtype) { return wgrad_way(g, dtype).nsplit; }

size_t inner_fprop_scratch(const Geom& g, int dtype);
size_t inner_dgrad_scratch(const Geom& g, int dtype);
// Elements of the largest fp32 buffer of partial sums a problem's kernels would write: the split copies of dw' and
// the partial outputs of convolutions whose reduced channels are divided over workgroups.  Only problems large
// enough to come near the limit are planned here (every split count is far below 1024, every channel split below 64).
long long widest_partial_elems(const Geom& g0, int dtype) {
  const long long lim = 0x7fffffffLL;
  const long long pp = (long long)g0.Cout * g0.kH * g0.kW * ((g0.Cin + 7) / 8 * 8);
  const long long act = (long long)(g0.M > g0.Min ? g0.M : g0.Min) * (g0.Cout > g0.Cin ? g0.Cout : g0.Cin);
  if (pp <= lim / 1024 && act <= lim / 64) return 0;
  const Geom g = needs_cin_pad(g0, dtype) ? padded_geom(g0) : g0;
  long long widest = (long long)wgrad_way(g0, dtype).nsplit * g.Cout * g.K;
  const long long conv = (long long)((inner_fprop_scratch(g, dtype) > inner_dgrad_scratch(g, dtype)
                                          ? inner_fprop_scratch(g, dtype) : inner_dgrad_scratch(g, dtype)) / 4);
  return widest > conv ? widest : conv;
}

size_t fprop_scratch_bytes(const Geom& g, int dtype);
size_t dgrad_scratch_bytes(const Geom& g, int dtype);
size_t wgrad_scratch_bytes(const Geom& g, int dtype);

// Workspace carving.  Every section starts on a 256-byte boundary.
struct Carve {
  char* base;
  size_t off = 0;
  explicit Carve(void* p) : base(static_cast<char*>(p)) {}
  void* take(size_t bytes) {
    void* r = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return r;
  }
};

struct TuneFwdWs { void* w_krsc; float* bfold; float* conv_scratch; size_t bytes; };
TuneFwdWs carve_tune_fwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  TuneFwdWs r;
  r.w_krsc = c.take((size_t)g.Cout * g.K * esize(dtype));
  r.bfold = (float*)c.take((size_t)g.Cout * 4);
  r.conv_scratch = (float*)c.take(fprop_scratch_bytes(g, dtype));
  r.bytes = c.off;
  return r;
}

// Eval forward needs only the convolution's own scratch.
struct EvalFwdWs { float* conv_scratch; size_t bytes; };
EvalFwdWs carve_eval_fwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  EvalFwdWs r;
  r.conv_scratch = (float*)c.take(fprop_scratch_bytes(g, dtype));
  r.bytes = c.off;
  return r;
}

struct TuneBwdWs { void* w_crsk; float* dwf_part; float* r_part; float* conv_scratch; void* wgrad_scratch; int nsplit; int nrpart; size_t bytes; };
TuneBwdWs carve_tune_bwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  TuneBwdWs r;
  const WgradWay way = wgrad_way(g, dtype);
  r.nsplit = way.nsplit;
  r.nrpart = way.nrpart;
  r.w_crsk = c.take((size_t)g.Cout * g.K * esize(dtype));
  r.dwf_part = (float*)c.take((size_t)r.nsplit * g.Cout * g.K * 4);
  r.r_part = (float*)c.take((size_t)r.nrpart * g.Cout * 4);
  r.conv_scratch = (float*)c.take(dgrad_scratch_bytes(g, dtype));
  r.wgrad_scratch = c.take(wgrad_scratch_bytes(g, dtype));
  r.bytes = c.off;
  return r;
}

struct EvalBwdWs { void* dy; void* w_crsk; float* dwf_part; float* bn_part; float* conv_scratch; void* wgrad_scratch; int nsplit; int nparts; size_t bytes; };
EvalBwdWs carve_eval_bwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  EvalBwdWs r;
  r.nsplit = nsplit_for(g, dtype);
  r.nparts = bn_bwd_parts(g);
  r.dy = c.take((size_t)g.M * g.Cout * esize(dtype));
  r.w_crsk = c.take((size_t)g.Cout * g.K * esize(dtype));
  r.dwf_part = (float*)c.take((size_t)r.nsplit * g.Cout * g.K * 4);
  r.bn_part = (float*)c.take((size_t)r.nparts * 2 * g.Cout * 4);
  r.conv_scratch = (float*)c.take(dgrad_scratch_bytes(g, dtype));
  r.wgrad_scratch = c.take(wgrad_scratch_bytes(g, dtype));
  r.bytes = c.off;
  return r;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

#define REQUIRE_PTR(p)                                                            \
  do {                                                                            \
    if (!(p)) return fail(CONVBN_ERR_NULL, "required pointer '%s' is NULL", #p);   \
    if (misaligned(p))                                                            \
      return fail(CONVBN_ERR_UNSUPPORTED, "pointer '%s' is not 16-byte aligned", #p); \
  } while (0)
#define OPTIONAL_PTR(p)                                                           \
  do {                                                                            \
    if ((p) && misaligned(p))                                                     \
      return fail(CONVBN_ERR_UNSUPPORTED, "pointer '%s' is not 16-byte aligned", #p); \
  } while (0)
#define LAUNCH(expr)                                                              \
  do {                                                                            \
    hipError_t e_ = (expr);                                                       \
    if (e_ != hipSuccess)                                                         \
      return fail(CONVBN_ERR_LAUNCH, "%s: %s", #expr, hipGetErrorString(e_));      \
  } while (0)

convbn_status check_ws(size_t need, void* ws, size_t ws_bytes) {
  if (need == 0) return CONVBN_OK;
  if (!ws) return fail(CONVBN_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
  if (misaligned(ws)) return fail(CONVBN_ERR_UNSUPPORTED, "workspace is not 16-byte aligned");
  if (ws_bytes < need)
    return fail(CONVBN_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
  return CONVBN_OK;
}

// Scratch the three convolutions of a problem need (0 for most): fp32 partial outputs when the
// reduced channels are split over workgroups, and the zero-padded copies of needs_cin_pad().
size_t inner_fprop_scratch(const Geom& g, int dtype) {
  if (pw_fprop_supported(g, dtype) || rw_fprop_supported(g, dtype) || st_fprop_supported(g, dtype)) return 0;
  return tile_fprop_supported(g, dtype) ? align_up(tile_fprop_partial_bytes(g), 256) : 0;
}
size_t inner_dgrad_scratch(const Geom& g, int dtype) {
  if (pw_dgrad_supported(g, dtype) || rw_dgrad_supported(g, dtype) || st_dgrad_supported(g, dtype)) return 0;
  return tile_dgrad_supported(g, dtype) ? align_up(tile_dgrad_partial_bytes(g), 256) : 0;
}
size_t fprop_scratch_bytes(const Geom& g, int dtype) {
  if (!needs_cin_pad(g, dtype)) return inner_fprop_scratch(g, dtype);
  if (stem_fprop_supported(g, dtype))
    return align_up(stem_packed_weight_bytes(g), 256) + align_up(stem_input_copy_bytes(g), 256);
  const Geom q = padded_geom(g);
  return align_up((size_t)q.Min * q.Cin * 2, 256) + align_up((size_t)q.Cout * q.K * 2, 256) +
         inner_fprop_scratch(q, dtype);
}
size_t dgrad_scratch_bytes(const Geom& g, int dtype) {
  if (!needs_cin_pad(g, dtype)) return inner_dgrad_scratch(g, dtype);
  if (stem_dgrad_supported(g, dtype)) return align_up(stem_dgrad_weight_bytes(g), 256);
  const Geom q = padded_geom(g);
  return align_up((size_t)q.Cout * q.K * 2, 256) + align_up((size_t)q.Min * q.Cin * 2, 256) +
         inner_dgrad_scratch(q, dtype);
}
size_t wgrad_scratch_bytes(const Geom& g, int dtype) {
  if (!needs_cin_pad(g, dtype)) return 0;
  if (stem_wgrad_supported(g, dtype)) return align_up(stem_input_copy_bytes(g), 256);
  const Geom q = padded_geom(g);
  return align_up((size_t)q.Min * q.Cin * 2, 256) +
         align_up((size_t)wgrad_way(g, dtype).nsplit * q.Cout * q.K * 4, 256);
}

// The post-operation of g (addend, ReLU, mask) as passes of their own over `out` (n elements): for the kernels that
// do not apply it in their epilogue.
hipError_t post_op_pass(const Geom& g, int dtype, void* out, size_t n, hipStream_t st) {
  if (g.post_add) {
    hipError_t e = launch_eltwise(3 /* a + b */, dtype, out, g.post_add, nullptr, n, st);
    if (e != hipSuccess) return e;
  }
  if (g.post_relu) {
    hipError_t e = launch_eltwise(0 /* max(a, 0) */, dtype, out, nullptr, nullptr, n, st);
    if (e != hipSuccess) return e;
  }
  if (g.post_mask) return launch_eltwise(1 /* b > 0 ? a : 0 */, dtype, out, g.post_mask, nullptr, n, st);
  return hipSuccess;
}
bool has_post_op(const Geom& g) { return g.post_relu || g.post_mask || g.post_add; }

// FUSED_*: the kernel applies g's post-operation itself.
constexpr bool FUSED_PW = true, FUSED_RW = true, FUSED_ST = true, FUSED_TILE = true;

hipError_t fprop_any(const Geom& g, int dtype, const void* x, const void* w_krsc, const float* bias,
                     void* z, float* scratch, hipStream_t st) {
  hipError_t e;
  bool fused = false;
  if (pw_fprop_supported(g, dtype)) { e = launch_fprop_pw(g, x, w_krsc, bias, z, st); fused = FUSED_PW; }
  else if (rw_fprop_supported(g, dtype)) { e = launch_fprop_rw(g, x, w_krsc, bias, z, st); fused = FUSED_RW; }
  else if (st_fprop_supported(g, dtype)) { e = launch_fprop_st(g, x, w_krsc, bias, z, st); fused = FUSED_ST; }
  else if (tile_fprop_supported(g, dtype)) { e = launch_fprop_tile(g, x, w_krsc, bias, z, scratch, st); fused = FUSED_TILE; }
  else e = igemm_supported(g, dtype) ? launch_fprop_igemm(g, x, w_krsc, bias, z, st)
                                     : launch_fprop_direct(g, dtype, x, w_krsc, bias, z, st);
  if (e != hipSuccess || fused || !has_post_op(g)) return e;
  return post_op_pass(g, dtype, z, (size_t)g.M * g.Cout, st);
}
hipError_t dgrad_any(const Geom& g, int dtype, const void* dz, const void* w_crsk, const float* bias, void* dx,
                     float* scratch, hipStream_t st) {
  hipError_t e;
  bool fused = false;
  if (pw_dgrad_supported(g, dtype)) { e = launch_dgrad_pw(g, dz, w_crsk, bias, dx, st); fused = FUSED_PW; }
  else if (rw_dgrad_supported(g, dtype)) { e = launch_dgrad_rw(g, dz, w_crsk, bias, dx, st); fused = FUSED_RW; }
  else if (st_dgrad_supported(g, dtype)) { e = launch_dgrad_st(g, dz, w_crsk, bias, dx, st); fused = FUSED_ST; }
  else if (tile_dgrad_supported(g, dtype)) { e = launch_dgrad_tile(g, dz, w_crsk, bias, dx, scratch, st); fused = FUSED_TILE; }
  else e = igemm_supported(g, dtype) ? launch_dgrad_igemm(g, dz, w_crsk, bias, dx, st)
                                     : launch_dgrad_direct(g, dtype, dz, w_crsk, bias, dx, st);
  if (e != hipSuccess || fused || !has_post_op(g)) return e;
  return post_op_pass(g, dtype, dx, (size_t)g.Min * g.Cin, st);
}

#define TRY(expr)                       \
  do {                                  \
    hipError_t e_ = (expr);             \
    if (e_ != hipSuccess) return e_;    \
  } while (0)

hipError_t run_fprop(const Geom& g, int dtype, const void* x, const void* w_krsc, const float* bias,
                     void* z, float* scratch, hipStream_t st) {
  if (!needs_cin_pad(g, dtype)) return fprop_any(g, dtype, x, w_krsc, bias, z, scratch, st);
  if (stem_fprop_supported(g, dtype)) {   // a first layer: its own kernel; the scratch holds the padded weight
    char* sp = reinterpret_cast<char*>(scratch);
    void* wpad = sp;
    sp += align_up(stem_packed_weight_bytes(g), 256);
    if (stem_input_copy_bytes(g) == 0) {
      TRY(launch_fprop_stem(g, x, w_krsc, wpad, bias, z, st));
    } else {
      TRY(launch_repitch(2, (size_t)g.Min, g.Cin, 4, x, sp, st));   // ... and a 4-channel copy of the input
      TRY(launch_fprop_stem(g, sp, w_krsc, wpad, bias, z, st));
    }
    return post_op_pass(g, dtype, z, (size_t)g.M * g.Cout, st);
  }
  const Geom q = padded_geom(g);
  char* s = reinterpret_cast<char*>(scratch);
  void* xp = s; s += align_up((size_t)q.Min * q.Cin * 2, 256);
  void* wp = s; s += align_up((size_t)q.Cout * q.K * 2, 256);
  TRY(launch_repitch(2, (size_t)g.Min, g.Cin, q.Cin, x, xp, st));
  TRY(launch_repitch(2, (size_t)g.Cout * g.kH * g.kW, g.Cin, q.Cin, w_krsc, wp, st));
  return fprop_any(q, dtype, xp, wp, bias, z, reinterpret_cast<float*>(s), st);
}
hipError_t run_dgrad(const Geom& g, int dtype, const void* dz, const void* w_crsk, void* dx,
                     float* scratch, hipStream_t st) {
  if (!needs_cin_pad(g, dtype)) return dgrad_any(g, dtype, dz, w_crsk, nullptr, dx, scratch, st);
  if (stem_dgrad_supported(g, dtype)) {   // a first layer: its own kernel; the scratch holds its packed weight
    TRY(launch_dgrad_stem(g, dz, w_crsk, scratch, dx, st));
    return post_op_pass(g, dtype, dx, (size_t)g.Min * g.Cin, st);
  }
  Geom q = padded_geom(g);
  q.post_relu = 0; q.post_mask = nullptr; q.post_add = nullptr;   // mask and addend are laid out like dx, not like its padded copy: applied at the end
  char* s = reinterpret_cast<char*>(scratch);
  void* wp = s; s += align_up((size_t)q.Cout * q.K * 2, 256);
  void* dxp = s; s += align_up((size_t)q.Min * q.Cin * 2, 256);
  // [Cin][taps*Cout] -> [Cin_p][taps*Cout]: the extra rows are zero
  const size_t row = (size_t)g.kH * g.kW * g.Cout;
  TRY(launch_repitch(2, 1, (size_t)g.Cin * row, (size_t)q.Cin * row, w_crsk, wp, st));
  TRY(dgrad_any(q, dtype, dz, wp, nullptr, dxp, reinterpret_cast<float*>(s), st));
  TRY(launch_repitch(2, (size_t)g.Min, q.Cin, g.Cin, dxp, dx, st));
  return post_op_pass(g, dtype, dx, (size_t)g.Min * g.Cin, st);
}
// dw' partials and, when r_part != nullptr, the partial per-channel sums of dz.
hipError_t wgrad_any(const Geom& g, int dtype, const void* x, const void* dz, float* part, float* r_part,
                     const WgradWay& way, hipStream_t st) {
  if (way.sq) return launch_wgrad_sq(g, x, dz, part, r_part, st);
  if (way.fused_r) return launch_wgrad_tile(g, x, dz, part, r_part, st);
  hipError_t e = igemm_supported(g, dtype) ? launch_wgrad_igemm(g, x, dz, part, way.nsplit, st)
                                           : launch_wgrad_direct(g, dtype, x, dz, part, st);
  if (e != hipSuccess || !r_part) return e;
  return launch_colsum(g, dtype, dz, r_part, st);
}
hipError_t run_wgrad(const Geom& g, int dtype, const void* x, const void* dz, float* part, float* r_part,
                     void* scratch, hipStream_t st) {
  const WgradWay way = wgrad_way(g, dtype);
  if (!needs_cin_pad(g, dtype)) return wgrad_any(g, dtype, x, dz, part, r_part, way, st);
  if (stem_wgrad_supported(g, dtype)) {
    if (stem_input_copy_bytes(g) == 0) return launch_wgrad_stem(g, x, dz, part, r_part, st);
    TRY(launch_repitch(2, (size_t)g.Min, g.Cin, 4, x, scratch, st));   // a 4-channel copy of the input
    return launch_wgrad_stem(g, scratch, dz, part, r_part, st);
  }
  const Geom q = padded_geom(g);
  char* s = reinterpret_cast<char*>(scratch);
  void* xp = s; s += align_up((size_t)q.Min * q.Cin * 2, 256);
  float* pp = reinterpret_cast<float*>(s);
  TRY(launch_repitch(2, (size_t)g.Min, g.Cin, q.Cin, x, xp, st));
  TRY(wgrad_any(q, dtype, xp, dz, pp, r_part, way, st));
  return launch_repitch(4, (size_t)way.nsplit * g.Cout * g.kH * g.kW, q.Cin, g.Cin, pp, part, st);
}

// ---- TransposedConv-BN block (Sec. 3.2.1) ----------------------------------------------------------
// A transposed convolution is the adjoint of a convolution with the same window, stride and padding that
// maps the block's OUTPUT (Cout channels, Hout x Wout) back to its input.  `g` is that convolution: the
// block's forward pass is its input-gradient kernel, the block's input gradient its forward kernel, and
// the weight gradient is its weight gradient with the two feature maps exchanged.
convbn_status make_tgeom(const convbn_desc* d, Geom* g) {
  if (!d) return fail(CONVBN_ERR_NULL, "descriptor is NULL");
  if (d->N < 1 || d->Cin < 1 || d->Hin < 1 || d->Win < 1 || d->Cout < 1 || d->kH < 1 || d->kW < 1)
    return fail(CONVBN_ERR_SHAPE, "non-positive dimension in descriptor");
  if (d->stride_h < 1 || d->stride_w < 1) return fail(CONVBN_ERR_SHAPE, "stride must be >= 1");
  if (d->pad_h < 0 || d->pad_w < 0) return fail(CONVBN_ERR_SHAPE, "padding must be >= 0");
  const long long ho = (long long)(d->Hin - 1) * d->stride_h - 2LL * d->pad_h + d->kH;
  const long long wo = (long long)(d->Win - 1) * d->stride_w - 2LL * d->pad_w + d->kW;
  if (ho < 1 || wo < 1) return fail(CONVBN_ERR_SHAPE, "padding removes the whole output of the transposed convolution");
  if (ho > 0x7fffffffLL || wo > 0x7fffffffLL) return fail(CONVBN_ERR_UNSUPPORTED, "output size overflows");
  convbn_desc c = *d;
  c.Cin = d->Cout; c.Cout = d->Cin; c.Hin = (int32_t)ho; c.Win = (int32_t)wo;
  const convbn_status s = make_geom(&c, g);
  if (s != CONVBN_OK) return s;
  if (g->Hout != d->Hin || g->Wout != d->Win) return fail(CONVBN_ERR_SHAPE, "inconsistent transposed geometry");
  return CONVBN_OK;
}
// the block's output seen as rows of Cout channels (for the per-channel sums of dZ)
Geom tconv_out_rows(const Geom& g) {
  Geom r = g;
  r.M = g.Min;
  r.Cout = g.Cin;
  return r;
}
// bf16 blocks whose output-channel count is not a multiple of 8 run the forward pass on the any-shape kernel
bool tconv_fwd_direct(const Geom& g, int dtype) { return needs_cin_pad(g, dtype); }

struct TconvFwdWs { void* w_swap; float* bfold; float* conv_scratch; size_t bytes; };
TconvFwdWs carve_tconv_fwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  TconvFwdWs r;
  r.w_swap = c.take((size_t)g.Cout * g.K * esize(dtype));
  r.bfold = (float*)c.take((size_t)g.Cin * g.kH * g.kW * 4);   // room for one copy per tap (the single-product forward)
  r.conv_scratch = (float*)c.take(tconv_fwd_direct(g, dtype) ? 0 : inner_dgrad_scratch(g, dtype));
  r.bytes = c.off;
  return r;
}
struct TconvBwdWs { void* w_same; float* dwf_part; float* r_part; float* dot_part; float* conv_scratch; void* wgrad_scratch; int nsplit; int nrpart; size_t bytes; };
TconvBwdWs carve_tconv_bwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  TconvBwdWs r;
  r.nsplit = nsplit_for(g, dtype);
  r.nrpart = colsum_parts(tconv_out_rows(g));
  r.w_same = c.take((size_t)g.Cout * g.K * esize(dtype));
  r.dwf_part = (float*)c.take((size_t)r.nsplit * g.Cout * g.K * 4);
  r.r_part = (float*)c.take((size_t)r.nrpart * g.Cin * 4);
  r.dot_part = (float*)c.take((size_t)fold_back_t_chunks(g.Cout, g.kH * g.kW) * g.Cin * 4);
  r.conv_scratch = (float*)c.take(fprop_scratch_bytes(g, dtype));
  r.wgrad_scratch = c.take(wgrad_scratch_bytes(g, dtype));
  r.bytes = c.off;
  return r;
}

// Eval comparison path of the transposed block: Y kept, separate affine; backward through dY
struct TconvEvalBwdWs { void* dy; float* dwf_part; float* bn_part; float* conv_scratch; void* wgrad_scratch; int nsplit; int nparts; size_t bytes; };
TconvEvalBwdWs carve_tconv_eval_bwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  TconvEvalBwdWs r;
  r.nsplit = nsplit_for(g, dtype);
  r.nparts = bn_bwd_parts(tconv_out_rows(g));
  r.dy = c.take((size_t)g.Min * g.Cin * esize(dtype));
  r.dwf_part = (float*)c.take((size_t)r.nsplit * g.Cout * g.K * 4);
  r.bn_part = (float*)c.take((size_t)r.nparts * 2 * g.Cin * 4);
  r.conv_scratch = (float*)c.take(fprop_scratch_bytes(g, dtype));
  r.wgrad_scratch = c.take(wgrad_scratch_bytes(g, dtype));
  r.bytes = c.off;
  return r;
}

// ---- depthwise block -----------------------------------------------------------------------------------
convbn_status make_dwgeom(const convbn_desc* d, Geom* g) {
  const convbn_status s = make_geom(d, g);
  if (s != CONVBN_OK) return s;
  if (d->Cin != d->Cout) return fail(CONVBN_ERR_SHAPE, "a depthwise block has Cin == Cout (one filter per channel)");
  return CONVBN_OK;
}
struct DwFwdWs { void* wf; float* bfold; size_t bytes; };
DwFwdWs carve_dw_fwd(const Geom& g, int dtype, void* ws) {
  Carve c(ws);
  DwFwdWs r;
  r.wf = c.take((size_t)g.kH * g.kW * g.Cin * esize(dtype));
  r.bfold = (float*)c.take((size_t)g.Cin * 4);
  r.bytes = c.off;
  return r;
}
struct DwBwdWs { void* wf; void* dy; float* part; float* r_part; float* sums; float* bn_part; int slices; int nparts; size_t bytes; };
DwBwdWs carve_dw_bwd(const Geom& g, int dtype, int mode, void* ws) {
  Carve c(ws);
  DwBwdWs r;
  const int taps = g.kH * g.kW;
  r.slices = dw_wgrad_slices(g, dtype);
  r.nparts = bn_bwd_parts(g);
  r.wf = c.take((size_t)taps * g.Cin * esize(dtype));
  r.part = (float*)c.take((size_t)r.slices * taps * g.Cin * 4);
  r.r_part = (float*)c.take((size_t)r.slices * g.Cin * 4);
  r.sums = (float*)c.take((size_t)(taps + 1) * g.Cin * 4);
  r.dy = nullptr; r.bn_part = nullptr;
  if (mode == CONVBN_MODE_EVAL) {
    r.dy = c.take((size_t)g.M * g.Cout * esize(dtype));
    r.bn_part = (float*)c.take((size_t)r.nparts * 2 * g.Cout * 4);
  }
  r.bytes = c.off;
  return r;
}

// ---- grouped block -------------------------------------------------------------------------------------
convbn_status make_ggeom(const convbn_desc* d, int groups, Geom* g, Geom* gf) {
  const convbn_status s = make_geom(d, g);
  if (s != CONVBN_OK) return s;
  if (groups < 1 || d->Cin % groups != 0 || d->Cout % groups != 0)
    return fail(CONVBN_ERR_SHAPE, "groups = %d must be >= 1 and divide Cin and Cout", groups);
  // the weight as the fold and the fold-back see it: a [Cout][kH kW cg] matrix
  *gf = *g;
  gf->Cin = d->Cin / groups;
  gf->K = d->kH * d->kW * gf->Cin;
  return CONVBN_OK;
}
// The two limits of the grouped block have calls of their own with the same buffer layouts (W [Cout][kH][kW][cg] with
// cg = Cin is the dense weight, with cg = 1 the depthwise filter [C][kH][kW]; likewise w_folded): the grouped entry
// points pass them on, so that the limits run on those blocks' kernels.
enum GroupedRoute { G_ROUTE_GROUPED, G_ROUTE_DENSE, G_ROUTE_DEPTHWISE };
GroupedRoute grouped_route(const convbn_desc* d, int groups) {
  if (groups == 1) return G_ROUTE_DENSE;
  if (groups == d->Cin && d->Cin == d->Cout) return G_ROUTE_DEPTHWISE;
  return G_ROUTE_GROUPED;
}
struct GFwdWs { void* w_krsc; float* bfold; size_t bytes; };
GFwdWs carve_g_fwd(const Geom& gf, int dtype, void* ws) {
  Carve c(ws);
  GFwdWs r;
  r.w_krsc = c.take((size_t)gf.Cout * gf.K * esize(dtype));
  r.bfold = (float*)c.take((size_t)gf.Cout * 4);
  r.bytes = c.off;
  return r;
}
struct GBwdWs { void* w_crsk; void* dy; float* part; float* r_part; float* bn_part; int slices; int nrpart; int nparts; size_t bytes; };
GBwdWs carve_g_bwd(const Geom& g, const Geom& gf, int groups, int dtype, int mode, void* ws) {
  Carve c(ws);
  GBwdWs r;
  r.slices = g_wgrad_slices(g, groups, dtype);
  r.nrpart = g_wgrad_makes_rsum(g, groups, dtype) ? r.slices : colsum_parts(g);
  r.nparts = bn_bwd_parts(g);
  r.w_crsk = c.take((size_t)gf.Cout * gf.K * esize(dtype));
  r.part = (float*)c.take((size_t)r.slices * gf.Cout * gf.K * 4);
  r.r_part = (float*)c.take((size_t)r.nrpart * g.Cout * 4);
  r.dy = nullptr; r.bn_part = nullptr;
  if (mode == CONVBN_MODE_EVAL) {
    r.dy = c.take((size_t)g.M * g.Cout * esize(dtype));
    r.bn_part = (float*)c.take((size_t)r.nparts * 2 * g.Cout * 4);
  }
  r.bytes = c.off;
  return r;
}

}  // namespace

extern "C" {

int32_t convbn_hout(const convbn_desc* desc) {
  Geom g;
  return make_geom(desc, &g) == CONVBN_OK ? g.Hout : 0;
}

int32_t convbn_wout(const convbn_desc* desc) {
  Geom g;
  return make_geom(desc, &g) == CONVBN_OK ? g.Wout : 0;
}

size_t convbn_workspace_bytes(const convbn_desc* desc, int mode, int pass) {
  Geom g;
  if (make_geom(desc, &g) != CONVBN_OK) return 0;
  if (mode == CONVBN_MODE_TUNE)
    return pass == CONVBN_PASS_FWD ? carve_tune_fwd(g, desc->dtype, nullptr).bytes
                                   : carve_tune_bwd(g, desc->dtype, nullptr).bytes;
  if (mode == CONVBN_MODE_EVAL)
    return pass == CONVBN_PASS_FWD ? carve_eval_fwd(g, desc->dtype, nullptr).bytes
                                   : carve_eval_bwd(g, desc->dtype, nullptr).bytes;
  return 0;
}

size_t convbn_saved_bytes(const convbn_desc* desc, int mode, int refold) {
  Geom g;
  if (make_geom(desc, &g) != CONVBN_OK) return 0;
  if (mode == CONVBN_MODE_EVAL) return (size_t)g.M * g.Cout * esize(desc->dtype);
  return refold ? 0 : (size_t)g.Cout * g.K * esize(desc->dtype);
}

const char* convbn_last_error(void) { return g_err; }

// ---- Tune forward for callers that cannot allocate ---------------------------------------------------
// The forward workspace (w' in the forward order, b', split sums) lives in a file-scope device array.  Every
// GPU the library runs on holds its own copy of the array at its own address; the address is looked up once
// per device, with that device current, and kept.  Host code never passes the array's name to a kernel.
#define CONVBN_STATIC_WS_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[CONVBN_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call per device).
convbn_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(CONVBN_ERR_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(CONVBN_ERR_UNSUPPORTED, "device index %d is not below %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(CONVBN_ERR_LAUNCH, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CONVBN_OK;
}
}  // namespace

size_t convbn_static_workspace_limit(void) { return CONVBN_STATIC_WS_BYTES; }

convbn_status convbn_tune_fwd_static(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                     const float* gamma, const float* beta, const float* mean, const float* var,
                                     void* z, void* w_folded, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  const size_t need = carve_tune_fwd(g, desc->dtype, nullptr).bytes;
  if (need > CONVBN_STATIC_WS_BYTES)
    return fail(CONVBN_ERR_WORKSPACE, "this block needs %zu workspace bytes, the built-in buffer has %u: use convbn_tune_fwd",
                need, CONVBN_STATIC_WS_BYTES);
  void* ptr = nullptr;
  s = static_scratch(&ptr);
  if (s != CONVBN_OK) return s;
  // nothing in the forward workspace has to start at zero: every byte a kernel reads is written first by this call
  return convbn_tune_fwd(desc, x, W, b, gamma, beta, mean, var, z, w_folded, ptr, CONVBN_STATIC_WS_BYTES, stream);
}

convbn_status convbn_tune_fwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                              const float* gamma, const float* beta, const float* mean,
                              const float* var, void* z, void* w_folded, void* ws, size_t ws_bytes,
                              void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded);
  const int dt = desc->dtype;
  s = check_ws(carve_tune_fwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const TuneFwdWs w = carve_tune_fwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  g.post_relu = g.act & CONVBN_ACT_RELU_OUT; g.post_add = g.add_out;
  const size_t nz = (size_t)g.M * g.Cout;
  if (!needs_cin_pad(g, dt) && !pw_fprop_supported(g, dt) && (g.kH > 1 || g.kW > 1)) {
    // The scale is per output channel, so Z = s (w (*) X) + b' (Sec. 3.3): the convolution reads the unfolded
    // weight and applies s and b' in its epilogue, and -- where w' is kept for backward -- its workgroups each
    // write a slice of w' on the side.  The forward pass is one launch; no w' is materialised for it.
    const BnEpilogue bn{gamma, beta, mean, var, b, g.eps, w_folded, g.kH * g.kW, g.Cin, g.Cout};
    if (rw_fprop_supported(g, dt)) {
      LAUNCH(launch_fprop_rw(g, x, W, nullptr, z, st, &bn));
      if (!FUSED_RW) LAUNCH(post_op_pass(g, dt, z, nz, st));
      return CONVBN_OK;
    }
    if (st_fprop_supported(g, dt)) {
      LAUNCH(launch_fprop_st(g, x, W, nullptr, z, st, &bn));
      if (!FUSED_ST) LAUNCH(post_op_pass(g, dt, z, nz, st));
      return CONVBN_OK;
    }
    if (tile_fprop_scaled_supported(g, dt)) {
      LAUNCH(launch_fprop_tile(g, x, W, nullptr, z, nullptr, st, &bn));
      if (!FUSED_TILE) LAUNCH(post_op_pass(g, dt, z, nz, st));
      return CONVBN_OK;
    }
  }
  // w' = s w (both orders), b' = (b - mu) s + beta; then Z = w' (*) X + b'
  LAUNCH(launch_fold(g, dt, W, b, gamma, beta, mean, var, 0, w.w_krsc, w_folded, w.bfold, st));
  LAUNCH(run_fprop(g, dt, x, w.w_krsc, w.bfold, z, w.conv_scratch, st));
  return CONVBN_OK;
}

convbn_status convbn_tune_bwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                              const float* gamma, const float* mean, const float* var,
                              const void* w_folded, const void* dz, void* dx, void* dW, float* db,
                              float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;   // false: input gradient only (Sec. 4.3's adversarial-example use)
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_tune_bwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const TuneBwdWs w = carve_tune_bwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (g.act & CONVBN_ACT_RELU_IN) g.post_mask = x;   // dx comes out masked with x > 0
  g.post_add = g.add_in;                             // ... after the addend
  if (params && convbn_tune_bwd_is_fused(desc)) {
    // deep layers: dw', r and the fold-back in one launch (the fp32 dw' never reaches memory); the space of the
    // fp32 copy holds the few partial sums the workgroups exchange.  Where nothing was kept, the same launch leaves
    // w' for the input gradient, which then runs second: no fold launch.
    void* refold = (dx && !w_folded) ? w.w_crsk : nullptr;
    LAUNCH(launch_wgrad_sq_fused(g, x, dz, W, b, gamma, mean, var, dW, db, dgamma, dbeta, w.dwf_part, refold, st));
    if (dx) LAUNCH(run_dgrad(g, dt, dz, w_folded ? w_folded : w.w_crsk, dx, w.conv_scratch, st));   // dX = w'_rot (*) dZ
    return CONVBN_OK;
  }
  if (dx) {
    const void* wt = w_folded;
    if (!wt) {  // nothing was kept: fold again, transposed order only
      LAUNCH(launch_fold(g, dt, W, b, gamma, nullptr, mean, var, 0, nullptr, w.w_crsk, nullptr, st));
      wt = w.w_crsk;
    }
    if (params && !needs_cin_pad(g, dt) && wgrad_way(g, dt).sq && wgrad_dgrad_pair_supported(g, dt)) {
      // shallow layers: the two gradient passes are independent and share one launch (see wgrad_sq.hip)
      LAUNCH(launch_wgrad_dgrad_pair(g, x, dz, wt, dx, w.dwf_part, w.r_part, st));
      if (!FUSED_RW) LAUNCH(post_op_pass(g, dt, dx, (size_t)g.Min * g.Cin, st));
      LAUNCH(launch_fold_back(g, dt, w.dwf_part, w.nsplit, w.r_part, w.nrpart, W, b, gamma, mean, var, 0,
                              dW, db, dgamma, dbeta, st));
      return CONVBN_OK;
    }
    LAUNCH(run_dgrad(g, dt, dz, wt, dx, w.conv_scratch, st));   // dX = w'_rot (*) dZ
  }
  if (!params) return CONVBN_OK;
  LAUNCH(run_wgrad(g, dt, x, dz, w.dwf_part, w.r_part, w.wgrad_scratch, st));   // dw' = dZ (.) X and r = sum dZ (fp32 partials)
  LAUNCH(launch_fold_back(g, dt, w.dwf_part, w.nsplit, w.r_part, w.nrpart, W, b, gamma, mean, var, 0,
                          dW, db, dgamma, dbeta, st));
  return CONVBN_OK;
}

convbn_status convbn_eval_fwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                              const float* gamma, const float* beta, const float* mean,
                              const float* var, void* z, void* y_saved, void* ws, size_t ws_bytes,
                              void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z); REQUIRE_PTR(y_saved);
  OPTIONAL_PTR(b);
  const int dt = desc->dtype;
  s = check_ws(carve_eval_fwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const EvalFwdWs w = carve_eval_fwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  LAUNCH(run_fprop(g, dt, x, W, b, y_saved, w.conv_scratch, st));         // Y = w (*) X + b
  g.post_relu = g.act & CONVBN_ACT_RELU_OUT; g.post_add = g.add_out;   // applied to Z, not to the stored Y
  LAUNCH(launch_bn_affine_fwd(g, dt, y_saved, gamma, beta, mean, var, z, st));  // Z from Y
  return CONVBN_OK;
}

convbn_status convbn_eval_bwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                              const float* gamma, const float* mean, const float* var,
                              const void* y_saved, const void* dz, void* dx, void* dW, float* db,
                              float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(y_saved); REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;   // false: input gradient only
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_eval_bwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const EvalBwdWs w = carve_eval_bwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (g.act & CONVBN_ACT_RELU_IN) g.post_mask = x;   // dx comes out masked with x > 0
  g.post_add = g.add_in;                             // ... after the addend
  // dY = s dZ, partial per-channel sums of dZ and dZ (Y-mu)/sqrt(var+eps)
  LAUNCH(launch_bn_bwd(g, dt, dz, y_saved, gamma, mean, var, w.dy, w.bn_part, st));
  if (params) LAUNCH(launch_bn_bwd_finalize(g, w.bn_part, w.nparts, gamma, var, dgamma, dbeta, db, st));
  if (dx) {
    // the input-gradient pass reads the weight as [Cin][kH][kW][Cout]
    LAUNCH(launch_fold(g, dt, W, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, w.w_crsk,
                       nullptr, st));
    LAUNCH(run_dgrad(g, dt, w.dy, w.w_crsk, dx, w.conv_scratch, st));   // dX = w_rot (*) dY
  }
  if (!params) return CONVBN_OK;
  LAUNCH(run_wgrad(g, dt, x, w.dy, w.dwf_part, nullptr, w.wgrad_scratch, st));   // dW = dY (.) X
  LAUNCH(launch_fold_back(g, dt, w.dwf_part, w.nsplit, nullptr, 0, W, nullptr, nullptr, nullptr,
                          nullptr, 1, dW, nullptr, nullptr, nullptr, st));
  return CONVBN_OK;
}

int32_t convbn_tconv_hout(const convbn_desc* desc) {
  Geom g;
  return make_tgeom(desc, &g) == CONVBN_OK ? g.Hin : 0;
}

int32_t convbn_tconv_wout(const convbn_desc* desc) {
  Geom g;
  return make_tgeom(desc, &g) == CONVBN_OK ? g.Win : 0;
}

size_t convbn_tconv_workspace_bytes(const convbn_desc* desc, int mode, int pass) {
  Geom g;
  if (make_tgeom(desc, &g) != CONVBN_OK) return 0;
  if (pass == CONVBN_PASS_FWD) return carve_tconv_fwd(g, desc->dtype, nullptr).bytes;   // the same for both modes
  if (mode == CONVBN_MODE_TUNE) return carve_tconv_bwd(g, desc->dtype, nullptr).bytes;
  return mode == CONVBN_MODE_EVAL ? carve_tconv_eval_bwd(g, desc->dtype, nullptr).bytes : 0;
}

size_t convbn_tconv_saved_bytes(const convbn_desc* desc, int mode, int refold) {
  Geom g;
  if (make_tgeom(desc, &g) != CONVBN_OK) return 0;
  if (mode == CONVBN_MODE_EVAL) return (size_t)g.Min * g.Cin * esize(desc->dtype);   // Y: the block's output size
  return refold ? 0 : (size_t)g.Cout * g.K * esize(desc->dtype);
}

convbn_status convbn_tconv_tune_fwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                    const float* gamma, const float* beta, const float* mean, const float* var,
                                    void* z, void* w_folded, void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_tgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded);
  const int dt = desc->dtype;
  s = check_ws(carve_tconv_fwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const TconvFwdWs w = carve_tconv_fwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // w' = s w in both orders, b'; then Z = (transposed convolution of X with w') + b'
  const bool one_product = pw_tconv_supported(g, dt);   // stride = window: a product with a depth-to-space store
  LAUNCH(launch_fold_t(dt, g.Cout, g.Cin, g.kH * g.kW, W, b, gamma, beta, mean, var, g.eps, one_product, w_folded,
                       w.w_swap, w.bfold, st));
  if (one_product) LAUNCH(launch_tconv_pw(g, x, w.w_swap, w.bfold, z, st));
  else if (tconv_fwd_direct(g, dt)) LAUNCH(launch_dgrad_direct(g, dt, x, w.w_swap, w.bfold, z, st));
  else LAUNCH(dgrad_any(g, dt, x, w.w_swap, w.bfold, z, w.conv_scratch, st));
  return CONVBN_OK;
}

convbn_status convbn_tconv_tune_bwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                    const float* gamma, const float* mean, const float* var, const void* w_folded,
                                    const void* dz, void* dx, void* dW, float* db, float* dgamma, float* dbeta,
                                    void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_tgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;   // false: input gradient only
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_tconv_bwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const TconvBwdWs w = carve_tconv_bwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int taps = g.kH * g.kW;
  if (dx) {
    const void* wf = w_folded;
    if (!wf) {  // nothing was kept: fold again, in the order this pass reads
      LAUNCH(launch_fold_t(dt, g.Cout, g.Cin, taps, W, b, gamma, nullptr, mean, var, g.eps, 0, w.w_same, nullptr,
                           nullptr, st));
      wf = w.w_same;
    }
    LAUNCH(run_fprop(g, dt, dz, wf, nullptr, dx, w.conv_scratch, st));   // dX = w' (*) dZ: a plain convolution
  }
  if (!params) return CONVBN_OK;
  // dw'[ci][tap][co] = sum X[ci] dZ[co]: the associated convolution's weight gradient with dZ as its input
  LAUNCH(run_wgrad(g, dt, dz, x, w.dwf_part, nullptr, w.wgrad_scratch, st));
  LAUNCH(launch_colsum(tconv_out_rows(g), dt, dz, w.r_part, st));       // r = sum dZ
  LAUNCH(launch_fold_back_t(dt, g.Cout, g.Cin, taps, w.dwf_part, w.nsplit, w.r_part, w.nrpart, W, b, gamma, mean,
                            var, g.eps, w.dot_part, dW, db, dgamma, dbeta, st));
  return CONVBN_OK;
}

convbn_status convbn_tconv_eval_fwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                    const float* gamma, const float* beta, const float* mean, const float* var,
                                    void* z, void* y_saved, void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_tgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z); REQUIRE_PTR(y_saved);
  OPTIONAL_PTR(b);
  const int dt = desc->dtype;
  s = check_ws(carve_tconv_fwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const TconvFwdWs w = carve_tconv_fwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool one_product = pw_tconv_supported(g, dt);
  // the weight in the order the forward kernel reads (no scaling), Y = transposed convolution + b, then Z from Y
  LAUNCH(launch_fold_t(dt, g.Cout, g.Cin, g.kH * g.kW, W, b, nullptr, nullptr, nullptr, nullptr, g.eps, one_product,
                       nullptr, w.w_swap, w.bfold, st));
  if (one_product) LAUNCH(launch_tconv_pw(g, x, w.w_swap, w.bfold, y_saved, st));
  else if (tconv_fwd_direct(g, dt)) LAUNCH(launch_dgrad_direct(g, dt, x, w.w_swap, w.bfold, y_saved, st));
  else LAUNCH(dgrad_any(g, dt, x, w.w_swap, w.bfold, y_saved, w.conv_scratch, st));
  LAUNCH(launch_bn_affine_fwd(tconv_out_rows(g), dt, y_saved, gamma, beta, mean, var, z, st));
  return CONVBN_OK;
}

convbn_status convbn_tconv_eval_bwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                    const float* gamma, const float* mean, const float* var, const void* y_saved,
                                    const void* dz, void* dx, void* dW, float* db, float* dgamma, float* dbeta,
                                    void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_tgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(y_saved); REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_tconv_eval_bwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const TconvEvalBwdWs w = carve_tconv_eval_bwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Geom rows = tconv_out_rows(g);
  LAUNCH(launch_bn_bwd(rows, dt, dz, y_saved, gamma, mean, var, w.dy, w.bn_part, st));   // dY = s dZ and the channel sums
  if (params) LAUNCH(launch_bn_bwd_finalize(rows, w.bn_part, w.nparts, gamma, var, dgamma, dbeta, db, st));
  if (dx) LAUNCH(run_fprop(g, dt, w.dy, W, nullptr, dx, w.conv_scratch, st));            // dX = w (*) dY
  if (!params) return CONVBN_OK;
  LAUNCH(run_wgrad(g, dt, w.dy, x, w.dwf_part, nullptr, w.wgrad_scratch, st));           // dW = sum X dY
  LAUNCH(launch_fold_back_t(dt, g.Cout, g.Cin, g.kH * g.kW, w.dwf_part, w.nsplit, nullptr, 0, W, nullptr, nullptr,
                            nullptr, nullptr, g.eps, nullptr, dW, nullptr, nullptr, nullptr, st));
  return CONVBN_OK;
}

size_t convbn_dw_workspace_bytes(const convbn_desc* desc, int mode, int pass) {
  Geom g;
  if (make_dwgeom(desc, &g) != CONVBN_OK) return 0;
  if (mode != CONVBN_MODE_TUNE && mode != CONVBN_MODE_EVAL) return 0;
  return pass == CONVBN_PASS_FWD ? carve_dw_fwd(g, desc->dtype, nullptr).bytes
                                 : carve_dw_bwd(g, desc->dtype, mode, nullptr).bytes;
}

size_t convbn_dw_saved_bytes(const convbn_desc* desc, int mode, int refold) {
  Geom g;
  if (make_dwgeom(desc, &g) != CONVBN_OK) return 0;
  if (mode == CONVBN_MODE_EVAL) return (size_t)g.M * g.Cout * esize(desc->dtype);
  return refold ? 0 : (size_t)g.kH * g.kW * g.Cin * esize(desc->dtype);
}

convbn_status convbn_dw_tune_fwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                 const float* gamma, const float* beta, const float* mean, const float* var,
                                 void* z, void* w_folded, void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_dwgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded);
  const int dt = desc->dtype;
  s = check_ws(carve_dw_fwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const DwFwdWs w = carve_dw_fwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  void* wf = w_folded ? w_folded : w.wf;
  LAUNCH(launch_dw_fold(g, dt, W, b, gamma, beta, mean, var, wf, w.bfold, st));   // w' = s w (tap-major), b'
  LAUNCH(launch_dw_fprop(g, dt, x, wf, w.bfold, z, st));                          // Z = w' (*) X + b'
  return CONVBN_OK;
}

convbn_status convbn_dw_tune_bwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                 const float* gamma, const float* mean, const float* var, const void* w_folded,
                                 const void* dz, void* dx, void* dW, float* db, float* dgamma, float* dbeta,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_dwgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_dw_bwd(g, dt, CONVBN_MODE_TUNE, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const DwBwdWs w = carve_dw_bwd(g, dt, CONVBN_MODE_TUNE, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dx) {
    const void* wf = w_folded;
    if (!wf) {
      LAUNCH(launch_dw_fold(g, dt, W, b, gamma, nullptr, mean, var, w.wf, nullptr, st));
      wf = w.wf;
    }
    LAUNCH(launch_dw_dgrad(g, dt, dz, wf, dx, st));                                // dX = w'_rot (*) dZ
  }
  if (!params) return CONVBN_OK;
  LAUNCH(launch_dw_wgrad(g, dt, x, dz, w.part, w.r_part, st));                     // dw' = dZ (.) X, r = sum dZ
  LAUNCH(launch_dw_fold_back(g, dt, w.part, w.r_part, w.slices, w.sums, W, b, gamma, mean, var, dW, db, dgamma,
                             dbeta, st));
  return CONVBN_OK;
}

convbn_status convbn_dw_eval_fwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                 const float* gamma, const float* beta, const float* mean, const float* var,
                                 void* z, void* y_saved, void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_dwgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z); REQUIRE_PTR(y_saved);
  OPTIONAL_PTR(b);
  const int dt = desc->dtype;
  s = check_ws(carve_dw_fwd(g, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const DwFwdWs w = carve_dw_fwd(g, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  LAUNCH(launch_dw_fold(g, dt, W, b, nullptr, nullptr, nullptr, nullptr, w.wf, w.bfold, st));   // reorder only
  LAUNCH(launch_dw_fprop(g, dt, x, w.wf, w.bfold, y_saved, st));                                 // Y = w (*) X + b
  LAUNCH(launch_bn_affine_fwd(g, dt, y_saved, gamma, beta, mean, var, z, st));                   // Z from Y
  return CONVBN_OK;
}

convbn_status convbn_dw_eval_bwd(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                 const float* gamma, const float* mean, const float* var, const void* y_saved,
                                 const void* dz, void* dx, void* dW, float* db, float* dgamma, float* dbeta,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g;
  convbn_status s = make_dwgeom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(y_saved); REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_dw_bwd(g, dt, CONVBN_MODE_EVAL, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const DwBwdWs w = carve_dw_bwd(g, dt, CONVBN_MODE_EVAL, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  LAUNCH(launch_bn_bwd(g, dt, dz, y_saved, gamma, mean, var, w.dy, w.bn_part, st));
  if (params) LAUNCH(launch_bn_bwd_finalize(g, w.bn_part, w.nparts, gamma, var, dgamma, dbeta, db, st));
  if (dx) {
    LAUNCH(launch_dw_fold(g, dt, W, nullptr, nullptr, nullptr, nullptr, nullptr, w.wf, nullptr, st));
    LAUNCH(launch_dw_dgrad(g, dt, w.dy, w.wf, dx, st));
  }
  if (!params) return CONVBN_OK;
  LAUNCH(launch_dw_wgrad(g, dt, x, w.dy, w.part, nullptr, st));
  LAUNCH(launch_dw_fold_back(g, dt, w.part, nullptr, w.slices, w.sums, W, nullptr, nullptr, nullptr, nullptr, dW,
                             nullptr, nullptr, nullptr, st));
  return CONVBN_OK;
}

size_t convbn_grouped_workspace_bytes(const convbn_desc* desc, int groups, int mode, int pass) {
  Geom g, gf;
  if (make_ggeom(desc, groups, &g, &gf) != CONVBN_OK) return 0;
  if (grouped_route(desc, groups) == G_ROUTE_DENSE) return convbn_workspace_bytes(desc, mode, pass);
  if (grouped_route(desc, groups) == G_ROUTE_DEPTHWISE) return convbn_dw_workspace_bytes(desc, mode, pass);
  if (mode != CONVBN_MODE_TUNE && mode != CONVBN_MODE_EVAL) return 0;
  return pass == CONVBN_PASS_FWD ? carve_g_fwd(gf, desc->dtype, nullptr).bytes
                                 : carve_g_bwd(g, gf, groups, desc->dtype, mode, nullptr).bytes;
}

size_t convbn_grouped_saved_bytes(const convbn_desc* desc, int groups, int mode, int refold) {
  Geom g, gf;
  if (make_ggeom(desc, groups, &g, &gf) != CONVBN_OK) return 0;
  if (grouped_route(desc, groups) == G_ROUTE_DENSE) return convbn_saved_bytes(desc, mode, refold);
  if (grouped_route(desc, groups) == G_ROUTE_DEPTHWISE) return convbn_dw_saved_bytes(desc, mode, refold);
  if (mode == CONVBN_MODE_EVAL) return (size_t)g.M * g.Cout * esize(desc->dtype);
  return refold ? 0 : (size_t)gf.Cout * gf.K * esize(desc->dtype);
}

convbn_status convbn_grouped_tune_fwd(const convbn_desc* desc, int groups, const void* x, const void* W,
                                      const float* b, const float* gamma, const float* beta, const float* mean,
                                      const float* var, void* z, void* w_folded, void* ws, size_t ws_bytes,
                                      void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g, gf;
  convbn_status s = make_ggeom(desc, groups, &g, &gf);
  if (s != CONVBN_OK) return s;
  if (grouped_route(desc, groups) == G_ROUTE_DENSE) return convbn_tune_fwd(desc, x, W, b, gamma, beta, mean, var, z, w_folded, ws, ws_bytes, stream);
  if (grouped_route(desc, groups) == G_ROUTE_DEPTHWISE) return convbn_dw_tune_fwd(desc, x, W, b, gamma, beta, mean, var, z, w_folded, ws, ws_bytes, stream);
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded);
  const int dt = desc->dtype;
  s = check_ws(carve_g_fwd(gf, dt, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const GFwdWs w = carve_g_fwd(gf, dt, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // w' = s w in both orders ([Cout][taps][cg] for this pass, [cg][taps][Cout] kept for backward), b'
  LAUNCH(launch_fold(gf, dt, W, b, gamma, beta, mean, var, 0, w.w_krsc, w_folded, w.bfold, st));
  LAUNCH(launch_g_fprop(g, groups, dt, x, w.w_krsc, w.bfold, z, st));              // Z = w' (*) X + b'
  return CONVBN_OK;
}

convbn_status convbn_grouped_tune_bwd(const convbn_desc* desc, int groups, const void* x, const void* W,
                                      const float* b, const float* gamma, const float* mean, const float* var,
                                      const void* w_folded, const void* dz, void* dx, void* dW, float* db,
                                      float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g, gf;
  convbn_status s = make_ggeom(desc, groups, &g, &gf);
  if (s != CONVBN_OK) return s;
  if (grouped_route(desc, groups) == G_ROUTE_DENSE) return convbn_tune_bwd(desc, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma, dbeta, ws, ws_bytes, stream);
  if (grouped_route(desc, groups) == G_ROUTE_DEPTHWISE) return convbn_dw_tune_bwd(desc, x, W, b, gamma, mean, var, w_folded, dz, dx, dW, db, dgamma, dbeta, ws, ws_bytes, stream);
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(w_folded); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_g_bwd(g, gf, groups, dt, CONVBN_MODE_TUNE, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const GBwdWs w = carve_g_bwd(g, gf, groups, dt, CONVBN_MODE_TUNE, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dx) {
    const void* wf = w_folded;
    if (!wf) {   // not kept: fold again (Sec. 3.3 recomputes w' from the parameters)
      LAUNCH(launch_fold(gf, dt, W, b, gamma, nullptr, mean, var, 0, nullptr, w.w_crsk, nullptr, st));
      wf = w.w_crsk;
    }
    LAUNCH(launch_g_dgrad(g, groups, dt, dz, wf, dx, st));                          // dX = w'_rot (*) dZ
  }
  if (!params) return CONVBN_OK;
  const bool own_r = g_wgrad_makes_rsum(g, groups, dt);
  LAUNCH(launch_g_wgrad(g, groups, dt, x, dz, w.part, own_r ? w.r_part : nullptr, st));   // dw' = dZ (.) X
  if (!own_r) LAUNCH(launch_colsum(g, dt, dz, w.r_part, st));                              // r = sum dZ
  LAUNCH(launch_fold_back(gf, dt, w.part, w.slices, w.r_part, w.nrpart, W, b, gamma, mean, var, 0, dW, db, dgamma,
                          dbeta, st));
  return CONVBN_OK;
}

convbn_status convbn_grouped_eval_fwd(const convbn_desc* desc, int groups, const void* x, const void* W,
                                      const float* b, const float* gamma, const float* beta, const float* mean,
                                      const float* var, void* z, void* y_saved, void* ws, size_t ws_bytes,
                                      void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g, gf;
  convbn_status s = make_ggeom(desc, groups, &g, &gf);
  if (s != CONVBN_OK) return s;
  if (grouped_route(desc, groups) == G_ROUTE_DENSE) return convbn_eval_fwd(desc, x, W, b, gamma, beta, mean, var, z, y_saved, ws, ws_bytes, stream);
  if (grouped_route(desc, groups) == G_ROUTE_DEPTHWISE) return convbn_dw_eval_fwd(desc, x, W, b, gamma, beta, mean, var, z, y_saved, ws, ws_bytes, stream);
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z); REQUIRE_PTR(y_saved);
  OPTIONAL_PTR(b);
  const int dt = desc->dtype;
  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)ws; (void)ws_bytes;
  LAUNCH(launch_g_fprop(g, groups, dt, x, W, b, y_saved, st));                        // Y = w (*) X + b
  LAUNCH(launch_bn_affine_fwd(g, dt, y_saved, gamma, beta, mean, var, z, st));        // Z from Y
  return CONVBN_OK;
}

convbn_status convbn_grouped_eval_bwd(const convbn_desc* desc, int groups, const void* x, const void* W,
                                      const float* b, const float* gamma, const float* mean, const float* var,
                                      const void* y_saved, const void* dz, void* dx, void* dW, float* db,
                                      float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream) {
  if (desc && desc->act) return fail(CONVBN_ERR_UNSUPPORTED, "this entry point takes no activation bits (act must be 0)");
  Geom g, gf;
  convbn_status s = make_ggeom(desc, groups, &g, &gf);
  if (s != CONVBN_OK) return s;
  if (grouped_route(desc, groups) == G_ROUTE_DENSE) return convbn_eval_bwd(desc, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma, dbeta, ws, ws_bytes, stream);
  if (grouped_route(desc, groups) == G_ROUTE_DEPTHWISE) return convbn_dw_eval_bwd(desc, x, W, b, gamma, mean, var, y_saved, dz, dx, dW, db, dgamma, dbeta, ws, ws_bytes, stream);
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  REQUIRE_PTR(y_saved); REQUIRE_PTR(dz);
  OPTIONAL_PTR(b); OPTIONAL_PTR(dx); OPTIONAL_PTR(db);
  OPTIONAL_PTR(dW); OPTIONAL_PTR(dgamma); OPTIONAL_PTR(dbeta);
  const bool params = dW != nullptr;
  if (!params && (dgamma || dbeta || db || !dx))
    return fail(CONVBN_ERR_NULL, "without dW only dx may be asked for (dgamma, dbeta, db NULL, dx given)");
  if (params && (!dgamma || !dbeta))
    return fail(CONVBN_ERR_NULL, "dgamma and dbeta are required together with dW");
  if (params && (b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const int dt = desc->dtype;
  s = check_ws(carve_g_bwd(g, gf, groups, dt, CONVBN_MODE_EVAL, nullptr).bytes, ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  const GBwdWs w = carve_g_bwd(g, gf, groups, dt, CONVBN_MODE_EVAL, ws);
  hipStream_t st = static_cast<hipStream_t>(stream);
  LAUNCH(launch_bn_bwd(g, dt, dz, y_saved, gamma, mean, var, w.dy, w.bn_part, st));   // dY = s dZ, sums for dgamma, dbeta
  if (params) LAUNCH(launch_bn_bwd_finalize(g, w.bn_part, w.nparts, gamma, var, dgamma, dbeta, db, st));
  if (dx) {
    LAUNCH(launch_fold(gf, dt, W, nullptr, nullptr, nullptr, nullptr, nullptr, 1, nullptr, w.w_crsk, nullptr, st));
    LAUNCH(launch_g_dgrad(g, groups, dt, w.dy, w.w_crsk, dx, st));
  }
  if (!params) return CONVBN_OK;
  LAUNCH(launch_g_wgrad(g, groups, dt, x, w.dy, w.part, nullptr, st));
  LAUNCH(launch_fold_back(gf, dt, w.part, w.slices, nullptr, 0, W, nullptr, nullptr, nullptr, nullptr, 1, dW, nullptr,
                          nullptr, nullptr, st));
  return CONVBN_OK;
}

convbn_status convbn_tune_fwd_scale_epilogue(const convbn_desc* desc, const void* x, const void* W, const float* b,
                                             const float* gamma, const float* beta, const float* mean,
                                             const float* var, void* z, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(beta); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(z);
  OPTIONAL_PTR(b);
  const int dt = desc->dtype;
  const BnEpilogue bn{gamma, beta, mean, var, b, g.eps, nullptr, g.kH * g.kW, g.Cin, g.Cout};
  hipStream_t st = static_cast<hipStream_t>(stream);
  g.post_relu = g.act & CONVBN_ACT_RELU_OUT; g.post_add = g.add_out;
  const size_t nz = (size_t)g.M * g.Cout;
  // Z = s (w (*) X) + b': the unfolded weight goes straight into the convolution, one launch in all
  if (!needs_cin_pad(g, dt) && !pw_fprop_supported(g, dt) && rw_fprop_supported(g, dt)) {
    LAUNCH(launch_fprop_rw(g, x, W, nullptr, z, st, &bn));
    if (!FUSED_RW) LAUNCH(post_op_pass(g, dt, z, nz, st));
    return CONVBN_OK;
  }
  if (!needs_cin_pad(g, dt) && !pw_fprop_supported(g, dt) && st_fprop_supported(g, dt)) {
    LAUNCH(launch_fprop_st(g, x, W, nullptr, z, st, &bn));
    if (!FUSED_ST) LAUNCH(post_op_pass(g, dt, z, nz, st));
    return CONVBN_OK;
  }
  if (pw_fprop_scaled_supported(g, dt)) {
    LAUNCH(launch_fprop_pw(g, x, W, nullptr, z, st, &bn));
    if (!FUSED_PW) LAUNCH(post_op_pass(g, dt, z, nz, st));
    return CONVBN_OK;
  }
  if (!pw_fprop_supported(g, dt) && tile_fprop_scaled_supported(g, dt)) {
    LAUNCH(launch_fprop_tile(g, x, W, nullptr, z, nullptr, st, &bn));
    if (!FUSED_TILE) LAUNCH(post_op_pass(g, dt, z, nz, st));
    return CONVBN_OK;
  }
  return fail(CONVBN_ERR_UNSUPPORTED, "the scale-in-the-epilogue forward is built for a few plans of the LDS-tile "
              "kernels only (the benchmark's 3x3 and 1x1 shapes): use convbn_tune_fwd");
}

size_t convbn_fold_group_table_bytes(int n) { return n > 0 ? (size_t)n * fold_group_item_bytes() : 0; }

convbn_status convbn_fold_group_plan(int n, const convbn_fold_item* items, void* table_host, size_t table_bytes,
                                     int* grid_blocks) {
  if (n <= 0) return fail(CONVBN_ERR_SHAPE, "a fold group needs at least one block");
  if (!items || !table_host || !grid_blocks) return fail(CONVBN_ERR_NULL, "items, table_host and grid_blocks are required");
  if (table_bytes < convbn_fold_group_table_bytes(n))
    return fail(CONVBN_ERR_WORKSPACE, "table_host holds %zu bytes, %zu are needed", table_bytes,
                convbn_fold_group_table_bytes(n));
  int total = 0;
  for (int i = 0; i < n; ++i) {
    const convbn_fold_item& it = items[i];
    Geom g;
    convbn_status s = make_geom(it.desc, &g);
    if (s != CONVBN_OK) return s;
    const void* W = it.W; const float* b = it.b; const float* gamma = it.gamma; const float* beta = it.beta;
    const float* mean = it.mean; const float* var = it.var;
    void* w_fprop = it.w_fprop; void* w_folded = it.w_folded; float* b_folded = it.b_folded;
    REQUIRE_PTR(W);
    if (!it.identity) { REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var); }
    OPTIONAL_PTR(b); OPTIONAL_PTR(beta); OPTIONAL_PTR(w_fprop); OPTIONAL_PTR(w_folded); OPTIONAL_PTR(b_folded);
    if (b_folded && !it.identity && !beta) return fail(CONVBN_ERR_NULL, "beta is required when b_folded is wanted");
    int blocks = 0;
    if (!fold_group_item(g, it.desc->dtype, W, b, gamma, beta, mean, var, it.identity, w_fprop, w_folded, b_folded,
                         total, static_cast<char*>(table_host) + (size_t)i * fold_group_item_bytes(), &blocks))
      return fail(CONVBN_ERR_UNSUPPORTED, "block %d: a fold group takes bf16 blocks whose Cout and Cin*kH*kW are "
                  "multiples of 8 (fold the others with convbn_fold)", i);
    total += blocks;
  }
  *grid_blocks = total;
  return CONVBN_OK;
}

convbn_status convbn_fold_group(int n, const void* table_dev, int grid_blocks, void* stream) {
  if (n <= 0 || grid_blocks <= 0) return fail(CONVBN_ERR_SHAPE, "empty fold group");
  REQUIRE_PTR(table_dev);
  LAUNCH(launch_fold_group(table_dev, n, grid_blocks, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

int32_t convbn_tune_bwd_is_fused(const convbn_desc* desc) {
  Geom g;
  if (make_geom(desc, &g) != CONVBN_OK) return 0;
  const int dt = desc->dtype;
  return !needs_cin_pad(g, dt) && wgrad_sq_fused_supported(g, dt) &&
         wgrad_sq_fused_scratch_bytes(g) <= (size_t)wgrad_way(g, dt).nsplit * g.Cout * g.K * 4;
}

size_t convbn_fold_back_group_table_bytes(int n) { return n > 0 ? (size_t)n * fold_back_group_item_bytes() : 0; }

convbn_status convbn_fold_back_group_plan(int n, const convbn_fold_back_item* items, void* table_host,
                                          size_t table_bytes, int* grid_blocks) {
  if (n <= 0) return fail(CONVBN_ERR_SHAPE, "a fold-back group needs at least one block");
  if (!items || !table_host || !grid_blocks) return fail(CONVBN_ERR_NULL, "items, table_host and grid_blocks are required");
  if (table_bytes < convbn_fold_back_group_table_bytes(n))
    return fail(CONVBN_ERR_WORKSPACE, "table_host holds %zu bytes, %zu are needed", table_bytes,
                convbn_fold_back_group_table_bytes(n));
  int total = 0;
  for (int i = 0; i < n; ++i) {
    const convbn_fold_back_item& it = items[i];
    Geom g;
    convbn_status s = make_geom(it.desc, &g);
    if (s != CONVBN_OK) return s;
    const float* dw_part = it.dw_part; const float* r_part = it.r_part; const void* W = it.W; const float* b = it.b;
    const float* gamma = it.gamma; const float* mean = it.mean; const float* var = it.var; void* dW = it.dW;
    float* db = it.db; float* dgamma = it.dgamma; float* dbeta = it.dbeta;
    REQUIRE_PTR(dw_part); REQUIRE_PTR(r_part); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
    REQUIRE_PTR(dW); REQUIRE_PTR(dgamma); REQUIRE_PTR(dbeta);
    OPTIONAL_PTR(b); OPTIONAL_PTR(db);
    if ((b == nullptr) != (db == nullptr)) return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
    const WgradWay way = wgrad_way(g, it.desc->dtype);
    int blocks = 0;
    if (!fold_back_group_item(g, it.desc->dtype, dw_part, way.nsplit, r_part, way.nrpart, W, b, gamma, mean, var, dW, db,
                              dgamma, dbeta, total, static_cast<char*>(table_host) + (size_t)i * fold_back_group_item_bytes(),
                              &blocks))
      return fail(CONVBN_ERR_UNSUPPORTED, "block %d: a fold-back group takes bf16 blocks whose Cin*kH*kW is a multiple "
                  "of 4 (use convbn_fold_back for the others)", i);
    total += blocks;
  }
  *grid_blocks = total;
  return CONVBN_OK;
}

convbn_status convbn_fold_back_group(int n, const void* table_dev, int grid_blocks, void* stream) {
  if (n <= 0 || grid_blocks <= 0) return fail(CONVBN_ERR_SHAPE, "empty fold-back group");
  REQUIRE_PTR(table_dev);
  LAUNCH(launch_fold_back_group(table_dev, n, grid_blocks, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_fold(const convbn_desc* desc, const void* W, const float* b, const float* gamma,
                          const float* beta, const float* mean, const float* var, void* w_fprop,
                          void* w_folded, float* b_folded, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean); REQUIRE_PTR(var);
  OPTIONAL_PTR(b); OPTIONAL_PTR(beta); OPTIONAL_PTR(w_fprop); OPTIONAL_PTR(w_folded);
  OPTIONAL_PTR(b_folded);
  if (b_folded && !beta) return fail(CONVBN_ERR_NULL, "beta is required when b_folded is wanted");
  LAUNCH(launch_fold(g, desc->dtype, W, b, gamma, beta, mean, var, 0, w_fprop, w_folded, b_folded,
                     static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

size_t convbn_conv_workspace_bytes(const convbn_desc* desc, int pass) {
  Geom g;
  if (make_geom(desc, &g) != CONVBN_OK) return 0;
  const size_t bwd = dgrad_scratch_bytes(g, desc->dtype) > wgrad_scratch_bytes(g, desc->dtype)
                         ? dgrad_scratch_bytes(g, desc->dtype) : wgrad_scratch_bytes(g, desc->dtype);
  return align_up(pass == CONVBN_PASS_FWD ? fprop_scratch_bytes(g, desc->dtype) : bwd, 256);
}

convbn_status convbn_conv_fprop(const convbn_desc* desc, const void* x, const void* w,
                                const float* bias, void* z, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(w); REQUIRE_PTR(z); OPTIONAL_PTR(bias);
  s = check_ws(fprop_scratch_bytes(g, desc->dtype), ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  g.post_relu = g.act & CONVBN_ACT_RELU_OUT; g.post_add = g.add_out;
  LAUNCH(run_fprop(g, desc->dtype, x, w, bias, z, (float*)ws, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_conv_dgrad(const convbn_desc* desc, const void* dz, const void* w_t, void* dx,
                                void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(dz); REQUIRE_PTR(w_t); REQUIRE_PTR(dx);
  s = check_ws(dgrad_scratch_bytes(g, desc->dtype), ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  g.post_add = g.add_in;
  LAUNCH(run_dgrad(g, desc->dtype, dz, w_t, dx, (float*)ws, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_conv_dgrad_masked(const convbn_desc* desc, const void* dz, const void* w_t, const void* x,
                                       void* dx, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(dz); REQUIRE_PTR(w_t); REQUIRE_PTR(x); REQUIRE_PTR(dx);
  s = check_ws(dgrad_scratch_bytes(g, desc->dtype), ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  g.post_mask = x; g.post_add = g.add_in;
  LAUNCH(run_dgrad(g, desc->dtype, dz, w_t, dx, (float*)ws, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

int32_t convbn_wgrad_parts(const convbn_desc* desc) {
  Geom g;
  return make_geom(desc, &g) == CONVBN_OK ? nsplit_for(g, desc->dtype) : 0;
}

int32_t convbn_rsum_parts(const convbn_desc* desc) {
  Geom g;
  return make_geom(desc, &g) == CONVBN_OK ? wgrad_way(g, desc->dtype).nrpart : 0;
}

convbn_status convbn_conv_wgrad(const convbn_desc* desc, const void* x, const void* dz,
                                float* dw_part, float* r_part, void* ws, size_t ws_bytes, void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(x); REQUIRE_PTR(dz); REQUIRE_PTR(dw_part); OPTIONAL_PTR(r_part);
  s = check_ws(wgrad_scratch_bytes(g, desc->dtype), ws, ws_bytes);
  if (s != CONVBN_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  LAUNCH(run_wgrad(g, desc->dtype, x, dz, dw_part, r_part, ws, st));
  return CONVBN_OK;
}

convbn_status convbn_fold_back(const convbn_desc* desc, const float* dw_part, const float* r_part,
                               const void* W, const float* b, const float* gamma, const float* mean,
                               const float* var, void* dW, float* db, float* dgamma, float* dbeta,
                               void* stream) {
  Geom g;
  convbn_status s = make_geom(desc, &g);
  if (s != CONVBN_OK) return s;
  REQUIRE_PTR(dw_part); REQUIRE_PTR(r_part); REQUIRE_PTR(W); REQUIRE_PTR(gamma); REQUIRE_PTR(mean);
  REQUIRE_PTR(var); REQUIRE_PTR(dW); REQUIRE_PTR(dgamma); REQUIRE_PTR(dbeta);
  OPTIONAL_PTR(b); OPTIONAL_PTR(db);
  if ((b == nullptr) != (db == nullptr))
    return fail(CONVBN_ERR_NULL, "db must be given exactly when b is given");
  const WgradWay way = wgrad_way(g, desc->dtype);
  LAUNCH(launch_fold_back(g, desc->dtype, dw_part, way.nsplit, r_part, way.nrpart,
                          W, b, gamma, mean, var, 0, dW, db, dgamma, dbeta,
                          static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_aux_eltwise(int op, int dtype, void* a, const void* b, size_t n, void* stream) {
  if (op < 0 || op > 3) return fail(CONVBN_ERR_UNSUPPORTED, "unknown elementwise op %d", op);
  if (dtype != CONVBN_F32 && dtype != CONVBN_BF16) return fail(CONVBN_ERR_UNSUPPORTED, "dtype %d", dtype);
  REQUIRE_PTR(a);
  if (op != 0) REQUIRE_PTR(b);
  LAUNCH(launch_eltwise(op, dtype, a, b, nullptr, n, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_aux_add_relu_bwd(int dtype, void* a, const void* b, const void* y, size_t n, void* stream) {
  if (dtype != CONVBN_F32 && dtype != CONVBN_BF16) return fail(CONVBN_ERR_UNSUPPORTED, "dtype %d", dtype);
  REQUIRE_PTR(a); REQUIRE_PTR(b); REQUIRE_PTR(y);
  LAUNCH(launch_eltwise(4, dtype, a, b, y, n, static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_aux_maxpool_fwd(int dtype, const void* x, void* y, void* idx, int32_t N, int32_t H,
                                     int32_t W, int32_t C, void* stream) {
  if (dtype != CONVBN_F32 && dtype != CONVBN_BF16) return fail(CONVBN_ERR_UNSUPPORTED, "dtype %d", dtype);
  if (N < 1 || H < 1 || W < 1 || C < 1) return fail(CONVBN_ERR_SHAPE, "non-positive dimension");
  if ((long long)N * H * W * C > 0x7fffffffLL) return fail(CONVBN_ERR_UNSUPPORTED, "the input has more than 2^31-1 elements");
  REQUIRE_PTR(x); REQUIRE_PTR(y); REQUIRE_PTR(idx);
  LAUNCH(launch_maxpool_fwd(dtype, x, y, static_cast<unsigned char*>(idx), N, H, W, C,
                            static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

convbn_status convbn_aux_maxpool_bwd(int dtype, const void* dy, const void* idx, void* dx, int32_t N, int32_t H,
                                     int32_t W, int32_t C, void* stream) {
  if (dtype != CONVBN_F32 && dtype != CONVBN_BF16) return fail(CONVBN_ERR_UNSUPPORTED, "dtype %d", dtype);
  if (N < 1 || H < 1 || W < 1 || C < 1) return fail(CONVBN_ERR_SHAPE, "non-positive dimension");
  if ((long long)N * H * W * C > 0x7fffffffLL) return fail(CONVBN_ERR_UNSUPPORTED, "the input has more than 2^31-1 elements");
  REQUIRE_PTR(dy); REQUIRE_PTR(idx); REQUIRE_PTR(dx);
  LAUNCH(launch_maxpool_bwd(dtype, dy, static_cast<const unsigned char*>(idx), dx, N, H, W, C,
                            static_cast<hipStream_t>(stream)));
  return CONVBN_OK;
}

}  // extern "C"
