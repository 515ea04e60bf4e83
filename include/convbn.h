/*
 * convbn.h -- C ABI of the MI355X (gfx950) ConvBN-block library.
 *
 * One block = a 2-D convolution followed by a BatchNorm layer whose statistics are
 * frozen (Sec. 3.1 of "Efficient ConvBN Blocks for Transfer Learning and Beyond"):
 *
 *     Y = w (*) X + b                       X: [N,Cin,Hin,Win]   w: [Cout,Cin,kH,kW]
 *     Z = gamma (Y - mu)/sqrt(var+eps) + beta          Y,Z: [N,Cout,Hout,Wout]
 *
 * Two ways of running it, with identical results (Sec. 3.4.1):
 *   Tune mode (the paper's proposal, Sec. 3.3-3.4, Table 2 row "Tune"): on every call
 *     fold the BatchNorm into the weights, w' = s w, b' = (b - mu) s + beta with
 *     s = gamma/sqrt(var+eps), run ONE convolution, and in backward route dJ/dw'
 *     back to w, gamma, beta through s.  Only X and w' are kept for backward.
 *   Eval mode (Sec. 3.1, App. C, Table 2 row "Eval"): convolution, stored Y, separate
 *     per-channel affine; backward needs X and Y.  Built as the comparison path.
 *
 * GENERAL CONVENTIONS
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing, frees nothing and keeps no state between calls.
 *   - All work is enqueued asynchronously on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream).  No call synchronises with the host.
 *   - Arguments are validated on the host before anything is launched: a call that
 *     returns a validation error (codes 1-4) has had no effect on device memory.
 *     CONVBN_ERR_LAUNCH can come from any of the kernels a call enqueues; what the
 *     earlier ones wrote (workspace, w_folded, dx) then stays written.
 *   - Outputs are overwritten, never accumulated into.
 *   - mu and var are frozen buffers: read-only, no gradient.
 *   - Device-side value preconditions (var + eps > 0) are documented, not checked.
 *
 * MEMORY LAYOUT (the descriptor's dimensions are always the logical ones above)
 *   The one supported layout is channels-last, CONVBN_LAYOUT_NHWC:
 *     x, dx          [N][Hin][Win][Cin]
 *     z, y, dz       [N][Hout][Wout][Cout]
 *     W, dW          [Cout][kH][kW][Cin]
 *     w_folded       [Cin][kH][kW][Cout]   (the folded weight w', stored transposed:
 *                                           the order the input-gradient pass reads)
 *   dense, no padding between rows.  Element type of these tensors is desc->dtype;
 *   every [Cout] vector (b, gamma, beta, mean, var, db, dgamma, dbeta) is fp32.
 *   With dtype BF16 all accumulation is fp32; w' = bf16(float(W) * s) and
 *   dW = bf16(s * dJ/dw'_fp32) are each rounded once.
 *
 * Hout = floor((Hin + 2 pad_h - kH)/stride_h) + 1, likewise Wout.
 */
#ifndef CONVBN_H_
#define CONVBN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CONVBN_OK = 0,
  CONVBN_ERR_NULL = 1,        /* a required pointer is NULL                          */
  CONVBN_ERR_SHAPE = 2,       /* non-positive dim, negative pad, empty output, ...   */
  CONVBN_ERR_UNSUPPORTED = 3, /* unknown dtype / layout, tensor too large for int32  */
  CONVBN_ERR_WORKSPACE = 4,   /* ws is NULL or ws_bytes < convbn_workspace_bytes()   */
  CONVBN_ERR_LAUNCH = 5       /* the HIP runtime refused a launch                    */
} convbn_status;

typedef enum { CONVBN_F32 = 0, CONVBN_BF16 = 1 } convbn_dtype;
typedef enum { CONVBN_LAYOUT_NHWC = 0 } convbn_layout;
typedef enum { CONVBN_MODE_TUNE = 0, CONVBN_MODE_EVAL = 1 } convbn_mode;
typedef enum { CONVBN_PASS_FWD = 0, CONVBN_PASS_BWD = 1 } convbn_pass;

/* Problem descriptor: plain data, passed by pointer, caller-owned, read-only.
 * Dilation is 1 and groups is 1 (the paper's blocks use a single k, Sec. 3.1). */
typedef struct {
  int32_t N, Cin, Hin, Win;   /* logical dims of X (Sec. 3.1)                       */
  int32_t Cout, kH, kW;       /* W is logically [Cout,Cin,kH,kW] (App. C)           */
  int32_t stride_h, stride_w;
  int32_t pad_h, pad_w;       /* zero padding                                       */
  float eps;                  /* BatchNorm epsilon, inside the square root          */
  int32_t dtype;              /* convbn_dtype of x, W, z, y, dz, dx, dW, w_folded   */
  int32_t layout;             /* convbn_layout                                      */
  int32_t act;                /* CONVBN_ACT_* bits, 0 = none (see below)            */
  const void *add_out;        /* device tensor laid out like z  (CONVBN_ACT_ADD_OUT) */
  const void *add_in;         /* device tensor laid out like dx (CONVBN_ACT_ADD_IN)  */
} convbn_desc;

/* Activations around a block.  What follows a block does not change the block's computation (Sec. 3.1); these
 * bits only let the convolution kernels apply a neighbouring ReLU while the values are still in registers,
 * instead of a separate pass over the tensor.  Honoured by convbn_tune_fwd / _bwd, convbn_eval_fwd / _bwd,
 * convbn_tune_fwd_static, convbn_tune_fwd_scale_epilogue and convbn_conv_fprop; the transposed, depthwise and
 * grouped entry points reject a descriptor with act != 0.
 *   CONVBN_ACT_RELU_OUT  the forward calls return max(z, 0) in z.  Backward is unchanged: dz stays the gradient
 *                        with respect to the block's own output Z, i.e. the caller (or the next block, see the
 *                        other bit) has already applied the ReLU's backward mask.
 *   CONVBN_ACT_RELU_IN   x is the output of a ReLU: the backward calls return dx masked with x > 0, which is the
 *                        gradient with respect to that ReLU's input.
 *   CONVBN_ACT_ADD_OUT   a residual connection joins behind the block: the forward calls return z + add_out (the sum
 *                        of the two tensors, each rounded to dtype, rounded once more), before the ReLU of
 *                        CONVBN_ACT_RELU_OUT if that bit is set too.  add_out must not overlap z.
 *   CONVBN_ACT_ADD_IN    x also feeds a second branch whose gradient is add_in: the backward calls (and
 *                        convbn_conv_dgrad / convbn_conv_dgrad_masked) return dx + add_in, before the mask of
 *                        CONVBN_ACT_RELU_IN.  add_in must not overlap dx.
 * The addend pointers are read only when their bit is set (then they must not be NULL); they are caller-owned and
 * only read. */
enum { CONVBN_ACT_RELU_OUT = 1, CONVBN_ACT_RELU_IN = 2, CONVBN_ACT_ADD_OUT = 4, CONVBN_ACT_ADD_IN = 8 };

/* Output spatial size for a descriptor (0 on a NULL / invalid descriptor). */
int32_t convbn_hout(const convbn_desc *desc);
int32_t convbn_wout(const convbn_desc *desc);

/* Bytes of device workspace the given call needs (mode: convbn_mode, pass:
 * convbn_pass).  Depends on the descriptor only.  The backward figure covers the
 * case w_folded == NULL (re-fold).  Returns 0 for an invalid descriptor.  The
 * workspace carries nothing from one call to the next. */
size_t convbn_workspace_bytes(const convbn_desc *desc, int mode, int pass);

/* Tune-mode forward (Sec. 3.3: definitions of w', b'; Sec. 3.4: the folded
 * parameters are recomputed on every call, then a single convolution runs).
 *   in : x, W, b (nullable = no conv bias), gamma, beta, mean, var
 *   out: z            block output
 *        w_folded     nullable.  If given, receives w' ([Cin][kH][kW][Cout]) -- the
 *                     tensor Tune mode keeps for backward instead of Y.  If NULL
 *                     nothing but x needs to be kept and backward folds again.
 */
convbn_status convbn_tune_fwd(const convbn_desc *desc, const void *x, const void *W,
                              const float *b, const float *gamma, const float *beta,
                              const float *mean, const float *var, void *z, void *w_folded,
                              void *ws, size_t ws_bytes, void *stream);

/* Tune-mode backward (Table 2, row "Tune"; broadcast sums of App. B restored):
 *   dX = w'_rot (*) dZ            dw' = dZ (.) X            r_c = sum_{n,h,w} dZ
 *   dW = s dw'      db = s r      dgamma = (<dw'_c, w_c> + r_c (b_c - mu_c))/sqrt(var_c+eps)
 *   dbeta = r
 *   in : x, W, b (nullable), gamma, mean, var, dz,
 *        w_folded (nullable: the buffer convbn_tune_fwd filled; NULL = fold again
 *        into the workspace)
 *   out: dx (nullable = skip the input-gradient pass), dW, db (must be NULL exactly
 *        when b is NULL), dgamma, dbeta.
 *        Input gradient only (the frozen-model use of Sec. 4.3): dW, db, dgamma and
 *        dbeta all NULL and dx given -- the weight-gradient and fold-back passes are
 *        skipped.  Any other mix of NULLs is CONVBN_ERR_NULL.
 */
convbn_status convbn_tune_bwd(const convbn_desc *desc, const void *x, const void *W,
                              const float *b, const float *gamma, const float *mean,
                              const float *var, const void *w_folded, const void *dz, void *dx,
                              void *dW, float *db, float *dgamma, float *dbeta, void *ws,
                              size_t ws_bytes, void *stream);

/* Eval-mode forward (Sec. 3.1; App. C "Eval Mode"): convolution, then the
 * per-channel normalisation + affine as a separate pass over the stored Y.
 *   out: z, y_saved (required: the conv output Eval mode keeps for backward). */
convbn_status convbn_eval_fwd(const convbn_desc *desc, const void *x, const void *W,
                              const float *b, const float *gamma, const float *beta,
                              const float *mean, const float *var, void *z, void *y_saved,
                              void *ws, size_t ws_bytes, void *stream);

/* Eval-mode backward (Table 2, row "Eval"):
 *   dY = s dZ;  dgamma = sum dZ (Y - mu)/sqrt(var+eps);  dbeta = sum dZ;
 *   dX = w_rot (*) dY;  dW = dY (.) X;  db = sum dY.
 *   in : x, W, b (nullable; only its NULL-ness matters), gamma, mean, var, y_saved, dz
 *   out: dx (nullable), dW, db (NULL exactly when b is NULL), dgamma, dbeta;
 *        or dx alone (dW, db, dgamma, dbeta all NULL), as for convbn_tune_bwd */
convbn_status convbn_eval_bwd(const convbn_desc *desc, const void *x, const void *W,
                              const float *b, const float *gamma, const float *mean,
                              const float *var, const void *y_saved, const void *dz, void *dx,
                              void *dW, float *db, float *dgamma, float *dbeta, void *ws,
                              size_t ws_bytes, void *stream);

/* convbn_tune_fwd for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as convbn_tune_fwd, without ws / ws_bytes: the forward workspace is a device array
 * built into the library (convbn_static_workspace_limit() bytes = 32 MiB, held by every GPU
 * the library runs on until the process ends).  The call allocates and frees nothing.  A block
 * whose convbn_workspace_bytes(desc, CONVBN_MODE_TUNE, CONVBN_PASS_FWD) exceeds the limit is
 * refused with CONVBN_ERR_WORKSPACE before anything is launched.  All calls on one GPU share
 * that GPU's array: calls that overlap in time on one GPU (different streams, or different
 * threads) race; calls on one stream are ordered and safe.  The array keeps the previous
 * call's contents; nothing in it has to start at zero (every byte read is written first). */
convbn_status convbn_tune_fwd_static(const convbn_desc *desc, const void *x, const void *W,
                                     const float *b, const float *gamma, const float *beta,
                                     const float *mean, const float *var, void *z, void *w_folded,
                                     void *stream);
size_t convbn_static_workspace_limit(void);

/* Ablation of the fold (the forward of Sec. 3.3 without materialising w'): since the scale is per output
 * channel, Z = s (w (*) X) + b' -- the convolution reads the UNFOLDED W and its epilogue applies s and b',
 * which it works out from gamma, beta, mean, var (and b) itself.  One launch, no workspace, the same Z up to
 * rounding (w' is never rounded to bf16 here).  Backward still needs w' (convbn_tune_bwd with
 * w_folded == NULL folds it again).  Built as a measurement, for the kernel plans of the benchmark's 3x3
 * and 1x1 shapes; CONVBN_ERR_UNSUPPORTED otherwise (nothing is launched). */
convbn_status convbn_tune_fwd_scale_epilogue(const convbn_desc *desc, const void *x, const void *W,
                                             const float *b, const float *gamma, const float *beta,
                                             const float *mean, const float *var, void *z,
                                             void *stream);

/* ---- TransposedConv-BN block in Tune mode ----------------------------------------
 * Sec. 3.2.1 (last paragraph): scaling the weight along its output-channel index is
 * associative with a transposed convolution as well, so Tune mode covers
 * TransposedConv-BN blocks.  The operator is the adjoint of the convolution above with
 * respect to its input (dilation 1, groups 1, no output padding):
 *     Y[n, co, h sh - ph + i, w sw - pw + j] += W[ci, co, i, j] X[n, ci, h, w]   (+ b[co])
 *     Hout = (Hin - 1) stride_h - 2 pad_h + kH, likewise Wout; BatchNorm over the Cout channels.
 * The descriptor's fields keep their meaning (N, Cin, Hin, Win describe x; Cout, the
 * window, stride and padding the operator).  Layout (channels-last as everywhere):
 *     x, dx  [N][Hin][Win][Cin]        z, dz  [N][Hout][Wout][Cout]
 *     W, dW, w_folded  [Cin][kH][kW][Cout]      (logical [Cin, Cout, kH, kW])
 * Tune mode: w' = s w with s on the Cout index, b' as above; forward is ONE transposed
 * convolution with (w', b'); backward is Table 2's "Tune" row with the transposed
 * operator: dX = w' (*) dZ (a plain convolution), dw'[ci,co,i,j] = sum X dZ, r = sum dZ,
 * dW = s dw', dgamma_co = (sum_{ci,i,j} dw' w + r (b - mu)) / sqrt(var + eps), dbeta = r,
 * db = s r.  Arguments, NULL rules and error behaviour are those of convbn_tune_fwd /
 * convbn_tune_bwd; w_folded (nullable) is w' in the order of W.  Shapes whose padding
 * leaves no output are CONVBN_ERR_SHAPE. */
int32_t convbn_tconv_hout(const convbn_desc *desc);
int32_t convbn_tconv_wout(const convbn_desc *desc);
/* As convbn_workspace_bytes / convbn_saved_bytes, for the transposed block (Eval keeps Y, which has
 * the size of the block's output; Tune keeps w').  0 for an invalid descriptor. */
size_t convbn_tconv_workspace_bytes(const convbn_desc *desc, int mode, int pass);
size_t convbn_tconv_saved_bytes(const convbn_desc *desc, int mode, int refold);
convbn_status convbn_tconv_tune_fwd(const convbn_desc *desc, const void *x, const void *W,
                                    const float *b, const float *gamma, const float *beta,
                                    const float *mean, const float *var, void *z, void *w_folded,
                                    void *ws, size_t ws_bytes, void *stream);
convbn_status convbn_tconv_tune_bwd(const convbn_desc *desc, const void *x, const void *W,
                                    const float *b, const float *gamma, const float *mean,
                                    const float *var, const void *w_folded, const void *dz,
                                    void *dx, void *dW, float *db, float *dgamma, float *dbeta,
                                    void *ws, size_t ws_bytes, void *stream);

/* Eval mode of the transposed block (Sec. 3.1 with the transposed operator): Y = transposed
 * convolution + b stored in y_saved, then the per-channel affine as a separate pass; backward through
 * dY = s dZ as in Table 2's "Eval" row.  The comparison path for the two calls above; arguments as
 * convbn_eval_fwd / convbn_eval_bwd with W, dW in [Cin][kH][kW][Cout] order. */
convbn_status convbn_tconv_eval_fwd(const convbn_desc *desc, const void *x, const void *W,
                                    const float *b, const float *gamma, const float *beta,
                                    const float *mean, const float *var, void *z, void *y_saved,
                                    void *ws, size_t ws_bytes, void *stream);
convbn_status convbn_tconv_eval_bwd(const convbn_desc *desc, const void *x, const void *W,
                                    const float *b, const float *gamma, const float *mean,
                                    const float *var, const void *y_saved, const void *dz, void *dx,
                                    void *dW, float *db, float *dgamma, float *dbeta, void *ws,
                                    size_t ws_bytes, void *stream);

/* ---- Depthwise ConvBN block -------------------------------------------------------
 * A convolution with one filter per channel (groups = channels, Cin == Cout == C; CONVBN_ERR_SHAPE
 * otherwise) followed by the frozen BatchNorm.  The scale of Sec. 3.3 is per output channel, so Tune
 * mode is unchanged: w'[c] = s_c w[c], b' as above, one (depthwise) convolution, and Table 2's "Tune"
 * backward with <dw'_c, w_c> summed over the window only.  Layout:
 *     x, dx [N][Hin][Win][C]      z, dz, y [N][Hout][Wout][C]      W, dW [C][kH][kW]
 *     w_folded [kH][kW][C]        (w' tap-major: the order the kernels read)
 * Arguments, NULL rules and error behaviour as for the dense block's four calls. */
size_t convbn_dw_workspace_bytes(const convbn_desc *desc, int mode, int pass);
size_t convbn_dw_saved_bytes(const convbn_desc *desc, int mode, int refold);
convbn_status convbn_dw_tune_fwd(const convbn_desc *desc, const void *x, const void *W, const float *b,
                                 const float *gamma, const float *beta, const float *mean,
                                 const float *var, void *z, void *w_folded, void *ws, size_t ws_bytes,
                                 void *stream);
convbn_status convbn_dw_tune_bwd(const convbn_desc *desc, const void *x, const void *W, const float *b,
                                 const float *gamma, const float *mean, const float *var,
                                 const void *w_folded, const void *dz, void *dx, void *dW, float *db,
                                 float *dgamma, float *dbeta, void *ws, size_t ws_bytes, void *stream);
convbn_status convbn_dw_eval_fwd(const convbn_desc *desc, const void *x, const void *W, const float *b,
                                 const float *gamma, const float *beta, const float *mean,
                                 const float *var, void *z, void *y_saved, void *ws, size_t ws_bytes,
                                 void *stream);
convbn_status convbn_dw_eval_bwd(const convbn_desc *desc, const void *x, const void *W, const float *b,
                                 const float *gamma, const float *mean, const float *var,
                                 const void *y_saved, const void *dz, void *dx, void *dW, float *db,
                                 float *dgamma, float *dbeta, void *ws, size_t ws_bytes, void *stream);

/* ---- Grouped ConvBN block ----------------------------------------------------------
 * A convolution whose channels are split into `groups` equal parts, an output channel reading only
 * the input channels of its own part (the grouped layers of the ResNeXt / RegNet style models in
 * Sec. 4 and App. E), followed by the frozen BatchNorm.  groups must divide Cin and Cout
 * (CONVBN_ERR_SHAPE otherwise); with cg = Cin / groups and og = Cout / groups output channel o reads
 * input channels (o / og) cg .. (o / og) cg + cg - 1.  The scale of Sec. 3.3 is per output channel,
 * so Tune mode is unchanged: w'[o] = s_o w[o], b' as above, one (grouped) convolution, and Table 2's
 * "Tune" backward with <dw'_o, w_o> summed over the cg kH kW weights of channel o.  Layout:
 *     x, dx [N][Hin][Win][Cin]     z, dz, y [N][Hout][Wout][Cout]     W, dW [Cout][kH][kW][cg]
 *     w_folded [cg][kH][kW][Cout]  (w' in the order the input-gradient pass reads)
 * groups = 1 is the dense block and groups = Cin = Cout the depthwise one: their buffer layouts
 * coincide with this block's, and these calls pass such problems on to those blocks' calls (and
 * the queries to their queries).  Arguments, NULL rules and error behaviour as for the dense
 * block's four calls. */
size_t convbn_grouped_workspace_bytes(const convbn_desc *desc, int groups, int mode, int pass);
size_t convbn_grouped_saved_bytes(const convbn_desc *desc, int groups, int mode, int refold);
convbn_status convbn_grouped_tune_fwd(const convbn_desc *desc, int groups, const void *x, const void *W,
                                      const float *b, const float *gamma, const float *beta,
                                      const float *mean, const float *var, void *z, void *w_folded,
                                      void *ws, size_t ws_bytes, void *stream);
convbn_status convbn_grouped_tune_bwd(const convbn_desc *desc, int groups, const void *x, const void *W,
                                      const float *b, const float *gamma, const float *mean,
                                      const float *var, const void *w_folded, const void *dz, void *dx,
                                      void *dW, float *db, float *dgamma, float *dbeta, void *ws,
                                      size_t ws_bytes, void *stream);
convbn_status convbn_grouped_eval_fwd(const convbn_desc *desc, int groups, const void *x, const void *W,
                                      const float *b, const float *gamma, const float *beta,
                                      const float *mean, const float *var, void *z, void *y_saved,
                                      void *ws, size_t ws_bytes, void *stream);
convbn_status convbn_grouped_eval_bwd(const convbn_desc *desc, int groups, const void *x, const void *W,
                                      const float *b, const float *gamma, const float *mean,
                                      const float *var, const void *y_saved, const void *dz, void *dx,
                                      void *dW, float *db, float *dgamma, float *dbeta, void *ws,
                                      size_t ws_bytes, void *stream);

/* ---- The individual steps of the Tune-mode block (each is one kernel) -------------
 * convbn_tune_fwd is convbn_fold followed by convbn_conv_fprop; convbn_tune_bwd is
 * convbn_conv_dgrad, convbn_conv_wgrad and convbn_fold_back.  They are exported so that
 * each step can be checked and timed on its own.  Same conventions as above. */

/* Fold (Sec. 3.3):  w' = s w,  b' = (b - mu) s + beta,  s = gamma/sqrt(var+eps).
 *   out (each nullable = not wanted): w_fprop  w' as [Cout][kH][kW][Cin],
 *                                     w_folded w' as [Cin][kH][kW][Cout],
 *                                     b_folded [Cout] fp32. */
convbn_status convbn_fold(const convbn_desc *desc, const void *W, const float *b,
                          const float *gamma, const float *beta, const float *mean,
                          const float *var, void *w_fprop, void *w_folded, float *b_folded,
                          void *stream);

/* The folds of several blocks in ONE launch (Sec. 3.3: in Tune mode every training step starts by
 * folding each block's BatchNorm into its weights; a fold moves little data, so one launch per
 * block is bound by the launches).  Built for callers that own a whole network.
 *   convbn_fold_item: one block's convbn_fold arguments (device pointers; identity != 0 folds
 *     with s = 1, b' = b: the plain re-ordering of the weights the Eval-mode backward needs).
 *   convbn_fold_group_plan: HOST side.  Checks the n items (bf16 blocks with Cout and
 *     Cin*kH*kW multiples of 8; others are CONVBN_ERR_UNSUPPORTED: fold them with convbn_fold)
 *     and writes a table of convbn_fold_group_table_bytes(n) bytes into HOST memory
 *     `table_host`, and the launch size into *grid_blocks.  Launches nothing.  The caller
 *     copies the table to device memory (16-byte aligned) once; it stays valid while the
 *     pointers in the items do.
 *   convbn_fold_group: runs the table (`table_dev`, DEVICE memory) on `stream`; results are
 *     bit-identical to n convbn_fold calls. */
typedef struct {
  const convbn_desc *desc;
  const void *W;
  const float *b, *gamma, *beta, *mean, *var; /* b, beta nullable as for convbn_fold */
  void *w_fprop, *w_folded;                  /* each nullable = not wanted */
  float *b_folded;                           /* nullable */
  int32_t identity;
} convbn_fold_item;
size_t convbn_fold_group_table_bytes(int n);
convbn_status convbn_fold_group_plan(int n, const convbn_fold_item *items, void *table_host,
                                     size_t table_bytes, int *grid_blocks);
convbn_status convbn_fold_group(int n, const void *table_dev, int grid_blocks, void *stream);

/* 1 if convbn_tune_bwd computes this block's weight gradient and fold-back in one launch (deep 3x3
 * layers whose pixels need no split: the fp32 dw' never reaches memory), else 0.  A caller that groups
 * fold-backs (below) leaves such blocks to convbn_tune_bwd. */
int32_t convbn_tune_bwd_is_fused(const convbn_desc *desc);

/* The fold-backs of several blocks in ONE launch (Table 2 "Tune", last four lines: dW = s dw',
 * db = s r, dgamma = (<dw', w> + r (b - mu))/sqrt(var+eps), dbeta = r, for every block of the
 * group).  A fold-back moves little data, so one launch per block is bound by the launches.
 *   convbn_fold_back_item: one block's convbn_fold_back arguments (device pointers; dw_part and
 *     r_part as convbn_conv_wgrad leaves them).
 *   convbn_fold_back_group_plan: HOST side, like convbn_fold_group_plan.  Takes bf16 blocks
 *     whose Cin*kH*kW is a multiple of 4 (others: CONVBN_ERR_UNSUPPORTED).  Launches nothing.
 *   convbn_fold_back_group: runs the table on `stream`.  Same sums in the same order as
 *     convbn_fold_back's 256-thread kernel (the single call uses a 1024-thread kernel, whose
 *     partial sums are grouped differently, for blocks of at most 128 output channels with 16
 *     or more partial copies of short rows). */
typedef struct {
  const convbn_desc *desc;
  const float *dw_part, *r_part;
  const void *W;
  const float *b, *gamma, *mean, *var; /* b nullable */
  void *dW;
  float *db, *dgamma, *dbeta;          /* db NULL exactly when b is NULL */
} convbn_fold_back_item;
size_t convbn_fold_back_group_table_bytes(int n);
convbn_status convbn_fold_back_group_plan(int n, const convbn_fold_back_item *items,
                                          void *table_host, size_t table_bytes, int *grid_blocks);
convbn_status convbn_fold_back_group(int n, const void *table_dev, int grid_blocks, void *stream);

/* Workspace bytes convbn_conv_fprop (pass = CONVBN_PASS_FWD) or convbn_conv_dgrad /
 * convbn_conv_wgrad (CONVBN_PASS_BWD, enough for either) need; 0 for most shapes (then ws
 * may be NULL). */
size_t convbn_conv_workspace_bytes(const convbn_desc *desc, int pass);

/* Forward convolution  z = w (*) x + bias  (Sec. 3.1; cross-correlation, zero padding).
 *   w is [Cout][kH][kW][Cin]; bias [Cout] fp32, nullable. */
convbn_status convbn_conv_fprop(const convbn_desc *desc, const void *x, const void *w,
                                const float *bias, void *z, void *ws, size_t ws_bytes,
                                void *stream);

/* Input gradient  dx = w_rot (*) dz  (Sec. 3.2.1).  w_t is [Cin][kH][kW][Cout]. */
convbn_status convbn_conv_dgrad(const convbn_desc *desc, const void *dz, const void *w_t,
                                void *dx, void *ws, size_t ws_bytes, void *stream);
/* The same with the backward mask of a ReLU in front of the block (CONVBN_ACT_RELU_IN; desc->act itself is not
 * looked at here): dx = x > 0 ? (w_rot (*) dz) : 0, x being the block's input, laid out like dx. */
convbn_status convbn_conv_dgrad_masked(const convbn_desc *desc, const void *dz, const void *w_t,
                                       const void *x, void *dx, void *ws, size_t ws_bytes,
                                       void *stream);

/* Weight gradient  dw = dz (.) x  and  r_c = sum_{n,h,w} dz  (Sec. 3.2.1; App. B), left as
 * fp32 partial sums over slices of the output pixels:
 *   dw_part [convbn_wgrad_parts][Cout][kH][kW][Cin],  r_part [convbn_rsum_parts][Cout].
 * The true values are the sums over the leading index; convbn_fold_back adds them up. */
int32_t convbn_wgrad_parts(const convbn_desc *desc);
int32_t convbn_rsum_parts(const convbn_desc *desc);
/* r_part is nullable (then only the weight-gradient kernel runs). */
convbn_status convbn_conv_wgrad(const convbn_desc *desc, const void *x, const void *dz,
                                float *dw_part, float *r_part, void *ws, size_t ws_bytes,
                                void *stream);

/* Fold-back (Table 2, row "Tune", last four lines): from the partial sums of dw' and r,
 *   dW = s dw',  db = s r (nullable with b),  dgamma = (<dw'_c, w_c> + r_c (b_c - mu_c))/sqrt(var_c+eps),
 *   dbeta = r. */
convbn_status convbn_fold_back(const convbn_desc *desc, const float *dw_part, const float *r_part,
                               const void *W, const float *b, const float *gamma,
                               const float *mean, const float *var, void *dW, float *db,
                               float *dgamma, float *dbeta, void *stream);

/* ---- Glue between blocks (not part of the ConvBN block) ------------------------------
 * What follows a block does not change the block's computation (Sec. 3.1).  These three
 * calls exist only so that a whole backbone (ResNet-50: ReLU, residual add, 3x3/2 max-pool)
 * can be chained on the GPU for the end-to-end time / memory measurement (App. D).
 *   convbn_aux_eltwise, n elements, a is updated in place:
 *     op 0: a = max(a, 0)            op 1: a = b > 0 ? a : 0   (ReLU backward; b = ReLU output)
 *     op 2: a = max(a + b, 0)        op 3: a = a + b
 *   convbn_aux_maxpool_fwd: 3x3 window, stride 2, padding 1 over x [N][H][W][C] -> y
 *     [N][Ho][Wo][C], Ho = (H-1)/2+1; idx (one byte per output element) records the winner.
 *   convbn_aux_maxpool_bwd: dx [N][H][W][C] from dy and idx. */
convbn_status convbn_aux_eltwise(int op, int dtype, void *a, const void *b, size_t n, void *stream);
/* a = y > 0 ? a + b : 0 -- op 3 followed by op 1 (same rounding of the sum) in one pass: where the gradients of a
 * residual unit's two branches meet in front of the ReLU that produced y. */
convbn_status convbn_aux_add_relu_bwd(int dtype, void *a, const void *b, const void *y, size_t n,
                                      void *stream);
convbn_status convbn_aux_maxpool_fwd(int dtype, const void *x, void *y, void *idx, int32_t N,
                                     int32_t H, int32_t W, int32_t C, void *stream);
convbn_status convbn_aux_maxpool_bwd(int dtype, const void *dy, const void *idx, void *dx,
                                     int32_t N, int32_t H, int32_t W, int32_t C, void *stream);

/* Bytes a block must keep alive between its forward and its backward call in
 * addition to X (App. K.1): Eval keeps Y (N Cout Hout Wout elements); Tune keeps
 * w' (kH kW Cin Cout elements), or nothing when `refold` is non-zero. */
size_t convbn_saved_bytes(const convbn_desc *desc, int mode, int refold);

/* Human-readable description of the last error on the calling thread
 * (thread-local static storage; valid until the next failing call). */
const char *convbn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CONVBN_H_ */
