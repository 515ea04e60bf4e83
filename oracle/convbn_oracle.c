/*
 * CPU oracle for the ConvBN block (frozen BatchNorm), forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition the
 * GPU library is checked against.  It shares no code with the HIP path and must
 * never be called from it; only the tests, the smoke check and the CPU-baseline
 * leg of the benchmark may load it.
 *
 * Everything is double precision, logical NCHW indexing on dense row-major
 * arrays:  X[N][Cin][Hin][Win], W[Cout][Cin][kH][kW], Y/Z/G[N][Cout][Hout][Wout],
 * and per-channel vectors of length Cout.  "conv" is cross-correlation with zero
 * padding, dilation 1, groups 1 (the deep-learning convention; Sec. 3.1 writes
 * Y = w (*) X + b and Sec. 3.2.1 takes the rotated kernel for the input
 * gradient, which is the adjoint of cross-correlation).
 *
 * Two independent routes are provided:
 *   Eval mode  (Sec. 3.1; App. C "Eval Mode"; Table 2 row "Eval"):
 *       Y = w (*) X + b;  Z = gamma (Y - mu)/sqrt(var+eps) + beta,
 *       backward derived from those two lines with the broadcast sums of
 *       App. B written out.  This is the DEFINITION the GPU is compared with.
 *   Tune mode  (Sec. 3.3 definitions of w', b'; Table 2 row "Tune"):
 *       fold, one convolution, six backward equations.  Present only so the
 *       test-suite can assert Tune == Eval (Sec. 3.4.1) inside the oracle.
 *
 * The same two routes exist for the TransposedConv-BN block, for the depthwise
 * ConvBN block and for the grouped ConvBN block (end of file), pinned by identities
 * against the convolution above (adjoint; block-diagonal dense weight), a library
 * cross-check, finite differences and Tune == Eval.
 *
 * Parity pins (tests marked "not gpu"): library conv2d+batch_norm with autograd
 * on the CPU as an independent special-case check, 1x1 == matrix product,
 * delta kernel, single-pixel impulse response, central finite differences for
 * every gradient, the adjoint identities, and Tune == Eval.
 *
 * OpenMP is used only over independent output indices; there is no blocking,
 * no reordering and no vector intrinsics.
 */
#include <math.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int N, Cin, Hin, Win;
  int Cout, kH, kW;
  int sh, sw, ph, pw;
} cb_dims;

/* floor((in + 2p - k)/s) + 1 : the usual output-size rule (paper is silent). */
static int out_size(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

int cbo_hout(const cb_dims *d) { return out_size(d->Hin, d->kH, d->sh, d->ph); }
int cbo_wout(const cb_dims *d) { return out_size(d->Win, d->kW, d->sw, d->pw); }

int cbo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

#define XI(n, c, h, w) ((((size_t)(n) * d->Cin + (c)) * d->Hin + (h)) * d->Win + (w))
#define WI(o, c, i, j) ((((size_t)(o) * d->Cin + (c)) * d->kH + (i)) * d->kW + (j))
#define YI(n, o, h, w) ((((size_t)(n) * d->Cout + (o)) * Ho + (h)) * Wo + (w))

/* Y = w (*) X + b      (Sec. 3.1; Sec. 3.2.1).  b may be NULL (= 0). */
void cbo_conv_fwd(const cb_dims *d, const double *X, const double *W, const double *b, double *Y) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o)
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          double acc = b ? b[o] : 0.0;
          for (int c = 0; c < d->Cin; ++c)
            for (int i = 0; i < d->kH; ++i) {
              const int h = ho * d->sh + i - d->ph;
              if (h < 0 || h >= d->Hin) continue;
              for (int j = 0; j < d->kW; ++j) {
                const int w = wo * d->sw + j - d->pw;
                if (w < 0 || w >= d->Win) continue;
                acc += W[WI(o, c, i, j)] * X[XI(n, c, h, w)];
              }
            }
          Y[YI(n, o, ho, wo)] = acc;
        }
}

/* dJ/dX = w_rot (*) dJ/dY  (Sec. 3.2.1), written as the transpose of the forward
 * loop: every forward read of X[n,c,h,w] with weight W[o,c,i,j] into Y[n,o,ho,wo]
 * becomes an accumulation of W * dY into dX at the same indices. */
void cbo_conv_dgrad(const cb_dims *d, const double *W, const double *dY, double *dX) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  memset(dX, 0, sizeof(double) * (size_t)d->N * d->Cin * d->Hin * d->Win);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int c = 0; c < d->Cin; ++c)
      for (int o = 0; o < d->Cout; ++o)
        for (int ho = 0; ho < Ho; ++ho)
          for (int wo = 0; wo < Wo; ++wo) {
            const double g = dY[YI(n, o, ho, wo)];
            for (int i = 0; i < d->kH; ++i) {
              const int h = ho * d->sh + i - d->ph;
              if (h < 0 || h >= d->Hin) continue;
              for (int j = 0; j < d->kW; ++j) {
                const int w = wo * d->sw + j - d->pw;
                if (w < 0 || w >= d->Win) continue;
                dX[XI(n, c, h, w)] += W[WI(o, c, i, j)] * g;
              }
            }
          }
}

/* dJ/dw = dJ/dY (.) X  (cross-correlation of the output gradient with the
 * padded input, Sec. 3.2.1), summed over the batch. */
void cbo_conv_wgrad(const cb_dims *d, const double *X, const double *dY, double *dW) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int o = 0; o < d->Cout; ++o)
    for (int c = 0; c < d->Cin; ++c)
      for (int i = 0; i < d->kH; ++i)
        for (int j = 0; j < d->kW; ++j) {
          double acc = 0.0;
          for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho) {
              const int h = ho * d->sh + i - d->ph;
              if (h < 0 || h >= d->Hin) continue;
              for (int wo = 0; wo < Wo; ++wo) {
                const int w = wo * d->sw + j - d->pw;
                if (w < 0 || w >= d->Win) continue;
                acc += dY[YI(n, o, ho, wo)] * X[XI(n, c, h, w)];
              }
            }
          dW[WI(o, c, i, j)] = acc;
        }
}

/* Per-channel sum over N, Hout, Wout: the backward of a [Cout] -> [N,Cout,H,W]
 * broadcast (App. B).  If T is non-NULL the summand is A*T elementwise. */
static void channel_sum(const cb_dims *d, const double *A, const double *T, double *out) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
#pragma omp parallel for schedule(static)
  for (int o = 0; o < d->Cout; ++o) {
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          acc += T ? A[idx] * T[idx] : A[idx];
        }
    out[o] = acc;
  }
}

/* ------------------------------------------------------------------ Eval --- */

/* Eval forward (Sec. 3.1; App. C "Eval Mode"):
 *   Y = w (*) X + b ;  Ybar = (Y - mu)/sqrt(var + eps) ;  Z = gamma*Ybar + beta.
 * Y (the tensor Eval mode keeps for backward) and Z are both returned. */
void cbo_eval_fwd(const cb_dims *d, const double *X, const double *W, const double *b,
                  const double *gamma, const double *beta, const double *mu, const double *var,
                  double eps, double *Y, double *Z) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  cbo_conv_fwd(d, X, W, b, Y);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          const double ybar = (Y[idx] - mu[o]) / sd;
          Z[idx] = gamma[o] * ybar + beta[o];
        }
    }
}

/* Eval backward (Table 2, row "Eval", with App. B's sums restored).  G = dJ/dZ.
 *   dY     = gamma/sqrt(var+eps) * G
 *   dX     = w_rot (*) dY
 *   dW     = dY (.) X
 *   db     = sum dY                       (only if db != NULL)
 *   dgamma = sum G * (Y - mu)/sqrt(var+eps)
 *   dbeta  = sum G
 * scratch_dY must hold N*Cout*Hout*Wout doubles. */
void cbo_eval_bwd(const cb_dims *d, const double *X, const double *W, const double *gamma,
                  const double *mu, const double *var, double eps, const double *Y,
                  const double *G, double *scratch_dY, double *dX, double *dW, double *db,
                  double *dgamma, double *dbeta) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  double *dY = scratch_dY;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          dY[idx] = gamma[o] / sd * G[idx];
        }
    }
  if (dX) cbo_conv_dgrad(d, W, dY, dX);
  cbo_conv_wgrad(d, X, dY, dW);
  if (db) channel_sum(d, dY, NULL, db);
  /* dgamma: sum over the broadcast dims of G * Ybar */
#pragma omp parallel for schedule(static)
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          acc += G[idx] * ((Y[idx] - mu[o]) / sd);
        }
    dgamma[o] = acc;
  }
  channel_sum(d, G, NULL, dbeta);
}

/* ------------------------------------------------------------------ Tune --- */

/* Fold (Sec. 3.3):  w' = gamma/sqrt(var+eps) * w  (per output channel),
 *                   b' = (b - mu) * gamma/sqrt(var+eps) + beta.   b may be NULL. */
void cbo_fold(const cb_dims *d, const double *W, const double *b, const double *gamma,
              const double *beta, const double *mu, const double *var, double eps, double *Wf,
              double *bf) {
  const size_t row = (size_t)d->Cin * d->kH * d->kW;
  for (int o = 0; o < d->Cout; ++o) {
    const double s = gamma[o] / sqrt(var[o] + eps);
    for (size_t t = 0; t < row; ++t) Wf[o * row + t] = s * W[o * row + t];
    bf[o] = ((b ? b[o] : 0.0) - mu[o]) * s + beta[o];
  }
}

/* Tune forward (Sec. 3.4: fold on every call, then one convolution). */
void cbo_tune_fwd(const cb_dims *d, const double *X, const double *W, const double *b,
                  const double *gamma, const double *beta, const double *mu, const double *var,
                  double eps, double *Wf, double *bf, double *Z) {
  cbo_fold(d, W, b, gamma, beta, mu, var, eps, Wf, bf);
  cbo_conv_fwd(d, X, Wf, bf, Z);
}

/* Tune backward (Table 2, row "Tune").  Needs X and w' only (no Y).
 *   dX     = w'_rot (*) G
 *   dW'    = G (.) X                        (returned in dWf)
 *   dW     = gamma/sqrt(var+eps) * dW'
 *   db     = gamma/sqrt(var+eps) * sum G
 *   dgamma = <dW', w>/sqrt(var+eps) + (sum G)(b - mu)/sqrt(var+eps)
 *   dbeta  = sum G */
void cbo_tune_bwd(const cb_dims *d, const double *X, const double *W, const double *b,
                  const double *gamma, const double *mu, const double *var, double eps,
                  const double *Wf, const double *G, double *dX, double *dWf, double *dW,
                  double *db, double *dgamma, double *dbeta) {
  const size_t row = (size_t)d->Cin * d->kH * d->kW;
  if (dX) cbo_conv_dgrad(d, Wf, G, dX);
  cbo_conv_wgrad(d, X, G, dWf);
  channel_sum(d, G, NULL, dbeta);
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    const double s = gamma[o] / sd;
    double dot = 0.0;
    for (size_t t = 0; t < row; ++t) {
      dW[o * row + t] = s * dWf[o * row + t];
      dot += dWf[o * row + t] * W[o * row + t];
    }
    const double r = dbeta[o];
    if (db) db[o] = s * r;
    dgamma[o] = dot / sd + r * ((b ? b[o] : 0.0) - mu[o]) / sd;
  }
}

/* ------------------------------------------------- transposed convolution --- */
/*
 * TransposedConv-BN block (Sec. 3.2.1, closing remark: the associative law
 * gamma . (w (*) X) = (gamma . w) (*) X also holds for transposed convolution,
 * so Tune mode applies to it).  The paper gives no formula for the operator;
 * the usual definition is taken: a transposed convolution is the adjoint of the
 * cross-correlation of Sec. 3.1 with respect to its input.  The weight is
 * W[Cin][Cout][kH][kW], the BatchNorm acts on the Cout output channels, and
 *   Y[n,o,h*sh - ph + i, w*sw - pw + j] += W[c,o,i,j] * X[n,c,h,w]   (+ b[o]),
 * with Hout = (Hin-1) sh - 2 ph + kH (no output padding, dilation 1, groups 1).
 * The cb_dims fields keep their names: Cin/Hin/Win describe X, Cout the output.
 */
int cbo_thout(const cb_dims *d) { return (d->Hin - 1) * d->sh - 2 * d->ph + d->kH; }
int cbo_twout(const cb_dims *d) { return (d->Win - 1) * d->sw - 2 * d->pw + d->kW; }

#define TWI(c, o, i, j) ((((size_t)(c) * d->Cout + (o)) * d->kH + (i)) * d->kW + (j))

/* Y = transposed convolution of X with W (+ b): every input pixel spreads a
 * kernel-shaped patch into the output.  One thread owns one (n, o) plane. */
void cbo_tconv_fwd(const cb_dims *d, const double *X, const double *W, const double *b, double *Y) {
  const int Ho = cbo_thout(d), Wo = cbo_twout(d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) Y[YI(n, o, ho, wo)] = b ? b[o] : 0.0;
      for (int c = 0; c < d->Cin; ++c)
        for (int h = 0; h < d->Hin; ++h)
          for (int w = 0; w < d->Win; ++w) {
            const double x = X[XI(n, c, h, w)];
            for (int i = 0; i < d->kH; ++i) {
              const int ho = h * d->sh - d->ph + i;
              if (ho < 0 || ho >= Ho) continue;
              for (int j = 0; j < d->kW; ++j) {
                const int wo = w * d->sw - d->pw + j;
                if (wo < 0 || wo >= Wo) continue;
                Y[YI(n, o, ho, wo)] += W[TWI(c, o, i, j)] * x;
              }
            }
          }
    }
}

/* dJ/dX of the transposed convolution: each X[n,c,h,w] entered Y[n,o,ho,wo] with
 * weight W[c,o,i,j], so it collects W * dY over the same index pairs. */
void cbo_tconv_dgrad(const cb_dims *d, const double *W, const double *dY, double *dX) {
  const int Ho = cbo_thout(d), Wo = cbo_twout(d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int c = 0; c < d->Cin; ++c)
      for (int h = 0; h < d->Hin; ++h)
        for (int w = 0; w < d->Win; ++w) {
          double acc = 0.0;
          for (int o = 0; o < d->Cout; ++o)
            for (int i = 0; i < d->kH; ++i) {
              const int ho = h * d->sh - d->ph + i;
              if (ho < 0 || ho >= Ho) continue;
              for (int j = 0; j < d->kW; ++j) {
                const int wo = w * d->sw - d->pw + j;
                if (wo < 0 || wo >= Wo) continue;
                acc += W[TWI(c, o, i, j)] * dY[YI(n, o, ho, wo)];
              }
            }
          dX[XI(n, c, h, w)] = acc;
        }
}

/* dJ/dW of the transposed convolution, summed over the batch and all positions. */
void cbo_tconv_wgrad(const cb_dims *d, const double *X, const double *dY, double *dW) {
  const int Ho = cbo_thout(d), Wo = cbo_twout(d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int c = 0; c < d->Cin; ++c)
    for (int o = 0; o < d->Cout; ++o)
      for (int i = 0; i < d->kH; ++i)
        for (int j = 0; j < d->kW; ++j) {
          double acc = 0.0;
          for (int n = 0; n < d->N; ++n)
            for (int h = 0; h < d->Hin; ++h) {
              const int ho = h * d->sh - d->ph + i;
              if (ho < 0 || ho >= Ho) continue;
              for (int w = 0; w < d->Win; ++w) {
                const int wo = w * d->sw - d->pw + j;
                if (wo < 0 || wo >= Wo) continue;
                acc += X[XI(n, c, h, w)] * dY[YI(n, o, ho, wo)];
              }
            }
          dW[TWI(c, o, i, j)] = acc;
        }
}

/* Per-channel sum of A (times T if given) over a [N][Cout][Ho][Wo] tensor. */
static void plane_sum(const cb_dims *d, int Ho, int Wo, const double *A, const double *T, double *out) {
#pragma omp parallel for schedule(static)
  for (int o = 0; o < d->Cout; ++o) {
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          acc += T ? A[idx] * T[idx] : A[idx];
        }
    out[o] = acc;
  }
}

/* Eval mode of the transposed block: Y = tconv(X, W) + b kept, then the frozen
 * BatchNorm of Sec. 3.1 on the Cout channels.  This is the definition. */
void cbo_teval_fwd(const cb_dims *d, const double *X, const double *W, const double *b,
                   const double *gamma, const double *beta, const double *mu, const double *var,
                   double eps, double *Y, double *Z) {
  const int Ho = cbo_thout(d), Wo = cbo_twout(d);
  cbo_tconv_fwd(d, X, W, b, Y);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          Z[idx] = gamma[o] * ((Y[idx] - mu[o]) / sd) + beta[o];
        }
    }
}

/* Eval backward of the transposed block (Table 2 row "Eval" with the transposed
 * operator in place of the convolution).  scratch_dY: N*Cout*Hout*Wout doubles. */
void cbo_teval_bwd(const cb_dims *d, const double *X, const double *W, const double *gamma,
                   const double *mu, const double *var, double eps, const double *Y,
                   const double *G, double *scratch_dY, double *dX, double *dW, double *db,
                   double *dgamma, double *dbeta) {
  const int Ho = cbo_thout(d), Wo = cbo_twout(d);
  double *dY = scratch_dY;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          dY[idx] = gamma[o] / sd * G[idx];
        }
    }
  if (dX) cbo_tconv_dgrad(d, W, dY, dX);
  cbo_tconv_wgrad(d, X, dY, dW);
  if (db) plane_sum(d, Ho, Wo, dY, NULL, db);
#pragma omp parallel for schedule(static)
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          acc += G[idx] * ((Y[idx] - mu[o]) / sd);
        }
    dgamma[o] = acc;
  }
  plane_sum(d, Ho, Wo, G, NULL, dbeta);
}

/* Tune mode of the transposed block (Sec. 3.3 with the scale on the weight's
 * output-channel index, which is its second one here): fold, one transposed
 * convolution, and Table 2's "Tune" backward lines with the sums of <dW', w>
 * running over (Cin, kH, kW) for each output channel. */
void cbo_tfold(const cb_dims *d, const double *W, const double *b, const double *gamma,
               const double *beta, const double *mu, const double *var, double eps, double *Wf,
               double *bf) {
  for (int o = 0; o < d->Cout; ++o) {
    const double s = gamma[o] / sqrt(var[o] + eps);
    for (int c = 0; c < d->Cin; ++c)
      for (int i = 0; i < d->kH; ++i)
        for (int j = 0; j < d->kW; ++j) Wf[TWI(c, o, i, j)] = s * W[TWI(c, o, i, j)];
    bf[o] = ((b ? b[o] : 0.0) - mu[o]) * s + beta[o];
  }
}

void cbo_ttune_fwd(const cb_dims *d, const double *X, const double *W, const double *b,
                   const double *gamma, const double *beta, const double *mu, const double *var,
                   double eps, double *Wf, double *bf, double *Z) {
  cbo_tfold(d, W, b, gamma, beta, mu, var, eps, Wf, bf);
  cbo_tconv_fwd(d, X, Wf, bf, Z);
}

void cbo_ttune_bwd(const cb_dims *d, const double *X, const double *W, const double *b,
                   const double *gamma, const double *mu, const double *var, double eps,
                   const double *Wf, const double *G, double *dX, double *dWf, double *dW,
                   double *db, double *dgamma, double *dbeta) {
  const int Ho = cbo_thout(d), Wo = cbo_twout(d);
  if (dX) cbo_tconv_dgrad(d, Wf, G, dX);
  cbo_tconv_wgrad(d, X, G, dWf);
  plane_sum(d, Ho, Wo, G, NULL, dbeta);
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    const double s = gamma[o] / sd;
    double dot = 0.0;
    for (int c = 0; c < d->Cin; ++c)
      for (int i = 0; i < d->kH; ++i)
        for (int j = 0; j < d->kW; ++j) {
          const size_t t = TWI(c, o, i, j);
          dW[t] = s * dWf[t];
          dot += dWf[t] * W[t];
        }
    const double r = dbeta[o];
    if (db) db[o] = s * r;
    dgamma[o] = dot / sd + r * ((b ? b[o] : 0.0) - mu[o]) / sd;
  }
}

/* --------------------------------------------------- depthwise convolution --- */
/*
 * Depthwise ConvBN block: a convolution with as many groups as channels (every
 * output channel sees only its own input channel), followed by the frozen
 * BatchNorm of Sec. 3.1.  The scale of Sec. 3.3 is per output channel, so the fold
 * is unchanged; only the contraction differs (the experiments' GhostNet / MobileNet
 * style layers, Sec. 4).  W is [C][kH][kW]; cb_dims.Cin == cb_dims.Cout == C.
 *   Y[n,c,ho,wo] = b[c] + sum_{i,j} W[c,i,j] X[n,c,ho sh + i - ph, wo sw + j - pw]
 */
#define DWI(c, i, j) (((size_t)(c) * d->kH + (i)) * d->kW + (j))

void cbo_dw_fwd(const cb_dims *d, const double *X, const double *W, const double *b, double *Y) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int c = 0; c < d->Cout; ++c)
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          double acc = b ? b[c] : 0.0;
          for (int i = 0; i < d->kH; ++i) {
            const int h = ho * d->sh + i - d->ph;
            if (h < 0 || h >= d->Hin) continue;
            for (int j = 0; j < d->kW; ++j) {
              const int w = wo * d->sw + j - d->pw;
              if (w < 0 || w >= d->Win) continue;
              acc += W[DWI(c, i, j)] * X[XI(n, c, h, w)];
            }
          }
          Y[YI(n, c, ho, wo)] = acc;
        }
}

/* dJ/dX: the transpose of the loop above (scatter form, one thread per (n, c) plane). */
void cbo_dw_dgrad(const cb_dims *d, const double *W, const double *dY, double *dX) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  memset(dX, 0, sizeof(double) * (size_t)d->N * d->Cin * d->Hin * d->Win);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int c = 0; c < d->Cout; ++c)
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          const double g = dY[YI(n, c, ho, wo)];
          for (int i = 0; i < d->kH; ++i) {
            const int h = ho * d->sh + i - d->ph;
            if (h < 0 || h >= d->Hin) continue;
            for (int j = 0; j < d->kW; ++j) {
              const int w = wo * d->sw + j - d->pw;
              if (w < 0 || w >= d->Win) continue;
              dX[XI(n, c, h, w)] += W[DWI(c, i, j)] * g;
            }
          }
        }
}

void cbo_dw_wgrad(const cb_dims *d, const double *X, const double *dY, double *dW) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
#pragma omp parallel for schedule(static)
  for (int c = 0; c < d->Cout; ++c)
    for (int i = 0; i < d->kH; ++i)
      for (int j = 0; j < d->kW; ++j) {
        double acc = 0.0;
        for (int n = 0; n < d->N; ++n)
          for (int ho = 0; ho < Ho; ++ho) {
            const int h = ho * d->sh + i - d->ph;
            if (h < 0 || h >= d->Hin) continue;
            for (int wo = 0; wo < Wo; ++wo) {
              const int w = wo * d->sw + j - d->pw;
              if (w < 0 || w >= d->Win) continue;
              acc += dY[YI(n, c, ho, wo)] * X[XI(n, c, h, w)];
            }
          }
        dW[DWI(c, i, j)] = acc;
      }
}

/* Eval mode (the definition) and Tune mode (Sec. 3.3, Table 2 "Tune") of the depthwise block. */
void cbo_dw_eval_fwd(const cb_dims *d, const double *X, const double *W, const double *b,
                     const double *gamma, const double *beta, const double *mu, const double *var,
                     double eps, double *Y, double *Z) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  cbo_dw_fwd(d, X, W, b, Y);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          Z[idx] = gamma[o] * ((Y[idx] - mu[o]) / sd) + beta[o];
        }
    }
}

void cbo_dw_eval_bwd(const cb_dims *d, const double *X, const double *W, const double *gamma,
                     const double *mu, const double *var, double eps, const double *Y,
                     const double *G, double *scratch_dY, double *dX, double *dW, double *db,
                     double *dgamma, double *dbeta) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  double *dY = scratch_dY;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          dY[idx] = gamma[o] / sd * G[idx];
        }
    }
  if (dX) cbo_dw_dgrad(d, W, dY, dX);
  cbo_dw_wgrad(d, X, dY, dW);
  if (db) plane_sum(d, Ho, Wo, dY, NULL, db);
#pragma omp parallel for schedule(static)
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          acc += G[idx] * ((Y[idx] - mu[o]) / sd);
        }
    dgamma[o] = acc;
  }
  plane_sum(d, Ho, Wo, G, NULL, dbeta);
}

void cbo_dw_tune_fwd(const cb_dims *d, const double *X, const double *W, const double *b,
                     const double *gamma, const double *beta, const double *mu, const double *var,
                     double eps, double *Wf, double *bf, double *Z) {
  const size_t row = (size_t)d->kH * d->kW;
  for (int c = 0; c < d->Cout; ++c) {
    const double s = gamma[c] / sqrt(var[c] + eps);
    for (size_t t = 0; t < row; ++t) Wf[c * row + t] = s * W[c * row + t];
    bf[c] = ((b ? b[c] : 0.0) - mu[c]) * s + beta[c];
  }
  cbo_dw_fwd(d, X, Wf, bf, Z);
}

void cbo_dw_tune_bwd(const cb_dims *d, const double *X, const double *W, const double *b,
                     const double *gamma, const double *mu, const double *var, double eps,
                     const double *Wf, const double *G, double *dX, double *dWf, double *dW,
                     double *db, double *dgamma, double *dbeta) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  const size_t row = (size_t)d->kH * d->kW;
  if (dX) cbo_dw_dgrad(d, Wf, G, dX);
  cbo_dw_wgrad(d, X, G, dWf);
  plane_sum(d, Ho, Wo, G, NULL, dbeta);
  for (int c = 0; c < d->Cout; ++c) {
    const double sd = sqrt(var[c] + eps);
    const double s = gamma[c] / sd;
    double dot = 0.0;
    for (size_t t = 0; t < row; ++t) {
      dW[c * row + t] = s * dWf[c * row + t];
      dot += dWf[c * row + t] * W[c * row + t];
    }
    const double r = dbeta[c];
    if (db) db[c] = s * r;
    dgamma[c] = dot / sd + r * ((b ? b[c] : 0.0) - mu[c]) / sd;
  }
}

/* ------------------------------------------------------ grouped convolution --- */
/*
 * Grouped ConvBN block: the channels are split into `groups` equal parts and every
 * output channel sees only the input channels of its own part (the ResNeXt / RegNet
 * style layers among the experiments' models, Sec. 4 and App. E).  The BatchNorm of
 * Sec. 3.1 and the per-output-channel scale of Sec. 3.3 are unchanged; only the
 * contraction differs.  With cg = Cin / groups and og = Cout / groups, W is
 * [Cout][cg][kH][kW] and output channel o reads input channels (o / og) cg .. + cg - 1:
 *   Y[n,o,ho,wo] = b[o] + sum_{q<cg,i,j} W[o,q,i,j] X[n,(o/og) cg + q, ho sh + i - ph, wo sw + j - pw]
 */
#define GWI(o, q, i, j) ((((size_t)(o) * cg + (q)) * d->kH + (i)) * d->kW + (j))

void cbo_g_fwd(const cb_dims *d, int groups, const double *X, const double *W, const double *b, double *Y) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  const int cg = d->Cin / groups, og = d->Cout / groups;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o)
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo) {
          double acc = b ? b[o] : 0.0;
          const int c0 = (o / og) * cg;
          for (int q = 0; q < cg; ++q)
            for (int i = 0; i < d->kH; ++i) {
              const int h = ho * d->sh + i - d->ph;
              if (h < 0 || h >= d->Hin) continue;
              for (int j = 0; j < d->kW; ++j) {
                const int w = wo * d->sw + j - d->pw;
                if (w < 0 || w >= d->Win) continue;
                acc += W[GWI(o, q, i, j)] * X[XI(n, c0 + q, h, w)];
              }
            }
          Y[YI(n, o, ho, wo)] = acc;
        }
}

/* dJ/dX: the transpose of the loop above (scatter form; one thread per (n, group): the
 * input channels of a group receive contributions from that group's outputs only). */
void cbo_g_dgrad(const cb_dims *d, int groups, const double *W, const double *dY, double *dX) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  const int cg = d->Cin / groups, og = d->Cout / groups;
  memset(dX, 0, sizeof(double) * (size_t)d->N * d->Cin * d->Hin * d->Win);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int g = 0; g < groups; ++g)
      for (int oo = 0; oo < og; ++oo) {
        const int o = g * og + oo;
        for (int ho = 0; ho < Ho; ++ho)
          for (int wo = 0; wo < Wo; ++wo) {
            const double gy = dY[YI(n, o, ho, wo)];
            for (int q = 0; q < cg; ++q)
              for (int i = 0; i < d->kH; ++i) {
                const int h = ho * d->sh + i - d->ph;
                if (h < 0 || h >= d->Hin) continue;
                for (int j = 0; j < d->kW; ++j) {
                  const int w = wo * d->sw + j - d->pw;
                  if (w < 0 || w >= d->Win) continue;
                  dX[XI(n, g * cg + q, h, w)] += W[GWI(o, q, i, j)] * gy;
                }
              }
          }
      }
}

void cbo_g_wgrad(const cb_dims *d, int groups, const double *X, const double *dY, double *dW) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  const int cg = d->Cin / groups, og = d->Cout / groups;
#pragma omp parallel for collapse(2) schedule(static)
  for (int o = 0; o < d->Cout; ++o)
    for (int q = 0; q < cg; ++q)
      for (int i = 0; i < d->kH; ++i)
        for (int j = 0; j < d->kW; ++j) {
          const int c = (o / og) * cg + q;
          double acc = 0.0;
          for (int n = 0; n < d->N; ++n)
            for (int ho = 0; ho < Ho; ++ho) {
              const int h = ho * d->sh + i - d->ph;
              if (h < 0 || h >= d->Hin) continue;
              for (int wo = 0; wo < Wo; ++wo) {
                const int w = wo * d->sw + j - d->pw;
                if (w < 0 || w >= d->Win) continue;
                acc += dY[YI(n, o, ho, wo)] * X[XI(n, c, h, w)];
              }
            }
          dW[GWI(o, q, i, j)] = acc;
        }
}

/* Eval mode (the definition) and Tune mode (Sec. 3.3, Table 2 "Tune") of the grouped block. */
void cbo_g_eval_fwd(const cb_dims *d, int groups, const double *X, const double *W, const double *b,
                    const double *gamma, const double *beta, const double *mu, const double *var,
                    double eps, double *Y, double *Z) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  cbo_g_fwd(d, groups, X, W, b, Y);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          Z[idx] = gamma[o] * ((Y[idx] - mu[o]) / sd) + beta[o];
        }
    }
}

void cbo_g_eval_bwd(const cb_dims *d, int groups, const double *X, const double *W, const double *gamma,
                    const double *mu, const double *var, double eps, const double *Y,
                    const double *G, double *scratch_dY, double *dX, double *dW, double *db,
                    double *dgamma, double *dbeta) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  double *dY = scratch_dY;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->Cout; ++o) {
      const double sd = sqrt(var[o] + eps);
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          dY[idx] = gamma[o] / sd * G[idx];
        }
    }
  if (dX) cbo_g_dgrad(d, groups, W, dY, dX);
  cbo_g_wgrad(d, groups, X, dY, dW);
  if (db) plane_sum(d, Ho, Wo, dY, NULL, db);
#pragma omp parallel for schedule(static)
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n)
      for (int h = 0; h < Ho; ++h)
        for (int w = 0; w < Wo; ++w) {
          const size_t idx = YI(n, o, h, w);
          acc += G[idx] * ((Y[idx] - mu[o]) / sd);
        }
    dgamma[o] = acc;
  }
  plane_sum(d, Ho, Wo, G, NULL, dbeta);
}

void cbo_g_tune_fwd(const cb_dims *d, int groups, const double *X, const double *W, const double *b,
                    const double *gamma, const double *beta, const double *mu, const double *var,
                    double eps, double *Wf, double *bf, double *Z) {
  const size_t row = (size_t)(d->Cin / groups) * d->kH * d->kW;
  for (int o = 0; o < d->Cout; ++o) {
    const double s = gamma[o] / sqrt(var[o] + eps);
    for (size_t t = 0; t < row; ++t) Wf[o * row + t] = s * W[o * row + t];
    bf[o] = ((b ? b[o] : 0.0) - mu[o]) * s + beta[o];
  }
  cbo_g_fwd(d, groups, X, Wf, bf, Z);
}

void cbo_g_tune_bwd(const cb_dims *d, int groups, const double *X, const double *W, const double *b,
                    const double *gamma, const double *mu, const double *var, double eps,
                    const double *Wf, const double *G, double *dX, double *dWf, double *dW,
                    double *db, double *dgamma, double *dbeta) {
  const int Ho = cbo_hout(d), Wo = cbo_wout(d);
  const size_t row = (size_t)(d->Cin / groups) * d->kH * d->kW;
  if (dX) cbo_g_dgrad(d, groups, Wf, G, dX);
  cbo_g_wgrad(d, groups, X, G, dWf);
  plane_sum(d, Ho, Wo, G, NULL, dbeta);
  for (int o = 0; o < d->Cout; ++o) {
    const double sd = sqrt(var[o] + eps);
    const double s = gamma[o] / sd;
    double dot = 0.0;
    for (size_t t = 0; t < row; ++t) {
      dW[o * row + t] = s * dWf[o * row + t];
      dot += dWf[o * row + t] * W[o * row + t];
    }
    const double r = dbeta[o];
    if (db) db[o] = s * r;
    dgamma[o] = dot / sd + r * ((b ? b[o] : 0.0) - mu[o]) / sd;
  }
}
