/* cnnk_ref: fp64 CPU oracle of one CNN training step.  TEST INFRASTRUCTURE ONLY.
 *
 * The paper's Algorithm 1 (inner loop) says no more than: forward pass, loss, backward pass,
 * theta <- theta - eta * grad.  Each function below is therefore the textbook definition of
 * the operator written out as direct loops in double precision, with no blocking, fusion or
 * reordering, so that it can be checked against the definition by eye.  OpenMP only splits
 * independent output elements across threads; every output element is summed by one thread in
 * a fixed order.
 */
#include "cnnk_ref.h"
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int out_size(int H, int pad, int R, int stride) { return (H + 2 * pad - R) / stride + 1; }

int cnnk_ref_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Forward pass, convolution layer (Algorithm 1, "perform forward pass"):
 * y[n,ho,wo,k] = sum_{r,s,c} x[n, ho*st+r-p, wo*st+s-p, c] * w[k,r,s,c], zero outside the image. */
int cnnk_ref_conv2d_fwd(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                        const double* x, const double* w, double* y) {
  if (!x || !w || !y) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return 2;
  const int Ho = out_size(H, pad, R, stride), Wo = out_size(W, pad, S, stride);
  if (Ho <= 0 || Wo <= 0) return 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int k = 0; k < Cout; ++k) {
          double acc = 0.0;
          for (int r = 0; r < R; ++r) {
            const int hi = ho * stride + r - pad;
            if (hi < 0 || hi >= H) continue;
            for (int s = 0; s < S; ++s) {
              const int wi = wo * stride + s - pad;
              if (wi < 0 || wi >= W) continue;
              const double* xp = x + (((size_t)n * H + hi) * W + wi) * Cin;
              const double* wp = w + (((size_t)k * R + r) * S + s) * Cin;
              for (int c = 0; c < Cin; ++c) acc += xp[c] * wp[c];
            }
          }
          y[(((size_t)n * Ho + ho) * Wo + wo) * Cout + k] = acc;
        }
  return 0;
}

/* Backward pass, gradient w.r.t. the convolution input:
 * dx[n,h,w,c] = sum_{k,r,s} dy[n,(h+p-r)/st,(w+p-s)/st,k] * w[k,r,s,c]
 * over those (r,s) for which both quotients are integers inside the output image. */
int cnnk_ref_conv2d_dgrad(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                          const double* dy, const double* w, double* dx) {
  if (!dy || !w || !dx) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return 2;
  const int Ho = out_size(H, pad, R, stride), Wo = out_size(W, pad, S, stride);
  if (Ho <= 0 || Wo <= 0) return 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int h = 0; h < H; ++h)
      for (int ww = 0; ww < W; ++ww)
        for (int c = 0; c < Cin; ++c) {
          double acc = 0.0;
          for (int k = 0; k < Cout; ++k)
            for (int r = 0; r < R; ++r) {
              const int th = h + pad - r;
              if (th < 0 || th % stride != 0) continue;
              const int ho = th / stride;
              if (ho >= Ho) continue;
              for (int s = 0; s < S; ++s) {
                const int tw = ww + pad - s;
                if (tw < 0 || tw % stride != 0) continue;
                const int wo = tw / stride;
                if (wo >= Wo) continue;
                acc += dy[(((size_t)n * Ho + ho) * Wo + wo) * Cout + k] *
                       w[(((size_t)k * R + r) * S + s) * Cin + c];
              }
            }
          dx[(((size_t)n * H + h) * W + ww) * Cin + c] = acc;
        }
  return 0;
}

/* Backward pass, gradient w.r.t. the convolution weights:
 * dw[k,r,s,c] = sum_{n,ho,wo} dy[n,ho,wo,k] * x[n, ho*st+r-p, wo*st+s-p, c]. */
int cnnk_ref_conv2d_wgrad(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                          const double* x, const double* dy, double* dw) {
  if (!x || !dy || !dw) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0) return 2;
  const int Ho = out_size(H, pad, R, stride), Wo = out_size(W, pad, S, stride);
  if (Ho <= 0 || Wo <= 0) return 2;
#pragma omp parallel for collapse(4) schedule(static)
  for (int k = 0; k < Cout; ++k)
    for (int r = 0; r < R; ++r)
      for (int s = 0; s < S; ++s)
        for (int c = 0; c < Cin; ++c) {
          double acc = 0.0;
          for (int n = 0; n < N; ++n)
            for (int ho = 0; ho < Ho; ++ho) {
              const int hi = ho * stride + r - pad;
              if (hi < 0 || hi >= H) continue;
              for (int wo = 0; wo < Wo; ++wo) {
                const int wi = wo * stride + s - pad;
                if (wi < 0 || wi >= W) continue;
                acc += dy[(((size_t)n * Ho + ho) * Wo + wo) * Cout + k] *
                       x[(((size_t)n * H + hi) * W + wi) * Cin + c];
              }
            }
          dw[(((size_t)k * R + r) * S + s) * Cin + c] = acc;
        }
  return 0;
}

/* Forward pass, batch normalisation in training mode, optional residual add, optional ReLU.
 * m = N*H*W; mean_c = (1/m) sum x; var_c = (1/m) sum (x-mean_c)^2 (two passes, biased);
 * invstd = 1/sqrt(var+eps); xhat = (x-mean)*invstd; u = gamma*xhat + beta (+ residual);
 * y = max(u,0) if relu else u.  Side outputs (not on the gradient path):
 * running_mean <- (1-a)*running_mean + a*mean; running_var <- (1-a)*running_var + a*var*m/(m-1). */
int cnnk_ref_bn_relu_fwd(int N, int H, int W, int C, double eps, double momentum, int relu,
                         const double* x, const double* residual, const double* gamma,
                         const double* beta, double* y, double* save_mean, double* save_invstd,
                         double* running_mean, double* running_var) {
  if (!x || !gamma || !beta || !y || !save_mean || !save_invstd) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return 2;
  const size_t m = (size_t)N * H * W;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double sum = 0.0;
    for (size_t i = 0; i < m; ++i) sum += x[i * C + c];
    const double mean = sum / (double)m;
    double ss = 0.0;
    for (size_t i = 0; i < m; ++i) {
      const double d = x[i * C + c] - mean;
      ss += d * d;
    }
    const double var = ss / (double)m;
    const double invstd = 1.0 / sqrt(var + eps);
    save_mean[c] = mean;
    save_invstd[c] = invstd;
    if (running_mean) running_mean[c] = (1.0 - momentum) * running_mean[c] + momentum * mean;
    if (running_var) {
      const double unbiased = (m > 1) ? ss / (double)(m - 1) : var;
      running_var[c] = (1.0 - momentum) * running_var[c] + momentum * unbiased;
    }
    for (size_t i = 0; i < m; ++i) {
      double u = gamma[c] * ((x[i * C + c] - mean) * invstd) + beta[c];
      if (residual) u += residual[i * C + c];
      y[i * C + c] = (relu && !(u > 0.0)) ? 0.0 : u;
    }
  }
  return 0;
}

/* Inference-mode batch norm (validation pass of Algorithm 1's epoch loop): the batch statistics
 * are replaced by the running ones, y = act(gamma*(x - running_mean)/sqrt(running_var + eps) +
 * beta [+ residual]); nothing is updated. */
int cnnk_ref_bn_relu_infer(int N, int H, int W, int C, double eps, int relu, const double* x,
                           const double* residual, const double* gamma, const double* beta,
                           const double* running_mean, const double* running_var, double* y) {
  if (!x || !gamma || !beta || !running_mean || !running_var || !y) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return 2;
  const size_t m = (size_t)N * H * W;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const double invstd = 1.0 / sqrt(running_var[c] + eps);
    for (size_t i = 0; i < m; ++i) {
      double u = gamma[c] * ((x[i * C + c] - running_mean[c]) * invstd) + beta[c];
      if (residual) u += residual[i * C + c];
      y[i * C + c] = (relu && !(u > 0.0)) ? 0.0 : u;
    }
  }
  return 0;
}

/* Backward pass of the block above.  dz = dy * [y > 0] (strict; all ones without ReLU);
 * dresidual = dz; dbeta = sum dz; dgamma = sum dz*xhat;
 * dx = (gamma*invstd/m) * (m*dz - dbeta - xhat*dgamma). */
int cnnk_ref_bn_relu_bwd(int N, int H, int W, int C, int relu, const double* dy, const double* x,
                         const double* y, const double* gamma, const double* save_mean,
                         const double* save_invstd, double* dx, double* dresidual, double* dgamma,
                         double* dbeta) {
  if (!dy || !x || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return 1;
  if (relu && !y) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return 2;
  const size_t m = (size_t)N * H * W;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const double mean = save_mean[c], invstd = save_invstd[c];
    double db = 0.0, dg = 0.0;
    for (size_t i = 0; i < m; ++i) {
      const double dz = (relu && !(y[i * C + c] > 0.0)) ? 0.0 : dy[i * C + c];
      db += dz;
      dg += dz * ((x[i * C + c] - mean) * invstd);
    }
    dbeta[c] = db;
    dgamma[c] = dg;
    const double scale = gamma[c] * invstd / (double)m;
    for (size_t i = 0; i < m; ++i) {
      const double dz = (relu && !(y[i * C + c] > 0.0)) ? 0.0 : dy[i * C + c];
      const double xhat = (x[i * C + c] - mean) * invstd;
      dx[i * C + c] = scale * ((double)m * dz - db - xhat * dg);
      if (dresidual) dresidual[i * C + c] = dz;
    }
  }
  return 0;
}

/* Forward pass, pooling.  Max-pool: 2x2 window, stride 2, no padding; the recorded argmax is
 * the first maximal element in (row, col) scan order, coded 2*dr+dc.  Global average pool:
 * y[n,c] = (1/(H*W)) sum_{h,w} x[n,h,w,c]. */
int cnnk_ref_pool_fwd(int N, int H, int W, int C, int mode, const double* x, double* y,
                      unsigned char* argmax) {
  if (!x || !y) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return 2;
  if (mode == 0) {
    if (!argmax) return 1;
    if (H % 2 || W % 2) return 2;
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
      for (int ho = 0; ho < Ho; ++ho)
        for (int wo = 0; wo < Wo; ++wo)
          for (int c = 0; c < C; ++c) {
            double best = x[(((size_t)n * H + 2 * ho) * W + 2 * wo) * C + c];
            int code = 0;
            for (int dr = 0; dr < 2; ++dr)
              for (int dc = 0; dc < 2; ++dc) {
                const double v = x[(((size_t)n * H + 2 * ho + dr) * W + 2 * wo + dc) * C + c];
                if (v > best) { best = v; code = 2 * dr + dc; }
              }
            const size_t o = (((size_t)n * Ho + ho) * Wo + wo) * C + c;
            y[o] = best;
            argmax[o] = (unsigned char)code;
          }
    return 0;
  }
  if (mode == 1) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
      for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (int i = 0; i < H * W; ++i) s += x[((size_t)n * H * W + i) * C + c];
        y[(size_t)n * C + c] = s / (double)(H * W);
      }
    return 0;
  }
  return 3;
}

/* Backward pass, pooling.  Max-pool: dy goes to the recorded argmax position, zero elsewhere.
 * Global average pool: dx[n,h,w,c] = dy[n,c]/(H*W). */
int cnnk_ref_pool_bwd(int N, int H, int W, int C, int mode, const double* dy,
                      const unsigned char* argmax, double* dx) {
  if (!dy || !dx) return 1;
  if (N <= 0 || H <= 0 || W <= 0 || C <= 0) return 2;
  if (mode == 0) {
    if (!argmax) return 1;
    if (H % 2 || W % 2) return 2;
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
      for (int h = 0; h < H; ++h)
        for (int w = 0; w < W; ++w)
          for (int c = 0; c < C; ++c) {
            const size_t o = (((size_t)n * Ho + h / 2) * Wo + w / 2) * C + c;
            const int code = 2 * (h % 2) + (w % 2);
            dx[(((size_t)n * H + h) * W + w) * C + c] = (argmax[o] == code) ? dy[o] : 0.0;
          }
    return 0;
  }
  if (mode == 1) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < H * W; ++i)
        for (int c = 0; c < C; ++c)
          dx[((size_t)n * H * W + i) * C + c] = dy[(size_t)n * C + c] / (double)(H * W);
    return 0;
  }
  return 3;
}

/* Forward pass head, loss, and their backward pass (Algorithm 1: "compute loss L(theta)").
 * z[n,j] = sum_f x[n,f]*W[j,f] + b[j]; zmax = max_j z; lse = zmax + log sum_j exp(z-zmax);
 * loss = (1/N) sum_n (lse_n - z[n,label_n]) (natural log); pred_n = smallest j with z[n,j]=zmax.
 * dz = (softmax(z) - onehot(label))/N; dW = dz^T x; db = sum_n dz; dx = dz W.
 * probs (optional) receives softmax(z). */
int cnnk_ref_fc_softmax_xent(int N, int F, int classes, const double* x, const double* W,
                             const double* b, const int* labels, double* loss, int* pred,
                             double* probs, double* dx, double* dW, double* db) {
  if (!x || !W || !b || !labels || !loss || !pred || !dx || !dW || !db) return 1;
  if (N <= 0 || F <= 0 || classes <= 0) return 2;
  for (int n = 0; n < N; ++n)
    if (labels[n] < 0 || labels[n] >= classes) return 2;
  double* dz = (double*)malloc(sizeof(double) * (size_t)N * classes);
  if (!dz) return 4;
  double total = 0.0;
  for (int n = 0; n < N; ++n) {
    double* z = dz + (size_t)n * classes;
    for (int j = 0; j < classes; ++j) {
      double acc = 0.0;
      for (int f = 0; f < F; ++f) acc += x[(size_t)n * F + f] * W[(size_t)j * F + f];
      z[j] = acc + b[j];
    }
    double zmax = z[0];
    int arg = 0;
    for (int j = 1; j < classes; ++j)
      if (z[j] > zmax) { zmax = z[j]; arg = j; }
    pred[n] = arg;
    double se = 0.0;
    for (int j = 0; j < classes; ++j) se += exp(z[j] - zmax);
    const double lse = zmax + log(se);
    total += lse - z[labels[n]];
    for (int j = 0; j < classes; ++j) {
      const double p = exp(z[j] - lse);
      if (probs) probs[(size_t)n * classes + j] = p;
      z[j] = (p - (j == labels[n] ? 1.0 : 0.0)) / (double)N;
    }
  }
  *loss = total / (double)N;
  for (int j = 0; j < classes; ++j) {
    double s = 0.0;
    for (int n = 0; n < N; ++n) s += dz[(size_t)n * classes + j];
    db[j] = s;
    for (int f = 0; f < F; ++f) {
      double a = 0.0;
      for (int n = 0; n < N; ++n) a += dz[(size_t)n * classes + j] * x[(size_t)n * F + f];
      dW[(size_t)j * F + f] = a;
    }
  }
  for (int n = 0; n < N; ++n)
    for (int f = 0; f < F; ++f) {
      double a = 0.0;
      for (int j = 0; j < classes; ++j) a += dz[(size_t)n * classes + j] * W[(size_t)j * F + f];
      dx[(size_t)n * F + f] = a;
    }
  free(dz);
  return 0;
}

/* Parameter update (Algorithm 1: theta <- theta - eta*grad), generalised to SGD with momentum:
 * g' = g + wd*w; v <- mu*v + g'; w <- w - lr*v.  With mu = 0 and wd = 0 this is the printed rule. */
int cnnk_ref_sgd_momentum(long n, double* w, double* v, const double* g, double lr, double momentum,
                          double weight_decay) {
  if (!w || !v || !g) return 1;
  if (n < 0) return 2;
  for (long i = 0; i < n; ++i) {
    const double gp = g[i] + weight_decay * w[i];
    v[i] = momentum * v[i] + gp;
    w[i] = w[i] - lr * v[i];
  }
  return 0;
}

/* Storage emulation for the bf16 mode (used when the comparison must take the ReLU / max-pool /
 * argmax decisions on values stored at the kernel's precision): round each double to the
 * nearest bfloat16 (8 significand bits, ties to even), in place.  The value is first rounded to
 * float (the kernel's accumulator type), then to bfloat16; overflow to infinity is not handled. */
int cnnk_ref_round_bf16(long n, double* a) {
  if (!a) return 1;
  if (n < 0) return 2;
  for (long i = 0; i < n; ++i) {
    const float f = (float)a[i];
    if (f != f || f == 0.0f) { a[i] = (double)f; continue; }
    int e;
    const double m = frexp((double)f, &e);          /* f = m * 2^e, 0.5 <= |m| < 1 */
    const double scaled = ldexp(m, 8);              /* 8 significand bits: |scaled| in [128, 256) */
    const double r = nearbyint(scaled);             /* default rounding mode: ties to even */
    a[i] = ldexp(r, e - 8);
  }
  return 0;
}
