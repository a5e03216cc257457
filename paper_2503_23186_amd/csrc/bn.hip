// Batch norm (+ residual) (+ ReLU), forward and backward, for NHWC tensors viewed as [m][C].
// Bandwidth-bound: every thread moves 16-byte (bf16) or 32-byte (fp32) vectors of 8 channels,
// per-channel reductions are per-thread partial sums -> LDS -> per-workgroup partials -> a small
// finalising kernel that sums the partials in double precision (fixed order, no atomics).
#include "common.h"
#include "conv.h"

namespace {

constexpr int kT = 256;
constexpr int kMaxBlocks = 2048;

struct RowMap {
  int lanes;   // threads per row = C/8
  int rows;    // rows per workgroup pass = 256 / lanes
};

__host__ __device__ inline int reduce_blocks(size_t m, int C) {
  const int rows = kT / (C / 8);
  size_t nb = (m + (size_t)rows * 4 - 1) / ((size_t)rows * 4);  // at least 4 rows per thread
  if (nb > kMaxBlocks) nb = kMaxBlocks;
  if (nb < 1) nb = 1;
  return (int)nb;
}

// Sum the NV per-thread vectors of 8 channels over the threads that share a channel octet and
// write them to part[v][c][blockIdx.x] (workgroup index fastest, so the finaliser reads rows).
template <int NV>
__device__ __forceinline__ void block_reduce_store(float (*acc)[8], int lanes, int rows, int C,
                                                   float* __restrict__ part) {
  __shared__ float red[kT * 8];
  const int tid = threadIdx.x;
  const int o = tid % lanes, rl = tid / lanes;
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    __syncthreads();
    if (rl < rows) {
#pragma unroll
      for (int e = 0; e < 8; ++e) red[(rl * lanes + o) * 8 + e] = acc[v][e];
    }
    __syncthreads();
    for (int i = tid; i < C; i += kT) {
      float s = 0.f;
      for (int r = 0; r < rows; ++r) s += red[(r * lanes) * 8 + i];
      part[((size_t)v * C + i) * gridDim.x + blockIdx.x] = s;
    }
  }
}

// Finalising reduction: one workgroup per channel sums the nb per-workgroup partials
// part[v][c][0..nb) in double (coalesced rows, fixed-order tree).  Result valid in thread 0.
__device__ __forceinline__ void finalize_sums(const float* __restrict__ part, int nb, int C, int c,
                                              double* s1_out, double* s2_out) {
  __shared__ double fred[2][kT];
  const int t = threadIdx.x;
  double s1 = 0.0, s2 = 0.0;
  const float* p1 = part + ((size_t)0 * C + c) * nb;
  const float* p2 = part + ((size_t)1 * C + c) * nb;
  for (int b = t; b < nb; b += kT) {
    s1 += (double)p1[b];
    s2 += (double)p2[b];
  }
  fred[0][t] = s1;
  fred[1][t] = s2;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if (t < o) {
      fred[0][t] += fred[0][t + o];
      fred[1][t] += fred[1][t + o];
    }
    __syncthreads();
  }
  *s1_out = fred[0][0];
  *s2_out = fred[1][0];
}

// Partial sums of (x - shift) and (x - shift)^2 with shift = x[0][c] (keeps fp32 sums benign).
template <typename T>
__global__ void __launch_bounds__(kT) stats_partial_kernel(const T* __restrict__ x, size_t m, int C,
                                                           float* __restrict__ part) {
  const int lanes = C / 8, rows = kT / lanes;
  const int tid = threadIdx.x, o = tid % lanes, rl = tid / lanes;
  float acc[2][8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[0][e] = acc[1][e] = 0.f;
  if (rl < rows) {
    float sh[8];
    load8(x + o * 8, sh);
#pragma unroll 4
    for (size_t r = (size_t)blockIdx.x * rows + rl; r < m; r += (size_t)gridDim.x * rows) {
      float v[8];
      load8(x + r * C + o * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = v[e] - sh[e];
        acc[0][e] += d;
        acc[1][e] = fmaf(d, d, acc[1][e]);
      }
    }
  }
  block_reduce_store<2>(acc, lanes, rows, C, part);
}

// mode 0: write save_mean / save_invstd (+ running stats); mode 1: write plain sum, sum of squares.
template <typename T>
__global__ void __launch_bounds__(kT) stats_finalize_kernel(const float* __restrict__ part, int nb,
                                                            const T* __restrict__ x, size_t m, int C, int mode,
                                                            float eps, float momentum, float* __restrict__ o0,
                                                            float* __restrict__ o1, float* __restrict__ rmean,
                                                            float* __restrict__ rvar) {
  const int c = blockIdx.x;
  double s1, s2;
  finalize_sums(part, nb, C, c, &s1, &s2);
  if (threadIdx.x != 0) return;
  const double sh = (double)Elem<T>::ld(x + c);
  const double dm = (double)m;
  if (mode == 1) {
    o0[c] = (float)(s1 + dm * sh);
    o1[c] = (float)(s2 + 2.0 * sh * s1 + dm * sh * sh);
    return;
  }
  const double mean_s = s1 / dm;
  double var = s2 / dm - mean_s * mean_s;
  if (var < 0.0) var = 0.0;
  o0[c] = (float)(sh + mean_s);
  o1[c] = (float)(1.0 / sqrt(var + (double)eps));
  if (rmean) {
    const double unb = m > 1 ? var * dm / (dm - 1.0) : var;
    rmean[c] = (float)((1.0 - momentum) * rmean[c] + momentum * (sh + mean_s));
    rvar[c] = (float)((1.0 - momentum) * rvar[c] + momentum * unb);
  }
}

__global__ void __launch_bounds__(kT) sums_finalize_kernel(const float* __restrict__ part, int nb, int C,
                                                           float* __restrict__ ch_sum, float* __restrict__ ch_sumsq) {
  const int c = blockIdx.x;
  double s1, s2;
  finalize_sums(part, nb, C, c, &s1, &s2);
  if (threadIdx.x != 0) return;
  ch_sum[c] = (float)s1;
  ch_sumsq[c] = (float)s2;
}

template <typename T>
__global__ void __launch_bounds__(kT) bn_apply_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                      const float* __restrict__ gamma,
                                                      const float* __restrict__ beta,
                                                      const float* __restrict__ mean,
                                                      const float* __restrict__ invstd, T* __restrict__ y,
                                                      size_t n8, int C, int relu) {
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n8; i += (size_t)gridDim.x * kT) {
    const int c0 = (int)((i * 8) % C);
    float v[8], g[8], b[8], mu[8], is[8];
    load8(x + i * 8, v);
    load8(gamma + c0, g);
    load8(beta + c0, b);
    load8(mean + c0, mu);
    load8(invstd + c0, is);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = fmaf(g[e], (v[e] - mu[e]) * is[e], b[e]);
    if (res) {
      float r[8];
      load8(res + i * 8, r);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += r[e];
    }
    if (relu) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
    }
    store8(y + i * 8, v);
  }
}

// Normalise (+ residual) (+ ReLU) with the statistics taken directly from per-channel sums
// (sum x, sum x^2 over m positions, e.g. from the convolution that produced x): every thread
// derives mean / invstd of its 8 channels itself, so no separate statistics kernel runs.
// Workgroup 0 also writes save_mean / save_invstd and updates the running statistics.
template <typename T>
__global__ void __launch_bounds__(kT) bn_apply_sums_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                           const float* __restrict__ gamma,
                                                           const float* __restrict__ beta,
                                                           const float* __restrict__ ch_sum,
                                                           const float* __restrict__ ch_sumsq, float inv_m,
                                                           float unbias, float eps, float momentum,
                                                           float* __restrict__ save_mean,
                                                           float* __restrict__ save_invstd,
                                                           float* __restrict__ rmean, float* __restrict__ rvar,
                                                           T* __restrict__ y, size_t n8, int C, int relu) {
  int cur_c0 = -1;
  float sc[8], bi[8];
  if (blockIdx.x == 0) {
    for (int c = threadIdx.x; c < C; c += kT) {
      const float mu = ch_sum[c] * inv_m;
      const float var = fmaxf(fmaf(ch_sumsq[c], inv_m, -mu * mu), 0.f);
      save_mean[c] = mu;
      save_invstd[c] = rsqrtf(var + eps);
      if (rmean) {
        rmean[c] = (1.f - momentum) * rmean[c] + momentum * mu;
        rvar[c] = (1.f - momentum) * rvar[c] + momentum * var * unbias;
      }
    }
  }
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n8; i += (size_t)gridDim.x * kT) {
    const int c0 = (int)((i * 8) % C);
    if (c0 != cur_c0) {
      cur_c0 = c0;
      float s1[8], s2[8], g[8], b[8];
      load8(ch_sum + c0, s1);
      load8(ch_sumsq + c0, s2);
      load8(gamma + c0, g);
      load8(beta + c0, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float mu = s1[e] * inv_m;
        const float var = fmaxf(fmaf(s2[e], inv_m, -mu * mu), 0.f);
        const float is = rsqrtf(var + eps);
        sc[e] = g[e] * is;
        bi[e] = fmaf(-mu, sc[e], b[e]);
      }
    }
    float v[8];
    load8(x + i * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = fmaf(v[e], sc[e], bi[e]);
    if (res) {
      float r[8];
      load8(res + i * 8, r);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += r[e];
    }
    if (relu) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
    }
    store8(y + i * 8, v);
  }
}

// Partial sums of dz and dz*xhat.
template <typename T>
__global__ void __launch_bounds__(kT) bwd_partial_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                         const T* __restrict__ y,
                                                         const float* __restrict__ mean,
                                                         const float* __restrict__ invstd, size_t m, int C,
                                                         int relu, float* __restrict__ part) {
  const int lanes = C / 8, rows = kT / lanes;
  const int tid = threadIdx.x, o = tid % lanes, rl = tid / lanes;
  float acc[2][8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[0][e] = acc[1][e] = 0.f;
  if (rl < rows) {
    float mu[8], is[8];
    load8(mean + o * 8, mu);
    load8(invstd + o * 8, is);
#pragma unroll 4
    for (size_t r = (size_t)blockIdx.x * rows + rl; r < m; r += (size_t)gridDim.x * rows) {
      float g[8], xv[8];
      load8(dy + r * C + o * 8, g);
      load8(x + r * C + o * 8, xv);
      if (relu) {
        float yv[8];
        load8(y + r * C + o * 8, yv);
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = yv[e] > 0.f ? g[e] : 0.f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[0][e] += g[e];
        acc[1][e] = fmaf(g[e], (xv[e] - mu[e]) * is[e], acc[1][e]);
      }
    }
  }
  block_reduce_store<2>(acc, lanes, rows, C, part);
}

__global__ void __launch_bounds__(kT) bwd_finalize_kernel(const float* __restrict__ part, int nb, int C,
                                                          float* __restrict__ dgamma, float* __restrict__ dbeta) {
  const int c = blockIdx.x;
  double s1, s2;
  finalize_sums(part, nb, C, c, &s1, &s2);
  if (threadIdx.x != 0) return;
  dbeta[c] = (float)s1;
  dgamma[c] = (float)s2;
}

template <typename T>
__global__ void __launch_bounds__(kT) bwd_apply_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                       const T* __restrict__ y, const float* __restrict__ gamma,
                                                       const float* __restrict__ mean,
                                                       const float* __restrict__ invstd,
                                                       const float* __restrict__ dgamma,
                                                       const float* __restrict__ dbeta, T* __restrict__ dx,
                                                       T* __restrict__ dres, size_t n8, int C, float inv_m,
                                                       int relu, int flags) {
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n8; i += (size_t)gridDim.x * kT) {
    const int c0 = (int)((i * 8) % C);
    float g[8], xv[8], ga[8], mu[8], is[8], dg[8], db[8], out[8];
    load8(dy + i * 8, g);
    load8(x + i * 8, xv);
    load8(gamma + c0, ga);
    load8(mean + c0, mu);
    load8(invstd + c0, is);
    load8(dgamma + c0, dg);
    load8(dbeta + c0, db);
    if (relu) {
      float yv[8];
      load8(y + i * 8, yv);
#pragma unroll
      for (int e = 0; e < 8; ++e) g[e] = yv[e] > 0.f ? g[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float xh = (xv[e] - mu[e]) * is[e];
      out[e] = ga[e] * is[e] * (g[e] - (db[e] + xh * dg[e]) * inv_m);
    }
    if (flags & 1) {
      float old[8];
      load8(dx + i * 8, old);
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] += old[e];
    }
    store8(dx + i * 8, out);
    if (dres) {
      if (flags & 2) {
        float old[8];
        load8(dres + i * 8, old);
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] += old[e];
      }
      store8(dres + i * 8, g);
    }
  }
}

inline unsigned ew_blocks(size_t n8) {
  size_t b = (n8 + kT - 1) / kT;
  if (b > 8192) b = 8192;
  return (unsigned)(b < 1 ? 1 : b);
}

int validate_bn(const cnnk_bn_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (d->C % 8 != 0 || d->C > 2048) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

}  // namespace

int channel_sums_finalize(const float* part, int nb, int C, float* ch_sum, float* ch_sumsq, hipStream_t st) {
  sums_finalize_kernel<<<C, kT, 0, st>>>(part, nb, C, ch_sum, ch_sumsq);
  return launch_status();
}

size_t channel_stats_ws(size_t m, int C) { return (size_t)reduce_blocks(m, C) * 2 * C * sizeof(float); }

int channel_stats(int dtype, const void* x, size_t m, int C, float* ch_sum, float* ch_sumsq, void* ws,
                  hipStream_t st) {
  const int nb = reduce_blocks(m, C);
  float* part = (float*)ws;
  if (dtype == CNNK_BF16) {
    stats_partial_kernel<bf16_t><<<nb, kT, 0, st>>>((const bf16_t*)x, m, C, part);
    stats_finalize_kernel<bf16_t><<<C, kT, 0, st>>>(part, nb, (const bf16_t*)x, m, C, 1, 0.f, 0.f,
                                                                    ch_sum, ch_sumsq, nullptr, nullptr);
  } else {
    stats_partial_kernel<float><<<nb, kT, 0, st>>>((const float*)x, m, C, part);
    stats_finalize_kernel<float><<<C, kT, 0, st>>>(part, nb, (const float*)x, m, C, 1, 0.f, 0.f,
                                                                   ch_sum, ch_sumsq, nullptr, nullptr);
  }
  return launch_status();
}

extern "C" size_t cnnk_bn_workspace_bytes(const cnnk_bn_desc* d) {
  if (validate_bn(d) != CNNK_OK) return 0;
  return align_up(channel_stats_ws((size_t)d->N * d->H * d->W, d->C), 256);
}

extern "C" int cnnk_bn_relu_fwd(const cnnk_bn_desc* d, const void* x, const void* residual, const float* gamma,
                                const float* beta, void* y, float* save_mean, float* save_invstd,
                                float* running_mean, float* running_var, const float* ch_sum,
                                const float* ch_sumsq, void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_bn(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !gamma || !beta || !y || !save_mean || !save_invstd) return CNNK_ERR_NULL;
  if ((running_mean == nullptr) != (running_var == nullptr)) return CNNK_ERR_NULL;
  if ((ch_sum == nullptr) != (ch_sumsq == nullptr)) return CNNK_ERR_NULL;
  const size_t m = (size_t)d->N * d->H * d->W;
  const int C = d->C;
  hipStream_t st = (hipStream_t)stream;
  if (!ch_sum) {
    if (!ws || ws_bytes < channel_stats_ws(m, C)) return CNNK_ERR_WORKSPACE;
    const int nb = reduce_blocks(m, C);
    float* part = (float*)ws;
    if (d->dtype == CNNK_BF16) {
      stats_partial_kernel<bf16_t><<<nb, kT, 0, st>>>((const bf16_t*)x, m, C, part);
      stats_finalize_kernel<bf16_t><<<C, kT, 0, st>>>(part, nb, (const bf16_t*)x, m, C, 0, d->eps,
                                                                      d->momentum, save_mean, save_invstd,
                                                                      running_mean, running_var);
    } else {
      stats_partial_kernel<float><<<nb, kT, 0, st>>>((const float*)x, m, C, part);
      stats_finalize_kernel<float><<<C, kT, 0, st>>>(part, nb, (const float*)x, m, C, 0, d->eps,
                                                                     d->momentum, save_mean, save_invstd,
                                                                     running_mean, running_var);
    }
  } else {
    // statistics handed in as sums: one fused kernel (statistics + normalise)
    const size_t n8s = m * C / 8;
    const float inv_m = (float)(1.0 / (double)m);
    const float unbias = m > 1 ? (float)((double)m / ((double)m - 1.0)) : 1.f;
    if (d->dtype == CNNK_BF16)
      bn_apply_sums_kernel<bf16_t><<<ew_blocks(n8s), kT, 0, st>>>((const bf16_t*)x, (const bf16_t*)residual, gamma, beta,
                                                                 ch_sum, ch_sumsq, inv_m, unbias, d->eps, d->momentum,
                                                                 save_mean, save_invstd, running_mean, running_var,
                                                                 (bf16_t*)y, n8s, C, d->relu);
    else
      bn_apply_sums_kernel<float><<<ew_blocks(n8s), kT, 0, st>>>((const float*)x, (const float*)residual, gamma, beta,
                                                                ch_sum, ch_sumsq, inv_m, unbias, d->eps, d->momentum,
                                                                save_mean, save_invstd, running_mean, running_var,
                                                                (float*)y, n8s, C, d->relu);
    return launch_status();
  }
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  const size_t n8 = m * C / 8;
  if (d->dtype == CNNK_BF16)
    bn_apply_kernel<bf16_t><<<ew_blocks(n8), kT, 0, st>>>((const bf16_t*)x, (const bf16_t*)residual, gamma, beta,
                                                          save_mean, save_invstd, (bf16_t*)y, n8, C, d->relu);
  else
    bn_apply_kernel<float><<<ew_blocks(n8), kT, 0, st>>>((const float*)x, (const float*)residual, gamma, beta,
                                                         save_mean, save_invstd, (float*)y, n8, C, d->relu);
  return launch_status();
}

extern "C" int cnnk_bn_relu_bwd(const cnnk_bn_desc* d, const void* dy, const void* x, const void* y,
                                const float* gamma, const float* save_mean, const float* save_invstd, void* dx,
                                void* dresidual, int flags, float* dgamma, float* dbeta, void* ws,
                                size_t ws_bytes, void* stream) {
  int rc = validate_bn(d);
  if (rc != CNNK_OK) return rc;
  if (!dy || !x || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return CNNK_ERR_NULL;
  if (d->relu && !y) return CNNK_ERR_NULL;
  const size_t m = (size_t)d->N * d->H * d->W;
  const int C = d->C;
  if (!ws || ws_bytes < channel_stats_ws(m, C)) return CNNK_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int nb = reduce_blocks(m, C);
  float* part = (float*)ws;
  const size_t n8 = m * C / 8;
  const float inv_m = (float)(1.0 / (double)m);
  if (d->dtype == CNNK_BF16) {
    bwd_partial_kernel<bf16_t><<<nb, kT, 0, st>>>((const bf16_t*)dy, (const bf16_t*)x, (const bf16_t*)y, save_mean,
                                                  save_invstd, m, C, d->relu, part);
    bwd_finalize_kernel<<<C, kT, 0, st>>>(part, nb, C, dgamma, dbeta);
    bwd_apply_kernel<bf16_t><<<ew_blocks(n8), kT, 0, st>>>((const bf16_t*)dy, (const bf16_t*)x, (const bf16_t*)y,
                                                           gamma, save_mean, save_invstd, dgamma, dbeta,
                                                           (bf16_t*)dx, (bf16_t*)dresidual, n8, C, inv_m, d->relu,
                                                           flags);
  } else {
    bwd_partial_kernel<float><<<nb, kT, 0, st>>>((const float*)dy, (const float*)x, (const float*)y, save_mean,
                                                 save_invstd, m, C, d->relu, part);
    bwd_finalize_kernel<<<C, kT, 0, st>>>(part, nb, C, dgamma, dbeta);
    bwd_apply_kernel<float><<<ew_blocks(n8), kT, 0, st>>>((const float*)dy, (const float*)x, (const float*)y, gamma,
                                                          save_mean, save_invstd, dgamma, dbeta, (float*)dx,
                                                          (float*)dresidual, n8, C, inv_m, d->relu, flags);
  }
  return launch_status();
}
