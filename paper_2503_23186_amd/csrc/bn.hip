// Batch norm (+ residual) (+ ReLU), forward and backward, for NHWC tensors viewed as [m][C].
// Bandwidth-bound: every thread moves 16-byte (bf16) or 32-byte (fp32) vectors of 8 channels,
// per-channel reductions are per-thread partial sums -> LDS -> per-workgroup partials -> a small
// finalising kernel that sums the partials in double precision (fixed order, no atomics).
#include "common.h"
#include <type_traits>
#include "conv.h"

namespace {

constexpr int kT = 256;
constexpr int kMaxBlocks = 2048;

struct RowMap {
  int lanes;   // threads per row = C/8
  int rows;    // rows per workgroup pass = 256 / lanes
};

inline int reduce_blocks(size_t m, int C) {
  const int rows = kT / (C / 8);
  // at least 8 rows per thread (ResNet-18 b256 step: 2.215 ms with 4, 2.195 with 8, 2.27 with 16)
  size_t nb = (m + (size_t)rows * 8 - 1) / ((size_t)rows * 8);
  if (nb > kMaxBlocks) nb = kMaxBlocks;
  // every workgroup ends with 2*C scattered 4-byte writes of its partial sums: with many channels
  // fewer, longer-lived workgroups are cheaper (C = 1024: 256 instead of 2048; ResNet-50
  // b256 step 9.57 -> 9.08 ms, 128 or 512 are worse or equal)
  size_t cap = (size_t)262144 / (size_t)C;
  if (cap < 256) cap = 256;
  if (nb > cap) nb = cap;
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
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wavefront per channel (four channels per workgroup): the lanes stride over the nb partials,
// the xor-butterfly gives every lane the total.  Fixed order, no LDS, no barrier.
constexpr int kFinCh = kT / 64;   // channels per finalising workgroup
inline unsigned fin_blocks(int C) { return (unsigned)((C + kFinCh - 1) / kFinCh); }

__device__ __forceinline__ void finalize_sums(const float* __restrict__ part, int nb, int C, int c,
                                              double* s1_out, double* s2_out) {
  const int lane = threadIdx.x & 63;
  double s1 = 0.0, s2 = 0.0;
  const float* p1 = part + ((size_t)0 * C + c) * nb;
  const float* p2 = part + ((size_t)1 * C + c) * nb;
  // up to eight partials per round, all loads issued before the first add (an index past the end
  // is not loaded and adds zero); same order of additions as a plain loop
  const int rounds = (nb + 63) / 64;
  for (int k0 = 0; k0 < rounds; k0 += 8) {
    float v1[8], v2[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int b = lane + (k0 + k) * 64;
      v1[k] = v2[k] = 0.f;
      if (b < nb) {
        v1[k] = p1[b];
        v2[k] = p2[b];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k0 + k < rounds) {
        s1 += (double)v1[k];
        s2 += (double)v2[k];
      }
  }
  *s1_out = wave_sum_f64(s1);
  *s2_out = wave_sum_f64(s2);
}

// Row walk of the reductions and of the element-wise kernels: a thread owns one octet of
// channels (o = tid % (C/8)) for the whole launch, keeps that octet's coefficients in registers, and
// walks rows blockIdx.x*rows + tid/(C/8), +gridDim.x*rows, ... four rows in flight.  No per-vector
// index arithmetic beyond one multiply-add, no per-vector coefficient loads.
template <typename T, typename F>
__device__ __forceinline__ void for_rows4(size_t m, int C, int lanes, int rows, F body) {
  const int tid = threadIdx.x, o = tid % lanes, rl = tid / lanes;
  if (rl >= rows) return;
  const size_t step = (size_t)gridDim.x * rows;
  size_t r = (size_t)blockIdx.x * rows + rl;
  for (; r + 3 * step < m; r += 4 * step) {
    const size_t i0 = r * C + o * 8, d = step * C;
    body(i0, i0 + d, i0 + 2 * d, i0 + 3 * d, std::integral_constant<int, 4>{});
  }
  for (; r < m; r += step) {
    const size_t i0 = r * C + o * 8;
    body(i0, i0, i0, i0, std::integral_constant<int, 1>{});
  }
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
    // four rows per round, all loads issued before the first use (a plain row loop is compiled to
    // one load in flight per thread)
    for_rows4<T>(m, C, lanes, rows, [&](size_t i0, size_t i1, size_t i2, size_t i3, auto NN) {
      constexpr int n = decltype(NN)::value;
      const size_t idx[4] = {i0, i1, i2, i3};
      float v[4][8];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (k < n) load8(x + idx[k], v[k]);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (k >= n) break;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float d = v[k][e] - sh[e];
          acc[0][e] += d;
          acc[1][e] = fmaf(d, d, acc[1][e]);
        }
      }
    });
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
  const int c = blockIdx.x * kFinCh + (threadIdx.x >> 6);
  if (c >= C) return;
  double s1, s2;
  finalize_sums(part, nb, C, c, &s1, &s2);
  if ((threadIdx.x & 63) != 0) return;
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
  const int c = blockIdx.x * kFinCh + (threadIdx.x >> 6);
  if (c >= C) return;
  double s1, s2;
  finalize_sums(part, nb, C, c, &s1, &s2);
  if ((threadIdx.x & 63) != 0) return;
  ch_sum[c] = (float)s1;
  ch_sumsq[c] = (float)s2;
}

// The same with a whole workgroup per channel, for many partials (a wavefront alone would walk
// them in nb/64 dependent rounds): threads stride the partials, butterfly per wavefront, the four
// wavefront sums added in order.
constexpr int kWideFinalize = 1024;   // partials per channel from which the wide kernels are used
__device__ __forceinline__ void finalize_sums_wide(const float* __restrict__ part, int nb, int C, int c,
                                                   double* s1_out, double* s2_out) {
  __shared__ double comb[2][kT / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* p1 = part + ((size_t)0 * C + c) * nb;
  const float* p2 = part + ((size_t)1 * C + c) * nb;
  double s1 = 0.0, s2 = 0.0;
  const int rounds = (nb + kT - 1) / kT;       // up to eight partials per round, as above
  for (int k0 = 0; k0 < rounds; k0 += 8) {
    float v1[8], v2[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int b = tid + (k0 + k) * kT;
      v1[k] = v2[k] = 0.f;
      if (b < nb) {
        v1[k] = p1[b];
        v2[k] = p2[b];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k0 + k < rounds) {
        s1 += (double)v1[k];
        s2 += (double)v2[k];
      }
  }
  s1 = wave_sum_f64(s1);
  s2 = wave_sum_f64(s2);
  if (lane == 0) { comb[0][wave] = s1; comb[1][wave] = s2; }
  __syncthreads();
  double t1 = comb[0][0], t2 = comb[1][0];
#pragma unroll
  for (int w_ = 1; w_ < kT / 64; ++w_) { t1 += comb[0][w_]; t2 += comb[1][w_]; }
  *s1_out = t1;
  *s2_out = t2;
}

__global__ void __launch_bounds__(kT) sums_finalize_wide_kernel(const float* __restrict__ part, int nb, int C,
                                                                float* __restrict__ ch_sum,
                                                                float* __restrict__ ch_sumsq) {
  double s1, s2;
  finalize_sums_wide(part, nb, C, blockIdx.x, &s1, &s2);
  if (threadIdx.x != 0) return;
  ch_sum[blockIdx.x] = (float)s1;
  ch_sumsq[blockIdx.x] = (float)s2;
}

// sc = gamma * invstd, bi = beta - mean * sc: the one place this is written, so that the forward
// kernels and the mask recomputation of the backward kernels round identically.
__device__ __forceinline__ void bn_scale_bias(float g, float b, float mu, float is, float* sc, float* bi) {
  *sc = g * is;
  *bi = fmaf(-mu, *sc, b);
}

template <typename T>
__device__ __forceinline__ void bn_apply_rows(const T* __restrict__ x, const T* __restrict__ res, T* __restrict__ y,
                                              size_t m, int C, int relu, const float* sc, const float* bi) {
  const int lanes = C / 8, rows = kT / lanes;
  for_rows4<T>(m, C, lanes, rows, [&](size_t i0, size_t i1, size_t i2, size_t i3, auto NN) {
    constexpr int n = decltype(NN)::value;
    const size_t idx[4] = {i0, i1, i2, i3};
    float v[4][8], r[4][8];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (k < n) load8(x + idx[k], v[k]);
    if (res) {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (k < n) load8(res + idx[k], r[k]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (k >= n) break;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[k][e] = fmaf(v[k][e], sc[e], bi[e]);
      if (res) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[k][e] += r[k][e];
      }
      if (relu) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[k][e] = v[k][e] > 0.f ? v[k][e] : 0.f;
      }
      store8(y + idx[k], v[k]);
    }
  });
}

// y = gamma * (x - mean) * invstd + beta (+ residual) (ReLU), as x * sc + bi with sc = gamma * invstd,
// bi = beta - mean * sc (the same two roundings whichever kernel produced the statistics).
template <typename T>
__global__ void __launch_bounds__(kT) bn_apply_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                      const float* __restrict__ gamma,
                                                      const float* __restrict__ beta,
                                                      const float* __restrict__ mean,
                                                      const float* __restrict__ invstd, T* __restrict__ y,
                                                      size_t m, int C, int relu) {
  const int o = threadIdx.x % (C / 8);
  float g[8], b[8], mu[8], is[8], sc[8], bi[8];
  load8(gamma + o * 8, g);
  load8(beta + o * 8, b);
  load8(mean + o * 8, mu);
  load8(invstd + o * 8, is);
#pragma unroll
  for (int e = 0; e < 8; ++e) bn_scale_bias(g[e], b[e], mu[e], is[e], &sc[e], &bi[e]);
  bn_apply_rows<T>(x, res, y, m, C, relu, sc, bi);
}

// Inference mode: the running statistics stand in for the batch's; nothing is reduced or updated.
template <typename T>
__global__ void __launch_bounds__(kT) bn_infer_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                      const float* __restrict__ gamma,
                                                      const float* __restrict__ beta,
                                                      const float* __restrict__ rmean,
                                                      const float* __restrict__ rvar, float eps,
                                                      T* __restrict__ y, size_t m, int C, int relu) {
  const int o = threadIdx.x % (C / 8);
  float g[8], b[8], mu[8], var[8], sc[8], bi[8];
  load8(gamma + o * 8, g);
  load8(beta + o * 8, b);
  load8(rmean + o * 8, mu);
  load8(rvar + o * 8, var);
#pragma unroll
  for (int e = 0; e < 8; ++e) bn_scale_bias(g[e], b[e], mu[e], 1.f / sqrtf(var[e] + eps), &sc[e], &bi[e]);
  bn_apply_rows<T>(x, res, y, m, C, relu, sc, bi);
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
                                                           T* __restrict__ y, size_t m, int C, int relu) {
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
  const int o = threadIdx.x % (C / 8);
  float s1[8], s2[8], g[8], b[8], sc[8], bi[8];
  load8(ch_sum + o * 8, s1);
  load8(ch_sumsq + o * 8, s2);
  load8(gamma + o * 8, g);
  load8(beta + o * 8, b);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float mu = s1[e] * inv_m;
    const float var = fmaxf(fmaf(s2[e], inv_m, -mu * mu), 0.f);
    const float is = rsqrtf(var + eps);
    bn_scale_bias(g[e], b[e], mu, is, &sc[e], &bi[e]);
  }
  bn_apply_rows<T>(x, res, y, m, C, relu, sc, bi);
}

// Partial sums of dz and dz*xhat.  MODE 0: no ReLU; 1: mask [y > 0]; 2: mask [x*sc + bi > 0]
// recomputed with the forward's arithmetic (y is not read).  The element-wise kernel also knows
// MODE 3: dz was written by this kernel into dres (the residual gradient is dz itself), read it there.
template <typename T, int MODE>
__global__ void __launch_bounds__(kT) bwd_partial_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                         const T* __restrict__ y,
                                                         const float* __restrict__ gamma,
                                                         const float* __restrict__ beta,
                                                         const float* __restrict__ mean,
                                                         const float* __restrict__ invstd, size_t m, int C,
                                                         float* __restrict__ part, T* __restrict__ dz_out) {
  const int lanes = C / 8, rows = kT / lanes;
  const int tid = threadIdx.x, o = tid % lanes, rl = tid / lanes;
  float acc[2][8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[0][e] = acc[1][e] = 0.f;
  if (rl < rows) {
    float mu[8], is[8], sc[8], bi[8];
    load8(mean + o * 8, mu);
    load8(invstd + o * 8, is);
    if (MODE == 2) {
      float ga[8], be[8];
      load8(gamma + o * 8, ga);
      load8(beta + o * 8, be);
#pragma unroll
      for (int e = 0; e < 8; ++e) bn_scale_bias(ga[e], be[e], mu[e], is[e], &sc[e], &bi[e]);
    }
    // four rows per round, all loads issued before the first use (a plain row loop is compiled to
    // one load in flight per thread)
    for_rows4<T>(m, C, lanes, rows, [&](size_t i0, size_t i1, size_t i2, size_t i3, auto NN) {
      constexpr int n = decltype(NN)::value;
      const size_t idx[4] = {i0, i1, i2, i3};
      float g[4][8], xv[4][8], yv[4][8];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (k < n) {
          load8(dy + idx[k], g[k]);
          load8(x + idx[k], xv[k]);
          if (MODE == 1) load8(y + idx[k], yv[k]);
        }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (k >= n) break;
        if (MODE == 1) {
#pragma unroll
          for (int e = 0; e < 8; ++e) g[k][e] = yv[k][e] > 0.f ? g[k][e] : 0.f;
        }
        if (MODE == 2) {
#pragma unroll
          for (int e = 0; e < 8; ++e) g[k][e] = fmaf(xv[k][e], sc[e], bi[e]) > 0.f ? g[k][e] : 0.f;
        }
        // the masked gradient is exact in the storage type (dy or 0): written here, it spares the
        // element-wise pass the reads of dy and y
        if (dz_out) store8(dz_out + idx[k], g[k]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          acc[0][e] += g[k][e];
          acc[1][e] = fmaf(g[k][e], xv[k][e] - mu[e], acc[1][e]);   // times invstd once, below
        }
      }
    });
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[1][e] *= is[e];
  }
  block_reduce_store<2>(acc, lanes, rows, C, part);
}

__global__ void __launch_bounds__(kT) bwd_finalize_kernel(const float* __restrict__ part, int nb, int C,
                                                          float* __restrict__ dgamma, float* __restrict__ dbeta) {
  const int c = blockIdx.x * kFinCh + (threadIdx.x >> 6);
  if (c >= C) return;
  double s1, s2;
  finalize_sums(part, nb, C, c, &s1, &s2);
  if ((threadIdx.x & 63) != 0) return;
  dbeta[c] = (float)s1;
  dgamma[c] = (float)s2;
}

__global__ void __launch_bounds__(kT) bwd_finalize_wide_kernel(const float* __restrict__ part, int nb, int C,
                                                               float* __restrict__ dgamma, float* __restrict__ dbeta) {
  double s1, s2;
  finalize_sums_wide(part, nb, C, blockIdx.x, &s1, &s2);
  if (threadIdx.x != 0) return;
  dbeta[blockIdx.x] = (float)s1;
  dgamma[blockIdx.x] = (float)s2;
}

template <typename T, int MODE>
__global__ void __launch_bounds__(kT) bwd_apply_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                       const T* __restrict__ y, const float* __restrict__ gamma,
                                                       const float* __restrict__ beta,
                                                       const float* __restrict__ mean,
                                                       const float* __restrict__ invstd,
                                                       const float* __restrict__ dgamma,
                                                       const float* __restrict__ dbeta, T* __restrict__ dx,
                                                       T* __restrict__ dres, size_t m, int C, float inv_m,
                                                       int flags) {
  const int lanes = C / 8, rows = kT / lanes;
  const int o = threadIdx.x % lanes;
  // dx = a * (dz - (dbeta + xhat * dgamma) / m), xhat = (x - mu) * is, a = gamma * is
  float a[8], mu[8], is[8], dgm[8], dbm[8], sc[8], bi[8];
  {
    float ga[8], dg[8], db[8];
    load8(gamma + o * 8, ga);
    load8(mean + o * 8, mu);
    load8(invstd + o * 8, is);
    load8(dgamma + o * 8, dg);
    load8(dbeta + o * 8, db);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[e] = ga[e] * is[e];
      dgm[e] = dg[e] * inv_m * is[e];   // xhat * dgamma / m = (x - mu) * (invstd * dgamma / m)
      dbm[e] = db[e] * inv_m;
    }
    if (MODE == 2) {
      float be[8];
      load8(beta + o * 8, be);
#pragma unroll
      for (int e = 0; e < 8; ++e) bn_scale_bias(ga[e], be[e], mu[e], is[e], &sc[e], &bi[e]);
    }
  }
  for_rows4<T>(m, C, lanes, rows, [&](size_t i0, size_t i1, size_t i2, size_t i3, auto NN) {
    constexpr int n = decltype(NN)::value;
    const size_t idx[4] = {i0, i1, i2, i3};
    float g[4][8], xv[4][8], yv[4][8];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (k < n) {
        load8((MODE == 3 ? dres : dy) + idx[k], g[k]);
        load8(x + idx[k], xv[k]);
        if (MODE == 1) load8(y + idx[k], yv[k]);
      }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (k >= n) break;
      float out[8];
      if (MODE == 1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) g[k][e] = yv[k][e] > 0.f ? g[k][e] : 0.f;
      }
      if (MODE == 2) {
#pragma unroll
        for (int e = 0; e < 8; ++e) g[k][e] = fmaf(xv[k][e], sc[e], bi[e]) > 0.f ? g[k][e] : 0.f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        out[e] = a[e] * (g[k][e] - fmaf(xv[k][e] - mu[e], dgm[e], dbm[e]));
      }
      if (flags & 1) {
        float old[8];
        load8(dx + idx[k], old);
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] += old[e];
      }
      store8(dx + idx[k], out);
      if (dres && MODE != 3) {
        if (flags & 2) {
          float old[8];
          load8(dres + idx[k], old);
#pragma unroll
          for (int e = 0; e < 8; ++e) g[k][e] += old[e];
        }
        store8(dres + idx[k], g[k]);
      }
    }
  });
}

// Grid of the element-wise kernels: every thread gets about eight rows, capped.
inline unsigned row_blocks(size_t m, int C) {
  const int rows = kT / (C / 8);
  size_t b = (m + (size_t)rows * 8 - 1) / ((size_t)rows * 8);
  if (b > 4096) b = 4096;
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
  if (nb >= kWideFinalize) sums_finalize_wide_kernel<<<C, kT, 0, st>>>(part, nb, C, ch_sum, ch_sumsq);
  else sums_finalize_kernel<<<fin_blocks(C), kT, 0, st>>>(part, nb, C, ch_sum, ch_sumsq);
  return launch_status();
}

size_t channel_stats_ws(size_t m, int C) { return (size_t)reduce_blocks(m, C) * 2 * C * sizeof(float); }

int channel_stats(int dtype, const void* x, size_t m, int C, float* ch_sum, float* ch_sumsq, void* ws,
                  hipStream_t st) {
  const int nb = reduce_blocks(m, C);
  float* part = (float*)ws;
  if (dtype == CNNK_BF16) {
    stats_partial_kernel<bf16_t><<<nb, kT, 0, st>>>((const bf16_t*)x, m, C, part);
    stats_finalize_kernel<bf16_t><<<fin_blocks(C), kT, 0, st>>>(part, nb, (const bf16_t*)x, m, C, 1, 0.f, 0.f,
                                                                    ch_sum, ch_sumsq, nullptr, nullptr);
  } else {
    stats_partial_kernel<float><<<nb, kT, 0, st>>>((const float*)x, m, C, part);
    stats_finalize_kernel<float><<<fin_blocks(C), kT, 0, st>>>(part, nb, (const float*)x, m, C, 1, 0.f, 0.f,
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
      stats_finalize_kernel<bf16_t><<<fin_blocks(C), kT, 0, st>>>(part, nb, (const bf16_t*)x, m, C, 0, d->eps,
                                                                      d->momentum, save_mean, save_invstd,
                                                                      running_mean, running_var);
    } else {
      stats_partial_kernel<float><<<nb, kT, 0, st>>>((const float*)x, m, C, part);
      stats_finalize_kernel<float><<<fin_blocks(C), kT, 0, st>>>(part, nb, (const float*)x, m, C, 0, d->eps,
                                                                     d->momentum, save_mean, save_invstd,
                                                                     running_mean, running_var);
    }
  } else {
    // statistics handed in as sums: one fused kernel (statistics + normalise)
    const float inv_m = (float)(1.0 / (double)m);
    const float unbias = m > 1 ? (float)((double)m / ((double)m - 1.0)) : 1.f;
    if (d->dtype == CNNK_BF16)
      bn_apply_sums_kernel<bf16_t><<<row_blocks(m, C), kT, 0, st>>>((const bf16_t*)x, (const bf16_t*)residual, gamma, beta,
                                                                 ch_sum, ch_sumsq, inv_m, unbias, d->eps, d->momentum,
                                                                 save_mean, save_invstd, running_mean, running_var,
                                                                 (bf16_t*)y, m, C, d->relu);
    else
      bn_apply_sums_kernel<float><<<row_blocks(m, C), kT, 0, st>>>((const float*)x, (const float*)residual, gamma, beta,
                                                                ch_sum, ch_sumsq, inv_m, unbias, d->eps, d->momentum,
                                                                save_mean, save_invstd, running_mean, running_var,
                                                                (float*)y, m, C, d->relu);
    return launch_status();
  }
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  if (d->dtype == CNNK_BF16)
    bn_apply_kernel<bf16_t><<<row_blocks(m, C), kT, 0, st>>>((const bf16_t*)x, (const bf16_t*)residual, gamma, beta,
                                                          save_mean, save_invstd, (bf16_t*)y, m, C, d->relu);
  else
    bn_apply_kernel<float><<<row_blocks(m, C), kT, 0, st>>>((const float*)x, (const float*)residual, gamma, beta,
                                                         save_mean, save_invstd, (float*)y, m, C, d->relu);
  return launch_status();
}

extern "C" int cnnk_bn_relu_infer(const cnnk_bn_desc* d, const void* x, const void* residual, const float* gamma,
                                  const float* beta, const float* running_mean, const float* running_var,
                                  void* y, void* stream) {
  int rc = validate_bn(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !gamma || !beta || !running_mean || !running_var || !y) return CNNK_ERR_NULL;
  const size_t m = (size_t)d->N * d->H * d->W;
  const int C = d->C;
  hipStream_t st = (hipStream_t)stream;
  if (d->dtype == CNNK_BF16)
    bn_infer_kernel<bf16_t><<<row_blocks(m, C), kT, 0, st>>>((const bf16_t*)x, (const bf16_t*)residual, gamma, beta,
                                                          running_mean, running_var, d->eps, (bf16_t*)y, m, C,
                                                          d->relu);
  else
    bn_infer_kernel<float><<<row_blocks(m, C), kT, 0, st>>>((const float*)x, (const float*)residual, gamma, beta,
                                                         running_mean, running_var, d->eps, (float*)y, m, C,
                                                         d->relu);
  return launch_status();
}

template <typename T, int MODE>
static int bn_bwd_launch(const cnnk_bn_desc* d, const void* dy, const void* x, const void* y, const float* gamma,
                         const float* beta, const float* save_mean, const float* save_invstd, void* dx,
                         void* dresidual, int flags, float* dgamma, float* dbeta, float* part, hipStream_t st) {
  const size_t m = (size_t)d->N * d->H * d->W;
  const int C = d->C;
  const int nb = reduce_blocks(m, C);
  const float inv_m = (float)(1.0 / (double)m);
  // a residual gradient that is written, not accumulated, is written by the first pass already
  const bool dz_first = MODE == 1 && dresidual && !(flags & 2);
  bwd_partial_kernel<T, MODE><<<nb, kT, 0, st>>>((const T*)dy, (const T*)x, (const T*)y, gamma, beta, save_mean,
                                                 save_invstd, m, C, part, dz_first ? (T*)dresidual : nullptr);
  if (nb >= kWideFinalize) bwd_finalize_wide_kernel<<<C, kT, 0, st>>>(part, nb, C, dgamma, dbeta);
  else bwd_finalize_kernel<<<fin_blocks(C), kT, 0, st>>>(part, nb, C, dgamma, dbeta);
  if (dz_first)
    bwd_apply_kernel<T, 3><<<row_blocks(m, C), kT, 0, st>>>((const T*)dy, (const T*)x, (const T*)y, gamma, beta,
                                                            save_mean, save_invstd, dgamma, dbeta, (T*)dx,
                                                            (T*)dresidual, m, C, inv_m, flags);
  else
    bwd_apply_kernel<T, MODE><<<row_blocks(m, C), kT, 0, st>>>((const T*)dy, (const T*)x, (const T*)y, gamma, beta,
                                                               save_mean, save_invstd, dgamma, dbeta, (T*)dx,
                                                               (T*)dresidual, m, C, inv_m, flags);
  return launch_status();
}

extern "C" int cnnk_bn_relu_bwd(const cnnk_bn_desc* d, const void* dy, const void* x, const void* y,
                                const float* gamma, const float* beta, const float* save_mean,
                                const float* save_invstd, void* dx, void* dresidual, int flags, float* dgamma,
                                float* dbeta, void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_bn(d);
  if (rc != CNNK_OK) return rc;
  if (!dy || !x || !gamma || !save_mean || !save_invstd || !dx || !dgamma || !dbeta) return CNNK_ERR_NULL;
  // ReLU mask: from y, or recomputed from x when y is withheld (no residual branch, beta given)
  if (d->relu && !y && (!beta || dresidual)) return CNNK_ERR_NULL;
  const int mode = !d->relu ? 0 : (y ? 1 : 2);
  const size_t m = (size_t)d->N * d->H * d->W;
  if (!ws || ws_bytes < channel_stats_ws(m, d->C)) return CNNK_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  float* part = (float*)ws;
#define CNNK_BN_BWD(T, MODE) \
  return bn_bwd_launch<T, MODE>(d, dy, x, y, gamma, beta, save_mean, save_invstd, dx, dresidual, flags, dgamma, \
                                dbeta, part, st)
  if (d->dtype == CNNK_BF16) {
    if (mode == 0) CNNK_BN_BWD(bf16_t, 0);
    if (mode == 1) CNNK_BN_BWD(bf16_t, 1);
    CNNK_BN_BWD(bf16_t, 2);
  }
  if (mode == 0) CNNK_BN_BWD(float, 0);
  if (mode == 1) CNNK_BN_BWD(float, 1);
  CNNK_BN_BWD(float, 2);
#undef CNNK_BN_BWD
}
