// Operators of the Vision Transformer step other than its matrix products (Section IV-A's second
// model; standard pre-norm ViT): layer normalisation, bias + GELU + residual, patch extraction and
// token assembly.  All are bound by memory traffic: 8- or 16-byte accesses, fp32 arithmetic,
// reductions over rows as per-workgroup partial sums that a second launch adds in a fixed order.
#include "common.h"
#include "../../include/cnnk_vit.h"

namespace {
constexpr int kT = 256;

// ---- 4 consecutive elements <-> 4 floats ---------------------------------------------------------
__device__ __forceinline__ void load4(const bf16_t* p, float* f) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
}
__device__ __forceinline__ void load4(const float* p, float* f) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
}
__device__ __forceinline__ void store4(bf16_t* p, const float* f) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]));
}
__device__ __forceinline__ void store4(float* p, const float* f) {
  *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
}

// ---- layer normalisation ---------------------------------------------------------------------------
// One wavefront per row; a lane holds NQ quads of the row (quad i of lane l covers elements
// (i * 64 + l) * 4 ...), so the row is read once and both passes of the variance run in registers.
template <typename T, int NQ>
__global__ void __launch_bounds__(kT) ln_fwd_kernel(const T* __restrict__ x, long long xs, const float* __restrict__ g,
                                                    const float* __restrict__ b, T* __restrict__ y,
                                                    float* __restrict__ stats, int rows, int C, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (kT / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* xr = x + (size_t)row * xs;
  float v[NQ][4];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < C) load4(xr + c, v[i]);
    else v[i][0] = v[i][1] = v[i][2] = v[i][3] = 0.f;
    s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
  }
  const float mean = wave_sum(s) / (float)C;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < C) {
#pragma unroll
      for (int k = 0; k < 4; ++k) { const float d = v[i][k] - mean; q += d * d; }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)C + eps);
  T* yr = y + (size_t)row * C;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < C) {
      const float4 gg = *reinterpret_cast<const float4*>(g + c);
      const float4 bb = *reinterpret_cast<const float4*>(b + c);
      float o[4] = {(v[i][0] - mean) * rstd * gg.x + bb.x, (v[i][1] - mean) * rstd * gg.y + bb.y,
                    (v[i][2] - mean) * rstd * gg.z + bb.z, (v[i][3] - mean) * rstd * gg.w + bb.w};
      store4(yr + c, o);
    }
  }
  if (lane == 0) { stats[2 * (size_t)row] = mean; stats[2 * (size_t)row + 1] = rstd; }
}

// A wavefront walks its rows RU at a time (1 as launched: two rows in flight cost the registers that
// a second resident workgroup needs, 40 against 27 us at ViT-B/16's shape); per row two
// wave reductions give the two projections that the normalisation removes; the lane keeps its
// columns' contributions to dgamma / dbeta in registers over all its rows.  The four wavefronts of a
// workgroup then add theirs in LDS one after the other (fixed order) and the workgroup writes one
// partial row.  VW elements per access (8 where C allows), NV vectors of the row per lane.
template <int VW, typename T> __device__ __forceinline__ void loadv(const T* p, float* f) {
  if (VW == 8) load8(p, f); else load4(p, f);
}
template <int VW, typename T> __device__ __forceinline__ void storev(T* p, const float* f) {
  if (VW == 8) store8(p, f); else store4(p, f);
}

template <typename T, int NV, int VW, int RU>
__global__ void __launch_bounds__(kT) ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x, long long xs,
                                                    const float* __restrict__ g, const float* __restrict__ stats,
                                                    const T* dres, T* dx, float* __restrict__ part, int rows, int C) {
  extern __shared__ float sm[];     // [2][C]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float gg[NV][VW], ag[NV][VW], ab[NV][VW];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 64 + lane) * VW;
#pragma unroll
    for (int k = 0; k < VW; ++k) { ag[i][k] = 0.f; ab[i][k] = 0.f; gg[i][k] = 0.f; }
    if (c < C) loadv<VW>(g + c, gg[i]);
  }
  const int stride = gridDim.x * (kT / 64);
  for (int row0 = blockIdx.x * (kT / 64) + wave; row0 < rows; row0 += RU * stride) {
    float d[RU][NV][VW], xh[RU][NV][VW], rr[RU][NV][VW];
    float mean[RU], rstd[RU];
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int row = row0 + u * stride;
      const bool live = row < rows;
      mean[u] = live ? stats[2 * (size_t)row] : 0.f;
      rstd[u] = live ? stats[2 * (size_t)row + 1] : 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * VW;
        if (live && c < C) {
          loadv<VW>(dy + (size_t)row * C + c, d[u][i]);
          loadv<VW>(x + (size_t)row * xs + c, xh[u][i]);
          if (dres) loadv<VW>(dres + (size_t)row * xs + c, rr[u][i]);
        } else {
#pragma unroll
          for (int k = 0; k < VW; ++k) { d[u][i][k] = 0.f; xh[u][i][k] = mean[u]; }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int row = row0 + u * stride;
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int k = 0; k < VW; ++k) {
          xh[u][i][k] = (xh[u][i][k] - mean[u]) * rstd[u];
          ab[i][k] += d[u][i][k];
          ag[i][k] += d[u][i][k] * xh[u][i][k];
          d[u][i][k] *= gg[i][k];
          s1 += d[u][i][k];
          s2 += d[u][i][k] * xh[u][i][k];
        }
      s1 = wave_sum(s1) / (float)C;
      s2 = wave_sum(s2) / (float)C;
      if (row < rows) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const int c = (i * 64 + lane) * VW;
          if (c < C) {
            float o[VW];
#pragma unroll
            for (int k = 0; k < VW; ++k) o[k] = rstd[u] * (d[u][i][k] - s1 - xh[u][i][k] * s2) + (dres ? rr[u][i][k] : 0.f);
            storev<VW>(dx + (size_t)row * xs + c, o);
          }
        }
      }
    }
  }
  for (int w = 0; w < kT / 64; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * 64 + lane) * VW;
        if (c < C) {
#pragma unroll
          for (int k = 0; k < VW; ++k) {
            sm[c + k] = (w ? sm[c + k] : 0.f) + ag[i][k];
            sm[C + c + k] = (w ? sm[C + c + k] : 0.f) + ab[i][k];
          }
        }
      }
    }
    __syncthreads();
  }
  for (int c = threadIdx.x; c < 2 * C; c += kT) part[(size_t)blockIdx.x * 2 * C + c] = sm[c];
}

// out[c] = sum_b part[b][c]; columns [0, n0) go to out0, the rest to out1.  A workgroup owns 64
// columns; four threads per column each add every fourth partial (sixteen loads in flight), then the
// four meet in LDS: a fixed order, so the sums are reproducible.
__global__ void __launch_bounds__(kT) colsum_finalize_kernel(const float* __restrict__ part, int nb, int n, int n0,
                                                             float* __restrict__ out0, float* __restrict__ out1) {
  __shared__ float sm[4][64];
  const int cl = threadIdx.x & 63, pl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  float s = 0.f;
  if (c < n) {
    int b = pl;
    for (; b + 60 < nb; b += 64) {
      float t[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) t[k] = part[(size_t)(b + 4 * k) * n + c];
#pragma unroll
      for (int k = 0; k < 16; ++k) s += t[k];
    }
    for (; b < nb; b += 4) s += part[(size_t)b * n + c];
  }
  sm[pl][cl] = s;
  __syncthreads();
  if (pl == 0 && c < n) {
    const float r = (sm[0][cl] + sm[1][cl]) + (sm[2][cl] + sm[3][cl]);
    if (c < n0) out0[c] = r; else out1[c - n0] = r;
  }
}

// ---- bias, GELU, residual ----------------------------------------------------------------------------
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * __expf(-0.5f * u * u) * 0.39894228040143268f;
}

template <typename T, int ACT, bool RES>
__global__ void __launch_bounds__(kT) bias_act_fwd_kernel(const T* z, const float* __restrict__ bias, const T* res, T* u,
                                                          T* y, size_t octets, int C8) {
  for (size_t o = (size_t)blockIdx.x * kT + threadIdx.x; o < octets; o += (size_t)gridDim.x * kT) {
    const int c = (int)(o % (size_t)C8) * 8;
    float v[8], bb[8];
    load8(z + o * 8, v);
    load8(bias + c, bb);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] += bb[k];
    if (ACT == CNNK_ACT_GELU) {
      store8(u + o * 8, v);
      // the activation is taken of the stored value, which the backward pass will read
      if (sizeof(T) == 2) {
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = bf16_to_f32(f32_to_bf16_hw(v[k]));
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = gelu_f(v[k]);
    }
    if (RES) {
      float r[8];
      load8(res + o * 8, r);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] += r[k];
    }
    store8(y + o * 8, v);
  }
}

// 32 column octets x 8 row lanes per workgroup; blockIdx.x = slab of 256 columns, blockIdx.y = row
// chunk.  A thread adds its column octet over its rows, the 8 row lanes meet in LDS.
template <typename T, int ACT>
__global__ void __launch_bounds__(kT) bias_act_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ u, T* dz,
                                                          float* __restrict__ part, long long rows, int C,
                                                          long long rows_per_chunk) {
  __shared__ float sm[8][257];
  const int oc = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int c = blockIdx.x * 256 + oc * 8;
  const long long r0 = (long long)blockIdx.y * rows_per_chunk;
  long long r1 = r0 + rows_per_chunk;
  if (r1 > rows) r1 = rows;
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  if (c < C) {
    long long r = r0 + rl;
    for (; r + 8 < r1; r += 16) {          // two rows in flight
      float a[8], b[8], ua[8], ub[8];
      load8(dy + (size_t)r * C + c, a);
      load8(dy + (size_t)(r + 8) * C + c, b);
      if (ACT == CNNK_ACT_GELU) {
        load8(u + (size_t)r * C + c, ua);
        load8(u + (size_t)(r + 8) * C + c, ub);
#pragma unroll
        for (int k = 0; k < 8; ++k) { a[k] *= gelu_grad_f(ua[k]); b[k] *= gelu_grad_f(ub[k]); }
        store8(dz + (size_t)r * C + c, a);
        store8(dz + (size_t)(r + 8) * C + c, b);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] += a[k];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] += b[k];
    }
    for (; r < r1; r += 8) {
      float a[8], ua[8];
      load8(dy + (size_t)r * C + c, a);
      if (ACT == CNNK_ACT_GELU) {
        load8(u + (size_t)r * C + c, ua);
#pragma unroll
        for (int k = 0; k < 8; ++k) a[k] *= gelu_grad_f(ua[k]);
        store8(dz + (size_t)r * C + c, a);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] += a[k];
    }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) sm[rl][oc * 8 + k] = acc[k];
  __syncthreads();
  const int cc = blockIdx.x * 256 + threadIdx.x;
  if (cc < C) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) s += sm[k][threadIdx.x];
    part[(size_t)blockIdx.y * C + cc] = s;
  }
}

// ---- patches and tokens --------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(kT) patchify_kernel(const T* __restrict__ x, T* __restrict__ out, size_t total, int image,
                                                      int p, int gw) {
  const int K = p * p * 3, n = gw * gw, rowlen = p * 3;
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < total; i += (size_t)gridDim.x * kT) {
    const int k = (int)(i % (size_t)K);
    const size_t bi = i / (size_t)K;
    const int pi = (int)(bi % (size_t)n);
    const size_t b = bi / (size_t)n;
    const int py = pi / gw, px = pi - py * gw;
    const int r = k / rowlen, sc = k - r * rowlen;
    out[i] = x[((b * image + (size_t)(py * p + r)) * image + (size_t)px * p) * 3 + sc];
  }
}

template <typename T>
__global__ void __launch_bounds__(kT) embed_fwd_kernel(const T* __restrict__ z, const float* __restrict__ be,
                                                       const float* __restrict__ cls, const float* __restrict__ pos,
                                                       T* __restrict__ tok, size_t octets, int Tn, int D8) {
  for (size_t o = (size_t)blockIdx.x * kT + threadIdx.x; o < octets; o += (size_t)gridDim.x * kT) {
    const int c = (int)(o % (size_t)D8) * 8;
    const size_t bt = o / (size_t)D8;
    const int t = (int)(bt % (size_t)Tn);
    const size_t b = bt / (size_t)Tn;
    float v[8], a[8], pp[8];
    load8(pos + (size_t)t * D8 * 8 + c, pp);
    if (t == 0) {
      load8(cls + c, v);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] += pp[k];
    } else {
      load8(z + ((b * (Tn - 1) + (size_t)(t - 1)) * D8) * 8 + c, v);
      load8(be + c, a);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = v[k] + a[k] + pp[k];
    }
    store8(tok + o * 8, v);
  }
}

// dz = the patch rows of dtok (a conversion to float and back is exact); dpos[t] = sum over the batch
// (b ascending) of dtok[b][t].  One thread per octet of one image's token block.
template <typename T>
__global__ void __launch_bounds__(kT) embed_bwd_kernel(const T* __restrict__ dtok, T* __restrict__ dz,
                                                       float* __restrict__ dpos, int B, int Tn, int D8) {
  const size_t o = (size_t)blockIdx.x * kT + threadIdx.x;
  if (o >= (size_t)Tn * D8) return;
  const int t = (int)(o / (size_t)D8);
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  for (int b = 0; b < B; ++b) {
    float v[8];
    load8(dtok + ((size_t)b * Tn * D8 + o) * 8, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] += v[k];
    if (t > 0) store8(dz + ((size_t)b * (Tn - 1) * D8 + (o - (size_t)D8)) * 8, v);
  }
  store8(dpos + o * 8, acc);
}

// dcls = dpos[0]; dbe[c] = sum over the patch positions t = 1.. (ascending) of dpos[t][c]
__global__ void __launch_bounds__(kT) embed_bwd_finalize_kernel(const float* __restrict__ dpos, float* __restrict__ dbe,
                                                                float* __restrict__ dcls, int Tn, int D) {
  const int c = blockIdx.x * kT + threadIdx.x;
  if (c >= D) return;
  dcls[c] = dpos[c];
  float s = 0.f;
  for (int t = 1; t < Tn; ++t) s += dpos[(size_t)t * D + c];
  dbe[c] = s;
}

__global__ void __launch_bounds__(kT) fill_zero_kernel(uint4* p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n16; i += (size_t)gridDim.x * kT) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

inline unsigned grid_for(size_t work_items, unsigned cap = 8192) {
  size_t b = (work_items + kT - 1) / kT;
  return (unsigned)(b < 1 ? 1 : (b > cap ? cap : b));
}
inline int ln_nq(int C) { return C <= 256 ? 1 : C <= 1024 ? 4 : 16; }
inline int ln_bwd_blocks(int rows) { int b = (rows + 7) / 8; return b < 1 ? 1 : (b > 768 ? 768 : b); }
inline bool aligned16(const void* p) { return (((size_t)p) & 15) == 0; }
}  // namespace

// ---- entry points ------------------------------------------------------------------------------------------
static int check_ln(const cnnk_ln_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->rows <= 0 || d->C <= 0 || d->x_stride < 0 || !(d->eps >= 0.f)) return CNNK_ERR_SHAPE;
  if (d->x_stride != 0 && d->x_stride < d->C) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (d->C % 4 != 0 || d->C > 4096 || (d->x_stride % 4) != 0) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

template <typename T>
static void launch_ln_fwd(const cnnk_ln_desc* d, long long xs, const void* x, const float* g, const float* b, void* y,
                          float* stats, hipStream_t st) {
  const unsigned grid = (unsigned)((d->rows + 3) / 4);
  switch (ln_nq(d->C)) {
    case 1: ln_fwd_kernel<T, 1><<<grid, kT, 0, st>>>((const T*)x, xs, g, b, (T*)y, stats, d->rows, d->C, d->eps); break;
    case 4: ln_fwd_kernel<T, 4><<<grid, kT, 0, st>>>((const T*)x, xs, g, b, (T*)y, stats, d->rows, d->C, d->eps); break;
    default: ln_fwd_kernel<T, 16><<<grid, kT, 0, st>>>((const T*)x, xs, g, b, (T*)y, stats, d->rows, d->C, d->eps); break;
  }
}

extern "C" int cnnk_layernorm_fwd(const cnnk_ln_desc* d, const void* x, const float* gamma, const float* beta, void* y,
                                  float* stats, void* stream) {
  const int rc = check_ln(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !gamma || !beta || !y || !stats) return CNNK_ERR_NULL;
  if (!aligned16(x) || !aligned16(y) || !aligned16(gamma) || !aligned16(beta)) return CNNK_ERR_UNSUPPORTED;
  const long long xs = d->x_stride ? d->x_stride : d->C;
  if (d->dtype == CNNK_BF16) launch_ln_fwd<bf16_t>(d, xs, x, gamma, beta, y, stats, (hipStream_t)stream);
  else launch_ln_fwd<float>(d, xs, x, gamma, beta, y, stats, (hipStream_t)stream);
  return launch_status();
}

extern "C" size_t cnnk_layernorm_workspace_bytes(const cnnk_ln_desc* d) {
  if (check_ln(d) != CNNK_OK) return 0;
  return align_up((size_t)ln_bwd_blocks(d->rows) * 2 * d->C * sizeof(float), 256);
}

template <typename T>
static void launch_ln_bwd(const cnnk_ln_desc* d, long long xs, int nb, const void* dy, const void* x, const float* g,
                          const float* stats, const void* dres, void* dx, float* part, hipStream_t st) {
  const size_t lds = (size_t)2 * d->C * sizeof(float);
#define LN_BWD(NV, VW) ln_bwd_kernel<T, NV, VW, 1><<<nb, kT, lds, st>>>((const T*)dy, (const T*)x, xs, g, stats, (const T*)dres, (T*)dx, part, d->rows, d->C)
  if (d->C % 8 == 0 && xs % 8 == 0) {
    if (d->C <= 512) LN_BWD(1, 8); else if (d->C <= 1024) LN_BWD(2, 8); else if (d->C <= 2048) LN_BWD(4, 8); else LN_BWD(8, 8);
  } else {
    if (d->C <= 256) LN_BWD(1, 4); else if (d->C <= 1024) LN_BWD(4, 4); else LN_BWD(16, 4);
  }
#undef LN_BWD
}

extern "C" int cnnk_layernorm_bwd(const cnnk_ln_desc* d, const void* dy, const void* x, const float* gamma,
                                  const float* stats, const void* dres, void* dx, float* dgamma, float* dbeta, void* ws,
                                  size_t ws_bytes, void* stream) {
  const int rc = check_ln(d);
  if (rc != CNNK_OK) return rc;
  if (!dy || !x || !gamma || !stats || !dx || !dgamma || !dbeta) return CNNK_ERR_NULL;
  if (!ws || ws_bytes < cnnk_layernorm_workspace_bytes(d)) return CNNK_ERR_WORKSPACE;
  if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(gamma) || (dres && !aligned16(dres)) || !aligned16(ws))
    return CNNK_ERR_UNSUPPORTED;
  const long long xs = d->x_stride ? d->x_stride : d->C;
  const int nb = ln_bwd_blocks(d->rows);
  hipStream_t st = (hipStream_t)stream;
  if (d->dtype == CNNK_BF16) launch_ln_bwd<bf16_t>(d, xs, nb, dy, x, gamma, stats, dres, dx, (float*)ws, st);
  else launch_ln_bwd<float>(d, xs, nb, dy, x, gamma, stats, dres, dx, (float*)ws, st);
  colsum_finalize_kernel<<<(2 * d->C + 63) / 64, kT, 0, st>>>((const float*)ws, nb, 2 * d->C, d->C, dgamma, dbeta);
  return launch_status();
}

static int check_rows(long long rows, int C, int dtype) {
  if (rows <= 0 || C <= 0) return CNNK_ERR_SHAPE;
  if (dtype != CNNK_F32 && dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (C % 8 != 0 || (double)rows * C > 2147483647.0 * 8) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

template <typename T>
static void launch_bias_fwd(int act, bool res, unsigned grid, const void* z, const float* bias, const void* r, void* u,
                            void* y, size_t octets, int C8, hipStream_t st) {
  if (act == CNNK_ACT_GELU)
    bias_act_fwd_kernel<T, CNNK_ACT_GELU, false><<<grid, kT, 0, st>>>((const T*)z, bias, nullptr, (T*)u, (T*)y, octets, C8);
  else if (res)
    bias_act_fwd_kernel<T, CNNK_ACT_NONE, true><<<grid, kT, 0, st>>>((const T*)z, bias, (const T*)r, nullptr, (T*)y, octets, C8);
  else
    bias_act_fwd_kernel<T, CNNK_ACT_NONE, false><<<grid, kT, 0, st>>>((const T*)z, bias, nullptr, nullptr, (T*)y, octets, C8);
}

extern "C" int cnnk_bias_act_fwd(long long rows, int C, int dtype, int act, const void* z, const float* bias,
                                 const void* res, void* u, void* y, void* stream) {
  const int rc = check_rows(rows, C, dtype);
  if (rc != CNNK_OK) return rc;
  if (act != CNNK_ACT_NONE && act != CNNK_ACT_GELU) return CNNK_ERR_UNSUPPORTED;
  if (!z || !bias || !y || (act == CNNK_ACT_GELU && !u)) return CNNK_ERR_NULL;
  if (act == CNNK_ACT_GELU && res) return CNNK_ERR_UNSUPPORTED;
  if (!aligned16(z) || !aligned16(y) || !aligned16(bias) || (res && !aligned16(res)) || (u && !aligned16(u)))
    return CNNK_ERR_UNSUPPORTED;
  const size_t octets = (size_t)rows * C / 8;
  const unsigned grid = grid_for(octets);
  if (dtype == CNNK_BF16) launch_bias_fwd<bf16_t>(act, res != nullptr, grid, z, bias, res, u, y, octets, C / 8, (hipStream_t)stream);
  else launch_bias_fwd<float>(act, res != nullptr, grid, z, bias, res, u, y, octets, C / 8, (hipStream_t)stream);
  return launch_status();
}

static int colsum_chunks(long long rows, int C) {
  const int slabs = (C + 255) / 256;
  long long want = 2048 / slabs;
  if (want < 1) want = 1;
  long long by_rows = (rows + 63) / 64;
  if (want > by_rows) want = by_rows;
  return (int)(want < 1 ? 1 : want);
}

extern "C" size_t cnnk_bias_act_workspace_bytes(long long rows, int C) {
  if (rows <= 0 || C <= 0) return 0;
  return align_up((size_t)colsum_chunks(rows, C) * C * sizeof(float), 256);
}

extern "C" int cnnk_bias_act_bwd(long long rows, int C, int dtype, int act, const void* dy, const void* u, void* dz,
                                 float* dbias, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_rows(rows, C, dtype);
  if (rc != CNNK_OK) return rc;
  if (act != CNNK_ACT_NONE && act != CNNK_ACT_GELU) return CNNK_ERR_UNSUPPORTED;
  if (!dy || !dbias || (act == CNNK_ACT_GELU && (!u || !dz))) return CNNK_ERR_NULL;
  if (!ws || ws_bytes < cnnk_bias_act_workspace_bytes(rows, C)) return CNNK_ERR_WORKSPACE;
  if (!aligned16(dy) || (u && !aligned16(u)) || (dz && !aligned16(dz)) || !aligned16(ws)) return CNNK_ERR_UNSUPPORTED;
  const int chunks = colsum_chunks(rows, C);
  const long long rpc = (rows + chunks - 1) / chunks;
  const dim3 grid((C + 255) / 256, chunks);
  hipStream_t st = (hipStream_t)stream;
  float* part = (float*)ws;
  if (dtype == CNNK_BF16) {
    if (act == CNNK_ACT_GELU) bias_act_bwd_kernel<bf16_t, CNNK_ACT_GELU><<<grid, kT, 0, st>>>((const bf16_t*)dy, (const bf16_t*)u, (bf16_t*)dz, part, rows, C, rpc);
    else bias_act_bwd_kernel<bf16_t, CNNK_ACT_NONE><<<grid, kT, 0, st>>>((const bf16_t*)dy, nullptr, nullptr, part, rows, C, rpc);
  } else {
    if (act == CNNK_ACT_GELU) bias_act_bwd_kernel<float, CNNK_ACT_GELU><<<grid, kT, 0, st>>>((const float*)dy, (const float*)u, (float*)dz, part, rows, C, rpc);
    else bias_act_bwd_kernel<float, CNNK_ACT_NONE><<<grid, kT, 0, st>>>((const float*)dy, nullptr, nullptr, part, rows, C, rpc);
  }
  colsum_finalize_kernel<<<(C + 63) / 64, kT, 0, st>>>(part, chunks, C, C, dbias, nullptr);
  return launch_status();
}

static int check_embed(const cnnk_embed_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->B <= 0 || d->image <= 0 || d->patch <= 0 || d->dim <= 0 || d->image % d->patch != 0) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (d->dim % 8 != 0) return CNNK_ERR_UNSUPPORTED;
  const double n = (double)(d->image / d->patch) * (d->image / d->patch);
  if ((double)d->B * d->image * d->image * 3 > 2147483647.0 || (double)d->B * (n + 1) * d->dim > 2147483647.0)
    return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

extern "C" int cnnk_vit_patchify(const cnnk_embed_desc* d, const void* x, void* patches, void* stream) {
  const int rc = check_embed(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !patches) return CNNK_ERR_NULL;
  const int gw = d->image / d->patch;
  const size_t total = (size_t)d->B * gw * gw * d->patch * d->patch * 3;
  if (d->dtype == CNNK_BF16)
    patchify_kernel<bf16_t><<<grid_for(total, 16384), kT, 0, (hipStream_t)stream>>>((const bf16_t*)x, (bf16_t*)patches, total, d->image, d->patch, gw);
  else
    patchify_kernel<float><<<grid_for(total, 16384), kT, 0, (hipStream_t)stream>>>((const float*)x, (float*)patches, total, d->image, d->patch, gw);
  return launch_status();
}

extern "C" int cnnk_vit_embed_fwd(const cnnk_embed_desc* d, const void* z, const float* be, const float* cls,
                                  const float* pos, void* tok, void* stream) {
  const int rc = check_embed(d);
  if (rc != CNNK_OK) return rc;
  if (!z || !be || !cls || !pos || !tok) return CNNK_ERR_NULL;
  if (!aligned16(z) || !aligned16(be) || !aligned16(cls) || !aligned16(pos) || !aligned16(tok)) return CNNK_ERR_UNSUPPORTED;
  const int Tn = (d->image / d->patch) * (d->image / d->patch) + 1;
  const size_t octets = (size_t)d->B * Tn * d->dim / 8;
  if (d->dtype == CNNK_BF16)
    embed_fwd_kernel<bf16_t><<<grid_for(octets), kT, 0, (hipStream_t)stream>>>((const bf16_t*)z, be, cls, pos, (bf16_t*)tok, octets, Tn, d->dim / 8);
  else
    embed_fwd_kernel<float><<<grid_for(octets), kT, 0, (hipStream_t)stream>>>((const float*)z, be, cls, pos, (float*)tok, octets, Tn, d->dim / 8);
  return launch_status();
}

extern "C" int cnnk_vit_embed_bwd(const cnnk_embed_desc* d, const void* dtok, void* dz, float* dbe, float* dcls,
                                  float* dpos, void* stream) {
  const int rc = check_embed(d);
  if (rc != CNNK_OK) return rc;
  if (!dtok || !dz || !dbe || !dcls || !dpos) return CNNK_ERR_NULL;
  if (!aligned16(dtok) || !aligned16(dz) || !aligned16(dpos)) return CNNK_ERR_UNSUPPORTED;
  const int Tn = (d->image / d->patch) * (d->image / d->patch) + 1;
  const size_t octets = (size_t)Tn * d->dim / 8;
  hipStream_t st = (hipStream_t)stream;
  if (d->dtype == CNNK_BF16)
    embed_bwd_kernel<bf16_t><<<(unsigned)((octets + kT - 1) / kT), kT, 0, st>>>((const bf16_t*)dtok, (bf16_t*)dz, dpos, d->B, Tn, d->dim / 8);
  else
    embed_bwd_kernel<float><<<(unsigned)((octets + kT - 1) / kT), kT, 0, st>>>((const float*)dtok, (float*)dz, dpos, d->B, Tn, d->dim / 8);
  embed_bwd_finalize_kernel<<<(d->dim + kT - 1) / kT, kT, 0, st>>>(dpos, dbe, dcls, Tn, d->dim);
  return launch_status();
}

// used by the step: zero n bytes (n % 16 == 0, p 16-byte aligned) without a memset node
int cnnk_fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return CNNK_OK;
  fill_zero_kernel<<<grid_for(bytes / 16, 4096), kT, 0, st>>>((uint4*)p, bytes / 16);
  return launch_status();
}
