// Pooling, element-wise sums and gradient routing: bandwidth-bound kernels moving vectors of 8
// channels per thread (NHWC, C a multiple of 8).
#include "common.h"

namespace {
constexpr int kT = 256;

inline unsigned ew_blocks(size_t n) {
  size_t b = (n + kT - 1) / kT;
  if (b > 16384) b = 16384;
  return (unsigned)(b < 1 ? 1 : b);
}

template <typename T>
__global__ void __launch_bounds__(kT) maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                         unsigned char* __restrict__ am, int N, int H, int W, int C) {
  const int Ho = H / 2, Wo = W / 2, C8 = C / 8;
  const size_t total = (size_t)N * Ho * Wo * C8;
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < total; i += (size_t)gridDim.x * kT) {
    const int c8 = (int)(i % C8);
    size_t p = i / C8;
    const int wo = (int)(p % Wo); p /= Wo;
    const int ho = (int)(p % Ho);
    const int n = (int)(p / Ho);
    float best[8];
    unsigned char code[8];
    const T* base = x + (((size_t)n * H + 2 * ho) * W + 2 * wo) * C + c8 * 8;
    load8(base, best);
#pragma unroll
    for (int e = 0; e < 8; ++e) code[e] = 0;
#pragma unroll
    for (int k = 1; k < 4; ++k) {
      float v[8];
      load8(base + ((size_t)(k >> 1) * W + (k & 1)) * C, v);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (v[e] > best[e]) { best[e] = v[e]; code[e] = (unsigned char)k; }
    }
    store8(y + i * 8, best);
    uint2 pk;
    pk.x = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
    pk.y = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
    *reinterpret_cast<uint2*>(am + i * 8) = pk;
  }
}

template <typename T>
__global__ void __launch_bounds__(kT) maxpool_bwd_kernel(const T* __restrict__ dy,
                                                         const unsigned char* __restrict__ am, T* __restrict__ dx,
                                                         int N, int H, int W, int C, int accumulate) {
  const int Ho = H / 2, Wo = W / 2, C8 = C / 8;
  const size_t total = (size_t)N * Ho * Wo * C8;
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < total; i += (size_t)gridDim.x * kT) {
    const int c8 = (int)(i % C8);
    size_t p = i / C8;
    const int wo = (int)(p % Wo); p /= Wo;
    const int ho = (int)(p % Ho);
    const int n = (int)(p / Ho);
    float g[8];
    load8(dy + i * 8, g);
    const uint2 pk = *reinterpret_cast<const uint2*>(am + i * 8);
    T* base = dx + (((size_t)n * H + 2 * ho) * W + 2 * wo) * C + c8 * 8;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float v[8];
      T* dst = base + ((size_t)(k >> 1) * W + (k & 1)) * C;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const unsigned code = ((e < 4 ? pk.x : pk.y) >> ((e & 3) * 8)) & 0xffu;
        v[e] = code == (unsigned)k ? g[e] : 0.f;
      }
      if (accumulate) {
        float o[8];
        load8(dst, o);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += o[e];
      }
      store8(dst, v);
    }
  }
}

template <typename T>
__global__ void __launch_bounds__(kT) gap_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int N, int HW,
                                                     int C) {
  const int C8 = C / 8;
  const size_t total = (size_t)N * C8;
  const size_t i = (size_t)blockIdx.x * kT + threadIdx.x;
  if (i >= total) return;
  const int c8 = (int)(i % C8);
  const size_t n = i / C8;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  // eight positions' loads in flight at a time; the additions keep the order p = 0, 1, 2, ...
  int p = 0;
  for (; p + 8 <= HW; p += 8) {
    float v[8][8];
#pragma unroll
    for (int k = 0; k < 8; ++k) load8(x + (n * HW + p + k) * C + c8 * 8, v[k]);
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[k][e];
  }
  for (; p < HW; ++p) {
    float v[8];
    load8(x + (n * HW + p) * C + c8 * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  const float inv = 1.f / (float)HW;
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] *= inv;
  store8(y + i * 8, acc);
}

template <typename T>
__global__ void __launch_bounds__(kT) gap_bwd_kernel(const T* __restrict__ dy, T* __restrict__ dx, int N, int HW,
                                                     int C, int accumulate) {
  const int C8 = C / 8;
  const size_t total = (size_t)N * HW * C8;
  const float inv = 1.f / (float)HW;
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < total; i += (size_t)gridDim.x * kT) {
    const int c8 = (int)(i % C8);
    const size_t n = i / ((size_t)C8 * HW);
    float g[8];
    load8(dy + n * C + c8 * 8, g);
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] *= inv;
    if (accumulate) {
      float o[8];
      load8(dx + i * 8, o);
#pragma unroll
      for (int e = 0; e < 8; ++e) g[e] += o[e];
    }
    store8(dx + i * 8, g);
  }
}

// mode 0: y = a + b; mode 1: y = a; mode 2: y += a      (scalar tail handled by the same loop)
template <typename T>
__global__ void __launch_bounds__(kT) ew_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ y,
                                                size_t n, int mode) {
  const size_t n8 = n / 8;
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n8; i += (size_t)gridDim.x * kT) {
    float u[8], v[8];
    load8(a + i * 8, u);
    if (mode == 0) load8(b + i * 8, v);
    if (mode == 2) load8(y + i * 8, v);
    if (mode != 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) u[e] += v[e];
    }
    store8(y + i * 8, u);
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 7)) {
    const size_t i = n8 * 8 + threadIdx.x;
    float u = Elem<T>::ld(a + i);
    if (mode == 0) u += Elem<T>::ld(b + i);
    if (mode == 2) u += Elem<T>::ld(y + i);
    Elem<T>::st(y + i, u);
  }
}

int validate_pool(const cnnk_pool_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->C <= 0) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (d->mode != CNNK_POOL_MAX2 && d->mode != CNNK_POOL_GAP) return CNNK_ERR_UNSUPPORTED;
  if (d->C % 8 != 0) return CNNK_ERR_UNSUPPORTED;
  if (d->mode == CNNK_POOL_MAX2 && ((d->H & 1) || (d->W & 1))) return CNNK_ERR_SHAPE;
  return CNNK_OK;
}
}  // namespace

extern "C" int cnnk_pool_fwd(const cnnk_pool_desc* d, const void* x, void* y, unsigned char* argmax, void* stream) {
  int rc = validate_pool(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !y || (d->mode == CNNK_POOL_MAX2 && !argmax)) return CNNK_ERR_NULL;
  hipStream_t st = (hipStream_t)stream;
  if (d->mode == CNNK_POOL_MAX2) {
    const size_t total = (size_t)d->N * (d->H / 2) * (d->W / 2) * (d->C / 8);
    if (d->dtype == CNNK_BF16)
      maxpool_fwd_kernel<bf16_t><<<ew_blocks(total), kT, 0, st>>>((const bf16_t*)x, (bf16_t*)y, argmax, d->N, d->H, d->W, d->C);
    else
      maxpool_fwd_kernel<float><<<ew_blocks(total), kT, 0, st>>>((const float*)x, (float*)y, argmax, d->N, d->H, d->W, d->C);
  } else {
    const size_t total = (size_t)d->N * (d->C / 8);
    const unsigned nb = (unsigned)((total + kT - 1) / kT);
    if (d->dtype == CNNK_BF16)
      gap_fwd_kernel<bf16_t><<<nb, kT, 0, st>>>((const bf16_t*)x, (bf16_t*)y, d->N, d->H * d->W, d->C);
    else
      gap_fwd_kernel<float><<<nb, kT, 0, st>>>((const float*)x, (float*)y, d->N, d->H * d->W, d->C);
  }
  return launch_status();
}

extern "C" int cnnk_pool_bwd(const cnnk_pool_desc* d, const void* dy, const unsigned char* argmax, void* dx,
                             int accumulate, void* stream) {
  int rc = validate_pool(d);
  if (rc != CNNK_OK) return rc;
  if (!dy || !dx || (d->mode == CNNK_POOL_MAX2 && !argmax)) return CNNK_ERR_NULL;
  hipStream_t st = (hipStream_t)stream;
  if (d->mode == CNNK_POOL_MAX2) {
    const size_t total = (size_t)d->N * (d->H / 2) * (d->W / 2) * (d->C / 8);
    if (d->dtype == CNNK_BF16)
      maxpool_bwd_kernel<bf16_t><<<ew_blocks(total), kT, 0, st>>>((const bf16_t*)dy, argmax, (bf16_t*)dx, d->N, d->H, d->W, d->C, accumulate);
    else
      maxpool_bwd_kernel<float><<<ew_blocks(total), kT, 0, st>>>((const float*)dy, argmax, (float*)dx, d->N, d->H, d->W, d->C, accumulate);
  } else {
    const size_t total = (size_t)d->N * d->H * d->W * (d->C / 8);
    if (d->dtype == CNNK_BF16)
      gap_bwd_kernel<bf16_t><<<ew_blocks(total), kT, 0, st>>>((const bf16_t*)dy, (bf16_t*)dx, d->N, d->H * d->W, d->C, accumulate);
    else
      gap_bwd_kernel<float><<<ew_blocks(total), kT, 0, st>>>((const float*)dy, (float*)dx, d->N, d->H * d->W, d->C, accumulate);
  }
  return launch_status();
}

static int launch_ew(size_t n, int dtype, const void* a, const void* b, void* y, int mode, hipStream_t st) {
  if (dtype != CNNK_F32 && dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (n == 0) return CNNK_OK;
  if (dtype == CNNK_BF16)
    ew_kernel<bf16_t><<<ew_blocks(n / 8 + 1), kT, 0, st>>>((const bf16_t*)a, (const bf16_t*)b, (bf16_t*)y, n, mode);
  else
    ew_kernel<float><<<ew_blocks(n / 8 + 1), kT, 0, st>>>((const float*)a, (const float*)b, (float*)y, n, mode);
  return launch_status();
}

extern "C" int cnnk_add(size_t n, int dtype, const void* a, const void* b, void* y, void* stream) {
  if (n && (!a || !b || !y)) return CNNK_ERR_NULL;
  return launch_ew(n, dtype, a, b, y, 0, (hipStream_t)stream);
}

extern "C" int cnnk_grad_route(size_t n, int dtype, const void* src, void* dst, int accumulate, void* stream) {
  if (n && (!src || !dst)) return CNNK_ERR_NULL;
  return launch_ew(n, dtype, src, nullptr, dst, accumulate ? 2 : 1, (hipStream_t)stream);
}
