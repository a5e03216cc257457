// Multi-head self-attention of the Vision Transformer step (Section IV-A's second model), forward
// and backward, for sequences that fit one workgroup's LDS (a ViT-B/16 image is 197 tokens).
//
// These are the general kernels (any storage type, head sizes 16 / 32 / 64); bf16 storage with head
// size 64 runs on the matrix cores instead (vit_attention_mfma.hip) unless cnnk_tune key 10 is -1.
// fp32 arithmetic on the vector ALUs, whatever the storage type: one workgroup per (image, head)
// holds the head's keys and values (or, for the key / value gradients, its queries and output
// gradients) in LDS as floats; a thread owns one query (or one key) and walks the other index, every
// LDS read being a broadcast of one row to all lanes.  The probabilities are never stored: the
// forward pass keeps log-sum-exp per query and the backward pass recomputes exp(s - lse).
#include "common.h"
#include "../../include/cnnk_vit.h"

// the matrix-core kernels (vit_attention_mfma.hip): bf16, head size 64, at most 256 tokens
bool attn_mfma_supported(const cnnk_attn_desc* d);
int attn_mfma_fwd(const cnnk_attn_desc* d, const void* qkv, void* o, float* lse, hipStream_t st);
int attn_mfma_bwd(const cnnk_attn_desc* d, const void* qkv, const void* o, const void* d_o, const float* lse, void* dqkv,
                  hipStream_t st);
extern int g_cnnk_tune[16];

namespace {
constexpr int kT = 256;

template <int DH>
__device__ __forceinline__ float dot_lds(const float* q, const float* row) {
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
  for (int k = 0; k < DH; k += 4) {
    const float4 r = *reinterpret_cast<const float4*>(row + k);
    s0 += q[k] * r.x; s1 += q[k + 1] * r.y; s2 += q[k + 2] * r.z; s3 += q[k + 3] * r.w;
  }
  return (s0 + s1) + (s2 + s3);
}
template <int DH>
__device__ __forceinline__ void axpy_lds(float* acc, float a, const float* row) {
#pragma unroll
  for (int k = 0; k < DH; k += 4) {
    const float4 r = *reinterpret_cast<const float4*>(row + k);
    acc[k] += a * r.x; acc[k + 1] += a * r.y; acc[k + 2] += a * r.z; acc[k + 3] += a * r.w;
  }
}
template <typename T, int DH>
__device__ __forceinline__ void load_row(const T* p, float* f, float scale) {
#pragma unroll
  for (int k = 0; k < DH; k += 8) {
    load8(p + k, f + k);
#pragma unroll
    for (int j = 0; j < 8; ++j) f[k + j] *= scale;
  }
}
template <typename T, int DH>
__device__ __forceinline__ void store_row(T* p, const float* f) {
#pragma unroll
  for (int k = 0; k < DH; k += 8) store8(p + k, f + k);
}
// rows [0, T) of one head's slice (column offset col0 of a [T][ld] matrix) into LDS as floats
template <typename T, int DH>
__device__ __forceinline__ void stage_rows(const T* base, size_t ld, int col0, int Tn, float* dst, float scale) {
  for (int i = threadIdx.x; i < Tn * (DH / 8); i += kT) {
    const int t = i / (DH / 8), j = (i % (DH / 8)) * 8;
    float v[8];
    load8(base + (size_t)t * ld + col0 + j, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) dst[t * DH + j + k] = v[k] * scale;
  }
}

template <typename T, int DH>
__global__ void __launch_bounds__(kT) attn_fwd_kernel(const T* __restrict__ qkv, T* __restrict__ o, float* __restrict__ lse,
                                                      int Tn, int heads) {
  extern __shared__ float sm[];
  float* Ks = sm;
  float* Vs = sm + (size_t)Tn * DH;
  const int b = blockIdx.x / heads, h = blockIdx.x % heads;
  const int d = heads * DH;
  const T* base = qkv + (size_t)b * Tn * 3 * d;
  stage_rows<T, DH>(base, 3 * (size_t)d, d + h * DH, Tn, Ks, 1.0f);
  stage_rows<T, DH>(base, 3 * (size_t)d, 2 * d + h * DH, Tn, Vs, 1.0f);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)DH);
  for (int t = threadIdx.x; t < Tn; t += kT) {
    float q[DH], acc[DH];
    load_row<T, DH>(base + (size_t)t * 3 * d + h * DH, q, scale);
    float m = -INFINITY, l = 0.f;
    for (int j = 0; j < Tn; ++j) {
      const float s = dot_lds<DH>(q, Ks + j * DH);
      const float mn = fmaxf(m, s);
      l = l * __expf(m - mn) + __expf(s - mn);
      m = mn;
    }
    const float L = m + __logf(l);
#pragma unroll
    for (int k = 0; k < DH; ++k) acc[k] = 0.f;
    for (int j = 0; j < Tn; ++j) {
      const float p = __expf(dot_lds<DH>(q, Ks + j * DH) - L);
      axpy_lds<DH>(acc, p, Vs + j * DH);
    }
    store_row<T, DH>(o + ((size_t)b * Tn + t) * d + h * DH, acc);
    lse[((size_t)b * heads + h) * Tn + t] = L;
  }
}

// dq: a thread owns a query; keys and values in LDS.
template <typename T, int DH>
__global__ void __launch_bounds__(kT) attn_bwd_q_kernel(const T* __restrict__ qkv, const T* __restrict__ o,
                                                        const T* __restrict__ d_o, const float* __restrict__ lse,
                                                        T* __restrict__ dqkv, int Tn, int heads) {
  extern __shared__ float sm[];
  float* Ks = sm;
  float* Vs = sm + (size_t)Tn * DH;
  const int b = blockIdx.x / heads, h = blockIdx.x % heads;
  const int d = heads * DH;
  const T* base = qkv + (size_t)b * Tn * 3 * d;
  stage_rows<T, DH>(base, 3 * (size_t)d, d + h * DH, Tn, Ks, 1.0f);
  stage_rows<T, DH>(base, 3 * (size_t)d, 2 * d + h * DH, Tn, Vs, 1.0f);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)DH);
  for (int t = threadIdx.x; t < Tn; t += kT) {
    float q[DH], g[DH], acc[DH];
    load_row<T, DH>(base + (size_t)t * 3 * d + h * DH, q, scale);
    load_row<T, DH>(d_o + ((size_t)b * Tn + t) * d + h * DH, g, 1.0f);
    float D = 0.f;
    {
      float ov[DH];
      load_row<T, DH>(o + ((size_t)b * Tn + t) * d + h * DH, ov, 1.0f);
#pragma unroll
      for (int k = 0; k < DH; ++k) D += g[k] * ov[k];
    }
    const float L = lse[((size_t)b * heads + h) * Tn + t];
#pragma unroll
    for (int k = 0; k < DH; ++k) acc[k] = 0.f;
    for (int j = 0; j < Tn; ++j) {
      const float p = __expf(dot_lds<DH>(q, Ks + j * DH) - L);
      const float ds = p * (dot_lds<DH>(g, Vs + j * DH) - D);
      axpy_lds<DH>(acc, ds, Ks + j * DH);
    }
#pragma unroll
    for (int k = 0; k < DH; ++k) acc[k] *= scale;
    store_row<T, DH>(dqkv + ((size_t)b * Tn + t) * 3 * d + h * DH, acc);
  }
}

// dk, dv: a thread owns a key; the (scaled) queries, the output gradients, lse and D = do . o per
// query in LDS.  Two walks over the queries so that at most three rows live in registers.
template <typename T, int DH>
__global__ void __launch_bounds__(kT) attn_bwd_kv_kernel(const T* __restrict__ qkv, const T* __restrict__ o,
                                                         const T* __restrict__ d_o, const float* __restrict__ lse,
                                                         T* __restrict__ dqkv, int Tn, int heads) {
  extern __shared__ float sm[];
  float* Qs = sm;
  float* Gs = sm + (size_t)Tn * DH;
  float* Ls = Gs + (size_t)Tn * DH;
  float* Ds = Ls + Tn;
  const int b = blockIdx.x / heads, h = blockIdx.x % heads;
  const int d = heads * DH;
  const T* base = qkv + (size_t)b * Tn * 3 * d;
  const float scale = 1.0f / sqrtf((float)DH);
  stage_rows<T, DH>(base, 3 * (size_t)d, h * DH, Tn, Qs, scale);
  stage_rows<T, DH>(d_o + (size_t)b * Tn * d, (size_t)d, h * DH, Tn, Gs, 1.0f);
  for (int t = threadIdx.x; t < Tn; t += kT) {
    float g[DH], ov[DH];
    load_row<T, DH>(d_o + ((size_t)b * Tn + t) * d + h * DH, g, 1.0f);
    load_row<T, DH>(o + ((size_t)b * Tn + t) * d + h * DH, ov, 1.0f);
    float D = 0.f;
#pragma unroll
    for (int k = 0; k < DH; ++k) D += g[k] * ov[k];
    Ds[t] = D;
    Ls[t] = lse[((size_t)b * heads + h) * Tn + t];
  }
  __syncthreads();
  for (int j = threadIdx.x; j < Tn; j += kT) {
    float kr[DH], acc[DH];
    load_row<T, DH>(base + (size_t)j * 3 * d + d + h * DH, kr, 1.0f);
#pragma unroll
    for (int k = 0; k < DH; ++k) acc[k] = 0.f;
    for (int t = 0; t < Tn; ++t) {                       // dv_j = sum_t p_tj do_t
      const float p = __expf(dot_lds<DH>(kr, Qs + t * DH) - Ls[t]);
      axpy_lds<DH>(acc, p, Gs + t * DH);
    }
    store_row<T, DH>(dqkv + ((size_t)b * Tn + j) * 3 * d + 2 * d + h * DH, acc);
    float vr[DH];
    load_row<T, DH>(base + (size_t)j * 3 * d + 2 * d + h * DH, vr, 1.0f);
#pragma unroll
    for (int k = 0; k < DH; ++k) acc[k] = 0.f;
    for (int t = 0; t < Tn; ++t) {                       // dk_j = sum_t ds_tj (q_t / sqrt(dh))
      const float p = __expf(dot_lds<DH>(kr, Qs + t * DH) - Ls[t]);
      const float ds = p * (dot_lds<DH>(vr, Gs + t * DH) - Ds[t]);
      axpy_lds<DH>(acc, ds, Qs + t * DH);
    }
    store_row<T, DH>(dqkv + ((size_t)b * Tn + j) * 3 * d + d + h * DH, acc);
  }
}

int check_attn(const cnnk_attn_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->B <= 0 || d->T <= 0 || d->heads <= 0 || d->dh <= 0) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if ((d->dh != 16 && d->dh != 32 && d->dh != 64) || (long long)d->T * d->dh > 16384) return CNNK_ERR_UNSUPPORTED;
  if ((double)d->B * d->T * 3 * d->heads * d->dh > 2147483647.0) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

template <typename K>
void raise_lds(K kernel, size_t bytes) {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <typename T, int DH>
void launch_fwd(const cnnk_attn_desc* d, const void* qkv, void* o, float* lse, hipStream_t st) {
  const size_t lds = (size_t)2 * d->T * DH * sizeof(float);
  raise_lds(attn_fwd_kernel<T, DH>, lds);
  attn_fwd_kernel<T, DH><<<d->B * d->heads, kT, lds, st>>>((const T*)qkv, (T*)o, lse, d->T, d->heads);
}
template <typename T, int DH>
void launch_bwd(const cnnk_attn_desc* d, const void* qkv, const void* o, const void* d_o, const float* lse, void* dqkv,
                hipStream_t st) {
  const size_t lds_q = (size_t)2 * d->T * DH * sizeof(float);
  const size_t lds_kv = lds_q + (size_t)2 * d->T * sizeof(float);
  raise_lds(attn_bwd_q_kernel<T, DH>, lds_q);
  raise_lds(attn_bwd_kv_kernel<T, DH>, lds_kv);
  attn_bwd_q_kernel<T, DH><<<d->B * d->heads, kT, lds_q, st>>>((const T*)qkv, (const T*)o, (const T*)d_o, lse, (T*)dqkv,
                                                                d->T, d->heads);
  attn_bwd_kv_kernel<T, DH><<<d->B * d->heads, kT, lds_kv, st>>>((const T*)qkv, (const T*)o, (const T*)d_o, lse, (T*)dqkv,
                                                                  d->T, d->heads);
}
inline bool aligned16(const void* p) { return (((size_t)p) & 15) == 0; }
}  // namespace

extern "C" int cnnk_attention_fwd(const cnnk_attn_desc* d, const void* qkv, void* o, float* lse, void* stream) {
  const int rc = check_attn(d);
  if (rc != CNNK_OK) return rc;
  if (!qkv || !o || !lse) return CNNK_ERR_NULL;
  if (!aligned16(qkv) || !aligned16(o)) return CNNK_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  if (attn_mfma_supported(d) && g_cnnk_tune[10] >= 0) return attn_mfma_fwd(d, qkv, o, lse, st);
  const bool bf = d->dtype == CNNK_BF16;
  switch (d->dh) {
    case 16: bf ? launch_fwd<bf16_t, 16>(d, qkv, o, lse, st) : launch_fwd<float, 16>(d, qkv, o, lse, st); break;
    case 32: bf ? launch_fwd<bf16_t, 32>(d, qkv, o, lse, st) : launch_fwd<float, 32>(d, qkv, o, lse, st); break;
    default: bf ? launch_fwd<bf16_t, 64>(d, qkv, o, lse, st) : launch_fwd<float, 64>(d, qkv, o, lse, st); break;
  }
  return launch_status();
}

extern "C" int cnnk_attention_bwd(const cnnk_attn_desc* d, const void* qkv, const void* o, const void* d_o,
                                  const float* lse, void* dqkv, void* stream) {
  const int rc = check_attn(d);
  if (rc != CNNK_OK) return rc;
  if (!qkv || !o || !d_o || !lse || !dqkv) return CNNK_ERR_NULL;
  if (!aligned16(qkv) || !aligned16(o) || !aligned16(d_o) || !aligned16(dqkv)) return CNNK_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  if (attn_mfma_supported(d) && g_cnnk_tune[10] >= 0) return attn_mfma_bwd(d, qkv, o, d_o, lse, dqkv, st);
  const bool bf = d->dtype == CNNK_BF16;
  switch (d->dh) {
    case 16: bf ? launch_bwd<bf16_t, 16>(d, qkv, o, d_o, lse, dqkv, st) : launch_bwd<float, 16>(d, qkv, o, d_o, lse, dqkv, st); break;
    case 32: bf ? launch_bwd<bf16_t, 32>(d, qkv, o, d_o, lse, dqkv, st) : launch_bwd<float, 32>(d, qkv, o, d_o, lse, dqkv, st); break;
    default: bf ? launch_bwd<bf16_t, 64>(d, qkv, o, d_o, lse, dqkv, st) : launch_bwd<float, 64>(d, qkv, o, d_o, lse, dqkv, st); break;
  }
  return launch_status();
}
