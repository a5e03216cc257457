// SGD with momentum: g' = g + wd*w; v <- mu*v + g'; w <- w - lr*v; optional bf16 copy of w.
// Bandwidth-bound (20 B per parameter, 22 B with the bf16 copy).  The multi-tensor variant
// updates up to kSgdMaxTensors parameter tensors per launch: the table travels in the kernel
// arguments, so nothing is staged through device memory.
#include "common.h"
#include "sgd.h"

namespace {
constexpr int kT = 256;
constexpr int kVec = 4;                    // float4 accesses
constexpr int kIters = 4;                  // float4 per thread, all loads issued before the arithmetic
constexpr int kPerBlock = kT * kVec * kIters;

__device__ __forceinline__ float sgd_one(float wi, float vi, float gi, float lr, float mu, float wd, float* vn) {
  const float gp = fmaf(wd, wi, gi);
  *vn = fmaf(mu, vi, gp);
  return fmaf(-lr, *vn, wi);
}

// Elements [begin, end) of one tensor; begin is a multiple of kPerBlock, the tensors are 16-byte
// aligned (checked on the host, else kVec-wide accesses are not used).
__device__ __forceinline__ void sgd_range(float* __restrict__ w, float* __restrict__ v, const float* __restrict__ g,
                                          bf16_t* __restrict__ wlp, size_t begin, size_t end, float lr, float mu,
                                          float wd, bool vec) {
  if (vec && begin + kPerBlock <= end) {
    float4 wv[kIters], vv[kIters], gv[kIters];
#pragma unroll
    for (int k = 0; k < kIters; ++k) {
      const size_t i = begin + ((size_t)k * kT + threadIdx.x) * kVec;
      wv[k] = *reinterpret_cast<const float4*>(w + i);
      vv[k] = *reinterpret_cast<const float4*>(v + i);
      gv[k] = *reinterpret_cast<const float4*>(g + i);
    }
#pragma unroll
    for (int k = 0; k < kIters; ++k) {
      const size_t i = begin + ((size_t)k * kT + threadIdx.x) * kVec;
      float4 vn, wn;
      wn.x = sgd_one(wv[k].x, vv[k].x, gv[k].x, lr, mu, wd, &vn.x);
      wn.y = sgd_one(wv[k].y, vv[k].y, gv[k].y, lr, mu, wd, &vn.y);
      wn.z = sgd_one(wv[k].z, vv[k].z, gv[k].z, lr, mu, wd, &vn.z);
      wn.w = sgd_one(wv[k].w, vv[k].w, gv[k].w, lr, mu, wd, &vn.w);
      *reinterpret_cast<float4*>(v + i) = vn;
      *reinterpret_cast<float4*>(w + i) = wn;
      if (wlp) {
        uint2 p;
        p.x = (unsigned)f32_to_bf16(wn.x) | ((unsigned)f32_to_bf16(wn.y) << 16);
        p.y = (unsigned)f32_to_bf16(wn.z) | ((unsigned)f32_to_bf16(wn.w) << 16);
        *reinterpret_cast<uint2*>(wlp + i) = p;
      }
    }
    return;
  }
  for (size_t i = begin + threadIdx.x; i < end; i += kT) {
    float vn;
    const float wn = sgd_one(w[i], v[i], g[i], lr, mu, wd, &vn);
    v[i] = vn;
    w[i] = wn;
    if (wlp) wlp[i] = f32_to_bf16(wn);
  }
}

__device__ __forceinline__ bool sgd_aligned(const float* w, const float* v, const float* g, const bf16_t* wlp) {
  return ((((size_t)w | (size_t)v | (size_t)g) & 15) == 0) && (((size_t)wlp & 7) == 0);
}

__global__ void __launch_bounds__(kT) sgd_kernel(float* w, float* v, const float* g, bf16_t* wlp, size_t n, float lr,
                                                 float mu, float wd) {
  const size_t begin = (size_t)blockIdx.x * kPerBlock;
  const size_t end = begin + kPerBlock < n ? begin + kPerBlock : n;
  sgd_range(w, v, g, wlp, begin, end, lr, mu, wd, sgd_aligned(w, v, g, wlp));
}

__global__ void __launch_bounds__(kT) sgd_multi_kernel(SgdTable t, float lr, float mu, float wd) {
  int k = 0;
  while (k + 1 < t.count && (int)blockIdx.x >= t.block_begin[k + 1]) ++k;
  const size_t begin = (size_t)(blockIdx.x - t.block_begin[k]) * kPerBlock;
  const size_t n = t.n[k];
  const size_t end = begin + kPerBlock < n ? begin + kPerBlock : n;
  bf16_t* wlp = reinterpret_cast<bf16_t*>(t.wlp[k]);
  sgd_range(t.w[k], t.v[k], t.g[k], wlp, begin, end, lr, mu, wd, sgd_aligned(t.w[k], t.v[k], t.g[k], wlp));
}
}  // namespace

int sgd_multi(SgdTable& t, float lr, float mu, float wd, hipStream_t st) {
  int blocks = 0;
  for (int k = 0; k < t.count; ++k) {
    t.block_begin[k] = blocks;
    blocks += (int)((t.n[k] + kPerBlock - 1) / kPerBlock);
  }
  t.block_begin[t.count] = blocks;
  if (blocks == 0) return CNNK_OK;
  sgd_multi_kernel<<<blocks, kT, 0, st>>>(t, lr, mu, wd);
  return launch_status();
}

extern "C" int cnnk_sgd_momentum(size_t n, float* w, float* v, const float* g, void* w_bf16, float lr, float momentum,
                                 float weight_decay, void* stream) {
  if (n == 0) return CNNK_OK;
  if (!w || !v || !g) return CNNK_ERR_NULL;
  if (n > ((size_t)1 << 40)) return CNNK_ERR_SHAPE;
  const unsigned blocks = (unsigned)((n + kPerBlock - 1) / kPerBlock);
  sgd_kernel<<<blocks, kT, 0, (hipStream_t)stream>>>(w, v, g, (bf16_t*)w_bf16, n, lr, momentum, weight_decay);
  return launch_status();
}
