// SGD with momentum: g' = g + wd*w; v <- mu*v + g'; w <- w - lr*v; optional bf16 copy of w.
// Bandwidth-bound (20 B per parameter, 22 B with the bf16 copy).  The multi-tensor variant
// updates up to kSgdMaxTensors parameter tensors per launch: the table travels in the kernel
// arguments, so nothing is staged through device memory.
#include "common.h"
#include "sgd.h"

namespace {
constexpr int kT = 256;
constexpr int kPerBlock = kT * 4;

__device__ __forceinline__ void sgd_range(float* __restrict__ w, float* __restrict__ v, const float* __restrict__ g,
                                          bf16_t* __restrict__ wlp, size_t begin, size_t end, float lr, float mu,
                                          float wd) {
  for (size_t i = begin + threadIdx.x; i < end; i += kT) {
    const float wi = w[i];
    const float gp = fmaf(wd, wi, g[i]);
    const float vn = fmaf(mu, v[i], gp);
    const float wn = fmaf(-lr, vn, wi);
    v[i] = vn;
    w[i] = wn;
    if (wlp) wlp[i] = f32_to_bf16(wn);
  }
}

__global__ void __launch_bounds__(kT) sgd_kernel(float* w, float* v, const float* g, bf16_t* wlp, size_t n, float lr,
                                                 float mu, float wd) {
  const size_t begin = (size_t)blockIdx.x * kPerBlock;
  const size_t end = begin + kPerBlock < n ? begin + kPerBlock : n;
  sgd_range(w, v, g, wlp, begin, end, lr, mu, wd);
}

__global__ void __launch_bounds__(kT) sgd_multi_kernel(SgdTable t, float lr, float mu, float wd) {
  int k = 0;
  while (k + 1 < t.count && (int)blockIdx.x >= t.block_begin[k + 1]) ++k;
  const size_t begin = (size_t)(blockIdx.x - t.block_begin[k]) * kPerBlock;
  const size_t n = t.n[k];
  const size_t end = begin + kPerBlock < n ? begin + kPerBlock : n;
  sgd_range(t.w[k], t.v[k], t.g[k], reinterpret_cast<bf16_t*>(t.wlp[k]), begin, end, lr, mu, wd);
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
