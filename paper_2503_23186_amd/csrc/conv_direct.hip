// Direct (non-MFMA) convolution kernels: the fp32 mode, and bf16 shapes the MFMA engine does
// not take (channel counts that are not multiples of 8, e.g. the 3-channel stem).
// One thread per output element, fp32 accumulation in a fixed order.
#include "common.h"
#include "conv.h"

namespace {

template <typename T>
__global__ void __launch_bounds__(256) direct_fwd_kernel(ConvGeom g, const T* __restrict__ x,
                                                         const T* __restrict__ w, T* __restrict__ y) {
  const size_t total = (size_t)g.N * g.Ho * g.Wo * g.Cout;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int k = (int)(idx % g.Cout);
  size_t m = idx / g.Cout;
  const int wo = (int)(m % g.Wo); m /= g.Wo;
  const int ho = (int)(m % g.Ho);
  const int n = (int)(m / g.Ho);
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int hi = ho * g.stride + r - g.pad;
    if (hi < 0 || hi >= g.H) continue;
    for (int s = 0; s < g.S; ++s) {
      const int wi = wo * g.stride + s - g.pad;
      if (wi < 0 || wi >= g.W) continue;
      const T* xp = x + (((size_t)n * g.H + hi) * g.W + wi) * g.Cin;
      const T* wp = w + (((size_t)k * g.R + r) * g.S + s) * g.Cin;
      for (int c = 0; c < g.Cin; ++c) acc = fmaf(Elem<T>::ld(xp + c), Elem<T>::ld(wp + c), acc);
    }
  }
  Elem<T>::st(y + idx, acc);
}

template <typename T>
__global__ void __launch_bounds__(256) direct_dgrad_kernel(ConvGeom g, const T* __restrict__ dy,
                                                           const T* __restrict__ w, T* __restrict__ dx,
                                                           int accumulate) {
  const size_t total = (size_t)g.N * g.H * g.W * g.Cin;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % g.Cin);
  size_t m = idx / g.Cin;
  const int wi = (int)(m % g.W); m /= g.W;
  const int hi = (int)(m % g.H);
  const int n = (int)(m / g.H);
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int th = hi + g.pad - r;
    if (th < 0 || th % g.stride != 0) continue;
    const int ho = th / g.stride;
    if (ho >= g.Ho) continue;
    for (int s = 0; s < g.S; ++s) {
      const int tw = wi + g.pad - s;
      if (tw < 0 || tw % g.stride != 0) continue;
      const int wo = tw / g.stride;
      if (wo >= g.Wo) continue;
      const T* dyp = dy + (((size_t)n * g.Ho + ho) * g.Wo + wo) * g.Cout;
      const T* wp = w + ((size_t)r * g.S + s) * g.Cin + c;
      const size_t wk = (size_t)g.R * g.S * g.Cin;
      for (int k = 0; k < g.Cout; ++k) acc = fmaf(Elem<T>::ld(dyp + k), Elem<T>::ld(wp + k * wk), acc);
    }
  }
  if (accumulate) acc += Elem<T>::ld(dx + idx);
  Elem<T>::st(dx + idx, acc);
}

// Partial weight gradient over the output positions [p*chunk, (p+1)*chunk) into part[p][i].
template <typename T>
__global__ void __launch_bounds__(256) direct_wgrad_kernel(ConvGeom g, const T* __restrict__ x,
                                                           const T* __restrict__ dy,
                                                           float* __restrict__ part, int chunk) {
  const int nw = g.Cout * g.R * g.S * g.Cin;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= nw) return;
  const int c = i % g.Cin;
  int t = i / g.Cin;
  const int s = t % g.S; t /= g.S;
  const int r = t % g.R;
  const int k = t / g.R;
  const long M = (long)g.N * g.Ho * g.Wo;
  const long m0 = (long)blockIdx.y * chunk;
  const long m1 = (m0 + chunk < M) ? m0 + chunk : M;
  float acc = 0.f;
  for (long m = m0; m < m1; ++m) {
    const int wo = (int)(m % g.Wo);
    const long q = m / g.Wo;
    const int ho = (int)(q % g.Ho);
    const int n = (int)(q / g.Ho);
    const int hi = ho * g.stride + r - g.pad;
    const int wi = wo * g.stride + s - g.pad;
    if (hi < 0 || hi >= g.H || wi < 0 || wi >= g.W) continue;
    acc = fmaf(Elem<T>::ld(dy + (size_t)m * g.Cout + k),
               Elem<T>::ld(x + (((size_t)n * g.H + hi) * g.W + wi) * g.Cin + c), acc);
  }
  part[(size_t)blockIdx.y * nw + i] = acc;
}

// out[i] = sum_p part[p][i], deterministic.  GROUPS thread groups share the P partials of a float4 column (group g takes p = g, g+GROUPS, ...);
// their sums are combined through LDS in group order.  More groups = more, shorter-lived threads:
// 16 for many partials (a 64x576 gradient split 108 ways is 16 MB to read), 4 otherwise.
struct SgdArgs {
  float* w;
  float* v;
  bf16_t* wlp;
  float lr, mu, wd;
};

__device__ __forceinline__ float sgd_apply(float wi, float vi, float gi, const SgdArgs& sg, float* vn) {
  const float gp = fmaf(sg.wd, wi, gi);
  *vn = fmaf(sg.mu, vi, gp);
  return fmaf(-sg.lr, *vn, wi);
}

template <int GROUPS, bool SGD>
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float* __restrict__ part,
                                                              float* __restrict__ out, int n, int P, SgdArgs sg) {
  constexpr int COLS = 256 / GROUPS;
  __shared__ float4 red[GROUPS][COLS];
  const int col = threadIdx.x % COLS, grp = threadIdx.x / COLS;
  const int i4 = blockIdx.x * COLS + col;   // float4 column
  const int n4 = n >> 2;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  // weight and momentum of the fused update are fetched under the partial sums
  float4 wv = make_float4(0.f, 0.f, 0.f, 0.f), vv = wv;
  if (SGD && grp == 0 && i4 < n4) {
    wv = *reinterpret_cast<const float4*>(sg.w + (size_t)i4 * 4);
    vv = *reinterpret_cast<const float4*>(sg.v + (size_t)i4 * 4);
  }
  if (i4 < n4) {
    // up to eight partials per round, all loads issued before the first add: the sum is a chain of
    // memory latencies otherwise (a partial past the end is not loaded and adds zero).  Same order
    // of additions as a plain loop.
    const float* base = part + (size_t)i4 * 4;
    const int rounds = (P + GROUPS - 1) / GROUPS;
    for (int k0 = 0; k0 < rounds; k0 += 8) {
      float4 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int p = grp + (k0 + k) * GROUPS;
        v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p < P) v[k] = *reinterpret_cast<const float4*>(base + (size_t)p * n);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k0 + k < rounds) { acc.x += v[k].x; acc.y += v[k].y; acc.z += v[k].z; acc.w += v[k].w; }
    }
  }
  red[grp][col] = acc;
  __syncthreads();
  if (grp == 0 && i4 < n4) {
    float4 s = red[0][col];
#pragma unroll
    for (int k = 1; k < GROUPS; ++k) { s.x += red[k][col].x; s.y += red[k][col].y; s.z += red[k][col].z; s.w += red[k][col].w; }
    *reinterpret_cast<float4*>(out + (size_t)i4 * 4) = s;
    if (SGD) {   // the parameter update on the gradient just summed (same arithmetic as the SGD kernel)
      const size_t i = (size_t)i4 * 4;
      float4 vn, wn;
      wn.x = sgd_apply(wv.x, vv.x, s.x, sg, &vn.x);
      wn.y = sgd_apply(wv.y, vv.y, s.y, sg, &vn.y);
      wn.z = sgd_apply(wv.z, vv.z, s.z, sg, &vn.z);
      wn.w = sgd_apply(wv.w, vv.w, s.w, sg, &vn.w);
      *reinterpret_cast<float4*>(sg.v + i) = vn;
      *reinterpret_cast<float4*>(sg.w + i) = wn;
      if (sg.wlp) {
        uint2 pk;
        pk.x = (unsigned)f32_to_bf16(wn.x) | ((unsigned)f32_to_bf16(wn.y) << 16);
        pk.y = (unsigned)f32_to_bf16(wn.z) | ((unsigned)f32_to_bf16(wn.w) << 16);
        *reinterpret_cast<uint2*>(sg.wlp + i) = pk;
      }
    }
  }
  // scalar tail (n not a multiple of 4)
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const int i = (n4 << 2) + threadIdx.x;
    float a = 0.f;
    for (int p = 0; p < P; ++p) a += part[(size_t)p * n + i];
    out[i] = a;
    if (SGD) {
      float vn;
      const float wn = sgd_apply(sg.w[i], sg.v[i], a, sg, &vn);
      sg.v[i] = vn;
      sg.w[i] = wn;
      if (sg.wlp) sg.wlp[i] = f32_to_bf16(wn);
    }
  }
}

void wgrad_split(const ConvGeom& g, int* chunk, int* P) {
  const long M = (long)g.N * g.Ho * g.Wo;
  const long nw = (long)g.Cout * g.R * g.S * g.Cin;
  const long out_blocks = (nw + 255) / 256;
  long want = (2048 + out_blocks - 1) / out_blocks;
  const long maxP = (M + 63) / 64;
  if (want > maxP) want = maxP;
  if (want > 4096) want = 4096;
  if (want < 1) want = 1;
  long ch = (M + want - 1) / want;
  *chunk = (int)ch;
  *P = (int)((M + ch - 1) / ch);
}

}  // namespace

size_t conv_direct_wgrad_ws(const ConvGeom& g) {
  int chunk, P;
  wgrad_split(g, &chunk, &P);
  return (size_t)P * g.Cout * g.R * g.S * g.Cin * sizeof(float);
}

int conv_direct_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, void* y, hipStream_t st) {
  const size_t total = (size_t)g.N * g.Ho * g.Wo * g.Cout;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dtype == CNNK_BF16)
    direct_fwd_kernel<bf16_t><<<blocks, 256, 0, st>>>(g, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y);
  else
    direct_fwd_kernel<float><<<blocks, 256, 0, st>>>(g, (const float*)x, (const float*)w, (float*)y);
  return launch_status();
}

int conv_direct_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                      hipStream_t st) {
  const size_t total = (size_t)g.N * g.H * g.W * g.Cin;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dtype == CNNK_BF16)
    direct_dgrad_kernel<bf16_t><<<blocks, 256, 0, st>>>(g, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, accumulate);
  else
    direct_dgrad_kernel<float><<<blocks, 256, 0, st>>>(g, (const float*)dy, (const float*)w, (float*)dx, accumulate);
  return launch_status();
}

int conv_direct_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                      hipStream_t st) {
  int chunk, P;
  wgrad_split(g, &chunk, &P);
  const int nw = g.Cout * g.R * g.S * g.Cin;
  dim3 grid((nw + 255) / 256, P);
  float* part = (float*)ws;
  if (dtype == CNNK_BF16)
    direct_wgrad_kernel<bf16_t><<<grid, 256, 0, st>>>(g, (const bf16_t*)x, (const bf16_t*)dy, part, chunk);
  else
    direct_wgrad_kernel<float><<<grid, 256, 0, st>>>(g, (const float*)x, (const float*)dy, part, chunk);
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  return reduce_partials(part, dw, nw, P, st);
}

thread_local SgdFuse* t_cnnk_sgd_fuse = nullptr;

int reduce_partials(const float* part, float* out, int n, int P, hipStream_t st) {
  const unsigned g16 = (unsigned)((n / 4 + 15) / 16 + 1), g4 = (unsigned)((n / 4 + 63) / 64 + 1);
  SgdFuse* f = t_cnnk_sgd_fuse;
  if (f && !f->done && ((((size_t)f->w | (size_t)f->v | (size_t)out) & 15) == 0) && (((size_t)f->wlp & 7) == 0)) {
    if (f->wait && hipStreamWaitEvent(st, f->wait, 0) != hipSuccess) return CNNK_ERR_HIP;
    const SgdArgs sg{f->w, f->v, static_cast<bf16_t*>(f->wlp), f->lr, f->mu, f->wd};
    if (P >= 32) reduce_partials_kernel<16, true><<<g16, 256, 0, st>>>(part, out, n, P, sg);
    else reduce_partials_kernel<4, true><<<g4, 256, 0, st>>>(part, out, n, P, sg);
    f->done = true;
    return launch_status();
  }
  const SgdArgs none{nullptr, nullptr, nullptr, 0.f, 0.f, 0.f};
  if (P >= 32) reduce_partials_kernel<16, false><<<g16, 256, 0, st>>>(part, out, n, P, none);
  else reduce_partials_kernel<4, false><<<g4, 256, 0, st>>>(part, out, n, P, none);
  return launch_status();
}
