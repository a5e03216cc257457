// Convolutions with fewer than 8 input channels (the 3-channel stem) in bf16 mode: the input and
// the weights are zero-padded to 8 channels in the workspace so that a pixel's channels form one
// 16-byte vector, then the bf16 MFMA kernels run on the padded problem.  The layer is bound by
// the 64-channel side (output write / dy read), so the padded reduction costs nothing.
#include "common.h"
#include "conv.h"

namespace {

// dst[m][0..8) = src[m][0..C) followed by zeros, for two tensors in one launch (the rows of the
// second one follow the rows of the first in the thread index; rows1 may be 0)
__global__ void __launch_bounds__(256) pad_channels_kernel(const bf16_t* __restrict__ src0, bf16_t* __restrict__ dst0,
                                                           size_t rows0, const bf16_t* __restrict__ src1,
                                                           bf16_t* __restrict__ dst1, size_t rows1, int C) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < rows0 + rows1; i += (size_t)gridDim.x * 256) {
    const bool first = i < rows0;
    const bf16_t* src = first ? src0 : src1;
    bf16_t* dst = first ? dst0 : dst1;
    const size_t m = first ? i : i - rows0;
    unsigned short v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = c < C ? src[m * C + c] : (unsigned short)0;
    uint4 o;
    o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16); o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
    *reinterpret_cast<uint4*>(dst + m * 8) = o;
  }
}

// dw[row][0..C) = sum over P partials of part[p][row][0..C) (rows of 8 padded channels; P = 1: a
// plain copy out of the padded layout).  16 thread groups share the partials of an element, their
// sums are added in group order (deterministic).
__global__ void __launch_bounds__(256) reduce_unpad_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                           int rows, int C, int P) {
  __shared__ float red[16][16];
  const int e = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int i = blockIdx.x * 16 + e;            // output element
  const size_t n8 = (size_t)rows * 8;
  float a = 0.f;
  if (i < rows * C) {
    const size_t src = (size_t)(i / C) * 8 + i % C;
    // up to eight partials per round, all loads issued before the first add (a partial past the end
    // is not loaded and adds zero)
    const int rounds = (P + 15) / 16;
    for (int k0 = 0; k0 < rounds; k0 += 8) {
      float v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int p = grp + (k0 + k) * 16;
        v[k] = 0.f;
        if (p < P) v[k] = part[(size_t)p * n8 + src];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k0 + k < rounds) a += v[k];
    }
  }
  red[grp][e] = a;
  __syncthreads();
  if (grp == 0 && i < rows * C) {
    float sum = red[0][e];
#pragma unroll
    for (int k = 1; k < 16; ++k) sum += red[k][e];
    dw[i] = sum;
  }
}

ConvGeom padded(const ConvGeom& g) {
  ConvGeom p = g;
  p.Cin = 8;
  return p;
}

inline unsigned pad_blocks(size_t rows) {
  size_t b = (rows + 255) / 256;
  return (unsigned)(b > 4096 ? 4096 : (b < 1 ? 1 : b));
}

size_t x8_bytes(const ConvGeom& g) { return align_up((size_t)g.N * g.H * g.W * 8 * sizeof(bf16_t), 256); }
size_t w8_bytes(const ConvGeom& g) { return align_up((size_t)g.Cout * g.R * g.S * 8 * sizeof(bf16_t), 256); }
size_t dw8_bytes(const ConvGeom& g) { return align_up((size_t)g.Cout * g.R * g.S * 8 * sizeof(float), 256); }

}  // namespace

thread_local X8Cache* t_cnnk_x8_cache = nullptr;
size_t conv_pad_x8_bytes(const ConvGeom& g) { return x8_bytes(g); }

bool conv_pad_supported(const ConvGeom& g) {
  return g.Cin < 8 && conv_mfma_supported(padded(g), CNNK_PASS_FWD);
}

size_t conv_pad_ws(const ConvGeom& g, int pass, bool want_stats) {
  const ConvGeom p = padded(g);
  if (pass == CNNK_PASS_FWD) return x8_bytes(g) + w8_bytes(g) + conv_mfma_ws(p, pass, want_stats);
  if (pass == CNNK_PASS_WGRAD) return x8_bytes(g) + dw8_bytes(g) + conv_mfma_ws(p, pass, false);
  return 0;
}

int conv_pad_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* ch_sum, float* ch_sumsq,
                 void* ws, hipStream_t st) {
  char* base = static_cast<char*>(ws);
  X8Cache* cache = t_cnnk_x8_cache;
  bf16_t* x8 = cache ? cache->buf : reinterpret_cast<bf16_t*>(base);
  bf16_t* w8 = reinterpret_cast<bf16_t*>(base + x8_bytes(g));
  void* rest = base + x8_bytes(g) + w8_bytes(g);
  const size_t px = (size_t)g.N * g.H * g.W, wr = (size_t)g.Cout * g.R * g.S;
  if (cache) cache->valid = true;
  pad_channels_kernel<<<pad_blocks(px + wr), 256, 0, st>>>(x, x8, px, w, w8, wr, g.Cin);
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  return conv_mfma_fwd(padded(g), x8, w8, y, ch_sum, ch_sumsq, rest, st);
}

int conv_pad_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st) {
  char* base = static_cast<char*>(ws);
  const X8Cache* cache = (t_cnnk_x8_cache && t_cnnk_x8_cache->valid) ? t_cnnk_x8_cache : nullptr;
  bf16_t* x8 = cache ? cache->buf : reinterpret_cast<bf16_t*>(base);
  float* dw8 = reinterpret_cast<float*>(base + x8_bytes(g));
  void* rest = base + x8_bytes(g) + dw8_bytes(g);
  const size_t px = (size_t)g.N * g.H * g.W;
  if (!cache) {
    pad_channels_kernel<<<pad_blocks(px), 256, 0, st>>>(x, x8, px, nullptr, nullptr, 0, g.Cin);
    if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  }
  // the padded problem's partial gradients, summed straight into the unpadded layout
  const float* part = nullptr;
  int P = 0;
  int rc = conv_mfma_wgrad_partials(padded(g), x8, dy, dw8, rest, &part, &P, st);
  if (rc != CNNK_OK) return rc;
  const int rows = g.Cout * g.R * g.S;
  reduce_unpad_kernel<<<(rows * g.Cin + 15) / 16, 256, 0, st>>>(part, dw, rows, g.Cin, P);
  return launch_status();
}
