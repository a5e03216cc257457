// Convolution kernels for very thin inputs (R*S*Cin <= 28, e.g. the 3-channel 3x3 stem), bf16
// storage.  The reduction is too short for the matrix cores to pay (K = 27) and the layer is
// bound by writing / reading the 64-channel side, so these are plain fp32 FMA kernels with the
// weights (forward) or the activation tiles (weight gradient) staged in LDS.
#include "common.h"
#include "conv.h"

namespace {

constexpr int kT = 256;
constexpr int kMaxK = 28;

// Host-built decode of the reduction index j = (r*S + s)*Cin + c, and magic-number divisors for
// the pixel index (integer division has no hardware instruction).
struct StemTab {
  int r[kMaxK], s[kMaxK], c[kMaxK];
  FastDiv dWo, dHo;
};

// Forward: one thread per output position; couts in register chunks of 32; weights in LDS as
// fp32 [K][Cout], read as broadcast float4.
__global__ void __launch_bounds__(kT) stem_fwd_kernel(ConvGeom g, StemTab tab, const bf16_t* __restrict__ x,
                                                      const bf16_t* __restrict__ w, bf16_t* __restrict__ y) {
  extern __shared__ __align__(16) float wl[];  // [K][Cout]
  const int K = g.R * g.S * g.Cin;
  for (int i = threadIdx.x; i < K * g.Cout; i += kT) {
    const int k = i % g.Cout, j = i / g.Cout;
    wl[i] = bf16_to_f32(w[(size_t)k * K + j]);
  }
  __syncthreads();
  const long M = (long)g.N * g.Ho * g.Wo;
  const long m = (long)blockIdx.x * kT + threadIdx.x;
  if (m >= M) return;
  int q, wo, n, ho;
  tab.dWo.divmod((int)m, &q, &wo);
  tab.dHo.divmod(q, &n, &ho);
  float xv[kMaxK];
#pragma unroll
  for (int j = 0; j < kMaxK; ++j) {
    float v = 0.f;
    if (j < K) {
      const int c = tab.c[j];
      const int hi = ho * g.stride + tab.r[j] - g.pad, wi = wo * g.stride + tab.s[j] - g.pad;
      if ((unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W)
        v = bf16_to_f32(x[(((size_t)n * g.H + hi) * g.W + wi) * g.Cin + c]);
    }
    xv[j] = v;
  }
  bf16_t* yp = y + (size_t)m * g.Cout;
  for (int k0 = 0; k0 < g.Cout; k0 += 32) {
    float acc[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) acc[e] = 0.f;
    const int kn = min(32, g.Cout - k0);  // multiple of 8
#pragma unroll
    for (int j = 0; j < kMaxK; ++j) {
      if (j < K) {
        const float* wr = wl + j * g.Cout + k0;
#pragma unroll
        for (int e4 = 0; e4 < 8; ++e4) {
          if (e4 * 4 < kn) {
            const float4 w4 = *reinterpret_cast<const float4*>(wr + e4 * 4);
            acc[e4 * 4 + 0] = fmaf(xv[j], w4.x, acc[e4 * 4 + 0]);
            acc[e4 * 4 + 1] = fmaf(xv[j], w4.y, acc[e4 * 4 + 1]);
            acc[e4 * 4 + 2] = fmaf(xv[j], w4.z, acc[e4 * 4 + 2]);
            acc[e4 * 4 + 3] = fmaf(xv[j], w4.w, acc[e4 * 4 + 3]);
          }
        }
      }
    }
#pragma unroll
    for (int e8 = 0; e8 < 4; ++e8)
      if (e8 * 8 < kn) store8(yp + k0 + e8 * 8, acc + e8 * 8);
  }
}

// Weight gradient.  A workgroup owns kPixPerBlock output positions and 64 (or fewer) output
// channels, walks them in sub-chunks of 128 positions staged in LDS (dy as bf16 [128][64], the
// K-long input patches as fp32 [128][32]); a thread accumulates a 4 (channels) x 8 (patch
// entries, 7 used) register tile over its slice of the positions; slices are
// combined through LDS and the workgroup writes one partial [Cout][K] to the workspace.
constexpr int kSub = 128;
constexpr int kPixPerBlock = 512;

__global__ void __launch_bounds__(kT) stem_wgrad_kernel(ConvGeom g, StemTab tab, const bf16_t* __restrict__ x,
                                                        const bf16_t* __restrict__ dy, float* __restrict__ part) {
  __shared__ __align__(16) float smem[kT * 32];             // 32 KB
  bf16_t* dyl = reinterpret_cast<bf16_t*>(smem);              // [kSub][64] bf16 = 16 KB
  float* xpl = smem + kSub * 32;                              // [kSub][32] fp32 = 16 KB
  float* red = smem;                                          // reused after the last sub-chunk
  const int K = g.R * g.S * g.Cin;
  const int k_base = blockIdx.y * 64;
  const int kc = min(64, g.Cout - k_base);  // channels of this workgroup (multiple of 4)
  const int KG = kc / 4;                     // channel groups of 4
  const int per_slice = KG * 4;              // threads per position slice
  const int nslice = kT / per_slice;
  const int tid = threadIdx.x;
  const int kg = tid % KG, jg = (tid / KG) % 4, ps = tid / per_slice;
  const bool active = ps < nslice;
  const long M = (long)g.N * g.Ho * g.Wo;
  const long m_begin = (long)blockIdx.x * kPixPerBlock;
  const long m_end = min(m_begin + kPixPerBlock, M);
  float acc[4][8];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = 0.f;

  for (long m0 = m_begin; m0 < m_end; m0 += kSub) {
    __syncthreads();
    // stage dy[sub][64] (zero beyond the range / channel count)
    for (int i = tid; i < kSub * 8; i += kT) {
      const int p = i / 8, c8 = i % 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (m0 + p < m_end && c8 * 8 < kc) v = *reinterpret_cast<const uint4*>(dy + (size_t)(m0 + p) * g.Cout + k_base + c8 * 8);
      *reinterpret_cast<uint4*>(dyl + p * 64 + c8 * 8) = v;
    }
    // stage the input patches: entry (p, jg*8+jj) holds patch element j = jg*7+jj (jj < 7), else 0
    for (int i = tid; i < kSub * 32; i += kT) {
      const int p = i / 32, e = i % 32;
      const int jj = e % 8, j = (e / 8) * 7 + jj;
      float v = 0.f;
      if (jj < 7 && j < K && m0 + p < m_end) {
        int q, wo, n, ho;
        tab.dWo.divmod((int)(m0 + p), &q, &wo);
        tab.dHo.divmod(q, &n, &ho);
        const int c = tab.c[j];
        const int hi = ho * g.stride + tab.r[j] - g.pad, wi = wo * g.stride + tab.s[j] - g.pad;
        if ((unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W)
          v = bf16_to_f32(x[(((size_t)n * g.H + hi) * g.W + wi) * g.Cin + c]);
      }
      xpl[i] = v;
    }
    __syncthreads();
    if (active) {
      for (int p = ps; p < kSub; p += nslice) {
        const uint2 d2 = *reinterpret_cast<const uint2*>(dyl + p * 64 + kg * 4);
        const float d[4] = {__uint_as_float(d2.x << 16), __uint_as_float(d2.x & 0xffff0000u),
                            __uint_as_float(d2.y << 16), __uint_as_float(d2.y & 0xffff0000u)};
        const float4 xa = *reinterpret_cast<const float4*>(xpl + p * 32 + jg * 8);
        const float4 xb = *reinterpret_cast<const float4*>(xpl + p * 32 + jg * 8 + 4);
        const float xs[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int b = 0; b < 8; ++b) acc[a][b] = fmaf(d[a], xs[b], acc[a][b]);
      }
    }
  }
  // combine the position slices: red[tid][32], then threads of slice 0 sum over slices
  __syncthreads();
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) red[tid * 32 + a * 8 + b] = active ? acc[a][b] : 0.f;
  __syncthreads();
  if (ps == 0) {
    float* out = part + (size_t)blockIdx.x * g.Cout * K;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 7; ++b) {
        const int j = jg * 7 + b;
        if (j >= K) continue;
        float s = 0.f;
        for (int sl = 0; sl < nslice; ++sl) s += red[(sl * per_slice + tid) * 32 + a * 8 + b];
        out[(size_t)(k_base + kg * 4 + a) * K + j] = s;
      }
  }
}

StemTab make_tab(const ConvGeom& g) {
  StemTab t{};
  for (int j = 0; j < g.R * g.S * g.Cin && j < kMaxK; ++j) {
    t.c[j] = j % g.Cin;
    t.s[j] = (j / g.Cin) % g.S;
    t.r[j] = j / g.Cin / g.S;
  }
  t.dWo.init(g.Wo);
  t.dHo.init(g.Ho);
  return t;
}

}  // namespace

bool conv_stem_supported(const ConvGeom& g) {
  // pixel indices are decoded with magic-number division: index * divisor must stay below 2^32
  const long M = (long)g.N * g.Ho * g.Wo;
  return g.R * g.S * g.Cin <= kMaxK && g.Cout % 8 == 0 && g.Cout <= 512 && M * g.Wo < (1L << 32) &&
         M / g.Wo * g.Ho < (1L << 32) && M < (1L << 31);
}

size_t conv_stem_wgrad_ws(const ConvGeom& g) {
  const long M = (long)g.N * g.Ho * g.Wo;
  const long nb = (M + kPixPerBlock - 1) / kPixPerBlock;
  return (size_t)nb * g.Cout * g.R * g.S * g.Cin * sizeof(float);
}

int conv_stem_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, hipStream_t st) {
  const long M = (long)g.N * g.Ho * g.Wo;
  const size_t smem = (size_t)g.R * g.S * g.Cin * g.Cout * sizeof(float);
  stem_fwd_kernel<<<(unsigned)((M + kT - 1) / kT), kT, smem, st>>>(g, make_tab(g), x, w, y);
  return launch_status();
}

int conv_stem_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st) {
  const long M = (long)g.N * g.Ho * g.Wo;
  const int nb = (int)((M + kPixPerBlock - 1) / kPixPerBlock);
  dim3 grid(nb, (g.Cout + 63) / 64);
  float* part = nb > 1 ? reinterpret_cast<float*>(ws) : dw;
  stem_wgrad_kernel<<<grid, kT, 0, st>>>(g, make_tab(g), x, dy, part);
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  if (nb > 1) return reduce_partials(part, dw, g.Cout * g.R * g.S * g.Cin, nb, st);
  return CNNK_OK;
}
