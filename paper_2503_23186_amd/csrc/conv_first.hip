// Forward pass of the first layer: a 3x3 stride-1 pad-1 convolution of a 3-channel image (the
// "stem" of the CIFAR-shaped networks), bf16 storage.  K = 27 is one padded 32-deep MFMA reduction,
// so the layer is bound by writing its output (64 channels per pixel against 3 read).  No operand
// staging at all: a pixel's nine 3-channel taps are three runs of nine contiguous bf16 values in
// the NHWC image, so every lane gathers the 16 reduction elements of its MFMA fragment straight
// from the (cache-resident) image with 2-byte loads, the weights (at most 64 x 27) sit in
// registers as MFMA fragments for the whole kernel, and the only LDS use is the wave-local
// transposition of the accumulators into 16-byte stores.
#include "common.h"
#include "conv.h"

namespace {

constexpr int kT = 256;          // four waves, 64 output pixels each
constexpr int kPixPerBlock = 256;

struct FirstArgs {
  const bf16_t* x;
  const bf16_t* w;
  bf16_t* y;
  float* stats;    // nullable: [2][Cout][nblocks] per-workgroup column sums and sums of squares
  int N, H, W, Cout, M, nblocks;
  FastDiv dW, dH;
};

__device__ __forceinline__ bf16x8_t pack8(const bf16_t* v) {
  typedef short s16x8_t __attribute__((ext_vector_type(8)));
  const s16x8_t s = {(short)v[0], (short)v[1], (short)v[2], (short)v[3], (short)v[4], (short)v[5], (short)v[6], (short)v[7]};
  return __builtin_bit_cast(bf16x8_t, s);
}

// TN: 32-column tiles of output channels (1: Cout <= 32, 2: Cout <= 64)
template <int TN>
__global__ void __launch_bounds__(kT) first_fwd_kernel(FirstArgs a) {
  constexpr int LDW = TN * 32 + 8;
  __shared__ __align__(16) bf16_t strips[kT / 64][8][LDW];
  __shared__ float sred[2][kT / 64][TN * 32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kg = lane >> 5;   // which 8 of a 16-deep reduction slice this lane holds

  // weights as B fragments: lane (channel n = lane % 32 of tile j, reduction elements ks*16 + kg*8 ...)
  bf16x8_t bw[TN][2];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int n = j * 32 + (lane & 31);
      bf16_t v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int k = ks * 16 + kg * 8 + e;
        v[e] = (n < a.Cout && k < 27) ? a.w[n * 27 + k] : (bf16_t)0;
      }
      bw[j][ks] = pack8(v);
    }

  f32x16_t acc[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int m0 = blockIdx.x * kPixPerBlock + wave * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    // A fragments of 32 pixels: lane (pixel m0 + i*32 + lane % 32, reduction elements ks*16 + kg*8 ...)
    const int p = m0 + i * 32 + (lane & 31);
    int q, wc, n, h;
    a.dW.divmod(p, &q, &wc);
    a.dH.divmod(q, &n, &h);
    const bool pok = p < a.M;
    bf16x8_t af[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16_t v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int k = ks * 16 + kg * 8 + e;      // = r*9 + s*3 + c
        const int r = (k * 57) >> 9;              // k / 9 for k < 32
        const int jj = k - r * 9;                 // s*3 + c
        const int s = (jj * 11) >> 5;             // jj / 3 for jj < 9
        const int hh = h + r - 1, ww = wc + s - 1;
        const bool ok = pok && k < 27 && (unsigned)hh < (unsigned)a.H && (unsigned)ww < (unsigned)a.W;
        v[e] = ok ? a.x[((size_t)(n * a.H + hh) * a.W + (wc - 1)) * 3 + jj] : (bf16_t)0;
      }
      af[ks] = pack8(v);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks], bw[j][ks], acc[i][j], 0, 0, 0);
  }

  // per-channel sums of the fp32 accumulators over the workgroup's 256 pixels (pixels beyond M
  // hold zeros): one partial row per workgroup
  if (a.stats) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float v = acc[i][j][r];
          s1 += v;
          s2 = fmaf(v, v, s2);
        }
      s1 += __shfl_xor(s1, 32, 64);
      s2 += __shfl_xor(s2, 32, 64);
      if (lane < 32) {
        sred[0][wave][j * 32 + lane] = s1;
        sred[1][wave][j * 32 + lane] = s2;
      }
    }
    __syncthreads();
    if (tid < 2 * TN * 32) {
      const int v = tid / (TN * 32), c = tid % (TN * 32);
      if (c < a.Cout) {
        float t = sred[v][0][c];
#pragma unroll
        for (int w_ = 1; w_ < kT / 64; ++w_) t += sred[v][w_][c];
        a.stats[((size_t)v * a.Cout + c) * a.nblocks + blockIdx.x] = t;
      }
    }
  }

  // wave-local epilogue: 8 rows x TN*32 columns at a time through the wave's LDS strip
  bf16_t* Cw = &strips[wave][0][0];
  constexpr int CH = TN * 4;   // 16-byte chunks per strip row
  const int lrow = lane / CH, ch = lane % CH;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int rho = 0; rho < 4; ++rho)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          Cw[((lane >> 5) * 4 + rho) * LDW + j * 32 + (lane & 31)] = f32_to_bf16_hw(acc[i][j][q * 4 + rho]);
      // the 16-byte reads below go through another type than the 2-byte writes above: tell the
      // compiler that they touch the same memory (the hardware keeps a wave's LDS operations in order)
      asm volatile("" ::: "memory");
      if (lrow < 8) {
        const int m = m0 + i * 32 + q * 8 + lrow, co = ch * 8;
        if (m < a.M && co < a.Cout)
          *reinterpret_cast<uint4*>(a.y + (size_t)m * a.Cout + co) = *reinterpret_cast<const uint4*>(Cw + lrow * LDW + ch * 8);
      }
      asm volatile("" ::: "memory");
    }
}

// ---- weight gradient ---------------------------------------------------------------------------
// dw[k][q] = sum over pixels of dy[p][k] * A[p][q], q = (tap, channel) as in the forward pass, as
// the MFMA product A^T (32 x pixels) * dy (pixels x 64): both fragments want eight consecutive
// PIXELS per lane, which for a lane's fixed column is a gather of 2-byte elements - from the
// cache-resident image for A, and for dy 32 adjacent lanes read 64 contiguous bytes of a pixel's
// channel row, so every line of dy still comes from memory once.  No LDS staging.  A wavefront
// walks whole image rows (16 pixels per MFMA step, so W % 16 == 0), workgroups write fp32 partials
// in accumulator layout, a second kernel sums them into dw[k][r][s][c] (and may apply the SGD
// update of the parameter in the same launch).
struct FirstWgArgs {
  const bf16_t* x;
  const bf16_t* dy;
  float* part;       // [workgroups][TN][16][64]
  int N, H, W, Cout, rows, rows_per_wave;
  FastDiv dH;
};

template <int TN>
__global__ void __launch_bounds__(kT) first_wgrad_kernel(FirstWgArgs a) {
  __shared__ float red[kT / 64][TN][16][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kg = lane >> 5, l31 = lane & 31;
  // this lane's column of A: q = l31 = r*9 + s*3 + c
  const int fr = (l31 * 57) >> 9, jj = l31 - fr * 9, fs = (jj * 11) >> 5;
  const bool qok = l31 < 27;
  f32x16_t acc[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

  const int row_begin = (blockIdx.x * (kT / 64) + wave) * a.rows_per_wave;
  const int row_end = min(row_begin + a.rows_per_wave, a.rows);
  for (int R = row_begin; R < row_end; ++R) {      // image row R = n*H + h
    int n, h;
    a.dH.divmod(R, &n, &h);
    const int hh = h + fr - 1;
    const bool rok = qok && (unsigned)hh < (unsigned)a.H;
    const long xbase = ((long)(R + fr - 1) * a.W + fs - 1) * 3 + (jj - fs * 3);   // element index at w = 0 (used only when in range)
    const bf16_t* dyrow = a.dy + (size_t)R * a.W * a.Cout + l31;
    for (int w0 = 0; w0 < a.W; w0 += 16) {
      bf16_t va[8], vb[TN][8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int wc = w0 + kg * 8 + e;
        const bool ok = rok && (unsigned)(wc + fs - 1) < (unsigned)a.W;
        va[e] = ok ? a.x[xbase + (long)wc * 3] : (bf16_t)0;
#pragma unroll
        for (int j = 0; j < TN; ++j)
          vb[j][e] = (j * 32 + l31 < a.Cout) ? dyrow[(size_t)wc * a.Cout + j * 32] : (bf16_t)0;
      }
      const bf16x8_t af = pack8(va);
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pack8(vb[j]), acc[j], 0, 0, 0);
    }
  }
  // four wavefront accumulators -> one partial per workgroup (accumulator layout kept)
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][j][r][lane] = acc[j][r];
  __syncthreads();
  for (int i = tid; i < TN * 16 * 64; i += kT) {
    const float* p0 = &red[0][0][0][0] + i;
    float t = p0[0];
#pragma unroll
    for (int w_ = 1; w_ < kT / 64; ++w_) t += p0[(size_t)w_ * TN * 16 * 64];
    a.part[(size_t)blockIdx.x * TN * 16 * 64 + i] = t;
  }
}

struct FirstSgd {
  float* w;
  float* v;
  bf16_t* wlp;
  float lr, mu, wd;
};

// dw[k*27 + q] = sum over P workgroup partials.  A thread owns one element of the accumulator
// layout (adjacent threads read adjacent floats of every partial), 16 thread groups share the
// partials of an element and their sums are added in group order; the element's (k, q) is decoded
// only for the final store.  SGD: also g' = g + wd*w; v <- mu*v + g'; w <- w - lr*v.
template <bool SGD>
__global__ void __launch_bounds__(256) first_wgrad_reduce_kernel(const float* __restrict__ part,
                                                                 float* __restrict__ dw, int Cout, int TN, int P,
                                                                 FirstSgd sg) {
  __shared__ float red[16][16];
  const int e = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int a = blockIdx.x * 16 + e;            // accumulator element: ((j*16 + r)*64 + lane)
  const int total = TN * 16 * 64;
  float acc = 0.f;
  if (a < total) {
    // up to sixteen partials per round, all loads issued before the first add (a partial past the
    // end is not loaded and adds zero); same order of additions as a plain loop
    const int rounds = (P + 15) / 16;
    for (int k0 = 0; k0 < rounds; k0 += 16) {
      float v[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        const int p = grp + (k0 + k) * 16;
        v[k] = 0.f;
        if (p < P) v[k] = part[(size_t)p * total + a];
      }
#pragma unroll
      for (int k = 0; k < 16; ++k)
        if (k0 + k < rounds) acc += v[k];
    }
  }
  red[grp][e] = acc;
  __syncthreads();
  if (grp != 0 || a >= total) return;
  float g = red[0][e];
#pragma unroll
  for (int k_ = 1; k_ < 16; ++k_) g += red[k_][e];
  // accumulator layout: row q = (r/4)*8 + (lane/32)*4 + r%4, column k = j*32 + lane%32
  const int ln = a & 63, r = (a >> 6) & 15, j = a >> 10;
  const int q = (r >> 2) * 8 + (ln >> 5) * 4 + (r & 3), k = j * 32 + (ln & 31);
  if (q >= 27 || k >= Cout) return;
  const int i = k * 27 + q;
  dw[i] = g;
  if (SGD) {
    const float wi = sg.w[i];
    const float gp = fmaf(sg.wd, wi, g);
    const float vn = fmaf(sg.mu, sg.v[i], gp);
    const float wn = fmaf(-sg.lr, vn, wi);
    sg.v[i] = vn;
    sg.w[i] = wn;
    if (sg.wlp) sg.wlp[i] = f32_to_bf16(wn);
  }
}

inline int first_wg_rows_per_wave(const ConvGeom& g) {
  const int rows = g.N * g.H;
  int rpw = (rows + 2047) / 2048;          // about 2048 wavefronts on the device
  return rpw < 1 ? 1 : rpw;
}
inline int first_wg_blocks(const ConvGeom& g) {
  const int rows = g.N * g.H, per_block = first_wg_rows_per_wave(g) * (kT / 64);
  return (rows + per_block - 1) / per_block;
}

}  // namespace

bool conv_first_supported(const ConvGeom& g) {
  if (g.Cin != 3 || g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1) return false;
  if (g.Cout % 8 != 0 || g.Cout > 64) return false;
  const long M = (long)g.N * g.H * g.W;
  return M * 64 < (1L << 31);   // 32-bit pixel indices and element offsets
}

int conv_first_stat_rows(const ConvGeom& g) {
  return (int)(((long)g.N * g.H * g.W + kPixPerBlock - 1) / kPixPerBlock);
}

size_t conv_first_ws(const ConvGeom& g) {
  return align_up((size_t)conv_first_stat_rows(g) * 2 * g.Cout * sizeof(float), 256);
}

int conv_first_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* ch_sum, float* ch_sumsq,
                   void* ws, hipStream_t st) {
  FirstArgs a{};
  a.x = x; a.w = w; a.y = y;
  a.stats = ch_sum ? reinterpret_cast<float*>(ws) : nullptr;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cout = g.Cout;
  a.M = g.N * g.H * g.W;
  a.nblocks = conv_first_stat_rows(g);
  a.dW.init((unsigned)g.W);
  a.dH.init((unsigned)g.H);
  if (g.Cout <= 32) first_fwd_kernel<1><<<a.nblocks, kT, 0, st>>>(a);
  else first_fwd_kernel<2><<<a.nblocks, kT, 0, st>>>(a);
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  if (!ch_sum) return CNNK_OK;
  return channel_sums_finalize(a.stats, a.nblocks, g.Cout, ch_sum, ch_sumsq, st);
}

bool conv_first_wgrad_supported(const ConvGeom& g) { return conv_first_supported(g) && g.W % 16 == 0; }

size_t conv_first_wgrad_ws(const ConvGeom& g) {
  const int TN = g.Cout <= 32 ? 1 : 2;
  return align_up((size_t)first_wg_blocks(g) * TN * 16 * 64 * sizeof(float), 256);
}

int conv_first_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st) {
  FirstWgArgs a{};
  a.x = x; a.dy = dy;
  a.part = reinterpret_cast<float*>(ws);
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cout = g.Cout;
  a.rows = g.N * g.H;
  a.rows_per_wave = first_wg_rows_per_wave(g);
  a.dH.init((unsigned)g.H);
  const int TN = g.Cout <= 32 ? 1 : 2, nblk = first_wg_blocks(g);
  if (TN == 1) first_wgrad_kernel<1><<<nblk, kT, 0, st>>>(a);
  else first_wgrad_kernel<2><<<nblk, kT, 0, st>>>(a);
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  const unsigned rblk = (unsigned)(TN * 16 * 64 / 16);
  SgdFuse* f = t_cnnk_sgd_fuse;
  if (f && !f->done) {
    if (f->wait && hipStreamWaitEvent(st, f->wait, 0) != hipSuccess) return CNNK_ERR_HIP;
    const FirstSgd sg{f->w, f->v, static_cast<bf16_t*>(f->wlp), f->lr, f->mu, f->wd};
    first_wgrad_reduce_kernel<true><<<rblk, 256, 0, st>>>(a.part, dw, g.Cout, TN, nblk, sg);
    f->done = true;
  } else {
    const FirstSgd none{nullptr, nullptr, nullptr, 0.f, 0.f, 0.f};
    first_wgrad_reduce_kernel<false><<<rblk, 256, 0, st>>>(a.part, dw, g.Cout, TN, nblk, none);
  }
  return launch_status();
}
