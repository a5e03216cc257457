// Weight gradient of a 3x3 stride-1 convolution with both operands read from LDS in their
// natural [pixel][channel] layout through the gfx950 transposing LDS load (ds_read_b64_tr_b16).
//
// dw[k][r][s][c] = sum_pixels dy[pixel][k] * x[pixel + (r-1, s-1)][c].  The reduction index (the
// pixel) is the slow index of both tensors, so the MFMA operands (8 consecutive reduction
// elements per lane) need a transposition; the transposing load does it on the way out of LDS,
// which leaves the x tile as a patch with a 1-pixel halo from which all nine taps are served
// (a tap is a pixel offset).  A workgroup owns 64 output channels x (9 taps x 64 input
// channels) of dw and a range of pixel tiles; each range writes an fp32 partial to the
// workspace and a fixed-order reduction kernel sums them (deterministic, no atomics).
#include "common.h"
#include "conv.h"

namespace {

constexpr int kThreads = 512;
constexpr int PS = 128;           // output pixels per stage
constexpr int CT = 64;            // channels per operand tile (64 k, 64 c)
constexpr int PITCH_B = CT * 2 + 32;  // LDS row pitch in bytes: 4 consecutive rows cover distinct banks
constexpr int kRowsPerPass = kThreads / 8;                  // tile rows staged per 16-byte load of the workgroup
constexpr int kDyLoads = PS / kRowsPerPass;                 // 16-byte loads per thread for the dy tile (2)

typedef short s16x4_t __attribute__((ext_vector_type(4)));

struct WgPatchArgs {
  const bf16_t* x;
  const bf16_t* dy;
  float* dw;
  int N, H, W, Cin, Cout;
  int TI, TH;          // stage = TI images x TH rows x W columns = PS pixels
  int ctiles;          // ceil(Cin / 64)
  int tiles_per_block; // pixel stages per workgroup
  int mtiles;          // total pixel stages
  int nw;              // Cout*9*Cin: stride between the partials of consecutive pixel ranges
  FastDiv dPW, dPH, dW, dTH, dH;
};

__device__ __forceinline__ bf16x8_t tr_read8(const unsigned char* lds, int off0, int off1) {
  // two transposing loads give this lane reduction slots 0..3 and 4..7 of its row / column
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4_t __attribute__((address_space(3)))*)(lds + off0));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4_t __attribute__((address_space(3)))*)(lds + off1));
  typedef short s16x8_t __attribute__((ext_vector_type(8)));
  const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8_t, v);
}

// Eight waves, two per SIMD.  A wave owns a 32 x 32 (k x c) corner of the 64 x 64 tile for four
// taps: waves 0..3 the taps 0..3, waves 4..7 the taps 5..8.  The centre tap (4) is shared: waves
// 0..3 take it on the even 16-pixel reduction steps, waves 4..7 on the odd ones, so both groups
// issue the same number of MFMAs per stage; the two halves of the centre tap are added through
// LDS, in that order, once at the end.
// The stages are double-buffered in LDS: the loads of stage t+1 are issued before the MFMAs of
// stage t and written to the other buffer after them, one barrier per stage.
// PL: 16-byte loads per thread for the x patch (patch holds at most PL * 64 pixels)
template <int PL>
__global__ void __launch_bounds__(kThreads, 2) wgrad_patch_kernel(WgPatchArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int PW = a.W + 2, PH = a.TH + 2;
  const int patch_px = a.TI * PH * PW;
  const int stage_bytes = (PS + patch_px) * PITCH_B;   // dy tile [PS][PITCH_B], then x patch [patch_px][PITCH_B]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, i16 = lane & 15;
  const int kt = blockIdx.x / a.ctiles, ct = blockIdx.x % a.ctiles;  // 64-channel tiles of k and c
  const int t_begin = blockIdx.y * a.tiles_per_block;
  const int t_end = min(t_begin + a.tiles_per_block, a.mtiles);
  const int M = a.N * a.H * a.W;

  const __amdgpu_buffer_rsrc_t x_rs = make_rsrc(a.x, (unsigned)M * a.Cin * 2u);
  const __amdgpu_buffer_rsrc_t dy_rs = make_rsrc(a.dy, (unsigned)M * a.Cout * 2u);

  const int grp = wave >> 2, row_half = wave & 1, col_half = (wave >> 1) & 1;
  // per-lane LDS byte offsets of the transposing loads
  //   A (dy): pixel = ks*16 + (g/2)*8 + i16/4 (+4), channel = row_half*32 + (g%2)*16 + (i16%4)*4
  //   (loop position j reads reduction step ks = j ^ grp)
  const int a_off = (((g >> 1) * 8 + (i16 >> 2)) * PITCH_B) + (row_half * 32 + (g & 1) * 16 + (i16 & 3) * 4) * 2;
  const int a_off_par[2] = {a_off + grp * 16 * PITCH_B, a_off - grp * 16 * PITCH_B};  // even / odd positions
  //   B (x): patch position of that pixel at tap (0,0), channel = col_half*32 + ...
  int b_off[PS / 16][2];
#pragma unroll
  for (int ks = 0; ks < PS / 16; ++ks)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int p = (ks ^ grp) * 16 + (g >> 1) * 8 + (i16 >> 2) + 4 * h;
      int q, tw, ti, th;
      a.dW.divmod(p, &q, &tw);
      a.dTH.divmod(q, &ti, &th);
      b_off[ks][h] = ((ti * PH + th) * PW + tw) * PITCH_B + (col_half * 32 + (g & 1) * 16 + (i16 & 3) * 4) * 2;
    }
  // patch byte offsets of this wave's four taps, and of the centre tap
  int toff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = grp * 5 + i;
    toff[i] = ((t / 3) * PW + t % 3) * PITCH_B;
  }
  const int toff_c = (PW + 1) * PITCH_B;

  f32x16_t acc[5];
#pragma unroll
  for (int t = 0; t < 5; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  const int kc = tid & 7;  // 16-byte chunk (8 channels) inside a 64-channel row
  uint4 dreg[kDyLoads], xreg[PL];
  // Per-thread load descriptors, fixed for the whole kernel: a stage only moves the origin
  // (image n0, row h0), which enters as one scalar byte offset per tensor.
  int xrel[PL], xdh[PL], xti[PL];   // byte offset relative to pixel (n0, h0, 0); row shift; image shift
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int pp = (tid >> 3) + j * kRowsPerPass;
    int q, pw, ti, ph;
    a.dPW.divmod(pp, &q, &pw);
    a.dPH.divmod(q, &ti, &ph);
    const bool ok = pp < patch_px && pw >= 1 && pw <= a.W && ct * CT + kc * 8 < a.Cin;   // ragged last channel tile
    xdh[j] = ok ? ph - 1 : -(1 << 20);   // a row shift that never passes the range test
    xti[j] = ti;
    xrel[j] = (((ti * a.H + ph - 1) * a.W + pw - 1) * a.Cin + ct * CT + kc * 8) * 2;
  }
  const int drel = ((tid >> 3) * a.Cout + kt * CT + kc * 8) * 2;
  const bool dch_ok = kt * CT + kc * 8 < a.Cout;   // ragged last channel tile: zeros

  // Stages at or past t_end are loaded from the out-of-range offset (zeros, no memory traffic), so
  // the loop body is the same for every stage.
  auto load_stage = [&](int t) {
    const bool live = t < t_end;
    const int m0 = t * PS;
    const unsigned dbase = (unsigned)m0 * a.Cout * 2u;
#pragma unroll
    for (int j = 0; j < kDyLoads; ++j) {
      const int p = (tid >> 3) + j * kRowsPerPass;
      const unsigned off = ((int)live & (int)(m0 + p < M) & (int)dch_ok) ? dbase + (unsigned)(drel + j * kRowsPerPass * a.Cout * 2) : kOobOffset;
      dreg[j] = buffer_load16(dy_rs, off, 0);
    }
    int q, wrem, n0, h0;
    a.dW.divmod(m0, &q, &wrem);
    a.dH.divmod(q, &n0, &h0);
    const int xbase = ((n0 * a.H + h0) * a.W) * a.Cin * 2;
#pragma unroll
    for (int j = 0; j < PL; ++j) {
      const int ok = (int)live & (int)((unsigned)(h0 + xdh[j]) < (unsigned)a.H) & (int)(n0 + xti[j] < a.N);
      xreg[j] = buffer_load16(x_rs, ok ? (unsigned)(xbase + xrel[j]) : kOobOffset, 0);
    }
  };
  auto store_stage = [&](int buf) {
    unsigned char* Dl = smem + buf * stage_bytes;
    unsigned char* Xl = Dl + PS * PITCH_B;
#pragma unroll
    for (int j = 0; j < kDyLoads; ++j) {
      const int p = (tid >> 3) + j * kRowsPerPass;
      *reinterpret_cast<uint4*>(Dl + p * PITCH_B + kc * 16) = dreg[j];
    }
#pragma unroll
    for (int j = 0; j < PL; ++j) {
      const int pp = (tid >> 3) + j * kRowsPerPass;
      if (pp < patch_px) *reinterpret_cast<uint4*>(Xl + pp * PITCH_B + kc * 16) = xreg[j];
    }
  };
  // The operands of position j+1 are read from LDS while the MFMAs of position j run (two
  // fragment sets); the scheduling fence after each position keeps the compiler from hoisting a
  // whole stage's reads, which would not fit the register file.
  auto compute = [&](int buf) {
    const unsigned char* Dl = smem + buf * stage_bytes;
    const unsigned char* Xl = Dl + PS * PITCH_B;
    bf16x8_t af[2], bf[2][5];
    // the tap offsets are loop invariants; hiding that from the compiler keeps it from
    // precomputing (and spilling) the 80 operand addresses of a stage
    int tof[4], tofc = toff_c;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      tof[i] = toff[i];
      asm volatile("" : "+s"(tof[i]));
    }
    asm volatile("" : "+s"(tofc));
    auto read_step = [&](int j, int set) {   // both arguments are constants after unrolling
      af[set] = tr_read8(Dl, a_off_par[j & 1] + j * 16 * PITCH_B, a_off_par[j & 1] + (j * 16 + 4) * PITCH_B);
#pragma unroll
      for (int i = 0; i < 4; ++i) bf[set][i] = tr_read8(Xl, b_off[j][0] + tof[i], b_off[j][1] + tof[i]);
      if ((j & 1) == 0) bf[set][4] = tr_read8(Xl, b_off[j][0] + tofc, b_off[j][1] + tofc);
    };
    read_step(0, 0);
#pragma unroll
    for (int j = 0; j < PS / 16; ++j) {
      if (j + 1 < PS / 16) read_step(j + 1, (j + 1) & 1);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[j & 1], bf[j & 1][i], acc[i], 0, 0, 0);
      if ((j & 1) == 0)
        acc[4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[j & 1], bf[j & 1][4], acc[4], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  load_stage(t_begin);
  store_stage(0);
  __syncthreads();
  for (int t = t_begin; t < t_end; ++t) {
    const int buf = (t - t_begin) & 1;
    load_stage(t + 1);
    compute(buf);
    store_stage(buf ^ 1);
    __syncthreads();
  }

  // centre tap: waves 4..7 hand their half to waves 0..3
  float* red = reinterpret_cast<float*>(smem);   // [4][16][64]
  if (grp == 1) {
#pragma unroll
    for (int r = 0; r < 16; ++r) red[((wave & 3) * 16 + r) * 64 + lane] = acc[4][r];
  }
  __syncthreads();
  if (grp == 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[4][r] += red[((wave & 3) * 16 + r) * 64 + lane];
  }

  // dw[k][tap][c]: this lane holds column c = ct*64 + col_half*32 + lane%32 and rows
  // k = kt*64 + row_half*32 + (r/4)*8 + (lane/32)*4 + r%4
  const int c = ct * CT + col_half * 32 + (lane & 31);
  float* out = a.dw + (size_t)blockIdx.y * a.nw;
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    if (i == 4 && grp == 1) break;
    const int t = i == 4 ? 4 : grp * 5 + i;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int k = kt * CT + row_half * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
      if (k < a.Cout && c < a.Cin) out[((size_t)k * 9 + t) * a.Cin + c] = acc[i][r];
    }
  }
}

bool wg_geometry(const ConvGeom& g, int* ti, int* th) {
  const int hw = g.H * g.W;
  if (hw <= PS) {
    if (PS % hw != 0) return false;
    *ti = PS / hw; *th = g.H;
  } else {
    if (PS % g.W != 0 || g.H % (PS / g.W) != 0) return false;
    *ti = 1; *th = PS / g.W;
  }
  return (*ti) * (*th + 2) * (g.W + 2) <= 5 * kRowsPerPass;
}

template <int PL>
int launch_wg(const WgPatchArgs& a, dim3 grid, size_t smem, hipStream_t st) {
  auto kern = wgrad_patch_kernel<PL>;
  static bool attr_done = false;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)(2 * (PS + PL * kRowsPerPass) * PITCH_B)) != hipSuccess)
      return CNNK_ERR_HIP;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, st, a);
  return launch_status();
}

}  // namespace

bool conv_wgrad_patch_supported(const ConvGeom& g) {
  if (g_cnnk_tune[6] < 0) return false;
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1) return false;
  // channel counts in whole 16-byte chunks; a ragged last 64-channel tile computes on zeros, so
  // only shapes that waste at most a third of the tile grid are taken (160 = 2.5 tiles: yes)
  if (g.Cin % 8 != 0 || g.Cout % 8 != 0) return false;
  if (((g.Cin + CT - 1) / CT) * CT * 3 > g.Cin * 4 || ((g.Cout + CT - 1) / CT) * CT * 3 > g.Cout * 4) return false;
  const long M = (long)g.N * g.H * g.W;
  if (M * g.Cin * 2 >= (1L << 31) || M * g.Cout * 2 >= (1L << 31)) return false;
  int ti, th;
  return wg_geometry(g, &ti, &th);
}

static void wg_plan(const ConvGeom& g, WgPatchArgs* a, int* splits, int cus = 256) {
  a->ctiles = (g.Cin + CT - 1) / CT;
  const int otiles = ((g.Cout + CT - 1) / CT) * a->ctiles;
  const long M = (long)g.N * g.H * g.W;
  a->mtiles = (int)((M + PS - 1) / PS);
  const int target = g_cnnk_tune[6] > 0 ? g_cnnk_tune[6] : cus;
  int sp = (target + otiles - 1) / otiles;
  if (sp > a->mtiles) sp = a->mtiles;
  if (sp < 1) sp = 1;
  a->tiles_per_block = (a->mtiles + sp - 1) / sp;
  *splits = (a->mtiles + a->tiles_per_block - 1) / a->tiles_per_block;
  a->nw = g.Cout * 9 * g.Cin;
}

size_t conv_wgrad_patch_ws(const ConvGeom& g) {
  WgPatchArgs a{};
  int splits;
  wg_plan(g, &a, &splits);
  return splits > 1 ? (size_t)splits * a.nw * sizeof(float) : 0;
}

int conv_wgrad_patch(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st) {
  WgPatchArgs a{};
  if (!wg_geometry(g, &a.TI, &a.TH)) return CNNK_ERR_UNSUPPORTED;
  int splits;
  wg_plan(g, &a, &splits, t_cnnk_wgrad_cus);
  a.x = x; a.dy = dy;
  a.dw = splits > 1 ? reinterpret_cast<float*>(ws) : dw;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.Cout = g.Cout;
  a.dPW.init(a.W + 2); a.dPH.init(a.TH + 2); a.dW.init(a.W); a.dTH.init(a.TH); a.dH.init(a.H);
  const int otiles = ((g.Cout + CT - 1) / CT) * a.ctiles;
  const int patch_px = a.TI * (a.TH + 2) * (a.W + 2);
  const size_t smem = (size_t)2 * (PS + patch_px) * PITCH_B;
  dim3 grid(otiles, splits);
  const int pl = (patch_px + kRowsPerPass - 1) / kRowsPerPass;
  int rc;
  if (g_cnnk_tune[10] >= 0)   // -1: the register-staged kernel of this file
    rc = conv_wgrad_dma_launch(g, x, dy, a.dw, a.TI, a.TH, a.ctiles, a.tiles_per_block, a.mtiles, a.nw, otiles, splits, st);
  else if (pl <= 4) rc = launch_wg<4>(a, grid, smem, st);
  else rc = launch_wg<5>(a, grid, smem, st);
  if (rc != CNNK_OK || splits == 1) return rc;
  return reduce_partials(a.dw, dw, a.nw, splits, st);
}
