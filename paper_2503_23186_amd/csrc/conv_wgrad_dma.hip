// Weight gradient of a 3x3 stride-1 convolution, variant of conv_wgrad_patch.hip whose operand
// tiles go from global memory straight into LDS (buffer_load ... lds: a wavefront's 64 lanes
// deposit 16 bytes each at consecutive LDS addresses; out-of-range offsets deposit zeros).
//
// Same arithmetic and wave roles as the register-staged kernel (eight waves, 32 x 32 (k x c) per
// wave for four taps, the centre tap shared between the two wave groups, partials + fixed-order
// reduce).  What changes is the staging: no load occupies a register, so with three LDS stage
// buffers the loads of stage t+2 are issued while stage t is multiplied - two stages of latency
// tolerance instead of one, with one workgroup per CU (the kernel is bound by the round trip of
// its operand loads, not by LDS reads or MFMA rate).
//
// LDS layout of a stage: operands split into planes of 32 channels with 64-byte rows,
//   dy: [2 planes][128 pixels][64 B],  x patch: [2 planes][PL*64 positions][64 B].
// A direct load fills 16 rows of one plane (lane -> row lane/4, 16-byte chunk lane%4).  Four
// consecutive 64-byte rows span all 64 banks once, which is exactly what a quarter-wave of the
// transposing LDS load reads, so no padding or swizzle is needed (and none is possible: the
// hardware fixes the LDS address of every lane).
#include "common.h"
#include "conv.h"

namespace {

constexpr int kThreads = 512;
constexpr int PS = 128;           // output pixels per stage
constexpr int CT = 64;            // channels per operand tile (64 k, 64 c)
constexpr int ROW_B = 64;         // bytes of a plane row (32 channels)
constexpr int DY_PLANE = PS * ROW_B;

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

// Buffer descriptor as four scalar words (base, no stride, size in bytes, raw 32-bit data format).
__device__ __forceinline__ i32x4_t make_desc(const void* p, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(p);
  return i32x4_t{(int)(unsigned)a, (int)((unsigned)(a >> 32) & 0xffffu), (int)bytes, 0x00020000};
}
// One direct load: lane i of the wave moves 16 bytes from byte offset voff of the buffer to LDS
// address lds_addr + 16*i (zeros when voff is out of range).  Written as assembly so that the
// compiler does not track it: it would otherwise make every LDS read that follows wait for all
// outstanding direct loads, which defeats the prefetch.  The waits are explicit in the kernel.
__device__ __forceinline__ void load16_to_lds(i32x4_t desc, unsigned lds_addr, unsigned voff) {
  // M0 carries the LDS address of such a load; it is put back so the statement is invisible to the
  // compiler's own uses of that register.
  unsigned keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "s"(lds_addr), "v"(voff), "s"(desc)
               : "memory");
}

struct WgDmaArgs {
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
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4_t __attribute__((address_space(3)))*)(lds + off0));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4_t __attribute__((address_space(3)))*)(lds + off1));
  typedef short s16x8_t __attribute__((ext_vector_type(8)));
  const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8_t, v);
}

// PL: the x patch holds at most PL*64 positions.  NBUF: LDS stage buffers (3 where they fit).
template <int PL, int NBUF>
__global__ void __launch_bounds__(kThreads, 2) wgrad_dma_kernel(WgDmaArgs a) {
  constexpr int X_PLANE = PL * 64 * ROW_B;
  constexpr int STAGE_B = 2 * DY_PLANE + 2 * X_PLANE;
  constexpr int NQ = 2 + PL;   // direct loads per wave and stage: two for dy, PL for the patch
  extern __shared__ __align__(16) unsigned char smem[];   // NBUF stage buffers; nothing else lives in LDS
  const int PW = a.W + 2, PH = a.TH + 2;
  const int patch_px = a.TI * PH * PW;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, i16 = lane & 15;
  const int kt = blockIdx.x / a.ctiles, ct = blockIdx.x % a.ctiles;  // 64-channel tiles of k and c
  const int t_begin = blockIdx.y * a.tiles_per_block;
  const int t_end = min(t_begin + a.tiles_per_block, a.mtiles);
  const int M = a.N * a.H * a.W;

  const i32x4_t x_rs = make_desc(a.x, (unsigned)M * a.Cin * 2u);
  const i32x4_t dy_rs = make_desc(a.dy, (unsigned)M * a.Cout * 2u);

  const int grp = wave >> 2, row_half = wave & 1, col_half = (wave >> 1) & 1;
  // per-lane LDS byte offsets of the transposing loads (inside a stage buffer)
  //   A (dy): plane row_half, pixel = ks*16 + (g/2)*8 + i16/4 (+4), channel in plane = (g%2)*16 + (i16%4)*4
  //   (loop position j reads reduction step ks = j ^ grp)
  const int inplane = ((g & 1) * 16 + (i16 & 3) * 4) * 2;
  const int a_off = row_half * DY_PLANE + ((g >> 1) * 8 + (i16 >> 2)) * ROW_B + inplane;
  const int a_off_par[2] = {a_off + grp * 16 * ROW_B, a_off - grp * 16 * ROW_B};  // even / odd positions
  //   B (x): plane col_half, patch position of that pixel at tap (0,0)
  int b_off[PS / 16][2];
#pragma unroll
  for (int ks = 0; ks < PS / 16; ++ks)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int p = (ks ^ grp) * 16 + (g >> 1) * 8 + (i16 >> 2) + 4 * h;
      int q, tw, ti, th;
      a.dW.divmod(p, &q, &tw);
      a.dTH.divmod(q, &ti, &th);
      b_off[ks][h] = 2 * DY_PLANE + col_half * X_PLANE + ((ti * PH + th) * PW + tw) * ROW_B + inplane;
    }
  // patch byte offsets of this wave's four taps, and of the centre tap
  int toff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = grp * 5 + i;
    toff[i] = ((t / 3) * PW + t % 3) * ROW_B;
  }
  const int toff_c = (PW + 1) * ROW_B;

  f32x16_t acc[5];
#pragma unroll
  for (int t = 0; t < 5; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  // Direct-load descriptors of this lane, fixed for the whole kernel.  Load slot j of wave w is
  // load q = j*8 + w of the stage: q < 16 fills 16 rows of a dy plane (plane q/8, rows (q%8)*16 ...),
  // the others 16 rows of an x plane.  A lane supplies row lane/4, 16-byte chunk lane%4.
  const int lrow = lane >> 2, lch = lane & 3;
  int drel[2];       // dy: byte offset relative to pixel m0 (or a marker for "never valid")
  int drow[2];
  int dlds[2];       // LDS byte offset of the 1 KB this wave's load fills
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int q = j * 8 + wave, plane = q >> 3, rg = q & 7;
    const int ch = kt * CT + plane * 32 + lch * 8;
    drow[j] = ch < a.Cout ? rg * 16 + lrow : (1 << 28);   // ragged last channel tile: zeros
    drel[j] = ((rg * 16 + lrow) * a.Cout + ch) * 2;
    dlds[j] = plane * DY_PLANE + rg * 16 * ROW_B;
  }
  int xrel[PL], xdh[PL], xti[PL], xlds[PL];   // byte offset relative to pixel (n0, h0, 0); row shift; image shift
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int qq = j * 8 + wave, plane = qq / (4 * PL), rg = qq % (4 * PL);
    const int pp = rg * 16 + lrow;
    int q, pw, ti, ph;
    a.dPW.divmod(pp, &q, &pw);
    a.dPH.divmod(q, &ti, &ph);
    const int ch = ct * CT + plane * 32 + lch * 8;
    const bool ok = pp < patch_px && pw >= 1 && pw <= a.W && ch < a.Cin;
    xdh[j] = ok ? ph - 1 : -(1 << 20);   // a row shift that never passes the range test
    xti[j] = ti;
    xrel[j] = (((ti * a.H + ph - 1) * a.W + pw - 1) * a.Cin + ch) * 2;
    xlds[j] = 2 * DY_PLANE + plane * X_PLANE + rg * 16 * ROW_B;
  }

  // Stages at or past t_end are loaded from the out-of-range offset (zeros, no memory traffic), so
  // the loop body is the same for every stage.
  auto dma_stage = [&](int t, int sb) __attribute__((always_inline)) {   // sb: LDS address of the stage buffer
    const bool live = t < t_end;
    const int m0 = t * PS;
    const unsigned dbase = (unsigned)m0 * a.Cout * 2u;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const unsigned off = ((int)live & (int)(m0 + drow[j] < M)) ? dbase + (unsigned)drel[j] : kOobOffset;
      load16_to_lds(dy_rs, (unsigned)(sb + dlds[j]), off);
    }
    int q, wrem, n0, h0;
    a.dW.divmod(m0, &q, &wrem);
    a.dH.divmod(q, &n0, &h0);
    const int xbase = ((n0 * a.H + h0) * a.W) * a.Cin * 2;
#pragma unroll
    for (int j = 0; j < PL; ++j) {
      const int ok = (int)live & (int)((unsigned)(h0 + xdh[j]) < (unsigned)a.H) & (int)(n0 + xti[j] < a.N);
      load16_to_lds(x_rs, (unsigned)(sb + xlds[j]), ok ? (unsigned)(xbase + xrel[j]) : kOobOffset);
    }
  };
  // The operands of position j+1 are read from LDS while the MFMAs of position j run (two
  // fragment sets); the scheduling fence after each position keeps the compiler from hoisting a
  // whole stage's reads, which would not fit the register file.
  auto compute = [&](int sboff) __attribute__((always_inline)) {
    const unsigned char* sb = smem + sboff;
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
      af[set] = tr_read8(sb, a_off_par[j & 1] + j * 16 * ROW_B, a_off_par[j & 1] + (j * 16 + 4) * ROW_B);
#pragma unroll
      for (int i = 0; i < 4; ++i) bf[set][i] = tr_read8(sb, b_off[j][0] + tof[i], b_off[j][1] + tof[i]);
      if ((j & 1) == 0) bf[set][4] = tr_read8(sb, b_off[j][0] + tofc, b_off[j][1] + tofc);
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
  // One iteration: wait until this wave's loads of stage t have landed (with three buffers the NQ
  // loads of stage t+1, issued after them, may stay in flight), meet the other waves (all of stage t
  // is in LDS, and everybody is done reading the buffer that is refilled next), issue the loads of
  // the stage NBUF-1 ahead into that buffer, multiply stage t.
  constexpr int RING = NBUF * STAGE_B;
  dma_stage(t_begin, 0);
  if constexpr (NBUF == 3) dma_stage(t_begin + 1, STAGE_B);
  int cur = 0;
  for (int t = t_begin; t < t_end; ++t) {
    if constexpr (NBUF == 3) __builtin_amdgcn_s_waitcnt(0x0f70 | NQ);   // vmcnt(NQ), NQ < 16
    else __builtin_amdgcn_s_waitcnt(0x0f70);                            // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    int fill = cur + (NBUF - 1) * STAGE_B;
    if (fill >= RING) fill -= RING;
    dma_stage(t + NBUF - 1, fill);
    compute(cur);
    cur += STAGE_B;
    if (cur == RING) cur = 0;
  }
  // all direct loads (the last ones fetched nothing) must have landed before LDS is reused
  __builtin_amdgcn_s_waitcnt(0x0f70);
  __syncthreads();

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

}  // namespace

// Launch for a geometry that conv_wgrad_patch_supported() accepted; the plan (pixel split) comes
// from the caller, shared with the register-staged kernel.
int conv_wgrad_dma_launch(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* part, int TI, int TH, int ctiles,
                          int tiles_per_block, int mtiles, int nw, int otiles, int splits, hipStream_t st) {
  WgDmaArgs a{};
  a.x = x; a.dy = dy; a.dw = part;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.Cout = g.Cout;
  a.TI = TI; a.TH = TH; a.ctiles = ctiles; a.tiles_per_block = tiles_per_block; a.mtiles = mtiles; a.nw = nw;
  a.dPW.init(a.W + 2); a.dPH.init(a.TH + 2); a.dW.init(a.W); a.dTH.init(a.TH); a.dH.init(a.H);
  const int patch_px = TI * (TH + 2) * (g.W + 2);
  dim3 grid(otiles, splits);
  auto launch = [&](auto kern, int stage_b, int nbuf, bool* attr_done) {
    const int smem = nbuf * stage_b;
    if (!*attr_done) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) !=
          hipSuccess)
        return (int)CNNK_ERR_HIP;
      *attr_done = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, st, a);
    return launch_status();
  };
  static bool attr43 = false, attr52 = false;
  if (patch_px <= 4 * 64) return launch(wgrad_dma_kernel<4, 3>, 2 * DY_PLANE + 2 * 4 * 64 * ROW_B, 3, &attr43);
  if (patch_px <= 5 * 64) return launch(wgrad_dma_kernel<5, 2>, 2 * DY_PLANE + 2 * 5 * 64 * ROW_B, 2, &attr52);
  return CNNK_ERR_UNSUPPORTED;
}
