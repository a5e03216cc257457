// bf16 implicit-GEMM convolution kernels on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16,
// fp32 accumulation).  Activations NHWC, weights [Cout][R][S][Cin].
//
//  * igemm_kernel: forward and data-gradient.  GEMM rows are output pixels, columns are output
//    channels, the reduction runs over (filter tap, source channel).  A tap is a (dh, dw) shift
//    of the source image plus an index into the weight array, so the same kernel serves the
//    forward pass (source x, shifts r-pad / s-pad, source step = stride) and the data gradient
//    (source dy, weights transposed to [Cin][tap][Cout], one launch class per output parity so
//    that a strided layer only visits the taps that really contribute).
//  * wgrad_kernel: weight gradient.  GEMM rows are output channels, columns are (tap, input
//    channel), the reduction runs over output pixels, split across workgroups; both operands
//    arrive channel-contiguous and are transposed in registers on their way into LDS.
#include <type_traits>
#include "common.h"
#include "conv.h"

int g_cnnk_tune[16] = {0};
thread_local int t_cnnk_wgrad_cus = 256;

namespace {

constexpr int kThreads = 256;
constexpr int kMaxTaps = 9;

struct TapTable {
  int nclass;
  int cls_begin[5];
  int dh[kMaxTaps], dw[kMaxTaps], widx[kMaxTaps];
  int Hm[4], Wm[4], oh[4], ow[4];
  FastDiv dW[4], dH[4];   // division by Wm / Hm of each class
};

struct IgemmArgs {
  const bf16_t* src;
  const bf16_t* wt;
  bf16_t* dst;
  int Nimg, Hs, Ws, Cs;  // source tensor
  int Hd, Wd, Cd;        // destination tensor; Cd = GEMM columns
  int T;                 // taps in the weight array: wt[Cd][T][Cs]
  int ss, os;            // source step per sub-grid index; destination step per sub-grid index
  int accumulate;
  int ntiles;
  float* stats;          // nullable: [2][Cd][mtiles * WM] per-wave column sums and sums of squares
  int mtiles;
  int tpb;               // tiles one workgroup walks
  FastDiv dNt;           // division by ntiles
  TapTable tt;
};

// OCC: workgroups per CU the register allocation must leave room for.
//
// A workgroup walks a.tpb consecutive tiles (tile t = (pixel tile t / ntiles, channel tile
// t % ntiles), so neighbours share their pixel rows).  The stage loads do not know about tile
// borders: the loads of the next tile's first stages are in flight while the current tile's last
// MFMAs and its epilogue run, which hides the prologue of every tile but the first.  The epilogue
// is wave-local (a wave transposes its own accumulators through a private LDS strip, 8 rows at a
// time, into 16-byte stores), so it needs no workgroup barrier and leaves the stage buffers alone.
template <int BM, int BN, int BK, int WM, int WN, int OCC>
__global__ void __launch_bounds__(kThreads, OCC) igemm_kernel(IgemmArgs a) {
  constexpr int LDK = BK + 8;  // padded row (elements): conflict-free 16-byte fragment reads
  constexpr int KC = BK / 8;
  constexpr int RPP = kThreads / KC;  // tile rows filled per pass of the workgroup
  constexpr int A_IT = (BM + RPP - 1) / RPP, B_IT = (BN + RPP - 1) / RPP;  // rows beyond the tile are skipped
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int LDW = TN * 32 + 8;   // row pitch (elements) of a wave's epilogue strip
  static_assert(WM * WN == 4 && A_IT >= 1 && B_IT >= 1 && TM >= 1 && (TN == 1 || TN == 2), "tile shape");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);  // [2][BM][LDK]
  bf16_t* Bs = As + 2 * BM * LDK;                    // [2][BN][LDK]
  bf16_t* strips = Bs + 2 * BN * LDK;                // [4 waves][8][LDW]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);  // consecutive workgroups share an XCD (and its L2)
  const int cls = blockIdx.y;
  const int Hm = a.tt.Hm[cls], Wm = a.tt.Wm[cls];
  const FastDiv dWm = a.tt.dW[cls], dHm = a.tt.dH[cls];
  const int M = a.Nimg * Hm * Wm;
  const int tiles_cls = ((M + BM - 1) / BM) * a.ntiles;
  const int t_begin = b * a.tpb;
  const int t_end = min(t_begin + a.tpb, tiles_cls);
  if (t_begin >= t_end) return;
  const int tap0 = a.tt.cls_begin[cls], ntap = a.tt.cls_begin[cls + 1] - tap0;
  const int oh = a.tt.oh[cls], ow = a.tt.ow[cls];
  const FastDiv dNt = a.dNt;
  if (ntap == 0 && !a.stats) {
    // An output parity class that no filter tap reaches (1x1 filters with stride 2: three of the
    // four): its values are zero.  Adding zero is a no-op; otherwise fill the tiles' rows.
    if (a.accumulate) return;
    for (int t = t_begin; t < t_end; ++t) {
      int mt, nt;
      dNt.divmod(t, &mt, &nt);
      for (int idx = tid; idx < BM * (BN / 8); idx += kThreads) {
        const int row = idx / (BN / 8), ch = idx % (BN / 8);
        const int m = mt * BM + row, co = nt * BN + ch * 8;
        if (m >= M || co >= a.Cd) continue;
        int q, j, n, i;
        dWm.divmod(m, &q, &j);
        dHm.divmod(q, &n, &i);
        bf16_t* dp = a.dst + (((size_t)n * a.Hd + (i * a.os + oh)) * a.Wd + (j * a.os + ow)) * a.Cd + co;
        *reinterpret_cast<uint4*>(dp) = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    return;
  }

  const int kc = tid % KC, r0 = tid / KC;
  const __amdgpu_buffer_rsrc_t src_rs = make_rsrc(a.src, (unsigned)a.Nimg * a.Hs * a.Ws * a.Cs * 2u);
  const __amdgpu_buffer_rsrc_t wt_rs = make_rsrc(a.wt, (unsigned)a.Cd * a.T * a.Cs * 2u);
  // Per tile row of the tile being loaded: source coordinates at tap (0,0) and the byte offset of
  // that pixel; a tap adds a uniform offset and two range tests, padding is an out-of-range buffer
  // offset (reads 0).
  int a_h[A_IT], a_w[A_IT];
  unsigned a_off[A_IT];
  unsigned b_off[B_IT];
  auto set_tile = [&](int t) __attribute__((always_inline)) {
    int mt, nt;
    dNt.divmod(t, &mt, &nt);
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int m = mt * BM + r0 + it * RPP;
      if (m < M && r0 + it * RPP < BM) {
        int q, j, n, i;
        dWm.divmod(m, &q, &j);
        dHm.divmod(q, &n, &i);
        a_h[it] = i * a.ss;
        a_w[it] = j * a.ss;
        a_off[it] = (unsigned)(((n * a.Hs + a_h[it]) * a.Ws + a_w[it]) * a.Cs + kc * 8) * 2u;
      } else {
        a_h[it] = -(1 << 20); a_w[it] = 0; a_off[it] = 0;
      }
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int row = r0 + it * RPP, ch = nt * BN + row;
      b_off[it] = (row < BN && ch < a.Cd) ? (unsigned)(ch * a.T * a.Cs + kc * 8) * 2u : kOobOffset;
    }
  };
  set_tile(t_begin);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int cchunks = (a.Cs + BK - 1) / BK;
  const int nstage = ntap * cchunks;              // stages per tile
  const int total = (t_end - t_begin) * nstage;   // stages of this workgroup
  // Two stages of global loads are kept in flight in registers (sets 0 and 1) while a third one
  // is consumed from LDS: a load issued at the top of iteration s is written to LDS at the end
  // of iteration s+1.
  uint4 ra[2][A_IT], rb[2][B_IT];
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  // Loads are issued in stage order, so (tile, tap, channel chunk) of the next stage is a running
  // triple; a stage past the workgroup's last one still issues its loads, all at the out-of-range
  // offset (they return zeros without touching memory).  Unconditional loads and stores keep the
  // main loop free of divergent joins around memory operations, which lets the compiler wait for
  // exactly the oldest loads in flight.
  int ld_t = t_begin, ld_tap = 0, ld_chunk = 0;
  auto load_stage = [&](auto SET) __attribute__((always_inline)) {
    constexpr int rs = decltype(SET)::value;
    const bool live = ld_t < t_end;
    const int t = ntap ? tap0 + ld_tap : 0;
    const int c0 = ld_chunk * BK;
    const int dh = a.tt.dh[t], dw = a.tt.dw[t], wi = a.tt.widx[t];
    const bool cok = live && c0 + kc * 8 < a.Cs;               // ragged last channel chunk
    const int tap_off = ((dh * a.Ws + dw) * a.Cs + c0) * 2;   // uniform
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const bool ok = cok && (unsigned)(a_h[it] + dh) < (unsigned)a.Hs && (unsigned)(a_w[it] + dw) < (unsigned)a.Ws;
      ra[rs][it] = buffer_load16(src_rs, ok ? a_off[it] + (unsigned)tap_off : kOobOffset, 0);
    }
    const unsigned so = (unsigned)(wi * a.Cs + c0) * 2u;
#pragma unroll
    for (int it = 0; it < B_IT; ++it) rb[rs][it] = buffer_load16(wt_rs, cok ? b_off[it] : kOobOffset, so);
    if (++ld_chunk == cchunks) {
      ld_chunk = 0;
      if (++ld_tap == ntap) {
        ld_tap = 0;
        if (++ld_t < t_end) set_tile(ld_t);
      }
    }
  };
  auto store_stage = [&](int buf, auto SET) __attribute__((always_inline)) {
    constexpr int rs = decltype(SET)::value;
#pragma unroll
    for (int it = 0; it < A_IT; ++it)
      if (BM % RPP == 0 || r0 + it * RPP < BM)
        *reinterpret_cast<uint4*>(As + (buf * BM + r0 + it * RPP) * LDK + kc * 8) = ra[rs][it];
#pragma unroll
    for (int it = 0; it < B_IT; ++it)
      if (BN % RPP == 0 || r0 + it * RPP < BN)
        *reinterpret_cast<uint4*>(Bs + (buf * BN + r0 + it * RPP) * LDK + kc * 8) = rb[rs][it];
  };
  // One stage of MFMAs: the operands of 16-element slice kk+1 are read from LDS between the MFMAs
  // of slice kk (two fragment sets; the scheduling directives pin the alternation, because left
  // alone the compiler reads just in time and exposes the LDS latency once per slice).
  auto compute = [&](int cur) __attribute__((always_inline)) {
    const bf16_t* Ab = As + (cur * BM + wm * TM * 32 + (lane & 31)) * LDK + (lane >> 5) * 8;
    const bf16_t* Bb = Bs + (cur * BN + wn * TN * 32 + (lane & 31)) * LDK + (lane >> 5) * 8;
    constexpr int KK = BK / 16;
    bf16x8_t af[2][TM], bfr[2][TN];
    auto read_slice = [&](int kk, int set) {   // both constants after unrolling
#pragma unroll
      for (int i = 0; i < TM; ++i) af[set][i] = *reinterpret_cast<const bf16x8_t*>(Ab + i * 32 * LDK + kk * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[set][j] = *reinterpret_cast<const bf16x8_t*>(Bb + j * 32 * LDK + kk * 16);
    };
    read_slice(0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) read_slice(kk + 1, (kk + 1) & 1);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
      if (kk + 1 < KK) {
#pragma unroll
        for (int q = 0; q < TM * TN; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one MFMA
          if (q < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Epilogue of tile t, wave-local.  Optional per-channel sum / sum of squares of the fp32
  // accumulators over this wave's rows (rows beyond M hold zeros): one partial row per wave and
  // pixel tile, reduced by a finalising kernel.  Then 8 rows x TN*32 columns at a time through the
  // wave's LDS strip so that a lane stores 16 contiguous bytes.
  auto epilogue = [&](int t) __attribute__((always_inline)) {
    int mt, nt;
    dNt.divmod(t, &mt, &nt);
    if (a.stats) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float v = acc[i][j][r];
            s1 += v;
            s2 = fmaf(v, v, s2);
          }
        s1 += __shfl_xor(s1, 32, 64);
        s2 += __shfl_xor(s2, 32, 64);
        const int col = nt * BN + wn * TN * 32 + j * 32 + (lane & 31);
        if (lane < 32 && col < a.Cd) {
          const size_t prow = (size_t)mt * WM + wm, nrow = (size_t)a.mtiles * WM;
          a.stats[((size_t)0 * a.Cd + col) * nrow + prow] = s1;
          a.stats[((size_t)1 * a.Cd + col) * nrow + prow] = s2;
        }
      }
    }
    bf16_t* Cw = strips + wave * 8 * LDW;
    constexpr int CH = TN * 4;               // 16-byte chunks per strip row
    const int lrow = lane / CH, ch = lane % CH;
#pragma unroll
    for (int i = 0; i < TM; ++i)
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
          const int m = mt * BM + wm * TM * 32 + i * 32 + q * 8 + lrow;
          const int co = nt * BN + wn * TN * 32 + ch * 8;
          if (m < M && co < a.Cd) {
            int qq, jj, n, ii;
            dWm.divmod(m, &qq, &jj);
            dHm.divmod(qq, &n, &ii);
            bf16_t* dp = a.dst + (((size_t)n * a.Hd + (ii * a.os + oh)) * a.Wd + (jj * a.os + ow)) * a.Cd + co;
            if (a.accumulate) {
              float o[8], nw[8];
              load8(dp, o);
              load8(Cw + lrow * LDW + ch * 8, nw);
#pragma unroll
              for (int e = 0; e < 8; ++e) o[e] += nw[e];
              store8(dp, o);
            } else {
              *reinterpret_cast<uint4*>(dp) = *reinterpret_cast<const uint4*>(Cw + lrow * LDW + ch * 8);
            }
          }
        }
        asm volatile("" ::: "memory");   // ... and the next pass's writes stay behind these reads
      }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  };

  if (nstage == 0) {   // no tap at all: the tiles are zero (the accumulators are)
    for (int t = t_begin; t < t_end; ++t) epilogue(t);
    return;
  }
  int c_t = t_begin, c_stage = 0;   // tile and in-tile stage of the MFMAs
  auto tile_end = [&]() __attribute__((always_inline)) {
    if (++c_stage == nstage) {
      epilogue(c_t);
      c_stage = 0;
      ++c_t;
    }
  };
  load_stage(S0{});
  load_stage(S1{});
  store_stage(0, S0{});
  __syncthreads();
  for (int s = 0; s < total; s += 2) {
    load_stage(S0{});       // stage s + 2
    compute(0);
    store_stage(1, S1{});   // stage s + 1 (zeros past the end, into the buffer nobody reads)
    tile_end();
    __syncthreads();
    if (s + 1 >= total) break;
    load_stage(S1{});       // stage s + 3
    compute(1);
    store_stage(0, S0{});   // stage s + 2
    tile_end();
    __syncthreads();
  }
}

// wt[c][t][k] = w[k][t][c]
__global__ void __launch_bounds__(256) transpose_weights_kernel(const bf16_t* __restrict__ w,
                                                                bf16_t* __restrict__ wt, int Cout, int T,
                                                                int Cin) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= Cout * T * Cin) return;
  const int k = idx % Cout;
  const int t = (idx / Cout) % T;
  const int c = idx / (Cout * T);
  wt[idx] = w[((size_t)k * T + t) * Cin + c];
}

// dst[c][t][k] = src[k][t][c] for every tensor of the table: one workgroup per (tap, 32x32 tile),
// staged through LDS so that both the reads (along c) and the writes (along k) are contiguous.
__global__ void __launch_bounds__(256) transpose_weights_multi_kernel(TransposeTable t) {
  __shared__ bf16_t tile[32][33];
  int k = 0;
  while (k + 1 < t.count && (int)blockIdx.x >= t.block_begin[k + 1]) ++k;
  const int Cout = t.Cout[k], T = t.T[k], Cin = t.Cin[k];
  const int ct = (Cin + 31) / 32, kt = (Cout + 31) / 32;
  int b = blockIdx.x - t.block_begin[k];
  const int c0 = (b % ct) * 32; b /= ct;
  const int k0 = (b % kt) * 32;
  const int tap = b / kt;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const bf16_t* src = t.src[k];
  bf16_t* dst = t.dst[k];
  // unconditional loads (an element outside the tensor reads element 0 and is never written out),
  // so that the four are in flight together
  bf16_t v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = ty + q * 8;
    const bool ok = k0 + r < Cout && c0 + tx < Cin;
    v[q] = src[ok ? ((size_t)(k0 + r) * T + tap) * Cin + c0 + tx : (size_t)0];
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) tile[ty + q * 8][tx] = v[q];
  __syncthreads();
#pragma unroll
  for (int r = ty; r < 32; r += 8)
    if (c0 + r < Cin && k0 + tx < Cout) dst[((size_t)(c0 + r) * T + tap) * Cout + k0 + tx] = tile[tx][r];
}

// ------------------------------------------------------------------------------------------
struct WgradArgs {
  const bf16_t* x;
  const bf16_t* dy;
  float* part;  // [splits][Cout][Q]
  int N, H, W, Cin, Cout, R, S, stride, pad, Ho, Wo;
  int M;      // N*Ho*Wo
  int chunk;  // output positions per split (multiple of 64)
  int Q;      // R*S*Cin
  int qtiles;
};

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 7); }

template <int BMK, int BNQ, int WM, int WN>
__global__ void __launch_bounds__(kThreads) wgrad_kernel(WgradArgs a) {
  constexpr int BKP = 64;  // output positions per stage
  constexpr int NA = (BMK / 8) * (BKP / 8), NB = (BNQ / 8) * (BKP / 8);
  constexpr int TM = BMK / WM / 32, TN = BNQ / WN / 32;
  static_assert(NA + NB <= kThreads && WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");
  __shared__ __align__(16) bf16_t At[2][BMK * BKP];
  __shared__ __align__(16) bf16_t Bt[2][BNQ * BKP];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const int qt = blockIdx.x % a.qtiles, kt = blockIdx.x / a.qtiles;
  const int m_begin = blockIdx.y * a.chunk;
  const int m_end = min(m_begin + a.chunk, a.M);
  const int nstage = (m_end - m_begin + BKP - 1) / BKP;

  // role of this thread in the staging: one 8-position x 8-channel block of dy or of x
  const bool isA = tid < NA, isB = !isA && tid < NA + NB;
  int oct, po;  // channel octet, position octet inside the stage
  if (isA) { oct = tid % (BMK / 8); po = tid / (BMK / 8); }
  else { oct = (tid - NA) % (BNQ / 8); po = (tid - NA) / (BNQ / 8); }
  int ch0 = 0, fr = 0, fs = 0;
  bool chan_ok = false;
  if (isA) {
    ch0 = kt * BMK + oct * 8;
    chan_ok = ch0 < a.Cout;
  } else if (isB) {
    const int q0 = qt * BNQ + oct * 8;
    chan_ok = q0 < a.Q;
    const int t = q0 / a.Cin;
    ch0 = q0 % a.Cin;
    fr = t / a.S;
    fs = t % a.S;
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Every thread issues the same eight loads every stage; rows that do not exist (past the split's
  // range, padding, a thread without a staging role) use the out-of-range buffer offset, which
  // returns zeros without touching memory.  Straight-line loads let the compiler wait for exactly
  // the loads it needs instead of draining the queue at every divergent join.
  const __amdgpu_buffer_rsrc_t dy_rs = make_rsrc(a.dy, (unsigned)a.M * a.Cout * 2u);
  const __amdgpu_buffer_rsrc_t x_rs = make_rsrc(a.x, (unsigned)a.N * a.H * a.W * a.Cin * 2u);
  uint4 rg[8];
  auto load_stage = [&](int s) __attribute__((always_inline)) {
    const int m0 = m_begin + s * BKP + po * 8;
    if (isA) {
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const bool ok = chan_ok && m0 + p < m_end;
        rg[p] = buffer_load16(dy_rs, ok ? (unsigned)((m0 + p) * a.Cout + ch0) * 2u : kOobOffset, 0);
      }
    } else {
      int wo = m0 % a.Wo, q = m0 / a.Wo;
      int ho = q % a.Ho, n = q / a.Ho;
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const int hi = ho * a.stride + fr - a.pad, wi = wo * a.stride + fs - a.pad;
        const bool ok = isB && chan_ok && m0 + p < m_end && (unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W;
        rg[p] = buffer_load16(x_rs, ok ? (unsigned)(((n * a.H + hi) * a.W + wi) * a.Cin + ch0) * 2u : kOobOffset, 0);
        if (++wo == a.Wo) { wo = 0; if (++ho == a.Ho) { ho = 0; ++n; } }
      }
    }
  };
  auto store_stage = [&](int buf) __attribute__((always_inline)) {
    if (!(isA || isB)) return;
    bf16_t* T_ = isA ? At[buf] : Bt[buf];
    const unsigned* rw = reinterpret_cast<const unsigned*>(rg);
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) {
      uint4 lo, hi;
      unsigned* lw = reinterpret_cast<unsigned*>(&lo);
      unsigned* hw = reinterpret_cast<unsigned*>(&hi);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const unsigned e = rw[(2 * j) * 4 + c2], o = rw[(2 * j + 1) * 4 + c2];
        lw[j] = (e & 0xffffu) | (o << 16);
        hw[j] = (e >> 16) | (o & 0xffff0000u);
      }
      const int rl = oct * 8 + 2 * c2, rh = rl + 1;
      *reinterpret_cast<uint4*>(T_ + rl * BKP + ((po ^ swz(rl)) << 3)) = lo;
      *reinterpret_cast<uint4*>(T_ + rh * BKP + ((po ^ swz(rh)) << 3)) = hi;
    }
  };
  // One stage of MFMAs: the operands of 16-position slice kk+1 are read from LDS between the MFMAs
  // of slice kk (two fragment sets, alternation pinned by the scheduling directives).
  auto compute = [&](int cur) __attribute__((always_inline)) {
    constexpr int KK = BKP / 16;
    bf16x8_t af[2][TM], bfr[2][TN];
    auto read_slice = [&](int kk, int set) {
      const int chunk = kk * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm * TM * 32 + i * 32 + (lane & 31);
        af[set][i] = *reinterpret_cast<const bf16x8_t*>(At[cur] + row * BKP + ((chunk ^ swz(row)) << 3));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int row = wn * TN * 32 + j * 32 + (lane & 31);
        bfr[set][j] = *reinterpret_cast<const bf16x8_t*>(Bt[cur] + row * BKP + ((chunk ^ swz(row)) << 3));
      }
    };
    read_slice(0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk + 1 < KK) read_slice(kk + 1, (kk + 1) & 1);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
      if (kk + 1 < KK) {
#pragma unroll
        for (int q = 0; q < TM * TN; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one MFMA
          if (q < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  load_stage(0);
  store_stage(0);
  __syncthreads();
  for (int s = 0; s < nstage; ++s) {
    const int cur = s & 1;
    load_stage(s + 1);        // past the last stage: zeros into the buffer nobody reads
    compute(cur);
    store_stage(cur ^ 1);
    __syncthreads();
  }

  float* out = a.part + (size_t)blockIdx.y * a.Cout * a.Q;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = kt * BMK + wm * TM * 32 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int col = qt * BNQ + wn * TN * 32 + j * 32 + (lane & 31);
        if (row < a.Cout && col < a.Q) out[(size_t)row * a.Q + col] = acc[i][j][r];
      }
}

// ---------------------------------------------------------------------------- host side ----
struct IgemmPlan {
  int bm, bn, bk;
};

// Tile choice.  g_cnnk_tune[0..2] (set through cnnk_tune) force BM / BN / BK for experiments.
IgemmPlan plan_igemm(long maxM, int Cd, int Cs) {
  IgemmPlan p;
  // Measured on MI355X (ResNet-18 b256 shapes): the kernels are bound by L2->CU traffic, so the
  // largest tile that still gives every CU two workgroups wins; small-M layers prefer 64x64.
  const long b128 = ((maxM + 127) / 128) * ((Cd + 127) / 128);
  if (Cd <= 64) { p.bm = 128; p.bn = 64; }
  else if (b128 >= 512) { p.bm = 128; p.bn = 128; }
  else { p.bm = 64; p.bn = 64; }
  if (g_cnnk_tune[0] > 0) p.bm = g_cnnk_tune[0];
  if (g_cnnk_tune[1] > 0) p.bn = g_cnnk_tune[1];
  p.bk = (Cs % 64 == 0) ? 64 : (Cs % 32 == 0) ? 32 : 16;
  if (p.bk == 64 && (p.bm + p.bn) > 256) p.bk = 32;   // keep two workgroups per CU in LDS
  if (p.bk == 64 && p.bm == 128 && p.bn == 64) p.bk = 32;   // three or four instead of two (64-channel outputs: 38 -> 33 us)
  if (g_cnnk_tune[2] > 0 && g_cnnk_tune[2] <= p.bk) p.bk = g_cnnk_tune[2];
  return p;
}

template <int BM, int BN, int BK, int WM, int WN, int OCC>
int launch_igemm(const IgemmArgs& a, long maxM, hipStream_t st) {
  constexpr int TN = BN / WN / 32;
  constexpr size_t stage_bytes = (size_t)2 * (BM + BN) * (BK + 8) * sizeof(bf16_t);
  constexpr size_t strip_bytes = (size_t)4 * 8 * (TN * 32 + 8) * sizeof(bf16_t);
  constexpr size_t smem = stage_bytes + strip_bytes;
  static_assert(smem <= 160 * 1024, "LDS budget");
  static bool attr_done = false;
  auto kern = igemm_kernel<BM, BN, BK, WM, WN, OCC>;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)smem) != hipSuccess)
      return CNNK_ERR_HIP;
    attr_done = true;
  }
  IgemmArgs b = a;
  b.ntiles = (a.Cd + BN - 1) / BN;
  const long mtiles = (maxM + BM - 1) / BM;
  b.mtiles = (int)mtiles;
  b.dNt.init((unsigned)b.ntiles);
  for (int c = 0; c < a.tt.nclass; ++c) {
    b.tt.dW[c].init((unsigned)a.tt.Wm[c]);
    b.tt.dH[c].init((unsigned)a.tt.Hm[c]);
  }
  // Tiles per workgroup: as many as still leave every CU its OCC workgroups (tune key 14 overrides).
  const long tiles = mtiles * b.ntiles;
  int tpb = 1;
  for (int t = 8; t > 1; t >>= 1)
    if ((tiles + t - 1) / t >= 256L * OCC) { tpb = t; break; }
  if (g_cnnk_tune[14] > 0) tpb = g_cnnk_tune[14];
  b.tpb = tpb;
  dim3 grid((unsigned)((tiles + tpb - 1) / tpb), a.tt.nclass);
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), smem, st, b);
  return launch_status();
}

// wavefront rows (WM) of the tile shape the dispatch below picks for a plan
int igemm_wm(const IgemmPlan& p) { return p.bn == 64 && p.bm >= 128 ? 4 : 2; }

int dispatch_igemm(const IgemmArgs& a, long maxM, const IgemmPlan& p, hipStream_t st) {
#define CNNK_IGEMM_CASE(BM, BN, WM, WN, OCC)                                         \
  if (p.bm == BM && p.bn == BN) {                                                    \
    if (p.bk == 64 && BM + BN <= 256) return launch_igemm<BM, BN, (BM + BN <= 256 ? 64 : 32), WM, WN, OCC>(a, maxM, st); \
    if (p.bk >= 32) return launch_igemm<BM, BN, 32, WM, WN, OCC>(a, maxM, st);       \
    return launch_igemm<BM, BN, 16, WM, WN, OCC>(a, maxM, st);                       \
  }
  CNNK_IGEMM_CASE(256, 128, 2, 2, 2)
  CNNK_IGEMM_CASE(128, 128, 2, 2, 2)
  CNNK_IGEMM_CASE(256, 64, 4, 1, 2)
  CNNK_IGEMM_CASE(128, 64, 4, 1, 3)
  CNNK_IGEMM_CASE(64, 64, 2, 2, 4)
#undef CNNK_IGEMM_CASE
  return CNNK_ERR_UNSUPPORTED;
}

void wgrad_plan(const ConvGeom& g, int* bmk, int* chunk, int* splits, int cus = 256) {
  const int Q = g.R * g.S * g.Cin;
  const long M = (long)g.N * g.Ho * g.Wo;
  *bmk = g.Cout > 64 ? 128 : 64;
  const long tiles = (long)((g.Cout + *bmk - 1) / *bmk) * ((Q + 127) / 128);
  const long target = g_cnnk_tune[3] > 0 ? g_cnnk_tune[3] : 3L * cus / (g.Cout <= 64 ? 1 : 2);   // 768 / 384 workgroups on the whole device
  long want = (target + tiles - 1) / tiles;
  const long maxs = (M + 255) / 256;
  if (want > maxs) want = maxs;
  if (want < 1) want = 1;
  long ch = (M + want - 1) / want;
  ch = (ch + 63) / 64 * 64;
  *chunk = (int)ch;
  *splits = (int)((M + ch - 1) / ch);
}

}  // namespace

bool conv_mfma_supported(const ConvGeom& g, int pass) {
  (void)pass;
  if (g.Cin % 8 != 0 || g.Cout % 8 != 0) return false;
  if (g.R != g.S || (g.R != 1 && g.R != 3)) return false;
  if (g.stride < 1 || g.stride > 2) return false;
  // 32-bit element offsets inside the kernels
  // byte offsets of the buffer loads must stay below their out-of-bounds marker (2 GiB)
  const long e_in = (long)g.N * g.H * g.W * g.Cin, e_out = (long)g.N * g.Ho * g.Wo * g.Cout;
  if (e_in >= (1L << 30) || e_out >= (1L << 30) || (long)g.Cout * g.R * g.S * g.Cin >= (1L << 30)) return false;
  return true;
}

size_t conv_mfma_ws(const ConvGeom& g, int pass, bool want_stats) {
  if (pass == CNNK_PASS_FWD)   // statistics partials: one row per wavefront and pixel tile, at the finest 32 pixels
                               // each; the last pixel tile is padded to whole wavefront rows (at most 8 of them)
    return want_stats ? align_up((((size_t)g.N * g.Ho * g.Wo + 31) / 32 + 8) * 2 * g.Cout * sizeof(float), 256) : 0;
  if (pass == CNNK_PASS_DGRAD) return align_up((size_t)g.Cout * g.R * g.S * g.Cin * sizeof(bf16_t), 256);
  if (pass == CNNK_PASS_WGRAD) {
    if (conv_wgrad_patch_supported(g)) return conv_wgrad_patch_ws(g);
    int bmk, chunk, splits;
    wgrad_plan(g, &bmk, &chunk, &splits);
    return splits > 1 ? (size_t)splits * g.Cout * g.R * g.S * g.Cin * sizeof(float) : 0;
  }
  return 0;
}

int conv_mfma_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* ch_sum,
                  float* ch_sumsq, void* ws, hipStream_t st) {
  if (conv_patch_supported(g, CNNK_PASS_FWD)) {
    float* stats = ch_sum ? reinterpret_cast<float*>(ws) : nullptr;
    int rc = conv_patch_fwd(g, x, w, y, stats, st);
    if (rc != CNNK_OK || !ch_sum) return rc;
    return channel_sums_finalize(stats, conv_patch_stat_rows(g), g.Cout, ch_sum, ch_sumsq, st);
  }
  IgemmArgs a{};
  a.src = x; a.wt = w; a.dst = y;
  a.stats = ch_sum ? reinterpret_cast<float*>(ws) : nullptr;
  a.Nimg = g.N; a.Hs = g.H; a.Ws = g.W; a.Cs = g.Cin;
  a.Hd = g.Ho; a.Wd = g.Wo; a.Cd = g.Cout;
  a.T = g.R * g.S; a.ss = g.stride; a.os = 1; a.accumulate = 0;
  a.tt.nclass = 1;
  a.tt.cls_begin[0] = 0; a.tt.cls_begin[1] = g.R * g.S;
  for (int r = 0; r < g.R; ++r)
    for (int s = 0; s < g.S; ++s) {
      const int t = r * g.S + s;
      a.tt.dh[t] = r - g.pad; a.tt.dw[t] = s - g.pad; a.tt.widx[t] = t;
    }
  a.tt.Hm[0] = g.Ho; a.tt.Wm[0] = g.Wo; a.tt.oh[0] = 0; a.tt.ow[0] = 0;
  const long M = (long)g.N * g.Ho * g.Wo;
  const IgemmPlan p = plan_igemm(M, a.Cd, a.Cs);
  int rc = dispatch_igemm(a, M, p, st);
  if (rc != CNNK_OK || !ch_sum) return rc;
  return channel_sums_finalize(a.stats, (int)((M + p.bm - 1) / p.bm) * igemm_wm(p), g.Cout, ch_sum, ch_sumsq, st);
}

int conv_transpose_weights_multi(TransposeTable& t, hipStream_t st) {
  int blocks = 0;
  for (int k = 0; k < t.count; ++k) {
    t.block_begin[k] = blocks;
    blocks += t.T[k] * ((t.Cout[k] + 31) / 32) * ((t.Cin[k] + 31) / 32);
  }
  t.block_begin[t.count] = blocks;
  if (blocks == 0) return CNNK_OK;
  transpose_weights_multi_kernel<<<blocks, 256, 0, st>>>(t);
  return launch_status();
}

int conv_mfma_dgrad(const ConvGeom& g, const bf16_t* dy, const bf16_t* w, bf16_t* dx, int accumulate,
                    void* ws, hipStream_t st) {
  const int T = g.R * g.S;
  bf16_t* wt = reinterpret_cast<bf16_t*>(ws);
  const int nw = g.Cout * T * g.Cin;
  transpose_weights_kernel<<<(nw + 255) / 256, 256, 0, st>>>(w, wt, g.Cout, T, g.Cin);
  if (launch_status() != CNNK_OK) return CNNK_ERR_HIP;
  return conv_mfma_dgrad_pt(g, dy, wt, dx, accumulate, st);
}

// wt: weights already transposed to [Cin][R*S][Cout]
int conv_mfma_dgrad_pt(const ConvGeom& g, const bf16_t* dy, const bf16_t* wt, bf16_t* dx, int accumulate,
                       hipStream_t st) {
  const int T = g.R * g.S;
  if (conv_patch_supported(g, CNNK_PASS_DGRAD)) return conv_patch_dgrad(g, dy, wt, dx, accumulate, st);
  IgemmArgs a{};
  a.src = dy; a.wt = wt; a.dst = dx;
  a.Nimg = g.N; a.Hs = g.Ho; a.Ws = g.Wo; a.Cs = g.Cout;
  a.Hd = g.H; a.Wd = g.W; a.Cd = g.Cin;
  a.T = T; a.ss = 1; a.os = g.stride; a.accumulate = accumulate;
  const int st_ = g.stride;
  int ncls = 0, ntap = 0;
  long maxM = 0;
  for (int eh = 0; eh < st_; ++eh)
    for (int ew = 0; ew < st_; ++ew) {
      a.tt.cls_begin[ncls] = ntap;
      for (int r = 0; r < g.R; ++r) {
        const int th = eh + g.pad - r;
        if (((th % st_) + st_) % st_ != 0) continue;
        for (int s = 0; s < g.S; ++s) {
          const int tw = ew + g.pad - s;
          if (((tw % st_) + st_) % st_ != 0) continue;
          // exact quotients (th, tw are multiples of the stride, possibly negative)
          a.tt.dh[ntap] = th / st_; a.tt.dw[ntap] = tw / st_; a.tt.widx[ntap] = r * g.S + s;
          ++ntap;
        }
      }
      a.tt.Hm[ncls] = (g.H - eh + st_ - 1) / st_;
      a.tt.Wm[ncls] = (g.W - ew + st_ - 1) / st_;
      a.tt.oh[ncls] = eh; a.tt.ow[ncls] = ew;
      const long m = (long)g.N * a.tt.Hm[ncls] * a.tt.Wm[ncls];
      if (m > maxM) maxM = m;
      ++ncls;
    }
  a.tt.cls_begin[ncls] = ntap;
  a.tt.nclass = ncls;
  return dispatch_igemm(a, maxM, plan_igemm(maxM, a.Cd, a.Cs), st);
}

int conv_mfma_wgrad_partials(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws,
                             const float** part, int* P, hipStream_t st) {
  if (conv_wgrad_patch_supported(g)) {
    *part = dw;
    *P = 1;
    return conv_wgrad_patch(g, x, dy, dw, ws, st);
  }
  int bmk, chunk, splits;
  wgrad_plan(g, &bmk, &chunk, &splits, t_cnnk_wgrad_cus);
  WgradArgs a{};
  a.x = x; a.dy = dy;
  a.part = splits > 1 ? reinterpret_cast<float*>(ws) : dw;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.Cout = g.Cout; a.R = g.R; a.S = g.S;
  a.stride = g.stride; a.pad = g.pad; a.Ho = g.Ho; a.Wo = g.Wo;
  a.M = g.N * g.Ho * g.Wo; a.chunk = chunk; a.Q = g.R * g.S * g.Cin;
  a.qtiles = (a.Q + 127) / 128;
  const int ktiles = (g.Cout + bmk - 1) / bmk;
  dim3 grid(ktiles * a.qtiles, splits);
  if (bmk == 128) hipLaunchKernelGGL((wgrad_kernel<128, 128, 2, 2>), grid, dim3(kThreads), 0, st, a);
  else hipLaunchKernelGGL((wgrad_kernel<64, 128, 1, 4>), grid, dim3(kThreads), 0, st, a);
  *part = a.part;
  *P = splits;
  return launch_status();
}

int conv_mfma_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws,
                    hipStream_t st) {
  const float* part = nullptr;
  int P = 0;
  const int rc = conv_mfma_wgrad_partials(g, x, dy, dw, ws, &part, &P, st);
  if (rc != CNNK_OK || P <= 1) return rc;
  return reduce_partials(part, dw, g.Cout * g.R * g.S * g.Cin, P, st);
}
