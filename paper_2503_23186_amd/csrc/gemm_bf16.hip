// Dense bf16 matrix products of the Vision Transformer step's linear layers on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): y = x W^T (+ bias, + GELU), dx = dy W,
// dW = dy^T x.  One kernel, three operand orientations.
//
// Workgroup tile 256 x 128 (or 192 x 128), four wavefronts of 128 x 64 (0.75 KB of LDS operand reads per MFMA), 32
// reduction elements per stage, three LDS stage buffers filled straight from memory
// (buffer_load ... lds, issued two stages ahead; out-of-range rows deposit zeros), one barrier per
// stage, two workgroups per CU.  An operand whose reduction index is its contiguous one ("natural":
// x and W of the forward product, dy of the data gradient) lies in LDS as [row][32 reduction
// elements] and is read with 16-byte loads; an operand whose reduction index is its row index (W of
// the data gradient, both operands of the weight gradient) lies as planes of [32 reduction
// rows][32 columns] and is read with the transposing load ds_read_b64_tr_b16, so no operand is ever
// transposed in memory.  Rows are 64 bytes with the 16-byte chunks XOR-swizzled by row bits 2-3: both
// kinds of read touch every bank once per pass.  Because the hardware fixes where a direct load's
// bytes land (lane i at base + 16 i), the layout is produced by which global bytes each lane asks for.
// Epilogue per wavefront through a private LDS strip (accumulator quads in, transposing reads out):
// 16-byte stores of 8 consecutive columns; bias and GELU are applied to the fp32 accumulator first, so
// an output is rounded once.  The weight gradient splits the row range over blockIdx.z and writes
// fp32 partials that a second kernel adds in a fixed order.
#include "common.h"
#include "gemm.h"

namespace {
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

constexpr int BN = 128, BK = 32, NST = 3;
constexpr int B_BYTES = BN * BK * 2;
constexpr int kThreads = 256;
// TM: 32-row blocks of a wavefront's tile (4: workgroup tile 256 x 128, 3: 192 x 128, for shapes whose
// tile count at 256 rows leaves much of the device idle in the last round of resident workgroups)
template <int TM> struct Cfg {
  static constexpr int BM = 64 * TM, A_BYTES = BM * BK * 2, STAGE_B = A_BYTES + B_BYTES;
  static constexpr int NLOAD = STAGE_B / 1024 / 4;      // direct loads per wavefront and stage (TM + 2)
};
constexpr int SP = 72;                         // epilogue strip pitch (bytes per column)

__device__ __forceinline__ i32x4_t make_desc(const void* p, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(p);
  return i32x4_t{(int)(unsigned)a, (int)((unsigned)(a >> 32) & 0xffffu), (int)bytes, 0x00020000};
}
// lane i of the wavefront moves 16 bytes from byte offset voff of the buffer to LDS address
// lds_addr + 16 i (zeros when voff is out of range).  Assembly, so that the compiler does not make
// every later LDS read wait for all outstanding direct loads; the waits are explicit below.
__device__ __forceinline__ void load16_to_lds(i32x4_t desc, unsigned lds_addr, unsigned voff) {
  unsigned keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
               : "=&s"(keep)
               : "s"(lds_addr), "v"(voff), "s"(desc)
               : "memory");
}
__device__ __forceinline__ int swz(int row, int c16) { return row * 64 + ((c16 ^ ((row >> 2) & 3)) << 4); }

struct Args {
  const bf16_t* A;
  const bf16_t* B;
  bf16_t* C;          // bf16 output [M][N] (EPI 0, 1)
  bf16_t* C2;         // EPI 1: gelu(C)
  float* part;        // EPI 2: fp32 partials [splits][M][N]
  const float* bias;  // [N] or null
  const bf16_t* res;  // EPI 3: [M][N] added to the rounded output (a residual connection)
  int M, N, K;        // output rows, output columns, reduction length
  int lda, ldb, ldc;
  int k_per_split;    // reduction elements per blockIdx.z (a multiple of BK)
  int mtiles, ntiles;
  unsigned a_bytes, b_bytes;
};

// gelu(u) = u Phi(u) with the complementary error function from the rational approximation 7.1.26 of
// Abramowitz & Stegun (absolute error of erf below 1.5e-7, far below a bf16 output's rounding): one
// reciprocal, one exponential and five multiply-adds, branch-free.  With q = erfc(|u| / sqrt 2) / 2:
// gelu(u) = u (1 - q) for u >= 0 and u q for u < 0.
__device__ __forceinline__ float gelu_f(float u) {
  const float x = fabsf(u) * 0.70710678118654752f;
  const float t = __frcp_rn(1.0f + 0.3275911f * x);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float q = 0.5f * poly * __expf(-x * x);
  return u >= 0.f ? u - u * q : u * q;
}

template <bool ATR, bool BTR, int EPI, int TM>
__global__ void __launch_bounds__(kThreads, 2) gemm_kernel(Args a) {
  constexpr int BM = Cfg<TM>::BM, A_BYTES = Cfg<TM>::A_BYTES, STAGE_B = Cfg<TM>::STAGE_B, NLOAD = Cfg<TM>::NLOAD;
  extern __shared__ __align__(16) unsigned char smem[];   // NST stage buffers, nothing else: LDS address 0
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1, h = lane >> 5, g = lane >> 4, i16 = lane & 15;
  // workgroups that share an XCD's L2 (every 8th) walk consecutive tiles: same rows of A, all of B
  // (the grid is 8 * ceil(tiles / 8) workgroups; the few past the end leave at once).  An XCD owns a
  // contiguous range of the row-major tile list, i.e. a band of tile rows, and walks it column by
  // column: the workgroups in flight on it then share the band's rows of A, which stay in its L2,
  // while B streams through once per XCD.
  const int ntot = a.mtiles * a.ntiles, chunk = (ntot + 7) >> 3;
  const int c0 = (blockIdx.x & 7) * chunk, c1 = min(c0 + chunk, ntot);
  int l = blockIdx.x >> 3;
  if (c0 + l >= c1) return;
  const int r0 = c0 / a.ntiles, s0 = c0 - r0 * a.ntiles, r1 = (c1 - 1) / a.ntiles, e1 = (c1 - 1) - r1 * a.ntiles + 1;
  int mt = r0, nt = 0;
  for (; nt < a.ntiles; ++nt) {
    const int first = nt >= s0 ? 1 : 0;                 // the band's first row has this column
    const int cnt = r0 == r1 ? ((nt >= s0 && nt < e1) ? 1 : 0) : (r1 - r0 - 1) + first + (nt < e1 ? 1 : 0);
    if (l < cnt) { mt = r0 + l + (1 - first); break; }
    l -= cnt;
  }
  const int m0 = mt * BM, n0 = nt * BN;
  const int kbeg = blockIdx.z * a.k_per_split;
  int kend = kbeg + a.k_per_split;
  if (kend > a.K) kend = a.K;
  const int nst = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;

  const i32x4_t a_rs = make_desc(a.A, a.a_bytes), b_rs = make_desc(a.B, a.b_bytes);
  // ---- this lane's six direct loads of a stage ----
  // kk0: reduction index of the lane's 16 bytes in stage 0 (its first element for a natural operand,
  // its row for a transposed one); a load of stage t is in range while kk0 + t * BK < kend
  unsigned voff[NLOAD], vinc[NLOAD];
  int ldsoff[NLOAD], kk0[NLOAD];
  bool isA[NLOAD];
#pragma unroll
  for (int j = 0; j < NLOAD; ++j) {
    const int q = j * 4 + wave;
    isA[j] = q < A_BYTES / 1024;
    const int qq = isA[j] ? q : q - A_BYTES / 1024;
    const bool tr = isA[j] ? ATR : BTR;
    const int ld = isA[j] ? a.lda : a.ldb;
    const int o0 = isA[j] ? m0 : n0, olim = isA[j] ? a.M : a.N;
    ldsoff[j] = (isA[j] ? 0 : A_BYTES) + qq * 1024;
    const int cp = lane & 3;
    if (!tr) {
      const int r = qq * 16 + (lane >> 2);
      const int c = cp ^ ((r >> 2) & 3);
      const int row = o0 + r;
      kk0[j] = row < olim ? kbeg + 8 * c : (1 << 30);
      voff[j] = (unsigned)((row * ld + kbeg + 8 * c) * 2);
      vinc[j] = BK * 2;
    } else {
      const int plane = qq >> 1, r = (qq & 1) * 16 + (lane >> 2);
      const int c = cp ^ ((r >> 2) & 3);
      const int col = o0 + plane * 32 + 8 * c;
      kk0[j] = col < olim ? kbeg + r : (1 << 30);
      voff[j] = (unsigned)(((kbeg + r) * ld + col) * 2);
      vinc[j] = (unsigned)(BK * ld * 2);
    }
  }
  auto issue = [&](int t, int sb) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
      const unsigned off = kk0[j] + t * BK < kend ? voff[j] + (unsigned)t * vinc[j] : kOobOffset;
      load16_to_lds(isA[j] ? a_rs : b_rs, (unsigned)(sb + ldsoff[j]), off);
    }
  };
  // ---- fragment addresses (stage-relative) ----
  int aoff[2][2], boff[2][2];     // [reduction step of the stage][first / second read of a transposing pair]
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    if (!ATR) {
      const int row = wm * (TM * 32) + (lane & 31);
      aoff[ks][0] = swz(row, ks * 2 + h);
      aoff[ks][1] = 0;
    } else {
      const int ch0 = (g & 1) * 16 + (i16 & 3) * 4, row = ks * 16 + h * 8 + (i16 >> 2);
      aoff[ks][0] = wm * TM * 2048 + swz(row, ch0 >> 3) + (ch0 & 7) * 2;
      aoff[ks][1] = wm * TM * 2048 + swz(row + 4, ch0 >> 3) + (ch0 & 7) * 2;
    }
    if (!BTR) {
      const int row = wn * 64 + (lane & 31);
      boff[ks][0] = A_BYTES + swz(row, ks * 2 + h);
      boff[ks][1] = 0;
    } else {
      const int ch0 = (g & 1) * 16 + (i16 & 3) * 4, row = ks * 16 + h * 8 + (i16 >> 2);
      boff[ks][0] = A_BYTES + wn * 2 * 2048 + swz(row, ch0 >> 3) + (ch0 & 7) * 2;
      boff[ks][1] = A_BYTES + wn * 2 * 2048 + swz(row + 4, ch0 >> 3) + (ch0 & 7) * 2;
    }
  }
  auto read_frag = [&](const unsigned char* sb, bool tr, int o0, int o1, int sub) __attribute__((always_inline)) -> bf16x8_t {
    // sub: 32-row (natural) or 32-column (transposing) block of the wave's tile: both 2048 bytes apart
    if (!tr) return *reinterpret_cast<const bf16x8_t*>(sb + o0 + sub * 2048);
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(sb + o0 + sub * 2048));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(sb + o1 + sub * 2048));
    const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  };

  f32x16_t acc[TM][2];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (nst > 0) issue(0, 0);
  if (nst > 1) issue(1, STAGE_B);
  int cur = 0;
  for (int t = 0; t < nst; ++t) {
    if (t + 1 < nst) __builtin_amdgcn_s_waitcnt(0x0f70 | NLOAD);   // this wave's loads of stage t have landed
    else __builtin_amdgcn_s_waitcnt(0x0f70);
    __builtin_amdgcn_s_barrier();
    if (t + 2 < nst) {
      int fill = cur + 2 * STAGE_B;
      if (fill >= NST * STAGE_B) fill -= NST * STAGE_B;
      issue(t + 2, fill);
    }
    const unsigned char* sb = smem + cur;
    bf16x8_t af[2][TM], bfr[2][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i) af[ks][i] = read_frag(sb, ATR, aoff[ks][0], aoff[ks][1], i);
#pragma unroll
      for (int j = 0; j < 2; ++j) bfr[ks][j] = read_frag(sb, BTR, boff[ks][0], boff[ks][1], j);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
    cur += STAGE_B;
    if (cur == NST * STAGE_B) cur = 0;
  }

  if (EPI == 2) {
    float* out = a.part + (size_t)blockIdx.z * a.M * a.ldc;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wm * (TM * 32) + i * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
          if (row < a.M && col < a.N) out[(size_t)row * a.ldc + col] = acc[i][j][r];
        }
      }
    return;
  }
  __syncthreads();     // every wave is done reading the stage buffers; all direct loads have landed (vmcnt(0) above)
  unsigned char* S = smem + wave * (32 * SP);
  const int wr_off = (lane & 31) * SP + h * 8;
  const int rd_off = (g * 8 + (i16 >> 2)) * SP + (i16 & 3) * 8;
  auto transpose_store = [&](const float* v, bf16_t* dst, int i, int j) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<uint2*>(S + wr_off + q * 16) = make_uint2(pack_bf16x2(v[q * 4], v[q * 4 + 1]), pack_bf16x2(v[q * 4 + 2], v[q * 4 + 3]));
    asm volatile("" ::: "memory");
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(S + rd_off + rb * 32));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(S + rd_off + 4 * SP + rb * 32));
      const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
      const int row = m0 + wm * (TM * 32) + i * 32 + rb * 16 + i16, col = n0 + wn * 64 + j * 32 + g * 8;
      if (row < a.M && col < a.N) {
        uint4 out = uint4{l2.x, l2.y, h2.x, h2.y};
        if (EPI == 3) {     // + residual: the sum of two stored values, rounded again
          float x[8], r[8];
          unpack8(out, x);
          load8(a.res + (size_t)row * a.ldc + col, r);
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] += r[e];
          out = uint4{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
        }
        *reinterpret_cast<uint4*>(dst + (size_t)row * a.ldc + col) = out;
      }
    }
    asm volatile("" ::: "memory");
  };
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int colv = n0 + wn * 64 + j * 32 + (lane & 31);
      const float bv = (a.bias && colv < a.N) ? a.bias[colv] : 0.f;
      float v[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = acc[i][j][r] + bv;
      transpose_store(v, a.C, i, j);
      if (EPI == 1) {
        // the activation of the value as stored
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = gelu_f(bf16_to_f32(f32_to_bf16_hw(v[r])));
        transpose_store(v, a.C2, i, j);
      }
    }
}

// out[i] = sum over splits (ascending) of part[z][i]; n a multiple of 4
__global__ void __launch_bounds__(256) sum_partials_kernel(const float* __restrict__ part, int splits, size_t n,
                                                           float* __restrict__ out) {
  for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += (size_t)gridDim.x * 1024) {
    float4 s = *reinterpret_cast<const float4*>(part + i);
    for (int z = 1; z < splits; ++z) {
      const float4 p = *reinterpret_cast<const float4*>(part + (size_t)z * n + i);
      s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    *reinterpret_cast<float4*>(out + i) = s;
  }
}

template <typename Kern>
int launch(Kern kern, bool* raised, int stage_b, const Args& a, int splits, hipStream_t st) {
  if (!*raised) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, NST * stage_b) != hipSuccess)
      return CNNK_ERR_HIP;
    *raised = true;
  }
  hipLaunchKernelGGL(kern, dim3(8 * ((a.mtiles * a.ntiles + 7) / 8), 1, splits), dim3(kThreads), NST * stage_b, st, a);
  return launch_status();
}
// one launch of the orientation / epilogue at either tile height
template <bool ATR, bool BTR, int EPI>
int launch_tm(int tm, Args& a, int out_rows, int splits, hipStream_t st) {
  static bool r4 = false, r3 = false;
  a.mtiles = (out_rows + 64 * tm - 1) / (64 * tm);
  if (tm == 3) return launch(gemm_kernel<ATR, BTR, EPI, 3>, &r3, Cfg<3>::STAGE_B, a, splits, st);
  return launch(gemm_kernel<ATR, BTR, EPI, 4>, &r4, Cfg<4>::STAGE_B, a, splits, st);
}
// Rows per workgroup tile (in 64s): the device holds 512 workgroups at once; the cost of a launch is
// about (rounds of resident workgroups) x (tile height).
int pick_tm(int out_rows, int ntiles) {
  auto cost = [&](int tm) { const int t = ((out_rows + 64 * tm - 1) / (64 * tm)) * ntiles; return ((t + 511) / 512) * tm; };
  return cost(3) < cost(4) ? 3 : 4;
}

bool fits32(long long rows, long long cols) { return rows * cols * 2 < 2147483647LL; }
int wgrad_splits(int rows, int tiles) {
  int s = (192 + tiles - 1) / tiles;           // workgroups of a launch: it runs beside the main stream's kernels (128-192 measured best)
  const int max_s = rows / (8 * BK);           // at least 8 stages each
  if (s > max_s) s = max_s;
  return s < 1 ? 1 : s;
}
}  // namespace

bool gemm_bf16_supported(long long rows, int K, int N) {
  return rows > 0 && K > 0 && N > 0 && K % 8 == 0 && N % 8 == 0 && fits32(rows, K) && fits32(rows, N) && fits32(N, K);
}

int gemm_bf16_fwd(long long rows, int K, int N, const bf16_t* x, const bf16_t* w, const float* bias, const bf16_t* res, bool gelu,
                  bf16_t* u, bf16_t* y, hipStream_t st) {
  Args a{};
  a.A = x; a.B = w; a.bias = bias; a.res = res;
  a.C = gelu ? u : y; a.C2 = gelu ? y : nullptr;
  a.M = (int)rows; a.N = N; a.K = K; a.lda = K; a.ldb = K; a.ldc = N; a.k_per_split = K;
  a.ntiles = (N + BN - 1) / BN;
  a.a_bytes = (unsigned)(rows * K * 2); a.b_bytes = (unsigned)((long long)N * K * 2);
  const int tm = pick_tm(a.M, a.ntiles);
  if (res) return launch_tm<false, false, 3>(tm, a, a.M, 1, st);
  return gelu ? launch_tm<false, false, 1>(tm, a, a.M, 1, st) : launch_tm<false, false, 0>(tm, a, a.M, 1, st);
}

int gemm_bf16_dgrad(long long rows, int K, int N, const bf16_t* dy, const bf16_t* w, bf16_t* dx, hipStream_t st) {
  Args a{};
  a.A = dy; a.B = w; a.C = dx;
  a.M = (int)rows; a.N = K; a.K = N; a.lda = N; a.ldb = K; a.ldc = K; a.k_per_split = N;
  a.ntiles = (K + BN - 1) / BN;
  a.a_bytes = (unsigned)(rows * N * 2); a.b_bytes = (unsigned)((long long)N * K * 2);
  return launch_tm<false, true, 0>(pick_tm(a.M, a.ntiles), a, a.M, 1, st);
}

size_t gemm_bf16_wgrad_ws(long long rows, int K, int N) {
  const int tiles = ((N + 255) / 256) * ((K + BN - 1) / BN);
  const int s = wgrad_splits((int)rows, tiles);
  return s > 1 ? (size_t)s * N * K * sizeof(float) : 0;
}

int gemm_bf16_wgrad(long long rows, int K, int N, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st) {
  Args a{};
  a.A = dy; a.B = x;
  a.M = N; a.N = K; a.K = (int)rows; a.lda = N; a.ldb = K; a.ldc = K;
  a.mtiles = (N + 255) / 256; a.ntiles = (K + BN - 1) / BN;
  const int splits = wgrad_splits((int)rows, a.mtiles * a.ntiles);
  const int stages = (((int)rows + BK - 1) / BK + splits - 1) / splits;
  a.k_per_split = stages * BK;
  a.part = splits > 1 ? (float*)ws : dw;
  a.a_bytes = (unsigned)(rows * N * 2); a.b_bytes = (unsigned)(rows * K * 2);
  const int rc = launch_tm<true, true, 2>(4, a, N, splits, st);
  if (rc != CNNK_OK || splits == 1) return rc;
  const size_t n = (size_t)N * K;
  size_t blocks = (n / 4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  sum_partials_kernel<<<(unsigned)blocks, 256, 0, st>>>((const float*)ws, splits, n, dw);
  return launch_status();
}
