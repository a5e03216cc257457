// Dense bf16 matrix products of the Vision Transformer step's linear layers on the gfx950 matrix
// cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): y = x W^T (+ bias, + GELU), dx = dy W,
// dW = dy^T x.  One kernel, three operand orientations.
//
// Workgroup tile 256 x 128 (or 192 x 128), four wavefronts of 128 x 64 (0.75 KB of LDS operand reads per
// MFMA), LDS stage buffers filled straight from memory (buffer_load ... lds; out-of-range rows deposit
// zeros), one barrier per stage, two workgroups per CU.  Two configurations: 32 reduction elements per
// stage in 64-byte LDS rows with three stage buffers (loads two stages ahead), or - for the long
// reductions of an operand whose reduction index is the contiguous one - 64 elements per stage in
// 128-byte rows with two buffers (see Cfg below for why).  An operand whose reduction index is its
// contiguous one ("natural": x and W of the forward product, dy of the data gradient) lies in LDS as
// [row][reduction elements of the stage] and is read with 16-byte loads; an operand whose reduction
// index is its row index (W of the data gradient, both operands of the weight gradient) lies as planes
// of [reduction rows][32 or 64 columns] and is read with the transposing load ds_read_b64_tr_b16, so no
// operand is ever transposed in memory.  The 16-byte chunks of a row are XOR-swizzled so that both kinds
// of read touch every bank once per pass (swz_of).  Because the hardware fixes where a direct load's
// bytes land (lane i at base + 16 i), the layout is produced by which global bytes each lane asks for.
// Epilogue per wavefront through a private LDS strip (accumulator quads in, transposing reads out):
// 16-byte stores of 8 consecutive columns; bias and GELU are applied to the fp32 accumulator first, so
// an output is rounded once.  The weight gradient splits the row range over blockIdx.z and writes
// fp32 partials that a second kernel adds in a fixed order.
#include "common.h"
#include "gemm.h"

extern int g_cnnk_tune[16];

namespace {
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));

// TM: 32-row blocks of a wavefront's tile (4: workgroup tile 256 x 128, 3: 192 x 128).
// RB: bytes of an LDS row = bytes of an operand row that one group of lanes fetches.  The path from L2
// into LDS moves a fixed number of requests per clock whatever their size up to a 128-byte line
// (measured: 16 TB/s with 64-byte row segments, 32 TB/s with 128-byte ones), and with 64-byte rows that
// path, not the matrix pipe, bounds the kernel.  128-byte rows of an operand whose reduction index is
// the contiguous one mean 64 reduction elements per stage, and then only two stage buffers of a
// 192 x 128 tile fit the 80 KB a workgroup may hold with two workgroups per CU; an operand read through
// the transposing load takes 128-byte rows by widening its planes to 64 columns, at any stage depth.
template <int TM, int BK_, int RB_> struct Cfg {
  static constexpr int BK = BK_, RB = RB_;
  static constexpr int NW = 4, THREADS = 64 * NW, BN = 128;   // four wavefronts, 2 x 2
  static constexpr int NST = BK == 64 ? 2 : 3;           // stage buffers; loads run NST - 1 stages ahead
  static constexpr int BM = 64 * TM, A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_B = A_BYTES + B_BYTES;
  static constexpr int NLOAD = STAGE_B / 1024 / NW;      // direct loads per wavefront and stage
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "every load of a wavefront belongs to one operand");
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
// What the index of a 16-byte chunk is XORed with to give its position in the LDS row.  64-byte rows
// read with 16-byte loads: row bits 2-3; read with the transposing load: nothing, four consecutive
// rows are the 64 banks whatever the order inside a row.
// 128-byte rows read with 16-byte loads (sixteen rows of one chunk per pass): with row bits 1-3, so that
// the eight rows of either parity - a row's parity picks the half of the banks - sit on eight different
// chunk positions.  128-byte rows read with the transposing load (four rows x 64 bytes per pass): the
// two 64-byte halves swap on every second pair of rows, which puts the four rows on four bank quarters.
template <int RB, bool TR> __device__ __forceinline__ int swz_of(int row) {
  if (RB == 64) return TR ? 0 : (row >> 2) & 3;
  return TR ? ((row >> 1) & 1) << 2 : (row >> 1) & 7;
}

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

// gelu(u) = u/2 (1 + erf(u / sqrt 2)) with erf(t) = t P(t^2) on |t| <= 3, P of degree 8 fitted to erf(t) / t
// (least squares on Chebyshev nodes, weighted so that the absolute error of erf is what is minimised;
// evaluated in fp32: 2.1e-5), and t clamped to that range beyond it (1 - erf(3) = 2.2e-5).  Fourteen
// full-rate instructions and no reciprocal or exponential: the epilogue runs on the vector ALU with
// nothing to overlap it, and the ~25 instructions per element of an erfc-based form were a tenth of the
// launch.  Absolute error of gelu below 4.4e-5 for every u, a hundredth of what the bf16 store rounds off.
__device__ __forceinline__ float gelu_f(float u) {
  const float t = fminf(fmaxf(u * 0.70710678118654752f, -3.0f), 3.0f);
  const float s = t * t;
  float p = 3.912539981e-08f;
  p = fmaf(p, s, -1.883036475e-06f);
  p = fmaf(p, s, 4.008835822e-05f);
  p = fmaf(p, s, -5.029218737e-04f);
  p = fmaf(p, s, 4.196857568e-03f);
  p = fmaf(p, s, -2.499890141e-02f);
  p = fmaf(p, s, 1.109308004e-01f);
  p = fmaf(p, s, -3.752196431e-01f);
  p = fmaf(p, s, 1.128250599e+00f);
  const float hu = 0.5f * u;
  return fmaf(hu, t * p, hu);
}

template <bool ATR, bool BTR, int EPI, int TM, int BK, int RB>
__global__ void __launch_bounds__(256, 2) gemm_kernel(Args a) {
  using C = Cfg<TM, BK, RB>;
  constexpr int NW = C::NW, BN = C::BN;
  constexpr int BM = C::BM, A_BYTES = C::A_BYTES, STAGE_B = C::STAGE_B, NLOAD = C::NLOAD, NST = C::NST;
  constexpr int LPR = RB / 16, RPL = 1024 / RB;       // lanes per LDS row, rows per direct load
  constexpr int PC = RB / 2, PLANE_B = BK * RB;       // a transposed operand: planes of BK reduction rows x PC columns
  constexpr int KS = BK / 16;                         // MFMA reduction steps per stage
  static_assert((ATR || BK * 2 == RB) && (BTR || BK * 2 == RB), "a natural operand's LDS row is its BK reduction elements");
  static_assert(BM % PC == 0 || !ATR, "whole planes");
  static_assert(NST == 2 || NLOAD < 16, "the wait below encodes the load count in four bits");
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
  // ---- this lane's direct loads of a stage ----
  // A load of the wavefront fills 1 KB of LDS: RPL rows of RB bytes, lane i the 16 bytes at 16 i, so
  // the LPR lanes of a row ask for the (swizzled) chunks of one RB-byte segment of memory.
  // kk0: reduction index of the lane's 16 bytes in stage 0 (its first element for a natural operand,
  // its row for a transposed one); a load of stage t is in range while kk0 + t * BK < kend
  unsigned voff[NLOAD];
  int kk0[NLOAD];
  const unsigned vinc_a = ATR ? (unsigned)(BK * a.lda * 2) : BK * 2, vinc_b = BTR ? (unsigned)(BK * a.ldb * 2) : BK * 2;
#pragma unroll
  for (int j = 0; j < NLOAD; ++j) {
    const bool isA = j * NW < A_BYTES / 1024;           // blocks j * NW + wave: a compile-time property
    const int qq = j * NW + wave - (isA ? 0 : A_BYTES / 1024);
    const bool tr = isA ? ATR : BTR;
    const int ld = isA ? a.lda : a.ldb;
    const int o0 = isA ? m0 : n0, olim = isA ? a.M : a.N;
    const int p = lane % LPR;
    if (!tr) {
      const int r = qq * RPL + lane / LPR;
      const int c = p ^ swz_of<RB, false>(r);
      const int row = o0 + r;
      kk0[j] = row < olim ? kbeg + 8 * c : (1 << 30);
      voff[j] = (unsigned)((row * ld + kbeg + 8 * c) * 2);
    } else {
      const int plane = qq / (BK / RPL), r = (qq % (BK / RPL)) * RPL + lane / LPR;
      const int c = p ^ swz_of<RB, true>(r);
      const int col = o0 + plane * PC + 8 * c;
      kk0[j] = col < olim ? kbeg + r : (1 << 30);
      voff[j] = (unsigned)(((kbeg + r) * ld + col) * 2);
    }
  }
  auto issue = [&](int t, int sb) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
      const bool isA = j * NW < A_BYTES / 1024;
      const unsigned off = kk0[j] + t * BK < kend ? voff[j] + (unsigned)t * (isA ? vinc_a : vinc_b) : kOobOffset;
      load16_to_lds(isA ? a_rs : b_rs, (unsigned)(sb + (j * NW + wave) * 1024), off);
    }
  };
  // ---- fragment addresses (stage-relative) ----
  // natural: 16 bytes = reduction elements ks * 16 + h * 8 .. + 8 of row lane % 32 of a 32-row block;
  // blocks lie 32 rows apart and the swizzle repeats every 16 rows.  The chunk index ks * 2 + h meets
  // the swizzle in an XOR, so step ks is the address of step 0 XOR ks * 32 (128-byte rows) and the next
  // row's 32 bytes on (64-byte rows).
  // transposed: a pair of transposing reads, reduction rows ks * 16 + h * 8 + (lane % 16) / 4 and + 4,
  // of 32-column block sub of the wavefront's tile.
  int a_n0 = 0, b_n0 = 0;            // natural: address of step 0, block 0
  int a_t0 = 0, b_t0 = 0;            // transposed: address of step 0 within a 32-column block at column 0
  int a_sub[TM], b_sub[2];           // transposed: where block sub lies (plane, and half of a 128-byte row)
  auto nat0 = [&](int row) { return row * RB + ((h ^ swz_of<RB, false>(row)) << 4); };
  auto tr0 = [&]() {
    const int ch0 = (g & 1) * 16 + (i16 & 3) * 4, row = h * 8 + (i16 >> 2);
    return row * RB + ((ch0 >> 3) << 4) + (ch0 & 7) * 2;        // 128-byte rows: which half of the row is in a_sub / b_sub
  };
  auto tr_sub = [&](int cb) {        // cb: 32-column block of the operand's tile
    if (RB == 64) return cb * PLANE_B;
    const int sw = swz_of<128, true>(i16 >> 2) >> 2;            // the same for every row this lane reads
    return (cb >> 1) * PLANE_B + (((cb & 1) ^ sw) << 6);
  };
  if (!ATR) a_n0 = nat0(wm * (TM * 32) + (lane & 31)); else a_t0 = tr0();
  if (!BTR) b_n0 = A_BYTES + nat0(wn * 64 + (lane & 31)); else b_t0 = A_BYTES + tr0();
#pragma unroll
  for (int i = 0; i < TM; ++i) a_sub[i] = ATR ? tr_sub(wm * TM + i) : i * 32 * RB;
#pragma unroll
  for (int j = 0; j < 2; ++j) b_sub[j] = BTR ? tr_sub(wn * 2 + j) : j * 32 * RB;
  auto read_frag = [&](const unsigned char* sb, bool tr, int n0a, int t0a, int subo, int ks) __attribute__((always_inline)) -> bf16x8_t {
    if (!tr) {
      return *reinterpret_cast<const bf16x8_t*>(sb + (n0a ^ (ks << 5)) + subo);
    }
    const unsigned char* q = sb + t0a + ks * 16 * RB + subo;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)q);
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(q + 4 * RB));
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

#pragma unroll
  for (int d = 0; d < NST - 1; ++d)
    if (d < nst) issue(d, d * STAGE_B);
  int cur = 0;
  for (int t = 0; t < nst; ++t) {
    // this wave's loads of stage t have landed; those of the stages issued after it may stay in flight
    if (NST == 3 && t + 1 < nst) __builtin_amdgcn_s_waitcnt(0x0f70 | NLOAD);
    else __builtin_amdgcn_s_waitcnt(0x0f70);
    __builtin_amdgcn_s_barrier();
    if (t + NST - 1 < nst) {
      int fill = cur + (NST - 1) * STAGE_B;
      if (fill >= NST * STAGE_B) fill -= NST * STAGE_B;
      issue(t + NST - 1, fill);
    }
    const unsigned char* sb = smem + cur;
    bf16x8_t af[2][TM], bfr[2][2];
#pragma unroll
    for (int kp = 0; kp < KS; kp += 2) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[ks][i] = read_frag(sb, ATR, a_n0, a_t0, a_sub[i], kp + ks);
#pragma unroll
        for (int j = 0; j < 2; ++j) bfr[ks][j] = read_frag(sb, BTR, b_n0, b_t0, b_sub[j], kp + ks);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0);
    }
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
int launch(Kern kern, bool* raised, int threads, int smem_bytes, const Args& a, int splits, hipStream_t st) {
  if (!*raised) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes) != hipSuccess)
      return CNNK_ERR_HIP;
    *raised = true;
  }
  hipLaunchKernelGGL(kern, dim3(8 * ((a.mtiles * a.ntiles + 7) / 8), 1, splits), dim3(threads), smem_bytes, st, a);
  return launch_status();
}
template <bool ATR, bool BTR, int EPI, int TM, int BK, int RB>
int launch_cfg(Args& a, int splits, hipStream_t st) {
  static bool raised = false;
  using C = Cfg<TM, BK, RB>;
  a.mtiles = (a.M + C::BM - 1) / C::BM;
  a.ntiles = (a.N + C::BN - 1) / C::BN;
  return launch(gemm_kernel<ATR, BTR, EPI, TM, BK, RB>, &raised, C::THREADS, C::NST * C::STAGE_B, a, splits, st);
}
// Rows per workgroup tile (in 64s): the device holds 512 workgroups at once; the cost of a launch is
// about (rounds of resident workgroups) x (tile height).
int pick_tm(int out_rows, int ntiles) {
  auto cost = [&](int tm) { const int t = ((out_rows + 64 * tm - 1) / (64 * tm)) * ntiles; return ((t + 511) / 512) * tm; };
  return cost(3) < cost(4) ? 3 : 4;
}
// One launch of an orientation with a natural operand.  128-byte rows (192 x 128 tiles, 64 reduction
// elements per stage, loads one stage ahead) pay from a reduction length of 2048 on: -15 % on
// 12608 x 3072 -> 768; shorter reductions run as fast or faster with 64-byte rows, three stage buffers
// and the choice of tile heights (the tuning table forces either: 15 = 1 / 2).
template <bool BTR, int EPI>
int launch_nat(Args& a, hipStream_t st) {
  const bool wide = g_cnnk_tune[15] == 2 || (g_cnnk_tune[15] != 1 && a.K >= 2048);
  if (wide) return launch_cfg<false, BTR, EPI, 3, 64, 128>(a, 1, st);
  if (pick_tm(a.M, (a.N + 127) / 128) == 3) return launch_cfg<false, BTR, EPI, 3, 32, 64>(a, 1, st);
  return launch_cfg<false, BTR, EPI, 4, 32, 64>(a, 1, st);
}

bool fits32(long long rows, long long cols) { return rows * cols * 2 < 2147483647LL; }
int wgrad_splits(int rows, int tiles) {
  int s = (192 + tiles - 1) / tiles;           // workgroups of a launch: it runs beside the main stream's kernels (128-192 measured best)
  const int max_s = rows / (8 * 32);           // at least 8 stages each
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
  a.a_bytes = (unsigned)(rows * K * 2); a.b_bytes = (unsigned)((long long)N * K * 2);
  if (res) return launch_nat<false, 3>(a, st);
  return gelu ? launch_nat<false, 1>(a, st) : launch_nat<false, 0>(a, st);
}

int gemm_bf16_dgrad(long long rows, int K, int N, const bf16_t* dy, const bf16_t* w, bf16_t* dx, hipStream_t st) {
  Args a{};
  a.A = dy; a.B = w; a.C = dx;
  a.M = (int)rows; a.N = K; a.K = N; a.lda = N; a.ldb = K; a.ldc = K; a.k_per_split = N;
  a.a_bytes = (unsigned)(rows * N * 2); a.b_bytes = (unsigned)((long long)N * K * 2);
  return launch_nat<true, 0>(a, st);
}

size_t gemm_bf16_wgrad_ws(long long rows, int K, int N) {
  const int tiles = ((N + 255) / 256) * ((K + 127) / 128);
  const int s = wgrad_splits((int)rows, tiles);
  return s > 1 ? (size_t)s * N * K * sizeof(float) : 0;
}

int gemm_bf16_wgrad(long long rows, int K, int N, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st) {
  Args a{};
  a.A = dy; a.B = x;
  a.M = N; a.N = K; a.K = (int)rows; a.lda = N; a.ldb = K; a.ldc = K;
  a.mtiles = (N + 255) / 256; a.ntiles = (K + 127) / 128;
  const int splits = wgrad_splits((int)rows, a.mtiles * a.ntiles);
  const int stages = (((int)rows + 31) / 32 + splits - 1) / splits;
  a.k_per_split = stages * 32;
  a.part = splits > 1 ? (float*)ws : dw;
  a.a_bytes = (unsigned)(rows * N * 2); a.b_bytes = (unsigned)(rows * K * 2);
  // 64-column planes (128-byte rows) measured 5-10 % slower here than 32-column ones; kept selectable
  const int rc = g_cnnk_tune[15] == 2 ? launch_cfg<true, true, 2, 4, 32, 128>(a, splits, st) : launch_cfg<true, true, 2, 4, 32, 64>(a, splits, st);
  if (rc != CNNK_OK || splits == 1) return rc;
  const size_t n = (size_t)N * K;
  size_t blocks = (n / 4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  sum_partials_kernel<<<(unsigned)blocks, 256, 0, st>>>((const float*)ws, splits, n, dw);
  return launch_status();
}
