// 3x3 stride-1 convolution (forward and data gradient) with the input patch resident in LDS.
//
// The plain implicit-GEMM kernel re-fetches the pixel tile for every filter tap, which makes it
// L2->CU traffic bound on MI355X.  Here a workgroup owns an output tile of TI images x TH rows
// x W columns, loads the matching input patch (+1 pixel halo, zero padded) for a 32-channel
// chunk ONCE into LDS in its natural [pixel][channel] layout, and serves all nine taps from it:
// a tap is just a pixel offset into the patch.  Only the weights stream (one [BN][32] slice per
// tap, two slices in flight in registers + a two-deep LDS ring).  bf16 MFMA 32x32x16, fp32
// accumulation, same LDS-transposed epilogue / optional channel statistics / accumulate as the
// implicit-GEMM kernel.
#include <type_traits>
#include "common.h"
#include "conv.h"

namespace {

constexpr int kThreads = 256;
constexpr int CK = 32;          // channels per chunk

typedef short s16x4_t __attribute__((ext_vector_type(4)));

constexpr int kPxPerLoad = kThreads / (CK / 8);  // patch pixels staged per 16-byte load of the workgroup

struct PatchArgs {
  const bf16_t* src;
  const bf16_t* wt;   // [Cd][9][Cs]
  bf16_t* dst;
  float* stats;       // nullable: [2][Cd][mtiles * WM]
  int N, H, W, Cs, Cd;
  int TI, TH;         // tile = TI images x TH rows x W columns (BM pixels)
  int accumulate, ntiles, mtiles;
  int tpb;            // pixel tiles a workgroup walks (consecutive, same channel tile); mtiles % tpb == 0
  int perm;           // row permutation of the pixel tile, see tile_pixel()
  int toff_h[9], toff_w[9], widx[9];  // patch offset (0..2, 0..2) and weight tap of each step
  FastDiv dPW, dPH, dW, dTH, dH;      // divisors used to decode pixel indices
};

// LDS rows are dense 64-byte rows (32 channels) whose four 16-byte chunks are XOR-swizzled with
// bits 2..3 of the row index: 16 lanes reading one chunk of 16 consecutive rows, and 16 lanes
// writing 4 whole rows, both touch every bank once.
__device__ __forceinline__ int swz_off(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4); }

// Which pixel of the tile (index (ti*TH + th)*W + tw) the GEMM row `rho` stands for.  The MFMA does
// not care which 32 pixels share a tile, but the LDS does: a quarter-wave reads 16 patch rows at
// once and they must differ modulo 16 (the bank pattern repeats every 16 rows).  With W >= 16 the
// 16 pixels are consecutive; narrower images put several image rows into one quarter-wave, whose
// patch rows collide unless they are picked apart:
//   perm 1 (W = 8, TH = 8): image rows th and th+4 share a quarter-wave (4 patch rows = 40 = 8 mod 16);
//   perm 2 (W = 4, TH = 4): row th of four consecutive images (one padded image = 36 = 4 mod 16).
__device__ __forceinline__ int tile_pixel(int rho, int perm) {
  if (perm == 1) {
    const int u = (rho >> 3) & 7;
    return (rho & ~0x38) | ((((u >> 1) | ((u & 1) << 2))) << 3);
  }
  if (perm == 2) {
    const int j = rho & 15, G = rho >> 4;
    return ((((G >> 2) * 4 + (j >> 2)) * 4 + (G & 3)) << 2) | (j & 3);
  }
  return rho;
}

// PL: 16-byte patch loads per thread, i.e. the patch holds at most PL * 64 pixels.
//
// Software pipeline.  A step is one filter row (three taps) of one 32-channel chunk, 24 MFMAs per
// wave between two barriers; g = 3 * chunk + row is the step index.
//   weights: the three taps of step g live in LDS buffer g % 2.  Those of step g+3 are loaded from
//            global memory into register set (g+1) % 2 at the start of step g and stored to LDS
//            buffer (g+1) % 2 at the start of step g+2, i.e. two steps in flight;
//   patch:   chunk c+1 is loaded at row 0 of chunk c and stored to the other patch buffer at row 2;
//   MFMA operands of the next tap are read from LDS between the MFMAs of the current tap (two
//   fragment sets; scheduling directives pin the interleaving, because left alone the compiler
//   reads just in time - read, wait, multiply - and exposes the LDS latency eight times per tap).
// Nothing in a step is conditional on "is there another chunk": past the last chunk the loads
// fetch in-range or zero-filled bytes that land in LDS buffers nobody reads any more.  Straight
// line code lets the compiler count the loads in flight exactly, so every wait is for the oldest
// load only.
//
// What bounds it: a 32x32x16 MFMA needs 2 KB of operands; with 64 x 64 wave tiles that is 1 KB of
// LDS reads per MFMA, 4 KB per 32 cycles and CU, against the ~180 B/clk that 16-byte LDS reads
// sustain: the LDS pipe is ~70 % busy when the matrix pipe is full, so the two have to overlap
// almost perfectly.  Measured: 45-65 % of the MFMA rate inside the main loop.
//
// KG = 2: two groups of four wavefronts share the output tile and split the reduction: group kg takes
// the channel chunks kg, kg + 2, ... with patch and weight buffers of its own, and hands its
// accumulators to group 0 through LDS at the end.  For the layers whose tile grid only gives every CU
// one workgroup (few pixels, many channels: 8 x 8 and 4 x 4 images) this puts two wavefronts on every
// SIMD without the second output tile per CU that the layer does not have.  The two groups fetch
// together: eight lanes take the 128 bytes that the two chunks of a pair occupy side by side in a pixel
// or weight row, and each lane stores its 16 bytes into the buffer of the group that owns the chunk.
// The path from L2 into a CU moves a fixed number of requests per clock whatever their size up to a
// 128-byte line, and a workgroup of these layers streams all 4.6 K reduction rows of its 64 filters
// (590 KB with 512 channels): in 64-byte pieces that alone took longer than the MFMAs.
template <int BM, int BN, int WM, int WN, int OCC, int PL, int KG>
__global__ void __launch_bounds__(kThreads * KG, OCC) patch_kernel(PatchArgs a) {
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int B_IT = (BN + 63) / 64;  // 64 weight rows per pass (4 chunks of 8 channels per row)
  constexpr int KK = CK / 16;
  static_assert(WM * WN == 4 && TM >= 1 && TN == 2 && KK == 2, "tile shape");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int PW = a.W + 2, PH = a.TH + 2;
  const int patch_px = a.TI * PH * PW;
  const int patch_bytes = max(patch_px * 64, 4 * 32 * 72);   // at least the epilogue's four transposition strips
  // (group 1's buffers start an odd multiple of 128 bytes after group 0's, so that the two 64-byte
  // halves of a staged 128-byte piece fall on different banks)
  const int group_bytes = 2 * patch_bytes + 6 * BN * 64 + (KG == 2 && (patch_bytes & 64) == 0 ? 128 : 0);
  const int kg = KG == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8);   // reduction group
  unsigned char* Pb = smem_raw + kg * group_bytes;   // [2][patch_px][64 B]
  unsigned char* Bb = Pb + 2 * patch_bytes;          // [2][3][BN][64 B]

  const int tid = threadIdx.x & (kThreads - 1), lane = tid & 63, wave = tid >> 6;   // within the group
  const int wm = wave % WM, wn = wave / WM;
  // The grid is (pixel-tile groups, channel tiles), walked as one linear index; the second
  // dimension only makes layers with the same number of workgroups tell apart in a kernel trace.
  int b = blockIdx.y * gridDim.x + blockIdx.x;
  const int nb = gridDim.x * gridDim.y;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);  // consecutive tiles share an XCD
  const int nt = b % a.ntiles;
  int mt = (b / a.ntiles) * a.tpb;            // current pixel tile; the workgroup walks tpb of them
  const int mt_end = mt + a.tpb;
  const int M = a.N * a.H * a.W;

  const __amdgpu_buffer_rsrc_t src_rs = make_rsrc(a.src, (unsigned)M * a.Cs * 2u);
  const __amdgpu_buffer_rsrc_t wt_rs = make_rsrc(a.wt, (unsigned)a.Cd * 9u * a.Cs * 2u);

  // Staging: LPP lanes fetch one row (a patch position, or a filter's tap) of a 64-row pass.  One group:
  // 4 lanes, the 64 bytes of the chunk.  Two groups: 8 lanes, the 128 bytes of a pair of chunks; group kg
  // stages rows kg * 32 .. + 32 of the pass, and a lane's piece goes to group piece / 4.
  constexpr int LPP = KG == 2 ? 8 : 4;
  const int piece = tid & (LPP - 1), kc = piece & 3;
  const int srow = KG == 2 ? kg * 32 + (tid >> 3) : tid >> 2;
  unsigned char* Pst = KG == 2 ? smem_raw + (piece >> 2) * group_bytes : Pb;
  unsigned char* Bst = Pst + 2 * patch_bytes;
  // Patch addressing.  What a thread loads for patch position pp = srow + 64*j is the same for
  // every tile up to the tile's origin: a byte offset relative to the tile's first pixel (prel),
  // and whether the position is real data - never (padding column, or a padding row of a tile of
  // whole images), always (interior row), or only if the band of rows has a row above / below it
  // inside the image (pcls: bit j interior, bit 8+j row above, bit 16+j row below).  A tile then
  // costs two scalar conditions instead of two divisions per position.  Images past the end of
  // the batch (ragged last tile of whole images) lie past the end of the buffer and read as zeros.
  int prel[PL];
  unsigned pcls = 0;
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int pp = srow + j * 64;
    int q, pw, ti, ph;
    a.dPW.divmod(pp, &q, &pw);
    a.dPH.divmod(q, &ti, &ph);
    if (pp < patch_px && pw >= 1 && pw <= a.W) {
      if (ph >= 1 && ph <= a.TH) pcls |= 1u << j;
      else if (a.TI == 1) pcls |= (ph == 0 ? 0x100u : 0x10000u) << j;
    }
    prel[j] = (((ti * a.H + ph - 1) * a.W + pw - 1) * a.Cs + piece * 8) * 2;
  }
  // the positions that are real data in pixel tile `mtile` (bit j), and the byte offset of its origin
  auto tile_mask = [&](int mtile, unsigned* base) __attribute__((always_inline)) {
    const int m0 = mtile * BM;
    int q0, wrem, n0, h0;
    a.dW.divmod(m0, &q0, &wrem);
    a.dH.divmod(q0, &n0, &h0);
    *base = (unsigned)m0 * (unsigned)a.Cs * 2u;
    if (mtile >= mt_end) return 0u;        // past the workgroup's range: all zero fill
    const unsigned sel = 0xffu | (h0 > 0 ? 0xff00u : 0u) | (h0 + a.TH < a.H ? 0xff0000u : 0u);
    const unsigned v = pcls & sel;
    return (v | (v >> 8) | (v >> 16)) & 0xffu;
  };
  unsigned cbase, nbase;                   // current tile and the one after it
  unsigned cmask = tile_mask(mt, &cbase), nmask = tile_mask(mt + 1, &nbase);
  auto patch_off = [&](unsigned mask, unsigned base, int j) __attribute__((always_inline)) {
    return (mask >> j) & 1u ? base + (unsigned)prel[j] : kOobOffset;
  };
  // its LDS byte offset inside a patch buffer is pst0 + j * 64 rows (the swizzle repeats every 16 rows)
  const int pst0 = swz_off(srow, kc);
  const int r0 = srow;      // weight row of this thread inside a 64-row pass
  unsigned boff[B_IT];
  int bst[B_IT];
#pragma unroll
  for (int it = 0; it < B_IT; ++it) {
    const int row = r0 + it * 64, ch = nt * BN + row;
    boff[it] = (row < BN && ch < a.Cd) ? (unsigned)(ch * 9 * a.Cs + piece * 8) * 2u : kOobOffset;
    bst[it] = swz_off(row, kc);
  }
  // patch pixel (tap (0,0)) under each of this lane's output rows, and the weight-row offsets
  int app[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int p = tile_pixel(wm * TM * 32 + i * 32 + (lane & 31), a.perm);
    int q, tw, ti, th;
    a.dW.divmod(p, &q, &tw);
    a.dTH.divmod(q, &ti, &th);
    app[i] = (ti * PH + th) * PW + tw;
  }
  const int khalf = lane >> 5;
  int bfo[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) bfo[j] = swz_off(wn * TN * 32 + j * 32 + (lane & 31), khalf);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nchunks = a.Cs / CK / KG;      // chunks of this group: kg, kg + KG, ...
  // byte offset, in a pixel or weight row, of what is staged for chunk c: the chunk, or the pair
  auto chunk_bytes = [&](int c) { return (unsigned)__builtin_amdgcn_readfirstlane(c * KG * (CK * 2)); };
  uint4 preg[PL];
  uint4 rb[2][3][B_IT];

  // the chunk after chunk c of the current tile: c + 1, or chunk 0 of the next tile
  int c_in_tile = 0;
  auto load_next_patch = [&]() __attribute__((always_inline)) {
    const bool last = c_in_tile + 1 == nchunks;
    const unsigned so = chunk_bytes(last ? 0 : c_in_tile + 1);
    const unsigned base = last ? nbase : cbase, mask = last ? nmask : cmask;
#pragma unroll
    for (int j = 0; j < PL; ++j) preg[j] = buffer_load16(src_rs, patch_off(mask, base, j), so);
  };
  auto store_patch = [&](int buf) {
#pragma unroll
    for (int j = 0; j < PL; ++j)
      if (srow + j * 64 < patch_px)
        *reinterpret_cast<uint4*>(Pst + buf * patch_bytes + pst0 + j * 64 * 64) = preg[j];
  };
  auto load_w = [&](int chunk, auto ROW, auto SET) {   // the three taps of (chunk, filter row ROW) -> register set SET
    constexpr int row = decltype(ROW)::value, rs = decltype(SET)::value;
#pragma unroll
    for (int s3 = 0; s3 < 3; ++s3) {
      const unsigned so = (unsigned)(a.widx[row * 3 + s3] * a.Cs) * 2u + chunk_bytes(chunk);
#pragma unroll
      for (int it = 0; it < B_IT; ++it) rb[rs][s3][it] = buffer_load16(wt_rs, boff[it], so);
    }
  };
  auto store_w = [&](auto SET, auto WB) {    // register set SET -> LDS weight buffer WB
    constexpr int rs = decltype(SET)::value, wb = decltype(WB)::value;
#pragma unroll
    for (int s3 = 0; s3 < 3; ++s3)
#pragma unroll
      for (int it = 0; it < B_IT; ++it)
        if (BN % 64 == 0 || r0 + it * 64 < BN)
          *reinterpret_cast<uint4*>(Bst + (wb * 3 + s3) * (BN * 64) + bst[it]) = rb[rs][s3][it];
  };
  bf16x8_t af[2][TM][KK], bfr[2][TN][KK];
  // MFMA operands of tap TAP from patch buffer `pbuf` and weight buffer WB into fragment set SET
  auto read_frags = [&](int pbuf, auto TAP, auto WB, auto SET) {
    constexpr int tap = decltype(TAP)::value, wb = decltype(WB)::value, fs = decltype(SET)::value;
    // per-tap patch offset; opaque to the optimiser so that the (tap, row) LDS addresses are
    // recomputed here (5 VALU each) instead of being hoisted out of the chunk loop into registers
    int tpx = __builtin_amdgcn_readfirstlane(a.toff_h[tap] * PW + a.toff_w[tap]);
    asm volatile("" : "+s"(tpx));
    const unsigned char* P = Pb + pbuf * patch_bytes;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int pp = app[i] + tpx;
      const int o = pp * 64 + ((khalf ^ ((pp >> 2) & 3)) << 4);
      af[fs][i][0] = *reinterpret_cast<const bf16x8_t*>(P + o);
      af[fs][i][1] = *reinterpret_cast<const bf16x8_t*>(P + (o ^ 32));   // chunk + 2
    }
    const unsigned char* B = Bb + (wb * 3 + tap % 3) * (BN * 64);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      bfr[fs][j][0] = *reinterpret_cast<const bf16x8_t*>(B + bfo[j]);
      bfr[fs][j][1] = *reinterpret_cast<const bf16x8_t*>(B + (bfo[j] ^ 32));
    }
  };
  auto mfmas = [&](auto SET) {
    constexpr int fs = decltype(SET)::value;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[fs][i][kk], bfr[fs][j][kk], acc[i][j], 0, 0, 0);
  };
  // the MFMAs of one tap with the operand reads of the next tap spread between them: the compiler
  // on its own reads just in time (read, wait, multiply), which leaves the LDS latency exposed
  auto interleave = [&]() {
    constexpr int n_mfma = TM * TN * KK, n_read = (TM + TN) * KK;
#pragma unroll
    for (int k = 0; k < n_mfma; ++k) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   // one MFMA
      if (k < n_read) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                   // one LDS read
    }
  };
  // PARC = chunk % 2 (patch buffer of this chunk); the weight buffer / register set parities follow
  // from (chunk + row) % 2
  auto step = [&](auto PARC, auto ROW) __attribute__((always_inline)) {
    constexpr int par = decltype(PARC)::value, row = decltype(ROW)::value;
    constexpr int cur = (par + row) % 2, nxt = cur ^ 1;
    using WB = std::integral_constant<int, cur>;
    using NX = std::integral_constant<int, nxt>;
    using F0 = std::integral_constant<int, 0>;
    using F1 = std::integral_constant<int, 1>;
    store_w(NX{}, NX{});                      // weights of step g+1
    load_w(__builtin_amdgcn_readfirstlane(c_in_tile + 1 == nchunks ? 0 : c_in_tile + 1), ROW, NX{});   // step g+3: same row of the next chunk
    if constexpr (row == 0) load_next_patch();
    if constexpr (row == 2) store_patch(par ^ 1);
    read_frags(par, std::integral_constant<int, row * 3 + 0>{}, WB{}, F0{});
    __builtin_amdgcn_sched_barrier(0);
    read_frags(par, std::integral_constant<int, row * 3 + 1>{}, WB{}, F1{});
    mfmas(F0{});
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(par, std::integral_constant<int, row * 3 + 2>{}, WB{}, F0{});
    mfmas(F1{});
    interleave();
    __builtin_amdgcn_sched_barrier(0);
    mfmas(F0{});
    __syncthreads();
  };
  // Epilogue of one pixel tile, wave-local (no workgroup barrier, 1.1 KB of LDS per wave): optional
  // per-channel sums of the fp32 accumulators over this wave's 64 rows (one partial row per wave:
  // mtiles * WM rows in all, reduced by a finalising kernel), then eight passes of 8 rows x 64
  // columns through LDS so that every lane stores 16 contiguous bytes.
  auto epilogue = [&](int mtile, int par) __attribute__((always_inline)) {
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
          const size_t prow = (size_t)mtile * WM + wm, nrow = (size_t)a.mtiles * WM;
          a.stats[((size_t)0 * a.Cd + col) * nrow + prow] = s1;
          a.stats[((size_t)1 * a.Cd + col) * nrow + prow] = s2;
        }
      }
    }
    // Transposition through LDS so that a lane stores 16 contiguous bytes (8 channels of a pixel).
    // A lane of the accumulator layout holds one column (channel) and, per register quad, four
    // consecutive rows: the quad goes out as one 8-byte write into a [channel][row] strip, and the
    // transposing LDS read hands each lane four consecutive channels of one row back.  Per 32x32
    // tile: 4 writes, 4 reads, 2 stores; the stores of a tile are issued behind the LDS traffic of
    // the next one.  The strip lives in the patch buffer of the chunk just finished (every wave is
    // past the barrier behind its last read, and the buffer is not refilled before two more barriers).
    constexpr int SP = 72;   // strip pitch in bytes per channel: 32 rows + 8 bytes, keeps writes and reads off shared banks
    unsigned char* S = Pb + par * patch_bytes + wave * (32 * SP);
    const int mbase = mtile * BM;
    const int g4 = lane >> 4, i16 = lane & 15;
    const int wr_off = (lane & 31) * SP + (lane >> 5) * 8;
    const int rd_off = (g4 * 8 + (i16 >> 2)) * SP + (i16 & 3) * 8;
    uint4 pend[2];
    int pend_i = 0, pend_j = 0;
    auto flush = [&](int i, int j) __attribute__((always_inline)) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const int row = wm * TM * 32 + i * 32 + rb * 16 + i16;
        const int m = mbase + tile_pixel(row, a.perm), co = nt * BN + wn * TN * 32 + j * 32 + g4 * 8;
        if (m < M && co < a.Cd) {
          bf16_t* dp = a.dst + (size_t)m * a.Cd + co;
          if (a.accumulate) {
            float o[8], nw[8];
            load8(dp, o);
            unpack8(pend[rb], nw);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += nw[e];
            store8(dp, o);
          } else {
            *reinterpret_cast<uint4*>(dp) = pend[rb];
          }
        }
      }
    };
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 v;
          v.x = pack_bf16x2(acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1]);
          v.y = pack_bf16x2(acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
          *reinterpret_cast<uint2*>(S + wr_off + q * 16) = v;
        }
        // the reads below go through another type than the writes above: tell the compiler that
        // they touch the same memory (the hardware keeps a wave's LDS operations in order)
        asm volatile("" ::: "memory");
        uint4 cur[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (s16x4_t __attribute__((address_space(3)))*)(S + rd_off + rb * 32));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (s16x4_t __attribute__((address_space(3)))*)(S + rd_off + 4 * SP + rb * 32));
          const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
          cur[rb] = uint4{l2.x, l2.y, h2.x, h2.y};
        }
        asm volatile("" ::: "memory");   // ... and the next tile's writes stay behind these reads
        if (i + j > 0) flush(pend_i, pend_j);
        pend[0] = cur[0]; pend[1] = cur[1];
        pend_i = i; pend_j = j;
      }
    flush(pend_i, pend_j);
  };

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  // One chunk = three steps; after the last chunk of a pixel tile the accumulators are written out
  // and the workgroup moves on to its next tile, whose first patch chunk and weights are already
  // on their way (the prefetches do not know about tile borders).
  auto chunk_body = [&](auto PARC) __attribute__((always_inline)) {
    step(PARC, std::integral_constant<int, 0>{});
    step(PARC, std::integral_constant<int, 1>{});
    step(PARC, std::integral_constant<int, 2>{});
    if (c_in_tile + 1 == nchunks) {
      if constexpr (KG == 2) {
        // every wavefront is past the barrier behind its last operand read, and nothing refills the
        // buffers of a workgroup's only tile: group 1's buffers take its accumulators
        float* R = reinterpret_cast<float*>(smem_raw + group_bytes);
        if (kg == 1) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
              for (int r = 0; r < 16; ++r) R[((i * TN + j) * 16 + r) * kThreads + tid] = acc[i][j][r];
        }
        __syncthreads();
        if (kg == 1) return;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] += R[((i * TN + j) * 16 + r) * kThreads + tid];
      }
      epilogue(mt, decltype(PARC)::value);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      ++mt;
      c_in_tile = 0;
      cbase = nbase; cmask = nmask;
      nmask = tile_mask(mt + 1, &nbase);
    } else {
      ++c_in_tile;
    }
  };

#pragma unroll
  for (int j = 0; j < PL; ++j) preg[j] = buffer_load16(src_rs, patch_off(cmask, cbase, j), chunk_bytes(0));
  load_w(0, I0{}, I0{});
  load_w(0, I1{}, I1{});
  store_patch(0);
  store_w(I0{}, I0{});
  load_w(0, I2{}, I0{});   // register set 0 is free again
  __syncthreads();
  const int total_chunks = a.tpb * nchunks;
  for (int g2 = 0; g2 < total_chunks; g2 += 2) {
    chunk_body(I0{});
    if (g2 + 1 < total_chunks) chunk_body(I1{});
  }
}

struct PatchPlan {
  int bm, bn, ti, th;
};

// Tile geometry for BM output pixels: whole images, or a band of whole rows of one image.
bool tile_geometry(const ConvGeom& g, int bm, int max_px, int* ti, int* th) {
  const int hw = g.H * g.W;
  if (hw <= bm) {
    if (bm % hw != 0) return false;
    *ti = bm / hw; *th = g.H;
  } else {
    if (bm % g.W != 0 || g.H % (bm / g.W) != 0) return false;
    *ti = 1; *th = bm / g.W;
  }
  return (*ti) * (*th + 2) * (g.W + 2) <= max_px;
}

template <int BM, int BN>
size_t patch_smem(int patch_px) {
  // two patch buffers (each at least the 9 KB the epilogue's transposition strips need), two weight
  // buffers of three taps
  return (size_t)2 * (patch_px * 64 < 4 * 32 * 72 ? 4 * 32 * 72 : patch_px * 64) + (size_t)6 * BN * 64;
}

template <int BM, int BN, int WM, int WN, int OCC, int PL, int KG>
int launch_patch_kg(PatchArgs& a, hipStream_t st) {
  auto kern = patch_kernel<BM, BN, WM, WN, KG == 1 ? OCC : 1, PL, KG>;
  static bool attr_done = false;
  if (!attr_done) {
    const int most = KG * (int)patch_smem<BM, BN>(PL * kPxPerLoad) + 128;   // the largest patch the template takes
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            most < 160 * 1024 ? most : 160 * 1024) != hipSuccess)
      return CNNK_ERR_HIP;
    attr_done = true;
  }
  const size_t smem = KG * patch_smem<BM, BN>(a.TI * (a.TH + 2) * (a.W + 2)) + (KG == 2 ? 128 : 0);
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.mtiles / a.tpb), (unsigned)a.ntiles), dim3(kThreads * KG), smem, st, a);
  return launch_status();
}

template <int BM, int BN, int WM, int WN, int OCC, int PL>
int launch_patch(PatchArgs& a, hipStream_t st) {
  const long M = (long)a.N * a.H * a.W;
  a.ntiles = (a.Cd + BN - 1) / BN;
  a.mtiles = (int)((M + BM - 1) / BM);
  // Pixel tiles per workgroup: as many as still leave two workgroups for every CU.  A workgroup
  // that walks several tiles hides the prologue of all but the first behind the MFMAs before it.
  a.tpb = 1;
  for (int t = 2; t <= 8; t *= 2)
    if (a.mtiles % t == 0 && (long)a.ntiles * (a.mtiles / t) >= 512) a.tpb = t;
  if (g_cnnk_tune[13] > 0 && a.mtiles % g_cnnk_tune[13] == 0) a.tpb = g_cnnk_tune[13];
  // Fewer than two workgroups per CU: two groups of wavefronts per workgroup split the reduction
  // (an even number of channel chunks, both groups' buffers within the CU's 160 KB)
  const bool split = a.tpb == 1 && (long)a.ntiles * a.mtiles < 512 && (a.Cs / CK) % 2 == 0 && g_cnnk_tune[13] >= 0 &&
                     2 * patch_smem<BM, BN>(a.TI * (a.TH + 2) * (a.W + 2)) + 128 <= 160 * 1024;
  return split ? launch_patch_kg<BM, BN, WM, WN, OCC, PL, 2>(a, st) : launch_patch_kg<BM, BN, WM, WN, OCC, PL, 1>(a, st);
}

bool plan_patch(const ConvGeom& g, int Cs, int Cd, PatchPlan* p) {
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1) return false;
  if (Cs % CK != 0 || Cd % 8 != 0) return false;
  // byte offsets must stay below the out-of-bounds marker of the buffer loads
  if ((long)g.N * g.H * g.W * Cs * 2 >= (1L << 31) || (long)Cd * 9 * Cs * 2 >= (1L << 31)) return false;
  if (g_cnnk_tune[4] < 0) return false;   // patch kernels switched off
  const long M = (long)g.N * g.H * g.W;
  // Candidates in order of preference (the larger the pixel tile, the less weight traffic):
  // the first one that gives every CU a workgroup, else the one with the most workgroups.
  const int cand[4][3] = {{256, 64, 7}, {128, 128, 5}, {128, 64, 5}, {256, 128, 6}};  // BM, BN, PL (last: forced only)
  int best = -1;
  long best_blocks = 0;
  for (int k = 0; k < 4; ++k) {
    const int bm = cand[k][0], bn = cand[k][1];
    if (g_cnnk_tune[4] > 0 && (bm != g_cnnk_tune[4] || bn != g_cnnk_tune[5])) continue;
    if (bn == 128 && Cd <= 64) continue;
    if (k == 3 && g_cnnk_tune[4] <= 0) continue;   // 256x128 needs more registers than two waves per SIMD leave
    int ti, th;
    if (!tile_geometry(g, bm, cand[k][2] * kPxPerLoad, &ti, &th)) continue;
    const long blocks = ((M + bm - 1) / bm) * ((Cd + bn - 1) / bn);
    if (blocks >= 256) { best = k; break; }
    if (blocks > best_blocks) { best = k; best_blocks = blocks; }
  }
  if (best < 0) return false;
  p->bm = cand[best][0]; p->bn = cand[best][1];
  return tile_geometry(g, p->bm, cand[best][2] * kPxPerLoad, &p->ti, &p->th);
}

int run_patch(const ConvGeom& g, PatchArgs& a, const PatchPlan& p, hipStream_t st) {
  a.TI = p.ti; a.TH = p.th;
  a.perm = (a.W == 8 && a.TH == 8) ? 1 : (a.W == 4 && a.TH == 4 && a.TI % 4 == 0) ? 2 : 0;
  if (g_cnnk_tune[7] < 0) a.perm = 0;
  a.dPW.init(a.W + 2); a.dPH.init(a.TH + 2); a.dW.init(a.W); a.dTH.init(a.TH); a.dH.init(a.H);
  if (p.bm == 256 && p.bn == 128) return launch_patch<256, 128, 2, 2, 2, 6>(a, st);
  if (p.bm == 256 && p.bn == 64)
    return a.TI * (a.TH + 2) * (a.W + 2) <= 6 * kPxPerLoad ? launch_patch<256, 64, 4, 1, 2, 6>(a, st)
                                                            : launch_patch<256, 64, 4, 1, 2, 7>(a, st);
  if (p.bm == 128 && p.bn == 128) return launch_patch<128, 128, 2, 2, 2, 5>(a, st);
  if (p.bm == 128 && p.bn == 64) return launch_patch<128, 64, 4, 1, 2, 5>(a, st);
  (void)g;
  return CNNK_ERR_UNSUPPORTED;
}

}  // namespace

bool conv_patch_supported(const ConvGeom& g, int pass) {
  PatchPlan p;
  if (pass == CNNK_PASS_FWD) return plan_patch(g, g.Cin, g.Cout, &p);
  if (pass == CNNK_PASS_DGRAD) return plan_patch(g, g.Cout, g.Cin, &p);
  return false;
}

// rows of the statistics partials that conv_patch_fwd writes: one per wave row of every pixel tile
int conv_patch_stat_rows(const ConvGeom& g) {
  PatchPlan p;
  if (!plan_patch(g, g.Cin, g.Cout, &p)) return 0;
  const int wm = p.bn == 64 ? 4 : 2;
  return (int)(((long)g.N * g.H * g.W + p.bm - 1) / p.bm) * wm;
}

int conv_patch_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* stats, hipStream_t st) {
  PatchPlan p;
  if (!plan_patch(g, g.Cin, g.Cout, &p)) return CNNK_ERR_UNSUPPORTED;
  PatchArgs a{};
  a.src = x; a.wt = w; a.dst = y; a.stats = stats;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cs = g.Cin; a.Cd = g.Cout; a.accumulate = 0;
  for (int r = 0; r < 3; ++r)
    for (int s = 0; s < 3; ++s) {
      a.toff_h[r * 3 + s] = r; a.toff_w[r * 3 + s] = s; a.widx[r * 3 + s] = r * 3 + s;
    }
  return run_patch(g, a, p, st);
}

// wt: weights already transposed to [Cin][9][Cout]
int conv_patch_dgrad(const ConvGeom& g, const bf16_t* dy, const bf16_t* wt, bf16_t* dx, int accumulate,
                     hipStream_t st) {
  PatchPlan p;
  if (!plan_patch(g, g.Cout, g.Cin, &p)) return CNNK_ERR_UNSUPPORTED;
  PatchArgs a{};
  a.src = dy; a.wt = wt; a.dst = dx; a.stats = nullptr;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cs = g.Cout; a.Cd = g.Cin; a.accumulate = accumulate;
  // dx[h,w] takes dy[h+1-r, w+1-s] with w[.,r,s,.]: patch offset (2-r, 2-s)
  for (int r = 0; r < 3; ++r)
    for (int s = 0; s < 3; ++s) {
      a.toff_h[r * 3 + s] = 2 - r; a.toff_w[r * 3 + s] = 2 - s; a.widx[r * 3 + s] = r * 3 + s;
    }
  return run_patch(g, a, p, st);
}
