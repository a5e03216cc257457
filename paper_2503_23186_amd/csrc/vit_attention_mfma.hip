// Self-attention on the matrix cores for bf16 storage, head size 64 and sequences of at most 256
// tokens (a ViT-B/16 image: 197): forward and backward of softmax(q k^T / 8) v for one (image, head)
// per workgroup, one 32-token block per wavefront (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Every matrix of the head (K, V; in the backward pass also Q and dO) sits in LDS once, in its natural
// [token][feature] layout: two planes of 32 features with 64-byte rows whose 16-byte chunks are
// XOR-swizzled by row bits 2-3.  Products that reduce over features read fragments with 16-byte loads
// (a token per lane); products that reduce over tokens read the same bytes with the transposing
// load ds_read_b64_tr_b16 (a feature per lane, four consecutive tokens per read).  Both patterns touch
// every LDS bank once per pass.
//
// Score tiles are computed transposed (rows = keys, columns = queries) where the softmax runs over
// keys, so that a query's row statistics are per-lane scalars, and the accumulator of a score tile is
// at once the B operand of the product that follows it: register i of lane l holds key
// (i/4)*8 + (l/32)*4 + i%4 of the tile, so registers 8j..8j+7 are the lane's eight reduction slots of
// 16-key step j, and the A operand is read with the same key-to-slot assignment (rows h*4..h*4+3 and
// 8+h*4..8+h*4+3 of the step for lane half h) instead of the usual 8 consecutive ones.
// Probabilities are not stored: the forward pass writes log-sum-exp per query and the backward pass
// recomputes exp(s - lse).  The backward pass runs two walks in one launch: by query block for dq,
// by key block for dk and dv (which recomputes the score tiles in the other orientation), so every
// sum has one owner and a fixed order: no atomics, bit-reproducible.
#include "common.h"
#include "../../include/cnnk_vit.h"

namespace {
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
constexpr int kDH = 64;
constexpr int ROW_B = 64;       // bytes of one token's 32 features of a plane

__device__ __forceinline__ int chunk_off(int row, int c16) { return row * ROW_B + ((c16 ^ ((row >> 2) & 3)) << 4); }

// 16-byte fragment read: token `row`, features d0 .. d0+7 (d0 a multiple of 8)
__device__ __forceinline__ bf16x8_t frag_read(const unsigned char* t, int plane_b, int row, int d0) {
  const unsigned char* p = t + (d0 >> 5) * plane_b + chunk_off(row, (d0 & 31) >> 3);
  return *reinterpret_cast<const bf16x8_t*>(p);
}
// Transposing fragment read for a product that reduces over tokens: the lane gets feature
// mt*32 + lane%32 of tokens rbase + h*4 + 0..3 and rbase + 8 + h*4 + 0..3 (h = lane / 32).
__device__ __forceinline__ bf16x8_t frag_read_tr(const unsigned char* t, int plane_b, int mt, int rbase, int lane) {
  const int g = lane >> 4, i16 = lane & 15;
  const int ch0 = (g & 1) * 16 + (i16 & 3) * 4;               // first of the 4 features this lane's address names
  const int row = rbase + (g >> 1) * 4 + (i16 >> 2);
  const unsigned char* base = t + mt * plane_b + (ch0 & 7) * 2;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4_t __attribute__((address_space(3)))*)(base + chunk_off(row, ch0 >> 3)));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4_t __attribute__((address_space(3)))*)(base + chunk_off(row + 8, ch0 >> 3)));
  const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8_t, v);
}
__device__ __forceinline__ bf16x8_t pack_frag(const f32x16_t& a, int j) {
  uint4 v;
  v.x = pack_bf16x2(a[8 * j + 0], a[8 * j + 1]);
  v.y = pack_bf16x2(a[8 * j + 2], a[8 * j + 3]);
  v.z = pack_bf16x2(a[8 * j + 4], a[8 * j + 5]);
  v.w = pack_bf16x2(a[8 * j + 6], a[8 * j + 7]);
  return __builtin_bit_cast(bf16x8_t, v);
}
__device__ __forceinline__ f32x16_t zero16() {
  f32x16_t z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}
// Rows [0, Tp) of a head's 64 features (global rows `ld` elements apart) into the two LDS planes; rows
// >= T are zero.  A workgroup has 64 threads per 32 rows, so every thread moves exactly four 16-byte
// pieces of a matrix: fetch() issues the four loads, put() stores them - a caller fetches all its
// matrices before it puts the first, so that a thread has all its loads in flight at once (as a loop of
// load-then-store the sixteen loads of the backward pass ran one after the other, a third of the launch).
struct Pieces { uint4 v[4]; };
__device__ __forceinline__ void fetch(const bf16_t* src, size_t ld, int T, Pieces* p) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = threadIdx.x + k * blockDim.x, r = i >> 3, c8 = i & 7;
    p->v[k] = make_uint4(0u, 0u, 0u, 0u);
    if (r < T) p->v[k] = *reinterpret_cast<const uint4*>(src + (size_t)r * ld + c8 * 8);
  }
}
__device__ __forceinline__ void put(const Pieces& p, unsigned char* dst, int plane_b) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = threadIdx.x + k * blockDim.x, r = i >> 3, c8 = i & 7;
    *reinterpret_cast<uint4*>(dst + (c8 >> 2) * plane_b + chunk_off(r, c8 & 3)) = p.v[k];
  }
}
// a 32 x 32 tile of X Y^T over the 64 features: rows = tokens arow0.. of the LDS matrix `a`, columns =
// the wave's own tokens, whose four fragments are in `b`
__device__ __forceinline__ f32x16_t tile_nt(const unsigned char* a, int plane_b, int arow0, const bf16x8_t* b, int lane) {
  f32x16_t acc = zero16();
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_read(a, plane_b, arow0 + (lane & 31), ks * 16 + (lane >> 5) * 8), b[ks], acc, 0, 0, 0);
  return acc;
}
// the accumulator of a [64 features] x [32 own tokens] product: 4 consecutive features per 8-byte store
__device__ __forceinline__ void store_cols(bf16_t* dst_row, const f32x16_t* acc, int h) {
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const uint2 v = make_uint2(pack_bf16x2(acc[mt][4 * i4], acc[mt][4 * i4 + 1]), pack_bf16x2(acc[mt][4 * i4 + 2], acc[mt][4 * i4 + 3]));
      *reinterpret_cast<uint2*>(dst_row + mt * 32 + i4 * 8 + h * 4) = v;
    }
}

__global__ void __launch_bounds__(512) attn_mfma_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                            float* __restrict__ lse, int T, int heads) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int NT = blockDim.x >> 6, Tp = NT * 32, plane_b = Tp * ROW_B;
  unsigned char* Ks = smem;
  unsigned char* Vs = smem + 2 * plane_b;
  const int b = blockIdx.x / heads, head = blockIdx.x % heads, d = heads * kDH;
  const bf16_t* base = qkv + (size_t)b * T * 3 * d + head * kDH;
  Pieces pk, pv;
  fetch(base + d, 3 * (size_t)d, T, &pk);
  fetch(base + 2 * d, 3 * (size_t)d, T, &pv);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, h = lane >> 5;
  const int q = wave * 32 + n;
  bf16x8_t bq[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (q < T) v = *reinterpret_cast<const uint4*>(base + (size_t)q * 3 * d + ks * 16 + h * 8);
    bq[ks] = __builtin_bit_cast(bf16x8_t, v);
  }
  put(pk, Ks, plane_b);
  put(pv, Vs, plane_b);
  __syncthreads();
  // exp(s / 8 - x) = exp2(s c - x c') with c = log2 e / 8: the scale rides in the multiply-add in front of
  // the exponential.  Keys past T exist only in the last tile, so only that tile masks.
  const float c2 = 0.125f * 1.44269504088896341f;
  // first walk over the keys: running maximum (of the raw scores) and sum of this lane's half of the keys
  float m = -INFINITY, l = 0.f;
  for (int kt = 0; kt < NT; ++kt) {
    f32x16_t s = tile_nt(Ks, plane_b, kt * 32, bq, lane);
    if (kt == NT - 1) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (kt * 32 + (i >> 2) * 8 + h * 4 + (i & 3) >= T) s[i] = -INFINITY;
    }
    float tm = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tm = fmaxf(tm, s[i]);
    const float mn = fmaxf(m, tm);
    if (mn > -INFINITY) {
      const float mc = mn * c2;
      float add = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) add += __builtin_amdgcn_exp2f(fmaf(s[i], c2, -mc));
      l = l * __builtin_amdgcn_exp2f(fmaf(m, c2, -mc)) + add;
      m = mn;
    }
  }
  {
    const float mo = __shfl_xor(m, 32, 64), lo = __shfl_xor(l, 32, 64);
    const float M = fmaxf(m, mo);
    l = l * __builtin_amdgcn_exp2f((m - M) * c2) + lo * __builtin_amdgcn_exp2f((mo - M) * c2);
    m = M;
  }
  const float L2 = fmaf(m, c2, __builtin_amdgcn_logf(l));      // log2 of the sum of exp(s / 8)
  const float L = L2 * 0.69314718055994531f;
  // second walk: probabilities, and o^T += v^T p^T
  f32x16_t oacc[2] = {zero16(), zero16()};
  for (int kt = 0; kt < NT; ++kt) {
    f32x16_t s = tile_nt(Ks, plane_b, kt * 32, bq, lane);
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c2, -L2));
    if (kt == NT - 1) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (kt * 32 + (i >> 2) * 8 + h * 4 + (i & 3) >= T) s[i] = 0.f;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const bf16x8_t pb = pack_frag(s, j);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
        oacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_read_tr(Vs, plane_b, mt, kt * 32 + 16 * j, lane), pb, oacc[mt], 0, 0, 0);
    }
  }
  if (q < T) {
    store_cols(o + ((size_t)b * T + q) * d + head * kDH, oacc, h);
    if (h == 0) lse[((size_t)b * heads + head) * T + q] = L;
  }
}

__global__ void __launch_bounds__(512) attn_mfma_bwd_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                            const bf16_t* __restrict__ d_o, const float* __restrict__ lse,
                                                            bf16_t* __restrict__ dqkv, int T, int heads) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int NT = blockDim.x >> 6, Tp = NT * 32, plane_b = Tp * ROW_B;
  unsigned char* Qs = smem;
  unsigned char* Ks = smem + 2 * plane_b;
  unsigned char* Vs = smem + 4 * plane_b;
  unsigned char* Gs = smem + 6 * plane_b;
  float* Ls = reinterpret_cast<float*>(smem + 8 * plane_b);
  float* Ds = Ls + Tp;
  const int b = blockIdx.x / heads, head = blockIdx.x % heads, d = heads * kDH;
  const bf16_t* base = qkv + (size_t)b * T * 3 * d + head * kDH;
  const bf16_t* gbase = d_o + (size_t)b * T * d + head * kDH;
  const bf16_t* obase = o + (size_t)b * T * d + head * kDH;
  bf16_t* dbase = dqkv + (size_t)b * T * 3 * d + head * kDH;
  {
    Pieces pq, pk, pv, pg;
    fetch(base, 3 * (size_t)d, T, &pq);
    fetch(base + d, 3 * (size_t)d, T, &pk);
    fetch(base + 2 * d, 3 * (size_t)d, T, &pv);
    fetch(gbase, (size_t)d, T, &pg);
    put(pq, Qs, plane_b);
    put(pk, Ks, plane_b);
    put(pv, Vs, plane_b);
    put(pg, Gs, plane_b);
  }
  for (int t = threadIdx.x; t < Tp; t += blockDim.x) {
    float D = 0.f, L = 0.f;
    if (t < T) {
#pragma unroll
      for (int c = 0; c < kDH; c += 8) {
        float a[8], g[8];
        load8(obase + (size_t)t * d + c, a);
        load8(gbase + (size_t)t * d + c, g);
#pragma unroll
        for (int k = 0; k < 8; ++k) D += a[k] * g[k];
      }
      L = lse[((size_t)b * heads + head) * T + t];
    }
    // stored as the walks use them: exp(s / 8 - L) = exp2(s c - L log2 e) with c = log2 e / 8, and
    // ds = p (dp - D) / 8 = p (dp / 8 - D / 8)
    Ds[t] = D * 0.125f;
    Ls[t] = L * 1.44269504088896341f;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, h = lane >> 5;
  const float scale = 0.125f, c2 = 0.125f * 1.44269504088896341f;
  const int own = wave * 32 + n;           // this lane's query (first walk) or key (second walk)
  // No score is masked in either walk.  Tokens past T are rows of zeros in all four matrices, with
  // L = D = 0: their probabilities are finite, and wherever one enters a sum it multiplies a zero row
  // of the other operand (a key past T: its row of K in dq; a query past T: its rows of dO and Q in dv
  // and dk), or lands in an output column that is not stored (the lane's own token past T).

  // ---- by query block: dq^T = k^T ds^T ----
  {
    bf16x8_t bq[4], bg[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bq[ks] = frag_read(Qs, plane_b, own, ks * 16 + h * 8);
      bg[ks] = frag_read(Gs, plane_b, own, ks * 16 + h * 8);
    }
    const float L2 = Ls[own], Dsc = Ds[own];
    f32x16_t acc[2] = {zero16(), zero16()};
    for (int kt = 0; kt < NT; ++kt) {
      const f32x16_t s = tile_nt(Ks, plane_b, kt * 32, bq, lane);     // [key][query]
      f32x16_t dp = tile_nt(Vs, plane_b, kt * 32, bg, lane);
#pragma unroll
      for (int i = 0; i < 16; ++i) dp[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c2, -L2)) * fmaf(dp[i], scale, -Dsc);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const bf16x8_t dsb = pack_frag(dp, j);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
          acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_read_tr(Ks, plane_b, mt, kt * 32 + 16 * j, lane), dsb, acc[mt], 0, 0, 0);
      }
    }
    if (own < T) store_cols(dbase + (size_t)own * 3 * d, acc, h);
  }
  // ---- by key block: dv^T = do^T p, dk^T = q^T ds ----
  {
    bf16x8_t bk[4], bv[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bk[ks] = frag_read(Ks, plane_b, own, ks * 16 + h * 8);
      bv[ks] = frag_read(Vs, plane_b, own, ks * 16 + h * 8);
    }
    f32x16_t dk[2] = {zero16(), zero16()}, dv[2] = {zero16(), zero16()};
    for (int qt = 0; qt < NT; ++qt) {
      f32x16_t p = tile_nt(Qs, plane_b, qt * 32, bk, lane);           // [query][key]
      f32x16_t dp = tile_nt(Gs, plane_b, qt * 32, bv, lane);
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int r0 = qt * 32 + i4 * 8 + h * 4;
        const float4 L4 = *reinterpret_cast<const float4*>(Ls + r0);
        const float4 D4 = *reinterpret_cast<const float4*>(Ds + r0);
        const float Lr[4] = {L4.x, L4.y, L4.z, L4.w}, Dr[4] = {D4.x, D4.y, D4.z, D4.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int i = i4 * 4 + k;
          const float pp = __builtin_amdgcn_exp2f(fmaf(p[i], c2, -Lr[k]));
          p[i] = pp;
          dp[i] = pp * fmaf(dp[i], scale, -Dr[k]);
        }
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const bf16x8_t pb = pack_frag(p, j), dsb = pack_frag(dp, j);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          dv[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_read_tr(Gs, plane_b, mt, qt * 32 + 16 * j, lane), pb, dv[mt], 0, 0, 0);
          dk[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_read_tr(Qs, plane_b, mt, qt * 32 + 16 * j, lane), dsb, dk[mt], 0, 0, 0);
        }
      }
    }
    if (own < T) {
      store_cols(dbase + (size_t)own * 3 * d + d, dk, h);
      store_cols(dbase + (size_t)own * 3 * d + 2 * d, dv, h);
    }
  }
}
}  // namespace

bool attn_mfma_supported(const cnnk_attn_desc* d) {
  return d->dtype == CNNK_BF16 && d->dh == kDH && d->T <= 256;
}

int attn_mfma_fwd(const cnnk_attn_desc* d, const void* qkv, void* o, float* lse, hipStream_t st) {
  const int NT = (d->T + 31) / 32;
  const size_t lds = (size_t)4 * NT * 32 * ROW_B;
  static bool raised = false;
  if (!raised) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_fwd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 8 * 32 * 4 * ROW_B) != hipSuccess)
      return CNNK_ERR_HIP;
    raised = true;
  }
  attn_mfma_fwd_kernel<<<d->B * d->heads, 64 * NT, lds, st>>>((const bf16_t*)qkv, (bf16_t*)o, lse, d->T, d->heads);
  return launch_status();
}

int attn_mfma_bwd(const cnnk_attn_desc* d, const void* qkv, const void* o, const void* d_o, const float* lse, void* dqkv,
                  hipStream_t st) {
  const int NT = (d->T + 31) / 32;
  const size_t lds = (size_t)8 * NT * 32 * ROW_B + (size_t)2 * NT * 32 * sizeof(float);
  static bool raised = false;
  if (!raised) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_bwd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            8 * 8 * 32 * ROW_B + 2 * 8 * 32 * 4) != hipSuccess)
      return CNNK_ERR_HIP;
    raised = true;
  }
  attn_mfma_bwd_kernel<<<d->B * d->heads, 64 * NT, lds, st>>>((const bf16_t*)qkv, (const bf16_t*)o, (const bf16_t*)d_o, lse,
                                                            (bf16_t*)dqkv, d->T, d->heads);
  return launch_status();
}
