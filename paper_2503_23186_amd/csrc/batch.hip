// Two small data-movement kernels of the loop around the step: the bf16 copy of fp32 master
// parameters (bf16 mode reads the convolution weights in bf16; cnnk_sgd_momentum refreshes the
// copy after every update, this call makes the first one) and the assembly of a mini-batch out of
// a device-resident data set (Algorithm 1: "for each mini-batch").
#include "common.h"

namespace {
constexpr int kT = 256;

__global__ void __launch_bounds__(kT) round_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst,
                                                        size_t n) {
  for (size_t i = (size_t)blockIdx.x * kT + threadIdx.x; i < n; i += (size_t)gridDim.x * kT) dst[i] = f32_to_bf16(src[i]);
}

// dst row i = src row idx[i]; rows of row_bytes bytes, moved as 16-byte vectors when VEC, else
// 4-byte words (row_bytes is a multiple of 4; rows start 16-byte aligned in the VEC case).  One
// workgroup walks whole rows, so the index is read once per row and workgroup.
template <bool VEC>
__global__ void __launch_bounds__(kT) gather_rows_kernel(const unsigned char* __restrict__ src,
                                                         const long long* __restrict__ idx,
                                                         unsigned char* __restrict__ dst, int n_rows,
                                                         long long n_src_rows, size_t row_bytes, int* bad) {
  for (int r = blockIdx.x; r < n_rows; r += gridDim.x) {
    const long long s = idx[r];
    if (s < 0 || s >= n_src_rows) {   // refused, not read: the row is zero-filled and the error flag set
      if (threadIdx.x == 0 && bad) *bad = 1;
      if (VEC) for (size_t o = (size_t)threadIdx.x * 16; o < row_bytes; o += (size_t)kT * 16)
        *reinterpret_cast<uint4*>(dst + (size_t)r * row_bytes + o) = make_uint4(0u, 0u, 0u, 0u);
      else for (size_t o = (size_t)threadIdx.x * 4; o < row_bytes; o += (size_t)kT * 4)
        *reinterpret_cast<unsigned*>(dst + (size_t)r * row_bytes + o) = 0u;
      continue;
    }
    const unsigned char* sp = src + (size_t)s * row_bytes;
    unsigned char* dp = dst + (size_t)r * row_bytes;
    if (VEC) for (size_t o = (size_t)threadIdx.x * 16; o < row_bytes; o += (size_t)kT * 16)
      *reinterpret_cast<uint4*>(dp + o) = *reinterpret_cast<const uint4*>(sp + o);
    else for (size_t o = (size_t)threadIdx.x * 4; o < row_bytes; o += (size_t)kT * 4)
      *reinterpret_cast<unsigned*>(dp + o) = *reinterpret_cast<const unsigned*>(sp + o);
  }
}
}  // namespace

extern "C" int cnnk_round_bf16(size_t n, const float* src, void* dst_bf16, void* stream) {
  if (n == 0) return CNNK_OK;
  if (!src || !dst_bf16) return CNNK_ERR_NULL;
  size_t blocks = (n + kT - 1) / kT;
  if (blocks > 4096) blocks = 4096;
  round_bf16_kernel<<<(unsigned)blocks, kT, 0, (hipStream_t)stream>>>(src, (bf16_t*)dst_bf16, n);
  return launch_status();
}

extern "C" int cnnk_gather_rows(int n_rows, long long n_src_rows, size_t row_bytes, const void* src,
                                const long long* idx, void* dst, int* bad_index, void* stream) {
  if (n_rows == 0) return CNNK_OK;
  if (n_rows < 0 || n_src_rows <= 0 || row_bytes == 0 || row_bytes % 4 != 0) return CNNK_ERR_SHAPE;
  if (!src || !idx || !dst) return CNNK_ERR_NULL;
  if ((((size_t)src | (size_t)dst) & 3) != 0) return CNNK_ERR_UNSUPPORTED;
  const bool vec = row_bytes % 16 == 0 && ((((size_t)src | (size_t)dst) & 15) == 0);
  const unsigned blocks = (unsigned)(n_rows < 4096 ? n_rows : 4096);
  if (vec)
    gather_rows_kernel<true><<<blocks, kT, 0, (hipStream_t)stream>>>((const unsigned char*)src, idx, (unsigned char*)dst,
                                                                   n_rows, n_src_rows, row_bytes, bad_index);
  else
    gather_rows_kernel<false><<<blocks, kT, 0, (hipStream_t)stream>>>((const unsigned char*)src, idx, (unsigned char*)dst,
                                                                    n_rows, n_src_rows, row_bytes, bad_index);
  return launch_status();
}
