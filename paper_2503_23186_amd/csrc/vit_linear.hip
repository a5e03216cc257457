// Linear layers of the Vision Transformer step (cnnk_linear_* of cnnk_vit.h): the choice between the
// dense bf16 matrix-core kernels (gemm_bf16.hip) and, for fp32 storage or shapes those do not take,
// the 1 x 1 convolution kernels followed by the bias / activation kernel.
#include "common.h"
#include "gemm.h"
#include "../../include/cnnk_vit.h"

extern int g_cnnk_tune[16];

namespace {
int check(long long rows, int K, int N, int dtype) {
  if (rows <= 0 || K <= 0 || N <= 0) return CNNK_ERR_SHAPE;
  if (dtype != CNNK_F32 && dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (rows > 2147483647LL || K % 8 != 0 || N % 8 != 0) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}
bool fast(long long rows, int K, int N, int dtype) {
  return dtype == CNNK_BF16 && g_cnnk_tune[15] >= 0 && gemm_bf16_supported(rows, K, N);
}
cnnk_conv_desc as_conv(long long rows, int K, int N, int dtype) {
  cnnk_conv_desc c;
  c.N = 1; c.H = (int)rows; c.W = 1; c.Cin = K; c.Cout = N; c.R = 1; c.S = 1; c.stride = 1; c.pad = 0; c.dtype = dtype;
  return c;
}
}  // namespace

extern "C" size_t cnnk_linear_workspace_bytes(long long rows, int K, int N, int dtype) {
  if (check(rows, K, N, dtype) != CNNK_OK) return 0;
  size_t w = 0;
  if (fast(rows, K, N, dtype)) w = gemm_bf16_wgrad_ws(rows, K, N);
  const cnnk_conv_desc c = as_conv(rows, K, N, dtype);
  for (int pass = 0; pass < 3; ++pass) {
    const size_t b = cnnk_conv2d_workspace_bytes(&c, pass);
    if (b > w) w = b;
  }
  return align_up(w, 256);
}

extern "C" int cnnk_linear_fwd(long long rows, int K, int N, int dtype, const void* x, const void* w, const float* bias,
                               const void* res, int act, void* u, void* y, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check(rows, K, N, dtype);
  if (rc != CNNK_OK) return rc;
  if (act != CNNK_ACT_NONE && act != CNNK_ACT_GELU) return CNNK_ERR_UNSUPPORTED;
  if (!x || !w || !y || (act == CNNK_ACT_GELU && (!u || !bias))) return CNNK_ERR_NULL;
  if ((act == CNNK_ACT_GELU && res) || (res && res == y)) return CNNK_ERR_UNSUPPORTED;
  if (((size_t)x | (size_t)w | (size_t)y | (size_t)u | (size_t)res) & 15) return CNNK_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  if (fast(rows, K, N, dtype))
    return gemm_bf16_fwd(rows, K, N, (const bf16_t*)x, (const bf16_t*)w, bias, (const bf16_t*)res, act == CNNK_ACT_GELU, (bf16_t*)u,
                         (bf16_t*)y, st);
  const cnnk_conv_desc c = as_conv(rows, K, N, dtype);
  void* z = act == CNNK_ACT_GELU ? u : y;
  int r2 = cnnk_conv2d_fwd(&c, x, w, z, nullptr, nullptr, ws, ws_bytes, stream);
  if (r2 == CNNK_OK && bias) r2 = cnnk_bias_act_fwd(rows, N, dtype, act, z, bias, nullptr, u, y, stream);
  if (r2 == CNNK_OK && res) r2 = cnnk_add((size_t)rows * N, dtype, res, y, y, stream);   // the same two roundings
  return r2;
}

extern "C" int cnnk_linear_dgrad(long long rows, int K, int N, int dtype, const void* dy, const void* w, void* dx, void* ws,
                                 size_t ws_bytes, void* stream) {
  const int rc = check(rows, K, N, dtype);
  if (rc != CNNK_OK) return rc;
  if (!dy || !w || !dx) return CNNK_ERR_NULL;
  if (((size_t)dy | (size_t)w | (size_t)dx) & 15) return CNNK_ERR_UNSUPPORTED;
  if (fast(rows, K, N, dtype)) return gemm_bf16_dgrad(rows, K, N, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, (hipStream_t)stream);
  const cnnk_conv_desc c = as_conv(rows, K, N, dtype);
  return cnnk_conv2d_dgrad(&c, dy, w, dx, 0, ws, ws_bytes, stream);
}

extern "C" int cnnk_linear_wgrad(long long rows, int K, int N, int dtype, const void* x, const void* dy, float* dw, void* ws,
                                 size_t ws_bytes, void* stream) {
  const int rc = check(rows, K, N, dtype);
  if (rc != CNNK_OK) return rc;
  if (!x || !dy || !dw) return CNNK_ERR_NULL;
  if (((size_t)x | (size_t)dy | (size_t)dw) & 15) return CNNK_ERR_UNSUPPORTED;
  if (fast(rows, K, N, dtype)) {
    const size_t need = gemm_bf16_wgrad_ws(rows, K, N);
    if (need && (!ws || ws_bytes < need)) return CNNK_ERR_WORKSPACE;
    return gemm_bf16_wgrad(rows, K, N, (const bf16_t*)x, (const bf16_t*)dy, dw, ws, (hipStream_t)stream);
  }
  const cnnk_conv_desc c = as_conv(rows, K, N, dtype);
  return cnnk_conv2d_wgrad(&c, x, dy, dw, ws, ws_bytes, stream);
}
