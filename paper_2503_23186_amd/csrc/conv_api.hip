// C-ABI front end of the convolution passes: validation, workspace sizing, and the choice
// between the bf16 MFMA implicit-GEMM kernels and the direct kernels.
#include "common.h"
#include "conv.h"

int cnnk_validate_conv(const cnnk_conv_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0 || d->R <= 0 || d->S <= 0 ||
      d->stride <= 0 || d->pad < 0)
    return CNNK_ERR_SHAPE;
  if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (d->R != d->S || (d->R != 1 && d->R != 3) || d->pad != d->R / 2 || d->stride > 2) return CNNK_ERR_UNSUPPORTED;
  const ConvGeom g = make_geom(d);
  const double lim = 2147483647.0;
  if ((double)g.N * g.H * g.W * g.Cin > lim || (double)g.N * g.Ho * g.Wo * g.Cout > lim ||
      (double)g.Cout * g.R * g.S * g.Cin > lim)
    return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}

static bool use_mfma(const cnnk_conv_desc* d, const ConvGeom& g, int pass) {
  return d->dtype == CNNK_BF16 && conv_mfma_supported(g, pass);
}
static bool use_pad(const cnnk_conv_desc* d, const ConvGeom& g, int pass) {
  return d->dtype == CNNK_BF16 && pass != CNNK_PASS_DGRAD && g_cnnk_tune[8] >= 0 && conv_pad_supported(g);
}
static bool use_first(const cnnk_conv_desc* d, const ConvGeom& g) {   // forward only
  return d->dtype == CNNK_BF16 && g_cnnk_tune[8] >= 0 && g_cnnk_tune[11] >= 0 && conv_first_supported(g);
}
static bool use_first_wgrad(const cnnk_conv_desc* d, const ConvGeom& g) {
  return d->dtype == CNNK_BF16 && g_cnnk_tune[8] >= 0 && g_cnnk_tune[11] >= 0 && conv_first_wgrad_supported(g);
}

extern "C" size_t cnnk_conv2d_workspace_bytes(const cnnk_conv_desc* d, int pass) {
  if (cnnk_validate_conv(d) != CNNK_OK) return 0;
  const ConvGeom g = make_geom(d);
  size_t b = 0;
  if (pass == CNNK_PASS_FWD) {
    // room for the per-channel statistics pass over y when the caller asks for ch_sum/ch_sumsq
    b = (g.Cout % 8 == 0 && g.Cout <= 2048) ? channel_stats_ws((size_t)g.N * g.Ho * g.Wo, g.Cout) : 0;
    if (use_mfma(d, g, pass)) { const size_t m = conv_mfma_ws(g, pass, true); if (m > b) b = m; }
    if (use_pad(d, g, pass)) { const size_t m = conv_pad_ws(g, pass, true); if (m > b) b = m; }
    if (use_first(d, g)) { const size_t m = conv_first_ws(g); if (m > b) b = m; }
  } else if (pass == CNNK_PASS_DGRAD) {
    b = use_mfma(d, g, pass) ? conv_mfma_ws(g, pass, false) : 0;
  } else if (pass == CNNK_PASS_WGRAD) {
    b = use_mfma(d, g, pass) ? conv_mfma_ws(g, pass, false)
        : use_first_wgrad(d, g) ? conv_first_wgrad_ws(g)
        : use_pad(d, g, pass) ? conv_pad_ws(g, pass, false) : conv_direct_wgrad_ws(g);
  }
  return align_up(b, 256);
}

extern "C" int cnnk_conv2d_fwd(const cnnk_conv_desc* d, const void* x, const void* w, void* y, float* ch_sum,
                               float* ch_sumsq, void* ws, size_t ws_bytes, void* stream) {
  int rc = cnnk_validate_conv(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !w || !y) return CNNK_ERR_NULL;
  if ((ch_sum == nullptr) != (ch_sumsq == nullptr)) return CNNK_ERR_NULL;
  const ConvGeom g = make_geom(d);
  if (ch_sum) {
    if (g.Cout % 8 != 0 || g.Cout > 2048) return CNNK_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < cnnk_conv2d_workspace_bytes(d, CNNK_PASS_FWD)) return CNNK_ERR_WORKSPACE;
  }
  hipStream_t st = (hipStream_t)stream;
  if (use_mfma(d, g, CNNK_PASS_FWD))
    return conv_mfma_fwd(g, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, ch_sum, ch_sumsq, ws, st);
  if (use_first(d, g))
    return conv_first_fwd(g, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, ch_sum, ch_sumsq, ws, st);
  if (use_pad(d, g, CNNK_PASS_FWD)) {
    if (!ws || ws_bytes < cnnk_conv2d_workspace_bytes(d, CNNK_PASS_FWD)) return CNNK_ERR_WORKSPACE;
    return conv_pad_fwd(g, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, ch_sum, ch_sumsq, ws, st);
  }
  rc = conv_direct_fwd(g, d->dtype, x, w, y, st);
  if (rc != CNNK_OK) return rc;
  if (ch_sum) rc = channel_stats(d->dtype, y, (size_t)g.N * g.Ho * g.Wo, g.Cout, ch_sum, ch_sumsq, ws, st);
  return rc;
}

extern "C" int cnnk_conv2d_dgrad(const cnnk_conv_desc* d, const void* dy, const void* w, void* dx, int accumulate,
                                 void* ws, size_t ws_bytes, void* stream) {
  int rc = cnnk_validate_conv(d);
  if (rc != CNNK_OK) return rc;
  if (!dy || !w || !dx) return CNNK_ERR_NULL;
  const ConvGeom g = make_geom(d);
  hipStream_t st = (hipStream_t)stream;
  if (use_mfma(d, g, CNNK_PASS_DGRAD)) {
    if (!ws || ws_bytes < cnnk_conv2d_workspace_bytes(d, CNNK_PASS_DGRAD)) return CNNK_ERR_WORKSPACE;
    return conv_mfma_dgrad(g, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, accumulate, ws, st);
  }
  return conv_direct_dgrad(g, d->dtype, dy, w, dx, accumulate, st);
}

extern "C" int cnnk_conv2d_wgrad(const cnnk_conv_desc* d, const void* x, const void* dy, float* dw, void* ws,
                                 size_t ws_bytes, void* stream) {
  int rc = cnnk_validate_conv(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !dy || !dw) return CNNK_ERR_NULL;
  const ConvGeom g = make_geom(d);
  hipStream_t st = (hipStream_t)stream;
  const size_t need = cnnk_conv2d_workspace_bytes(d, CNNK_PASS_WGRAD);
  if (need && (!ws || ws_bytes < need)) return CNNK_ERR_WORKSPACE;
  if (use_mfma(d, g, CNNK_PASS_WGRAD))
    return conv_mfma_wgrad(g, (const bf16_t*)x, (const bf16_t*)dy, dw, ws, st);
  if (use_first_wgrad(d, g)) return conv_first_wgrad(g, (const bf16_t*)x, (const bf16_t*)dy, dw, ws, st);
  if (use_pad(d, g, CNNK_PASS_WGRAD)) return conv_pad_wgrad(g, (const bf16_t*)x, (const bf16_t*)dy, dw, ws, st);
  return conv_direct_wgrad(g, d->dtype, x, dy, dw, ws, st);
}

extern "C" const char* cnnk_status_string(int s) {
  switch (s) {
    case CNNK_OK: return "ok";
    case CNNK_ERR_NULL: return "a required pointer is NULL";
    case CNNK_ERR_SHAPE: return "non-positive or inconsistent sizes";
    case CNNK_ERR_UNSUPPORTED: return "shape or dtype outside the supported set";
    case CNNK_ERR_WORKSPACE: return "workspace missing or too small";
    case CNNK_ERR_HIP: return "HIP runtime error at launch";
    default: return "unknown status";
  }
}

extern "C" int cnnk_tune(int key, int value) {
  if (key < 0 || key >= 16) return CNNK_ERR_SHAPE;
  g_cnnk_tune[key] = value;
  return CNNK_OK;
}

extern "C" const char* cnnk_version(void) { return "cnnk 0.1 (gfx950)"; }
