// Weight gradient of a 3x3 stride-1 convolution with both operands read from LDS in their
// natural [pixel][channel] layout through the gfx950 transposing LDS load (ds_read_b64_tr_b16):
// support test, split plan and launcher; the kernel is in conv_wgrad_dma.hip.
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
constexpr int kRowsPerPass = kThreads / 8;                  // patch positions per unit of the kernel's PL parameter

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
  int rc = conv_wgrad_dma_launch(g, x, dy, a.dw, a.TI, a.TH, a.ctiles, a.tiles_per_block, a.mtiles, a.nw, otiles, splits, st);
  if (rc != CNNK_OK || splits == 1) return rc;
  return reduce_partials(a.dw, dw, a.nw, splits, st);
}
