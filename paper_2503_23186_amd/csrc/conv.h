// Internal interfaces between the convolution front end (conv_api.hip) and its kernel families.
#pragma once
#include "common.h"

struct ConvGeom {
  int N, H, W, Cin, Cout, R, S, stride, pad, Ho, Wo;
};

static inline ConvGeom make_geom(const cnnk_conv_desc* d) {
  ConvGeom g;
  g.N = d->N; g.H = d->H; g.W = d->W; g.Cin = d->Cin; g.Cout = d->Cout;
  g.R = d->R; g.S = d->S; g.stride = d->stride; g.pad = d->pad;
  g.Ho = conv_out(d->H, d->pad, d->R, d->stride);
  g.Wo = conv_out(d->W, d->pad, d->S, d->stride);
  return g;
}

// direct kernels (any shape, both dtypes)
size_t conv_direct_wgrad_ws(const ConvGeom& g);
int conv_direct_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, void* y, hipStream_t st);
int conv_direct_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                      hipStream_t st);
int conv_direct_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                      hipStream_t st);
int reduce_partials(const float* part, float* out, int n, int P, hipStream_t st);

// bf16 MFMA implicit-GEMM kernels
bool conv_mfma_supported(const ConvGeom& g, int pass);
size_t conv_mfma_ws(const ConvGeom& g, int pass, bool want_stats);
int conv_mfma_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* ch_sum,
                  float* ch_sumsq, void* ws, hipStream_t st);
int conv_mfma_dgrad(const ConvGeom& g, const bf16_t* dy, const bf16_t* w, bf16_t* dx, int accumulate,
                    void* ws, hipStream_t st);
int conv_mfma_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws,
                    hipStream_t st);
// The same without the final reduction: *part points at *P partial gradients (each Cout*R*S*Cin
// floats; dw itself with *P = 1 when the reduction was not split), for a caller that reduces them
// in its own way.
int conv_mfma_wgrad_partials(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws,
                             const float** part, int* P, hipStream_t st);

// data gradient with weights already transposed to [Cin][R*S][Cout], and the batched transposition
constexpr int kMaxTranspose = 32;
struct TransposeTable {
  int count;
  int block_begin[kMaxTranspose + 1];
  const bf16_t* src[kMaxTranspose];
  bf16_t* dst[kMaxTranspose];
  int Cout[kMaxTranspose], T[kMaxTranspose], Cin[kMaxTranspose];
};
int conv_transpose_weights_multi(TransposeTable& t, hipStream_t st);
int conv_mfma_dgrad_pt(const ConvGeom& g, const bf16_t* dy, const bf16_t* wt, bf16_t* dx, int accumulate,
                       hipStream_t st);

// 3x3 stride-1 kernels with the input patch resident in LDS (forward, data gradient)
bool conv_patch_supported(const ConvGeom& g, int pass);
int conv_patch_stat_rows(const ConvGeom& g);
int conv_patch_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* stats, hipStream_t st);
int conv_patch_dgrad(const ConvGeom& g, const bf16_t* dy, const bf16_t* wt, bf16_t* dx, int accumulate,
                     hipStream_t st);

// 3x3 stride-1 weight gradient from LDS patches with transposing LDS loads
bool conv_wgrad_patch_supported(const ConvGeom& g);
size_t conv_wgrad_patch_ws(const ConvGeom& g);
int conv_wgrad_patch(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st);
// the same partial sums with the operand tiles loaded straight into LDS (conv_wgrad_dma.hip)
int conv_wgrad_dma_launch(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* part, int TI, int TH, int ctiles,
                          int tiles_per_block, int mtiles, int nw, int otiles, int splits, hipStream_t st);

// fewer than 8 input channels: zero-pad to 8 in the workspace, then the MFMA kernels
bool conv_pad_supported(const ConvGeom& g);
size_t conv_pad_ws(const ConvGeom& g, int pass, bool want_stats);
int conv_pad_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* ch_sum, float* ch_sumsq,
                 void* ws, hipStream_t st);
int conv_pad_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st);
// Hook 1 of 3 (see "Hooks between cnnk_train_step and the convolution entry points" below).
// The forward and the weight-gradient call of such a layer both need the 8-channel copy of x.  When
// set (per host thread), the forward call writes it to buf and sets valid, and a weight-gradient
// call that finds valid set reads it there instead of padding x again (the caller vouches that x
// and buf are unchanged in between).
size_t conv_pad_x8_bytes(const ConvGeom& g);
struct X8Cache {
  bf16_t* buf;
  bool valid;
};
extern thread_local X8Cache* t_cnnk_x8_cache;

// first layer (3 input channels, 3x3, stride 1, pad 1, at most 64 output channels): forward on MFMA
// without operand staging
bool conv_first_supported(const ConvGeom& g);
size_t conv_first_ws(const ConvGeom& g);
int conv_first_fwd(const ConvGeom& g, const bf16_t* x, const bf16_t* w, bf16_t* y, float* ch_sum, float* ch_sumsq,
                   void* ws, hipStream_t st);
bool conv_first_wgrad_supported(const ConvGeom& g);   // additionally W % 16 == 0
size_t conv_first_wgrad_ws(const ConvGeom& g);
int conv_first_wgrad(const ConvGeom& g, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st);

// ch_sum[c] = sum_b part[b][0][c], ch_sumsq[c] = sum_b part[b][1][c]  (double accumulation)
int channel_sums_finalize(const float* part, int nb, int C, float* ch_sum, float* ch_sumsq, hipStream_t st);

// ---- Hooks between cnnk_train_step and the convolution entry points -----------------------------
// cnnk_train_step calls the public entry points (cnnk_conv2d_fwd / _wgrad) and passes three extra
// pieces of context through the per-thread pointers below (t_cnnk_x8_cache above, t_cnnk_sgd_fuse,
// t_cnnk_wgrad_cus).  Contract, the same for all three: the step sets the pointer immediately
// before ONE entry-point call on the same host thread and resets it to its neutral value (nullptr /
// 256) right after that call returns, whatever the call's status; an entry point reads it once, at
// entry.  Outside cnnk_train_step the values are always neutral, so a direct caller of the C ABI
// never sees them, and calls from other host threads are unaffected (thread_local).  The library
// keeps no other state between calls except two process-wide tables that are written once or by
// an explicit call: the "dynamic LDS size already raised" flag of each kernel launcher (set on the
// first launch; harmless to set twice, so unsynchronised first launches from two threads are
// benign) and the cnnk_tune table (explicitly documented as not thread-safe).
//
// Hook 2 of 3.  When set (per host thread), the next split-K reduction of a weight gradient also applies the
// SGD-momentum update of that parameter in the same launch (out = sum of partials is still
// written as the gradient): g' = g + wd*w; v <- mu*v + g'; w <- w - lr*v; optional bf16 copy.
// wait (nullable): an event the stream waits for between the weight-gradient kernel and the
// reduction (the last reader of the old weights).  done is set when the fused launch was made;
// callers fall back to a separate update otherwise (unsplit reductions, other reducers).
struct SgdFuse {
  float* w;
  float* v;
  void* wlp;
  float lr, mu, wd;
  hipEvent_t wait;
  bool done;
};
extern thread_local SgdFuse* t_cnnk_sgd_fuse;

extern int g_cnnk_tune[16];
// Hook 3 of 3.  Compute units the weight-gradient kernels size their grids for (256 = the whole device).  The
// training step lowers it for the weight gradients it runs on its second stream, beside the rest
// of the backward pass: fewer, longer-lived workgroups leave the other stream room to run.
// Workspace sizes are always computed for the whole device (the upper bound).
extern thread_local int t_cnnk_wgrad_cus;

// per-channel sum / sum of squares of a tensor with C channels (used when the conv kernel
// itself does not produce them)
size_t channel_stats_ws(size_t m, int C);
int channel_stats(int dtype, const void* x, size_t m, int C, float* ch_sum, float* ch_sumsq, void* ws,
                  hipStream_t st);
