/* cnnk: one device's CNN training step (forward, loss, backward, SGD-momentum update) on gfx950.
 *
 * The operations are those of the inner mini-batch loop of the paper's Algorithm 1
 * ("perform forward pass", "compute loss L(theta)", "perform backward pass", "update
 * parameters theta = theta - eta * grad") as one data-parallel replica executes them
 * (Section III-A, data parallelism: every device holds the whole model and processes its own
 * share of the batch).  The model family is the image-classification CNN of Section IV-A
 * (ResNet-style networks on 32x32 RGB inputs, 100 classes).
 *
 * Conventions common to every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller; descriptors are host structs.
 *  - The library never allocates, frees or synchronises.  Work is enqueued on `stream` (a
 *    hipStream_t passed as void*, NULL = the default stream) and the call returns at once.
 *  - Layout: activations NHWC; convolution weights [Cout][R][S][Cin]; FC weight [classes][F].
 *  - dtype CNNK_F32: every tensor is float.  dtype CNNK_BF16: activations, activation gradients
 *    and the convolution weights handed to the conv calls are bfloat16 (round to nearest even);
 *    BN statistics and parameters, all parameter gradients, FC parameters, master weights,
 *    momentum, logits and the loss stay float.  Accumulation is always fp32.
 *  - Errors are return codes.  Arguments are validated on the host before anything is
 *    enqueued: a call that returns an error other than CNNK_ERR_HIP has launched nothing.
 *  - Outputs must not alias inputs unless stated.
 *  - Threads and streams: every entry point may be called from any host thread; calls that share
 *    device buffers or a workspace must be ordered by the caller (same stream, or events).  The
 *    library keeps no state between calls apart from cnnk_tune's table (process-wide, not
 *    thread-safe) and, inside cnnk_train_step only, per-thread context that the step hands to the
 *    convolution calls it makes (invisible to other threads and to direct callers).
 *  - Workspace (`ws`, `ws_bytes`): scratch device memory, at least the size the matching
 *    *_workspace_bytes query returns (may be NULL when that is 0), 256-byte aligned.
 *    Contents are undefined on entry and on return.
 */
#ifndef CNNK_H
#define CNNK_H
#include <stddef.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CNNK_OK = 0,
  CNNK_ERR_NULL = 1,        /* a required pointer is NULL */
  CNNK_ERR_SHAPE = 2,       /* non-positive or inconsistent sizes */
  CNNK_ERR_UNSUPPORTED = 3, /* valid but outside the supported set */
  CNNK_ERR_WORKSPACE = 4,   /* workspace missing or too small */
  CNNK_ERR_HIP = 5          /* the HIP runtime refused a launch */
} cnnk_status;

typedef enum { CNNK_F32 = 0, CNNK_BF16 = 1 } cnnk_dtype;
typedef enum { CNNK_POOL_MAX2 = 0, CNNK_POOL_GAP = 1 } cnnk_pool_mode;
typedef enum { CNNK_PASS_FWD = 0, CNNK_PASS_DGRAD = 1, CNNK_PASS_WGRAD = 2 } cnnk_conv_pass;

/* Output extent: Ho = (H + 2*pad - R)/stride + 1 (integer division), same for Wo. */
typedef struct { int N, H, W, Cin, Cout, R, S, stride, pad; int dtype; } cnnk_conv_desc;
typedef struct { int N, H, W, C; int dtype; float eps, momentum; int relu; } cnnk_bn_desc;
typedef struct { int N, H, W, C; int dtype; int mode; } cnnk_pool_desc;
typedef struct { int N, F, classes; int dtype; } cnnk_fc_desc;

const char* cnnk_status_string(int status);
/* Library version, and the code-object architecture the kernels were built for ("gfx950"). */
const char* cnnk_version(void);

/* Tuning hook for benchmarking, not needed for normal use: overrides one of the library's
 * launch heuristics (value 0 restores the built-in choice).  Keys: 0/1/2 = rows / columns /
 * reduction depth of the implicit-GEMM tile of the forward and data-gradient kernels
 * (unsupported combinations make the conv calls return CNNK_ERR_UNSUPPORTED); 3 = target
 * number of workgroups of the weight-gradient kernel; 4/5 = pixel / channel tile of the 3x3
 * stride-1 LDS-patch kernels (4 = -1 switches them off); 6 = target number of workgroups of
 * the 3x3 stride-1 weight-gradient kernel (-1 switches it off); 10 = -1 keeps cnnk_attention_fwd / _bwd (cnnk_vit.h) on the vector-ALU kernels, 15 = -1 keeps cnnk_linear_* on the 1 x 1 convolution kernels, 1 / 2 keeps their matrix-core kernels on 64-byte / 128-byte operand rows in LDS whatever the shape; 7 = -1 switches off the pixel
 * permutation that keeps narrow images (W < 16) free of LDS bank conflicts; 8 = -1 keeps convolutions with
 * fewer than 8 input channels on the direct (plain-FMA) kernels; 11 = -1 keeps the first layer's forward
 * pass on the padded-input path; 9 = -1 makes cnnk_train_step hand y to
 * every batch-norm backward call (no mask recomputation); 12 = -1 keeps the weight transposes of
 * the data-gradient kernels on the main stream when cnnk_train_step has a second one; 14 = tiles that one workgroup of the
 * gathered implicit-GEMM kernels walks (0: as many as still fill every CU); 13 = pixel tiles that one workgroup of
 * the 3x3 stride-1 LDS-patch kernels walks (0: as many as still leave two workgroups per CU; -1: one, and no
 * split of the reduction over two groups of wavefronts on grids of fewer than 512 workgroups).
 * Process-wide, not thread-safe. */
int cnnk_tune(int key, int value);

/* ---- convolution (Algorithm 1: forward pass / backward pass of a conv layer) -------------- */

/* Scratch bytes needed by the given pass (cnnk_conv_pass) of this convolution. */
size_t cnnk_conv2d_workspace_bytes(const cnnk_conv_desc* d, int pass);

/* y[n,ho,wo,k] = sum_{r,s,c} x[n,ho*stride+r-pad,wo*stride+s-pad,c] * w[k,r,s,c], zero padding,
 * no bias.  x: N*H*W*Cin, w: Cout*R*S*Cin, y: N*Ho*Wo*Cout, all of d->dtype.
 * ch_sum / ch_sumsq (both or neither; nullable): Cout floats each, receive sum_m y and
 * sum_m y^2 over the N*Ho*Wo output positions of the fp32 accumulators (input to batch norm).
 * Supported: R==S in {1,3}, stride in {1,2}, pad == R/2. */
int cnnk_conv2d_fwd(const cnnk_conv_desc* d, const void* x, const void* w, void* y,
                    float* ch_sum, float* ch_sumsq, void* ws, size_t ws_bytes, void* stream);

/* dx[n,h,w,c] = sum_{k,r,s} dy[n,(h+pad-r)/stride,(w+pad-s)/stride,k] * w[k,r,s,c] over the
 * (r,s) whose quotients are integers inside the output image.  accumulate != 0 adds the result
 * to the existing contents of dx (a tensor with two consumers receives the sum of both
 * gradients), otherwise dx is overwritten. */
int cnnk_conv2d_dgrad(const cnnk_conv_desc* d, const void* dy, const void* w, void* dx,
                      int accumulate, void* ws, size_t ws_bytes, void* stream);

/* dw[k,r,s,c] = sum_{n,ho,wo} dy[n,ho,wo,k] * x[n,ho*stride+r-pad,wo*stride+s-pad,c].
 * dw is float in both dtypes and is overwritten. */
int cnnk_conv2d_wgrad(const cnnk_conv_desc* d, const void* x, const void* dy, float* dw,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- batch norm (+ residual) (+ ReLU) ------------------------------------------------------ */

size_t cnnk_bn_workspace_bytes(const cnnk_bn_desc* d);

/* Training-mode batch norm over m = N*H*W positions per channel:
 * mean = (1/m) sum x; var = (1/m) sum (x-mean)^2; invstd = 1/sqrt(var+eps);
 * y = act(gamma*(x-mean)*invstd + beta [+ residual]), act = max(.,0) if d->relu else identity.
 * save_mean, save_invstd: C floats each (needed by the backward call).
 * running_mean/var (both or neither; nullable, updated in place): r <- (1-momentum)*r +
 * momentum*stat, with the unbiased variance var*m/(m-1).
 * ch_sum/ch_sumsq (both or neither; nullable): per-channel sum x and sum x^2 produced by
 * cnnk_conv2d_fwd; when given, the statistics pass over x is skipped. */
int cnnk_bn_relu_fwd(const cnnk_bn_desc* d, const void* x, const void* residual,
                     const float* gamma, const float* beta, void* y, float* save_mean,
                     float* save_invstd, float* running_mean, float* running_var,
                     const float* ch_sum, const float* ch_sumsq, void* ws, size_t ws_bytes,
                     void* stream);

/* Inference-mode batch norm, for the validation pass of Algorithm 1's epoch loop ("if validation
 * metric improved"): y = act(gamma*(x - running_mean)/sqrt(running_var + eps) + beta [+ residual]).
 * Reads C floats each of running_mean / running_var (as maintained by cnnk_bn_relu_fwd); writes
 * only y.  residual is nullable.  d->momentum is ignored. */
int cnnk_bn_relu_infer(const cnnk_bn_desc* d, const void* x, const void* residual,
                       const float* gamma, const float* beta, const float* running_mean,
                       const float* running_var, void* y, void* stream);

/* dz = dy*[y>0] (strict; dz = dy without ReLU); dbeta = sum dz; dgamma = sum dz*xhat;
 * dx = (gamma*invstd/m)*(m*dz - dbeta - xhat*dgamma), xhat = (x-mean)*invstd; dresidual = dz.
 * y may be NULL when d->relu == 0; dresidual is nullable.
 * With ReLU and no residual branch (dresidual == NULL) y may also be NULL if beta is given: the
 * mask is then recomputed as [x*sc + bi > 0] with sc = gamma*invstd, bi = beta - mean*sc, the
 * arithmetic (and rounding) of cnnk_bn_relu_fwd on the same x, gamma, beta and saved statistics,
 * which saves reading y.  beta is nullable otherwise.
 * flags bit 0: add into dx instead of overwriting; bit 1: add into dresidual. */
int cnnk_bn_relu_bwd(const cnnk_bn_desc* d, const void* dy, const void* x, const void* y,
                     const float* gamma, const float* beta, const float* save_mean,
                     const float* save_invstd,
                     void* dx, void* dresidual, int flags, float* dgamma, float* dbeta,
                     void* ws, size_t ws_bytes, void* stream);

/* ---- pooling --------------------------------------------------------------------------------- */

/* CNNK_POOL_MAX2: 2x2 window, stride 2, no padding (H, W even); y: N*(H/2)*(W/2)*C; argmax
 * (one byte per output element) = 2*dr+dc of the first maximal element in (row, col) order.
 * CNNK_POOL_GAP: y[n,c] = mean over H*W; argmax unused (may be NULL). */
int cnnk_pool_fwd(const cnnk_pool_desc* d, const void* x, void* y, unsigned char* argmax,
                  void* stream);
/* MAX2: dx = dy at the recorded argmax, 0 elsewhere.  GAP: dx = dy/(H*W) everywhere.
 * accumulate != 0 adds into dx. */
int cnnk_pool_bwd(const cnnk_pool_desc* d, const void* dy, const unsigned char* argmax, void* dx,
                  int accumulate, void* stream);

/* ---- element-wise helpers for residual sums without a following batch norm --------------- */

/* y = a + b over n elements of dtype. */
int cnnk_add(size_t n, int dtype, const void* a, const void* b, void* y, void* stream);
/* dst = src (accumulate == 0) or dst += src, n elements of dtype: gradient fan-out of cnnk_add. */
int cnnk_grad_route(size_t n, int dtype, const void* src, void* dst, int accumulate, void* stream);

/* ---- classifier head and loss (Algorithm 1: "compute loss L(theta)") ---------------------- */

size_t cnnk_fc_workspace_bytes(const cnnk_fc_desc* d);

/* z = x W^T + b; loss = (1/N) sum_n (logsumexp(z_n) - z[n,label_n]) (natural log);
 * pred[n] = smallest j attaining max_j z[n,j] (the scan starts at class 0 and moves on a strictly
 * greater logit only, so a row whose logits are all -inf or NaN, or whose first logit is NaN,
 * predicts class 0); dz = (softmax(z) - onehot)/N; dW = dz^T x; db = sum_n dz; dx = dz W.
 * x, dx: N*F of dtype; W, dW: classes*F float; b, db: classes float; labels, pred: N int32.
 * labels live on the device, so the host cannot validate them: a label outside [0, classes)
 * makes that sample's loss, and therefore *loss, NaN (its row of dz has no target term);
 * loss: 1 float; probs (nullable): N*classes float softmax output.
 * dx, dW, db: all three, or all NULL for the forward half only (loss, pred, probs). */
int cnnk_fc_softmax_xent(const cnnk_fc_desc* d, const void* x, const float* W, const float* b,
                         const int* labels, float* loss, int* pred, float* probs, void* dx,
                         float* dW, float* db, void* ws, size_t ws_bytes, void* stream);

/* The same operation for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc) and so have no workspace to hand
 * over: identical arguments and results (the same kernels), but the scratch (N*classes + N floats)
 * lives in an array inside the library's code object, CNNK_FC_STATIC_SCRATCH_BYTES per device,
 * resident from the moment the library is loaded until the process ends.  The call allocates and
 * frees nothing.  Shapes whose cnnk_fc_workspace_bytes exceeds that size are refused with
 * CNNK_ERR_WORKSPACE and nothing is launched.  The device that `stream` belongs to must be the
 * current device.  All calls on one device share the one array: two calls that may overlap in
 * time on one device (different streams, or different host threads) race and must be ordered by
 * the caller; calls on one stream are ordered by the stream.  Nothing in the array has to be
 * cleared between calls: each call writes every element it later reads. */
#define CNNK_FC_STATIC_SCRATCH_BYTES (1 << 20)
int cnnk_fc_softmax_xent_static(const cnnk_fc_desc* d, const void* x, const float* W, const float* b,
                                const int* labels, float* loss, int* pred, float* probs, void* dx,
                                float* dW, float* db, void* stream);

/* *n_correct += #{i < n : pred[i] == labels[i]} (device int; the caller zeroes it, so that the
 * count can run over several validation batches).  Integer addition: order-independent. */
int cnnk_count_correct(int n, const int* pred, const int* labels, int* n_correct, void* stream);

/* ---- parameter update (Algorithm 1: theta = theta - eta * grad, with momentum) ------------ */

/* g' = g + weight_decay*w; v <- momentum*v + g'; w <- w - lr*v, in place over n floats.
 * w_bf16 (nullable): n bfloat16 values refreshed with the rounded new w. */
int cnnk_sgd_momentum(size_t n, float* w, float* v, const float* g, void* w_bf16, float lr,
                      float momentum, float weight_decay, void* stream);

/* w_bf16[i] = round-to-nearest-even bfloat16 of w[i], n values: the first bf16 copy of fp32 master
 * weights (cnnk_sgd_momentum refreshes the copy after every update). */
int cnnk_round_bf16(size_t n, const float* w, void* w_bf16, void* stream);

/* Mini-batch assembly (Algorithm 1, "for each mini-batch"): dst row i = src row idx[i] for
 * i < n_rows; rows are row_bytes bytes (a multiple of 4; src and dst 4-byte aligned), idx holds
 * n_rows int64 row numbers on the device.  The indices are device data and cannot be validated on
 * the host: a row number outside [0, n_src_rows) is never dereferenced; its destination row is
 * zero-filled and *bad_index (device int, nullable, zeroed by the caller) is set to 1. */
int cnnk_gather_rows(int n_rows, long long n_src_rows, size_t row_bytes, const void* src,
                     const long long* idx, void* dst, int* bad_index, void* stream);

/* ---- the whole step over a layer list ------------------------------------------------------ */

typedef enum { CNNK_OP_CONV = 0, CNNK_OP_BN = 1, CNNK_OP_POOL = 2, CNNK_OP_ADD = 3,
               CNNK_OP_FC_LOSS = 4 } cnnk_op;

/* One layer.  in0/in1/out are tensor-slot ids, p0/p1 parameter-slot ids, -1 = unused.
 *   CONV: x=in0, y=out, w=p0            BN: x=in0, residual=in1, y=out, gamma=p0, beta=p1
 *   POOL: x=in0, y=out                  ADD: a=in0, b=in1, y=out (d.pool describes the shape)
 *   FC_LOSS: x=in0, W=p0, b=p1 (must be the last layer).
 * Slot 0 is the network input and receives no gradient. */
typedef struct cnnk_layer {
  int op, in0, in1, out, p0, p1;
  union { cnnk_conv_desc conv; cnnk_bn_desc bn; cnnk_pool_desc pool; cnnk_fc_desc fc; } d;
} cnnk_layer;

/* Caller-owned device buffers, arrays indexed by slot / parameter / layer id (host arrays of
 * device pointers).  Element types follow the dtype rules at the top of this file. */
typedef struct cnnk_buffers {
  int n_slots, n_params;
  void** act;               /* [n_slots] activations */
  void** dact;              /* [n_slots] activation gradients; dact[0] may be NULL */
  float** param;            /* [n_params] float master parameters (updated in place) */
  void** param_lp;          /* [n_params] bf16 copies of conv weights (bf16 mode), else NULL */
  float** grad;             /* [n_params] parameter gradients (overwritten) */
  float** mom;              /* [n_params] momentum buffers (updated in place) */
  float** bn_save;          /* [n_layers] BN layers: 2*C floats (mean, then invstd) */
  float** bn_running;       /* [n_layers] BN layers: 2*C floats (mean, then var) or NULL */
  unsigned char** pool_idx; /* [n_layers] MAX2 layers: one byte per output element */
  float* probs;             /* N*classes softmax output, nullable */
  void* ws; size_t ws_bytes;
  void** events;            /* nullable: hipEvent_t handles for per-call timing, see below */
  int n_events;             /* number of handles in events */
  /* Optional second stream (all three handles or none; ignored while per-call timing is on).
   * Work that the rest of the step does not wait for runs there, beside the main stream:
   *  - every weight gradient: it depends only on tensors that are final when the backward pass
   *    reaches the layer, and only the parameter update consumes it;
   *  - the update of each convolution's weights, right after their gradient and after the data
   *    gradient that still reads them;
   *  - in the forward pass, a projection shortcut (a convolution and the plain batch norm behind
   *    it whose output is only the residual input of a later batch norm), launched when the main
   *    stream reaches the first other reader of the same input.
   * The step forks with ev_fork (recorded on `stream`, waited for on aux_stream) and joins with
   * ev_join (the other way round), the last time in front of the update of the remaining
   * parameters.  aux_stream must not carry other work during the call and must have the default
   * priority; both events are hipEvent_t handles created by the caller (timing may be disabled).
   * With an aux stream the workspace must be twice cnnk_train_step_workspace_bytes.  Results are
   * bit-reproducible for a given mode; between the modes they differ by fp32 rounding (the forked
   * weight gradients split their reduction over fewer workgroups). */
  void* aux_stream;
  void* ev_fork;
  void* ev_join;
} cnnk_buffers;

size_t cnnk_train_step_workspace_bytes(const cnnk_layer* layers, int n_layers);

/* Per-call timing (the measured analogue of the per-component execution-time profile that the
 * paper's scheduler consumes, Section III-B step 2).  The step is a sequence of "groups", one per
 * call of an entry point above, in this order: forward layer i -> group i (i = 0..n-1); backward
 * layer i (i = n-2..0) -> groups n + 2*(n-2-i) (weight gradient of a CONV, or the whole backward
 * call of any other layer) and n + 2*(n-2-i) + 1 (data gradient of a CONV; empty otherwise); the
 * parameter update -> the last group.  cnnk_train_step_event_groups returns their number,
 * 3*n_layers - 1.  When cnnk_buffers.events holds at least twice that many handles (created by
 * the caller with timing enabled), handle 2g is recorded on the stream before group g and handle
 * 2g+1 after it (both are recorded for an empty group).  Otherwise nothing is recorded. */
int cnnk_train_step_event_groups(int n_layers);

/* Forward over the list, loss, backward over the reversed list, then the update of every
 * parameter, all on one stream without host synchronisation.  labels: N int32 (device);
 * loss: 1 float (device); pred: N int32 (device).  The first gradient written to a slot in
 * the backward pass overwrites it, later ones are added. */
int cnnk_train_step(const cnnk_layer* layers, int n_layers, const cnnk_buffers* buf,
                    const int* labels, float lr, float momentum, float weight_decay,
                    float* loss, int* pred, void* stream);

/* Validation pass of Algorithm 1's epoch loop on one batch: the forward half of cnnk_train_step
 * over the same layer list in inference mode (every batch norm normalises with
 * buf->bn_running, which must be given), then loss, pred and, if n_correct is not NULL,
 * *n_correct += #{pred == label}.  Reads param / param_lp and bn_running; overwrites act[1..],
 * pool_idx, probs (if given) and the workspace; leaves parameters, gradients, momentum, saved and
 * running statistics untouched.  Runs on `stream` alone (aux_stream and events are ignored); the
 * workspace of cnnk_train_step_workspace_bytes suffices. */
int cnnk_eval_step(const cnnk_layer* layers, int n_layers, const cnnk_buffers* buf,
                   const int* labels, float* loss, int* pred, int* n_correct, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CNNK_H */
