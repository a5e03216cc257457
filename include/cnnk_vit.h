/* cnnk_vit.h - C ABI of the Vision Transformer training step (gfx950 / MI355X), the second model
 * family of the paper (Section IV-A: ViT-B/16; the step is the inner loop of Algorithm 1: forward
 * pass, loss, backward pass, parameter update).  Same conventions as cnnk.h: plain device pointers
 * and sizes, status codes of cnnk_status, nothing is allocated or synchronised, every call is
 * enqueued on `stream` (a hipStream_t, NULL = the default stream), `dtype` is CNNK_F32 or
 * CNNK_BF16 and names the storage type of activations and activation gradients; parameters,
 * parameter gradients, statistics and the loss are always float.  All matrices are row-major with
 * the feature index contiguous.  Host-side checks come before any launch.
 *
 * The paper names the model only.  The operators below are those of the standard pre-norm ViT:
 *   tokens   X[b, 0] = cls + pos[0];  X[b, 1 + i] = patch_i(b) @ We^T + be + pos[1 + i]
 *   block    X += Attn(LN(X)) @ Wo^T + bo;   X += gelu(LN(X) @ W1^T + c1) @ W2^T + c2
 *   head     logits = LN(X[:, 0]) @ Wh^T + bh, mean softmax cross-entropy
 */
#ifndef CNNK_VIT_ABI_H_
#define CNNK_VIT_ABI_H_
#include "cnnk.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- layer normalisation over the feature axis ----------------------------------------------------
 * y[r, c] = (x[r, c] - mean_r) * rstd_r * gamma[c] + beta[c],  mean_r and the biased variance over
 * the C features of row r, rstd_r = 1 / sqrt(var_r + eps).  C % 4 == 0, C <= 4096.
 * x_stride: elements between consecutive rows of x (and of dx / dres in the backward call); 0 means
 * C.  y and dy are dense.  stats [rows][2] = (mean, rstd), written by fwd and read by bwd. */
typedef struct { int rows, C; int dtype; float eps; long long x_stride; } cnnk_ln_desc;

int cnnk_layernorm_fwd(const cnnk_ln_desc* d, const void* x, const float* gamma, const float* beta,
                       void* y, float* stats, void* stream);

/* dx = d loss / d x given dy (+ dres[r, c] when dres is not NULL: the gradient that reaches x along
 * a residual connection, same layout as dx; dx may alias dres);  dgamma[c] = sum_r dy * xhat,
 * dbeta[c] = sum_r dy.  The sums over rows are per-workgroup partial sums in `ws`, added in a fixed
 * order by a second launch: results are reproducible bit for bit. */
size_t cnnk_layernorm_workspace_bytes(const cnnk_ln_desc* d);
int cnnk_layernorm_bwd(const cnnk_ln_desc* d, const void* dy, const void* x, const float* gamma,
                       const float* stats, const void* dres, void* dx, float* dgamma, float* dbeta,
                       void* ws, size_t ws_bytes, void* stream);

/* ---- bias, activation, residual ---------------------------------------------------------------------
 * act = CNNK_ACT_NONE:  y = z + bias (+ res when not NULL);  u is not used.
 * act = CNNK_ACT_GELU:  u = z + bias (stored: the backward pass needs it), y = gelu(u) with the exact
 *                       gelu(u) = u * Phi(u), Phi the standard normal distribution function; res
 *                       must be NULL.
 * z, res, u, y: [rows][C] of dtype; u may alias z, y may alias z or res.  C % 8 == 0. */
enum { CNNK_ACT_NONE = 0, CNNK_ACT_GELU = 1 };
int cnnk_bias_act_fwd(long long rows, int C, int dtype, int act, const void* z, const float* bias,
                      const void* res, void* u, void* y, void* stream);

/* act = NONE: dbias[c] = sum_r dy[r, c]; dz and u are not used (the gradient of z is dy itself).
 * act = GELU: dz = dy * gelu'(u), dbias[c] = sum_r dz[r, c] (the sum of the unrounded products).
 * Column sums as in cnnk_layernorm_bwd: partials in ws, fixed order. */
size_t cnnk_bias_act_workspace_bytes(long long rows, int C);
int cnnk_bias_act_bwd(long long rows, int C, int dtype, int act, const void* dy, const void* u,
                      void* dz, float* dbias, void* ws, size_t ws_bytes, void* stream);

/* ---- linear layers ---------------------------------------------------------------------------------------
 * x [rows][K], w [N][K] (of dtype: in the bf16 mode the bf16 copy of the fp32 master), bias [N]
 * float or NULL.  fwd: act = NONE: y = x w^T + bias, and with res [rows][N] not NULL (a residual
 * connection; y must not alias res) y = res + (x w^T + bias as stored: in bf16 storage the product is
 * rounded before the sum and the sum again, whichever kernels run);  act = GELU (bias required, no
 * res): u = x w^T + bias is stored and y = gelu(u as stored), as in cnnk_bias_act_fwd.
 * dgrad: dx [rows][K] = dy w.
 * wgrad: dw [N][K] float = dy^T x (the bias gradient is cnnk_bias_act_bwd's column sum).
 * K % 8 == 0, N % 8 == 0.  bf16 runs on dedicated matrix-core kernels (an output is rounded once,
 * after bias); fp32 on the 1 x 1 convolution kernels of cnnk.h followed by cnnk_bias_act_fwd
 * (cnnk_tune key 15 = -1 forces that path for bf16 too).  The weight
 * gradient is a fixed-order sum of per-row-range partials: reproducible bit for bit. */
size_t cnnk_linear_workspace_bytes(long long rows, int K, int N, int dtype);
int cnnk_linear_fwd(long long rows, int K, int N, int dtype, const void* x, const void* w,
                    const float* bias, const void* res, int act, void* u, void* y, void* ws,
                    size_t ws_bytes, void* stream);
int cnnk_linear_dgrad(long long rows, int K, int N, int dtype, const void* dy, const void* w, void* dx,
                      void* ws, size_t ws_bytes, void* stream);
int cnnk_linear_wgrad(long long rows, int K, int N, int dtype, const void* x, const void* dy, float* dw,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- multi-head self-attention ------------------------------------------------------------------------
 * qkv [B][T][3 * heads * dh]: per token the queries of all heads, then the keys, then the values.
 * o[b, t, h*dh + j] = sum_u A[b, h, t, u] v[b, u, h, j],  A = softmax over u of q.k / sqrt(dh).
 * lse [B][heads][T] = log sum_u exp(q.k / sqrt(dh)): written by fwd, read by bwd (the probabilities
 * are recomputed, not stored).  dh in {16, 32, 64}, T * dh <= 16384. */
typedef struct { int B, T, heads, dh; int dtype; } cnnk_attn_desc;
int cnnk_attention_fwd(const cnnk_attn_desc* d, const void* qkv, void* o, float* lse, void* stream);
int cnnk_attention_bwd(const cnnk_attn_desc* d, const void* qkv, const void* o, const void* d_o,
                       const float* lse, void* dqkv, void* stream);

/* ---- patch embedding ------------------------------------------------------------------------------------
 * x [B][image][image][3] (NHWC); n = (image / patch)^2 patches per image, row-major over the patch
 * grid; a patch is flattened in (row, column, channel) order: patches [B * n][patch * patch * 3].
 * embed_fwd: tok [B][n + 1][dim] from z [B * n][dim] = patches @ We^T as documented above.
 * embed_bwd: dz [B * n][dim] = the rows of dtok that belong to patches; dbe, dcls [dim],
 *            dpos [n + 1][dim] (sums over the batch, fixed order). */
typedef struct { int B, image, patch, dim; int dtype; } cnnk_embed_desc;
int cnnk_vit_patchify(const cnnk_embed_desc* d, const void* x, void* patches, void* stream);
int cnnk_vit_embed_fwd(const cnnk_embed_desc* d, const void* z, const float* be, const float* cls,
                       const float* pos, void* tok, void* stream);
int cnnk_vit_embed_bwd(const cnnk_embed_desc* d, const void* dtok, void* dz, float* dbe, float* dcls,
                       float* dpos, void* stream);

/* ---- the whole training step -----------------------------------------------------------------------------
 * Parameter order (n_params = 4 + 12 * layers + 4): We [dim][patch*patch*3], be [dim], cls [dim],
 * pos [tokens][dim]; per block g1, b1, Wqkv [3 dim][dim], bqkv, Wo [dim][dim], bo, g2, b2,
 * W1 [mlp][dim], c1, W2 [dim][mlp], c2; then gf, bf, Wh [classes][dim], bh.
 * param / grad / mom: float tensors.  param_lp[k]: bf16 copy of parameter k, required in the bf16
 * mode for the matrices We, Wqkv, Wo, W1, W2 (refreshed by the update), NULL elsewhere.
 * arena: activations, statistics and activation gradients of the step, laid out by the library
 * (cnnk_vit_arena_bytes; cnnk_vit_tensor finds a tensor in it).  Nothing in it has to survive
 * between steps.  ws: scratch of the single calls (cnnk_vit_workspace_bytes).
 * events (optional): 2 * cnnk_vit_step_calls(d) hipEvent_t; the step records one pair around each
 * call it makes, in the order that cnnk_vit_step_call_name lists.
 * aux_stream (optional, with the two events ev_fork and ev_join; default priority): a second stream
 * for work that only the update waits for - the weight gradients of the linear layers and the bias
 * gradients that are plain column sums.  They depend only on tensors that are final when the backward
 * pass reaches them, so the step forks each onto aux_stream and joins before the update; beside the
 * main stream they fill the compute units that its launches leave idle.  ws must then hold twice
 * cnnk_vit_workspace_bytes (the forked calls use the upper half).  Ignored while `events` is set (a
 * call's time is then its own).  Results are bit-identical with and without it. */
typedef struct { int B, image, patch, dim, heads, layers, mlp, classes; int dtype; float ln_eps; } cnnk_vit_desc;
typedef struct cnnk_vit_buffers {
  int n_params;
  void** param;
  void** param_lp;
  void** grad;
  void** mom;
  const void* x;          /* [B][image][image][3] */
  const int* labels;      /* [B] */
  float* loss;            /* [1] */
  int* pred;              /* [B] */
  float* probs;           /* [B][classes] or NULL */
  void* arena;
  size_t arena_bytes;
  void* ws;
  size_t ws_bytes;
  void** events;
  int n_events;
  void* aux_stream;       /* hipStream_t or NULL */
  void* ev_fork;          /* hipEvent_t */
  void* ev_join;          /* hipEvent_t */
} cnnk_vit_buffers;

/* tensors of the arena; `layer` is the block index (ignored for the first and last group).
 * Activations: TOK (input of block 0), per block H, QKV, O, XMID, H2, U, G, XOUT (= input of the
 * next block), then F (normalised class-token features).  D* are the gradients of the same. */
typedef enum { CNNK_VIT_PATCHES = 0, CNNK_VIT_TOK, CNNK_VIT_H, CNNK_VIT_QKV, CNNK_VIT_O, CNNK_VIT_XMID,
               CNNK_VIT_H2, CNNK_VIT_U, CNNK_VIT_G, CNNK_VIT_XOUT, CNNK_VIT_F,
               CNNK_VIT_DTOK, CNNK_VIT_DH, CNNK_VIT_DQKV, CNNK_VIT_DO, CNNK_VIT_DXMID, CNNK_VIT_DH2,
               CNNK_VIT_DU, CNNK_VIT_DG, CNNK_VIT_DXOUT, CNNK_VIT_DF, CNNK_VIT_TENSORS } cnnk_vit_tensor_id;

size_t cnnk_vit_arena_bytes(const cnnk_vit_desc* d);
size_t cnnk_vit_workspace_bytes(const cnnk_vit_desc* d);
/* byte offset and size of a tensor inside the arena; returns a status. */
int cnnk_vit_tensor(const cnnk_vit_desc* d, int tensor_id, int layer, size_t* offset, size_t* bytes);
int cnnk_vit_step_calls(const cnnk_vit_desc* d);
/* name of call i ("block3.fc1.wgrad", ...) copied into buf (at most n bytes incl. the terminator). */
int cnnk_vit_step_call_name(const cnnk_vit_desc* d, int i, char* buf, int n);

/* One step: forward, loss, backward, then v <- momentum * v + (grad + weight_decay * w),
 * w <- w - lr * v on every parameter (and the bf16 copies). */
int cnnk_vit_train_step(const cnnk_vit_desc* d, const cnnk_vit_buffers* buf, float lr, float momentum,
                        float weight_decay, void* stream);

/* The validation pass of the epoch loop (Algorithm 1: "evaluate model on validation data"): the
 * forward pass and the loss of the same model on buf->x / buf->labels; writes *loss, pred, probs (if
 * not NULL) and, if n_correct is not NULL, adds the number of correct predictions to *n_correct
 * (device int, as cnnk_count_correct).  The model has no batch statistics, so this is the training
 * step's own forward pass; parameters, gradients and momentum buffers are not touched (grad and mom
 * may be NULL).  One stream; events and aux_stream are ignored. */
int cnnk_vit_eval_step(const cnnk_vit_desc* d, const cnnk_vit_buffers* buf, int* n_correct, void* stream);

#ifdef __cplusplus
}
#endif
#endif
