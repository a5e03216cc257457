/* cnnk_ref: fp64 CPU oracle of one CNN training step (test infrastructure, not product code).
 *
 * Plain, slow, direct-loop definitions of the operators that make up the inner mini-batch
 * loop of the paper's Algorithm 1 (forward pass, loss, backward pass, parameter update) for
 * an image-classification CNN.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may call this library; the HIP library shares no code with it.
 *
 * All tensors are host double arrays.  Activations are NHWC, convolution weights are
 * [Cout][R][S][Cin], the FC weight is [classes][F].  Functions return 0 on success and a
 * non-zero value on an argument error (null pointer, non-positive size, empty output).
 */
#ifndef CNNK_REF_H
#define CNNK_REF_H
#ifdef __cplusplus
extern "C" {
#endif

int cnnk_ref_conv2d_fwd(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                        const double* x, const double* w, double* y);
int cnnk_ref_conv2d_dgrad(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                          const double* dy, const double* w, double* dx);
int cnnk_ref_conv2d_wgrad(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad,
                          const double* x, const double* dy, double* dw);
int cnnk_ref_bn_relu_fwd(int N, int H, int W, int C, double eps, double momentum, int relu,
                         const double* x, const double* residual, const double* gamma,
                         const double* beta, double* y, double* save_mean, double* save_invstd,
                         double* running_mean, double* running_var);
/* Inference mode: running statistics in place of the batch's; updates nothing. */
int cnnk_ref_bn_relu_infer(int N, int H, int W, int C, double eps, int relu, const double* x,
                           const double* residual, const double* gamma, const double* beta,
                           const double* running_mean, const double* running_var, double* y);
int cnnk_ref_bn_relu_bwd(int N, int H, int W, int C, int relu, const double* dy, const double* x,
                         const double* y, const double* gamma, const double* save_mean,
                         const double* save_invstd, double* dx, double* dresidual, double* dgamma,
                         double* dbeta);
/* mode 0: 2x2 stride-2 max-pool (argmax code 2*dr+dc, first maximum in scan order);
 * mode 1: global average pool (argmax unused). */
int cnnk_ref_pool_fwd(int N, int H, int W, int C, int mode, const double* x, double* y,
                      unsigned char* argmax);
int cnnk_ref_pool_bwd(int N, int H, int W, int C, int mode, const double* dy,
                      const unsigned char* argmax, double* dx);
int cnnk_ref_fc_softmax_xent(int N, int F, int classes, const double* x, const double* W,
                             const double* b, const int* labels, double* loss, int* pred,
                             double* probs, double* dx, double* dW, double* db);
int cnnk_ref_sgd_momentum(long n, double* w, double* v, const double* g, double lr, double momentum,
                          double weight_decay);
int cnnk_ref_round_bf16(long n, double* a);
int cnnk_ref_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
