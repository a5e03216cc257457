// Dense bf16 matrix products of linear layers (gemm_bf16.hip).  rows = tokens, K = input features,
// N = output features; x [rows][K], w [N][K], y / dy [rows][N], dw [N][K] float.
#pragma once
#include "common.h"

// K and N multiples of 8, every matrix below 2 GiB
bool gemm_bf16_supported(long long rows, int K, int N);
// y = x w^T + bias (bias may be null); with res (not with gelu): y = res + (x w^T + bias as stored);
// with gelu: u = x w^T + bias, y = gelu(u as stored)
int gemm_bf16_fwd(long long rows, int K, int N, const bf16_t* x, const bf16_t* w, const float* bias, const bf16_t* res, bool gelu,
                  bf16_t* u, bf16_t* y, hipStream_t st);
// dx = dy w
int gemm_bf16_dgrad(long long rows, int K, int N, const bf16_t* dy, const bf16_t* w, bf16_t* dx, hipStream_t st);
// dw = dy^T x (fp32); ws: gemm_bf16_wgrad_ws bytes of partial sums
size_t gemm_bf16_wgrad_ws(long long rows, int K, int N);
int gemm_bf16_wgrad(long long rows, int K, int N, const bf16_t* x, const bf16_t* dy, float* dw, void* ws, hipStream_t st);
