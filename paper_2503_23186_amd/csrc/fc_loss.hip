// Classifier head: logits, softmax cross-entropy (mean over the batch, natural log), class
// prediction, and the gradients of the head.  The work is tiny (N x F x classes); the kernels
// are written for determinism: every sum has a fixed order, no atomics.
#include <mutex>
#include "common.h"

namespace {
constexpr int kT = 256;
constexpr int kMaxClasses = 4096;
constexpr int kLT = 1024;   // threads of the logits kernel

// One workgroup per sample: z = W x + b by wave-level dot products, then the softmax.  The kernel
// is latency-bound (a sample's 100 dot products), so the workgroup is wide: 16 wavefronts take 4
// classes each per round.
template <typename T>
__global__ void __launch_bounds__(kLT) logits_softmax_kernel(const T* __restrict__ x, const float* __restrict__ W,
                                                            const float* __restrict__ b,
                                                            const int* __restrict__ labels, int N, int F, int K,
                                                            int vec, float* __restrict__ dz, float* __restrict__ loss_n,
                                                            int* __restrict__ pred, float* __restrict__ probs) {
  __shared__ float z[kMaxClasses];
  __shared__ float red[kLT / 64];
  __shared__ int redi[kLT / 64];
  const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* xr = x + (size_t)n * F;
  if (vec) {
    // F % 8 == 0 and F <= 2048: the sample's features stay in registers (8 consecutive per lane
    // and 512-feature chunk), weight rows stream in as 32-byte pieces, four classes in flight
    float xv[4][8];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int f0 = (lane + 64 * c) * 8;
      if (c * 512 < F) load8(xr + (f0 < F ? f0 : 0), xv[c]);   // uniform condition: the chunks load together
      if (f0 >= F)
#pragma unroll
        for (int e = 0; e < 8; ++e) xv[c][e] = 0.f;
    }
    for (int j0 = wave; j0 < K; j0 += 4 * (kLT / 64)) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      // Unconditional loads, so that the four classes' weight pieces are in flight together (under
      // per-lane conditions the compiler waits for every load before it issues the next): a class
      // past the end re-reads the last one (its logit is not stored), a lane past the end of the
      // features reads the row's start against features that are zero.
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (c * 512 >= F) break;           // uniform
        const int f0 = (lane + 64 * c) * 8;
        const int fl = f0 < F ? f0 : 0;
        float wv[4][8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int j = min(j0 + q * (kLT / 64), K - 1);
          load8(W + (size_t)j * F + fl, wv[q]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[q] = fmaf(xv[c][e], wv[q][e], acc[q]);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int j = j0 + q * (kLT / 64);
        const float sq = wave_sum(acc[q]);
        if (lane == 0 && j < K) z[j] = sq + b[j];
      }
    }
  } else {
    // four classes per pass of a wave: independent dot products keep several loads in flight
    for (int j0 = wave * 4; j0 < K; j0 += (kLT / 64) * 4) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
      for (int f = lane; f < F; f += 64) {
        const float xv = Elem<T>::ld(xr + f);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (j0 + q < K) acc[q] = fmaf(xv, W[(size_t)(j0 + q) * F + f], acc[q]);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float sq = wave_sum(acc[q]);
        if (lane == 0 && j0 + q < K) z[j0 + q] = sq + b[j0 + q];
      }
    }
  }
  __syncthreads();
  // max and its lowest index
  float mx = -INFINITY;
  int arg = 0x7fffffff;
  for (int j = tid; j < K; j += kLT)
    if (z[j] > mx) { mx = z[j]; arg = j; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(mx, o, 64);
    const int oa = __shfl_xor(arg, o, 64);
    if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
  }
  if (lane == 0) { red[wave] = mx; redi[wave] = arg; }
  __syncthreads();
  mx = red[0]; arg = redi[0];
  for (int w = 1; w < kLT / 64; ++w)
    if (red[w] > mx || (red[w] == mx && redi[w] < arg)) { mx = red[w]; arg = redi[w]; }
  // A scan that starts from class 0 and moves only on a strictly greater logit stays at class 0
  // when no logit exceeds -inf (a row of -inf or NaN) and when the first logit is NaN (nothing
  // compares greater than NaN): the predicted class of such a row is 0.
  if (arg == 0x7fffffff || z[0] != z[0]) arg = 0;
  __syncthreads();
  float se = 0.f;
  for (int j = tid; j < K; j += kLT) se += expf(z[j] - mx);
  se = wave_sum(se);
  if (lane == 0) red[wave] = se;
  __syncthreads();
  se = 0.f;
  for (int w = 0; w < kLT / 64; ++w) se += red[w];
  const float lse = mx + logf(se);
  const int lab = labels[n];
  if (tid == 0) {
    pred[n] = arg;
    // a label outside [0, K) has no target logit: the sample's loss, and with it the mean, is NaN
    loss_n[n] = (lab >= 0 && lab < K) ? lse - z[lab] : __builtin_nanf("");
  }
  const float invN = 1.f / (float)N;
  for (int j = tid; j < K; j += kLT) {
    const float p = expf(z[j] - lse);
    if (probs) probs[(size_t)n * K + j] = p;
    dz[(size_t)n * K + j] = (p - (j == lab ? 1.f : 0.f)) * invN;
  }
}

// loss = mean(loss_n)      (single workgroup, fixed order)
__device__ __forceinline__ void loss_body(const float* __restrict__ loss_n, int N, float* __restrict__ loss) {
  __shared__ float red[kT];
  const int tid = threadIdx.x;
  float s = 0.f;
  for (int n = tid; n < N; n += kT) s += loss_n[n];
  red[tid] = s;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) loss[0] = red[0] / (float)N;
}

__global__ void __launch_bounds__(kT) loss_kernel(const float* __restrict__ loss_n, int N, float* __restrict__ loss) {
  loss_body(loss_n, N, loss);
}

// One workgroup per class j: dW[j][f] = sum_n dz[n][j] * x[n][f] (threads over f), and
// db[j] = sum_n dz[n][j] (threads over n, fixed-order tree).
template <typename T>
__device__ __forceinline__ void fc_dw_db_body(int j, const float* __restrict__ dz, const T* __restrict__ x, int N,
                                              int F, int K, float* __restrict__ dW, float* __restrict__ db) {
  __shared__ float red[kT];
  const int tid = threadIdx.x;
  for (int f = tid; f < F; f += kT) {
    float a = 0.f;
#pragma unroll 8
    for (int n = 0; n < N; ++n) a = fmaf(dz[(size_t)n * K + j], Elem<T>::ld(x + (size_t)n * F + f), a);
    dW[(size_t)j * F + f] = a;
  }
  float s = 0.f;
  for (int n = tid; n < N; n += kT) s += dz[(size_t)n * K + j];
  red[tid] = s;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) db[j] = red[0];
}

// The same for F % 8 == 0: wave w takes the samples n = w, w+4, ..., a lane 8 consecutive features
// (16- or 32-byte loads); the four per-wave sums are combined through LDS in wave order.
template <typename T>
__device__ __forceinline__ void fc_dw_db_vec_body(int j, const float* __restrict__ dz, const T* __restrict__ x,
                                                  int N, int F, int K, float* __restrict__ dW,
                                                  float* __restrict__ db) {
  __shared__ float part[kT / 64][512];
  __shared__ float red[kT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int fb = 0; fb < F; fb += 512) {
    const int f0 = fb + lane * 8;
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (f0 < F) {
#pragma unroll 4
      for (int n = wave; n < N; n += kT / 64) {
        float xv[8];
        load8(x + (size_t)n * F + f0, xv);
        const float g = dz[(size_t)n * K + j];
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = fmaf(g, xv[e], a[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[wave][lane * 8 + e] = a[e];
    __syncthreads();
    for (int f = tid; f < 512 && fb + f < F; f += kT) {
      float sum = part[0][f];
#pragma unroll
      for (int w = 1; w < kT / 64; ++w) sum += part[w][f];
      dW[(size_t)j * F + fb + f] = sum;
    }
    __syncthreads();
  }
  float sacc = 0.f;
  for (int n = tid; n < N; n += kT) sacc += dz[(size_t)n * K + j];
  red[tid] = sacc;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) db[j] = red[0];
}

// dx[n][f] = sum_j dz[n][j] * W[j][f]
template <typename T>
__device__ __forceinline__ void fc_dx_body(int fblk, int n, const float* __restrict__ dz,
                                           const float* __restrict__ W, int N, int F, int K, T* __restrict__ dx) {
  const int f = fblk * kT + threadIdx.x;
  if (f >= F) return;
  float a = 0.f;
#pragma unroll 4
  for (int j = 0; j < K; ++j) a = fmaf(dz[(size_t)n * K + j], W[(size_t)j * F + f], a);
  Elem<T>::st(dx + (size_t)n * F + f, a);
}

// Everything behind the softmax in one launch, by workgroup role: workgroups [0, K) one class each
// of dW and db, workgroup K the mean of the per-sample losses, the rest one (feature block, sample)
// each of dx.  The roles are independent (all read dz and loss_n of the previous launch), each sum
// keeps its fixed order.
template <typename T, int VEC>
__global__ void __launch_bounds__(kT) fc_bwd_kernel(const float* __restrict__ dz, const float* __restrict__ loss_n,
                                                    const T* __restrict__ x, const float* __restrict__ W, int N,
                                                    int F, int K, int fblocks, float* __restrict__ loss,
                                                    float* __restrict__ dW, float* __restrict__ db,
                                                    T* __restrict__ dx) {
  const int b = blockIdx.x;
  if (b < K) {
    if (VEC) fc_dw_db_vec_body<T>(b, dz, x, N, F, K, dW, db);
    else fc_dw_db_body<T>(b, dz, x, N, F, K, dW, db);
  } else if (b == K) {
    loss_body(loss_n, N, loss);
  } else {
    const int r = b - K - 1;
    fc_dx_body<T>(r % fblocks, r / fblocks, dz, W, N, F, K, dx);
  }
}

// *n_correct += number of samples with pred == label (integer atomic: order-independent).
__global__ void __launch_bounds__(kT) count_correct_kernel(const int* __restrict__ pred,
                                                           const int* __restrict__ labels, int N,
                                                           int* __restrict__ n_correct) {
  __shared__ int red[kT];
  const int tid = threadIdx.x;
  int c = 0;
  for (int n = tid; n < N; n += kT) c += pred[n] == labels[n] ? 1 : 0;
  red[tid] = c;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) atomicAdd(n_correct, red[0]);
}

int validate_fc(const cnnk_fc_desc* d) {
  if (!d) return CNNK_ERR_NULL;
  if (d->N <= 0 || d->F <= 0 || d->classes <= 0) return CNNK_ERR_SHAPE;
  if (d->dtype != CNNK_F32 && d->dtype != CNNK_BF16) return CNNK_ERR_UNSUPPORTED;
  if (d->classes > kMaxClasses || d->N > 65535) return CNNK_ERR_UNSUPPORTED;
  return CNNK_OK;
}
}  // namespace

extern "C" size_t cnnk_fc_workspace_bytes(const cnnk_fc_desc* d) {
  if (validate_fc(d) != CNNK_OK) return 0;
  return align_up(((size_t)d->N * d->classes + d->N) * sizeof(float), 256);
}

namespace {
// Both entry points of the classifier head: `scratch` holds dz (N * classes floats) and the
// per-sample losses (N floats); every element is written by the first launch before the second
// reads it, so its previous contents do not matter.
int fc_enqueue(const cnnk_fc_desc* d, const void* x, const float* W, const float* b, const int* labels, float* loss,
               int* pred, float* probs, void* dx, float* dW, float* db, float* scratch, hipStream_t st) {
  const bool backward = dx || dW || db;   // all three or none
  const int N = d->N, F = d->F, K = d->classes;
  float* dz = scratch;
  float* loss_n = dz + (size_t)N * K;
  const int fblocks = (F + kT - 1) / kT;
  const unsigned nblk = (unsigned)(K + 1 + fblocks * N);
  // the vector paths read x and W in 16-byte pieces: rows stay aligned when F % 8 == 0 and the
  // tensors themselves start on a 16-byte boundary
  const bool aligned = (((uintptr_t)x | (uintptr_t)W) & 15u) == 0;
  const bool vec8 = F % 8 == 0 && aligned;
  const int vec = (vec8 && F <= 2048) ? 1 : 0;
  if (d->dtype == CNNK_BF16) {
    logits_softmax_kernel<bf16_t><<<N, kLT, 0, st>>>((const bf16_t*)x, W, b, labels, N, F, K, vec, dz, loss_n, pred, probs);
    if (!backward) loss_kernel<<<1, kT, 0, st>>>(loss_n, N, loss);
    else if (vec8)
      fc_bwd_kernel<bf16_t, 1><<<nblk, kT, 0, st>>>(dz, loss_n, (const bf16_t*)x, W, N, F, K, fblocks, loss, dW, db, (bf16_t*)dx);
    else
      fc_bwd_kernel<bf16_t, 0><<<nblk, kT, 0, st>>>(dz, loss_n, (const bf16_t*)x, W, N, F, K, fblocks, loss, dW, db, (bf16_t*)dx);
  } else {
    logits_softmax_kernel<float><<<N, kLT, 0, st>>>((const float*)x, W, b, labels, N, F, K, vec, dz, loss_n, pred, probs);
    if (!backward) loss_kernel<<<1, kT, 0, st>>>(loss_n, N, loss);
    else if (vec8)
      fc_bwd_kernel<float, 1><<<nblk, kT, 0, st>>>(dz, loss_n, (const float*)x, W, N, F, K, fblocks, loss, dW, db, (float*)dx);
    else
      fc_bwd_kernel<float, 0><<<nblk, kT, 0, st>>>(dz, loss_n, (const float*)x, W, N, F, K, fblocks, loss, dW, db, (float*)dx);
  }
  return launch_status();
}

int fc_check_args(const cnnk_fc_desc* d, const void* x, const float* W, const float* b, const int* labels,
                  const float* loss, const int* pred, const void* dx, const float* dW, const float* db) {
  int rc = validate_fc(d);
  if (rc != CNNK_OK) return rc;
  if (!x || !W || !b || !labels || !loss || !pred) return CNNK_ERR_NULL;
  if ((dx || dW || db) && (!dx || !dW || !db)) return CNNK_ERR_NULL;
  return CNNK_OK;
}

// Scratch of the entry point that allocates nothing: one array per device, part of the code object
// (it exists from the moment the library is loaded until the process ends).  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels and copies get the address that
// call returns for the device that is current, looked up once per device.
static __device__ __align__(256) unsigned char g_fc_scratch[CNNK_FC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_fc_scratch_mu;
void* g_fc_scratch_ptr[kMaxDevices];   // zero-initialised: not looked up yet

int fc_static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CNNK_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_fc_scratch_mu);
  if (!g_fc_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_fc_scratch)) != hipSuccess || !p) return CNNK_ERR_HIP;
    g_fc_scratch_ptr[dev] = p;
  }
  *out = static_cast<float*>(g_fc_scratch_ptr[dev]);
  return CNNK_OK;
}
}  // namespace

extern "C" int cnnk_fc_softmax_xent(const cnnk_fc_desc* d, const void* x, const float* W, const float* b,
                                    const int* labels, float* loss, int* pred, float* probs, void* dx, float* dW,
                                    float* db, void* ws, size_t ws_bytes, void* stream) {
  int rc = fc_check_args(d, x, W, b, labels, loss, pred, dx, dW, db);
  if (rc != CNNK_OK) return rc;
  if (!ws || ws_bytes < cnnk_fc_workspace_bytes(d)) return CNNK_ERR_WORKSPACE;
  return fc_enqueue(d, x, W, b, labels, loss, pred, probs, dx, dW, db, (float*)ws, (hipStream_t)stream);
}

extern "C" int cnnk_fc_softmax_xent_static(const cnnk_fc_desc* d, const void* x, const float* W, const float* b,
                                           const int* labels, float* loss, int* pred, float* probs, void* dx,
                                           float* dW, float* db, void* stream) {
  int rc = fc_check_args(d, x, W, b, labels, loss, pred, dx, dW, db);
  if (rc != CNNK_OK) return rc;
  if (cnnk_fc_workspace_bytes(d) > (size_t)CNNK_FC_STATIC_SCRATCH_BYTES) return CNNK_ERR_WORKSPACE;
  float* scratch = nullptr;
  rc = fc_static_scratch(&scratch);
  if (rc != CNNK_OK) return rc;
  return fc_enqueue(d, x, W, b, labels, loss, pred, probs, dx, dW, db, scratch, (hipStream_t)stream);
}

extern "C" int cnnk_count_correct(int n, const int* pred, const int* labels, int* n_correct, void* stream) {
  if (!pred || !labels || !n_correct) return CNNK_ERR_NULL;
  if (n <= 0) return CNNK_ERR_SHAPE;
  count_correct_kernel<<<1, kT, 0, (hipStream_t)stream>>>(pred, labels, n, n_correct);
  return launch_status();
}
