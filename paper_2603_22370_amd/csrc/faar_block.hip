// Glue between the quantised linears of a transformer block, for a Stage-2-style joint step (paper Sec. 3.5 "Stage 2";
// Table 2 steps 15-17 and 23: the assembled quantised model runs forward and one loss is back-propagated into every
// layer's rounding variables).  The operations are those of the Llama3 / Qwen3 blocks the paper evaluates: pre-norm
// RMSNorm, the gated SiLU MLP, the residual connection, and the squared error of the block output.  HBM-bound
// kernels; activations and their gradients are stored in bf16 between kernels (the rounding points a bf16 model
// declares), all arithmetic is float32.
#include "faar_internal.h"

namespace faar {
namespace {

constexpr int kRowThreads = 256;

__device__ __forceinline__ float row_sum(float a) {   // sum over the 256 threads of a workgroup, result in every thread
  __shared__ float s[kRowThreads / 64];
  __shared__ float total;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
  __syncthreads();                                     // a previous use of `total` is finished
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) total = (s[0] + s[1]) + (s[2] + s[3]);
  __syncthreads();
  return total;
}

// h = x g / sqrt(mean(x^2) + eps), one workgroup per token row; the row is read twice (the second time from cache)
template <typename XT>
__global__ void __launch_bounds__(kRowThreads)
k_rmsnorm_fwd(const XT* __restrict__ X, int64_t D8, const float* __restrict__ g, float eps, bf16_t* __restrict__ H,
              float* __restrict__ rstd) {
  const int64_t row = blockIdx.x;
  const XT* x = X + row * D8 * 8;
  float ss = 0.0f;
  for (int64_t c = threadIdx.x; c < D8; c += kRowThreads) {
    float v[8];
    W8<XT>::load(x + c * 8, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
  }
  ss = row_sum(ss);
  const float r = 1.0f / sqrtf(ss / static_cast<float>(D8 * 8) + eps);
  if (threadIdx.x == 0) rstd[row] = r;
  for (int64_t c = threadIdx.x; c < D8; c += kRowThreads) {
    float v[8], gg[8], o[8];
    W8<XT>::load(x + c * 8, v);
    load8(g + c * 8, gg);
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (v[j] * r) * gg[j];
    W8<bf16_t>::store(H + (row * D8 + c) * 8, o);
  }
}

// the gradient entering the norm's output: dh1 (+ dh2) (+ dh3), each stored in bf16, added in float32 in that order
__device__ __forceinline__ void load_dh(const bf16_t* dH1, const bf16_t* dH2, const bf16_t* dH3, int64_t at, float (&d1)[8]) {
  float d2[8];
  W8<bf16_t>::load(dH1 + at, d1);
  if (dH2) {
    W8<bf16_t>::load(dH2 + at, d2);
#pragma unroll
    for (int j = 0; j < 8; ++j) d1[j] += d2[j];
  }
  if (dH3) {
    W8<bf16_t>::load(dH3 + at, d2);
#pragma unroll
    for (int j = 0; j < 8; ++j) d1[j] += d2[j];
  }
}

// dx = r g dh - x r^3 / D * sum(x g dh) + d_res,  dh = dh1 + dh2 + dh3
template <typename XT>
__global__ void __launch_bounds__(kRowThreads)
k_rmsnorm_bwd(const bf16_t* __restrict__ dH1, const bf16_t* __restrict__ dH2, const bf16_t* __restrict__ dH3,
              const XT* __restrict__ X, int64_t D8, const float* __restrict__ g, const float* __restrict__ rstd,
              const bf16_t* __restrict__ d_res, bf16_t* __restrict__ dX) {
  const int64_t row = blockIdx.x, base = row * D8;
  const float r = rstd[row];
  float dot = 0.0f;
  for (int64_t c = threadIdx.x; c < D8; c += kRowThreads) {
    float v[8], gg[8], d1[8];
    W8<XT>::load(X + (base + c) * 8, v);
    load8(g + c * 8, gg);
    load_dh(dH1, dH2, dH3, (base + c) * 8, d1);
#pragma unroll
    for (int j = 0; j < 8; ++j) dot += v[j] * (gg[j] * d1[j]);
  }
  dot = row_sum(dot);
  const float k = (r * r * r) * (dot / static_cast<float>(D8 * 8));
  for (int64_t c = threadIdx.x; c < D8; c += kRowThreads) {
    float v[8], gg[8], d1[8], d2[8], o[8];
    W8<XT>::load(X + (base + c) * 8, v);
    load8(g + c * 8, gg);
    load_dh(dH1, dH2, dH3, (base + c) * 8, d1);
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = r * (gg[j] * d1[j]) - v[j] * k;
    if (d_res) {
      W8<bf16_t>::load(d_res + (base + c) * 8, d2);
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] += d2[j];
    }
    W8<bf16_t>::store(dX + (base + c) * 8, o);
  }
}

// Rows of at most 512 entries (the per-head norm of q and k: dh = 128): LPR lanes per row (the power of two that holds the
// row's 16-byte chunks, one per lane), 64 / LPR rows per wavefront, sums within a row's lanes by shuffles
template <int LPR>
__device__ __forceinline__ float row_group_sum(float a) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) a += __shfl_xor(a, o);
  return a;
}

template <typename XT, int LPR>
__global__ void __launch_bounds__(kRowThreads)
k_rmsnorm_fwd_short(const XT* __restrict__ X, int64_t rows, int D8, const float* __restrict__ g, float eps,
                    bf16_t* __restrict__ H, float* __restrict__ rstd) {
  constexpr int RPB = kRowThreads / LPR;           // rows per workgroup
  const int sub = threadIdx.x % LPR;
  const int64_t row = blockIdx.x * (int64_t)RPB + threadIdx.x / LPR;
  const bool on = row < rows && sub < D8;
  float v[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f}, gg[8], o[8];
  if (on) W8<XT>::load(X + (row * D8 + sub) * 8, v);
  float ss = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) ss += v[j] * v[j];
  ss = row_group_sum<LPR>(ss);
  const float r = 1.0f / sqrtf(ss / static_cast<float>(D8 * 8) + eps);
  if (row < rows && sub == 0) rstd[row] = r;
  if (!on) return;
  load8(g + sub * 8, gg);
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (v[j] * r) * gg[j];
  W8<bf16_t>::store(H + (row * D8 + sub) * 8, o);
}

template <typename XT, int LPR>
__global__ void __launch_bounds__(kRowThreads)
k_rmsnorm_bwd_short(const bf16_t* __restrict__ dH1, const bf16_t* __restrict__ dH2, const bf16_t* __restrict__ dH3,
                    const XT* __restrict__ X, int64_t rows, int D8, const float* __restrict__ g,
                    const float* __restrict__ rstd, const bf16_t* __restrict__ d_res, bf16_t* __restrict__ dX) {
  constexpr int RPB = kRowThreads / LPR;
  const int sub = threadIdx.x % LPR;
  const int64_t row = blockIdx.x * (int64_t)RPB + threadIdx.x / LPR;
  const bool on = row < rows && sub < D8;
  const int64_t at = (row * D8 + sub) * 8;
  float v[8], gg[8], d1[8], o[8];
  float dot = 0.0f;
  if (on) {
    W8<XT>::load(X + at, v);
    load8(g + sub * 8, gg);
    load_dh(dH1, dH2, dH3, at, d1);
#pragma unroll
    for (int j = 0; j < 8; ++j) dot += v[j] * (gg[j] * d1[j]);
  }
  dot = row_group_sum<LPR>(dot);
  if (!on) return;
  const float r = rstd[row];
  const float k = (r * r * r) * (dot / static_cast<float>(D8 * 8));
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = r * (gg[j] * d1[j]) - v[j] * k;
  if (d_res) {
    float d2[8];
    W8<bf16_t>::load(d_res + at, d2);
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] += d2[j];
  }
  W8<bf16_t>::store(dX + at, o);
}

__device__ __forceinline__ float sigmoidf_(float p) { return 1.0f / (1.0f + __expf(-p)); }

// a = SiLU(p) q
__global__ void __launch_bounds__(kEltThreads)
k_silu_mul_fwd(const bf16_t* __restrict__ P, const bf16_t* __restrict__ Q, int64_t n8, bf16_t* __restrict__ A) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  float p[8], q[8], a[8];
  W8<bf16_t>::load(P + i * 8, p);
  W8<bf16_t>::load(Q + i * 8, q);
#pragma unroll
  for (int j = 0; j < 8; ++j) a[j] = (p[j] * sigmoidf_(p[j])) * q[j];
  W8<bf16_t>::store(A + i * 8, a);
}

// dp = da q s (1 + p (1 - s)),  dq = da p s,  s = sigmoid(p)
__global__ void __launch_bounds__(kEltThreads)
k_silu_mul_bwd(const bf16_t* __restrict__ dA, const bf16_t* __restrict__ P, const bf16_t* __restrict__ Q, int64_t n8,
               bf16_t* __restrict__ dP, bf16_t* __restrict__ dQ) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  float da[8], p[8], q[8], dp[8], dq[8];
  W8<bf16_t>::load(dA + i * 8, da);
  W8<bf16_t>::load(P + i * 8, p);
  W8<bf16_t>::load(Q + i * 8, q);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float s = sigmoidf_(p[j]);
    dp[j] = (da[j] * q[j]) * (s * (1.0f + p[j] * (1.0f - s)));
    dq[j] = da[j] * (p[j] * s);
  }
  W8<bf16_t>::store(dP + i * 8, dp);
  W8<bf16_t>::store(dQ + i * 8, dq);
}

// y = x + d;  r = y - y_fp;  per-workgroup sum of r^2 (double);  dy = bf16(two_scale r)
template <typename XT, typename YT>
__global__ void __launch_bounds__(kEltThreads)
k_block_output_loss(const XT* __restrict__ X, const bf16_t* __restrict__ Dm, const YT* __restrict__ Yfp, int64_t n8,
                    float two_scale, bf16_t* __restrict__ Y, bf16_t* __restrict__ dY, double* __restrict__ partials) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  float sq = 0.0f;
  if (i < n8) {
    float x[8], d[8], yf[8], y[8], g[8];
    W8<XT>::load(X + i * 8, x);
    W8<bf16_t>::load(Dm + i * 8, d);
    W8<YT>::load(Yfp + i * 8, yf);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      y[j] = x[j] + d[j];
      const float r = y[j] - yf[j];
      sq += r * r;
      g[j] = two_scale * r;
    }
    if (Y) W8<bf16_t>::store(Y + i * 8, y);
    W8<bf16_t>::store(dY + i * 8, g);
  }
  __shared__ double s[kEltThreads / 64];
  double a = static_cast<double>(sq);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) partials[blockIdx.x] = (s[0] + s[1]) + (s[2] + s[3]);
}

// y = x + d (the residual connection between the two halves of a block)
template <typename XT>
__global__ void __launch_bounds__(kEltThreads)
k_residual_add(const XT* __restrict__ X, const bf16_t* __restrict__ Dm, int64_t n8, bf16_t* __restrict__ Y) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  float x[8], d[8];
  W8<XT>::load(X + i * 8, x);
  W8<bf16_t>::load(Dm + i * 8, d);
#pragma unroll
  for (int j = 0; j < 8; ++j) x[j] += d[j];
  W8<bf16_t>::store(Y + i * 8, x);
}

inline unsigned blocks_for(int64_t n8) { return static_cast<unsigned>((n8 + kEltThreads - 1) / kEltThreads); }

}  // namespace

inline int lanes_per_row(int64_t D) { return D <= 64 ? 8 : D <= 128 ? 16 : D <= 256 ? 32 : 64; }

hipError_t launch_rmsnorm_fwd(const void* X, bool x_bf16, int64_t T, int64_t D, const float* g, float eps, bf16_t* H,
                              float* rstd, hipStream_t st) {
  const dim3 block(kRowThreads);
  if (D <= 512) {
    const int lpr = lanes_per_row(D), rpb = kRowThreads / lpr, d8 = static_cast<int>(D / 8);
    const dim3 grid(static_cast<unsigned>((T + rpb - 1) / rpb));
#define FAAR_RF(XT, LPR) \
  hipLaunchKernelGGL((k_rmsnorm_fwd_short<XT, LPR>), grid, block, 0, st, static_cast<const XT*>(X), T, d8, g, eps, H, rstd)
#define FAAR_RF_T(XT) \
  do { if (lpr == 8) FAAR_RF(XT, 8); else if (lpr == 16) FAAR_RF(XT, 16); else if (lpr == 32) FAAR_RF(XT, 32); else FAAR_RF(XT, 64); } while (0)
    if (x_bf16) FAAR_RF_T(bf16_t); else FAAR_RF_T(float);
#undef FAAR_RF_T
#undef FAAR_RF
    return hipGetLastError();
  }
  const dim3 grid(static_cast<unsigned>(T));
  if (x_bf16)
    hipLaunchKernelGGL(k_rmsnorm_fwd<bf16_t>, grid, block, 0, st, static_cast<const bf16_t*>(X), D / 8, g, eps, H, rstd);
  else
    hipLaunchKernelGGL(k_rmsnorm_fwd<float>, grid, block, 0, st, static_cast<const float*>(X), D / 8, g, eps, H, rstd);
  return hipGetLastError();
}

hipError_t launch_rmsnorm_bwd(const bf16_t* dH1, const bf16_t* dH2, const bf16_t* dH3, const void* X, bool x_bf16, int64_t T,
                              int64_t D, const float* g, const float* rstd, const bf16_t* d_res, bf16_t* dX, hipStream_t st) {
  const dim3 block(kRowThreads);
  if (D <= 512) {
    const int lpr = lanes_per_row(D), rpb = kRowThreads / lpr, d8 = static_cast<int>(D / 8);
    const dim3 grid(static_cast<unsigned>((T + rpb - 1) / rpb));
#define FAAR_RB(XT, LPR) \
  hipLaunchKernelGGL((k_rmsnorm_bwd_short<XT, LPR>), grid, block, 0, st, dH1, dH2, dH3, static_cast<const XT*>(X), T, d8, g, rstd, d_res, dX)
#define FAAR_RB_T(XT) \
  do { if (lpr == 8) FAAR_RB(XT, 8); else if (lpr == 16) FAAR_RB(XT, 16); else if (lpr == 32) FAAR_RB(XT, 32); else FAAR_RB(XT, 64); } while (0)
    if (x_bf16) FAAR_RB_T(bf16_t); else FAAR_RB_T(float);
#undef FAAR_RB_T
#undef FAAR_RB
    return hipGetLastError();
  }
  const dim3 grid(static_cast<unsigned>(T));
  if (x_bf16)
    hipLaunchKernelGGL(k_rmsnorm_bwd<bf16_t>, grid, block, 0, st, dH1, dH2, dH3, static_cast<const bf16_t*>(X), D / 8, g, rstd, d_res, dX);
  else
    hipLaunchKernelGGL(k_rmsnorm_bwd<float>, grid, block, 0, st, dH1, dH2, dH3, static_cast<const float*>(X), D / 8, g, rstd, d_res, dX);
  return hipGetLastError();
}

hipError_t launch_silu_mul_fwd(const bf16_t* P, const bf16_t* Q, int64_t n, bf16_t* A, hipStream_t st) {
  hipLaunchKernelGGL(k_silu_mul_fwd, dim3(blocks_for(n / 8)), dim3(kEltThreads), 0, st, P, Q, n / 8, A);
  return hipGetLastError();
}

hipError_t launch_silu_mul_bwd(const bf16_t* dA, const bf16_t* P, const bf16_t* Q, int64_t n, bf16_t* dP, bf16_t* dQ,
                               hipStream_t st) {
  hipLaunchKernelGGL(k_silu_mul_bwd, dim3(blocks_for(n / 8)), dim3(kEltThreads), 0, st, dA, P, Q, n / 8, dP, dQ);
  return hipGetLastError();
}

hipError_t launch_residual_add(const void* X, bool x_bf16, const bf16_t* Dm, int64_t n, bf16_t* Y, hipStream_t st) {
  const dim3 grid(blocks_for(n / 8)), block(kEltThreads);
  if (x_bf16)
    hipLaunchKernelGGL(k_residual_add<bf16_t>, grid, block, 0, st, static_cast<const bf16_t*>(X), Dm, n / 8, Y);
  else
    hipLaunchKernelGGL(k_residual_add<float>, grid, block, 0, st, static_cast<const float*>(X), Dm, n / 8, Y);
  return hipGetLastError();
}

int64_t block_loss_blocks(int64_t n) { return (n / 8 + kEltThreads - 1) / kEltThreads; }

hipError_t launch_block_output_loss(const void* X, bool x_bf16, const bf16_t* Dm, const void* Yfp, bool y_bf16, int64_t n,
                                    float two_scale, bf16_t* Y, bf16_t* dY, double* partials, hipStream_t st) {
  const dim3 grid(blocks_for(n / 8)), block(kEltThreads);
#define FAAR_BL(XT, YT) \
  hipLaunchKernelGGL((k_block_output_loss<XT, YT>), grid, block, 0, st, static_cast<const XT*>(X), Dm, static_cast<const YT*>(Yfp), \
                     n / 8, two_scale, Y, dY, partials)
  if (x_bf16) { if (y_bf16) FAAR_BL(bf16_t, bf16_t); else FAAR_BL(bf16_t, float); }
  else        { if (y_bf16) FAAR_BL(float, bf16_t);  else FAAR_BL(float, float); }
#undef FAAR_BL
  return hipGetLastError();
}

}  // namespace faar
