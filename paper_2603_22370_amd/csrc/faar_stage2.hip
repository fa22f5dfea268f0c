// Stage-2 objective on given model outputs (paper Sec. 3.5 "Stage 2", Eq. 6; Table 2 steps 18-22):
// temperature softmax of two logit tensors, KL(P_fp || P_q) and its gradient with respect to the quantised
// model's logits, the Frobenius MSE of the last hidden states and its gradient, and the sum of the layers'
// Round Losses.  HBM-bound row kernels: one workgroup per token row, a single pass for the loss (online
// max / sum / weighted-sum), a second pass over the same row (served from cache) only when the gradient is wanted.
#include <cmath>

#include "faar_device.h"
#include "faar_internal.h"

namespace faar {
namespace {

constexpr int kRowThreads = 1024;

// Running statistics of one row for a = z_fp / tau and b = z_q / tau:
//   ma = max a, sa = sum exp(a - ma), w = sum exp(a - ma) (a - b);  mb = max b, sb = sum exp(b - mb)
struct RowStats { float ma, sa, w, mb, sb; };

__device__ __forceinline__ RowStats merge(const RowStats& x, const RowStats& y) {
  RowStats r;
  // a side that has seen no element has max -inf and sums 0: its factor is exp(-inf) = 0, or 1 when both are empty
  r.ma = fmaxf(x.ma, y.ma);
  const float fx = x.ma == r.ma ? 1.0f : __expf(x.ma - r.ma), fy = y.ma == r.ma ? 1.0f : __expf(y.ma - r.ma);
  r.sa = x.sa * fx + y.sa * fy;
  r.w = x.w * fx + y.w * fy;
  r.mb = fmaxf(x.mb, y.mb);
  const float gx = x.mb == r.mb ? 1.0f : __expf(x.mb - r.mb), gy = y.mb == r.mb ? 1.0f : __expf(y.mb - r.mb);
  r.sb = x.sb * gx + y.sb * gy;
  return r;
}

__device__ __forceinline__ RowStats shuffle_xor(const RowStats& x, int o) {
  RowStats r;
  r.ma = __shfl_xor(x.ma, o); r.sa = __shfl_xor(x.sa, o); r.w = __shfl_xor(x.w, o);
  r.mb = __shfl_xor(x.mb, o); r.sb = __shfl_xor(x.sb, o);
  return r;
}

// One vocabulary entry added to the running sums (st.ma / st.mb already cover it).  A logit of -inf (a masked
// entry) has probability 0: it adds nothing to either sum, and by the convention 0 log 0 = 0 nothing to the KL
// term either -- also where only z_fp is -inf.  Where P_fp > 0 and z_q = -inf the term, and the row's KL, is +inf.
// A row whose logits are all -inf has no softmax; its results are NaN.
__device__ __forceinline__ void accumulate(RowStats& st, float a, float b) {
  const float ea = a == -INFINITY ? 0.0f : __expf(a - st.ma);
  st.sa += ea;
  if (ea != 0.0f) st.w += ea * (a - b);
  st.sb += b == -INFINITY ? 0.0f : __expf(b - st.mb);
}

template <typename ZT>
__global__ void __launch_bounds__(kRowThreads)
k_stage2_kl(const ZT* __restrict__ Zf, const ZT* __restrict__ Zq, int64_t v8, float inv_tau, float grad_coef,
            ZT* __restrict__ dZq, double* __restrict__ kl_rows) {
  const int64_t row = blockIdx.x;
  const ZT* zf = Zf + row * v8 * 8;
  const ZT* zq = Zq + row * v8 * 8;
  const float ninf = -INFINITY;
  RowStats st{ninf, 0.0f, 0.0f, ninf, 0.0f};
  for (int64_t c = threadIdx.x; c < v8; c += kRowThreads) {
    float a[8], b[8];
    W8<ZT>::load(zf + c * 8, a);
    W8<ZT>::load(zq + c * 8, b);
    float ca = ninf, cb = ninf;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      a[j] *= inv_tau;
      b[j] *= inv_tau;
      ca = fmaxf(ca, a[j]);
      cb = fmaxf(cb, b[j]);
    }
    if (ca > st.ma) {  // rescale the running sums to the new maximum
      const float f = __expf(st.ma - ca);
      st.sa *= f;
      st.w *= f;
      st.ma = ca;
    }
    if (cb > st.mb) {
      st.sb *= __expf(st.mb - cb);
      st.mb = cb;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) accumulate(st, a[j], b[j]);
  }
  // fixed-order reduction: butterfly inside each wavefront, then the wavefronts in index order
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) st = merge(st, shuffle_xor(st, o));
  __shared__ RowStats per_wave[kRowThreads / 64];
  __shared__ RowStats row_stats;
  if ((threadIdx.x & 63) == 0) per_wave[threadIdx.x >> 6] = st;
  __syncthreads();
  if (threadIdx.x == 0) {
    RowStats t = per_wave[0];
    for (int i = 1; i < kRowThreads / 64; ++i) t = merge(t, per_wave[i]);
    row_stats = t;
    // sum_j P_fp (log P_fp - log P_q) = w / sa - (ma - mb) - log(sa / sb); combined in double, with the two
    // log-sum-exp terms taken as one difference so that nearly equal distributions do not cancel at size log(vocab)
    kl_rows[row] = static_cast<double>(t.w) / static_cast<double>(t.sa) -
                   (static_cast<double>(t.ma) - static_cast<double>(t.mb)) -
                   log(static_cast<double>(t.sa) / static_cast<double>(t.sb));
  }
  if (!dZq) return;
  __syncthreads();
  const RowStats t = row_stats;
  const float ia = 1.0f / t.sa, ib = 1.0f / t.sb;
  ZT* g = dZq + row * v8 * 8;
  for (int64_t c = threadIdx.x; c < v8; c += kRowThreads) {
    float a[8], b[8], o[8];
    W8<ZT>::load(zf + c * 8, a);
    W8<ZT>::load(zq + c * 8, b);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      o[j] = grad_coef * (__expf(b[j] * inv_tau - t.mb) * ib - __expf(a[j] * inv_tau - t.ma) * ia);
    W8<ZT>::store(g + c * 8, o);
  }
}

// bf16 rows of up to NC * 1024 chunks (8 logits each): the row of Z_fp stays in registers (packed bf16, NC x 4
// VGPRs per lane) and the first kLdsChunks chunks per lane of Z_q's row stay in LDS between the loss pass and
// the gradient pass, so that only the rest of Z_q is read a second time.
constexpr int kLdsChunks = 9;  // 9 x 1024 lanes x 16 B = 144 KB of the 160 KB LDS

__device__ __forceinline__ void unpack8(const uint4& q, float (&x)[8]) {
  const uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(r[i] << 16);
    x[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
  }
}

template <int NC>
__global__ void __launch_bounds__(kRowThreads)
k_stage2_kl_resident(const bf16_t* __restrict__ Zf, const bf16_t* __restrict__ Zq, int64_t v8, float inv_tau,
                     float grad_coef, bf16_t* __restrict__ dZq, double* __restrict__ kl_rows) {
  static_assert(NC >= kLdsChunks, "the LDS part is a prefix of the per-lane chunks");
  __shared__ uint4 q_lds[kLdsChunks][kRowThreads];
  const int64_t row = blockIdx.x;
  const uint4* zf = reinterpret_cast<const uint4*>(Zf + row * v8 * 8);
  const uint4* zq = reinterpret_cast<const uint4*>(Zq + row * v8 * 8);
  const float ninf = -INFINITY;
  RowStats st{ninf, 0.0f, 0.0f, ninf, 0.0f};
  uint4 rf[NC];
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int64_t c = threadIdx.x + (int64_t)k * kRowThreads;
    rf[k] = make_uint4(0u, 0u, 0u, 0u);
    if (c < v8) {
      rf[k] = zf[c];
      const uint4 rq = zq[c];
      if (k < kLdsChunks) q_lds[k][threadIdx.x] = rq;
      float a[8], b[8];
      unpack8(rf[k], a);
      unpack8(rq, b);
      float ca = ninf, cb = ninf;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        a[j] *= inv_tau;
        b[j] *= inv_tau;
        ca = fmaxf(ca, a[j]);
        cb = fmaxf(cb, b[j]);
      }
      if (ca > st.ma) {
        const float f = __expf(st.ma - ca);
        st.sa *= f;
        st.w *= f;
        st.ma = ca;
      }
      if (cb > st.mb) {
        st.sb *= __expf(st.mb - cb);
        st.mb = cb;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) accumulate(st, a[j], b[j]);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) st = merge(st, shuffle_xor(st, o));
  __shared__ RowStats per_wave[kRowThreads / 64];
  __shared__ RowStats row_stats;
  if ((threadIdx.x & 63) == 0) per_wave[threadIdx.x >> 6] = st;
  __syncthreads();
  if (threadIdx.x == 0) {
    RowStats t = per_wave[0];
    for (int i = 1; i < kRowThreads / 64; ++i) t = merge(t, per_wave[i]);
    row_stats = t;
    kl_rows[row] = static_cast<double>(t.w) / static_cast<double>(t.sa) -
                   (static_cast<double>(t.ma) - static_cast<double>(t.mb)) -
                   log(static_cast<double>(t.sa) / static_cast<double>(t.sb));
  }
  if (!dZq) return;
  __syncthreads();
  const RowStats t = row_stats;
  const float ia = 1.0f / t.sa, ib = 1.0f / t.sb;
  uint4* g = reinterpret_cast<uint4*>(dZq + row * v8 * 8);
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int64_t c = threadIdx.x + (int64_t)k * kRowThreads;
    if (c < v8) {
      const uint4 rq = k < kLdsChunks ? q_lds[k][threadIdx.x] : zq[c];   // each lane reads back its own LDS slots
      float a[8], b[8];
      unpack8(rf[k], a);
      unpack8(rq, b);
      uint32_t o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        o[j] = f32_to_bf16(grad_coef * (__expf(b[j] * inv_tau - t.mb) * ib - __expf(a[j] * inv_tau - t.ma) * ia));
      g[c] = make_uint4(o[0] | (o[1] << 16), o[2] | (o[3] << 16), o[4] | (o[5] << 16), o[6] | (o[7] << 16));
    }
  }
}

template <typename HT>
__global__ void __launch_bounds__(kEltThreads)
k_stage2_mse(const HT* __restrict__ Hf, const HT* __restrict__ Hq, int64_t n8, float two_scale, HT* __restrict__ dHq,
             double* __restrict__ partials) {
  float s = 0.0f;
  for (int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x; i < n8; i += (int64_t)gridDim.x * kEltThreads) {
    float f[8], q[8], o[8];
    W8<HT>::load(Hf + i * 8, f);
    W8<HT>::load(Hq + i * 8, q);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float d = q[j] - f[j];
      s += d * d;
      o[j] = two_scale * d;
    }
    if (dHq) W8<HT>::store(dHq + i * 8, o);
  }
  double a = static_cast<double>(s);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
  __shared__ double sw[kEltThreads / 64];
  if ((threadIdx.x & 63) == 0) sw[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kEltThreads / 64; ++i) t += sw[i];
    partials[blockIdx.x] = t;
  }
}

// losses[0] = kl_scale * sum kl_rows, [1] = mse_scale * sum partials, [2] = sum round_losses,
// [3] = lambda_kl [0] + [1] + lambda_round [2]; sums in a fixed order, in double
__global__ void __launch_bounds__(kEltThreads)
k_stage2_finalize(const double* __restrict__ kl_rows, int64_t n_rows, float kl_scale, const double* __restrict__ mse_partials,
                  int64_t n_mse, float mse_scale, const float* __restrict__ round_losses, int64_t n_layers, float lambda_kl,
                  float lambda_round, float* __restrict__ losses) {
  double a = 0.0, b = 0.0, c = 0.0;
  for (int64_t i = threadIdx.x; i < n_rows; i += kEltThreads) a += kl_rows[i];
  for (int64_t i = threadIdx.x; i < n_mse; i += kEltThreads) b += mse_partials[i];
  for (int64_t i = threadIdx.x; i < n_layers; i += kEltThreads) c += static_cast<double>(round_losses[i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_xor(a, o);
    b += __shfl_xor(b, o);
    c += __shfl_xor(c, o);
  }
  __shared__ double sa[kEltThreads / 64], sb[kEltThreads / 64], sc[kEltThreads / 64];
  if ((threadIdx.x & 63) == 0) {
    sa[threadIdx.x >> 6] = a;
    sb[threadIdx.x >> 6] = b;
    sc[threadIdx.x >> 6] = c;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = b = c = 0.0;
    for (int i = 0; i < kEltThreads / 64; ++i) {
      a += sa[i];
      b += sb[i];
      c += sc[i];
    }
    const double kl = a * static_cast<double>(kl_scale), mse = b * static_cast<double>(mse_scale);
    losses[0] = static_cast<float>(kl);
    losses[1] = static_cast<float>(mse);
    losses[2] = static_cast<float>(c);
    losses[3] = static_cast<float>(static_cast<double>(lambda_kl) * kl + mse + static_cast<double>(lambda_round) * c);
  }
}

}  // namespace

int64_t stage2_mse_blocks(int64_t n) {
  const int64_t b = (n / 8 + kEltThreads - 1) / kEltThreads;
  return b < kStepBwdMaxBlocks ? (b > 0 ? b : 1) : kStepBwdMaxBlocks;
}

hipError_t launch_stage2(const Stage2Args& a, hipStream_t st) {
  const float inv_tau = 1.0f / a.tau;
  const float grad_coef = a.lambda_kl * a.kl_scale * inv_tau;
  const int64_t v8 = a.vocab / 8;
  if (a.z_bf16 && v8 <= 16 * kRowThreads)
    hipLaunchKernelGGL(k_stage2_kl_resident<16>, dim3(static_cast<unsigned>(a.T)), dim3(kRowThreads), 0, st,
                       static_cast<const bf16_t*>(a.Z_fp), static_cast<const bf16_t*>(a.Z_q), v8, inv_tau, grad_coef,
                       static_cast<bf16_t*>(a.dZ_q), a.kl_rows);
  else if (a.z_bf16 && v8 <= 19 * kRowThreads)
    hipLaunchKernelGGL(k_stage2_kl_resident<19>, dim3(static_cast<unsigned>(a.T)), dim3(kRowThreads), 0, st,
                       static_cast<const bf16_t*>(a.Z_fp), static_cast<const bf16_t*>(a.Z_q), v8, inv_tau, grad_coef,
                       static_cast<bf16_t*>(a.dZ_q), a.kl_rows);
  else if (a.z_bf16)
    hipLaunchKernelGGL(k_stage2_kl<bf16_t>, dim3(static_cast<unsigned>(a.T)), dim3(kRowThreads), 0, st,
                       static_cast<const bf16_t*>(a.Z_fp), static_cast<const bf16_t*>(a.Z_q), a.vocab / 8, inv_tau, grad_coef,
                       static_cast<bf16_t*>(a.dZ_q), a.kl_rows);
  else
    hipLaunchKernelGGL(k_stage2_kl<float>, dim3(static_cast<unsigned>(a.T)), dim3(kRowThreads), 0, st,
                       static_cast<const float*>(a.Z_fp), static_cast<const float*>(a.Z_q), a.vocab / 8, inv_tau, grad_coef,
                       static_cast<float*>(a.dZ_q), a.kl_rows);
  if (hipError_t e = hipGetLastError()) return e;
  const int64_t nh = a.T * a.D;
  const int64_t blocks = stage2_mse_blocks(nh);
  const float two_scale = 2.0f * a.mse_scale;
  if (a.h_bf16)
    hipLaunchKernelGGL(k_stage2_mse<bf16_t>, dim3(static_cast<unsigned>(blocks)), dim3(kEltThreads), 0, st,
                       static_cast<const bf16_t*>(a.H_fp), static_cast<const bf16_t*>(a.H_q), nh / 8, two_scale,
                       static_cast<bf16_t*>(a.dH_q), a.mse_partials);
  else
    hipLaunchKernelGGL(k_stage2_mse<float>, dim3(static_cast<unsigned>(blocks)), dim3(kEltThreads), 0, st,
                       static_cast<const float*>(a.H_fp), static_cast<const float*>(a.H_q), nh / 8, two_scale,
                       static_cast<float*>(a.dH_q), a.mse_partials);
  if (hipError_t e = hipGetLastError()) return e;
  hipLaunchKernelGGL(k_stage2_finalize, dim3(1), dim3(kEltThreads), 0, st, a.kl_rows, a.T, a.kl_scale, a.mse_partials, blocks,
                     a.mse_scale, a.round_losses, a.round_losses ? a.n_layers : 0, a.lambda_kl, a.lambda_round, a.losses);
  return hipGetLastError();
}

}  // namespace faar
