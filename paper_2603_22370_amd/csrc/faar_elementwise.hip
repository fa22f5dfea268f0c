// HBM-bound elementwise / codec kernels of the FAAR layer step (paper Sec. 3.1, 3.4; Table 2;
// Eq. 2-5, 7).  Every kernel uses the same mapping: one thread owns 8 consecutive weights (16 B
// of bf16, 32 B of float32), so a 16-weight scale block is an even/odd lane pair and its amax is
// one cross-lane exchange.  Loads and stores are 16 B per lane and fully coalesced.
#include <type_traits>

#include "faar_internal.h"

namespace faar {
namespace {

__device__ __forceinline__ float pair_max(float a) {
  return fmaxf(a, __shfl_xor(a, 1));
}

__device__ __forceinline__ float wave_max(float a) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a = fmaxf(a, __shfl_xor(a, o));
  return a;
}

__device__ __forceinline__ double wave_sum(double a) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
  return a;
}

// Fixed-order block sum of one double per thread (kEltThreads threads); result valid in thread 0.
__device__ __forceinline__ double block_sum(double a) {
  __shared__ double s[kEltThreads / 64];
  a = wave_sum(a);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  double r = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < kEltThreads / 64; ++i) r += s[i];
  }
  return r;
}

// ---- tensor amax -> s_global (Sec. 3.1: FP32 scale of scales) -------------------------------
template <typename WT>
__global__ void __launch_bounds__(kEltThreads) k_amax_partial(const WT* __restrict__ W, int64_t n8,
                                                              float* __restrict__ partials) {
  float a = 0.0f;
  for (int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x; i < n8;
       i += (int64_t)gridDim.x * kEltThreads) {
    float w[8];
    W8<WT>::load(W + i * 8, w);
#pragma unroll
    for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(w[j]));
  }
  __shared__ float s[kEltThreads / 64];
  a = wave_max(a);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 1; i < kEltThreads / 64; ++i) a = fmaxf(a, s[i]);
    partials[blockIdx.x] = a;
  }
}

__global__ void __launch_bounds__(kEltThreads) k_amax_final(const float* __restrict__ partials, int n,
                                                            float* __restrict__ s_global) {
  float a = 0.0f;
  for (int i = threadIdx.x; i < n; i += kEltThreads) a = fmaxf(a, partials[i]);
  __shared__ float s[kEltThreads / 64];
  a = wave_max(a);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 1; i < kEltThreads / 64; ++i) a = fmaxf(a, s[i]);
    *s_global = (a == 0.0f) ? 1.0f : a / 2688.0f;  // 2688 = 6 (largest node) * 448 (largest E4M3)
  }
}

// ---- codec operations on one chunk of 8 weights (thread i of a tensor owns weights 8i .. 8i+7) ----------------
// Shared by the single-tensor kernels and the batched ones below.  Inputs that a kernel reads exactly once are
// loaded with the nontemporal hint.

// Round-to-nearest quantisation (Sec. 3.1; Table 2 steps 2-3).  Both lanes of an even/odd pair must be active.
template <typename WT, bool kDequant>
__device__ __forceinline__ void quant_chunk(const WT* __restrict__ W, int64_t i, float sg, uint8_t* __restrict__ scales,
                                            uint32_t* __restrict__ codes, WT* __restrict__ W_dq, bool dq_in_units) {
  float w[8];
  W8<WT>::load_stream(W + i * 8, w);
  float a = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(w[j]));
  a = pair_max(a);
  const uint32_t byte = block_scale_byte(a, sg);
  const float sgv = e4m3_value(byte);
  const float s = sgv * sg;
  uint32_t packed = 0;
  float dq[8];
  const BlockDivider div(s, a);
  auto encode = [&](auto fast) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float wt = div.quotient<decltype(fast)::value>(fabsf(w[j]));
      // a zero weight has wt == 0 and therefore magnitude code 0; its nibble keeps the sign bit of w
      const uint32_t nib = ((__float_as_uint(w[j]) >> 31) << 3) | nearest_magnitude_code(wt);
      packed |= nib << (4 * j);
      if (kDequant) dq[j] = dequant(nib, sgv, dq_in_units ? 1.0f : sg);  // in units of s_global: an exact product
    }
  };
  if (div.fast) encode(std::true_type{}); else encode(std::false_type{});
  codes[i] = packed;
  if ((i & 1) == 0) scales[i >> 1] = static_cast<uint8_t>(byte);
  if (kDequant) W8<WT>::store(W_dq + i * 8, dq);
}

// V initialisation (Eq. 4)
template <typename WT>
__device__ __forceinline__ void init_v_chunk(const WT* __restrict__ W, int64_t i, float sg, const uint8_t* __restrict__ scales,
                                             float* __restrict__ V, uint32_t* __restrict__ floor_codes) {
  const float s = effective_scale(scales[i >> 1], sg);
  float w[8], v[8];
  W8<WT>::load_stream(W + i * 8, w);
  uint32_t packed = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const Interval iv = find_interval(w[j], s);
    v[j] = iv.v_init;
    packed |= (((__float_as_uint(w[j]) >> 31) << 3) | static_cast<uint32_t>(iv.k_lo)) << (4 * j);
  }
  store8(V + i * 8, v);
  if (floor_codes) floor_codes[i] = packed;
}

// Hardening + NVFP4 packing (Eq. 7; Table 2 steps 25-26); returns how many of the 8 nibbles differ from round-to-nearest
template <typename WT>
__device__ __forceinline__ unsigned harden_chunk(const WT* __restrict__ W, int64_t i, float sg, const uint8_t* __restrict__ scales,
                                                 const float* __restrict__ V, uint32_t* __restrict__ codes,
                                                 uint8_t* __restrict__ decisions, WT* __restrict__ W_final) {
  const float sgv = e4m3_value(scales[i >> 1]);
  const float s = sgv * sg;
  float w[8], v[8], dq[8];
  W8<WT>::load_stream(W + i * 8, w);
  W8<float>::load_stream(V + i * 8, v);
  uint32_t packed = 0, bits = 0;
  unsigned flips = 0;
  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(w[j]));
  const BlockDivider div(s, amax);
  auto encode = [&](auto fast) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float wt = div.quotient<decltype(fast)::value>(fabsf(w[j]));
      const int k_lo = interval_index(wt);
      const int up = v[j] >= 0.5f;
      const uint32_t nib = nibble(w[j], k_lo, up);
      flips += (nib & 7u) != nearest_magnitude_code(wt);  // differs from round-to-nearest (never for a zero weight)
      packed |= nib << (4 * j);
      bits |= static_cast<uint32_t>(up) << j;
      if (W_final) dq[j] = dequant(nib, sgv, sg);
    }
  };
  if (div.fast) encode(std::true_type{}); else encode(std::false_type{});
  codes[i] = packed;
  if (decisions) decisions[i] = static_cast<uint8_t>(bits);
  if (W_final) W8<WT>::store(W_final + i * 8, dq);
  return flips;
}

__device__ __forceinline__ void add_flips(unsigned flips, unsigned long long* __restrict__ flip_count) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) flips += __shfl_xor(flips, o);
  if ((threadIdx.x & 63) == 0 && flips) atomicAdd(flip_count, (unsigned long long)flips);
}

// ---- single-tensor kernels: one chunk per thread, as many blocks as chunks / 256 ---------------------------------
// (the shape that streams best on this part: a plain copy written this way moves 6.3 TB/s, the same copy as a
// grid-stride loop over a few thousand blocks, or with several chunks per thread, 4.4 - 5.9 TB/s)
template <typename WT, bool kDequant>
__global__ void __launch_bounds__(kEltThreads)
k_quant_rtn(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
            uint8_t* __restrict__ scales, uint32_t* __restrict__ codes, WT* __restrict__ W_dq, bool dq_in_units) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;  // n8 is even: both lanes of a pair leave together
  quant_chunk<WT, kDequant>(W, i, *s_global_p, scales, codes, W_dq, dq_in_units);
}

template <typename WT>
__global__ void __launch_bounds__(kEltThreads)
k_init_v(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
         const uint8_t* __restrict__ scales, float* __restrict__ V, uint32_t* __restrict__ floor_codes) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  init_v_chunk<WT>(W, i, *s_global_p, scales, V, floor_codes);
}

template <typename WT>
__global__ void __launch_bounds__(kEltThreads)
k_harden_pack(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
              const uint8_t* __restrict__ scales, const float* __restrict__ V,
              uint32_t* __restrict__ codes, uint8_t* __restrict__ decisions, WT* __restrict__ W_final,
              unsigned long long* __restrict__ flip_count) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  unsigned flips = 0;
  if (i < n8) flips = harden_chunk<WT>(W, i, *s_global_p, scales, V, codes, decisions, W_final);
  if (flip_count) add_flips(flips, flip_count);  // uniform branch: every lane of the block reaches the reduction
}

// ---- batched kernels: many tensors, one launch ----------------------------------------------------------------------
// A model's weight tensors are quantised, initialised and packed tensor by tensor, and most of them are small (a
// 2 M-weight projection is a 5 us launch, half of it ramp-up and tail).  The batched entry points put up to
// kBatchMax tensors into one launch: the descriptors travel in the kernel arguments, workgroup b finds its tensor by
// a binary search over the tensors' first workgroup indices (uniform: scalar loads) and then runs the same chunk code.
__device__ __forceinline__ int batch_item(const CodecBatch& B, uint32_t block) {
  int lo = 0, hi = B.n;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (B.first_block[mid] <= block) lo = mid; else hi = mid;
  }
  return lo;
}

// Per-tensor amax: kBatchAmaxBlocks workgroups per tensor walk its chunks with a stride; a tensor's partial maxima
// are finished by k_batch_amax_final (one workgroup per tensor).
template <typename WT>
__global__ void __launch_bounds__(kEltThreads) k_batch_amax_partial(CodecBatch B, float* __restrict__ partials) {
  const int item = blockIdx.x / kBatchAmaxBlocks, part = blockIdx.x % kBatchAmaxBlocks;
  const WT* W = static_cast<const WT*>(B.it[item].W);
  const int64_t n8 = B.it[item].n8;
  float a = 0.0f;
  for (int64_t i = part * (int64_t)kEltThreads + threadIdx.x; i < n8; i += (int64_t)kBatchAmaxBlocks * kEltThreads) {
    float w[8];
    W8<WT>::load(W + i * 8, w);   // read again by the quantise kernel: keep it cached
#pragma unroll
    for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(w[j]));
  }
  __shared__ float s[kEltThreads / 64];
  a = wave_max(a);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 1; i < kEltThreads / 64; ++i) a = fmaxf(a, s[i]);
    partials[blockIdx.x] = a;
  }
}

__global__ void __launch_bounds__(kEltThreads) k_batch_amax_final(CodecBatch B, const float* __restrict__ partials) {
  const int item = blockIdx.x;
  float a = 0.0f;
  for (int i = threadIdx.x; i < kBatchAmaxBlocks; i += kEltThreads) a = fmaxf(a, partials[item * kBatchAmaxBlocks + i]);
  __shared__ float s[kEltThreads / 64];
  a = wave_max(a);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 1; i < kEltThreads / 64; ++i) a = fmaxf(a, s[i]);
    *B.it[item].s_global = (a == 0.0f) ? 1.0f : a / 2688.0f;
  }
}

template <typename WT>
__global__ void __launch_bounds__(kEltThreads) k_batch_quant_rtn(CodecBatch B) {
  const int item = batch_item(B, blockIdx.x);
  const CodecItem& t = B.it[item];
  const int64_t i = (blockIdx.x - B.first_block[item]) * (int64_t)kEltThreads + threadIdx.x;
  if (i >= t.n8) return;
  quant_chunk<WT, false>(static_cast<const WT*>(t.W), i, *t.s_global, t.scales, t.codes, nullptr, false);
}

template <typename WT>
__global__ void __launch_bounds__(kEltThreads) k_batch_init_v(CodecBatch B) {
  const int item = batch_item(B, blockIdx.x);
  const CodecItem& t = B.it[item];
  const int64_t i = (blockIdx.x - B.first_block[item]) * (int64_t)kEltThreads + threadIdx.x;
  if (i >= t.n8) return;
  init_v_chunk<WT>(static_cast<const WT*>(t.W), i, *t.s_global, t.scales, t.V, t.codes);
}

template <typename WT>
__global__ void __launch_bounds__(kEltThreads) k_batch_harden_pack(CodecBatch B) {
  const int item = batch_item(B, blockIdx.x);
  const CodecItem& t = B.it[item];
  const int64_t i = (blockIdx.x - B.first_block[item]) * (int64_t)kEltThreads + threadIdx.x;
  if (i >= t.n8) return;
  (void)harden_chunk<WT>(static_cast<const WT*>(t.W), i, *t.s_global, t.scales, t.V, t.codes, nullptr, nullptr);
}

// ---- soft quantisation forward (Eq. 2-3) ----------------------------------------------------
__device__ __forceinline__ float h_beta(float v, float beta) {
  return 1.0f / (1.0f + __expf(-beta * (v - 0.5f)));
}

template <typename WT, bool kDelta, bool kFull>
__global__ void __launch_bounds__(kEltThreads)
k_softquant_fwd(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
                const uint8_t* __restrict__ scales, const float* __restrict__ V, float beta,
                bf16_t* __restrict__ Wt, bf16_t* __restrict__ Wq_full) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  const float s = effective_scale(scales[i >> 1], *s_global_p);
  float w[8], v[8], out[8], full[8];
  W8<WT>::load(W + i * 8, w);
  load8(V + i * 8, v);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const Interval iv = find_interval(w[j], s);
    const float wq = sign_of(w[j]) * ((iv.lo + h_beta(v[j], beta) * iv.width) * s);
    out[j] = kDelta ? wq - w[j] : wq;
    if (kFull) full[j] = wq;
  }
  W8<bf16_t>::store(Wt + i * 8, out);
  if (kFull) W8<bf16_t>::store(Wq_full + i * 8, full);
}

// dL/dv of Eq. 5 for one weight given g = dL/dW_q, plus its Round-Loss term.
__device__ __forceinline__ float grad_v(float g, float w, float s, float v, float beta, float lam_over_n,
                                        float& round_term) {
  const Interval iv = find_interval(w, s);
  const float h = h_beta(v, beta);
  const float t = 2.0f * v - 1.0f;
  round_term = 1.0f - t * t;
  return g * (sign_of(w) * s * iv.width * beta * (h * (1.0f - h))) + lam_over_n * (4.0f - 8.0f * v);
}

template <typename WT>
__global__ void __launch_bounds__(kEltThreads)
k_softquant_bwd(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
                const uint8_t* __restrict__ scales, const float* __restrict__ V, float beta,
                const float* __restrict__ G, int n_split, int64_t split_stride, float lam_over_n,
                float* __restrict__ dV, double* __restrict__ round_partials) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  float rsum = 0.0f;
  if (i < n8) {
    const float s = effective_scale(scales[i >> 1], *s_global_p);
    float w[8], v[8], g[8], d[8];
    W8<WT>::load(W + i * 8, w);
    load8(V + i * 8, v);
    load8(G + i * 8, g);
    for (int sp = 1; sp < n_split; ++sp) {
      float g2[8];
      load8(G + sp * split_stride + i * 8, g2);
#pragma unroll
      for (int j = 0; j < 8; ++j) g[j] += g2[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float rt;
      d[j] = grad_v(g[j], w[j], s, v[j], beta, lam_over_n, rt);
      rsum += rt;
    }
    store8(dV + i * 8, d);
  }
  const double bs = block_sum(static_cast<double>(rsum));
  if (threadIdx.x == 0) round_partials[blockIdx.x] = bs;
}



// ---- layer-step kernels on cached interval codes -------------------------------------------
// The interval of a weight (Table 2 step 3) depends only on W and the scales, which are frozen for the
// whole layer, so faar_layer_prepare stores it once as a nibble  signbit(w) << 3 | (w == 0 ? 7 : k_lo)
// and the per-step kernels skip the division and the node search.  Code 7 marks a zero weight
// (sign(0) = 0 in Eq. 2: no contribution to W_q and no data gradient).

template <typename WT>
__global__ void __launch_bounds__(kEltThreads)
k_interval_codes(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
                 const uint8_t* __restrict__ scales, uint32_t* __restrict__ icodes) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  const float s = effective_scale(scales[i >> 1], *s_global_p);
  float w[8];
  W8<WT>::load(W + i * 8, w);
  uint32_t packed = 0;
  float amax = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf(w[j]));
  const BlockDivider div(s, amax);
  auto encode = [&](auto fast) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float wt = div.quotient<decltype(fast)::value>(fabsf(w[j]));
      const uint32_t k = (w[j] == 0.0f) ? 7u : static_cast<uint32_t>(interval_index(wt));
      packed |= (((__float_as_uint(w[j]) >> 31) << 3) | k) << (4 * j);
    }
  };
  if (div.fast) encode(std::true_type{}); else encode(std::false_type{});
  icodes[i] = packed;
}

// lower node and interval width of magnitude code k in 0..6
__device__ __forceinline__ float node_lo(uint32_t k) {
  return k < 2u ? 0.5f * static_cast<float>(k) : __uint_as_float(((126u + (k >> 1)) << 23) | ((k & 1u) << 22));
}
__device__ __forceinline__ float node_width(uint32_t k) { return k < 4u ? 0.5f : (k < 6u ? 1.0f : 2.0f); }
// sigmoid through the hardware exp2 / reciprocal units (about 1 ulp each; not decision arithmetic)
__device__ __forceinline__ float h_beta_fast(float v, float beta) {
  return __builtin_amdgcn_rcpf(1.0f + __expf(-beta * (v - 0.5f)));
}
// signed scale  sign(w) * s  of a coded weight (0 for a zero weight)
__device__ __forceinline__ float signed_scale(uint32_t nib, float s) {
  return (nib & 7u) == 7u ? 0.0f : ((nib & 8u) ? -s : s);
}

// soft-quantised weight of one coded element
__device__ __forceinline__ float soft_weight(uint32_t nib, float s, float v, float beta) {
  const uint32_t k = nib & 7u;
  return signed_scale(nib, s) * (node_lo(k) + h_beta_fast(v, beta) * node_width(k));
}

__device__ __forceinline__ void store_bf16x8(bf16_t* p, const float (&x)[8]) {
  *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]),
                                            pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7]));
}

// delta = bf16(W_q - W) (and bf16(W_q)) for eight weights, plus their Round-Loss terms sum(1 - (2v - 1)^2) and, when
// the layer carries the constant H = C^T X_q (use_h; hh its eight values), the cross term sum(delta * H) of the loss, taken on the
// ROUNDED delta -- the operand the residual GEMM actually multiplies
template <typename WT, bool kFull>
__device__ __forceinline__ float forward8(const WT* __restrict__ W, int64_t i, uint32_t codes, float s,
                                          const float (&v)[8], float beta, bf16_t* __restrict__ delta,
                                          bf16_t* __restrict__ Wq_full, bool use_h, const float (&hh)[8], float& cross) {
  float w[8], out[8], full[8];
  W8<WT>::load(W + i * 8, w);
  float rsum = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float wq = soft_weight((codes >> (4 * j)) & 15u, s, v[j], beta);
    out[j] = wq - w[j];
    if (kFull) full[j] = wq;
    const float t = 2.0f * v[j] - 1.0f;
    rsum += 1.0f - t * t;
  }
  const uint4 packed = make_uint4(pack_bf16x2(out[0], out[1]), pack_bf16x2(out[2], out[3]),
                                  pack_bf16x2(out[4], out[5]), pack_bf16x2(out[6], out[7]));
  *reinterpret_cast<uint4*>(delta + i * 8) = packed;
  if (use_h) {   // hh stays in registers: indexed by constants only
    const uint32_t r[4] = {packed.x, packed.y, packed.z, packed.w};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      cross += __uint_as_float(r[j] << 16) * hh[2 * j] + __uint_as_float(r[j] & 0xFFFF0000u) * hh[2 * j + 1];
  }
  if (kFull) store_bf16x8(Wq_full + i * 8, full);
  return rsum;
}

template <typename WT, bool kFull>
__global__ void __launch_bounds__(kEltThreads)
k_step_fwd(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
           const uint8_t* __restrict__ scales, const uint32_t* __restrict__ icodes, const float* __restrict__ V,
           float beta, bf16_t* __restrict__ delta, bf16_t* __restrict__ Wq_full, double* __restrict__ round_partials,
           uint32_t* __restrict__ guard_slot, const float* __restrict__ H, double* __restrict__ cross_partials) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {  // a fresh forward: whatever tag the workspace held is void, verdict 1
    for (int i = 0; i < kTagWords; ++i) guard_slot[i] = 0u;
    guard_slot[kTagWords] = 1u;
  }
  float rsum = 0.0f, cross = 0.0f;
  const float sg = *s_global_p;
  for (int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x; i < n8; i += (int64_t)gridDim.x * kEltThreads) {
    float v[8], hh[8];
    load8(V + i * 8, v);
    if (H) load8(H + i * 8, hh);
    rsum += forward8<WT, kFull>(W, i, icodes[i], effective_scale(scales[i >> 1], sg), v, beta, delta, Wq_full,
                                H != nullptr, hh, cross);
  }
  const double bs = block_sum(static_cast<double>(rsum));
  if (threadIdx.x == 0) round_partials[blockIdx.x] = bs;
  if (H) {
    __syncthreads();                      // block_sum's scratch is reused
    const double cs = block_sum(static_cast<double>(cross));
    if (threadIdx.x == 0) cross_partials[blockIdx.x] = cs;
  }
}

// The forward-tag check of a step that consumes a prepared forward, for steps whose first kernel is not the residual
// GEMM (which otherwise does it): compare, clear, write the verdict.
__global__ void k_check_forward_tag(ForwardGuard guard) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    bool ok = true;
    for (int i = 0; i < kTagWords; ++i) ok = ok && guard.slot[i] == guard.expect.w[i];
    for (int i = 0; i < kTagWords; ++i) guard.slot[i] = 0u;
    guard.slot[kTagWords] = ok ? 1u : 0u;
  }
}

// ---- loss finalisation: fixed-order sums of the per-block partials (one block) ---------------
struct LossSums {
  const double* mse_partials;
  int64_t n_mse;
  float mse_scale;
  // with the constant part of the residual carried separately (R = A - C, A = x_scale * acc):
  // ||R||^2 = sum A^2 - 2 x_scale <delta, H> + ||C||^2; cross_partials sum to <delta, H>.  Null: mse_partials are ||R||^2.
  const double* cross_partials;
  int64_t n_cross;
  const double* c_norm2;
  const float* x_scale;
  const double* round_partials;
  int64_t n_round;
  double inv_n;
  float lambda_round;
  float *loss_mse, *loss_round, *loss_total;
};

__device__ __forceinline__ void finalize_block(const LossSums& f, bool valid = true) {
  if (!valid) {  // the step ran on a forward pass that is not the one its caller described: no result
    if (threadIdx.x == 0) {
      const float nan = __uint_as_float(0x7FC00000u);
      if (f.loss_mse) *f.loss_mse = nan;
      if (f.loss_round) *f.loss_round = nan;
      if (f.loss_total) *f.loss_total = nan;
    }
    return;
  }
  double a = 0.0, b = 0.0, c = 0.0;
  // per-thread partial sums in a fixed order; loads of one batch are independent
#pragma unroll 4
  for (int64_t i = threadIdx.x; i < f.n_mse; i += kEltThreads) a += f.mse_partials[i];
#pragma unroll 4
  for (int64_t i = threadIdx.x; i < f.n_round; i += kEltThreads) b += f.round_partials[i];
  if (f.cross_partials) {
#pragma unroll 4
    for (int64_t i = threadIdx.x; i < f.n_cross; i += kEltThreads) c += f.cross_partials[i];
  }
  __shared__ double sa[kEltThreads / 64], sb[kEltThreads / 64], sc[kEltThreads / 64];
  a = wave_sum(a);
  b = wave_sum(b);
  c = wave_sum(c);
  if ((threadIdx.x & 63) == 0) {
    sa[threadIdx.x >> 6] = a;
    sb[threadIdx.x >> 6] = b;
    sc[threadIdx.x >> 6] = c;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = 0.0;
    b = 0.0;
    c = 0.0;
    for (int i = 0; i < kEltThreads / 64; ++i) {
      a += sa[i];
      b += sb[i];
      c += sc[i];
    }
    if (f.cross_partials) a += *f.c_norm2 - 2.0 * static_cast<double>(f.x_scale ? *f.x_scale : 1.0f) * c;
    const double mse = a * static_cast<double>(f.mse_scale);
    const double rl = b * f.inv_n;
    if (f.loss_mse) *f.loss_mse = static_cast<float>(mse);
    if (f.loss_round) *f.loss_round = static_cast<float>(rl);
    if (f.loss_total) *f.loss_total = static_cast<float>(mse + static_cast<double>(f.lambda_round) * rl);
  }
}

__global__ void __launch_bounds__(kEltThreads) k_finalize_losses(LossSums f) { finalize_block(f); }

// Backward + Adam + clip over grid-stride blocks 0..gridDim.x-2.  With kEmit the same pass writes the next
// step's delta (and W_q) from the updated V at beta_next, with that V's Round-Loss partials.  The last block
// takes no weights: it finishes this step's losses from partial sums that earlier kernels completed.
template <typename WT, bool kEmit, bool kFull>
__global__ void __launch_bounds__(kEltThreads)
k_step_bwd_adam(int64_t n8, const float* __restrict__ s_global_p, const uint8_t* __restrict__ scales,
                const uint32_t* __restrict__ icodes, float* __restrict__ V, float* __restrict__ M,
                float* __restrict__ U, float beta, const float* __restrict__ G, int n_split, int64_t split_stride,
                const float* __restrict__ x_scale_p, float lam_over_n, AdamScalars o, LossSums fin, const WT* __restrict__ W, float beta_next,
                bf16_t* __restrict__ delta, bf16_t* __restrict__ Wq_full, double* __restrict__ round_next,
                uint32_t* __restrict__ guard_slot, ForwardTag next_tag, const float* __restrict__ H, float two_alpha_h,
                double* __restrict__ cross_next) {
  const int workers = static_cast<int>(gridDim.x) - 1;
  const bool valid = guard_slot[kTagWords] != 0u;  // written by an earlier kernel of this step
  if (static_cast<int>(blockIdx.x) == workers) {
    finalize_block(fin, valid);
    if (kEmit && valid && threadIdx.x == 0) {      // nobody in this launch reads the tag words
      for (int i = 0; i < kTagWords; ++i) guard_slot[i] = next_tag.w[i];
    }
    return;
  }
  if (!valid) return;
  float rsum = 0.0f, cross = 0.0f;
  const float sg = *s_global_p;
  const float xs = x_scale_p ? *x_scale_p : 1.0f;  // G = x_scale * (dY^T X_q-in-units)
  for (int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x; i < n8; i += (int64_t)workers * kEltThreads) {
    const float s = effective_scale(scales[i >> 1], sg);
    const uint32_t codes = icodes[i];
    float v[8], g[8], m[8], u[8], hh[8];
    load8(V + i * 8, v);
    load8(M + i * 8, m);
    load8(U + i * 8, u);
    load8(G + i * 8, g);
    for (int sp = 1; sp < n_split; ++sp) {
      float g2[8];
      load8(G + sp * split_stride + i * 8, g2);
#pragma unroll
      for (int j = 0; j < 8; ++j) g[j] += g2[j];
    }
    if (H) {  // the constant part of the gradient, -2 alpha C^T X_q (two_alpha_h is 0 when dY came from upstream)
      load8(H + i * 8, hh);
#pragma unroll
      for (int j = 0; j < 8; ++j) g[j] -= two_alpha_h * hh[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t nib = (codes >> (4 * j)) & 15u;
      const float h = h_beta_fast(v[j], beta);
      const float d = (xs * g[j]) * (signed_scale(nib, s) * node_width(nib & 7u) * beta * (h * (1.0f - h))) +
                      lam_over_n * (4.0f - 8.0f * v[j]);
      m[j] = o.beta1 * m[j] + (1.0f - o.beta1) * d;
      u[j] = o.beta2 * u[j] + (1.0f - o.beta2) * (d * d);
      const float step = o.lr * (m[j] * o.inv_bc1) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(u[j] * o.inv_bc2) + o.eps);
      v[j] = fminf(fmaxf(v[j] - step, 0.0f), 1.0f);  // V clipped to [0, 1] after every update
    }
    store8(V + i * 8, v);
    store8(M + i * 8, m);
    store8(U + i * 8, u);
    if (kEmit) rsum += forward8<WT, kFull>(W, i, codes, s, v, beta_next, delta, Wq_full, H != nullptr, hh, cross);
  }
  if (kEmit) {
    const double bs = block_sum(static_cast<double>(rsum));
    if (threadIdx.x == 0) round_next[blockIdx.x] = bs;
    if (H) {
      __syncthreads();                    // block_sum's scratch is reused
      const double cs = block_sum(static_cast<double>(cross));
      if (threadIdx.x == 0) cross_next[blockIdx.x] = cs;
    }
  }
}

// ---- stochastic-rounding candidates and the loss of a hardened candidate (Sec. 3.2, Table 1) ----
// Philox-4x32 with 10 rounds (Salmon et al., SC'11): counter-based, so any implementation draws the same words.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
    c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
    k.x += 0x9E3779B9u;
    k.y += 0xBB67AE85u;
  }
  return c;
}

// v = 1 with probability v_init (Eq. 4), else 0: element i draws word i % 4 of
// Philox(counter = (i / 4 low, i / 4 high, sample, 0), key = seed); u = (word >> 8) * 2^-24; up iff u < v_init
template <typename WT>
__global__ void __launch_bounds__(kEltThreads)
k_stochastic_v(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
               const uint8_t* __restrict__ scales, uint32_t seed_lo, uint32_t seed_hi, uint32_t sample,
               float* __restrict__ V) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n8) return;
  const float s = effective_scale(scales[i >> 1], *s_global_p);
  float w[8], v[8];
  W8<WT>::load(W + i * 8, w);
  uint32_t word[8];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint64_t blk = static_cast<uint64_t>(i) * 2 + h;
    const uint4 r = philox4x32_10(make_uint4(static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32), sample, 0u),
                                  make_uint2(seed_lo, seed_hi));
    word[4 * h] = r.x; word[4 * h + 1] = r.y; word[4 * h + 2] = r.z; word[4 * h + 3] = r.w;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float u = static_cast<float>(word[j] >> 8) * 0x1p-24f;
    v[j] = u < find_interval(w[j], s).v_init ? 1.0f : 0.0f;
  }
  store8(V + i * 8, v);
}

// delta = bf16(W_final - W) with W_final = sign * node * block scale * tensor scale in float32 (the value an
// NVFP4 decoder produces, not rounded to W's storage type): the perturbation whose reconstruction loss ranks a
// rounding candidate
template <typename WT>
__global__ void __launch_bounds__(kEltThreads)
k_hardened_delta(const WT* __restrict__ W, int64_t n8, const float* __restrict__ s_global_p,
                 const uint8_t* __restrict__ scales, const float* __restrict__ V, bf16_t* __restrict__ delta,
                 uint32_t* __restrict__ guard_slot) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i == 0) {
    for (int k = 0; k < kTagWords; ++k) guard_slot[k] = 0u;   // delta replaces whatever forward the workspace held
  }
  if (i >= n8) return;
  const float sg = *s_global_p;
  const float sgv = e4m3_value(scales[i >> 1]);
  const float s = sgv * sg;
  float w[8], v[8], out[8];
  W8<WT>::load(W + i * 8, w);
  load8(V + i * 8, v);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int k_lo = interval_index(normalised(w[j], s));
    out[j] = dequant(nibble(w[j], k_lo, v[j] >= 0.5f), sgv, sg) - w[j];
  }
  store_bf16x8(delta + i * 8, out);
}

// ---- bf16 transpose with zero padding (X_q^T for the dW GEMM) -------------------------------
// 64 x 64 tiles through LDS; 16-byte global accesses on both sides (rows of the tile are 128 contiguous bytes).
// The LDS row pitch of 33 words makes the transposed 2-byte reads of a wavefront hit 32 distinct banks.
__global__ void __launch_bounds__(256)
k_transpose_bf16(const bf16_t* __restrict__ in, int64_t rows, int64_t cols, bf16_t* __restrict__ out,
                 int64_t ld_out, unsigned tiles_c) {
  __shared__ uint32_t tile[64][33];
  const int64_t r0 = (blockIdx.x / tiles_c) * 64LL, c0 = (blockIdx.x % tiles_c) * 64LL;
  const int sub = threadIdx.x >> 3, ch = threadIdx.x & 7;
  const bool vec_in = (cols % 8) == 0;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int r = p * 32 + sub;
    const int64_t rr = r0 + r, cc = c0 + ch * 8;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (rr < rows) {
      if (vec_in && cc + 8 <= cols) {
        v = *reinterpret_cast<const uint4*>(in + rr * cols + cc);
      } else {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = (cc + j < cols) ? in[rr * cols + cc + j] : 0u;
        v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
      }
    }
    tile[r][ch * 4 + 0] = v.x;
    tile[r][ch * 4 + 1] = v.y;
    tile[r][ch * 4 + 2] = v.z;
    tile[r][ch * 4 + 3] = v.w;
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int oc = p * 32 + sub;                       // output row within the tile = input column
    const int64_t cc = c0 + oc, rr = r0 + ch * 8;      // eight consecutive input rows -> 16 contiguous output bytes
    if (cc < cols && rr < ld_out) {                    // ld_out is a multiple of 64: a chunk is inside or outside as a whole
      uint32_t e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = (tile[ch * 8 + j][oc >> 1] >> ((oc & 1) * 16)) & 0xFFFFu;
      *reinterpret_cast<uint4*>(out + cc * ld_out + rr) =
          make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
  }
}

// ---- the constant part of the gradient, H = C^T X_q (once per layer) -----------------------------------------------
// C (float32, tokens interleaved in groups of four: [ceil(T/4)][O][4]) -> one of its three bf16 terms hi / mid / lo
// (each the rounding of the running remainder: together all 24 significand bits), transposed to [O, ld_out] with
// zero padding, i.e. in the operand layout of the dW GEMM.  64 outputs x 64 tokens per workgroup through LDS; both
// sides move whole 128-byte (or longer) runs.  With sq_partials != null the workgroup also writes its sum of C^2.
__global__ void __launch_bounds__(256)
k_c_term_transposed(const float* __restrict__ C, int64_t T, int64_t O, int term, bf16_t* __restrict__ out, int64_t ld_out,
                    unsigned tiles_o, double* __restrict__ sq_partials) {
  __shared__ uint32_t tile[64][33];            // [output][token pair], pitch 33 words
  const int64_t o0 = (blockIdx.x % tiles_o) * 64LL, t0 = (blockIdx.x / tiles_o) * 64LL;
  const int og = threadIdx.x & 63, gq = threadIdx.x >> 6;
  const int64_t groups = (T + 3) / 4;
  float sq = 0.0f;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int g = gq + 4 * it;                 // token group within the tile
    const int64_t gg = t0 / 4 + g, o = o0 + og;
    float4 c = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (gg < groups && o < O) c = *reinterpret_cast<const float4*>(C + (gg * O + o) * 4);
    const float x[4] = {c.x, c.y, c.z, c.w};
    uint32_t b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sq += x[q] * x[q];
      const uint32_t h = f32_to_bf16(x[q]);
      const float r1 = x[q] - bf16_to_f32(h);
      const uint32_t m = f32_to_bf16(r1);
      const float r2 = r1 - bf16_to_f32(m);
      b[q] = term == 0 ? h : (term == 1 ? m : f32_to_bf16(r2));
    }
    tile[og][2 * g] = b[0] | (b[1] << 16);
    tile[og][2 * g + 1] = b[2] | (b[3] << 16);
  }
  __syncthreads();
  const int sub = threadIdx.x >> 3, ch = threadIdx.x & 7;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int row = p * 32 + sub;
    const int64_t o = o0 + row, t = t0 + ch * 8;
    if (o < O && t < ld_out)                   // ld_out is a multiple of 64: a chunk is inside or outside as a whole
      *reinterpret_cast<uint4*>(out + o * ld_out + t) =
          make_uint4(tile[row][ch * 4], tile[row][ch * 4 + 1], tile[row][ch * 4 + 2], tile[row][ch * 4 + 3]);
  }
  if (sq_partials) {
    __syncthreads();
    const double bs = block_sum(static_cast<double>(sq));
    if (threadIdx.x == 0) sq_partials[blockIdx.x] = bs;
  }
}

// H = (first ? 0 : H) + sum over the splits of the partial products
__global__ void __launch_bounds__(kEltThreads)
k_accumulate_partials(float* __restrict__ H, const float* __restrict__ partials, int n_split, int64_t stride, int64_t n4,
                      bool first) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n4) return;
  float4 a = first ? make_float4(0.0f, 0.0f, 0.0f, 0.0f) : reinterpret_cast<const float4*>(H)[i];
  for (int s = 0; s < n_split; ++s) {
    const float4 p = *reinterpret_cast<const float4*>(partials + s * stride + i * 4);
    a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
  }
  reinterpret_cast<float4*>(H)[i] = a;
}

// The token Gram matrix of a layer, from the split partial products: rounded to bf16 for the matrix cores, with the
// rounding error of each diagonal entry kept in float32
__global__ void __launch_bounds__(kEltThreads)
k_gram_finish(const float* __restrict__ partials, int n_split, int64_t K, bf16_t* __restrict__ gram,
              float* __restrict__ diag_lo) {
  const int64_t n4 = K * K / 4;
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n4) return;
  float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  for (int s = 0; s < n_split; ++s) {
    const float4 p = *reinterpret_cast<const float4*>(partials + s * K * K + i * 4);
    a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
  }
  const float v[4] = {a.x, a.y, a.z, a.w};
  uint32_t b[4];
  const int64_t row = (i * 4) / K, col = (i * 4) % K;   // K is a multiple of 4: the four share a row
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    b[j] = f32_to_bf16(v[j]);
    if (col + j == row) diag_lo[row] = v[j] - __uint_as_float(b[j] << 16);
  }
  *reinterpret_cast<uint2*>(gram + i * 4) = make_uint2(b[0] | (b[1] << 16), b[2] | (b[3] << 16));
}

// out[0] = sum of n doubles, in a fixed order (one workgroup)
__global__ void __launch_bounds__(kEltThreads) k_sum_doubles(const double* __restrict__ p, int64_t n, double* __restrict__ out) {
  double a = 0.0;
  for (int64_t i = threadIdx.x; i < n; i += kEltThreads) a += p[i];
  const double t = block_sum(a);
  if (threadIdx.x == 0) *out = t;
}

// float32 -> hi + mid + lo bf16 terms (24 significand bits covered by 3 x 8).
__global__ void __launch_bounds__(kEltThreads)
k_split_f32(const float* __restrict__ in, int64_t n, bf16_t* __restrict__ hi, bf16_t* __restrict__ mid,
            bf16_t* __restrict__ lo) {
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  if (i >= n) return;
  const float x = in[i];
  const uint32_t h = f32_to_bf16(x);
  const float r1 = x - bf16_to_f32(h);
  const uint32_t m = f32_to_bf16(r1);
  const float r2 = r1 - bf16_to_f32(m);
  hi[i] = static_cast<bf16_t>(h);
  mid[i] = static_cast<bf16_t>(m);
  lo[i] = static_cast<bf16_t>(f32_to_bf16(r2));
}

inline unsigned blocks_for(int64_t n8) { return static_cast<unsigned>((n8 + kEltThreads - 1) / kEltThreads); }

}  // namespace

hipError_t launch_amax(const void* W, bool w_bf16, int64_t n, float* partials, float* s_global,
                       hipStream_t st) {
  const int64_t n8 = n / 8;
  const int grid = static_cast<int>(std::min<int64_t>(kAmaxPartials, (n8 + kEltThreads - 1) / kEltThreads));
  if (w_bf16)
    hipLaunchKernelGGL(k_amax_partial<bf16_t>, dim3(grid), dim3(kEltThreads), 0, st,
                       static_cast<const bf16_t*>(W), n8, partials);
  else
    hipLaunchKernelGGL(k_amax_partial<float>, dim3(grid), dim3(kEltThreads), 0, st,
                       static_cast<const float*>(W), n8, partials);
  hipLaunchKernelGGL(k_amax_final, dim3(1), dim3(kEltThreads), 0, st, partials, grid, s_global);
  return hipGetLastError();
}

hipError_t launch_quant_rtn(const void* W, bool w_bf16, int64_t n, const float* s_global,
                            uint8_t* scales, uint8_t* codes, void* W_dq, bool dq_in_units, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  uint32_t* c32 = reinterpret_cast<uint32_t*>(codes);
#define FAAR_Q(WT, DQ) \
  hipLaunchKernelGGL((k_quant_rtn<WT, DQ>), g, b, 0, st, static_cast<const WT*>(W), n8, s_global, scales, c32, static_cast<WT*>(W_dq), dq_in_units)
  if (w_bf16) { if (W_dq) FAAR_Q(bf16_t, true); else FAAR_Q(bf16_t, false); }
  else        { if (W_dq) FAAR_Q(float, true);  else FAAR_Q(float, false); }
#undef FAAR_Q
  return hipGetLastError();
}

hipError_t launch_codec_batch(int op, const CodecBatch& B, bool w_bf16, bool sglobal_given, float* partials, hipStream_t st) {
  const dim3 b(kEltThreads);
  const dim3 g(B.first_block[B.n]);
  if (op == kBatchQuant) {
    if (!sglobal_given) {
      const dim3 ga(static_cast<unsigned>(B.n * kBatchAmaxBlocks));
      if (w_bf16) hipLaunchKernelGGL(k_batch_amax_partial<bf16_t>, ga, b, 0, st, B, partials);
      else hipLaunchKernelGGL(k_batch_amax_partial<float>, ga, b, 0, st, B, partials);
      hipLaunchKernelGGL(k_batch_amax_final, dim3(static_cast<unsigned>(B.n)), b, 0, st, B, partials);
    }
    if (w_bf16) hipLaunchKernelGGL(k_batch_quant_rtn<bf16_t>, g, b, 0, st, B);
    else hipLaunchKernelGGL(k_batch_quant_rtn<float>, g, b, 0, st, B);
  } else if (op == kBatchInitV) {
    if (w_bf16) hipLaunchKernelGGL(k_batch_init_v<bf16_t>, g, b, 0, st, B);
    else hipLaunchKernelGGL(k_batch_init_v<float>, g, b, 0, st, B);
  } else {
    if (w_bf16) hipLaunchKernelGGL(k_batch_harden_pack<bf16_t>, g, b, 0, st, B);
    else hipLaunchKernelGGL(k_batch_harden_pack<float>, g, b, 0, st, B);
  }
  return hipGetLastError();
}

hipError_t launch_init_v(const void* W, bool w_bf16, int64_t n, const float* s_global,
                         const uint8_t* scales, float* V, uint8_t* floor_codes, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  uint32_t* c32 = reinterpret_cast<uint32_t*>(floor_codes);
  if (w_bf16)
    hipLaunchKernelGGL(k_init_v<bf16_t>, g, b, 0, st, static_cast<const bf16_t*>(W), n8, s_global, scales, V, c32);
  else
    hipLaunchKernelGGL(k_init_v<float>, g, b, 0, st, static_cast<const float*>(W), n8, s_global, scales, V, c32);
  return hipGetLastError();
}

hipError_t launch_harden_pack(const void* W, bool w_bf16, int64_t n, const float* s_global,
                              const uint8_t* scales, const float* V, uint8_t* codes,
                              uint8_t* decisions, void* W_final, unsigned long long* flip_count,
                              hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  uint32_t* c32 = reinterpret_cast<uint32_t*>(codes);
  if (w_bf16)
    hipLaunchKernelGGL(k_harden_pack<bf16_t>, g, b, 0, st, static_cast<const bf16_t*>(W), n8, s_global, scales, V,
                       c32, decisions, static_cast<bf16_t*>(W_final), flip_count);
  else
    hipLaunchKernelGGL(k_harden_pack<float>, g, b, 0, st, static_cast<const float*>(W), n8, s_global, scales, V,
                       c32, decisions, static_cast<float*>(W_final), flip_count);
  return hipGetLastError();
}

hipError_t launch_softquant_fwd(const void* W, bool w_bf16, int64_t n, const float* s_global,
                                const uint8_t* scales, const float* V, float beta, bool delta,
                                bf16_t* Wt, bf16_t* Wq_full, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
#define FAAR_F(WT, D, F) \
  hipLaunchKernelGGL((k_softquant_fwd<WT, D, F>), g, b, 0, st, static_cast<const WT*>(W), n8, s_global, scales, V, beta, Wt, Wq_full)
#define FAAR_F2(WT) \
  do { if (delta) { if (Wq_full) FAAR_F(WT, true, true); else FAAR_F(WT, true, false); } \
       else       { if (Wq_full) FAAR_F(WT, false, true); else FAAR_F(WT, false, false); } } while (0)
  if (w_bf16) FAAR_F2(bf16_t); else FAAR_F2(float);
#undef FAAR_F2
#undef FAAR_F
  return hipGetLastError();
}

int64_t softquant_bwd_blocks(int64_t n) { return (n / 8 + kEltThreads - 1) / kEltThreads; }
// the fused step kernel walks its elements with a grid-stride loop so that the partial count stays small
int64_t step_bwd_blocks(int64_t n) { return std::min<int64_t>(softquant_bwd_blocks(n), kStepBwdMaxBlocks); }

hipError_t launch_softquant_bwd(const void* W, bool w_bf16, int64_t n, const float* s_global,
                                const uint8_t* scales, const float* V, float beta, const float* G,
                                int n_split, int64_t split_stride, float lambda_round, float* dV,
                                double* round_partials, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  const float lam_over_n = static_cast<float>(static_cast<double>(lambda_round) / static_cast<double>(n));
  if (w_bf16)
    hipLaunchKernelGGL(k_softquant_bwd<bf16_t>, g, b, 0, st, static_cast<const bf16_t*>(W), n8, s_global, scales, V,
                       beta, G, n_split, split_stride, lam_over_n, dV, round_partials);
  else
    hipLaunchKernelGGL(k_softquant_bwd<float>, g, b, 0, st, static_cast<const float*>(W), n8, s_global, scales, V,
                       beta, G, n_split, split_stride, lam_over_n, dV, round_partials);
  return hipGetLastError();
}

hipError_t launch_interval_codes(const void* W, bool w_bf16, int64_t n, const float* s_global,
                                 const uint8_t* scales, uint8_t* icodes, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  uint32_t* c32 = reinterpret_cast<uint32_t*>(icodes);
  if (w_bf16)
    hipLaunchKernelGGL(k_interval_codes<bf16_t>, g, b, 0, st, static_cast<const bf16_t*>(W), n8, s_global, scales, c32);
  else
    hipLaunchKernelGGL(k_interval_codes<float>, g, b, 0, st, static_cast<const float*>(W), n8, s_global, scales, c32);
  return hipGetLastError();
}

hipError_t launch_step_fwd(const void* W, bool w_bf16, int64_t n, const float* s_global, const uint8_t* scales,
                           const uint8_t* icodes, const float* V, float beta, bf16_t* delta, bf16_t* Wq_full,
                           double* round_partials, uint32_t* guard_slot, const float* H, double* cross_partials,
                           hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(static_cast<unsigned>(step_bwd_blocks(n))), b(kEltThreads);
  const uint32_t* c32 = reinterpret_cast<const uint32_t*>(icodes);
#define FAAR_SF(WT, F) \
  hipLaunchKernelGGL((k_step_fwd<WT, F>), g, b, 0, st, static_cast<const WT*>(W), n8, s_global, scales, c32, V, beta, delta, Wq_full, round_partials, guard_slot, H, cross_partials)
  if (w_bf16) { if (Wq_full) FAAR_SF(bf16_t, true); else FAAR_SF(bf16_t, false); }
  else        { if (Wq_full) FAAR_SF(float, true);  else FAAR_SF(float, false); }
#undef FAAR_SF
  return hipGetLastError();
}

hipError_t launch_step_bwd_adam(const StepBwdArgs& a, hipStream_t st) {
  const int64_t n8 = a.n / 8;
  const int64_t workers = step_bwd_blocks(a.n);
  const dim3 g(static_cast<unsigned>(workers + 1)), b(kEltThreads);  // the extra block finishes the losses
  const float lam_over_n = static_cast<float>(static_cast<double>(a.lambda_round) / static_cast<double>(a.n));
  const LossSums fin{a.mse_partials, a.n_mse, a.mse_scale, a.H ? a.cross_partials : nullptr, workers, a.c_norm2, a.x_scale,
                     a.round_partials, workers, 1.0 / static_cast<double>(a.n),
                     a.lambda_round, a.losses, a.losses + 1, a.losses + 2};
  const uint32_t* c32 = reinterpret_cast<const uint32_t*>(a.icodes);
#define FAAR_SB(WT, E, F) \
  hipLaunchKernelGGL((k_step_bwd_adam<WT, E, F>), g, b, 0, st, n8, a.s_global, a.scales, c32, a.V, a.m, a.u, a.beta, a.G, \
                     a.n_split, a.split_stride, a.x_scale, lam_over_n, a.opt, fin, static_cast<const WT*>(a.W), a.beta_next, \
                     a.delta_next, a.wq_full_next, a.round_next, a.guard_slot, a.next_tag, a.H, a.two_alpha_h, a.cross_next)
  const bool emit = a.beta_next > 0.0f;
  if (!emit) { if (a.w_bf16) FAAR_SB(bf16_t, false, false); else FAAR_SB(float, false, false); }
  else if (a.wq_full_next) { if (a.w_bf16) FAAR_SB(bf16_t, true, true); else FAAR_SB(float, true, true); }
  else { if (a.w_bf16) FAAR_SB(bf16_t, true, false); else FAAR_SB(float, true, false); }
#undef FAAR_SB
  return hipGetLastError();
}

hipError_t launch_finalize_losses(const double* mse_partials, int64_t n_mse, float mse_scale,
                                  const double* round_partials, int64_t n_round, double inv_n,
                                  float lambda_round, float* loss_mse, float* loss_round,
                                  float* loss_total, hipStream_t st) {
  const LossSums f{mse_partials, n_mse, mse_scale, nullptr, 0, nullptr, nullptr, round_partials, n_round, inv_n, lambda_round,
                   loss_mse, loss_round, loss_total};
  hipLaunchKernelGGL(k_finalize_losses, dim3(1), dim3(kEltThreads), 0, st, f);
  return hipGetLastError();
}

hipError_t launch_stochastic_v(const void* W, bool w_bf16, int64_t n, const float* s_global, const uint8_t* scales,
                               uint64_t seed, uint32_t sample, float* V, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  const uint32_t lo = static_cast<uint32_t>(seed), hi = static_cast<uint32_t>(seed >> 32);
  if (w_bf16)
    hipLaunchKernelGGL(k_stochastic_v<bf16_t>, g, b, 0, st, static_cast<const bf16_t*>(W), n8, s_global, scales, lo, hi, sample, V);
  else
    hipLaunchKernelGGL(k_stochastic_v<float>, g, b, 0, st, static_cast<const float*>(W), n8, s_global, scales, lo, hi, sample, V);
  return hipGetLastError();
}

hipError_t launch_hardened_delta(const void* W, bool w_bf16, int64_t n, const float* s_global, const uint8_t* scales,
                                 const float* V, bf16_t* delta, uint32_t* guard_slot, hipStream_t st) {
  const int64_t n8 = n / 8;
  const dim3 g(blocks_for(n8)), b(kEltThreads);
  if (w_bf16)
    hipLaunchKernelGGL(k_hardened_delta<bf16_t>, g, b, 0, st, static_cast<const bf16_t*>(W), n8, s_global, scales, V, delta, guard_slot);
  else
    hipLaunchKernelGGL(k_hardened_delta<float>, g, b, 0, st, static_cast<const float*>(W), n8, s_global, scales, V, delta, guard_slot);
  return hipGetLastError();
}

hipError_t launch_transpose_bf16(const bf16_t* in, int64_t rows, int64_t cols, bf16_t* out,
                                 int64_t ld_out, hipStream_t st) {
  if (ld_out % 64 != 0) return hipErrorInvalidValue;  // the kernel stores whole 8-element chunks
  // the grid covers rows up to ld_out so that the zero padding is written too; one flat grid dimension (limit
  // 2^31 - 1 workgroups) so that neither extent is bounded by the 65535 of the other dimensions
  const int64_t tiles_c = (cols + 63) / 64, tiles_r = (ld_out + 63) / 64;
  if (tiles_c * tiles_r > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_transpose_bf16, dim3(static_cast<unsigned>(tiles_c * tiles_r)), dim3(256), 0, st, in, rows, cols, out,
                     ld_out, static_cast<unsigned>(tiles_c));
  return hipGetLastError();
}

hipError_t launch_check_forward_tag(const ForwardGuard& guard, hipStream_t st) {
  hipLaunchKernelGGL(k_check_forward_tag, dim3(1), dim3(64), 0, st, guard);
  return hipGetLastError();
}

int64_t c_term_blocks(int64_t T, int64_t O) { return ((O + 63) / 64) * (padded_tokens(T) / 64); }

hipError_t launch_c_term_transposed(const float* C, int64_t T, int64_t O, int term, bf16_t* out, int64_t ld_out,
                                    double* sq_partials, hipStream_t st) {
  if (ld_out != padded_tokens(T)) return hipErrorInvalidValue;
  const int64_t tiles_o = (O + 63) / 64, blocks = c_term_blocks(T, O);
  if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_c_term_transposed, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, st, C, T, O, term, out, ld_out,
                     static_cast<unsigned>(tiles_o), sq_partials);
  return hipGetLastError();
}

hipError_t launch_accumulate_partials(float* H, const float* partials, int n_split, int64_t stride, int64_t n, bool first,
                                      hipStream_t st) {
  const int64_t n4 = n / 4;   // n = O * K is a multiple of 16
  hipLaunchKernelGGL(k_accumulate_partials, dim3(static_cast<unsigned>((n4 + kEltThreads - 1) / kEltThreads)), dim3(kEltThreads),
                     0, st, H, partials, n_split, stride, n4, first);
  return hipGetLastError();
}

hipError_t launch_gram_finish(const float* partials, int n_split, int64_t K, bf16_t* gram, float* diag_lo, hipStream_t st) {
  const int64_t n4 = K * K / 4;
  hipLaunchKernelGGL(k_gram_finish, dim3(static_cast<unsigned>((n4 + kEltThreads - 1) / kEltThreads)), dim3(kEltThreads), 0, st,
                     partials, n_split, K, gram, diag_lo);
  return hipGetLastError();
}

hipError_t launch_sum_doubles(const double* p, int64_t n, double* out, hipStream_t st) {
  hipLaunchKernelGGL(k_sum_doubles, dim3(1), dim3(kEltThreads), 0, st, p, n, out);
  return hipGetLastError();
}

hipError_t launch_split_f32(const float* in, int64_t n, bf16_t* hi, bf16_t* mid, bf16_t* lo,
                            hipStream_t st) {
  hipLaunchKernelGGL(k_split_f32, dim3(static_cast<unsigned>((n + kEltThreads - 1) / kEltThreads)),
                     dim3(kEltThreads), 0, st, in, n, hi, mid, lo);
  return hipGetLastError();
}

}  // namespace faar
