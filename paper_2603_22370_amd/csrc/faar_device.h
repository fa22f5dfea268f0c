// Device-side building blocks shared by the FAAR kernels: bf16 <-> float, FP8-E4M3 scale
// codec, E2M1 interval lookup (paper Sec. 3.1; Table 2 steps 2-4; Eq. 4).
// All "decision" arithmetic here is plain IEEE float32, one operation at a time; the library is
// compiled with -ffp-contract=off and without fast-math so that results are bit-reproducible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace faar {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// two floats -> two bf16 (the first in the low half), round to nearest even, with the hardware's pair conversion
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2_t f = {a, b};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&h);
}

// 16 bytes that are read once and not again by this kernel: a load with the nontemporal hint, which lets the
// caches drop the line early (measured on a plain copy of 1 GiB: 6.5 instead of 6.3 TB/s)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Eight consecutive weights as float, from bf16 or float storage (16-byte aligned).
template <typename WT> struct W8;
template <> struct W8<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&w)[8]) {
    const uint4 q = *reinterpret_cast<const uint4*>(p);
    const uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[2 * i] = __uint_as_float(r[i] << 16);
      w[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void load_stream(const bf16_t* p, float (&w)[8]) {
    const uint4 q = load16_stream(p);
    const uint32_t r[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[2 * i] = __uint_as_float(r[i] << 16);
      w[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
  // float32 values -> rounded to bf16 -> stored
  static __device__ __forceinline__ void store(bf16_t* p, const float (&w)[8]) {
    uint32_t r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16(w[2 * i]) | (f32_to_bf16(w[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(r[0], r[1], r[2], r[3]);
  }
};
template <> struct W8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&w)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
    w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
  }
  static __device__ __forceinline__ void load_stream(const float* p, float (&w)[8]) {
    const uint4 a = load16_stream(p), b = load16_stream(p + 4);
    w[0] = __uint_as_float(a.x); w[1] = __uint_as_float(a.y); w[2] = __uint_as_float(a.z); w[3] = __uint_as_float(a.w);
    w[4] = __uint_as_float(b.x); w[5] = __uint_as_float(b.y); w[6] = __uint_as_float(b.z); w[7] = __uint_as_float(b.w);
  }
  static __device__ __forceinline__ void store(float* p, const float (&w)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(w[0], w[1], w[2], w[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(w[4], w[5], w[6], w[7]);
  }
};

__device__ __forceinline__ void load8(const float* p, float (&v)[8]) { W8<float>::load(p, v); }
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) { W8<float>::store(p, v); }

// FP8 E4M3 (1-4-3, bias 7, no inf) value of a non-negative byte 0x00..0x7E.
__device__ __forceinline__ float e4m3_value(uint32_t b) {
  const uint32_t e = b >> 3, m = b & 7u;
  return e == 0 ? static_cast<float>(m) * 0x1p-9f : __uint_as_float(((e + 120u) << 23) | (m << 20));
}

// Non-negative finite float -> nearest E4M3 byte, ties to even, saturating at 448 (0x7E).
__device__ __forceinline__ uint32_t e4m3_encode_sat(float t) {
  if (!(t < 448.0f)) return 0x7Eu;
  if (t < 0x1p-6f) return static_cast<uint32_t>(rintf(t * 512.0f));  // subnormal grid: m * 2^-9
  uint32_t u = __float_as_uint(t);
  u += 0x7FFFFu + ((u >> 20) & 1u);  // round mantissa to 3 bits, nearest even (carry may bump the exponent)
  return (u >> 20) - (120u << 3);
}

// Block scale byte from the block's largest magnitude: E4M3((a_b / 6) / s_global).
__device__ __forceinline__ uint32_t block_scale_byte(float a_b, float s_global) {
  return e4m3_encode_sat((a_b / 6.0f) / s_global);
}

// s = E4M3_value(byte) * s_global, one float32 product.
__device__ __forceinline__ float effective_scale(uint32_t byte, float s_global) {
  return e4m3_value(byte) * s_global;
}

// What Eq. 2 needs for one weight.
struct Interval {
  int k_lo;      // 0..6
  float lo;      // N[k_lo]
  float width;   // N[k_lo+1] - N[k_lo]
  float v_init;  // Eq. 4, clamped to [0, 1]
};

// Number of nodes among 0.5, 1, 1.5, 2, 3, 4 that are <= wt, for finite wt >= 0.  From 1 upwards the
// nodes are exactly the floats with one significand bit, so exponent and leading significand bit index them:
// (bits >> 22) is 254 at 1.0, 255 at 1.5, 256 at 2.0 ... ; 252 and 253 cover [0.5, 1).
__device__ __forceinline__ int interval_index(float wt) {
  const int d = (static_cast<int>(__float_as_uint(wt)) >> 22) - 252;  // arithmetic shift: a negative input gives 0
  return d < 0 ? 0 : min(max(d, 1), 6);
}
// N[k] for k in 0..6
__device__ __forceinline__ float interval_lo(int k) {
  return k < 2 ? 0.5f * static_cast<float>(k)
               : __uint_as_float(((126u + (static_cast<uint32_t>(k) >> 1)) << 23) | ((static_cast<uint32_t>(k) & 1u) << 22));
}

// Magnitude code 0..7 of the node nearest to wt (finite, >= 0), exact midpoints going up: the same decision as
// "k_lo + (wt >= midpoint of interval k_lo)", taken in one step.  From 1 upwards an E2M1 code is the float's exponent
// and leading significand bit, so adding half an E2M1 ulp to the bit pattern (bit 21) and truncating rounds the
// magnitude half-up; below 1 the nodes are 0, 0.5 and 1 with midpoints 0.25 and 0.75.  A zero weight gives code 0.
__device__ __forceinline__ uint32_t nearest_magnitude_code(float wt) {
  const int hi = static_cast<int>((__float_as_uint(wt) + 0x200000u) >> 22) - 252;
  const int lo = static_cast<int>(wt >= 0.25f) + static_cast<int>(wt >= 0.75f);
  return static_cast<uint32_t>(wt < 1.0f ? lo : min(hi, 7));
}

// Midpoint of interval k: round-to-nearest goes up exactly when w~ >= midpoint (w~ - lo is exact and
// the widths are powers of two, so this is the same decision as v_init >= 0.5).
__device__ __forceinline__ float interval_mid(int k) {
  return k < 2 ? 0.25f + 0.5f * static_cast<float>(k) : __uint_as_float(__float_as_uint(interval_lo(k)) | (1u << 21));
}
// w~ = |w| / s, one correctly rounded division; 0 when the block scale is 0
__device__ __forceinline__ float normalised(float w, float s) { return (s == 0.0f) ? 0.0f : fabsf(w) / s; }

// |w| / s for several weights of one block, for kernels that need w~ only to DECIDE (interval index,
// round-to-nearest direction).  With y = 1/s correctly rounded (hardware estimate plus one Newton step; checked
// against the IEEE quotient for every float32 significand), q0 = a*y, r = fma(-q0, s, a) is the exact remainder
// and fma(r, y, q0) is the correctly rounded quotient a/s (Markstein's theorem) as long as nothing underflows:
// guaranteed here for quotients >= 2^-40 because s is kept within [2^-60, 2^60] and the numerators below 2^60.
// A quotient below 2^-40 may come out inexact but stays far below the first threshold (0.25), so every decision
// is still that of the IEEE division.  Outside those ranges the plain division is used.
struct BlockDivider {
  float s, y;
  bool fast;
  __device__ __forceinline__ BlockDivider(float s_, float amax) : s(s_) {
    fast = (s_ >= 0x1p-60f) && (s_ <= 0x1p60f) && (amax <= 0x1p60f);
    const float y0 = __builtin_amdgcn_rcpf(s_);
    y = __builtin_fmaf(__builtin_fmaf(-s_, y0, 1.0f), y0, y0);
  }
  template <bool kFast> __device__ __forceinline__ float quotient(float a) const {
    if (kFast) {
      const float q0 = a * y;
      return __builtin_fmaf(__builtin_fmaf(-q0, s, a), y, q0);
    }
    return (s == 0.0f) ? 0.0f : a / s;
  }
};

// Table 2 steps 2-4 for one weight: w~ = |w| / s (0 when s == 0), interval, relative position.
// (w~ - lo) / width is evaluated as a product with 1 / width: the widths are powers of two, so both are
// the correctly rounded value of the same real number.
__device__ __forceinline__ Interval find_interval(float w, float s) {
  const float wt = normalised(w, s);
  Interval r;
  r.k_lo = interval_index(wt);
  r.lo = interval_lo(r.k_lo);
  r.width = r.k_lo <= 3 ? 0.5f : (r.k_lo == 6 ? 2.0f : 1.0f);
  const float inv_width = r.k_lo <= 3 ? 2.0f : (r.k_lo == 6 ? 0.5f : 1.0f);
  const float v = (wt - r.lo) * inv_width;
  r.v_init = fminf(fmaxf(v, 0.0f), 1.0f);
  return r;
}

// Magnitude value of E2M1 code 0..7.
__device__ __forceinline__ float e2m1_magnitude(uint32_t c) {
  return c <= 4u ? 0.5f * static_cast<float>(c) : (c == 5u ? 3.0f : (c == 6u ? 4.0f : 6.0f));
}

// nibble = signbit(w) << 3 | (w == 0 ? 0 : k_lo + up)
__device__ __forceinline__ uint32_t nibble(float w, int k_lo, int up) {
  const uint32_t mag = (w == 0.0f) ? 0u : static_cast<uint32_t>(k_lo + up);
  return ((__float_as_uint(w) >> 31) << 3) | mag;
}

// Dequantised value of a nibble: sign * ((N[code] * E4M3_value(byte)) * s_global).
__device__ __forceinline__ float dequant(uint32_t nib, float sg_value, float s_global) {
  const float mag = (e2m1_magnitude(nib & 7u) * sg_value) * s_global;
  return (nib & 8u) ? -mag : mag;
}

// sign(w) in {-1, 0, +1}
__device__ __forceinline__ float sign_of(float w) { return w > 0.0f ? 1.0f : (w < 0.0f ? -1.0f : 0.0f); }

}  // namespace faar
