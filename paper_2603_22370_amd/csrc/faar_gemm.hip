// bf16 MFMA GEMMs of the FAAR layer step for gfx950 (paper Table 2 steps 8-10 and the chain rule
// of Eq. 5): the residual GEMM  X_q (W_q - W)^T - C  with its loss / dY epilogue, the weight
// gradient  dY^T X_q  and the optional input gradient  dY W_q.
//
// Every product is computed as an "NT" GEMM  acc[m][n] = sum_k A[m][k] B[n][k]  with both operands
// row-major and the contraction index contiguous; operands that the mathematics wants transposed
// (X_q^T, dY^T, W_q^T) are produced in that layout by the kernel that writes them, so one tuned
// main loop serves all of them.  The one exception is the weight gradient of LLM-sized layers, whose
// contraction index is the token -- the row index of everything the layers produce: k_gemm_dma64 has a
// token-major form (acc[m][n] = sum_t A[t][m] B[t][n], LDS transposing reads) that takes dY and X_q as
// they are.
//
// Three main loops:
//  * k_gemm_dma64 (contraction length a multiple of 64 -- every GEMM of an LLM-shaped layer): 256x256 or
//    256x128 output tile per 512-thread workgroup (8 wavefronts, 2 per SIMD), BK = 64 slices copied
//    global -> LDS by global_load_lds_dwordx4 (no VGPR staging) into two or three stages, 128-byte LDS rows,
//    v_mfma_f32_16x16x32_bf16, one workgroup barrier per slice.  Described at the kernel.
//  * k_gemm_dma (contraction length a multiple of 32, and all 128x128 tiles): BK = 32 slices in a 4-stage
//    ring; LDS rows are 64 B, un-padded, with the 16-byte chunk index XOR-swizzled by (row / 4) % 4 so that the
//    fragment reads of 16 consecutive rows hit 16 distinct bank groups (measured: zero LDS bank conflicts);
//    fragments are prefetched one MFMA phase ahead, also across the slice boundary, and the ds_reads / DMA
//    issues are interleaved one by one between the v_mfma_f32_32x32x16_bf16 instructions.
//    In both, workgroups are dealt to the 8 XCDs in contiguous chunks of a grouped tile order so that each
//    XCD's L2 sees a compact sub-grid.
//  * k_gemm_nt (generic fallback for ragged contraction lengths): 128x128 tile, register-staged,
//    padded LDS, bounds-checked loads.
#include <algorithm>

#include "faar_internal.h"

namespace faar {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;            // contraction slice per stage
constexpr int LDS_LD = BK + 8;    // padded LDS row, elements (144 B)
constexpr int GEMM_THREADS = 256;

template <int BM_, int BN_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_;
  static constexpr int WM = BM / 2, WN = BN / 2;   // 2 x 2 wavefronts
  static constexpr int TM = WM / 32, TN = WN / 32; // 32x32 MFMA tiles per wavefront
  static constexpr int A_CHUNKS = BM * (BK / 8) / GEMM_THREADS;  // 16-byte chunks per thread
  static constexpr int B_CHUNKS = BN * (BK / 8) / GEMM_THREADS;
  static constexpr int STAGE = (BM + BN) * LDS_LD;               // elements per LDS stage
};

// Output coordinates held by one lane for accumulator register v of a 32x32 tile:
// column = lane % 32, row = 8 * (v / 4) + 4 * (lane / 32) + v % 4.
struct Out {
  int64_t M, N;
};

template <class T, class Epi>
__global__ void __launch_bounds__(GEMM_THREADS)
k_gemm_nt(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, GemmDims d, int tiles_m, int tiles_n,
          int64_t k_per_split, Epi epi) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * T::STAGE];
  epi.once();
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * T::WM, wn = (wave & 1) * T::WN;

  int pid = blockIdx.x;
  const int split = pid / (tiles_m * tiles_n);
  pid -= split * tiles_m * tiles_n;
  const int tm = pid % tiles_m, tn = pid / tiles_m;   // consecutive workgroups share the B panel
  const int64_t m0 = (int64_t)tm * T::BM, n0 = (int64_t)tn * T::BN;
  const int64_t k_begin = split * k_per_split;
  const int64_t k_end = k_begin + k_per_split < d.Kd ? k_begin + k_per_split : d.Kd;
  const int nk = static_cast<int>((k_end - k_begin + BK - 1) / BK);

  uint4 ra[T::A_CHUNKS], rb[T::B_CHUNKS];
  auto g_load = [&](int kt) {
    const int64_t k0 = k_begin + (int64_t)kt * BK;
#pragma unroll
    for (int j = 0; j < T::A_CHUNKS; ++j) {
      const int c = tid + j * GEMM_THREADS, row = c >> 3, kc = (c & 7) * 8;
      const int64_t m = m0 + row, k = k0 + kc;
      ra[j] = (m < d.M && k < k_end) ? *reinterpret_cast<const uint4*>(A + m * d.lda + k) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < T::B_CHUNKS; ++j) {
      const int c = tid + j * GEMM_THREADS, row = c >> 3, kc = (c & 7) * 8;
      const int64_t n = n0 + row, k = k0 + kc;
      rb[j] = (n < d.N && k < k_end) ? *reinterpret_cast<const uint4*>(B + n * d.ldb + k) : make_uint4(0, 0, 0, 0);
    }
  };
  auto s_store = [&](int stage) {
    bf16_t* sa = lds + stage * T::STAGE;
    bf16_t* sb = sa + T::BM * LDS_LD;
#pragma unroll
    for (int j = 0; j < T::A_CHUNKS; ++j) {
      const int c = tid + j * GEMM_THREADS, row = c >> 3, kc = (c & 7) * 8;
      *reinterpret_cast<uint4*>(sa + row * LDS_LD + kc) = ra[j];
    }
#pragma unroll
    for (int j = 0; j < T::B_CHUNKS; ++j) {
      const int c = tid + j * GEMM_THREADS, row = c >> 3, kc = (c & 7) * 8;
      *reinterpret_cast<uint4*>(sb + row * LDS_LD + kc) = rb[j];
    }
  };

  f32x16 acc[T::TM][T::TN];
#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  if (nk > 0) {
    g_load(0);
    s_store(0);
  }
  __syncthreads();
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) g_load(kt + 1);
    const bf16_t* sa = lds + (kt & 1) * T::STAGE;
    const bf16_t* sb = sa + T::BM * LDS_LD;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 fa[T::TM], fb[T::TN];
#pragma unroll
      for (int i = 0; i < T::TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(sa + (wm + i * 32 + frag_row) * LDS_LD + kk + frag_k);
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(sb + (wn + j * 32 + frag_row) * LDS_LD + kk + frag_k);
#pragma unroll
      for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) s_store((kt + 1) & 1);
    __syncthreads();
  }

  // epilogue: hand every group of 4 consecutive rows (one column) to the functor
  epi.begin();
  const int col = lane & 31, hi = lane >> 5;
#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j) {
      const int64_t n = n0 + wn + j * 32 + col;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int64_t m = m0 + wm + i * 32 + 8 * g + 4 * hi;
        const float r[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        epi.rows4(r, m, n, split, d);
      }
    }
  epi.finish(blockIdx.x);
}

// ---- epilogues -----------------------------------------------------------------------------

// fixed-order sum of one float per lane over the workgroup's wavefronts (4 or 8), as a double, to partials[item]
__device__ __forceinline__ void finish_sum(float sum, double* partials, int item) {
  __shared__ double s[8];
  double a = static_cast<double>(sum);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    const int nw = blockDim.x >> 6;
    for (int i = 0; i < nw; ++i) t += s[i];
    partials[item] = t;
  }
}

// kWithC:  R = x_scale * acc - C;  sum R^2;  dYt[n][m] = bf16(two_alpha R) (zero-padded to ldt); optional dY[m][n].
// !kWithC: the V-dependent part alone, for steps that carry the constant part of the gradient separately
//          (G = dY^T X_q = (2 alpha x_scale acc)^T X_q - 2 alpha C^T X_q):  A = x_scale * acc;  sum A^2;
//          dYt[n][m] = bf16(two_alpha A).  Nothing is read in the epilogue.
template <bool kWithC>
struct EpiResidualT {
  static constexpr bool kRowStaged = false;
  static constexpr bool kTransposedOut = true;  // the fast kernel stages dYt through LDS for full-line stores
  static constexpr int kMode = 0;               // 0: the whole main loop (1, 2: measurement variants, see EpiProbe)
  // The GEMM that follows (dW = dY^T X_q) reads X_q^T, which the pass that updates V has meanwhile pushed out of the
  // last-level cache; with either operand coming from HBM that GEMM runs ~25 % slower.  The BK = 64 main loop of this
  // kernel therefore reads `warm` (X_q^T, warm_chunks KB) on the side, 1 KB per wavefront and slice, and keeps nothing.
  static constexpr bool kWarm = true;
  const float* C;
  const float* x_scale;  // device scalar multiplying the A operand (activations stored in units of it); null = 1
  float xs;
  __device__ __forceinline__ void begin() { xs = x_scale ? *x_scale : 1.0f; }
  // first thing workgroup 0 does: is the forward in the workspace the one this step's caller says it is?
  ForwardGuard guard;
  __device__ __forceinline__ void once() {
    if (guard.slot && blockIdx.x == 0 && threadIdx.x == 0) {
      bool ok = true;
      for (int i = 0; i < kTagWords; ++i) ok = ok && guard.slot[i] == guard.expect.w[i];
      for (int i = 0; i < kTagWords; ++i) guard.slot[i] = 0u;   // consumed: a replay of this step must not match
      guard.slot[kTagWords] = ok ? 1u : 0u;
    }
  }
  float two_alpha;
  bf16_t* dYt;
  int64_t ldt;
  bf16_t* dY;
  double* partials;
  float sum;
  const void* warm;      // null: nothing to read on the side
  int64_t warm_chunks;   // its size in KB (whole 1 KB chunks)
  // C of rows m..m+3 (m a multiple of 4) of column n: one 16-byte load from the row-group-interleaved layout
  // [ceil(M/4)][N][4] (zero outside the matrix); kept separate from value4 so that a whole slab's loads can be
  // issued before the first dependent store
  __device__ __forceinline__ float4 load4(int64_t m, int64_t n, const GemmDims& d) const {
    if (kWithC && n < d.N && m < d.M) return *reinterpret_cast<const float4*>(C + ((m >> 2) * d.N + n) * 4);
    return make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  }
  // four consecutive rows m..m+3 of column n -> four bf16 dY values (zero outside the matrix)
  __device__ __forceinline__ uint2 value4(const float (&acc)[4], const float4& c4, int64_t m, int64_t n, const GemmDims& d) {
    uint32_t b[4] = {0u, 0u, 0u, 0u};
    const float c[4] = {c4.x, c4.y, c4.z, c4.w};
    if (n < d.N) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (m + q < d.M) {
          const float r = kWithC ? xs * acc[q] - c[q] : xs * acc[q];
          sum += r * r;
          b[q] = f32_to_bf16(two_alpha * r);
          if (kWithC && dY) dY[(m + q) * d.N + n] = static_cast<bf16_t>(b[q]);
        }
      }
    }
    return make_uint2(b[0] | (b[1] << 16), b[2] | (b[3] << 16));
  }
  __device__ __forceinline__ void store_chunk(const uint4& v, int64_t m, int64_t n, const GemmDims& d) {
    if (n < d.N && m < ldt) *reinterpret_cast<uint4*>(dYt + n * ldt + m) = v;  // m, ldt multiples of 8
  }
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N || m >= ldt) return;
    *reinterpret_cast<uint2*>(dYt + n * ldt + m) = value4(acc, load4(m, n, d), m, n, d);
  }
  // fixed-order sum over the workgroup's wavefronts (4 or 8)
  __device__ __forceinline__ void finish(int item) { finish_sum(sum, partials, item); }
};
typedef EpiResidualT<true> EpiResidual;
typedef EpiResidualT<false> EpiPerturbation;

// The V-dependent part of the residual with dY stored TOKEN-major, for the token-major dW GEMM that follows:
// A = x_scale * acc;  sum A^2 per work item;  dY[m][n] = bf16(two_alpha * A)  ([M, N] row-major, N a multiple of 8).
struct EpiPerturbationRows {
  static constexpr bool kTransposedOut = false;
  static constexpr bool kRowStaged = true;
  static constexpr bool kWarm = false;
  static constexpr int kMode = 0;
  const float* x_scale;
  float xs;
  ForwardGuard guard;
  float two_alpha;
  bf16_t* dY;
  double* partials;
  float sum;
  __device__ __forceinline__ void once() {
    if (guard.slot && blockIdx.x == 0 && threadIdx.x == 0) {
      bool ok = true;
      for (int i = 0; i < kTagWords; ++i) ok = ok && guard.slot[i] == guard.expect.w[i];
      for (int i = 0; i < kTagWords; ++i) guard.slot[i] = 0u;
      guard.slot[kTagWords] = ok ? 1u : 0u;
    }
  }
  __device__ __forceinline__ void begin() { xs = x_scale ? *x_scale : 1.0f; }
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) {
        const float r = xs * acc[q];
        sum += r * r;
        dY[(m + q) * d.N + n] = static_cast<bf16_t>(f32_to_bf16(two_alpha * r));
      }
  }
  __device__ __forceinline__ void run8(const float (&acc)[8], int64_t m, int64_t n, int, const GemmDims& d) {
    if (m >= d.M || n >= d.N) return;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float r0 = xs * acc[2 * j], r1 = xs * acc[2 * j + 1];
      sum += r0 * r0;
      sum += r1 * r1;
      w[j] = f32_to_bf16(two_alpha * r0) | (f32_to_bf16(two_alpha * r1) << 16);
    }
    *reinterpret_cast<uint4*>(dY + m * d.N + n) = make_uint4(w[0], w[1], w[2], w[3]);
  }
  __device__ __forceinline__ void finish(int item) { finish_sum(sum, partials, item); }
};

// sum of (x_scale * acc)^2 per work item and nothing else: the loss of a step whose dY comes from upstream
struct EpiSumSq {
  static constexpr bool kRowStaged = false;
  static constexpr bool kWarm = false;
  static constexpr bool kTransposedOut = false;
  static constexpr int kMode = 0;
  const float* x_scale;
  float xs;
  ForwardGuard guard;
  double* partials;
  float sum;
  __device__ __forceinline__ void once() {
    if (guard.slot && blockIdx.x == 0 && threadIdx.x == 0) {
      bool ok = true;
      for (int i = 0; i < kTagWords; ++i) ok = ok && guard.slot[i] == guard.expect.w[i];
      for (int i = 0; i < kTagWords; ++i) guard.slot[i] = 0u;
      guard.slot[kTagWords] = ok ? 1u : 0u;
    }
  }
  __device__ __forceinline__ void begin() { xs = x_scale ? *x_scale : 1.0f; }
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) {
        const float r = xs * acc[q];
        sum += r * r;
      }
  }
  __device__ __forceinline__ void finish(int item) { finish_sum(sum, partials, item); }
};

// out[split][m][n] = acc
struct EpiF32 {
  static constexpr bool kWarm = false;
  static constexpr bool kRowStaged = true;   // the BK = 64 kernel hands it runs of 8 columns of a row (run8)
  static constexpr bool kTransposedOut = false;
  static constexpr int kMode = 0;
  float* out;
  __device__ __forceinline__ void once() {}
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int split, const GemmDims& d) {
    if (n >= d.N) return;
    float* o = out + (int64_t)split * d.M * d.N;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) o[(m + q) * d.N + n] = acc[q];
  }
  // columns n..n+7 of row m (n and N multiples of 8)
  __device__ __forceinline__ void run8(const float (&r)[8], int64_t m, int64_t n, int split, const GemmDims& d) {
    if (m >= d.M || n >= d.N) return;
    float4* o = reinterpret_cast<float4*>(out + (int64_t)split * d.M * d.N + m * d.N + n);
    o[0] = make_float4(r[0], r[1], r[2], r[3]);
    o[1] = make_float4(r[4], r[5], r[6], r[7]);
  }
  __device__ __forceinline__ void finish(int) {}
};

// C_out(m, n) = (first ? Y[m][n] : C_out(m, n)) - x_scale * acc, with C_out in the row-group-interleaved layout
// [ceil(M/4)][N][4]: element (m, n) at ((m / 4) * N + n) * 4 + m % 4, so that the four consecutive rows a lane
// holds of one column are one 16-byte access and the 16 or 32 lanes of a row group touch contiguous memory.
// Rows M..4*ceil(M/4)-1 are written as zero.
template <bool kYbf16>
struct EpiSub {
  static constexpr bool kRowStaged = false;
  static constexpr bool kWarm = false;
  static constexpr bool kTransposedOut = false;
  static constexpr int kMode = 0;
  const void* Y;
  bool first;
  float* C_out;
  const float* x_scale;  // as in EpiResidual
  float xs;
  __device__ __forceinline__ void once() {}
  __device__ __forceinline__ void begin() { xs = x_scale ? *x_scale : 1.0f; }
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N || m >= d.M) return;  // m is a multiple of 4
    float4* p = reinterpret_cast<float4*>(C_out + ((m >> 2) * d.N + n) * 4);
    float y[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!first) {
      const float4 c = *p;
      y[0] = c.x; y[1] = c.y; y[2] = c.z; y[3] = c.w;
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (m + q < d.M) {
          const int64_t idx = (m + q) * d.N + n;
          y[q] = kYbf16 ? bf16_to_f32(static_cast<const bf16_t*>(Y)[idx]) : static_cast<const float*>(Y)[idx];
        }
    }
    float o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = (m + q < d.M) ? y[q] - xs * acc[q] : 0.0f;
    *p = make_float4(o[0], o[1], o[2], o[3]);
  }
  __device__ __forceinline__ void finish(int) {}
};

// out[m][n] = bf16(scale * acc)
struct EpiBf16 {
  static constexpr bool kRowStaged = true;    // the DMA kernels hand it runs of 8 columns of a row (run8)
  static constexpr bool kWarm = false;
  static constexpr bool kTransposedOut = false;
  static constexpr int kMode = 0;
  bf16_t* out;
  const float* scale;   // device scalar multiplying the product (activations stored in units of it); null = 1
  float sc;
  __device__ __forceinline__ void once() {}
  __device__ __forceinline__ void begin() { sc = scale ? *scale : 1.0f; }
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) out[(m + q) * d.N + n] = static_cast<bf16_t>(f32_to_bf16(sc * acc[q]));
  }
  // columns n..n+7 of row m (n a multiple of 8): one 16-byte store when the row pitch allows it
  __device__ __forceinline__ void run8(const float (&r)[8], int64_t m, int64_t n, int, const GemmDims& d) {
    if (m >= d.M || n >= d.N) return;
    bf16_t* o = out + m * d.N + n;
    if (n + 8 <= d.N && (d.N & 7) == 0) {
      uint32_t w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = f32_to_bf16(sc * r[2 * j]) | (f32_to_bf16(sc * r[2 * j + 1]) << 16);
      *reinterpret_cast<uint4*>(o) = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
      for (int j = 0; j < 8 && n + j < d.N; ++j) o[j] = static_cast<bf16_t>(f32_to_bf16(sc * r[j]));
    }
  }
  __device__ __forceinline__ void finish(int) {}
};

// Gram-matrix form of the step: A = W_q - W (M x N = O x K outputs, the contraction runs over K as well), B = bf16(Xq^T Xq).
// t = acc + (split 0: A[m][n] * diag_lo[n]) restores what the rounding took from B's diagonal;
// out[split][m][n] = two_alpha * x_scale * t  (what the dW GEMM of the token form leaves for the pass that updates V);
// per work item the partial sum of x_scale^2 * t * A[m][n], which over all items is ||x_scale Xq (W_q - W)^T||^2.
struct EpiGram {
  static constexpr bool kWarm = false;
  static constexpr bool kRowStaged = true;
  static constexpr bool kTransposedOut = false;
  static constexpr int kMode = 0;
  const bf16_t* delta;     // the A operand, [M, N] row-major
  const float* diag_lo;    // [N]
  const float* x_scale;
  float xs;
  ForwardGuard guard;
  float two_alpha;
  float* out;
  double* partials;
  float sum;
  __device__ __forceinline__ void once() {
    if (guard.slot && blockIdx.x == 0 && threadIdx.x == 0) {
      bool ok = true;
      for (int i = 0; i < kTagWords; ++i) ok = ok && guard.slot[i] == guard.expect.w[i];
      for (int i = 0; i < kTagWords; ++i) guard.slot[i] = 0u;
      guard.slot[kTagWords] = ok ? 1u : 0u;
    }
  }
  __device__ __forceinline__ void begin() { xs = x_scale ? *x_scale : 1.0f; }
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int split, const GemmDims& d) {
    if (n >= d.N) return;
    float* o = out + (int64_t)split * d.M * d.N;
    const float lo = split == 0 ? diag_lo[n] : 0.0f;
    const float k_out = two_alpha * xs, k_sum = xs * xs;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) {
        const float a = bf16_to_f32(delta[(m + q) * d.N + n]);
        const float t = acc[q] + a * lo;
        o[(m + q) * d.N + n] = k_out * t;
        sum += k_sum * (t * a);
      }
  }
  // columns n..n+7 of row m (n and N multiples of 8): one 16-byte load of delta, two of diag_lo, two 16-byte stores
  __device__ __forceinline__ void run8(const float (&r)[8], int64_t m, int64_t n, int split, const GemmDims& d) {
    if (m >= d.M || n >= d.N) return;
    const uint4 dv = *reinterpret_cast<const uint4*>(delta + m * d.N + n);
    const uint32_t dw[4] = {dv.x, dv.y, dv.z, dv.w};
    float lo[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    if (split == 0) {
      const float4 l0 = *reinterpret_cast<const float4*>(diag_lo + n), l1 = *reinterpret_cast<const float4*>(diag_lo + n + 4);
      lo[0] = l0.x; lo[1] = l0.y; lo[2] = l0.z; lo[3] = l0.w; lo[4] = l1.x; lo[5] = l1.y; lo[6] = l1.z; lo[7] = l1.w;
    }
    const float k_out = two_alpha * xs, k_sum = xs * xs;
    float o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float a = __uint_as_float((j & 1) ? (dw[j >> 1] & 0xFFFF0000u) : (dw[j >> 1] << 16));
      const float t = r[j] + a * lo[j];
      o[j] = k_out * t;
      sum += k_sum * (t * a);
    }
    float4* op = reinterpret_cast<float4*>(out + (int64_t)split * d.M * d.N + m * d.N + n);
    op[0] = make_float4(o[0], o[1], o[2], o[3]);
    op[1] = make_float4(o[4], o[5], o[6], o[7]);
  }
  __device__ __forceinline__ void finish(int item) { finish_sum(sum, partials, item); }
};

// Measurement epilogue (faar_gemm_probe): no output; every work item reports how many shader-clock cycles and how
// many ticks of the constant 100 MHz counter it took, so that the clock the compute units ran at can be read off.
// kMode selects what the main loop of k_gemm_dma64 keeps: 0 everything, 1 only the matrix instructions and their
// LDS reads (the stages are filled once and never refilled), 2 only the global->LDS copies.
template <int MODE>
struct EpiProbe {
  static constexpr bool kTransposedOut = false;
  static constexpr bool kWarm = false;
  static constexpr bool kRowStaged = false;
  static constexpr int kMode = MODE;
  unsigned long long* clocks;   // [items][2]
  float* sink;
  long long t0, w0;
  float sum;
  __device__ __forceinline__ void once() { t0 = clock64(); w0 = wall_clock64(); sum = 0.0f; }
  __device__ __forceinline__ void begin() {}
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t, int64_t, int, const GemmDims&) {
    sum += (acc[0] + acc[1]) + (acc[2] + acc[3]);
  }
  __device__ __forceinline__ void finish(int item) {
    if (sum == 1.2345e-30f) *sink = sum;   // keeps the accumulators alive; never true for real operands
    if (threadIdx.x == 0) {
      clocks[2 * item] = static_cast<unsigned long long>(clock64() - t0);
      clocks[2 * item + 1] = static_cast<unsigned long long>(wall_clock64() - w0);
    }
  }
};

// ---- fast path: direct-to-LDS ring, swizzled LDS, interleaved schedule ------------------------------

constexpr int DBK = 32;   // contraction slice per stage
constexpr int DNS = 4;    // ring stages

template <int BM_, int BN_, int WGM_, int WGN_>
struct DmaCfg {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_;
  static constexpr int NW = WGM * WGN, THREADS = 64 * NW;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int CPR = DBK / 8;            // 16-byte chunks per LDS row (4)
  static constexpr int RPI = 64 / CPR;           // rows written by one wave-wide DMA instruction (16)
  static constexpr int RB = 16 / CPR;            // rows per 256-byte bank cycle (4)
  static constexpr int STAGE = (BM + BN) * DBK;  // elements per stage
  static constexpr int P = (BM + BN) / RPI / NW; // DMA instructions per wavefront per stage
  static constexpr int KK = DBK / 16;            // MFMA phases per stage
  static constexpr int NF = TM + TN, NM = TM * TN;
  static_assert(NF <= NM, "every phase must have room to prefetch the next phase's fragments");
  static_assert((BM + BN) % (RPI * NW) == 0 && (KK * NM) / P >= 1, "DMA schedule");
};

// 16 bytes per lane from global memory straight into LDS at lds_addr + 16 * lane (lds_addr wave-uniform).
// Written as inline assembly so that the compiler's wait-count bookkeeping for ordinary LDS reads stays
// exact; completion is tracked by hand through vmcnt (wait_vmcnt) and the workgroup barrier.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)p));
}
#define FAAR_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N)&0xF) | (((N) >> 4) << 14))

// Work item -> (tile, split).  Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; XCD x
// takes the x-th contiguous chunk of the item list, and the list walks the tile grid in column-major
// groups of 8 tile rows, so the 32 workgroups resident on an XCD cover a compact 8 x 4 block of tiles.
__device__ __forceinline__ bool item_coords(int pid, int tiles_m, int tiles_n, int n_split, int& tm, int& tn, int& split,
                                            int& item) {
  const int nt = tiles_m * tiles_n, items = nt * n_split;
  const int chunk = (items + 7) / 8;
  item = (pid % 8) * chunk + pid / 8;
  if (pid / 8 >= chunk || item >= items) return false;
  split = item / nt;
  const int lin = item - split * nt;
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int g = lin / per_group;
  const int first_m = g * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int r = lin - g * per_group;
  tm = first_m + r % gsz;
  tn = r / gsz;
  return true;
}

template <class C, class Epi>
__global__ void __launch_bounds__(C::THREADS)
k_gemm_dma(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, GemmDims d, int tiles_m, int tiles_n, int n_split,
           int ksteps_per_split, Epi epi) {
  __shared__ __attribute__((aligned(1024))) bf16_t lds[DNS * C::STAGE];
  epi.once();
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / C::WGN) * C::WM, wn = (wave % C::WGN) * C::WN;
  int tm, tn, split, item;
  if (!item_coords(blockIdx.x, tiles_m, tiles_n, n_split, tm, tn, split, item)) return;
  const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;
  const int ksteps = static_cast<int>(d.Kd / DBK);
  const int kbeg = split * ksteps_per_split;
  const int kend = kbeg + ksteps_per_split < ksteps ? kbeg + ksteps_per_split : ksteps;
  const int nk = kend - kbeg;
  constexpr int P = C::P, KK = C::KK, NF = C::NF, NM = C::NM;

  f32x16 acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  if (nk > 0) {
    // DMA instruction q of this wavefront fills rows [(wave*P + q)*RPI, +RPI) of the stacked [A rows; B rows]
    // stage: lane -> row = base + lane / CPR, LDS slot = lane % CPR, global chunk = slot ^ ((row / RB) % CPR).
    // Rows beyond M (or N) are clamped to the last valid row: their products are never stored.
    const bf16_t* gsrc[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
      const int trow = (wave * P + q) * C::RPI + lane / C::CPR;
      const int chunk = (lane % C::CPR) ^ ((trow / C::RB) % C::CPR);
      if (trow < C::BM) {
        const int64_t m = m0 + trow < d.M ? m0 + trow : d.M - 1;
        gsrc[q] = A + m * d.lda + chunk * 8;
      } else {
        const int64_t n = n0 + (trow - C::BM) < d.N ? n0 + (trow - C::BM) : d.N - 1;
        gsrc[q] = B + n * d.ldb + chunk * 8;
      }
    }
#pragma unroll
    for (int s = 0; s < DNS - 1; ++s) {
      const int t = kbeg + (s < nk ? s : nk - 1);
#pragma unroll
      for (int q = 0; q < P; ++q)
        dma16(gsrc[q] + (int64_t)t * DBK,
              __builtin_amdgcn_readfirstlane(lds_addr_of(lds + s * C::STAGE + (wave * P + q) * C::RPI * DBK)));
    }

    // fragment addresses: row = w? + i*32 + lane % 32, chunk = 2*kk + lane / 32, slot = chunk ^ ((row / RB) % CPR)
    const int fr = lane & 31, hi = lane >> 5;
    const int sw = (fr / C::RB) % C::CPR;
    int a_off[KK], b_off[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int slot = ((2 * kk + hi) ^ sw) * 8;
      a_off[kk] = (wm + fr) * DBK + slot;
      b_off[kk] = C::BM * DBK + (wn + fr) * DBK + slot;
    }
    bf16x8 fa[2][C::TM], fb[2][C::TN];

    FAAR_WAIT_VMCNT(P * (DNS - 2));  // slice 0 has landed (mine); barrier: everybody's
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < C::TM; ++i) fa[0][i] = *reinterpret_cast<const bf16x8*>(lds + a_off[0] + i * 32 * DBK);
#pragma unroll
    for (int j = 0; j < C::TN; ++j) fb[0][j] = *reinterpret_cast<const bf16x8*>(lds + b_off[0] + j * 32 * DBK);

    for (int it = 0; it < nk; ++it) {
      // slice it+1 must have landed before its first fragments are prefetched at the end of this iteration;
      // the barrier also guarantees that every wavefront has finished reading the stage refilled below.
      FAAR_WAIT_VMCNT(P * (DNS - 3));
      __builtin_amdgcn_s_barrier();
      const bf16_t* st = lds + (it % DNS) * C::STAGE;
      const bf16_t* st_next = lds + ((it + 1) % DNS) * C::STAGE;
      const int dma_k = kbeg + (it + DNS - 1 < nk ? it + DNS - 1 : nk - 1);  // past the end: a harmless reload
      const bf16_t* dma_base = lds + ((it + DNS - 1) % DNS) * C::STAGE + wave * P * C::RPI * DBK;
      constexpr int DSTEP = (KK * NM) / P;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const int cur = kk & 1;
        const bf16_t* src = (kk + 1 < KK) ? st : st_next;
        const int nkk = (kk + 1 < KK) ? kk + 1 : 0;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const int mi = m / C::TN, mj = m % C::TN;
          acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][mi], fb[cur][mj], acc[mi][mj], 0, 0, 0);
          if (m < NF) {  // fragment m of the next phase, in the order A0, B0..B(TN-1), A1..A(TM-1)
            if (m == 0) fa[cur ^ 1][0] = *reinterpret_cast<const bf16x8*>(src + a_off[nkk]);
            else if (m <= C::TN) fb[cur ^ 1][m - 1] = *reinterpret_cast<const bf16x8*>(src + b_off[nkk] + (m - 1) * 32 * DBK);
            else fa[cur ^ 1][m - C::TN] = *reinterpret_cast<const bf16x8*>(src + a_off[nkk] + (m - C::TN) * 32 * DBK);
          }
          const int g = kk * NM + m;
          if (g % DSTEP == DSTEP / 2 && g / DSTEP < P) {
            const int q = g / DSTEP;
            dma16(gsrc[q] + (int64_t)dma_k * DBK, __builtin_amdgcn_readfirstlane(lds_addr_of(dma_base + q * C::RPI * DBK)));
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    FAAR_WAIT_VMCNT(0);  // no copy may still be in flight into this workgroup's LDS when it retires
  }

  epi.begin();
  const int col = lane & 31, hi2 = lane >> 5;
  if constexpr (Epi::kTransposedOut) {
    // Output is wanted transposed ([n][m], m contiguous) while a lane holds 4 consecutive m of one n: stage
    // one 32-column slab per wavefront column through LDS and write whole 2*BM-byte rows with 16 B per lane.
    // staging row: BM elements + 4, i.e. a pitch of 2 words more than a multiple of 32: the 16 lanes that write one
    // 8-byte group of four rows each then fall into 32 distinct LDS banks (a pitch of BM + 8 made rows r and r + 8 collide)
    constexpr int LDT = C::BM + 4;
    constexpr int ROWS = C::WGN * 32;       // staged n-rows per pass
    constexpr int CPRW = C::BM / 8;         // 16-byte chunks per staged row
    static_assert(ROWS * LDT <= DNS * C::STAGE, "staging buffer fits in the ring");
    bf16_t* stg = lds;
    const int wc = wave % C::WGN;
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
      __syncthreads();                      // ring (or previous slab) no longer read by anybody
      const int64_t n = n0 + wn + j * 32 + col;
      float4 cv[C::TM][4];
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) cv[i][g] = epi.load4(m0 + wm + i * 32 + 8 * g + 4 * hi2, n, d);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int ml = wm + i * 32 + 8 * g + 4 * hi2;
          const float r[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          *reinterpret_cast<uint2*>(stg + (wc * 32 + col) * LDT + ml) = epi.value4(r, cv[i][g], m0 + ml, n, d);
        }
      __syncthreads();
      for (int idx = tid; idx < ROWS * CPRW; idx += C::THREADS) {
        const int row = idx / CPRW, ch = idx % CPRW;
        const uint2* src = reinterpret_cast<const uint2*>(stg + row * LDT + ch * 8);   // 8-byte aligned
        const uint2 lo = src[0], hi = src[1];
        epi.store_chunk(make_uint4(lo.x, lo.y, hi.x, hi.y), m0 + ch * 8, n0 + (row / 32) * C::WN + j * 32 + (row % 32), d);
      }
    }
  } else if constexpr (Epi::kRowStaged) {
    // as in k_gemm_dma64: one 32 x WN row of accumulator tiles per wavefront at a time through its own piece of LDS, handed
    // to the epilogue as runs of 8 consecutive columns of a row
    constexpr int PITCH = C::WN + 4;
    constexpr int RUNS = 32 * (C::WN / 8) / 64;
    static_assert(C::NW * 32 * PITCH * 4 <= DNS * C::STAGE * 2 && (32 * (C::WN / 8)) % 64 == 0, "staging fits in the ring");
    float* stg = reinterpret_cast<float*>(lds) + wave * 32 * PITCH;
    __syncthreads();                                 // nobody reads the ring any more
#pragma unroll
    for (int i = 0; i < C::TM; ++i) {
#pragma unroll
      for (int j = 0; j < C::TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int v = 0; v < 4; ++v) stg[(8 * g + 4 * hi2 + v) * PITCH + j * 32 + col] = acc[i][j][4 * g + v];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int t = 0; t < RUNS; ++t) {
        const int idx = lane + 64 * t, row = idx / (C::WN / 8), cg = idx % (C::WN / 8);
        const float4 a = *reinterpret_cast<const float4*>(stg + row * PITCH + cg * 8);
        const float4 b = *reinterpret_cast<const float4*>(stg + row * PITCH + cg * 8 + 4);
        const float r[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        epi.run8(r, m0 + wm + i * 32 + row, n0 + wn + cg * 8, split, d);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  } else {
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
      for (int j = 0; j < C::TN; ++j) {
        const int64_t n = n0 + wn + j * 32 + col;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int64_t m = m0 + wm + i * 32 + 8 * g + 4 * hi2;
          const float r[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          epi.rows4(r, m, n, split, d);
        }
      }
  }
  epi.finish(item);
}

// ---- fast path for contractions that are a multiple of 64: 128-byte LDS rows, two stages, 16x16x32 MFMAs ----
//
// The chip runs this loop power-limited, and two things lower the energy per flop: global->LDS copies whose
// eight lanes per row make one 128-byte request (BK = 64) instead of two 64-byte ones, and the 16x16x32 MFMA,
// which reads and writes a quarter of the accumulator values per instruction of the 32x32x16 form for half
// its flops.  With BK = 64 only two stages fit next to a 256x256 tile (2 x 64 KB; three for 256x128), so a stage
// is refilled as soon as the workgroup has read it: ONE barrier per slice, placed before the slice's last MFMA phase, at
// which point every wavefront holds the last fragments of the slice in registers and the copies of the next
// slice (issued NS - 1 slices earlier, right after a barrier) have landed.

constexpr int DBK64 = 64;

// kTokenMajor_: both operands are stored with the contraction index as the ROW index (A [Kd, lda], B [Kd, ldb]; "TN" product
// acc[m][n] = sum_t A[t][m] B[t][n]) -- activations and their gradients as the layers produce them, token-major.  A stage then
// holds 64 rows (tokens) of BM + BN columns, and a wavefront gathers the 8 tokens x 1 column an MFMA lane needs with two of the
// LDS transposing reads of this architecture (ds_read_b64_tr_b16) instead of one 16-byte read.
template <int BM_, int BN_, int WGM_, int WGN_, int NS_, bool kTokenMajor_ = false>
struct Dma64Cfg {
  static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, NS = NS_;  // NS ring stages (2 or 3)
  static constexpr bool kTokenMajor = kTokenMajor_;
  static_assert(!kTokenMajor_ || ((BM_ == 256 || BM_ == 192) && (BN_ == 256 || BN_ == 192)),
                "the token-major stage layout is written for 256 and 192 columns per operand");
  static constexpr int NW = WGM * WGN, THREADS = 64 * NW;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 16, TN = WN / 16;
  static constexpr int CPR = DBK64 / 8;            // 16-byte chunks per LDS row (8)
  static constexpr int RPI = 64 / CPR;             // rows written by one wave-wide DMA instruction (8)
  static constexpr int RB = 2;                     // rows per 256-byte bank cycle
  static constexpr int STAGE = (BM + BN) * DBK64;  // elements per stage
  static constexpr int P = (BM + BN) / RPI / NW;   // DMA instructions per wavefront per stage
  static constexpr int KK = DBK64 / 32;            // MFMA phases per stage (2)
  static constexpr int NF = TM + TN, NM = TM * TN;
  static constexpr int FSTEP = NM / NF >= 2 ? 2 : 1;  // one fragment prefetch every FSTEP MFMAs
  static constexpr int DSTEP = NM / P;                // one DMA issue every DSTEP MFMAs of the last phase
  static_assert(NF * FSTEP <= NM && P * DSTEP <= NM && DSTEP >= 1, "phase schedule");
  static_assert((BM + BN) % (RPI * NW) == 0 && TN % 2 == 0 && (NS == 2 || NS == 3), "tile shape");
};

// Eight consecutive tokens of one column for every lane, from a token-major stage: two transposing reads of 4 tokens each.
// Within a group of 16 lanes, lane r supplies the address of 4 consecutive columns of one token; lane i receives column
// i % 4 of the tokens that lanes i / 4 + {0, 4, 8, 12} pointed at.  With lane r pointing at token r / 4, columns 4 (r % 4) ..,
// lane i therefore receives column i of tokens 0..3: an MFMA operand row per lane.  `p`: this lane's address for the first
// read; the second reads 4 tokens (4 * pitch elements) further on.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
template <int PITCH>
__device__ __forceinline__ bf16x8 read_tokens8(const bf16_t* p) {
  typedef __attribute__((address_space(3))) s16x4* lds_ptr;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * PITCH));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
// XOR key of a token row's pairs of 16-byte chunks (32 bytes = the 16 columns one transposing read takes from a token) in a
// token-major stage of COLS columns per token.  One read touches 16 token rows -- 4 consecutive tokens in each of 4 groups 8
// apart -- and they must fall into the 8 different 32-byte bank groups, two rows each (the two cycles 512 bytes take anyway).
// 256 columns: a row is 512 bytes, every row starts at bank 0, so the key has 3 bits (token bits 0, 1, 3) and permutes a row's
// pairs within aligned groups of 8.  192 columns: a row is 384 bytes, odd rows start half-way round the banks, so token bit 0 is
// taken care of and the key has 2 bits (token bits 1, 3), permuting pairs within aligned groups of 4 -- which 12 pairs divide into.
template <int COLS>
__device__ __forceinline__ int token_key(int t) {
  static_assert(COLS == 256 || COLS == 192, "token-major operand width");
  return COLS == 256 ? (t & 3) | (((t >> 3) & 1) << 2) : ((t >> 1) & 1) | (((t >> 3) & 1) << 1);
}

template <class C, class Epi>
__global__ void __launch_bounds__(C::THREADS)
k_gemm_dma64(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, GemmDims d, int tiles_m, int tiles_n, int n_split,
             int ksteps_per_split, Epi epi) {
  __shared__ __attribute__((aligned(1024))) bf16_t lds[C::NS * C::STAGE];
  // where the side reads of an epilogue with kWarm land: 1 KB per wavefront, never read
  __shared__ __attribute__((aligned(1024))) uint32_t warm_sink[Epi::kWarm ? C::NW * 256 : 4];
  epi.once();
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / C::WGN) * C::WM, wn = (wave % C::WGN) * C::WN;
  int tm, tn, split, item;
  if (!item_coords(blockIdx.x, tiles_m, tiles_n, n_split, tm, tn, split, item)) return;
  const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;
  const int ksteps = static_cast<int>(d.Kd / DBK64);
  const int kbeg = split * ksteps_per_split;
  const int kend = kbeg + ksteps_per_split < ksteps ? kbeg + ksteps_per_split : ksteps;
  const int nk = kend - kbeg;
  constexpr int P = C::P, KK = C::KK, NF = C::NF, NM = C::NM, TM = C::TM, TN = C::TN;
  // vector-memory instructions a wavefront issues per slice: the copies, and one side read with kWarm.  Loads complete
  // in order, so the wait counts below are in units of this
  constexpr int PW = P + (Epi::kWarm ? 1 : 0);
  static_assert(PW * (C::NS - 1) < 64, "vmcnt is a 6-bit counter");

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;

  if (nk > 0) {
    // DMA instruction q of this wavefront fills rows [(wave*P + q)*RPI, +RPI) of the stacked [A rows; B rows]
    // stage: lane -> row = base + lane / CPR, LDS slot = lane % CPR, global chunk = slot ^ ((row / RB) % CPR).
    // Rows beyond M (or N) are clamped to the last valid row: their products are never stored.
    const bf16_t* gsrc[P];
    int64_t gstep[P];   // elements from one slice to the next
#pragma unroll
    for (int q = 0; q < P; ++q) {
      if constexpr (C::kTokenMajor) {
        // instruction u = wave * P + q fills 64 consecutive 16-byte slots of the stage; an operand of COLS columns owns
        // 64 tokens x COLS / 8 slots (a whole number of instructions), slot -> token = slot / (COLS / 8), LDS chunk =
        // slot % (COLS / 8), global chunk = that ^ 2 key(token).  Columns beyond M (or N) are clamped to the last whole chunk:
        // their products are never stored.
        const int u = wave * P + q;
        const bool is_a = u < C::BM / 8;
        int t, chunk;
        if constexpr (C::BM == 256 && C::BN == 256) {   // two whole token rows per instruction
          t = 2 * (is_a ? u : u - C::BM / 8) + lane / 32;
          chunk = (lane % 32) ^ (2 * token_key<256>(t));
        } else {
          const int slot = (is_a ? u : u - C::BM / 8) * 64 + lane;
          t = is_a ? slot / (C::BM / 8) : slot / (C::BN / 8);
          chunk = is_a ? (slot % (C::BM / 8)) ^ (2 * token_key<C::BM>(t)) : (slot % (C::BN / 8)) ^ (2 * token_key<C::BN>(t));
        }
        const int64_t first = is_a ? m0 : n0, width = is_a ? d.M : d.N, ld = is_a ? d.lda : d.ldb;
        const int64_t col = first + chunk * 8 <= width - 8 ? first + chunk * 8 : width - 8;
        gsrc[q] = (is_a ? A : B) + t * ld + col;
        gstep[q] = DBK64 * ld;
      } else {
        const int trow = (wave * P + q) * C::RPI + lane / C::CPR;
        const int chunk = (lane % C::CPR) ^ ((trow / C::RB) % C::CPR);
        if (trow < C::BM) {
          const int64_t m = m0 + trow < d.M ? m0 + trow : d.M - 1;
          gsrc[q] = A + m * d.lda + chunk * 8;
        } else {
          const int64_t n = n0 + (trow - C::BM) < d.N ? n0 + (trow - C::BM) : d.N - 1;
          gsrc[q] = B + n * d.ldb + chunk * 8;
        }
        gstep[q] = DBK64;
      }
    }
    // side read (kWarm) that goes with slice `rel` of this work item: the 1 KB chunk of the epilogue's buffer whose number
    // counts (workgroup, slice, wavefront) triples from the END of the launch (workgroups are dispatched in the order of
    // their ids), so that the buffer is read late, close to the kernel that wants it; triples beyond the buffer re-read one
    // valid address (the instruction count per slice stays uniform)
    const uint32_t warm_dst = __builtin_amdgcn_readfirstlane(lds_addr_of(warm_sink + (Epi::kWarm ? wave * 256 : 0)));
    const int64_t warm_last = ((int64_t)gridDim.x - blockIdx.x) * nk - 1;   // triple number of slice 0, before the wavefront
    static_assert(!Epi::kWarm || (P - 1) * C::DSTEP + 1 < NM, "room for the side read after the slice's last copy");
#define FAAR_SIDE_READ(REL)                                                                                              \
  if constexpr (Epi::kWarm) {                                                                                            \
    const int64_t chunk_ = (warm_last - (REL)) * C::NW + wave;                                                           \
    const bool in_ = epi.warm != nullptr && (REL) < nk && chunk_ < epi.warm_chunks;                                      \
    dma16(in_ ? static_cast<const char*>(epi.warm) + chunk_ * 1024 + lane * 16 : reinterpret_cast<const char*>(A), warm_dst); \
  }
#pragma unroll
    for (int s = 0; s < C::NS; ++s) {
      const int t = kbeg + (s < nk ? s : nk - 1);
#pragma unroll
      for (int q = 0; q < P; ++q)
        dma16(gsrc[q] + (int64_t)t * gstep[q],
              __builtin_amdgcn_readfirstlane(lds_addr_of(lds + s * C::STAGE + (wave * P + q) * C::RPI * DBK64)));
      FAAR_SIDE_READ(s)
    }

    // fragment addresses: row = w? + i*16 + lane % 16, chunk = 4*kk + lane / 16, slot = chunk ^ ((row / RB) % CPR);
    // the 16 lanes that share a chunk index then cover 16 distinct 16-byte bank groups
    const int fr = lane & 15, kc = lane >> 4;
    const int sw = (fr / C::RB) % C::CPR;
    int a_off[KK], b_off[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int slot = ((4 * kk + kc) ^ sw) * 8;
      a_off[kk] = (wm + fr) * DBK64 + slot;
      b_off[kk] = C::BM * DBK64 + (wn + fr) * DBK64 + slot;
    }
    // token-major stage: element offset of this lane's first transposing read for fragment i (A) / j (B) of phase 0.  The
    // lane points at token 8 (lane / 16) + (lane % 16) / 4 of the phase's 32 and at columns w? + 16 i + 4 (lane % 4); that
    // token's XOR key is the same in every phase and for both reads of a fragment (no key uses token bits 2, 4 or 5)
    int a_tr[TM] = {}, b_tr[TN] = {};
    if constexpr (C::kTokenMajor) {
      const int tok = 8 * kc + (fr >> 2);
      const int key_a = token_key<C::BM>(tok), key_b = token_key<C::BN>(tok);
#pragma unroll
      for (int i = 0; i < TM; ++i) a_tr[i] = tok * C::BM + (((wm / 16 + i) ^ key_a) * 16) + (fr & 3) * 4;
#pragma unroll
      for (int j = 0; j < TN; ++j) b_tr[j] = C::BM * DBK64 + tok * C::BN + (((wn / 16 + j) ^ key_b) * 16) + (fr & 3) * 4;
    }
    // fragment i of the A rows (j of the B rows) for phase kk, from the stage at `src`
#define FAAR_FRAG_A(SRC, KKI, I)                                                                                         \
  (C::kTokenMajor ? read_tokens8<C::BM>((SRC) + a_tr[I] + 32 * (KKI) * C::BM)                                            \
                  : *reinterpret_cast<const bf16x8*>((SRC) + a_off[KKI] + (I) * 16 * DBK64))
#define FAAR_FRAG_B(SRC, KKI, J)                                                                                         \
  (C::kTokenMajor ? read_tokens8<C::BN>((SRC) + b_tr[J] + 32 * (KKI) * C::BN)                                            \
                  : *reinterpret_cast<const bf16x8*>((SRC) + b_off[KKI] + (J) * 16 * DBK64))
    bf16x8 fa[2][TM], fb[2][TN];

    FAAR_WAIT_VMCNT(PW * (C::NS - 1));  // slice 0 has landed (mine); barrier: everybody's
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      fa[0][i] = FAAR_FRAG_A(lds, 0, i);
      fa[1][i] = fa[0][i];
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      fb[0][j] = FAAR_FRAG_B(lds, 0, j);
      fb[1][j] = fb[0][j];
    }

    for (int it = 0; it < nk; ++it) {
      bf16_t* st = lds + (it % C::NS) * C::STAGE;
      const bf16_t* sn = lds + ((it + 1) % C::NS) * C::STAGE;
      const bool more = it + C::NS < nk;
      const int64_t gslice = kbeg + it + C::NS;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const int cur = kk & 1;
        if (kk == KK - 1) {
          // this wavefront's copies of slice it+1 have landed and its reads of slice it are complete;
          // after the barrier that holds for the workgroup: stage `st` may be refilled, `sn` may be read
          constexpr int kInFlight = PW * (C::NS - 2);  // copies of later slices may stay in flight
          __builtin_amdgcn_s_waitcnt(0x0070 | (kInFlight & 0xF) | ((kInFlight >> 4) << 14));  // vmcnt(kInFlight) lgkmcnt(0)
          __builtin_amdgcn_s_barrier();
        }
        const bf16_t* src = (kk + 1 < KK) ? st : sn;
        const int nkk = (kk + 1 < KK) ? kk + 1 : 0;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          // boustrophedon over the tile grid: consecutive MFMAs share one operand
          const int mi = m / TN, mj = (mi & 1) ? TN - 1 - m % TN : m % TN;
          if constexpr (Epi::kMode != 2)
            acc[mi][mj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[cur][mi], fb[cur][mj], acc[mi][mj], 0, 0, 0);
          if constexpr (Epi::kMode != 2 && C::kTokenMajor && C::FSTEP == 2) {
            // token-major: a fragment is two transposing reads; one of them per MFMA instead of both every other MFMA
            // (in a slice's last phase, where the copies are issued too, spread over all of the phase's MFMAs: every
            // SKIP-th one goes without; in the others the reads have to be complete at the next barrier, so they go first)
            constexpr int SKIP = NM / (NM - 2 * NF);
            static_assert(NM % (NM - 2 * NF) == 0, "read schedule");
            const bool spread = kk == KK - 1;
            const int r = spread ? m - m / SKIP : m;
            if (r < 2 * NF && !(spread && m % SKIP == SKIP - 1)) {
              const int f = r / 2, h = r % 2;
              typedef __attribute__((address_space(3))) s16x4* lds_ptr;
              if (f == 0 || f > TN) {
                const int i = f == 0 ? 0 : f - TN;
                const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + a_tr[i] + 32 * nkk * C::BM + h * 4 * C::BM));
                s16x8 t = __builtin_bit_cast(s16x8, fa[cur ^ 1][i]);
                if (h == 0) t.lo = v; else t.hi = v;
                fa[cur ^ 1][i] = __builtin_bit_cast(bf16x8, t);
              } else {
                const int j = f - 1;
                const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + b_tr[j] + 32 * nkk * C::BN + h * 4 * C::BN));
                s16x8 t = __builtin_bit_cast(s16x8, fb[cur ^ 1][j]);
                if (h == 0) t.lo = v; else t.hi = v;
                fb[cur ^ 1][j] = __builtin_bit_cast(bf16x8, t);
              }
            }
          } else
          if (Epi::kMode != 2 && m % C::FSTEP == 0 && m / C::FSTEP < NF) {  // next phase's fragments: A0, B0..B(TN-1), A1..A(TM-1)
            const int f = m / C::FSTEP;
            if (f == 0) fa[cur ^ 1][0] = FAAR_FRAG_A(src, nkk, 0);
            else if (f <= TN) fb[cur ^ 1][f - 1] = FAAR_FRAG_B(src, nkk, f - 1);
            else fa[cur ^ 1][f - TN] = FAAR_FRAG_A(src, nkk, f - TN);
          }
          if (Epi::kMode != 1 && kk == KK - 1 && m % C::DSTEP == 0 && m / C::DSTEP < P) {
            // slice it+NS into the stage just released; past the end every lane re-reads one valid address
            const int q = m / C::DSTEP;
            const bf16_t* g = more ? gsrc[q] + gslice * gstep[q] : A;
            dma16(g, __builtin_amdgcn_readfirstlane(lds_addr_of(st + (wave * P + q) * C::RPI * DBK64)));
          }
          if (Epi::kMode != 1 && kk == KK - 1 && m == (P - 1) * C::DSTEP + 1) {   // right after the slice's last copy
            FAAR_SIDE_READ(it + C::NS)
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    FAAR_WAIT_VMCNT(0);  // no copy may still be in flight into this workgroup's LDS when it retires
#undef FAAR_SIDE_READ
#undef FAAR_FRAG_A
#undef FAAR_FRAG_B
  }

  // accumulator layout of the 16x16 tile: lane -> column lane % 16, rows 4 * (lane / 16) + 0..3
  epi.begin();
  const int col = lane & 15, rq = lane >> 4;
  if constexpr (Epi::kTransposedOut) {
    // as in k_gemm_dma: stage a 32-column slab (two 16-column tiles) per wavefront column through LDS and
    // write whole rows of the transposed output with 16 B per lane
    constexpr int LDT = C::BM + 4;          // pitch of 2 words beyond a multiple of 32: conflict-free 8-byte writes
    constexpr int ROWS = C::WGN * 32;
    constexpr int CPRW = C::BM / 8;
    static_assert(ROWS * LDT <= C::NS * C::STAGE, "staging buffer fits in the ring");
    bf16_t* stg = lds;
    const int wc = wave % C::WGN;
#pragma unroll
    for (int jj = 0; jj < TN / 2; ++jj) {
      __syncthreads();
      float4 cv[TM][2];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          cv[i][h] = epi.load4(m0 + wm + i * 16 + 4 * rq, n0 + wn + (2 * jj + h) * 16 + col, d);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int ml = wm + i * 16 + 4 * rq;
          const float r[4] = {acc[i][2 * jj + h][0], acc[i][2 * jj + h][1], acc[i][2 * jj + h][2], acc[i][2 * jj + h][3]};
          *reinterpret_cast<uint2*>(stg + (wc * 32 + h * 16 + col) * LDT + ml) =
              epi.value4(r, cv[i][h], m0 + ml, n0 + wn + (2 * jj + h) * 16 + col, d);
        }
      __syncthreads();
      for (int idx = tid; idx < ROWS * CPRW; idx += C::THREADS) {
        const int row = idx / CPRW, ch = idx % CPRW;
        const uint2* src = reinterpret_cast<const uint2*>(stg + row * LDT + ch * 8);   // 8-byte aligned
        const uint2 lo = src[0], hi = src[1];
        epi.store_chunk(make_uint4(lo.x, lo.y, hi.x, hi.y), m0 + ch * 8, n0 + (row / 32) * C::WN + jj * 32 + (row % 32), d);
      }
    }
  } else if constexpr (Epi::kRowStaged) {
    // every wavefront stages one 16 x WN row of its accumulator tiles at a time through its own piece of LDS and hands the
    // epilogue runs of 8 consecutive columns of a row: 16-byte operand loads and stores, a quarter of the instructions
    constexpr int PITCH = C::WN + 4;                 // floats; 4 * PITCH = 16 mod 32: the two row groups of a half-wave miss each other
    constexpr int RUNS = 16 * (C::WN / 8) / 64;      // runs per lane and staged row
    static_assert(C::NW * 16 * PITCH * 4 <= C::NS * C::STAGE * 2 && (16 * (C::WN / 8)) % 64 == 0, "staging fits in the ring");
    float* stg = reinterpret_cast<float*>(lds) + wave * 16 * PITCH;
    __syncthreads();                                 // nobody reads the ring any more
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) stg[(4 * rq + v) * PITCH + j * 16 + col] = acc[i][j][v];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int t = 0; t < RUNS; ++t) {
        const int idx = lane + 64 * t, row = idx / (C::WN / 8), cg = idx % (C::WN / 8);
        const float4 a = *reinterpret_cast<const float4*>(stg + row * PITCH + cg * 8);
        const float4 b = *reinterpret_cast<const float4*>(stg + row * PITCH + cg * 8 + 4);
        const float r[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        epi.run8(r, m0 + wm + i * 16 + row, n0 + wn + cg * 8, split, d);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const float r[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
        epi.rows4(r, m0 + wm + i * 16 + 4 * rq, n0 + wn + j * 16 + col, split, d);
      }
  }
  epi.finish(item);
}

typedef Tile<128, 128> T128;
typedef DmaCfg<256, 256, 2, 4> CfgL;  // large problems
typedef DmaCfg<256, 128, 4, 2> CfgM;  // one tile per compute unit at ~256 tiles
typedef DmaCfg<128, 128, 2, 2> CfgS;  // small outputs, two workgroups per compute unit
typedef Dma64Cfg<256, 256, 2, 4, 2> CfgL64;  // 2 x 64 KB
typedef Dma64Cfg<256, 128, 4, 2, 3> CfgM64;  // 3 x 48 KB: copies stay in flight for two slices
typedef Dma64Cfg<256, 256, 2, 4, 2, true> CfgT64;  // CfgL64 on token-major operands
// ... and with 192 rows (columns) per tile: 6144 x 2048 is 24 x 8 = 192 tiles of 256 x 256 -- a quarter of the 256 compute units
// idle -- but 32 x 8 = 256 tiles of 192 x 256
typedef Dma64Cfg<192, 256, 2, 4, 2, true> CfgT64A;
typedef Dma64Cfg<256, 192, 4, 2, 2, true> CfgT64B;

inline int ceil_div(int64_t a, int64_t b) { return static_cast<int>((a + b - 1) / b); }

enum { KIND_GENERIC = 0, KIND_L = 1, KIND_M = 2, KIND_S = 3, KIND_L64 = 4, KIND_M64 = 5 };

struct Plan {
  int kind, tiles_m, tiles_n, n_split;
  int64_t items() const { return (int64_t)tiles_m * tiles_n * n_split; }
};

inline Plan make_plan(int kind, const GemmDims& d, int n_split) {
  const int bm = kind == KIND_S || kind == KIND_GENERIC ? 128 : 256;
  const int bn = kind == KIND_L || kind == KIND_L64 ? 256 : 128;
  return Plan{kind, ceil_div(d.M, bm), ceil_div(d.N, bn), n_split};
}

// Tile shape and contraction split, chosen by a small cost model (all times in microseconds, calibrated on
// MI355X with every compute unit busy).  A compute unit works through one BK-slice of a tile in c_kind;
// an item's epilogue costs a fixed part plus its global traffic (reads count fully, writes half: they do not
// stall the wave) at one compute unit's share of the memory bandwidth.  Items are dealt in rounds of 256.
// Large tiles cut LDS and L2 traffic per flop but quantise badly on small outputs; splitting the contraction
// (allowed only where partial sums may be written separately) buys back occupancy at the price of one more
// float32 partial per split, which the consumer has to read.
struct EpiCost { float read_bytes, write_bytes; };  // per output element

Plan plan_gemm(const GemmDims& d, bool may_split, EpiCost epi) {
  if (d.Kd % DBK != 0) {
    Plan p = make_plan(KIND_GENERIC, d, 1);
    if (may_split)
      while (p.items() < 256 && d.Kd / (p.n_split * 2) >= 512 && p.n_split < 16) p.n_split *= 2;
    return p;
  }
  // contractions that are a multiple of 64 take the 128-byte-row kernels for the two large shapes
  const bool k64 = d.Kd % DBK64 == 0;
  const int kinds[3] = {k64 ? KIND_L64 : KIND_L, k64 ? KIND_M64 : KIND_M, KIND_S};
  const double slice_us[3] = {k64 ? 0.833 : 0.985, k64 ? 0.552 : 0.63, 0.36};  // per 32 of the contraction
  const double tile_outputs[3] = {256.0 * 256.0, 256.0 * 128.0, 128.0 * 128.0};
  const double cu_bytes_per_us = 17600.0;   // ~4.5 TB/s over 256 compute units
  Plan best{};
  double best_cost = 0.0;
  for (int i = 0; i < 3; ++i) {
    for (int sp = 1; sp <= (may_split ? 8 : 1); ++sp) {
      if (sp > 1 && d.Kd / sp < 512) break;
      const int64_t ksteps = d.Kd / (i < 2 && k64 ? DBK64 : DBK), per = (ksteps + sp - 1) / sp;
      if ((sp - 1) * per >= ksteps) continue;  // the last split would be empty
      const Plan p = make_plan(kinds[i], d, sp);
      const double rounds = static_cast<double>((p.items() + 255) / 256);
      const double epilogue = 3.0 + tile_outputs[i] * (epi.read_bytes + 0.5 * epi.write_bytes) / cu_bytes_per_us;
      double cost = rounds * (static_cast<double>(per) * (i < 2 && k64 ? 2.0 : 1.0) * slice_us[i] + epilogue);
      // every extra split is one more float32 partial written here and read back by the consumer
      cost += (sp - 1) * static_cast<double>(d.M) * static_cast<double>(d.N) * 8.0 / 5.0e6;
      if (best.kind == 0 || cost < best_cost) {
        best = p;
        best_cost = cost;
      }
    }
  }
  return best;
}

constexpr EpiCost kEpiGram{2.0f, 4.0f}, kEpiResidual{4.0f, 2.0f}, kEpiF32{0.0f, 4.0f}, kEpiSub{4.0f, 4.0f}, kEpiBf16{0.0f, 2.0f}, kEpiNone{0.0f, 0.0f};

template <class Epi>
hipError_t run(const bf16_t* A, const bf16_t* B, GemmDims d, Plan p, Epi epi, hipStream_t st) {
  if (p.kind == KIND_GENERIC) {
    const int64_t k_per_split = round_up((d.Kd + p.n_split - 1) / p.n_split, BK);
    const dim3 grid(static_cast<unsigned>(p.items()));
    hipLaunchKernelGGL((k_gemm_nt<T128, Epi>), grid, dim3(GEMM_THREADS), 0, st, A, B, d, p.tiles_m, p.tiles_n, k_per_split, epi);
    return hipGetLastError();
  }
  const bool k64 = p.kind == KIND_L64 || p.kind == KIND_M64;
  const int ksteps = static_cast<int>(d.Kd / (k64 ? DBK64 : DBK));
  const int per_split = (ksteps + p.n_split - 1) / p.n_split;
  const dim3 grid(static_cast<unsigned>((p.items() + 7) / 8 * 8));
#define FAAR_LAUNCH(KERNEL, CFG) \
  hipLaunchKernelGGL((KERNEL<CFG, Epi>), grid, dim3(CFG::THREADS), 0, st, A, B, d, p.tiles_m, p.tiles_n, p.n_split, per_split, epi)
  if (p.kind == KIND_L64) FAAR_LAUNCH(k_gemm_dma64, CfgL64);
  else if (p.kind == KIND_M64) FAAR_LAUNCH(k_gemm_dma64, CfgM64);
  else if (p.kind == KIND_L) FAAR_LAUNCH(k_gemm_dma, CfgL);
  else if (p.kind == KIND_M) FAAR_LAUNCH(k_gemm_dma, CfgM);
  else FAAR_LAUNCH(k_gemm_dma, CfgS);
#undef FAAR_LAUNCH
  return hipGetLastError();
}

}  // namespace

int64_t gemm_residual_partials(int64_t M, int64_t N, int64_t Kd) {  // the most any of the three epilogues writes
  const GemmDims d{M, N, Kd, Kd, Kd};
  return std::max(plan_gemm(d, false, kEpiResidual).items(),
                  std::max(plan_gemm(d, false, kEpiBf16).items(), plan_gemm(d, false, kEpiNone).items()));
}

hipError_t launch_gemm_residual_rows(const bf16_t* A, const bf16_t* B, GemmDims d, const float* x_scale, float two_alpha,
                                     bf16_t* dY, double* mse_partials, int64_t* n_partials, const ForwardGuard& guard,
                                     hipStream_t st) {
  if (d.N % 8 != 0) return hipErrorInvalidValue;
  EpiPerturbationRows e{x_scale, 1.0f, guard, two_alpha, dY, mse_partials, 0.0f};
  const Plan p = plan_gemm(d, false, kEpiBf16);
  *n_partials = p.items();
  return run(A, B, d, p, e, st);
}

hipError_t launch_gemm_residual(const bf16_t* A, const bf16_t* B, GemmDims d, const float* C, const float* x_scale,
                                float two_alpha, bf16_t* dYt, int64_t ldt, bf16_t* dY,
                                double* mse_partials, int64_t* n_partials, const ForwardGuard& guard, const void* warm,
                                int64_t warm_bytes, hipStream_t st) {
  const int64_t warm_chunks = warm ? warm_bytes / 1024 : 0;
  if (C) {
    EpiResidual e{C, x_scale, 1.0f, guard, two_alpha, dYt, ldt, dY, mse_partials, 0.0f, warm, warm_chunks};
    const Plan p = plan_gemm(d, false, kEpiResidual);
    *n_partials = p.items();
    return run(A, B, d, p, e, st);
  }
  if (dY) return hipErrorInvalidValue;   // the un-transposed dY exists only with the constant
  if (dYt) {
    EpiPerturbation e{nullptr, x_scale, 1.0f, guard, two_alpha, dYt, ldt, nullptr, mse_partials, 0.0f, warm, warm_chunks};
    const Plan p = plan_gemm(d, false, kEpiBf16);
    *n_partials = p.items();
    return run(A, B, d, p, e, st);
  }
  EpiSumSq e{x_scale, 1.0f, guard, mse_partials, 0.0f};
  const Plan p = plan_gemm(d, false, kEpiNone);
  *n_partials = p.items();
  return run(A, B, d, p, e, st);
}

int choose_split(int64_t M, int64_t N, int64_t Kd) { return plan_gemm(GemmDims{M, N, Kd, Kd, Kd}, true, kEpiF32).n_split; }

GemmPlanInfo gemm_plan_info(int epilogue, int64_t M, int64_t N, int64_t Kd) {
  const GemmDims d{M, N, Kd, Kd, Kd};
  const Plan p = epilogue == kGemmEpiResidual ? plan_gemm(d, false, kEpiResidual)
               : epilogue == kGemmEpiF32    ? plan_gemm(d, true, kEpiF32)
               : epilogue == kGemmEpiSub    ? plan_gemm(d, false, kEpiSub)
               : epilogue == kGemmEpiNone   ? plan_gemm(d, false, kEpiNone)
               : epilogue == kGemmEpiGram   ? plan_gemm(d, true, kEpiGram)
                                            : plan_gemm(d, false, kEpiBf16);
  const int bm = p.kind == KIND_S || p.kind == KIND_GENERIC ? 128 : 256;
  const int bn = p.kind == KIND_L || p.kind == KIND_L64 ? 256 : 128;
  return GemmPlanInfo{p.kind, bm, bn, p.n_split};
}

hipError_t launch_gemm_f32(const bf16_t* A, const bf16_t* B, GemmDims d, float* out, int n_split,
                           hipStream_t st) {
  EpiF32 e{out};
  Plan p = plan_gemm(d, true, kEpiF32);
  if (p.n_split != n_split) return hipErrorInvalidValue;  // the caller sized its workspace with choose_split
  return run(A, B, d, p, e, st);
}

int choose_split_gram(int64_t O, int64_t K) { return plan_gemm(GemmDims{O, K, K, K, K}, true, kEpiGram).n_split; }
int64_t gemm_gram_partials(int64_t O, int64_t K) { return plan_gemm(GemmDims{O, K, K, K, K}, true, kEpiGram).items(); }

hipError_t launch_gemm_gram(const bf16_t* delta, const bf16_t* gram, int64_t O, int64_t K, const float* diag_lo,
                            const float* x_scale, float two_alpha, float* out, int n_split, double* partials,
                            int64_t* n_partials, const ForwardGuard& guard, hipStream_t st) {
  const GemmDims d{O, K, K, K, K};
  const Plan p = plan_gemm(d, true, kEpiGram);
  if (p.n_split != n_split) return hipErrorInvalidValue;  // the caller sized its workspace with choose_split_gram
  *n_partials = p.items();
  EpiGram e{delta, diag_lo, x_scale, 1.0f, guard, two_alpha, out, partials, 0.0f};
  return run(delta, gram, d, p, e, st);
}

// Tile shape of the token-major product: 0 not usable, 1 256 x 256, 2 192 x 256, 3 256 x 192.  The contraction split is the
// one planned for 256 x 256 tiles.  fill_device: the kernel has the device to itself, so a 192-wide shape is taken when its
// work items need fewer rounds of the 256 compute units, weighted by the tile's area (6144 x 2048, one split: 192 items of
// 65536 -> one round at 65536; 256 items of 49152 -> one round at 49152).  Otherwise other kernels run on whatever units this
// one leaves idle, and the tile with the most work per byte moved wins: 256 x 256.
int gemm_tn_tiles(int64_t M, int64_t N, int64_t T, bool fill_device) {
  if (T <= 0 || T % DBK64 != 0 || M % 8 != 0 || N % 8 != 0) return 0;
  const Plan p = plan_gemm(GemmDims{M, N, T, T, T}, true, kEpiF32);
  if (p.kind != KIND_L64) return 0;
  if (!fill_device) return 1;
  const int64_t cus = 256;
  auto rounds_area = [&](int64_t bm, int64_t bn) {
    const int64_t items = (int64_t)ceil_div(M, bm) * ceil_div(N, bn) * p.n_split;
    return (items + cus - 1) / cus * bm * bn;
  };
  const int64_t c1 = rounds_area(256, 256), c2 = rounds_area(192, 256), c3 = rounds_area(256, 192);
  if (c2 < c1 && c2 <= c3) return 2;
  if (c3 < c1) return 3;
  return 1;
}
bool gemm_tn_usable(int64_t M, int64_t N, int64_t T) { return gemm_tn_tiles(M, N, T, false) != 0; }

template <class C, class Epi>
static hipError_t run_tn(const bf16_t* A, const bf16_t* B, const GemmDims& d, int n_split, Epi epi, hipStream_t st) {
  const int tiles_m = ceil_div(d.M, C::BM), tiles_n = ceil_div(d.N, C::BN);
  const int ksteps = static_cast<int>(d.Kd / DBK64);
  const int per_split = (ksteps + n_split - 1) / n_split;
  const int64_t items = (int64_t)tiles_m * tiles_n * n_split;
  const dim3 grid(static_cast<unsigned>((items + 7) / 8 * 8));
  hipLaunchKernelGGL((k_gemm_dma64<C, Epi>), grid, dim3(C::THREADS), 0, st, A, B, d, tiles_m, tiles_n, n_split, per_split, epi);
  return hipGetLastError();
}

hipError_t launch_gemm_f32_tn(const bf16_t* A, const bf16_t* B, GemmDims d, float* out, int n_split, bool fill_device,
                              hipStream_t st) {
  const int tiles = gemm_tn_tiles(d.M, d.N, d.Kd, fill_device);
  if (tiles == 0 || d.lda % 8 != 0 || d.ldb % 8 != 0) return hipErrorInvalidValue;
  const Plan p = plan_gemm(GemmDims{d.M, d.N, d.Kd, d.Kd, d.Kd}, true, kEpiF32);
  if (p.n_split != n_split) return hipErrorInvalidValue;
  if (tiles == 2) return run_tn<CfgT64A>(A, B, d, n_split, EpiF32{out}, st);
  if (tiles == 3) return run_tn<CfgT64B>(A, B, d, n_split, EpiF32{out}, st);
  return run_tn<CfgT64>(A, B, d, n_split, EpiF32{out}, st);
}

hipError_t launch_gemm_probe(int mode, const bf16_t* A, const bf16_t* B, GemmDims d, unsigned long long* clocks,
                             int64_t capacity, float* sink, int* kind, int64_t* items, hipStream_t st) {
  const Plan p = plan_gemm(d, false, kEpiF32);
  *kind = p.kind;
  *items = p.items();
  if (p.kind != KIND_L64 && p.kind != KIND_M64) return hipErrorNotSupported;   // only the BK = 64 loop has the variants
  if (p.items() > capacity) return hipErrorInvalidValue;
  if (mode & 4) {   // the same loops on token-major operands: the buffers are read as A [Kd, M], B [Kd, N]
    if (!gemm_tn_usable(d.M, d.N, d.Kd)) return hipErrorNotSupported;
    const GemmDims t{d.M, d.N, d.Kd, d.M, d.N};
    if (mode & 8) {   // ... on 192-wide tiles (whole loop only), whichever of the two shapes divides the product better
      if ((mode & 3) != 0) return hipErrorNotSupported;
      const bool a192 = ceil_div(d.M, 192) * (int64_t)ceil_div(d.N, 256) <= ceil_div(d.M, 256) * (int64_t)ceil_div(d.N, 192);
      *items = a192 ? ceil_div(d.M, 192) * (int64_t)ceil_div(d.N, 256) : ceil_div(d.M, 256) * (int64_t)ceil_div(d.N, 192);
      if (*items > capacity) return hipErrorInvalidValue;
      const EpiProbe<0> e{clocks, sink, 0, 0, 0.0f};
      return a192 ? run_tn<CfgT64A>(A, B, t, 1, e, st) : run_tn<CfgT64B>(A, B, t, 1, e, st);
    }
    if ((mode & 3) == 0) return run_tn<CfgT64>(A, B, t, 1, EpiProbe<0>{clocks, sink, 0, 0, 0.0f}, st);
    if ((mode & 3) == 1) return run_tn<CfgT64>(A, B, t, 1, EpiProbe<1>{clocks, sink, 0, 0, 0.0f}, st);
    return run_tn<CfgT64>(A, B, t, 1, EpiProbe<2>{clocks, sink, 0, 0, 0.0f}, st);
  }
  if (mode & 8) return hipErrorNotSupported;
  if (mode == 0) return run(A, B, d, p, EpiProbe<0>{clocks, sink, 0, 0, 0.0f}, st);
  if (mode == 1) return run(A, B, d, p, EpiProbe<1>{clocks, sink, 0, 0, 0.0f}, st);
  return run(A, B, d, p, EpiProbe<2>{clocks, sink, 0, 0, 0.0f}, st);
}

hipError_t launch_gemm_sub(const bf16_t* A, const bf16_t* B, GemmDims d, const void* Y, bool y_bf16,
                           bool first, float* C_out, const float* x_scale, hipStream_t st) {
  const Plan p = plan_gemm(d, false, kEpiSub);
  if (y_bf16) {
    EpiSub<true> e{Y, first, C_out, x_scale, 1.0f};
    return run(A, B, d, p, e, st);
  }
  EpiSub<false> e{Y, first, C_out, x_scale, 1.0f};
  return run(A, B, d, p, e, st);
}

hipError_t launch_gemm_bf16(const bf16_t* A, const bf16_t* B, GemmDims d, bf16_t* out, const float* scale, hipStream_t st) {
  EpiBf16 e{out, scale, 1.0f};
  return run(A, B, d, plan_gemm(d, false, kEpiBf16), e, st);
}

}  // namespace faar
