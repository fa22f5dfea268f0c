// bf16 MFMA GEMMs of the FAAR layer step for gfx950 (paper Table 2 steps 8-10 and the chain rule
// of Eq. 5): the residual GEMM  X_q (W_q - W)^T - C  with its loss / dY epilogue, the weight
// gradient  dY^T X_q  and the optional input gradient  dY W_q.
//
// Every product is computed as an "NT" GEMM  acc[m][n] = sum_k A[m][k] B[n][k]  with both operands
// row-major and the contraction index contiguous; operands that the mathematics wants transposed
// (X_q^T, dY^T, W_q^T) are produced in that layout by the kernel that writes them, so one tuned
// main loop serves all of them.
//
// Main loop: a BM x BN output tile per 256-thread workgroup (2 x 2 wavefronts), BK = 64 slices
// staged global -> registers -> LDS with two LDS stages, v_mfma_f32_32x32x16_bf16 with float32
// accumulators.  LDS rows are padded by 16 B so that the 16-byte fragment reads of 16 consecutive
// rows fall in distinct banks.
#include "faar_internal.h"

namespace faar {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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

// R = acc - C; sum R^2; dYt[n][m] = bf16(two_alpha R) (zero-padded to ldt); optional dY[m][n].
struct EpiResidual {
  const float* C;
  float two_alpha;
  bf16_t* dYt;
  int64_t ldt;
  bf16_t* dY;
  double* partials;
  float sum;
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N || m >= ldt) return;
    uint32_t b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float r = 0.0f;
      if (m + q < d.M) {
        r = acc[q] - C[(m + q) * d.N + n];
        sum += r * r;
      }
      b[q] = f32_to_bf16(two_alpha * r);
      if (dY && m + q < d.M) dY[(m + q) * d.N + n] = static_cast<bf16_t>(b[q]);
    }
    *reinterpret_cast<uint2*>(dYt + n * ldt + m) = make_uint2(b[0] | (b[1] << 16), b[2] | (b[3] << 16));
  }
  __device__ __forceinline__ void finish(int block) {
    __shared__ double s[GEMM_THREADS / 64];
    double a = static_cast<double>(sum);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o);
    if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) partials[block] = (s[0] + s[1]) + (s[2] + s[3]);
  }
};

// out[split][m][n] = acc
struct EpiF32 {
  float* out;
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int split, const GemmDims& d) {
    if (n >= d.N) return;
    float* o = out + (int64_t)split * d.M * d.N;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) o[(m + q) * d.N + n] = acc[q];
  }
  __device__ __forceinline__ void finish(int) {}
};

// C_out[m][n] = (first ? Y[m][n] : C_out[m][n]) - acc
template <bool kYbf16>
struct EpiSub {
  const void* Y;
  bool first;
  float* C_out;
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) {
        const int64_t idx = (m + q) * d.N + n;
        float y;
        if (!first) y = C_out[idx];
        else if (kYbf16) y = bf16_to_f32(static_cast<const bf16_t*>(Y)[idx]);
        else y = static_cast<const float*>(Y)[idx];
        C_out[idx] = y - acc[q];
      }
  }
  __device__ __forceinline__ void finish(int) {}
};

// out[m][n] = bf16(acc)
struct EpiBf16 {
  bf16_t* out;
  __device__ __forceinline__ void rows4(const float (&acc)[4], int64_t m, int64_t n, int, const GemmDims& d) {
    if (n >= d.N) return;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (m + q < d.M) out[(m + q) * d.N + n] = static_cast<bf16_t>(f32_to_bf16(acc[q]));
  }
  __device__ __forceinline__ void finish(int) {}
};

typedef Tile<128, 128> T128;

inline int ceil_div(int64_t a, int64_t b) { return static_cast<int>((a + b - 1) / b); }

template <class T, class Epi>
hipError_t run(const bf16_t* A, const bf16_t* B, GemmDims d, int n_split, Epi epi, hipStream_t st) {
  const int tiles_m = ceil_div(d.M, T::BM), tiles_n = ceil_div(d.N, T::BN);
  const int64_t k_per_split = round_up((d.Kd + n_split - 1) / n_split, BK);
  const dim3 grid(static_cast<unsigned>(tiles_m) * tiles_n * n_split);
  hipLaunchKernelGGL((k_gemm_nt<T, Epi>), grid, dim3(GEMM_THREADS), 0, st, A, B, d, tiles_m, tiles_n, k_per_split, epi);
  return hipGetLastError();
}

}  // namespace

int64_t gemm_residual_tiles(int64_t M, int64_t N) {
  return (int64_t)ceil_div(M, T128::BM) * ceil_div(N, T128::BN);
}

hipError_t launch_gemm_residual(const bf16_t* A, const bf16_t* B, GemmDims d, const float* C,
                                float two_alpha, bf16_t* dYt, int64_t ldt, bf16_t* dY,
                                double* mse_partials, int64_t* n_partials, hipStream_t st) {
  EpiResidual e{C, two_alpha, dYt, ldt, dY, mse_partials, 0.0f};
  *n_partials = gemm_residual_tiles(d.M, d.N);
  return run<T128>(A, B, d, 1, e, st);
}

int choose_split(int64_t M, int64_t N, int64_t Kd) {
  // enough workgroups to fill 256 compute units, but at least 512 of contraction per split
  const int64_t tiles = (int64_t)ceil_div(M, T128::BM) * ceil_div(N, T128::BN);
  int s = 1;
  while (tiles * s < 256 && Kd / (s * 2) >= 512 && s < 16) s *= 2;
  return s;
}

hipError_t launch_gemm_f32(const bf16_t* A, const bf16_t* B, GemmDims d, float* out, int n_split,
                           hipStream_t st) {
  EpiF32 e{out};
  return run<T128>(A, B, d, n_split, e, st);
}

hipError_t launch_gemm_sub(const bf16_t* A, const bf16_t* B, GemmDims d, const void* Y, bool y_bf16,
                           bool first, float* C_out, hipStream_t st) {
  if (y_bf16) {
    EpiSub<true> e{Y, first, C_out};
    return run<T128>(A, B, d, 1, e, st);
  }
  EpiSub<false> e{Y, first, C_out};
  return run<T128>(A, B, d, 1, e, st);
}

hipError_t launch_gemm_bf16(const bf16_t* A, const bf16_t* B, GemmDims d, bf16_t* out, hipStream_t st) {
  EpiBf16 e{out};
  return run<T128>(A, B, d, 1, e, st);
}

}  // namespace faar
