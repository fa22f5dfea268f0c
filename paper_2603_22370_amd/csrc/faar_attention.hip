// The attention core between the q / k / v and the output projections of a block, for a Stage-2-style joint step (paper
// Sec. 3.5 "Stage 2"; Table 2 steps 15-17 and 23: the quantised model runs forward and one loss is back-propagated into
// every layer's rounding variables).  The operations are those of the Llama3 / Qwen3 blocks the paper evaluates: rotary
// position embedding ("rotate-half" form) and causal softmax attention with grouped key / value heads, forward and
// backward.  Activations and gradients are bf16 between kernels, arithmetic is float32, products run on the matrix
// cores (v_mfma_f32_16x16x32_bf16) with the probabilities and their gradients rounded to bf16 as operands.
//
// Layouts.  q, o, dO, dq: [T, n_q * dh]; k, v, dk, dv: [T, n_kv * dh]; T = n_seq * S tokens, sequence b = rows b*S ..
// (b+1)*S-1, S a multiple of 32; query head j reads key / value head j / (n_q / n_kv).  Every product is arranged so that
// its matrix-core operands are plain row reads, with no transpose inside the kernel:
//   * a product whose contraction runs over dh reads rows of q, k, v, dO ([token][dh], dh contiguous);
//   * a product whose contraction runs over tokens (P V, dS K, P^T dO, dS^T Q) reads rows of a transposed copy
//     ([head * dh + d][token], tokens contiguous) that the entry point makes once with the library's transpose kernel;
//   * the probabilities enter those products in the accumulator layout they were computed in: an accumulator tile holds,
//     per lane, 4 consecutive rows of one column, and two such tiles side by side are exactly the 8 contraction values a
//     lane must supply as the second operand -- with the contraction index permuted, which the first operand's reads follow.
// A workgroup of four wavefronts owns 128 query positions (forward, dq) or 128 key positions (dk, dv) of one head and
// sequence, 32 per wavefront, and walks the causal range in blocks of 32 tokens whose tiles it shares through LDS (Tile
// below): letting every wavefront fetch its own operand fragments from global memory costs 16 partial cache lines per
// load instruction and was 2.5 times slower.  This part is under 5 % of a block step's flops.
#include "faar_internal.h"

namespace faar {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;

union Frag {
  bf16x8 v;
  uint4 q;
  uint2 h[2];
  uint32_t w[4];
};

__device__ __forceinline__ bf16x8 load_frag16(const bf16_t* p) {   // 8 consecutive bf16
  Frag f;
  f.q = *reinterpret_cast<const uint4*>(p);
  return f.v;
}
// 4 consecutive bf16 at p and 4 at p + 16: the contraction slots (g, 0..3) and (g, 4..7) of a 32-token step, for the
// lane group g whose accumulator rows are tokens 4g .. 4g+3 of the first and of the second 16-token tile
__device__ __forceinline__ bf16x8 load_frag_split(const bf16_t* p) {
  Frag f;
  f.h[0] = *reinterpret_cast<const uint2*>(p);
  f.h[1] = *reinterpret_cast<const uint2*>(p + 16);
  return f.v;
}
__device__ __forceinline__ bf16x8 pack_tiles(const f32x4& a, const f32x4& b) {   // two accumulator tiles -> one operand
  Frag f;
  f.w[0] = pack_bf16x2(a[0], a[1]);
  f.w[1] = pack_bf16x2(a[2], a[3]);
  f.w[2] = pack_bf16x2(b[0], b[1]);
  f.w[3] = pack_bf16x2(b[2], b[3]);
  return f.v;
}
__device__ __forceinline__ f32x4 mfma(const bf16x8& a, const bf16x8& b, const f32x4& c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float group_max(float x) {   // over the 4 lanes that share lane % 16
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float group_sum(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}
__device__ __forceinline__ void store4_bf16(bf16_t* p, const f32x4& a, float s) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(a[0] * s, a[1] * s), pack_bf16x2(a[2] * s, a[3] * s));
}

struct AttnDims {
  int S, n_q, n_kv;
  int64_t T, Tp;      // tokens, and the row pitch of the transposed copies
  float scale;        // of the scores (1 / sqrt(dh) for the models here)
};

// 2^x by the hardware instruction alone: the arguments here are at most a few units above zero and results far below one
// may flush to zero
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// o = softmax(q k^T scale, causal) v and lse = log sum exp of the scaled scores per query ([n_q][T]).
// The running maximum of a query's scores is only raised when a block exceeds it by more than 2^kLazy (the probabilities are
// then at most 2^kLazy instead of 1, harmless in float32 and bf16): the accumulators are rescaled in a branch that is
// rarely taken after the first blocks, and otherwise only matrix instructions touch them.
constexpr float kLazy = 8.0f;

// A workgroup of four wavefronts shares the keys and values of a block through LDS: its 256 threads copy the block's
// [32 keys][dh] tile of k and [dh][32 keys] tile of the transposed v global -> LDS, row-contiguous 16-byte chunks, two blocks
// ahead of their use, so the cache sees whole rows once per workgroup instead of 16 partial lines per matrix-operand load
// of every wavefront.  The 16-byte chunks of a row are stored XOR-swizzled by the row so that the operand reads (16 rows at
// the same chunk index) spread over the banks.
// 16 bytes per lane from global memory straight into LDS at lds_addr + 16 * lane (lds_addr wave-uniform).  Inline assembly:
// the compiler does not see the LDS write, so completion is tracked by hand (wait_vmcnt, then the workgroup barrier); its own
// wait counts for ordinary loads stay sufficient, since memory operations return in order.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)p));
}
#define FAAR_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N)&0xF) | (((N) >> 4) << 14))

template <int DH>
struct Tile {
  static constexpr int CPR = DH / 8;                  // 16-byte chunks per row of a [32 tokens][dh] tile
  static constexpr int RCH = 32 * CPR / 256;          // chunks of such a tile per thread
  static constexpr int CCH = DH * 4 / 256;            // chunks of a [dh][32 tokens] tile per thread (rows of 4 chunks)
  static constexpr int ELEMS = 32 * DH;               // per tile, either kind

  // [32 tokens][dh] out of a token-major tensor (rows row0 .. row0+31, columns col0 .. col0+dh-1), copied global -> LDS
  // without passing through registers: chunk i = tid + 256 j of the tile lands at byte 16 i, and holds the row's chunk
  // (i % CPR) ^ (row % CPR)
  static __device__ __forceinline__ void dma_rows(const bf16_t* __restrict__ src, int64_t row0, int64_t ld, int64_t col0,
                                                  const bf16_t* tile, int tid) {
    const uint32_t base = lds_addr_of(tile) + 16u * (static_cast<uint32_t>(tid) & ~63u);
#pragma unroll
    for (int j = 0; j < RCH; ++j) {
      const int i = tid + 256 * j, row = i / CPR, ch = (i % CPR) ^ (row % CPR);
      dma16(src + (row0 + row) * ld + col0 + ch * 8, __builtin_amdgcn_readfirstlane(base + 4096u * j));
    }
  }
  // [dh][32 tokens] out of a transposed copy: rows row0 .. row0+dh-1, columns col0 .. col0+31
  static __device__ __forceinline__ void dma_cols(const bf16_t* __restrict__ src, int64_t row0, int64_t ld, int64_t col0,
                                                  const bf16_t* tile, int tid) {
    const uint32_t base = lds_addr_of(tile) + 16u * (static_cast<uint32_t>(tid) & ~63u);
#pragma unroll
    for (int j = 0; j < CCH; ++j) {
      const int i = tid + 256 * j, row = i / 4, ch = (i % 4) ^ ((row / 4) % 4);
      dma16(src + (row0 + row) * ld + col0 + ch * 8, __builtin_amdgcn_readfirstlane(base + 4096u * j));
    }
  }
  // matrix operands out of the tiles: 16 token rows x 32 of dh (tile, dh chunk group ks) of a row tile; 16 dh rows x 32 tokens
  // of a column tile, the tokens in the slot order 4g .. 4g+3, 16+4g .. 16+4g+3
  static __device__ __forceinline__ bf16x8 row_frag(const bf16_t* t, int tile, int ks, int n, int g) {
    const int row = tile * 16 + n, ch = ks * 4 + g;
    return *reinterpret_cast<const bf16x8*>(t + row * DH + ((ch ^ (row % CPR)) * 8));
  }
  static __device__ __forceinline__ bf16x8 col_frag(const bf16_t* t, int tile, int n, int g) {
    const int row = tile * 16 + n, sw = (row / 4) % 4;
    Frag f;
    f.h[0] = *reinterpret_cast<const uint2*>(t + row * 32 + (((g / 2) ^ sw) * 8) + (g % 2) * 4);
    f.h[1] = *reinterpret_cast<const uint2*>(t + row * 32 + (((2 + g / 2) ^ sw) * 8) + (g % 2) * 4);
    return f.v;
  }
};

template <int DH>
struct FwdState {
  static constexpr int KS = DH / 32, DT = DH / 16;
  bf16x8 qf[2][KS];
  f32x4 oacc[2][DT];
  float m[2], l[2];     // reference maximum (raw score units) and this lane's share of the denominator, per query tile
};

template <int DH, bool kDiagonal>
__device__ __forceinline__ void fwd_block(FwdState<DH>& st, const bf16_t* kt_lds, const bf16_t* vt_lds, float c, int n, int g) {
  constexpr int KS = DH / 32, DT = DH / 16;
  f32x4 s[2][2];   // [query tile][key tile]: rows = keys 4g .. 4g+3 of the tile, column = query n
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    bf16x8 kf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ks] = Tile<DH>::row_frag(kt_lds, kt, ks, n, g);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      f32x4 a = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) a = mfma(kf[ks], st.qf[qt][ks], a);
      s[qt][kt] = a;
    }
  }
  float mx[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    float v = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (kDiagonal && kt * 16 + 4 * g + r > qt * 16 + n) s[qt][kt][r] = -INFINITY;   // a key after the query
        v = fmaxf(v, s[qt][kt][r]);
      }
    mx[qt] = group_max(v);   // finite: a query's own position is never masked
  }
  if (__any(mx[0] * c > st.m[0] * c + kLazy || mx[1] * c > st.m[1] * c + kLazy)) {
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      const float nm = fmaxf(st.m[qt], mx[qt]);
      const float alpha = fast_exp2((st.m[qt] - nm) * c);
      st.m[qt] = nm;
      st.l[qt] *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) st.oacc[qt][dt] *= alpha;
    }
  }
  bf16x8 pf[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const float off = -st.m[qt] * c;
    float ps = 0.0f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float p = fast_exp2(fmaf(s[qt][kt][r], c, off));
        s[qt][kt][r] = p;
        ps += p;
      }
    st.l[qt] += ps;       // this lane's keys only; the four lanes of a query add up at the end
    pf[qt] = pack_tiles(s[qt][0], s[qt][1]);
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const bf16x8 vf = Tile<DH>::col_frag(vt_lds, dt, n, g);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) st.oacc[qt][dt] = mfma(vf, pf[qt], st.oacc[qt][dt]);
  }
}

// workgroup -> (sequence, head, group of 128 query positions); wavefront w of it owns positions 32w .. 32w+31 of the group
template <int DH>
__global__ void __launch_bounds__(256, 3)
k_attn_fwd(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ Vt, AttnDims d,
           bf16_t* __restrict__ O, float* __restrict__ lse) {
  constexpr int KS = DH / 32, DT = DH / 16;
  typedef Tile<DH> Tl;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[3][2][Tl::ELEMS];   // [stage][k, v^T]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, g = lane >> 4;
  const int blocks = d.S / 32, groups = (blocks + 3) / 4;
  const int grp = blockIdx.x % groups;
  const int head = (blockIdx.x / groups) % d.n_q;
  const int64_t b = blockIdx.x / groups / d.n_q;
  const int kvh = head / (d.n_q / d.n_kv);
  const int64_t t0 = b * d.S, ldq = (int64_t)d.n_q * DH, ldk = (int64_t)d.n_kv * DH;
  const int qb = grp * 4 + wave;                   // this wavefront's block of 32 positions
  const bool active = qb < blocks;                 // the last group of a sequence may be short
  const int last = min(grp * 4 + 3, blocks - 1);   // last key block any wavefront of the group needs
  const int p0 = qb * 32;
  const float c = d.scale * kLog2e;     // scores in units of log 2

  FwdState<DH> st;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      st.qf[qt][ks] = active ? load_frag16(Q + (t0 + p0 + qt * 16 + n) * ldq + head * DH + ks * 32 + 8 * g) : bf16x8{};
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) st.oacc[qt][dt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    st.m[qt] = -INFINITY;
    st.l[qt] = 0.0f;
  }
  // Three LDS stages: a block's tiles are requested two blocks ahead (one was not enough: half of a wavefront's time went
  // into waiting), by copies that bypass the registers.  Past the last block the copies repeat it (unused).
  const int64_t kvcol = (int64_t)kvh * DH;
  constexpr int kCopies = Tl::RCH + Tl::CCH;      // per wavefront and block
#define FAAR_FWD_COPY(KB)                                            \
  do {                                                               \
    const int64_t at_ = t0 + ((KB) < last ? (KB) : last) * 32;       \
    Tl::dma_rows(K, at_, ldk, kvcol, lds[(KB) % 3][0], tid);         \
    Tl::dma_cols(Vt, kvcol, d.Tp, at_, lds[(KB) % 3][1], tid);       \
  } while (0)
  FAAR_FWD_COPY(0);
  FAAR_FWD_COPY(1);
  FAAR_WAIT_VMCNT(kCopies);                        // block 0 has landed (mine); the barrier: everybody's
  __syncthreads();
  for (int kb = 0; kb <= last; ++kb) {
    const int cur = kb % 3;
    FAAR_FWD_COPY(kb + 2);                         // into the stage read one block ago: everybody is past that barrier
    if (active) {
      if (kb < qb) fwd_block<DH, false>(st, lds[cur][0], lds[cur][1], c, n, g);
      else if (kb == qb) fwd_block<DH, true>(st, lds[cur][0], lds[cur][1], c, n, g);   // the queries' own positions
    }
    FAAR_WAIT_VMCNT(kCopies);                      // all but the copies just issued: block kb + 1 has landed
    __syncthreads();
  }
  FAAR_WAIT_VMCNT(0);                              // no copy may still be in flight into this workgroup's LDS when it retires
#undef FAAR_FWD_COPY
  if (!active) return;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const float lt = group_sum(st.l[qt]);
    const float inv = 1.0f / lt;
    const int64_t t = t0 + p0 + qt * 16 + n;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) store4_bf16(O + t * ldq + head * DH + dt * 16 + 4 * g, st.oacc[qt][dt], inv);
    if (g == 0) lse[(int64_t)head * d.T + t] = st.m[qt] * c * kLn2 + logf(lt);
  }
}

// delta[head][t] = sum_d dO[t][head, d] * O[t][head, d]  (= sum_k P dP of that query: the softmax Jacobian's second term)
template <int DH>
__global__ void __launch_bounds__(kEltThreads)
k_attn_rowdot(const bf16_t* __restrict__ dO, const bf16_t* __restrict__ O, int64_t T, int n_q, float* __restrict__ delta) {
  constexpr int LPR = DH / 8;   // lanes per (token, head): 8 or 16, a divisor of the wavefront
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;
  const int64_t row = i / LPR;      // = t * n_q + head
  float a[8], bb[8], acc = 0.0f;
  if (row < T * n_q) {
    W8<bf16_t>::load(dO + i * 8, a);
    W8<bf16_t>::load(O + i * 8, bb);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc += a[j] * bb[j];
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if (row < T * n_q && (threadIdx.x % LPR) == 0) delta[(row % n_q) * T + row / n_q] = acc;
}

// dq = scale * dS k with dS = P * (dP - delta), P = exp(scores - lse), dP = dO v^T.  Workgroups and wavefronts as in the
// forward kernel; per key block the tiles of k, v ([32 keys][dh]) and of the transposed k ([dh][32 keys]) go through LDS.
template <int DH, bool kDiagonal>
__device__ __forceinline__ void dq_block(f32x4 (&acc)[2][DH / 16], const bf16x8 (&qf)[2][DH / 32], const bf16x8 (&dof)[2][DH / 32],
                                         const float (&lse2)[2], const float (&dl)[2], const bf16_t* k_lds, const bf16_t* v_lds,
                                         const bf16_t* kt_lds, float c, int n, int g) {
  constexpr int KS = DH / 32, DT = DH / 16;
  f32x4 ds[2][2];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = Tile<DH>::row_frag(k_lds, kt, ks, n, g);
      vf[ks] = Tile<DH>::row_frag(v_lds, kt, ks, n, g);
    }
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f}, dp = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s = mfma(kf[ks], qf[qt][ks], s);
        dp = mfma(vf[ks], dof[qt][ks], dp);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float p = fast_exp2(fmaf(s[r], c, -lse2[qt]));
        if (kDiagonal && kt * 16 + 4 * g + r > qt * 16 + n) p = 0.0f;   // a key after the query
        ds[qt][kt][r] = p * (dp[r] - dl[qt]);
      }
    }
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const bf16x8 ktf = Tile<DH>::col_frag(kt_lds, dt, n, g);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) acc[qt][dt] = mfma(ktf, pack_tiles(ds[qt][0], ds[qt][1]), acc[qt][dt]);
  }
}

template <int DH>
__global__ void __launch_bounds__(256, 2)
k_attn_bwd_dq(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
              const bf16_t* __restrict__ Kt, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
              const float* __restrict__ delta, AttnDims d, bf16_t* __restrict__ dQ) {
  constexpr int KS = DH / 32, DT = DH / 16;
  typedef Tile<DH> Tl;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[3][3][Tl::ELEMS];   // [stage][k, v, k^T]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, g = lane >> 4;
  const int blocks = d.S / 32, groups = (blocks + 3) / 4;
  const int grp = blockIdx.x % groups;
  const int head = (blockIdx.x / groups) % d.n_q;
  const int64_t b = blockIdx.x / groups / d.n_q;
  const int kvh = head / (d.n_q / d.n_kv);
  const int64_t t0 = b * d.S, ldq = (int64_t)d.n_q * DH, ldk = (int64_t)d.n_kv * DH;
  const int qb = grp * 4 + wave;
  const bool active = qb < blocks;
  const int last = min(grp * 4 + 3, blocks - 1);
  const int p0 = qb * 32;
  const float c = d.scale * kLog2e;

  bf16x8 qf[2][KS], dof[2][KS];
  float lse2[2] = {0.0f, 0.0f}, dl[2] = {0.0f, 0.0f};
  f32x4 acc[2][DT];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const int64_t t = t0 + p0 + qt * 16 + n;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[qt][ks] = active ? load_frag16(Q + t * ldq + head * DH + ks * 32 + 8 * g) : bf16x8{};
      dof[qt][ks] = active ? load_frag16(dO + t * ldq + head * DH + ks * 32 + 8 * g) : bf16x8{};
    }
    if (active) {
      lse2[qt] = lse[(int64_t)head * d.T + t] * kLog2e;
      dl[qt] = delta[(int64_t)head * d.T + t];
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[qt][dt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  }
  const int64_t kvcol = (int64_t)kvh * DH;
  constexpr int kCopies = 2 * Tl::RCH + Tl::CCH;    // per wavefront and block
#define FAAR_DQ_COPY(KB)                                             \
  do {                                                               \
    const int64_t at_ = t0 + ((KB) < last ? (KB) : last) * 32;       \
    Tl::dma_rows(K, at_, ldk, kvcol, lds[(KB) % 3][0], tid);         \
    Tl::dma_rows(V, at_, ldk, kvcol, lds[(KB) % 3][1], tid);         \
    Tl::dma_cols(Kt, kvcol, d.Tp, at_, lds[(KB) % 3][2], tid);       \
  } while (0)
  FAAR_DQ_COPY(0);
  FAAR_DQ_COPY(1);
  FAAR_WAIT_VMCNT(kCopies);
  __syncthreads();
  for (int kb = 0; kb <= last; ++kb) {
    const int cur = kb % 3;
    FAAR_DQ_COPY(kb + 2);
    if (active) {
      if (kb < qb) dq_block<DH, false>(acc, qf, dof, lse2, dl, lds[cur][0], lds[cur][1], lds[cur][2], c, n, g);
      else if (kb == qb) dq_block<DH, true>(acc, qf, dof, lse2, dl, lds[cur][0], lds[cur][1], lds[cur][2], c, n, g);
    }
    FAAR_WAIT_VMCNT(kCopies);
    __syncthreads();
  }
  FAAR_WAIT_VMCNT(0);
#undef FAAR_DQ_COPY
  if (!active) return;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const int64_t t = t0 + p0 + qt * 16 + n;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) store4_bf16(dQ + t * ldq + head * DH + dt * 16 + 4 * g, acc[qt][dt], d.scale);
  }
}

// dv = P^T dO and dk = scale * dS^T q, summed over the query heads that share the key / value head.  A workgroup owns
// 64 * KT key positions of a key / value head and sequence (wavefront w: 16 * KT of them) and walks the blocks of 32 queries
// at or after them, for each query head of the group in turn; per step the tiles of q, dO ([32 queries][dh]) and of their
// transposed copies ([dh][32 queries]) go through LDS.  KT = 2 everywhere: with KT = 1 at dh = 128 two workgroups fit a compute
// unit, but every tile operand read from LDS then feeds half as many matrix instructions, and the kernel is slower (418 vs
// 360 us on 32 x 512 tokens, 16 / 8 heads).
template <int DH, int KT, bool kDiagonal>
__device__ __forceinline__ void dkv_block(f32x4 (&dk)[KT][DH / 16], f32x4 (&dv)[KT][DH / 16], const bf16x8 (&kf)[KT][DH / 32],
                                          const bf16x8 (&vf)[KT][DH / 32], const float* __restrict__ lse_q,
                                          const float* __restrict__ delta_q, const bf16_t* q_lds, const bf16_t* do_lds,
                                          const bf16_t* qt_lds, const bf16_t* dot_lds, float c, int key_minus_q0, int n, int g) {
  constexpr int KS = DH / 32, DT = DH / 16;
  f32x4 p[2][KT], ds[2][KT];    // [query tile][key tile]: rows = queries 4g .. 4g+3 of the tile, column = key n
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    bf16x8 qa[KS], da[KS];    // first operands: row = query n of the tile, contraction = dh
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qa[ks] = Tile<DH>::row_frag(q_lds, qt, ks, n, g);
      da[ks] = Tile<DH>::row_frag(do_lds, qt, ks, n, g);
    }
    const float4 l4 = *reinterpret_cast<const float4*>(lse_q + qt * 16 + 4 * g);
    const float4 d4 = *reinterpret_cast<const float4*>(delta_q + qt * 16 + 4 * g);
    const float lr[4] = {l4.x, l4.y, l4.z, l4.w}, dr[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f}, dp = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s = mfma(qa[ks], kf[kt][ks], s);
        dp = mfma(da[ks], vf[kt][ks], dp);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float pr = fast_exp2(fmaf(s[r], c, -lr[r] * kLog2e));
        // key_minus_q0 = position of this wavefront's first key relative to the block's first query
        if (kDiagonal && key_minus_q0 + kt * 16 + n > qt * 16 + 4 * g + r) pr = 0.0f;   // the key comes after the query
        p[qt][kt][r] = pr;
        ds[qt][kt][r] = pr * (dp[r] - dr[r]);
      }
    }
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const bf16x8 dotf = Tile<DH>::col_frag(dot_lds, dt, n, g);
    const bf16x8 qtf = Tile<DH>::col_frag(qt_lds, dt, n, g);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      dv[kt][dt] = mfma(dotf, pack_tiles(p[0][kt], p[1][kt]), dv[kt][dt]);
      dk[kt][dt] = mfma(qtf, pack_tiles(ds[0][kt], ds[1][kt]), dk[kt][dt]);
    }
  }
}

template <int DH, int KT>
__global__ void __launch_bounds__(256, (DH * KT <= 128 ? 2 : 1))
k_attn_bwd_dkv(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
               const bf16_t* __restrict__ Qt, const bf16_t* __restrict__ dO, const bf16_t* __restrict__ dOt,
               const float* __restrict__ lse, const float* __restrict__ delta, AttnDims d, bf16_t* __restrict__ dK,
               bf16_t* __restrict__ dV) {
  constexpr int KS = DH / 32, DT = DH / 16, WK = 16 * KT;    // WK keys per wavefront
  typedef Tile<DH> Tl;
  __shared__ __attribute__((aligned(1024))) bf16_t lds[3][4][Tl::ELEMS];   // [stage][q, dO, q^T, dO^T]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, g = lane >> 4;
  const int blocks = d.S / 32, groups = (d.S + 4 * WK - 1) / (4 * WK);
  const int grp = blockIdx.x % groups;
  const int kvh = (blockIdx.x / groups) % d.n_kv;
  const int64_t b = blockIdx.x / groups / d.n_kv;
  const int rep = d.n_q / d.n_kv;
  const int64_t t0 = b * d.S, ldq = (int64_t)d.n_q * DH, ldk = (int64_t)d.n_kv * DH;
  const int k0 = (grp * 4 + wave) * WK;          // this wavefront's first key position
  const bool active = k0 < d.S;                  // S is a multiple of 32 and WK divides 32: a wavefront is in or out as a whole
  const int first = grp * 4 * WK / 32;           // first query block any wavefront of the group needs
  const int my_first = k0 / 32;                  // ... and this wavefront
  const float c = d.scale * kLog2e;

  bf16x8 kf[KT][KS], vf[KT][KS];  // second operands: column = key n of the tile, contraction = dh
  f32x4 dk[KT][DT], dv[KT][DT];   // rows = dh 4g .. 4g+3 of the tile, column = key n
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[kt][ks] = active ? load_frag16(K + (t0 + k0 + kt * 16 + n) * ldk + kvh * DH + ks * 32 + 8 * g) : bf16x8{};
      vf[kt][ks] = active ? load_frag16(V + (t0 + k0 + kt * 16 + n) * ldk + kvh * DH + ks * 32 + 8 * g) : bf16x8{};
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      dk[kt][dt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      dv[kt][dt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
  }
  // steps: query head hj of the group (outer) x query block first .. blocks-1 (inner)
  const int per_head = blocks - first, steps = rep * per_head;
  constexpr int kCopies = 2 * Tl::RCH + 2 * Tl::CCH;    // per wavefront and step
#define FAAR_DKV_COPY(IT)                                                   \
  do {                                                                      \
    const int it_ = (IT) < steps ? (IT) : steps - 1;                        \
    const int64_t hcol_ = (int64_t)(kvh * rep + it_ / per_head) * DH;       \
    const int64_t q0_ = t0 + (first + it_ % per_head) * 32;                 \
    Tl::dma_rows(Q, q0_, ldq, hcol_, lds[(IT) % 3][0], tid);                \
    Tl::dma_rows(dO, q0_, ldq, hcol_, lds[(IT) % 3][1], tid);               \
    Tl::dma_cols(Qt, hcol_, d.Tp, q0_, lds[(IT) % 3][2], tid);              \
    Tl::dma_cols(dOt, hcol_, d.Tp, q0_, lds[(IT) % 3][3], tid);             \
  } while (0)
  FAAR_DKV_COPY(0);
  FAAR_DKV_COPY(1);
  FAAR_WAIT_VMCNT(kCopies);
  __syncthreads();
  for (int it = 0; it < steps; ++it) {
    const int cur = it % 3;
    FAAR_DKV_COPY(it + 2);                          // past the end: the last step again, unused
    const int head = kvh * rep + it / per_head, qb = first + it % per_head;
    if (active && qb >= my_first) {
      const float* lse_q = lse + (int64_t)head * d.T + t0 + qb * 32;
      const float* delta_q = delta + (int64_t)head * d.T + t0 + qb * 32;
      if (qb > my_first)
        dkv_block<DH, KT, false>(dk, dv, kf, vf, lse_q, delta_q, lds[cur][0], lds[cur][1], lds[cur][2], lds[cur][3], c, 0, n, g);
      else
        dkv_block<DH, KT, true>(dk, dv, kf, vf, lse_q, delta_q, lds[cur][0], lds[cur][1], lds[cur][2], lds[cur][3], c, k0 - qb * 32,
                                n, g);
    }
    FAAR_WAIT_VMCNT(kCopies);
    __syncthreads();
  }
  FAAR_WAIT_VMCNT(0);
#undef FAAR_DKV_COPY
  if (!active) return;
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) {
    const int64_t t = t0 + k0 + kt * 16 + n;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      store4_bf16(dK + t * ldk + kvh * DH + dt * 16 + 4 * g, dk[kt][dt], d.scale);
      store4_bf16(dV + t * ldk + kvh * DH + dt * 16 + 4 * g, dv[kt][dt], 1.0f);
    }
  }
}

// rotate-half rotary embedding of every head: pair (i, i + dh/2) by the angle whose cosine / sine are in the tables' row
// t % S; sign = -1 rotates back (the backward pass)
__global__ void __launch_bounds__(kEltThreads)
k_rope(const bf16_t* X, int64_t n_chunks, int H, int dh, const float* __restrict__ cos_t,
       const float* __restrict__ sin_t, int S, float sign, bf16_t* Y) {   // Y may be X: a thread reads what it overwrites first
  const int64_t i = blockIdx.x * (int64_t)kEltThreads + threadIdx.x;   // one 8-element chunk of a head's first half
  if (i >= n_chunks) return;
  const int cph = dh / 16;                       // chunks per half head
  const int ch = static_cast<int>(i % cph);
  const int64_t th = i / cph;                    // = t * H + head
  const int64_t t = th / H;
  const int64_t base = th * dh + ch * 8;
  const int64_t tab = (t % S) * (dh / 2) + ch * 8;
  float a[8], b[8], c[8], s[8], ya[8], yb[8];
  W8<bf16_t>::load(X + base, a);
  W8<bf16_t>::load(X + base + dh / 2, b);
  load8(cos_t + tab, c);
  load8(sin_t + tab, s);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float sj = sign * s[j];
    ya[j] = a[j] * c[j] - b[j] * sj;
    yb[j] = b[j] * c[j] + a[j] * sj;
  }
  W8<bf16_t>::store(Y + base, ya);
  W8<bf16_t>::store(Y + base + dh / 2, yb);
}

}  // namespace

hipError_t launch_rope(const bf16_t* X, int64_t T, int64_t H, int64_t dh, const float* cos_t, const float* sin_t, int64_t S,
                       bool inverse, bf16_t* Y, hipStream_t st) {
  const int64_t n_chunks = T * H * (dh / 16);
  hipLaunchKernelGGL(k_rope, dim3(static_cast<unsigned>((n_chunks + kEltThreads - 1) / kEltThreads)), dim3(kEltThreads), 0, st, X,
                     n_chunks, static_cast<int>(H), static_cast<int>(dh), cos_t, sin_t, static_cast<int>(S), inverse ? -1.0f : 1.0f, Y);
  return hipGetLastError();
}

hipError_t launch_attention_fwd(const bf16_t* Q, const bf16_t* K, const bf16_t* Vt, int64_t n_seq, int64_t S, int64_t n_q,
                                int64_t n_kv, int64_t dh, int64_t Tp, float scale, bf16_t* O, float* lse, hipStream_t st) {
  const AttnDims d{static_cast<int>(S), static_cast<int>(n_q), static_cast<int>(n_kv), n_seq * S, Tp, scale};
  const int64_t groups = n_seq * n_q * ((S / 32 + 3) / 4);    // one workgroup per 128 query positions of a head and sequence
  if (dh == 128)
    hipLaunchKernelGGL(k_attn_fwd<128>, dim3(static_cast<unsigned>(groups)), dim3(256), 0, st, Q, K, Vt, d, O, lse);
  else
    hipLaunchKernelGGL(k_attn_fwd<64>, dim3(static_cast<unsigned>(groups)), dim3(256), 0, st, Q, K, Vt, d, O, lse);
  return hipGetLastError();
}

hipError_t launch_attention_bwd(const bf16_t* dO, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* O,
                                const float* lse, const bf16_t* Qt, const bf16_t* Kt, const bf16_t* dOt, float* delta,
                                int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv, int64_t dh, int64_t Tp, float scale,
                                bf16_t* dQ, bf16_t* dK, bf16_t* dV, hipStream_t st) {
  const int64_t T = n_seq * S;
  const AttnDims d{static_cast<int>(S), static_cast<int>(n_q), static_cast<int>(n_kv), T, Tp, scale};
  const int64_t lanes = T * n_q * (dh / 8);
  const dim3 rgrid(static_cast<unsigned>((lanes + kEltThreads - 1) / kEltThreads));
  const unsigned gq = static_cast<unsigned>(n_seq * n_q * ((S / 32 + 3) / 4));
  const unsigned gk = static_cast<unsigned>(n_seq * n_kv * ((S + 127) / 128));
  if (dh == 128) {
    hipLaunchKernelGGL(k_attn_rowdot<128>, rgrid, dim3(kEltThreads), 0, st, dO, O, T, static_cast<int>(n_q), delta);
    hipLaunchKernelGGL(k_attn_bwd_dq<128>, dim3(gq), dim3(256), 0, st, Q, K, V, Kt, dO, lse, delta, d, dQ);
    hipLaunchKernelGGL((k_attn_bwd_dkv<128, 2>), dim3(gk), dim3(256), 0, st, Q, K, V, Qt, dO, dOt, lse, delta, d, dK, dV);
  } else {
    hipLaunchKernelGGL(k_attn_rowdot<64>, rgrid, dim3(kEltThreads), 0, st, dO, O, T, static_cast<int>(n_q), delta);
    hipLaunchKernelGGL(k_attn_bwd_dq<64>, dim3(gq), dim3(256), 0, st, Q, K, V, Kt, dO, lse, delta, d, dQ);
    hipLaunchKernelGGL((k_attn_bwd_dkv<64, 2>), dim3(gk), dim3(256), 0, st, Q, K, V, Qt, dO, dOt, lse, delta, d, dK, dV);
  }
  return hipGetLastError();
}

}  // namespace faar
