// extern "C" entry points of libfaar (declared and documented in include/faar.h): argument
// validation, workspace carving and kernel sequencing.  Nothing here allocates device memory or synchronises.
#include <cmath>
#include <mutex>
#include <vector>

#include "../../include/faar.h"
#include "faar_internal.h"

using namespace faar;

// ---- scratch memory that lives in the code object, for faar_softquant_fwd_bwd_static ----
// One double per block of the backward kernel (kEltThreads lanes x 8 weights each), for tensors of up to
// kStaticMaxWeights weights.  Every GPU the library runs on holds its own copy of the array at its own address
// until the process ends; the address is looked up once per device, with that device current, and kept
// (static_scratch below).  Kernels receive that address as an argument like any other buffer.
constexpr int64_t kStaticMaxWeights = (int64_t)1 << 27;
constexpr int64_t kStaticPartials = kStaticMaxWeights / (8 * kEltThreads);   // 65536 doubles = 512 KB
static __device__ __align__(256) double scratch[kStaticPartials];

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_status(hipError_t e) {
  if (e == hipSuccess) return FAAR_OK;
  g_last_hip_error = static_cast<int>(e);
  return FAAR_E_HIP;
}

// Optional event bracket around one kernel of the path (faar_time_kernel).
struct Probe { int which = FAAR_K_NONE; std::vector<hipEvent_t> events; int64_t count = 0; };   // events: start 0, stop 0, ...
thread_local Probe g_probe;
struct Bracket {
  bool on;
  hipStream_t st;
  hipEvent_t stop;
  Bracket(int id, hipStream_t s) : on(g_probe.which == id), st(s), stop(nullptr) {
    if (!on) return;
    const size_t pair = static_cast<size_t>(g_probe.count++) % (g_probe.events.size() / 2);
    stop = g_probe.events[2 * pair + 1];
    (void)hipEventRecord(g_probe.events[2 * pair], st);
  }
  ~Bracket() { if (on) (void)hipEventRecord(stop, st); }
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

// Largest tensor / activation extents accepted: index arithmetic is 64-bit, grids are 32-bit.
constexpr int64_t kMaxElems = (int64_t)1 << 36;

int check_shape(int64_t O, int64_t K) {
  if (O <= 0 || K <= 0 || K % 16 != 0) return FAAR_E_SHAPE;
  if (O > kMaxElems / K) return FAAR_E_SHAPE;
  return FAAR_OK;
}
int check_wdt(faar_dtype dt) { return (dt == FAAR_F32 || dt == FAAR_BF16) ? FAAR_OK : FAAR_E_DTYPE; }

// Carves 256-byte aligned regions out of the caller's workspace.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <typename T> T* take(size_t count) {
    T* r = reinterpret_cast<T*>(base + off);
    off += align256(count * sizeof(T));
    return r;
  }
};

struct StepLayout {
  size_t guard, delta, dYt, G, mse_partials, round_partials, cross_partials, wq_full, wqt, dY, total;
  int n_split;
  int64_t Tp, Op;
};

StepLayout step_layout(int64_t O, int64_t K, int64_t T, bool chained) {
  StepLayout L{};
  L.Tp = padded_tokens(T);
  L.Op = round_up(O, 64);
  L.n_split = choose_split(O, K, L.Tp);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off += align256(bytes); return r; };
  L.guard = take((size_t)(kTagWords + 1) * 4);  // first, so that every user of a step workspace finds it
  L.delta = take((size_t)O * K * 2);
  L.dYt = take((size_t)O * L.Tp * 2);
  L.G = take((size_t)L.n_split * O * K * 4);
  L.mse_partials = take((size_t)gemm_residual_partials(T, O, K) * 8);
  L.round_partials = take((size_t)2 * kStepBwdMaxBlocks * 8);  // two sets: steps of even / odd index
  L.cross_partials = take((size_t)2 * kStepBwdMaxBlocks * 8);  // likewise; used when the layer carries H
  if (chained) {
    L.wq_full = take((size_t)O * K * 2);
    L.wqt = take((size_t)K * L.Op * 2);
    L.dY = take((size_t)T * O * 2);
  }
  L.total = off;
  return L;
}

// Workspace of faar_layer_step_gram: the guard first, as in every step workspace
struct GramLayout {
  size_t guard, delta, G, mse_partials, round_partials, cross_partials, total;
  int n_split;
};

GramLayout gram_layout(int64_t O, int64_t K) {
  GramLayout L{};
  L.n_split = choose_split_gram(O, K);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off += align256(bytes); return r; };
  L.guard = take((size_t)(kTagWords + 1) * 4);
  L.delta = take((size_t)O * K * 2);
  L.G = take((size_t)L.n_split * O * K * 4);
  L.mse_partials = take((size_t)gemm_gram_partials(O, K) * 8);
  L.round_partials = take((size_t)2 * kStepBwdMaxBlocks * 8);
  L.cross_partials = take((size_t)2 * kStepBwdMaxBlocks * 8);
  L.total = off;
  return L;
}

// Tag of the forward pass "W_q - W (and W_q when dX is wanted) of step t of this layer at this beta".
ForwardTag forward_tag(int32_t t, float beta, const void* V, const void* W, const void* scales, int64_t n, bool with_wq,
                       const void* H) {
  ForwardTag g{};
  uint32_t bits;
  static_assert(sizeof(bits) == sizeof(beta), "float is 32 bits");
  __builtin_memcpy(&bits, &beta, sizeof(bits));
  auto lo = [](uint64_t x) { return static_cast<uint32_t>(x); };
  auto hi = [](uint64_t x) { return static_cast<uint32_t>(x >> 32); };
  const uint64_t v = reinterpret_cast<uintptr_t>(V), w = reinterpret_cast<uintptr_t>(W), s = reinterpret_cast<uintptr_t>(scales);
  g.w[0] = 0xFAA2F0D1u;
  g.w[1] = static_cast<uint32_t>(t);
  g.w[2] = bits;
  g.w[3] = lo(v); g.w[4] = hi(v);
  g.w[5] = lo(w); g.w[6] = hi(w);
  g.w[7] = lo(s); g.w[8] = hi(s);
  g.w[9] = lo(static_cast<uint64_t>(n)); g.w[10] = hi(static_cast<uint64_t>(n));
  // with H the forward also left the loss's cross term <delta, H>: fold H's address in
  g.w[11] = (with_wq ? 1u : 0u) | (H ? 2u : 0u) | (lo(reinterpret_cast<uintptr_t>(H)) & ~3u);
  g.w[9] ^= hi(reinterpret_cast<uintptr_t>(H));
  return g;
}

// ---- soft quantisation forward / backward, shared by the two entry points that differ in where the per-block
// Round-Loss partial sums live ----
int softquant_check(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global, const uint8_t* scales,
                    const float* V, float beta, void* Wt, const float* dWt, float lambda_round, float* dV, uint32_t flags) {
  if (!W || !s_global || !scales || !V || !Wt) return FAAR_E_NULL;
  if (dWt && !dV) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (flags & ~(uint32_t)FAAR_EMIT_DELTA) return FAAR_E_ARG;
  if (!(beta > 0.0f) || !std::isfinite(beta) || !std::isfinite(lambda_round)) return FAAR_E_ARG;
  if (!aligned16(W) || !aligned16(V) || !aligned16(Wt) || !aligned16(dWt) || !aligned16(dV)) return FAAR_E_ARG;
  return FAAR_OK;
}

int softquant_run(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global, const uint8_t* scales,
                  const float* V, float beta, void* Wt, const float* dWt, float lambda_round, float* dV, float* round_loss,
                  uint32_t flags, double* partials, hipStream_t st) {
  const bool bf = wdt == FAAR_BF16;
  const int64_t n = O * K;
  if (int e = hip_status(launch_softquant_fwd(W, bf, n, s_global, scales, V, beta, (flags & FAAR_EMIT_DELTA) != 0,
                                              static_cast<bf16_t*>(Wt), nullptr, st)))
    return e;
  if (!dWt) return FAAR_OK;
  if (int e = hip_status(launch_softquant_bwd(W, bf, n, s_global, scales, V, beta, dWt, 1, 0, lambda_round, dV,
                                              partials, st)))
    return e;
  if (round_loss)
    return hip_status(launch_finalize_losses(nullptr, 0, 0.0f, partials, softquant_bwd_blocks(n), 1.0 / (double)n,
                                             lambda_round, nullptr, round_loss, nullptr, st));
  return FAAR_OK;
}

// The address of `scratch` (declared at file scope above) on the current device.  In host code the array's name is
// only a handle for this lookup, never a device address.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(double** out) {
  int dev = -1;
  if (int e = hip_status(hipGetDevice(&dev))) return e;
  if (dev < 0 || dev >= kMaxDevices) return FAAR_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (int e = hip_status(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)))) return e;
    if (!p) return FAAR_E_HIP;
    g_scratch_ptr[dev] = static_cast<double*>(p);
  }
  *out = g_scratch_ptr[dev];
  return FAAR_OK;
}

}  // namespace

extern "C" {

int faar_version(void) { return 100; }

int faar_last_hip_error(void) { return g_last_hip_error; }

int faar_time_kernel(int which, void* start_event, void* stop_event) {
  if (which < FAAR_K_NONE || which > FAAR_K_GEMM_GRAM || which == FAAR_K_GEMM_C) return FAAR_E_ARG;  // FAAR_K_GEMM_C has no bracket
  if (which != FAAR_K_NONE && (!start_event || !stop_event)) return FAAR_E_ARG;
  void* const pair[2] = {start_event, stop_event};
  return faar_time_kernel_ring(which, pair, 1);
}

int faar_time_kernel_ring(int which, void* const* events, int n) {
  if (which < FAAR_K_NONE || which > FAAR_K_GEMM_GRAM || which == FAAR_K_GEMM_C) return FAAR_E_ARG;
  g_probe.which = FAAR_K_NONE;
  g_probe.events.clear();
  g_probe.count = 0;
  if (which == FAAR_K_NONE) return FAAR_OK;
  if (!events || n < 1 || n > 4096) return FAAR_E_ARG;
  for (int i = 0; i < 2 * n; ++i)
    if (!events[i]) return FAAR_E_ARG;
  for (int i = 0; i < 2 * n; ++i) g_probe.events.push_back(static_cast<hipEvent_t>(events[i]));
  g_probe.which = which;
  return FAAR_OK;
}

int64_t faar_time_kernel_count(void) { return g_probe.count; }

int faar_dw_split(int64_t O, int64_t K, int64_t T) {
  if (check_shape(O, K) != FAAR_OK || T <= 0) return 0;
  return choose_split(O, K, padded_tokens(T));
}

int64_t faar_padded_tokens(int64_t T) { return T > 0 ? padded_tokens(T) : 0; }

int faar_dw_token_major(int64_t O, int64_t K, int64_t T, uint32_t flags) {
  if (check_shape(O, K) != FAAR_OK || T <= 0) return 0;
  return gemm_tn_tiles(O, K, T, (flags & FAAR_STEP_WHOLE_DEVICE) != 0);
}

int faar_gemm_probe(int mode, int64_t M, int64_t N, int64_t Kd, const void* A, const void* B,
                    unsigned long long* clocks, int64_t capacity, float* sink, int32_t* info, void* stream) {
  if (!A || !B || !clocks || !sink || !info) return FAAR_E_NULL;
  if (mode < 0 || mode > 12 || (mode & 3) == 3) return FAAR_E_ARG;
  if (M <= 0 || N <= 0 || Kd <= 0 || Kd % 64 != 0 || M > kMaxElems / Kd || N > kMaxElems / Kd) return FAAR_E_SHAPE;
  if (!aligned16(A) || !aligned16(B) || (reinterpret_cast<uintptr_t>(clocks) & 7u)) return FAAR_E_ARG;
  int kind = 0;
  int64_t items = 0;
  const hipError_t e = launch_gemm_probe(mode, static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(B),
                                         GemmDims{M, N, Kd, Kd, Kd}, clocks, capacity, sink, &kind, &items,
                                         static_cast<hipStream_t>(stream));
  info[0] = static_cast<int32_t>(items);
  info[1] = kind;
  if (e == hipErrorNotSupported) return FAAR_E_UNSUPPORTED;
  if (e == hipErrorInvalidValue) return FAAR_E_WORKSPACE;
  return hip_status(e);
}

int faar_gemm_plan(int which, int64_t O, int64_t K, int64_t T, int32_t* out) {
  if (!out) return FAAR_E_NULL;
  if (int e = check_shape(O, K)) return e;
  if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return FAAR_E_SHAPE;
  GemmPlanInfo p{};
  switch (which) {
    case FAAR_K_GEMM_RESIDUAL: p = gemm_plan_info(kGemmEpiResidual, T, O, K); break;
    case FAAR_K_GEMM_DW: p = gemm_plan_info(kGemmEpiF32, O, K, padded_tokens(T)); break;
    case FAAR_K_GEMM_DX: p = gemm_plan_info(kGemmEpiBf16, T, K, O); break;
    case FAAR_K_GEMM_C: p = gemm_plan_info(kGemmEpiSub, T, O, K); break;
    case FAAR_K_GEMM_FWD: p = gemm_plan_info(kGemmEpiBf16, T, O, K); break;
    case FAAR_K_GEMM_GRAM: p = gemm_plan_info(kGemmEpiGram, O, K, K); break;
    default: return FAAR_E_ARG;
  }
  out[0] = p.kind; out[1] = p.bm; out[2] = p.bn; out[3] = p.n_split;
  return FAAR_OK;
}

size_t faar_workspace_bytes(int op, int64_t O, int64_t K, int64_t T, uint32_t flags) {
  if (op == FAAR_OP_STAGE2_LOSSES) {  // O = vocabulary size, K = hidden size, T = tokens
    if (T <= 0 || O <= 0 || K <= 0 || T > kMaxElems / K) return 0;
    return align256((size_t)T * sizeof(double)) + align256((size_t)stage2_mse_blocks(T * K) * sizeof(double));
  }
  if (check_shape(O, K) != FAAR_OK) return 0;
  switch (op) {
    case FAAR_OP_QUANT_RTN:
      return align256(kAmaxPartials * sizeof(float));
    case FAAR_OP_LINEAR_FORWARD:
      return align256((size_t)O * K * 2);   // W_q in bf16
    case FAAR_OP_ATTENTION_FWD:             // O = n_q * dh, K = n_kv * dh: V transposed
      if (T <= 0) return 0;
      return align256((size_t)K * (padded_tokens(T) + 64) * 2);
    case FAAR_OP_ATTENTION_BWD:             // Q, dO, K transposed; one float per head and query (at most O / 64 heads)
      if (T <= 0) return 0;
      return align256((size_t)O * (padded_tokens(T) + 64) * 2) * 2 + align256((size_t)K * (padded_tokens(T) + 64) * 2) +
             align256((size_t)(O / 64) * T * sizeof(float));
    case FAAR_OP_BLOCK_OUTPUT_LOSS:         // O = D (row length), T rows
      if (T <= 0 || O % 8 != 0) return 0;
      return align256((size_t)block_loss_blocks(T * O) * sizeof(double));
    case FAAR_OP_QUANT_RTN_BATCH:   // whatever the number and sizes of the tensors: launches reuse it in stream order
      return align256((size_t)kBatchMax * kBatchAmaxBlocks * sizeof(float));
    case FAAR_OP_INIT_V:
    case FAAR_OP_HARDEN_PACK:
      return 256;  // none needed; a non-zero size keeps callers' allocation code uniform
    case FAAR_OP_SOFTQUANT:
      return align256((size_t)softquant_bwd_blocks(O * K) * sizeof(double));
    case FAAR_OP_LAYER_PREPARE: {
      if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return 0;
      size_t need = 3 * align256((size_t)O * K * 2);  // hi/mid/lo bf16 terms of a float32 W
      if (flags & FAAR_WS_GRADIENT_CONSTANT) {        // one bf16 term of C^T, the partial products, sums of C^2
        const int64_t Tp = padded_tokens(T);
        const size_t h = align256((size_t)O * Tp * 2) + align256((size_t)choose_split(O, K, Tp) * O * K * 4) +
                         align256((size_t)c_term_blocks(T, O) * 8);
        need = need > h ? need : h;
      }
      return need;
    }
    case FAAR_OP_LAYER_STEP:
      if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return 0;
      return step_layout(O, K, T, (flags & FAAR_WS_CHAINED) != 0).total;
    case FAAR_OP_GRAM_PREPARE:              // the split partial products of the K x K matrix
      if (T <= 0 || T > kMaxElems / K || K > kMaxElems / K) return 0;
      return align256((size_t)choose_split(K, K, padded_tokens(T)) * K * K * 4);
    case FAAR_OP_LAYER_STEP_GRAM:
      return gram_layout(O, K).total;
    default:
      return 0;
  }
}

int faar_quant_rtn(const void* W, faar_dtype wdt, int64_t O, int64_t K, float* s_global,
                   uint8_t* scales, uint8_t* codes, void* W_dq, uint32_t flags, void* ws,
                   size_t ws_bytes, void* stream) {
  if (!W || !s_global || !scales || !codes) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (flags & ~(uint32_t)(FAAR_SGLOBAL_GIVEN | FAAR_DQ_IN_UNITS)) return FAAR_E_ARG;
  if (!aligned16(W) || !aligned16(codes) || !aligned16(W_dq) || (reinterpret_cast<uintptr_t>(s_global) & 3u))
    return FAAR_E_ARG;
  const bool given = (flags & FAAR_SGLOBAL_GIVEN) != 0;
  if (!given && (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_QUANT_RTN, O, K, 0, flags))) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = wdt == FAAR_BF16;
  if (!given)
    if (int e = hip_status(launch_amax(W, bf, O * K, static_cast<float*>(ws), s_global, st))) return e;
  Bracket b(FAAR_K_QUANT_RTN, st);
  return hip_status(launch_quant_rtn(W, bf, O * K, s_global, scales, codes, W_dq, (flags & FAAR_DQ_IN_UNITS) != 0, st));
}

int faar_init_v(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                const uint8_t* scales, float* V, uint8_t* floor_codes, void* stream) {
  if (!W || !s_global || !scales || !V) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (!aligned16(W) || !aligned16(V) || !aligned16(floor_codes)) return FAAR_E_ARG;
  Bracket b(FAAR_K_INIT_V, static_cast<hipStream_t>(stream));
  return hip_status(launch_init_v(W, wdt == FAAR_BF16, O * K, s_global, scales, V, floor_codes,
                                  static_cast<hipStream_t>(stream)));
}

// ---- batched codec entry points -----------------------------------------------------------------------------------
static int codec_batch(int op, const faar_tensor* items, int64_t n_items, faar_dtype wdt, uint32_t flags, void* ws,
                       size_t ws_bytes, void* stream) {
  if (!items) return FAAR_E_NULL;
  if (n_items <= 0 || n_items > (1 << 20)) return FAAR_E_SHAPE;
  if (int e = check_wdt(wdt)) return e;
  const bool given = (flags & FAAR_SGLOBAL_GIVEN) != 0;
  if (flags & ~(uint32_t)(op == kBatchQuant ? FAAR_SGLOBAL_GIVEN : 0)) return FAAR_E_ARG;
  for (int64_t k = 0; k < n_items; ++k) {   // validate everything before the first launch
    const faar_tensor& t = items[k];
    if (!t.W || !t.s_global || !t.scales) return FAAR_E_NULL;
    if (op != kBatchInitV && !t.codes) return FAAR_E_NULL;
    if (op != kBatchQuant && !t.V) return FAAR_E_NULL;
    if (t.n <= 0 || t.n % 16 != 0 || t.n > kMaxElems) return FAAR_E_SHAPE;
    if (!aligned16(t.W) || !aligned16(t.V) || !aligned16(t.codes) || (reinterpret_cast<uintptr_t>(t.s_global) & 3u))
      return FAAR_E_ARG;
  }
  const bool need_ws = op == kBatchQuant && !given;
  if (need_ws && (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_QUANT_RTN_BATCH, 16, 16, 0, 0))) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // A launch takes up to kBatchMax tensors and at most 2^31 - 1 workgroups.  (Cutting the two-pass quantisation's launches
  // at ~100 MB of weights, so that the second pass would find them in the last-level cache, was measured: the extra
  // launches cost more than the cache gives back, 2.4 against 1.5 ms on the 1.4 G-weight sweep.)
  int64_t k = 0;
  while (k < n_items) {
    CodecBatch B{};
    int64_t blocks = 0;
    int j = 0;
    for (; j < kBatchMax && k < n_items; ++j, ++k) {
      const faar_tensor& t = items[k];
      const int64_t tb = (t.n / 8 + kEltThreads - 1) / kEltThreads;
      if (j > 0 && blocks + tb > 0x7FFFFFFFll) break;
      if (tb > 0x7FFFFFFFll) return FAAR_E_SHAPE;   // unreachable below kMaxElems; kept next to the limit it protects
      B.first_block[j] = static_cast<uint32_t>(blocks);
      B.it[j] = CodecItem{t.W, t.s_global, t.scales, t.V, reinterpret_cast<uint32_t*>(t.codes), t.n / 8};
      blocks += tb;
    }
    B.n = j;
    B.first_block[j] = static_cast<uint32_t>(blocks);
    if (int e = hip_status(launch_codec_batch(op, B, wdt == FAAR_BF16, given, static_cast<float*>(ws), st))) return e;
  }
  return FAAR_OK;
}

int faar_quant_rtn_batch(const faar_tensor* items, int64_t n_items, faar_dtype wdt, uint32_t flags, void* ws,
                         size_t ws_bytes, void* stream) {
  return codec_batch(kBatchQuant, items, n_items, wdt, flags, ws, ws_bytes, stream);
}

int faar_init_v_batch(const faar_tensor* items, int64_t n_items, faar_dtype wdt, void* stream) {
  return codec_batch(kBatchInitV, items, n_items, wdt, 0, nullptr, 0, stream);
}

int faar_harden_pack_batch(const faar_tensor* items, int64_t n_items, faar_dtype wdt, void* stream) {
  return codec_batch(kBatchHardenPack, items, n_items, wdt, 0, nullptr, 0, stream);
}

int faar_softquant_fwd_bwd(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                           const uint8_t* scales, const float* V, float beta, void* Wt,
                           const float* dWt, float lambda_round, float* dV, float* round_loss,
                           uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
  if (int e = softquant_check(W, wdt, O, K, s_global, scales, V, beta, Wt, dWt, lambda_round, dV, flags)) return e;
  if (dWt && (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_SOFTQUANT, O, K, 0, flags))) return FAAR_E_WORKSPACE;
  return softquant_run(W, wdt, O, K, s_global, scales, V, beta, Wt, dWt, lambda_round, dV, round_loss, flags,
                       static_cast<double*>(ws), static_cast<hipStream_t>(stream));
}

int faar_softquant_fwd_bwd_static(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                                  const uint8_t* scales, const float* V, float beta, void* Wt,
                                  const float* dWt, float lambda_round, float* dV, float* round_loss,
                                  uint32_t flags, void* stream) {
  if (int e = softquant_check(W, wdt, O, K, s_global, scales, V, beta, Wt, dWt, lambda_round, dV, flags)) return e;
  if (O * K > kStaticMaxWeights) return FAAR_E_SHAPE;  // the resident partial-sum array holds no more blocks
  double* partials = nullptr;
  if (dWt)
    if (int e = static_scratch(&partials)) return e;
  return softquant_run(W, wdt, O, K, s_global, scales, V, beta, Wt, dWt, lambda_round, dV, round_loss, flags, partials,
                       static_cast<hipStream_t>(stream));
}

int faar_layer_prepare(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                       const uint8_t* scales, const void* Xq, const float* x_scale, const void* Y_fp, faar_dtype ydt,
                       int64_t T, void* Xt, float* C, uint8_t* icodes, float* H, double* c_norm2, void* ws, size_t ws_bytes,
                       void* stream) {
  if (!W || !s_global || !scales || !Xq || !Xt || !icodes) return FAAR_E_NULL;
  if ((Y_fp != nullptr) != (C != nullptr)) return FAAR_E_NULL;   // no reference output: only Xt and the interval codes
  if (!Y_fp && H) return FAAR_E_NULL;
  if ((H != nullptr) != (c_norm2 != nullptr)) return FAAR_E_NULL;
  if (!aligned16(H) || (reinterpret_cast<uintptr_t>(c_norm2) & 7u)) return FAAR_E_ARG;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_wdt(ydt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return FAAR_E_SHAPE;
  if (!aligned16(W) || !aligned16(Xq) || !aligned16(Y_fp) || !aligned16(Xt) || !aligned16(C) || !aligned16(icodes))
    return FAAR_E_ARG;
  const bool bf = wdt == FAAR_BF16;
  if (((!bf && Y_fp) || H) &&
      (!ws || !aligned16(ws) || ws_bytes < faar_workspace_bytes(FAAR_OP_LAYER_PREPARE, O, K, T, H ? FAAR_WS_GRADIENT_CONSTANT : 0)))
    return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bf16_t* xq = static_cast<const bf16_t*>(Xq);
  const int64_t Tp = padded_tokens(T);
  if (int e = hip_status(launch_interval_codes(W, bf, O * K, s_global, scales, icodes, st))) return e;
  if (int e = hip_status(launch_transpose_bf16(xq, T, K, static_cast<bf16_t*>(Xt), Tp, st))) return e;
  if (!Y_fp) return FAAR_OK;
  const GemmDims d{T, O, K, K, K};
  if (bf) {
    if (int e = hip_status(launch_gemm_sub(xq, static_cast<const bf16_t*>(W), d, Y_fp, ydt == FAAR_BF16, true, C, x_scale, st)))
      return e;
  } else {
    Carver cv(ws);
    bf16_t* term[3];
    for (auto& t : term) t = cv.take<bf16_t>((size_t)O * K);
    if (int e = hip_status(launch_split_f32(static_cast<const float*>(W), O * K, term[0], term[1], term[2], st))) return e;
    for (int i = 0; i < 3; ++i)
      if (int e = hip_status(launch_gemm_sub(xq, term[i], d, Y_fp, ydt == FAAR_BF16, i == 0, C, x_scale, st))) return e;
  }
  if (!H) return FAAR_OK;
  // H = C^T Xq (the activations as stored, i.e. in units of x_scale): C is split into three bf16 terms, each
  // transposed into the operand layout of the dW GEMM and multiplied with Xt on the matrix cores (exact products,
  // float32 accumulation); the terms' partial products are summed into H.  ||C||^2 comes from the first pass over C.
  Carver cv(ws);   // the float32-W terms above are no longer needed
  bf16_t* ct = cv.take<bf16_t>((size_t)O * Tp);
  const int n_split = choose_split(O, K, Tp);
  float* part = cv.take<float>((size_t)n_split * O * K);
  double* sq = cv.take<double>((size_t)c_term_blocks(T, O));
  const GemmDims d2{O, K, Tp, Tp, Tp};
  for (int term = 0; term < 3; ++term) {
    if (int e = hip_status(launch_c_term_transposed(C, T, O, term, ct, Tp, term == 0 ? sq : nullptr, st))) return e;
    if (int e = hip_status(launch_gemm_f32(ct, static_cast<const bf16_t*>(Xt), d2, part, n_split, st))) return e;
    if (int e = hip_status(launch_accumulate_partials(H, part, n_split, (int64_t)O * K, O * K, term == 0, st))) return e;
  }
  return hip_status(launch_sum_doubles(sq, c_term_blocks(T, O), c_norm2, st));
}

int faar_layer_step(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                    const uint8_t* scales, float* V, float* adam_m, float* adam_v, const void* Xq, const float* x_scale,
                    const void* Xt, const float* C, const uint8_t* icodes, const float* H, const double* c_norm2,
                    int64_t T, const void* dY_ext, void* dX,
                    float beta, float beta_next, float lambda_round, float mse_scale, const faar_adam* opt,
                    float* losses, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
  const bool joint = (flags & FAAR_STEP_JOINT) != 0;
  if (!W || !s_global || !scales || !V || !adam_m || !adam_v || !Xq || !Xt || (!C && !joint) || !icodes || !opt || !losses)
    return FAAR_E_NULL;
  if (joint && (!dY_ext || H)) return FAAR_E_ARG;   // the loss lives outside the layer: its gradient must be given
  if ((H != nullptr) != (c_norm2 != nullptr)) return FAAR_E_NULL;
  if (!aligned16(H) || (reinterpret_cast<uintptr_t>(c_norm2) & 7u)) return FAAR_E_ARG;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return FAAR_E_SHAPE;
  const bool chained = dY_ext || dX;
  if (chained && O % 8 != 0) return FAAR_E_SHAPE;
  if (flags & ~(uint32_t)(FAAR_WS_CHAINED | FAAR_WS_FORWARD_READY | FAAR_STEP_JOINT | FAAR_STEP_XT_READY | FAAR_STEP_WHOLE_DEVICE))
    return FAAR_E_ARG;
  if ((flags & FAAR_STEP_XT_READY) && !joint) return FAAR_E_ARG;
  if (!(beta > 0.0f) || !std::isfinite(beta) || !std::isfinite(lambda_round) || !std::isfinite(mse_scale))
    return FAAR_E_ARG;
  if (!(beta_next >= 0.0f) || !std::isfinite(beta_next)) return FAAR_E_ARG;
  if (!(opt->lr >= 0.0f) || !std::isfinite(opt->lr) || !(opt->beta1 >= 0.0f && opt->beta1 < 1.0f) ||
      !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) || !(opt->eps >= 0.0f) || !std::isfinite(opt->eps) || opt->t < 1)
    return FAAR_E_ARG;
  if (!aligned16(W) || !aligned16(V) || !aligned16(adam_m) || !aligned16(adam_v) || !aligned16(Xq) ||
      !aligned16(Xt) || !aligned16(C) || !aligned16(icodes) || !aligned16(dY_ext) || !aligned16(dX) || !aligned16(ws))
    return FAAR_E_ARG;
  const StepLayout L = step_layout(O, K, T, chained);
  if (!ws || ws_bytes < L.total) return FAAR_E_WORKSPACE;

  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = wdt == FAAR_BF16;
  const int64_t n = O * K;
  char* base = static_cast<char*>(ws);
  bf16_t* delta = reinterpret_cast<bf16_t*>(base + L.delta);
  bf16_t* dYt = reinterpret_cast<bf16_t*>(base + L.dYt);
  float* G = reinterpret_cast<float*>(base + L.G);
  double* mse_p = reinterpret_cast<double*>(base + L.mse_partials);
  // Round-Loss partials of the V a step starts from: set t % 2, so that a step which also prepares the
  // next one writes the other set while its last block reads this one
  double* round_p = reinterpret_cast<double*>(base + L.round_partials) + (opt->t & 1) * kStepBwdMaxBlocks;
  double* round_next = reinterpret_cast<double*>(base + L.round_partials) + ((opt->t + 1) & 1) * kStepBwdMaxBlocks;
  double* cross_p = reinterpret_cast<double*>(base + L.cross_partials) + (opt->t & 1) * kStepBwdMaxBlocks;
  double* cross_next = reinterpret_cast<double*>(base + L.cross_partials) + ((opt->t + 1) & 1) * kStepBwdMaxBlocks;
  // The constant part of the gradient is carried separately when the caller provides it -- unless dX has to come
  // from the locally derived dY, which then must contain the constant
  const float* Hs = (H && !(dX && !dY_ext)) ? H : nullptr;
  bf16_t* wq_full = chained && dX ? reinterpret_cast<bf16_t*>(base + L.wq_full) : nullptr;
  bf16_t* wqt = chained ? reinterpret_cast<bf16_t*>(base + L.wqt) : nullptr;
  bf16_t* dY = chained ? reinterpret_cast<bf16_t*>(base + L.dY) : nullptr;
  const bf16_t* xq = static_cast<const bf16_t*>(Xq);

  // s1: W_q - W (bf16), W_q itself when dX is wanted, Round-Loss partials -- unless the previous step left them,
  // in which case the residual GEMM first checks that what the workspace holds is this step's forward
  uint32_t* guard_slot = reinterpret_cast<uint32_t*>(base + L.guard);
  ForwardGuard guard{nullptr, {}};
  if (!(flags & FAAR_WS_FORWARD_READY)) {
    Bracket b(FAAR_K_SOFTQUANT_FWD, st);
    if (int e = hip_status(launch_step_fwd(W, bf, n, s_global, scales, icodes, V, beta, delta, wq_full, round_p, guard_slot, Hs,
                                           cross_p, st)))
      return e;
  } else {
    guard.slot = guard_slot;
    guard.expect = forward_tag(opt->t, beta, V, W, scales, n, wq_full != nullptr, Hs);
  }
  // s2: residual GEMM + loss + dY -- not in a joint step, whose loss is computed downstream of the layer; there the
  // activations change from step to step, so their transpose for the dW GEMM is refreshed here
  int64_t n_mse = 0;
  const GemmDims d1{T, O, K, K, K};
  const bool need_local_dY = dX && !dY_ext;
  // An upstream gradient arrives token-major, as the activations are: where the token-major form of the dW GEMM applies, it
  // takes both as they are -- no dY^T, and X_q^T is neither read nor (in a joint step) written
  const bool token_major = dY_ext && gemm_tn_usable(O, K, T);
  // ... and so does the step's own gradient when the constant is carried separately (nothing but the GEMM's product goes
  // into dY then) and no dX has to be derived from it
  const bool rows_form = !joint && Hs && !dY_ext && !dX && gemm_tn_usable(O, K, T);
  if (joint) {
    if (flags & FAAR_WS_FORWARD_READY) {   // nobody else consumes the tag: check it in a kernel of its own
      if (int e = hip_status(launch_check_forward_tag(guard, st))) return e;
    }
    if (!(flags & FAAR_STEP_XT_READY) && !token_major) {
      if (int e = hip_status(launch_transpose_bf16(xq, T, K, static_cast<bf16_t*>(const_cast<void*>(Xt)), L.Tp, st))) return e;
    }
  } else {
    Bracket b(FAAR_K_GEMM_RESIDUAL, st);
    // X_q^T, which the dW GEMM reads next, was pushed out of the 256 MB last-level cache by the previous step's pass over
    // V, m, u: the residual GEMM reads it on the side (when it is at most half that cache, and the dW GEMM will use it)
    const int64_t xt_bytes = (int64_t)K * L.Tp * 2;
    const bool warm_xt = xt_bytes <= ((int64_t)128 << 20);
    if (rows_form) {
      // with H and the token-major dW GEMM: dY stays token-major ([T, O], in the place of dY^T), no transposed staging,
      // and the dW GEMM re-reads the X_q this GEMM has just read: nothing to fetch on the side
      if (int e = hip_status(launch_gemm_residual_rows(xq, delta, d1, x_scale, 2.0f * mse_scale, dYt, mse_p, &n_mse, guard, st)))
        return e;
    } else if (int e = hip_status(launch_gemm_residual(xq, delta, d1, Hs ? nullptr : C, x_scale, 2.0f * mse_scale,
                                                       (Hs && dY_ext) ? nullptr : dYt, L.Tp, need_local_dY ? dY : nullptr, mse_p,
                                                       &n_mse, guard, warm_xt ? Xt : nullptr, xt_bytes, st))) {
      // with H: no constant in the epilogue, and no dY^T at all when the gradient comes from upstream
      return e;
    }
  }
  // otherwise the upstream gradient is transposed over dY^T
  const bf16_t* dY_used = dY;
  if (dY_ext) {
    dY_used = static_cast<const bf16_t*>(dY_ext);
    if (!token_major)
      if (int e = hip_status(launch_transpose_bf16(dY_used, T, O, dYt, L.Tp, st))) return e;
  }
  // s3: G = dY^T X_q, contraction over tokens, split for occupancy
  {
    Bracket b(FAAR_K_GEMM_DW, st);
    if (token_major || rows_form) {
      if (int e = hip_status(launch_gemm_f32_tn(rows_form ? dYt : dY_used, xq, GemmDims{O, K, T, O, K}, G, L.n_split,
                                                (flags & FAAR_STEP_WHOLE_DEVICE) != 0, st)))
        return e;
    } else {
      const GemmDims d2{O, K, L.Tp, L.Tp, L.Tp};
      if (int e = hip_status(launch_gemm_f32(dYt, static_cast<const bf16_t*>(Xt), d2, G, L.n_split, st))) return e;
    }
  }
  // s4: dX = dY W_q
  if (dX) {
    if (int e = hip_status(launch_transpose_bf16(wq_full, O, K, wqt, L.Op, st))) return e;
    const GemmDims d3{T, K, O, O, L.Op};
    Bracket b(FAAR_K_GEMM_DX, st);
    if (int e = hip_status(launch_gemm_bf16(dY_used, wqt, d3, static_cast<bf16_t*>(dX), nullptr, st))) return e;
  }
  // s5 + s6: dV, Adam, clip; the same launch sums the losses (both kinds of partials are complete by now:
  // they come from earlier kernels) and, when asked, runs s1 of the next step on the updated V
  StepBwdArgs a{};
  a.W = W; a.w_bf16 = bf; a.n = n;
  a.s_global = s_global; a.scales = scales; a.icodes = icodes;
  a.V = V; a.m = adam_m; a.u = adam_v;
  a.beta = beta; a.G = G; a.n_split = L.n_split; a.split_stride = (int64_t)O * K; a.x_scale = x_scale;
  a.lambda_round = lambda_round;
  a.opt.lr = opt->lr; a.opt.beta1 = opt->beta1; a.opt.beta2 = opt->beta2; a.opt.eps = opt->eps;
  a.opt.inv_bc1 = static_cast<float>(1.0 / (1.0 - std::pow((double)opt->beta1, (double)opt->t)));
  a.opt.inv_bc2 = static_cast<float>(1.0 / (1.0 - std::pow((double)opt->beta2, (double)opt->t)));
  a.mse_partials = mse_p; a.n_mse = n_mse; a.mse_scale = mse_scale; a.round_partials = round_p; a.losses = losses;
  a.beta_next = beta_next; a.delta_next = delta; a.wq_full_next = wq_full; a.round_next = round_next;
  a.guard_slot = guard_slot;
  a.next_tag = forward_tag(opt->t + 1, beta_next, V, W, scales, n, wq_full != nullptr, Hs);
  a.H = Hs; a.two_alpha_h = (Hs && !dY_ext) ? 2.0f * mse_scale : 0.0f;
  a.cross_partials = cross_p; a.c_norm2 = c_norm2; a.cross_next = cross_next;
  Bracket b(FAAR_K_BWD_ADAM, st);
  return hip_status(launch_step_bwd_adam(a, st));
}

// ---- the step in its Gram-matrix form (constant activations) --------------------------------------------------------
int faar_gram_prepare(const void* Xt, int64_t K, int64_t T, void* gram, float* gram_lo, void* ws, size_t ws_bytes,
                      void* stream) {
  if (!Xt || !gram || !gram_lo || !ws) return FAAR_E_NULL;
  if (int e = check_shape(K, K)) return e;
  if (T <= 0 || T > kMaxElems / K) return FAAR_E_SHAPE;
  if (!aligned16(Xt) || !aligned16(gram) || !aligned16(ws) || (reinterpret_cast<uintptr_t>(gram_lo) & 3u)) return FAAR_E_ARG;
  if (ws_bytes < faar_workspace_bytes(FAAR_OP_GRAM_PREPARE, K, K, T, 0)) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t Tp = padded_tokens(T);
  const int n_split = choose_split(K, K, Tp);
  const bf16_t* xt = static_cast<const bf16_t*>(Xt);
  float* part = static_cast<float*>(ws);
  if (int e = hip_status(launch_gemm_f32(xt, xt, GemmDims{K, K, Tp, Tp, Tp}, part, n_split, st))) return e;
  return hip_status(launch_gram_finish(part, n_split, K, static_cast<bf16_t*>(gram), gram_lo, st));
}

int faar_layer_step_gram(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global, const uint8_t* scales,
                         float* V, float* adam_m, float* adam_v, const float* x_scale, const uint8_t* icodes, const float* H,
                         const double* c_norm2, const void* gram, const float* gram_lo, float beta, float beta_next,
                         float lambda_round, float mse_scale, const faar_adam* opt, float* losses, uint32_t flags, void* ws,
                         size_t ws_bytes, void* stream) {
  if (!W || !s_global || !scales || !V || !adam_m || !adam_v || !icodes || !H || !c_norm2 || !gram || !gram_lo || !opt || !losses)
    return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (K > kMaxElems / K) return FAAR_E_SHAPE;
  if (flags & ~(uint32_t)FAAR_WS_FORWARD_READY) return FAAR_E_ARG;
  if (!(beta > 0.0f) || !std::isfinite(beta) || !std::isfinite(lambda_round) || !std::isfinite(mse_scale))
    return FAAR_E_ARG;
  if (!(beta_next >= 0.0f) || !std::isfinite(beta_next)) return FAAR_E_ARG;
  if (!(opt->lr >= 0.0f) || !std::isfinite(opt->lr) || !(opt->beta1 >= 0.0f && opt->beta1 < 1.0f) ||
      !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) || !(opt->eps >= 0.0f) || !std::isfinite(opt->eps) || opt->t < 1)
    return FAAR_E_ARG;
  if (!aligned16(W) || !aligned16(V) || !aligned16(adam_m) || !aligned16(adam_v) || !aligned16(icodes) || !aligned16(H) ||
      !aligned16(gram) || !aligned16(ws) || (reinterpret_cast<uintptr_t>(c_norm2) & 7u) ||
      (reinterpret_cast<uintptr_t>(gram_lo) & 3u))
    return FAAR_E_ARG;
  const GramLayout L = gram_layout(O, K);
  if (!ws || ws_bytes < L.total) return FAAR_E_WORKSPACE;

  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = wdt == FAAR_BF16;
  const int64_t n = O * K;
  char* base = static_cast<char*>(ws);
  bf16_t* delta = reinterpret_cast<bf16_t*>(base + L.delta);
  float* G = reinterpret_cast<float*>(base + L.G);
  double* mse_p = reinterpret_cast<double*>(base + L.mse_partials);
  double* round_p = reinterpret_cast<double*>(base + L.round_partials) + (opt->t & 1) * kStepBwdMaxBlocks;
  double* round_next = reinterpret_cast<double*>(base + L.round_partials) + ((opt->t + 1) & 1) * kStepBwdMaxBlocks;
  double* cross_p = reinterpret_cast<double*>(base + L.cross_partials) + (opt->t & 1) * kStepBwdMaxBlocks;
  double* cross_next = reinterpret_cast<double*>(base + L.cross_partials) + ((opt->t + 1) & 1) * kStepBwdMaxBlocks;
  uint32_t* guard_slot = reinterpret_cast<uint32_t*>(base + L.guard);
  ForwardGuard guard{nullptr, {}};
  // s1: W_q - W (bf16), Round-Loss partials and <W_q - W, H> partials -- unless the previous step left them
  if (!(flags & FAAR_WS_FORWARD_READY)) {
    Bracket b(FAAR_K_SOFTQUANT_FWD, st);
    if (int e = hip_status(launch_step_fwd(W, bf, n, s_global, scales, icodes, V, beta, delta, nullptr, round_p, guard_slot, H,
                                           cross_p, st)))
      return e;
  } else {
    guard.slot = guard_slot;
    guard.expect = forward_tag(opt->t, beta, V, W, scales, n, false, H);
  }
  // s2 + s3 in one product: (W_q - W) Gm, with the quadratic term of the loss summed in the epilogue
  int64_t n_mse = 0;
  {
    Bracket b(FAAR_K_GEMM_GRAM, st);
    if (int e = hip_status(launch_gemm_gram(delta, static_cast<const bf16_t*>(gram), O, K, gram_lo, x_scale, 2.0f * mse_scale, G,
                                            L.n_split, mse_p, &n_mse, guard, st)))
      return e;
  }
  // s5 + s6 as in faar_layer_step
  StepBwdArgs a{};
  a.W = W; a.w_bf16 = bf; a.n = n;
  a.s_global = s_global; a.scales = scales; a.icodes = icodes;
  a.V = V; a.m = adam_m; a.u = adam_v;
  a.beta = beta; a.G = G; a.n_split = L.n_split; a.split_stride = (int64_t)O * K; a.x_scale = x_scale;
  a.lambda_round = lambda_round;
  a.opt.lr = opt->lr; a.opt.beta1 = opt->beta1; a.opt.beta2 = opt->beta2; a.opt.eps = opt->eps;
  a.opt.inv_bc1 = static_cast<float>(1.0 / (1.0 - std::pow((double)opt->beta1, (double)opt->t)));
  a.opt.inv_bc2 = static_cast<float>(1.0 / (1.0 - std::pow((double)opt->beta2, (double)opt->t)));
  a.mse_partials = mse_p; a.n_mse = n_mse; a.mse_scale = mse_scale; a.round_partials = round_p; a.losses = losses;
  a.beta_next = beta_next; a.delta_next = delta; a.wq_full_next = nullptr; a.round_next = round_next;
  a.guard_slot = guard_slot;
  a.next_tag = forward_tag(opt->t + 1, beta_next, V, W, scales, n, false, H);
  a.H = H; a.two_alpha_h = 2.0f * mse_scale;
  a.cross_partials = cross_p; a.c_norm2 = c_norm2; a.cross_next = cross_next;
  Bracket b(FAAR_K_BWD_ADAM, st);
  return hip_status(launch_step_bwd_adam(a, st));
}

// ---- glue of a block for joint (Stage-2-style) steps ---------------------------------------------------------------
static int check_rows(int64_t T, int64_t D) {
  if (T <= 0 || D <= 0 || D % 8 != 0 || T > 0x7FFFFFFF || T > kMaxElems / D) return FAAR_E_SHAPE;
  return FAAR_OK;
}

int faar_linear_forward(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global, const uint8_t* scales,
                        const float* V, float beta, const void* Xq, const float* x_scale, int64_t T, void* Y, void* ws,
                        size_t ws_bytes, void* stream) {
  if (!W || !s_global || !scales || !V || !Xq || !Y) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return FAAR_E_SHAPE;
  if (!(beta > 0.0f) || !std::isfinite(beta)) return FAAR_E_ARG;
  if (!aligned16(W) || !aligned16(V) || !aligned16(Xq) || !aligned16(Y) || !aligned16(ws)) return FAAR_E_ARG;
  if (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_LINEAR_FORWARD, O, K, T, 0)) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  bf16_t* wq = static_cast<bf16_t*>(ws);
  if (int e = hip_status(launch_softquant_fwd(W, wdt == FAAR_BF16, O * K, s_global, scales, V, beta, false, wq, nullptr, st)))
    return e;
  Bracket b(FAAR_K_GEMM_FWD, st);
  return hip_status(launch_gemm_bf16(static_cast<const bf16_t*>(Xq), wq, GemmDims{T, O, K, K, K}, static_cast<bf16_t*>(Y),
                                     x_scale, st));
}

int faar_rmsnorm_fwd(const void* x, faar_dtype xdt, int64_t T, int64_t D, const float* g, float eps, void* h, float* rstd,
                     void* stream) {
  if (!x || !g || !h || !rstd) return FAAR_E_NULL;
  if (int e = check_wdt(xdt)) return e;
  if (int e = check_rows(T, D)) return e;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return FAAR_E_ARG;
  if (!aligned16(x) || !aligned16(g) || !aligned16(h)) return FAAR_E_ARG;
  return hip_status(launch_rmsnorm_fwd(x, xdt == FAAR_BF16, T, D, g, eps, static_cast<bf16_t*>(h), rstd,
                                       static_cast<hipStream_t>(stream)));
}

int faar_rmsnorm_bwd(const void* dh1, const void* dh2, const void* dh3, const void* x, faar_dtype xdt, int64_t T, int64_t D,
                     const float* g, const float* rstd, const void* d_res, void* dx, void* stream) {
  if (!dh1 || !x || !g || !rstd || !dx) return FAAR_E_NULL;
  if (int e = check_wdt(xdt)) return e;
  if (int e = check_rows(T, D)) return e;
  if (!aligned16(dh1) || !aligned16(dh2) || !aligned16(dh3) || !aligned16(x) || !aligned16(g) || !aligned16(d_res) || !aligned16(dx))
    return FAAR_E_ARG;
  return hip_status(launch_rmsnorm_bwd(static_cast<const bf16_t*>(dh1), static_cast<const bf16_t*>(dh2),
                                       static_cast<const bf16_t*>(dh3), x, xdt == FAAR_BF16, T, D, g, rstd,
                                       static_cast<const bf16_t*>(d_res), static_cast<bf16_t*>(dx),
                                       static_cast<hipStream_t>(stream)));
}

int faar_rope(const void* x, int64_t T, int64_t H, int64_t dh, const float* cos_t, const float* sin_t, int64_t S, int32_t inverse,
              void* y, void* stream) {
  if (!x || !cos_t || !sin_t || !y) return FAAR_E_NULL;
  if (T <= 0 || H <= 0 || dh <= 0 || S <= 0 || dh % 16 != 0 || dh > 4096 || H > 65536 || T > kMaxElems / (H * dh)) return FAAR_E_SHAPE;
  if (!aligned16(x) || !aligned16(y) || !aligned16(cos_t) || !aligned16(sin_t)) return FAAR_E_ARG;
  return hip_status(launch_rope(static_cast<const bf16_t*>(x), T, H, dh, cos_t, sin_t, S, inverse != 0, static_cast<bf16_t*>(y),
                                static_cast<hipStream_t>(stream)));
}

// Row pitch of the transposed copies the attention kernels read column blocks of: the padded token count plus 64 entries,
// so that consecutive rows (one per head-dimension index, all read by one load instruction) do not sit a power of two apart
// and collide in the same cache sets and memory channels
static int64_t attention_pitch(int64_t T) { return padded_tokens(T) + 64; }

static int check_attention(int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv, int64_t dh, float scale) {
  if (n_seq <= 0 || S <= 0 || S % 32 != 0 || S > (1 << 20) || n_q <= 0 || n_kv <= 0 || n_q % n_kv != 0 || n_q > 4096) return FAAR_E_SHAPE;
  if (dh != 64 && dh != 128) return FAAR_E_SHAPE;
  if (n_seq > kMaxElems / (S * n_q * dh) || n_seq * n_q * (S / 32) > 0x7FFFFFFFLL) return FAAR_E_SHAPE;
  if (!(scale > 0.0f) || !std::isfinite(scale)) return FAAR_E_ARG;
  return FAAR_OK;
}

int faar_attention_fwd(const void* q, const void* k, const void* v, int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv,
                       int64_t dh, float scale, void* o, float* lse, void* ws, size_t ws_bytes, void* stream) {
  if (!q || !k || !v || !o || !lse) return FAAR_E_NULL;
  if (int e = check_attention(n_seq, S, n_q, n_kv, dh, scale)) return e;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(ws)) return FAAR_E_ARG;
  const int64_t T = n_seq * S, Tp = attention_pitch(T);
  if (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_ATTENTION_FWD, n_q * dh, n_kv * dh, T, 0)) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  bf16_t* vt = static_cast<bf16_t*>(ws);
  if (int e = hip_status(launch_transpose_bf16(static_cast<const bf16_t*>(v), T, n_kv * dh, vt, Tp, st))) return e;
  Bracket b(FAAR_K_ATTENTION_FWD, st);
  return hip_status(launch_attention_fwd(static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k), vt, n_seq, S, n_q, n_kv, dh,
                                         Tp, scale, static_cast<bf16_t*>(o), lse, st));
}

int faar_attention_bwd(const void* d_o, const void* q, const void* k, const void* v, const void* o, const float* lse,
                       int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv, int64_t dh, float scale, void* dq, void* dk,
                       void* dv, void* ws, size_t ws_bytes, void* stream) {
  if (!d_o || !q || !k || !v || !o || !lse || !dq || !dk || !dv) return FAAR_E_NULL;
  if (int e = check_attention(n_seq, S, n_q, n_kv, dh, scale)) return e;
  if (!aligned16(d_o) || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv) || !aligned16(ws))
    return FAAR_E_ARG;
  const int64_t T = n_seq * S, Tp = attention_pitch(T);
  if (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_ATTENTION_BWD, n_q * dh, n_kv * dh, T, 0)) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Carver c(ws);
  bf16_t* qt = c.take<bf16_t>((size_t)n_q * dh * Tp);
  bf16_t* dot = c.take<bf16_t>((size_t)n_q * dh * Tp);
  bf16_t* kt = c.take<bf16_t>((size_t)n_kv * dh * Tp);
  float* delta = c.take<float>((size_t)n_q * T);
  if (int e = hip_status(launch_transpose_bf16(static_cast<const bf16_t*>(q), T, n_q * dh, qt, Tp, st))) return e;
  if (int e = hip_status(launch_transpose_bf16(static_cast<const bf16_t*>(d_o), T, n_q * dh, dot, Tp, st))) return e;
  if (int e = hip_status(launch_transpose_bf16(static_cast<const bf16_t*>(k), T, n_kv * dh, kt, Tp, st))) return e;
  Bracket b(FAAR_K_ATTENTION_BWD, st);
  return hip_status(launch_attention_bwd(static_cast<const bf16_t*>(d_o), static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                                         static_cast<const bf16_t*>(v), static_cast<const bf16_t*>(o), lse, qt, kt, dot, delta, n_seq,
                                         S, n_q, n_kv, dh, Tp, scale, static_cast<bf16_t*>(dq), static_cast<bf16_t*>(dk),
                                         static_cast<bf16_t*>(dv), st));
}

int faar_silu_mul_fwd(const void* p, const void* q, int64_t n, void* a, void* stream) {
  if (!p || !q || !a) return FAAR_E_NULL;
  if (n <= 0 || n % 8 != 0 || n > kMaxElems) return FAAR_E_SHAPE;
  if (!aligned16(p) || !aligned16(q) || !aligned16(a)) return FAAR_E_ARG;
  return hip_status(launch_silu_mul_fwd(static_cast<const bf16_t*>(p), static_cast<const bf16_t*>(q), n, static_cast<bf16_t*>(a),
                                        static_cast<hipStream_t>(stream)));
}

int faar_silu_mul_bwd(const void* da, const void* p, const void* q, int64_t n, void* dp, void* dq, void* stream) {
  if (!da || !p || !q || !dp || !dq) return FAAR_E_NULL;
  if (n <= 0 || n % 8 != 0 || n > kMaxElems) return FAAR_E_SHAPE;
  if (!aligned16(da) || !aligned16(p) || !aligned16(q) || !aligned16(dp) || !aligned16(dq)) return FAAR_E_ARG;
  return hip_status(launch_silu_mul_bwd(static_cast<const bf16_t*>(da), static_cast<const bf16_t*>(p), static_cast<const bf16_t*>(q),
                                        n, static_cast<bf16_t*>(dp), static_cast<bf16_t*>(dq), static_cast<hipStream_t>(stream)));
}

int faar_residual_add(const void* x, faar_dtype xdt, const void* d, int64_t n, void* y, void* stream) {
  if (!x || !d || !y) return FAAR_E_NULL;
  if (int e = check_wdt(xdt)) return e;
  if (n <= 0 || n % 8 != 0 || n > kMaxElems) return FAAR_E_SHAPE;
  if (!aligned16(x) || !aligned16(d) || !aligned16(y)) return FAAR_E_ARG;
  return hip_status(launch_residual_add(x, xdt == FAAR_BF16, static_cast<const bf16_t*>(d), n, static_cast<bf16_t*>(y),
                                        static_cast<hipStream_t>(stream)));
}

int faar_block_output_loss(const void* x, faar_dtype xdt, const void* d, const void* y_fp, faar_dtype ydt, int64_t T, int64_t D,
                           float mse_scale, void* y, void* dy, float* loss, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !d || !y_fp || !dy || !loss) return FAAR_E_NULL;
  if (int e = check_wdt(xdt)) return e;
  if (int e = check_wdt(ydt)) return e;
  if (int e = check_rows(T, D)) return e;
  if (!std::isfinite(mse_scale)) return FAAR_E_ARG;
  if (!aligned16(x) || !aligned16(d) || !aligned16(y_fp) || !aligned16(y) || !aligned16(dy) || !aligned16(ws)) return FAAR_E_ARG;
  if (!ws || ws_bytes < faar_workspace_bytes(FAAR_OP_BLOCK_OUTPUT_LOSS, D, 16, T, 0)) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  double* partials = static_cast<double*>(ws);
  if (int e = hip_status(launch_block_output_loss(x, xdt == FAAR_BF16, static_cast<const bf16_t*>(d), y_fp, ydt == FAAR_BF16, T * D,
                                                  2.0f * mse_scale, static_cast<bf16_t*>(y), static_cast<bf16_t*>(dy), partials, st)))
    return e;
  return hip_status(launch_finalize_losses(partials, block_loss_blocks(T * D), mse_scale, nullptr, 0, 0.0, 0.0f, loss, nullptr,
                                           nullptr, st));
}

// ---- a whole block's joint step: the calls above in sequence, every intermediate in the caller's workspace ------------
namespace {

struct BlockDims {
  int64_t T, Tp, D, Qd, Kd, F;
  bool qk_norm;
  float scale;
};

struct BlockLayout {
  // offsets into the workspace (bytes)
  size_t h, q0, k0, v, q1, k1, rq, rk, o, lse, d1, x1, rstd1, rstd2, h2, p, u, a, d2, dy, da, dp, du, dh_a, dh_b, dh_c, dx1,
      d_o, dq, dk, dv, dq0, dk0, xt, fwd_ws, step_ws, attn_ws, loss_ws, total;
  size_t fwd_bytes, step_bytes, attn_bytes, loss_bytes;
};

int block_dims(const faar_block* b, BlockDims& d) {
  if (!b) return FAAR_E_NULL;
  if (b->n_seq <= 0 || b->S <= 0 || b->D <= 0 || b->F <= 0 || b->n_q <= 0 || b->n_kv <= 0) return FAAR_E_SHAPE;
  if (b->D % 16 != 0 || b->F % 16 != 0) return FAAR_E_SHAPE;
  const float scale = b->attn_scale == 0.0f ? 1.0f / std::sqrt(static_cast<float>(b->dh)) : b->attn_scale;
  if (int e = check_attention(b->n_seq, b->S, b->n_q, b->n_kv, b->dh, scale)) return e;
  if (int e = check_wdt(b->wdt)) return e;
  d.T = b->n_seq * b->S;
  d.Tp = padded_tokens(d.T);
  d.D = b->D; d.Qd = b->n_q * b->dh; d.Kd = b->n_kv * b->dh; d.F = b->F;
  const int64_t widest = std::max(std::max(d.D, d.F), d.Qd);
  if (d.T > kMaxElems / widest || d.D > kMaxElems / d.F) return FAAR_E_SHAPE;
  if ((b->g_q != nullptr) != (b->g_k != nullptr)) return FAAR_E_NULL;
  d.qk_norm = b->g_q != nullptr;
  d.scale = scale;
  if (!(b->eps >= 0.0f) || !std::isfinite(b->eps)) return FAAR_E_ARG;
  return FAAR_OK;
}

void lin_shape(const BlockDims& d, int slot, int64_t& O, int64_t& K) {
  switch (slot) {
    case FAAR_LIN_Q: O = d.Qd; K = d.D; break;
    case FAAR_LIN_K: case FAAR_LIN_V: O = d.Kd; K = d.D; break;
    case FAAR_LIN_O: O = d.D; K = d.Qd; break;
    case FAAR_LIN_GATE: case FAAR_LIN_UP: O = d.F; K = d.D; break;
    default: O = d.D; K = d.F; break;
  }
}

BlockLayout block_layout(const BlockDims& d, int64_t n_q, int64_t n_kv) {
  BlockLayout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
  const size_t T = d.T, td = T * d.D * 2, tq = T * d.Qd * 2, tk = T * d.Kd * 2, tf = T * d.F * 2;
  L.h = take(td); L.q0 = take(tq); L.k0 = take(tk); L.v = take(tk);
  L.q1 = take(tq); L.k1 = take(tk);                       // after the per-head norm (if any) and the rotary embedding
  L.rq = take(T * n_q * 4); L.rk = take(T * n_kv * 4);
  L.o = take(tq); L.lse = take(T * n_q * 4); L.d1 = take(td); L.x1 = take(td);
  L.rstd1 = take(T * 4); L.rstd2 = take(T * 4);
  L.h2 = take(td); L.p = take(tf); L.u = take(tf); L.a = take(tf); L.d2 = take(td); L.dy = take(td);
  L.da = take(tf); L.dp = take(tf); L.du = take(tf);
  L.dh_a = take(td); L.dh_b = take(td); L.dh_c = take(td); L.dx1 = take(td);
  L.d_o = take(tq); L.dq = take(tq); L.dk = take(tk); L.dv = take(tk); L.dq0 = take(tq); L.dk0 = take(tk);
  L.xt = take(static_cast<size_t>(std::max(std::max(d.D, d.F), d.Qd)) * d.Tp * 2);
  for (int s = 0; s < FAAR_LIN_COUNT; ++s) {
    int64_t O, K;
    lin_shape(d, s, O, K);
    L.fwd_bytes = std::max(L.fwd_bytes, faar_workspace_bytes(FAAR_OP_LINEAR_FORWARD, O, K, d.T, 0));
    L.step_bytes = std::max(L.step_bytes, faar_workspace_bytes(FAAR_OP_LAYER_STEP, O, K, d.T, FAAR_WS_CHAINED));
  }
  L.attn_bytes = std::max(faar_workspace_bytes(FAAR_OP_ATTENTION_FWD, d.Qd, d.Kd, d.T, 0),
                          faar_workspace_bytes(FAAR_OP_ATTENTION_BWD, d.Qd, d.Kd, d.T, 0));
  L.loss_bytes = faar_workspace_bytes(FAAR_OP_BLOCK_OUTPUT_LOSS, d.D, 16, d.T, 0);
  L.fwd_ws = take(L.fwd_bytes); L.step_ws = take(L.step_bytes); L.attn_ws = take(L.attn_bytes); L.loss_ws = take(L.loss_bytes);
  L.total = off;
  return L;
}

}  // namespace

size_t faar_block_workspace_bytes(const faar_block* blk) {
  BlockDims d;
  if (block_dims(blk, d) != FAAR_OK) return 0;
  return block_layout(d, blk->n_q, blk->n_kv).total;
}

int faar_block_joint_step(const faar_block* blk, const void* x, const void* y_fp, float mse_scale, float beta,
                          float lambda_round, const faar_adam* opt, float* block_loss, void* dx, void* ws, size_t ws_bytes,
                          void* stream) {
  BlockDims d;
  if (int e = block_dims(blk, d)) return e;
  if (!x || !y_fp || !opt || !block_loss || !blk->g_attn || !blk->g_mlp || !blk->cos_t || !blk->sin_t) return FAAR_E_NULL;
  for (int s = 0; s < FAAR_LIN_COUNT; ++s) {
    const faar_block_linear& l = blk->lin[s];
    if (!l.W || !l.s_global || !l.scales || !l.icodes || !l.V || !l.adam_m || !l.adam_u || !l.losses) return FAAR_E_NULL;
    if (!aligned16(l.W) || !aligned16(l.scales) || !aligned16(l.icodes) || !aligned16(l.V) || !aligned16(l.adam_m) ||
        !aligned16(l.adam_u))
      return FAAR_E_ARG;
  }
  if (!(beta > 0.0f) || !std::isfinite(beta) || !std::isfinite(lambda_round) || !std::isfinite(mse_scale)) return FAAR_E_ARG;
  if (!(opt->lr >= 0.0f) || !std::isfinite(opt->lr) || !(opt->beta1 >= 0.0f && opt->beta1 < 1.0f) ||
      !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) || !(opt->eps >= 0.0f) || !std::isfinite(opt->eps) || opt->t < 1)
    return FAAR_E_ARG;
  if (!aligned16(x) || !aligned16(y_fp) || !aligned16(dx) || (reinterpret_cast<uintptr_t>(ws) & 255u)) return FAAR_E_ARG;
  const BlockLayout L = block_layout(d, blk->n_q, blk->n_kv);
  if (!ws || ws_bytes < L.total) return FAAR_E_WORKSPACE;

  char* base = static_cast<char*>(ws);
  auto at = [&](size_t off) { return static_cast<void*>(base + off); };
  auto fl = [&](size_t off) { return reinterpret_cast<float*>(base + off); };
  const int64_t T = d.T, Hq = blk->n_q, Hk = blk->n_kv, dh = blk->dh;
  const faar_dtype bf = FAAR_BF16;

  auto forward = [&](int slot, const void* X, void* Y) {
    int64_t O, K;
    lin_shape(d, slot, O, K);
    const faar_block_linear& l = blk->lin[slot];
    return faar_linear_forward(l.W, blk->wdt, O, K, l.s_global, l.scales, l.V, beta, X, nullptr, T, Y, at(L.fwd_ws), L.fwd_bytes,
                               stream);
  };
  // xt_shared: the linear reads the same activations as the one stepped just before it.  The transpose in the scratch is
  // valid for it only if one of those earlier siblings needed it (a linear whose dW GEMM takes token-major operands
  // neither reads nor writes it)
  bool xt_valid = false;
  auto backward = [&](int slot, const void* X, const void* dY, void* dX, bool xt_shared) {
    int64_t O, K;
    lin_shape(d, slot, O, K);
    const faar_block_linear& l = blk->lin[slot];
    const bool xt_ready = xt_shared && xt_valid;
    xt_valid = (xt_shared && xt_valid) || !gemm_tn_usable(O, K, T);
    const uint32_t flags = FAAR_WS_CHAINED | FAAR_STEP_JOINT | (xt_ready ? FAAR_STEP_XT_READY : 0u);
    return faar_layer_step(l.W, blk->wdt, O, K, l.s_global, l.scales, l.V, l.adam_m, l.adam_u, X, nullptr, at(L.xt), nullptr,
                           l.icodes, nullptr, nullptr, T, dY, dX, beta, 0.0f, lambda_round, 0.0f, opt, l.losses, flags,
                           at(L.step_ws), L.step_bytes, stream);
  };
#define FAAR_TRY(call) do { if (int e_ = (call)) return e_; } while (0)

  // ---- forward: attention half
  FAAR_TRY(faar_rmsnorm_fwd(x, bf, T, d.D, blk->g_attn, blk->eps, at(L.h), fl(L.rstd1), stream));
  FAAR_TRY(forward(FAAR_LIN_Q, at(L.h), at(L.q0)));
  FAAR_TRY(forward(FAAR_LIN_K, at(L.h), at(L.k0)));
  FAAR_TRY(forward(FAAR_LIN_V, at(L.h), at(L.v)));
  const void *qn = at(L.q0), *kn = at(L.k0);
  if (d.qk_norm) {
    FAAR_TRY(faar_rmsnorm_fwd(at(L.q0), bf, T * Hq, dh, blk->g_q, blk->eps, at(L.q1), fl(L.rq), stream));
    FAAR_TRY(faar_rmsnorm_fwd(at(L.k0), bf, T * Hk, dh, blk->g_k, blk->eps, at(L.k1), fl(L.rk), stream));
    qn = at(L.q1);
    kn = at(L.k1);
  }
  FAAR_TRY(faar_rope(qn, T, Hq, dh, blk->cos_t, blk->sin_t, blk->S, 0, at(L.q1), stream));   // in place after the norm
  FAAR_TRY(faar_rope(kn, T, Hk, dh, blk->cos_t, blk->sin_t, blk->S, 0, at(L.k1), stream));
  FAAR_TRY(faar_attention_fwd(at(L.q1), at(L.k1), at(L.v), blk->n_seq, blk->S, Hq, Hk, dh, d.scale, at(L.o), fl(L.lse),
                              at(L.attn_ws), L.attn_bytes, stream));
  FAAR_TRY(forward(FAAR_LIN_O, at(L.o), at(L.d1)));
  FAAR_TRY(faar_residual_add(x, bf, at(L.d1), T * d.D, at(L.x1), stream));
  // ---- forward: MLP half and the loss
  FAAR_TRY(faar_rmsnorm_fwd(at(L.x1), bf, T, d.D, blk->g_mlp, blk->eps, at(L.h2), fl(L.rstd2), stream));
  FAAR_TRY(forward(FAAR_LIN_GATE, at(L.h2), at(L.p)));
  FAAR_TRY(forward(FAAR_LIN_UP, at(L.h2), at(L.u)));
  FAAR_TRY(faar_silu_mul_fwd(at(L.p), at(L.u), T * d.F, at(L.a), stream));
  FAAR_TRY(forward(FAAR_LIN_DOWN, at(L.a), at(L.d2)));
  FAAR_TRY(faar_block_output_loss(at(L.x1), bf, at(L.d2), y_fp, bf, T, d.D, mse_scale, nullptr, at(L.dy), block_loss,
                                  at(L.loss_ws), L.loss_bytes, stream));
  // ---- backward: MLP half
  FAAR_TRY(backward(FAAR_LIN_DOWN, at(L.a), at(L.dy), at(L.da), false));
  FAAR_TRY(faar_silu_mul_bwd(at(L.da), at(L.p), at(L.u), T * d.F, at(L.dp), at(L.du), stream));
  FAAR_TRY(backward(FAAR_LIN_GATE, at(L.h2), at(L.dp), at(L.dh_a), false));
  FAAR_TRY(backward(FAAR_LIN_UP, at(L.h2), at(L.du), at(L.dh_b), true));      // h2^T is still in the scratch
  FAAR_TRY(faar_rmsnorm_bwd(at(L.dh_a), at(L.dh_b), nullptr, at(L.x1), bf, T, d.D, blk->g_mlp, fl(L.rstd2), at(L.dy), at(L.dx1),
                            stream));
  // ---- backward: attention half
  FAAR_TRY(backward(FAAR_LIN_O, at(L.o), at(L.dx1), at(L.d_o), false));
  FAAR_TRY(faar_attention_bwd(at(L.d_o), at(L.q1), at(L.k1), at(L.v), at(L.o), fl(L.lse), blk->n_seq, blk->S, Hq, Hk, dh,
                              d.scale, at(L.dq), at(L.dk), at(L.dv), at(L.attn_ws), L.attn_bytes, stream));
  FAAR_TRY(faar_rope(at(L.dq), T, Hq, dh, blk->cos_t, blk->sin_t, blk->S, 1, at(L.dq), stream));
  FAAR_TRY(faar_rope(at(L.dk), T, Hk, dh, blk->cos_t, blk->sin_t, blk->S, 1, at(L.dk), stream));
  const void *dq0 = at(L.dq), *dk0 = at(L.dk);
  if (d.qk_norm) {
    FAAR_TRY(faar_rmsnorm_bwd(at(L.dq), nullptr, nullptr, at(L.q0), bf, T * Hq, dh, blk->g_q, fl(L.rq), nullptr, at(L.dq0), stream));
    FAAR_TRY(faar_rmsnorm_bwd(at(L.dk), nullptr, nullptr, at(L.k0), bf, T * Hk, dh, blk->g_k, fl(L.rk), nullptr, at(L.dk0), stream));
    dq0 = at(L.dq0);
    dk0 = at(L.dk0);
  }
  FAAR_TRY(backward(FAAR_LIN_Q, at(L.h), dq0, dx ? at(L.dh_a) : nullptr, false));
  FAAR_TRY(backward(FAAR_LIN_K, at(L.h), dk0, dx ? at(L.dh_b) : nullptr, true));
  FAAR_TRY(backward(FAAR_LIN_V, at(L.h), at(L.dv), dx ? at(L.dh_c) : nullptr, true));
  if (dx)
    FAAR_TRY(faar_rmsnorm_bwd(at(L.dh_a), at(L.dh_b), at(L.dh_c), x, bf, T, d.D, blk->g_attn, fl(L.rstd1), at(L.dx1), dx, stream));
#undef FAAR_TRY
  return FAAR_OK;
}

int faar_stochastic_v(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                      const uint8_t* scales, unsigned long long seed, uint32_t sample, float* V, void* stream) {
  if (!W || !s_global || !scales || !V) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (!aligned16(W) || !aligned16(V)) return FAAR_E_ARG;
  return hip_status(launch_stochastic_v(W, wdt == FAAR_BF16, O * K, s_global, scales, seed, sample, V,
                                        static_cast<hipStream_t>(stream)));
}

int faar_hardened_loss(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                       const uint8_t* scales, const float* V, const void* Xq, const float* x_scale, const float* C,
                       int64_t T, float mse_scale, float* loss, void* ws, size_t ws_bytes, void* stream) {
  if (!W || !s_global || !scales || !V || !Xq || !C || !loss) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (T <= 0 || T > kMaxElems / (O > K ? O : K)) return FAAR_E_SHAPE;
  if (!std::isfinite(mse_scale)) return FAAR_E_ARG;
  if (!aligned16(W) || !aligned16(V) || !aligned16(Xq) || !aligned16(C) || !aligned16(ws)) return FAAR_E_ARG;
  const StepLayout L = step_layout(O, K, T, false);
  if (!ws || ws_bytes < L.total) return FAAR_E_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  bf16_t* delta = reinterpret_cast<bf16_t*>(base + L.delta);
  bf16_t* dYt = reinterpret_cast<bf16_t*>(base + L.dYt);
  double* mse_p = reinterpret_cast<double*>(base + L.mse_partials);
  if (int e = hip_status(launch_hardened_delta(W, wdt == FAAR_BF16, O * K, s_global, scales, V, delta,
                                               reinterpret_cast<uint32_t*>(base + L.guard), st)))
    return e;
  int64_t n_mse = 0;
  const GemmDims d1{T, O, K, K, K};
  if (int e = hip_status(launch_gemm_residual(static_cast<const bf16_t*>(Xq), delta, d1, C, x_scale, 2.0f * mse_scale, dYt,
                                              L.Tp, nullptr, mse_p, &n_mse, ForwardGuard{nullptr, {}}, nullptr, 0, st)))
    return e;
  return hip_status(launch_finalize_losses(mse_p, n_mse, mse_scale, nullptr, 0, 0.0, 0.0f, loss, nullptr, nullptr, st));
}

int faar_stage2_losses(const void* Z_fp, const void* Z_q, faar_dtype zdt, int64_t T, int64_t vocab, float tau,
                       float kl_scale, const void* H_fp, const void* H_q, faar_dtype hdt, int64_t D, float mse_scale,
                       const float* round_losses, int64_t n_layers, float lambda_kl, float lambda_round, void* dZ_q,
                       void* dH_q, float* losses, void* ws, size_t ws_bytes, void* stream) {
  if (!Z_fp || !Z_q || !H_fp || !H_q || !losses) return FAAR_E_NULL;
  if (int e = check_wdt(zdt)) return e;
  if (int e = check_wdt(hdt)) return e;
  if (T <= 0 || vocab <= 0 || D <= 0 || vocab % 8 != 0 || D % 8 != 0 || n_layers < 0) return FAAR_E_SHAPE;
  if (T > kMaxElems / vocab || T > kMaxElems / D || T > 0x7FFFFFFF) return FAAR_E_SHAPE;
  if (!(tau > 0.0f) || !std::isfinite(tau) || !std::isfinite(kl_scale) || !std::isfinite(mse_scale) ||
      !std::isfinite(lambda_kl) || !std::isfinite(lambda_round))
    return FAAR_E_ARG;
  if (n_layers > 0 && !round_losses) return FAAR_E_NULL;
  if (!aligned16(Z_fp) || !aligned16(Z_q) || !aligned16(H_fp) || !aligned16(H_q) || !aligned16(dZ_q) || !aligned16(dH_q) ||
      !aligned16(ws))
    return FAAR_E_ARG;
  const size_t need = align256((size_t)T * sizeof(double)) + align256((size_t)stage2_mse_blocks(T * D) * sizeof(double));
  if (!ws || ws_bytes < need) return FAAR_E_WORKSPACE;
  Stage2Args a{};
  a.Z_fp = Z_fp; a.Z_q = Z_q; a.z_bf16 = zdt == FAAR_BF16; a.T = T; a.vocab = vocab; a.tau = tau; a.kl_scale = kl_scale;
  a.H_fp = H_fp; a.H_q = H_q; a.h_bf16 = hdt == FAAR_BF16; a.D = D; a.mse_scale = mse_scale;
  a.round_losses = n_layers > 0 ? round_losses : nullptr; a.n_layers = n_layers;
  a.lambda_kl = lambda_kl; a.lambda_round = lambda_round;
  a.dZ_q = dZ_q; a.dH_q = dH_q;
  a.kl_rows = static_cast<double*>(ws);
  a.mse_partials = reinterpret_cast<double*>(static_cast<char*>(ws) + align256((size_t)T * sizeof(double)));
  a.losses = losses;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Bracket b(FAAR_K_STAGE2_KL, st);
  return hip_status(launch_stage2(a, st));
}

int faar_harden_pack(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global,
                     const uint8_t* scales, const float* V, uint8_t* codes, uint8_t* decisions,
                     void* W_final, unsigned long long* flip_count, void* stream) {
  if (!W || !s_global || !scales || !V || !codes) return FAAR_E_NULL;
  if (int e = check_wdt(wdt)) return e;
  if (int e = check_shape(O, K)) return e;
  if (!aligned16(W) || !aligned16(V) || !aligned16(codes) || !aligned16(W_final) ||
      (reinterpret_cast<uintptr_t>(flip_count) & 7u))
    return FAAR_E_ARG;
  Bracket b(FAAR_K_HARDEN_PACK, static_cast<hipStream_t>(stream));
  return hip_status(launch_harden_pack(W, wdt == FAAR_BF16, O * K, s_global, scales, V, codes, decisions, W_final,
                                       flip_count, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
