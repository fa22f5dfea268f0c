// Host-side declarations shared by the translation units of libfaar: kernel launchers and
// workspace layouts.  Launchers return hipError_t; argument validation lives in faar_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "faar_device.h"

namespace faar {

constexpr int kAmaxPartials = 1024;     // partial maxima written by the first amax pass
constexpr int kEltThreads = 256;        // threads per block of every elementwise kernel
constexpr int kStepBwdMaxBlocks = 2048;  // grid cap of the fused backward + Adam kernel (grid-stride beyond)

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
inline int64_t padded_tokens(int64_t T) { return round_up(T, 64); }

// Identity of the forward pass (W_q - W at some beta, for some V) that a step leaves in its workspace for the step
// that follows.  The guard slot in the workspace holds kTagWords tag words followed by one verdict word: the first
// kernel of a step either produces a fresh forward (verdict 1) or compares the stored tag with the one its caller
// implies (verdict = equal), and in both cases clears the tag; the kernel that updates V reads the verdict, and
// writes the tag of the next step's forward when it produces one.
constexpr int kTagWords = 12;
struct ForwardTag { uint32_t w[kTagWords]; };
struct ForwardGuard { uint32_t* slot; ForwardTag expect; };  // slot == nullptr: nothing to check

// ---- elementwise kernels (faar_elementwise.hip) -------------------------------------------
hipError_t launch_amax(const void* W, bool w_bf16, int64_t n, float* partials, float* s_global,
                       hipStream_t st);
// dq_in_units: W_dq receives sign * node * E4M3 scale (exact in bf16), without the factor s_global
hipError_t launch_quant_rtn(const void* W, bool w_bf16, int64_t n, const float* s_global,
                            uint8_t* scales, uint8_t* codes, void* W_dq, bool dq_in_units, hipStream_t st);
hipError_t launch_init_v(const void* W, bool w_bf16, int64_t n, const float* s_global,
                         const uint8_t* scales, float* V, uint8_t* floor_codes, hipStream_t st);
hipError_t launch_harden_pack(const void* W, bool w_bf16, int64_t n, const float* s_global,
                              const uint8_t* scales, const float* V, uint8_t* codes,
                              uint8_t* decisions, void* W_final, unsigned long long* flip_count,
                              hipStream_t st);
// Batched codec operations: up to kBatchMax tensors per launch, descriptors passed in the kernel arguments.
constexpr int kBatchMax = 72;          // 72 descriptors of 48 bytes + the index table stay below the 4 KB argument limit
constexpr int kBatchAmaxBlocks = 64;   // workgroups (and partial maxima) per tensor in the batched amax pass
struct CodecItem {
  const void* W; float* s_global; uint8_t* scales; float* V; uint32_t* codes;
  int64_t n8;                          // chunks of 8 weights
};
struct CodecBatch {
  int n;                               // tensors in this launch
  uint32_t first_block[kBatchMax + 1]; // first workgroup of each tensor; [n] = grid size
  CodecItem it[kBatchMax];
};
static_assert(sizeof(CodecBatch) <= 4096, "kernel arguments are limited to 4 KB");
enum { kBatchQuant = 0, kBatchInitV = 1, kBatchHardenPack = 2 };
// partials: kBatchAmaxBlocks floats per tensor (quantise without given tensor scales only)
hipError_t launch_codec_batch(int op, const CodecBatch& B, bool w_bf16, bool sglobal_given, float* partials, hipStream_t st);

// Wt = bf16(W_q) or bf16(W_q - W); Wq_full (nullable) additionally receives bf16(W_q).
hipError_t launch_softquant_fwd(const void* W, bool w_bf16, int64_t n, const float* s_global,
                                const uint8_t* scales, const float* V, float beta, bool delta,
                                bf16_t* Wt, bf16_t* Wq_full, hipStream_t st);
// dV = sum_s G[s] * dWq/dV + lambda/N (4 - 8 v); per-block Round-Loss partial sums (double).
hipError_t launch_softquant_bwd(const void* W, bool w_bf16, int64_t n, const float* s_global,
                                const uint8_t* scales, const float* V, float beta, const float* G,
                                int n_split, int64_t split_stride, float lambda_round, float* dV,
                                double* round_partials, hipStream_t st);
int64_t softquant_bwd_blocks(int64_t n);
int64_t step_bwd_blocks(int64_t n);
struct AdamScalars { float lr, beta1, beta2, eps, inv_bc1, inv_bc2; };
// Interval codes signbit(w) << 3 | (w == 0 ? 7 : k_lo), two per byte, for the per-step kernels below.
hipError_t launch_interval_codes(const void* W, bool w_bf16, int64_t n, const float* s_global,
                                 const uint8_t* scales, uint8_t* icodes, hipStream_t st);
// Step forward on cached codes: delta = bf16(W_q - W) (+ bf16(W_q) when Wq_full), and the Round-Loss
// partial sums of V, one per block (step_bwd_blocks(n) of them).
hipError_t launch_step_fwd(const void* W, bool w_bf16, int64_t n, const float* s_global, const uint8_t* scales,
                           const uint8_t* icodes, const float* V, float beta, bf16_t* delta, bf16_t* Wq_full,
                           double* round_partials, uint32_t* guard_slot, const float* H, double* cross_partials,
                           hipStream_t st);
// Step backward + Adam + clip on cached codes.  One more block sums this step's losses (mse_partials from the
// residual GEMM, round_partials of the V the step started from) into losses[0..2].  beta_next > 0 also emits
// the next step's forward outputs from the updated V: delta_next (and wq_full_next when not null) and that
// V's Round-Loss partials in round_next (must not alias round_partials).
struct StepBwdArgs {
  const void* W; bool w_bf16; int64_t n;
  const float* s_global; const uint8_t* scales; const uint8_t* icodes;
  float *V, *m, *u;
  float beta; const float* G; int n_split; int64_t split_stride;
  const float* x_scale;  // device scalar multiplying G (activations stored in units of it); null = 1
  float lambda_round; AdamScalars opt;
  const double* mse_partials; int64_t n_mse; float mse_scale; const double* round_partials; float* losses;
  float beta_next; bf16_t* delta_next; bf16_t* wq_full_next; double* round_next;
  uint32_t* guard_slot;   // verdict of the step's first kernel; a failed check leaves V, m, u alone and gives NaN losses
  ForwardTag next_tag;    // written to the slot when beta_next > 0
  // Constant part of the gradient carried separately (null: not in use): H = C^T X_q [n]; G -= two_alpha_h * H;
  // L_mse = mse_scale * (sum mse_partials - 2 x_scale sum cross_partials + *c_norm2); cross_next: <delta_next, H> per block
  const float* H; float two_alpha_h; const double* cross_partials; const double* c_norm2; double* cross_next;
};
hipError_t launch_step_bwd_adam(const StepBwdArgs& a, hipStream_t st);
// losses[0] = mse_scale * sum(mse_partials), losses[1] = sum(round_partials) / n,
// losses[2] = losses[0] + lambda * losses[1].  Either partial array may be empty (count 0).
hipError_t launch_finalize_losses(const double* mse_partials, int64_t n_mse, float mse_scale,
                                  const double* round_partials, int64_t n_round, double inv_n,
                                  float lambda_round, float* loss_mse, float* loss_round,
                                  float* loss_total, hipStream_t st);
// out[c * ld_out + r] = in[r * cols + c] for r < rows, c < cols; columns rows..ld_out-1 zeroed.
hipError_t launch_transpose_bf16(const bf16_t* in, int64_t rows, int64_t cols, bf16_t* out,
                                 int64_t ld_out, hipStream_t st);
hipError_t launch_check_forward_tag(const ForwardGuard& guard, hipStream_t st);
// Term `term` (0 hi, 1 mid, 2 lo) of the float32 C [ceil(T/4)][O][4] as bf16, transposed to [O, ld_out] (ld_out =
// padded_tokens(T), zero padded); sq_partials (nullable): c_term_blocks(T, O) per-workgroup sums of C^2
int64_t c_term_blocks(int64_t T, int64_t O);
hipError_t launch_c_term_transposed(const float* C, int64_t T, int64_t O, int term, bf16_t* out, int64_t ld_out,
                                    double* sq_partials, hipStream_t st);
// H[0..n) = (first ? 0 : H) + sum_s partials[s * stride + i]
hipError_t launch_accumulate_partials(float* H, const float* partials, int n_split, int64_t stride, int64_t n, bool first,
                                      hipStream_t st);
hipError_t launch_sum_doubles(const double* p, int64_t n, double* out, hipStream_t st);
// gram[i] = bf16(sum_s partials[s * K * K + i]) for the K x K matrix; diag_lo[k] = that sum at (k, k) minus its bf16 rounding
hipError_t launch_gram_finish(const float* partials, int n_split, int64_t K, bf16_t* gram, float* diag_lo, hipStream_t st);
// float32 -> three bf16 terms hi + mid + lo (each the rounding of the running remainder).
hipError_t launch_split_f32(const float* in, int64_t n, bf16_t* hi, bf16_t* mid, bf16_t* lo,
                            hipStream_t st);

// V = 1 with probability v_init else 0, from Philox-4x32-10 keyed by (seed, sample)
hipError_t launch_stochastic_v(const void* W, bool w_bf16, int64_t n, const float* s_global, const uint8_t* scales,
                               uint64_t seed, uint32_t sample, float* V, hipStream_t st);
// delta = bf16(W_final(V) - W) for the hardened V; clears the forward tag in guard_slot (delta replaces that forward)
hipError_t launch_hardened_delta(const void* W, bool w_bf16, int64_t n, const float* s_global, const uint8_t* scales,
                                 const float* V, bf16_t* delta, uint32_t* guard_slot, hipStream_t st);

// ---- Stage-2 objective on given logits / hidden states (faar_stage2.hip) -------------------
struct Stage2Args {
  const void *Z_fp, *Z_q; bool z_bf16; int64_t T, vocab; float tau, kl_scale;
  const void *H_fp, *H_q; bool h_bf16; int64_t D; float mse_scale;
  const float* round_losses; int64_t n_layers; float lambda_kl, lambda_round;
  void *dZ_q, *dH_q;          // nullable outputs, dtypes of Z and H
  double *kl_rows, *mse_partials;  // workspace: T and stage2_mse_blocks(T*D) doubles
  float* losses;              // [4]: KL, MSE, Round-Loss sum, total
};
int64_t stage2_mse_blocks(int64_t n);
hipError_t launch_stage2(const Stage2Args& a, hipStream_t st);

// ---- glue between the linears of a block (faar_block.hip); activations and gradients bf16, D and n multiples of 8 ----
hipError_t launch_rmsnorm_fwd(const void* X, bool x_bf16, int64_t T, int64_t D, const float* g, float eps, bf16_t* H,
                              float* rstd, hipStream_t st);
hipError_t launch_rmsnorm_bwd(const bf16_t* dH1, const bf16_t* dH2, const bf16_t* dH3, const void* X, bool x_bf16, int64_t T,
                              int64_t D, const float* g, const float* rstd, const bf16_t* d_res, bf16_t* dX, hipStream_t st);
hipError_t launch_silu_mul_fwd(const bf16_t* P, const bf16_t* Q, int64_t n, bf16_t* A, hipStream_t st);
hipError_t launch_silu_mul_bwd(const bf16_t* dA, const bf16_t* P, const bf16_t* Q, int64_t n, bf16_t* dP, bf16_t* dQ,
                               hipStream_t st);
hipError_t launch_residual_add(const void* X, bool x_bf16, const bf16_t* Dm, int64_t n, bf16_t* Y, hipStream_t st);
int64_t block_loss_blocks(int64_t n);
hipError_t launch_block_output_loss(const void* X, bool x_bf16, const bf16_t* Dm, const void* Yfp, bool y_bf16, int64_t n,
                                    float two_scale, bf16_t* Y, bf16_t* dY, double* partials, hipStream_t st);

// ---- rotary embedding and the attention core (faar_attention.hip); T = n_seq * S, S % 32 == 0, dh 64 or 128 ----
// Y (may be X) = every head of X [T, H * dh] rotated by the angles of the tables' row t % S (cos_t, sin_t [S, dh / 2])
hipError_t launch_rope(const bf16_t* X, int64_t T, int64_t H, int64_t dh, const float* cos_t, const float* sin_t, int64_t S,
                       bool inverse, bf16_t* Y, hipStream_t st);
// Vt = V transposed, [n_kv * dh, Tp]; lse [n_q, T]
hipError_t launch_attention_fwd(const bf16_t* Q, const bf16_t* K, const bf16_t* Vt, int64_t n_seq, int64_t S, int64_t n_q,
                                int64_t n_kv, int64_t dh, int64_t Tp, float scale, bf16_t* O, float* lse, hipStream_t st);
// Qt, dOt [n_q * dh, Tp], Kt [n_kv * dh, Tp]: transposed copies; delta [n_q, T] scratch
hipError_t launch_attention_bwd(const bf16_t* dO, const bf16_t* Q, const bf16_t* K, const bf16_t* V, const bf16_t* O,
                                const float* lse, const bf16_t* Qt, const bf16_t* Kt, const bf16_t* dOt, float* delta,
                                int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv, int64_t dh, int64_t Tp, float scale,
                                bf16_t* dQ, bf16_t* dK, bf16_t* dV, hipStream_t st);

// ---- bf16 MFMA GEMMs (faar_gemm.hip) ------------------------------------------------------
// All GEMMs are "NT": acc[m][n] = sum_k A[m][k] * B[n][k], A [M, lda], B [N, ldb] bf16 row-major
// with the contraction index contiguous, lda/ldb/Kd multiples of 8.
struct GemmDims { int64_t M, N, Kd, lda, ldb; };

// Residual epilogue (Table 2 steps 9-10): R = x_scale * acc - C(m, n), C in the row-group-interleaved layout
// [ceil(M/4)][N][4], x_scale a device scalar (null = 1); partial sum of R^2 per tile (double);
// dYt[n][m] = bf16(two_alpha * R) with row stride ldt (rows n < N, columns m < ldt, zero for m >= M);
// dY (nullable) [M, N] the same values un-transposed.
// C == nullptr: the V-dependent part alone -- A = x_scale * acc, sum A^2 per tile, dYt = bf16(two_alpha * A) (dY must
// be null); with dYt == nullptr too, only the sums are produced.
// guard: when its slot is set, workgroup 0 first compares the stored forward tag with guard.expect (see ForwardTag)
// warm (nullable), warm_bytes: a buffer the BK = 64 kernels read on the side during the main loop and discard, so that the
// next kernel finds it in the last-level cache (X_q^T for the dW GEMM); 16-byte aligned, whole KB are read
hipError_t launch_gemm_residual(const bf16_t* A, const bf16_t* B, GemmDims d, const float* C, const float* x_scale,
                                float two_alpha, bf16_t* dYt, int64_t ldt, bf16_t* dY,
                                double* mse_partials, int64_t* n_partials, const ForwardGuard& guard, const void* warm,
                                int64_t warm_bytes, hipStream_t st);
// The C == nullptr form with dY stored token-major instead of transposed: dY[m][n] = bf16(two_alpha * x_scale * acc), [M, N]
// row-major, N a multiple of 8 (for the token-major dW GEMM); the same per-item sums and the same tile plan
hipError_t launch_gemm_residual_rows(const bf16_t* A, const bf16_t* B, GemmDims d, const float* x_scale, float two_alpha,
                                     bf16_t* dY, double* mse_partials, int64_t* n_partials, const ForwardGuard& guard,
                                     hipStream_t st);
// number of per-work-item loss partials the residual GEMM writes for these sizes
int64_t gemm_residual_partials(int64_t M, int64_t N, int64_t Kd);
// Plain float32 output with the contraction split n_split ways: out[s][m][n] (split stride M*N).
hipError_t launch_gemm_f32(const bf16_t* A, const bf16_t* B, GemmDims d, float* out, int n_split,
                           hipStream_t st);
int choose_split(int64_t M, int64_t N, int64_t Kd);
// The same product from token-major operands: out[s][m][n] = sum_t A[t][m] * B[t][n], A [T, lda], B [T, ldb] (the contraction
// index is the row index; d.Kd = T).  Only where gemm_tn_usable says so (T a multiple of 64, M and N multiples of 8, a shape
// the planner gives 256 x 256 tiles); n_split = choose_split(M, N, T) as for launch_gemm_f32.
bool gemm_tn_usable(int64_t M, int64_t N, int64_t T);
// 0 not usable, 1 256 x 256 tiles, 2 192 x 256, 3 256 x 192 (the last two only with fill_device: the kernel runs alone)
int gemm_tn_tiles(int64_t M, int64_t N, int64_t T, bool fill_device);
hipError_t launch_gemm_f32_tn(const bf16_t* A, const bf16_t* B, GemmDims d, float* out, int n_split, bool fill_device,
                              hipStream_t st);
// The kernel variant, tile shape and contraction split the launchers above pick for an M x N x Kd product
// (kind: 0 generic, 1 / 2 / 3 the BK = 32 kernels with 256x256 / 256x128 / 128x128 tiles, 4 / 5 the BK = 64
// kernels with 256x256 / 256x128 tiles).  Pure host function.
enum { kGemmEpiResidual = 0, kGemmEpiF32 = 1, kGemmEpiSub = 2, kGemmEpiBf16 = 3, kGemmEpiNone = 4, kGemmEpiGram = 5 };
struct GemmPlanInfo { int kind, bm, bn, n_split; };
GemmPlanInfo gemm_plan_info(int epilogue, int64_t M, int64_t N, int64_t Kd);
// C_out(m, n) = (first ? Y[m][n] : C_out(m, n)) - x_scale * acc   (Y bf16 or float32 row-major; C_out interleaved)
hipError_t launch_gemm_sub(const bf16_t* A, const bf16_t* B, GemmDims d, const void* Y, bool y_bf16,
                           bool first, float* C_out, const float* x_scale, hipStream_t st);
// Measurement variants of the main loop (mode 0 whole, 1 matrix instructions only, 2 copies only) on an M x N x Kd
// product, no output: clocks[2 i], clocks[2 i + 1] = shader-clock cycles and 100 MHz ticks of work item i.
hipError_t launch_gemm_probe(int mode, const bf16_t* A, const bf16_t* B, GemmDims d, unsigned long long* clocks,
                             int64_t capacity, float* sink, int* kind, int64_t* items, hipStream_t st);
// Gram-matrix form of a step: delta [O, K] times gram [K, K] (symmetric, so the NT product is delta * gram);
// out[split][o][k] = two_alpha * x_scale * (acc + (split 0) delta[o][k] * diag_lo[k]); partials[item] = the item's share of
// x_scale^2 <delta gram, delta>; n_split must be choose_split_gram(O, K); guard as in launch_gemm_residual
int choose_split_gram(int64_t O, int64_t K);
int64_t gemm_gram_partials(int64_t O, int64_t K);
hipError_t launch_gemm_gram(const bf16_t* delta, const bf16_t* gram, int64_t O, int64_t K, const float* diag_lo,
                            const float* x_scale, float two_alpha, float* out, int n_split, double* partials,
                            int64_t* n_partials, const ForwardGuard& guard, hipStream_t st);
// out[m][n] = bf16(scale * acc), scale a device scalar (null = 1)
hipError_t launch_gemm_bf16(const bf16_t* A, const bf16_t* B, GemmDims d, bf16_t* out, const float* scale,
                            hipStream_t st);

}  // namespace faar
