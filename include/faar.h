/*
 * faar.h -- C ABI of the FAAR (Format-Aware Adaptive Rounding for NVFP4) per-layer
 * rounding-optimisation path for AMD MI355X (gfx950).
 *
 * Conventions, valid for every entry point unless its comment says otherwise
 * ---------------------------------------------------------------------------
 *  - A linear layer's weight W is [O, K] row-major (out_features x in_features, K contiguous).
 *    Calibration activations are [T, K] row-major, layer outputs [T, O] row-major.
 *    K must be a multiple of 16: a scale block is 16 consecutive weights along K and never
 *    straddles rows (paper Sec. 3.1: blocks of 16 elements, one FP8-E4M3 scale each, one FP32
 *    scale per tensor).
 *  - Every pointer is a DEVICE pointer owned by the caller, except `opt` of faar_layer_step
 *    (a host pointer, read during the call).  The library never allocates, frees or copies to
 *    the host, and never synchronises: all work is enqueued on `stream` (a hipStream_t passed
 *    as void*; NULL is the default stream).  Scalar results are written to device memory.
 *  - Device buffers must be 16-byte aligned.  Buffers must not overlap unless stated.
 *  - Scratch memory comes from a caller-provided workspace `ws` of at least
 *    faar_workspace_bytes(op, ...) bytes; its contents are undefined after the call (one exception:
 *    faar_layer_step can leave the next step's forward outputs there, see beta_next).  A FAAR_OP_LAYER_STEP
 *    workspace must be 16-byte aligned.
 *  - Return value: FAAR_OK, or a negative error code, in which case NOTHING was launched.
 *    FAAR_E_HIP means a HIP call failed; the raw hipError_t is kept per host thread and read
 *    with faar_last_hip_error().  No other global mutable state exists.
 *  - E2M1 nibble: bit 3 sign, bits 2..0 magnitude code 0..7 <-> {0, .5, 1, 1.5, 2, 3, 4, 6}
 *    (the node set of Sec. 3.1).  Packed codes are [O, K/2] bytes, element 2j of a row in the low
 *    nibble of byte j.  Block scales are [O, K/16] bytes, row-major, un-swizzled, always in
 *    0x00..0x7E (non-negative, finite).
 *  - Decision arithmetic (everything that ends in a byte, a nibble or a bit, and V_init) is IEEE
 *    float32, round-to-nearest-even, in the operation order documented at each entry point, so
 *    that results are reproducible bit for bit.  NaN/Inf in W are not supported (undefined codes).
 */
#ifndef FAAR_H_
#define FAAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FAAR_F32 = 0, FAAR_BF16 = 1 } faar_dtype;

enum {
  FAAR_OK = 0,
  FAAR_E_NULL = -1,      /* a required pointer is NULL */
  FAAR_E_SHAPE = -2,     /* O, K or T <= 0, K % 16 != 0, or a size beyond a documented limit */
  FAAR_E_DTYPE = -3,     /* dtype value not supported for that argument */
  FAAR_E_WORKSPACE = -4, /* ws == NULL or ws_bytes too small */
  FAAR_E_HIP = -5,       /* a HIP runtime call failed; see faar_last_hip_error() */
  FAAR_E_ARG = -6,       /* scalar out of domain (beta <= 0, lr < 0, non-finite), unknown flag or
                            unaligned pointer */
  FAAR_E_UNSUPPORTED = -7 /* combination of arguments not implemented */
};

/* flags */
enum {
  FAAR_SGLOBAL_GIVEN = 1u << 0, /* faar_quant_rtn: *s_global is an input instead of an output */
  FAAR_EMIT_DELTA = 1u << 1,    /* faar_softquant_fwd_bwd: Wt receives W_q - W instead of W_q */
  FAAR_WS_CHAINED = 1u << 2,    /* faar_workspace_bytes / faar_layer_step: size the workspace for a
                                   step that takes dY_ext and/or produces dX */
  FAAR_WS_FORWARD_READY = 1u << 3, /* faar_layer_step: the workspace already holds this step's soft-quantised
                                   weights, left there by the previous step (its beta_next) */
  FAAR_STEP_JOINT = 1u << 6,    /* faar_layer_step: the layer is one link of a jointly optimised chain (see there) */
  FAAR_STEP_XT_READY = 1u << 7, /* faar_layer_step with FAAR_STEP_JOINT: Xt already holds the transpose of Xq (written by the
                                   joint step of another linear that reads the same activations): do not transpose again */
  FAAR_STEP_WHOLE_DEVICE = 1u << 8, /* faar_layer_step: nothing else runs on the device beside this step.  The token-major
                                   dW GEMM then takes the tile that fills every compute unit (192 x 256 or 256 x 192 where
                                   256 x 256 tiles would leave units idle: 6144 x 2048 is 192 of those, but 256 of 192 x
                                   256).  Without the flag it stays on 256 x 256 tiles, which do more work per byte moved:
                                   what counts when kernels of other streams take up the idle units anyway.  Same sums in
                                   the same order either way: results are identical bit for bit. */
  FAAR_WS_GRADIENT_CONSTANT = 1u << 5, /* faar_workspace_bytes(FAAR_OP_LAYER_PREPARE): size the workspace for a call that
                                   also produces H and c_norm2 */
  FAAR_DQ_IN_UNITS = 1u << 4    /* faar_quant_rtn: W_dq receives sign * node * E4M3 scale, i.e. the dequantised
                                   value in units of s_global -- an exact product (at most 6 significant bits),
                                   so exactly representable in bf16 */
};

/* operations, for faar_workspace_bytes */
enum {
  FAAR_OP_QUANT_RTN = 0,
  FAAR_OP_INIT_V = 1,
  FAAR_OP_SOFTQUANT = 2,
  FAAR_OP_LAYER_PREPARE = 3,
  FAAR_OP_LAYER_STEP = 4,
  FAAR_OP_HARDEN_PACK = 5,
  FAAR_OP_STAGE2_LOSSES = 6, /* faar_workspace_bytes(op, O = vocabulary, K = hidden size, T = tokens, 0) */
  FAAR_OP_QUANT_RTN_BATCH = 7, /* independent of the tensors: pass any valid O, K (e.g. 16, 16) */
  FAAR_OP_LINEAR_FORWARD = 8,
  FAAR_OP_BLOCK_OUTPUT_LOSS = 9, /* faar_workspace_bytes(op, O = D (row length), K = 16, T = rows, 0) */
  FAAR_OP_ATTENTION_FWD = 10, /* faar_workspace_bytes(op, O = n_q * dh, K = n_kv * dh, T = tokens, 0) */
  FAAR_OP_ATTENTION_BWD = 11, /* likewise */
  FAAR_OP_GRAM_PREPARE = 12,  /* faar_workspace_bytes(op, O = K, K, T, 0) */
  FAAR_OP_LAYER_STEP_GRAM = 13 /* faar_workspace_bytes(op, O, K, T = 1, 0) */
};

/* kernels of the path, for faar_time_kernel */
enum {
  FAAR_K_NONE = 0,
  FAAR_K_SOFTQUANT_FWD = 1,  /* W_q - W                                 (faar_layer_step) */
  FAAR_K_GEMM_RESIDUAL = 2,  /* X_q (W_q - W)^T - C, loss, dY           (faar_layer_step) */
  FAAR_K_GEMM_DW = 3,        /* dY^T X_q                                (faar_layer_step) */
  FAAR_K_GEMM_DX = 4,        /* dY W_q                                  (faar_layer_step) */
  FAAR_K_BWD_ADAM = 5,       /* dV, Round Loss, Adam, clip              (faar_layer_step) */
  FAAR_K_QUANT_RTN = 6,      /* the quantise kernel of faar_quant_rtn (not its amax pass) */
  FAAR_K_INIT_V = 7,
  FAAR_K_HARDEN_PACK = 8,
  FAAR_K_STAGE2_KL = 9,      /* the three launches of faar_stage2_losses, bracketed together */
  FAAR_K_GEMM_C = 10,        /* Y_fp - X_q W^T of faar_layer_prepare (faar_gemm_plan only: it has no time bracket) */
  FAAR_K_GEMM_FWD = 11,      /* X_q W_q^T of faar_linear_forward */
  FAAR_K_ATTENTION_FWD = 12, /* the attention kernel of faar_attention_fwd (not the transpose before it) */
  FAAR_K_ATTENTION_BWD = 13, /* the three kernels of faar_attention_bwd (not the transposes before them) */
  FAAR_K_GEMM_GRAM = 14      /* (W_q - W) (X_q^T X_q), loss, gradient   (faar_layer_step_gram) */
};

/* GEMM kernel variants, as reported by faar_gemm_plan */
enum {
  FAAR_GEMM_GENERIC = 0,  /* register-staged 128x128 tile, any contraction length */
  FAAR_GEMM_L = 1,        /* contraction % 32 == 0: direct-to-LDS ring of 32-wide slices, 256x256 tile */
  FAAR_GEMM_M = 2,        /*   256x128 tile */
  FAAR_GEMM_S = 3,        /*   128x128 tile */
  FAAR_GEMM_L64 = 4,      /* contraction % 64 == 0: 64-wide slices, 256x256 tile */
  FAAR_GEMM_M64 = 5       /*   256x128 tile */
};

/* Library version, MAJOR*10000 + MINOR*100 + PATCH.  Pure host function. */
int faar_version(void);

/* hipError_t of the last failed HIP call made by this host thread (0 if none). */
int faar_last_hip_error(void);

/* Measurement hook for benchmarks: while `which` != FAAR_K_NONE, every launch of that kernel made
 * by this host thread is bracketed by hipEventRecord(start_event) / hipEventRecord(stop_event) on
 * the launch stream (hipEvent_t handles created by the caller with timing enabled).  Pass
 * FAAR_K_NONE to switch it off.  Returns FAAR_E_ARG for an unknown kernel or missing events. */
int faar_time_kernel(int which, void* start_event, void* stop_event);

/* The same hook with a ring of n event pairs, so that a kernel can be timed over many launches issued back to back
 * (no host synchronisation between them: the chip stays at the clocks it runs a real job at).  events: HOST array of
 * 2 n hipEvent_t handles (start 0, stop 0, start 1, ...), copied by the call; bracket number i (counted from this call)
 * uses pair i % n.  n in [1, 4096].  faar_time_kernel_count returns how many brackets were recorded since the hook was
 * last set. */
int faar_time_kernel_ring(int which, void* const* events, int n);
int64_t faar_time_kernel_count(void);

/* Workspace size in bytes that `op` needs for these sizes (T is ignored by ops that take no
 * activations; `flags` as passed to the op).  Pure host function; returns 0 for an unknown op or
 * invalid sizes. */
size_t faar_workspace_bytes(int op, int64_t O, int64_t K, int64_t T, uint32_t flags);

/* Number of ways faar_layer_step splits the token contraction of the dW GEMM for these sizes (the
 * float32 partial products are summed by the kernel that consumes them).  Pure host function. */
int faar_dw_split(int64_t O, int64_t K, int64_t T);

/* Which kernel variant, output tile and contraction split the library uses for one of the GEMMs of a layer of
 * these sizes: which = FAAR_K_GEMM_RESIDUAL (T x O x K), FAAR_K_GEMM_DW (O x K x padded T; the only one that may
 * split its contraction), FAAR_K_GEMM_DX (T x K x O), FAAR_K_GEMM_C (T x O x K, in faar_layer_prepare) or FAAR_K_GEMM_FWD (T x O x K, in
 * faar_linear_forward).
 * out[0..3] = variant (FAAR_GEMM_*), tile rows, tile columns, contraction splits.  Pure host function; lets tests
 * prove that their cases reach every variant. */
int faar_gemm_plan(int which, int64_t O, int64_t K, int64_t T, int32_t* out);

/* Measurement hook for benchmarks: runs the main loop of the library's GEMM kernel on the product
 * acc[m][n] = sum_k A[m][k] B[n][k]  (A [M, Kd], B [N, Kd] bf16 row-major, Kd a multiple of 64) WITHOUT storing a result,
 * whole (mode 0), with only its matrix instructions (mode 1: the LDS stages are filled once and never refilled) or
 * with only its global-to-LDS copies (mode 2).  Work item i (one output tile) writes the shader-clock cycles it took
 * to clocks[2 i] and the ticks of the constant 100 MHz counter to clocks[2 i + 1]: their ratio is the clock the
 * compute units ran at.  info (HOST, out): [0] work items, [1] kernel variant (FAAR_GEMM_*).  capacity: pairs that
 * fit in clocks (FAAR_E_WORKSPACE if too few); sink: one device float, never written for real operands.
 * mode + 4: the same three loops of the token-major kernel (the dW GEMM of a step whose operands are used as the layers
 * produce them): the two buffers are then read as A [Kd, M] and B [Kd, N] -- the same bytes, the contraction index as the row
 * index -- where faar_dw_token_major(M, N, Kd, 0) is non-zero.  mode 12: the whole token-major loop on 192 x 256 or 256 x 192
 * tiles, whichever covers the M x N outputs with fewer tiles.
 * FAAR_E_UNSUPPORTED when the product would not run on the 64-wide-slice kernels, or not in the token-major form asked for. */
int faar_gemm_probe(int mode, int64_t M, int64_t N, int64_t Kd, const void* A, const void* B,
                    unsigned long long* clocks, int64_t capacity, float* sink, int32_t* info, void* stream);

/* Padded leading dimension (in elements) of the transposed activations Xt written by
 * faar_layer_prepare and read by faar_layer_step: T rounded up to a multiple of 64. */
int64_t faar_padded_tokens(int64_t T);

/* Non-zero when a step of an O x K layer over T tokens that is given an upstream gradient (dY_ext) runs its dW GEMM on the
 * token-major operands as they are -- dY_ext [T, O] and Xq [T, K], no transposed copies -- else 0 (T not a multiple of 64, O or
 * K not a multiple of 8, or a shape too small for 256-wide tiles).  The value names the tile of that GEMM for a step with these
 * `flags` (only FAAR_STEP_WHOLE_DEVICE matters): 1 256 x 256, 2 192 x 256, 3 256 x 192.  Such a step neither reads nor, with
 * FAAR_STEP_JOINT, writes Xt.  The same holds for a step that derives its own gradient with the constant carried as H
 * (faar_layer_prepare_h) and no dX requested: its residual GEMM then leaves dY token-major and Xt is not read either.  Pure
 * host function. */
int faar_dw_token_major(int64_t O, int64_t K, int64_t T, uint32_t flags);

/*
 * Round-to-nearest NVFP4 quantisation of a tensor -- the baseline rounding of Sec. 3.1/3.2 and
 * the two-level scaling of Table 2 step 2.
 *
 *   amax      = max |w|                         ; s_global = amax / 2688   (2688 = 6 * 448; 1 if amax == 0)
 *   a_b       = max |w| over the block          ; byte = E4M3_rne_sat((a_b / 6) / s_global)
 *   s         = E4M3_value(byte) * s_global     ; w~ = |w| / s   (0 if s == 0)
 *   k_lo      = #{node in {.5,1,1.5,2,3,4} : node <= w~}   (interval [N[k_lo], N[k_lo+1]])
 *   v_init    = clamp((w~ - N[k_lo]) / (N[k_lo+1] - N[k_lo]), 0, 1)
 *   nibble    = signbit(w) << 3 | (w == 0 ? 0 : k_lo + (v_init >= 0.5))   -- exact midpoints go up
 *
 *   W        in  [O*K] of dtype wdt (FAAR_F32 or FAAR_BF16)
 *   s_global out float[1] (in, if flags & FAAR_SGLOBAL_GIVEN)
 *   scales   out uint8[O*K/16]
 *   codes    out uint8[O*K/2]
 *   W_dq     out, nullable: dequantised weights sign * N[code] * E4M3_value(byte) * s_global,
 *            dtype wdt (float32 product rounded once; then to bf16 if wdt is bf16).  With
 *            FAAR_DQ_IN_UNITS the factor s_global is left out and the value is exact: quantising
 *            ACTIVATIONS this way (tensor [T, K], blocks along K) gives the Xq / x_scale = s_global pair
 *            that faar_layer_prepare and faar_layer_step take.
 *   ws       FAAR_OP_QUANT_RTN workspace
 */
int faar_quant_rtn(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                   float* s_global, uint8_t* scales, uint8_t* codes, void* W_dq,
                   uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/*
 * Initial rounding variables -- Eq. 4 / Table 2 steps 2-5: V = v_init as defined above, from W and
 * the scales produced by faar_quant_rtn.
 *
 *   V           out float[O*K]
 *   floor_codes out, nullable uint8[O*K/2]: packed nibbles signbit(w) << 3 | k_lo
 */
int faar_init_v(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                const float* s_global, const uint8_t* scales,
                float* V, uint8_t* floor_codes, void* stream);

/*
 * Soft quantisation forward, and (when dWt != NULL) its backward -- Eq. 2, Eq. 3, and the
 * V-gradient of Eq. 5 (Table 2 steps 6-7 and 11-12).
 *
 *   h    = 1 / (1 + exp(-beta (v - 1/2)))
 *   W_q  = sign(w) (N[k_lo] + h (N[k_lo+1] - N[k_lo])) s          (sign(0) = 0)
 *   Wt   out bf16[O*K]: W_q, or W_q - W with FAAR_EMIT_DELTA, rounded to bf16
 *   dV   = dWt * sign(w) s (N[k_lo+1] - N[k_lo]) beta h (1 - h) + lambda_round / (O*K) * (4 - 8 v)
 *   round_loss = (1 / (O*K)) sum (1 - (2 v - 1)^2)
 *
 *   V          in  float[O*K]
 *   dWt        in, nullable float[O*K]: dL/dW_q; when NULL only the forward runs
 *   dV         out float[O*K], required iff dWt != NULL
 *   round_loss out, nullable float[1] (written only when dWt != NULL)
 *   beta > 0 and finite.  ws: FAAR_OP_SOFTQUANT workspace.  float32 arithmetic.
 */
int faar_softquant_fwd_bwd(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                           const float* s_global, const uint8_t* scales,
                           const float* V, float beta, void* Wt,
                           const float* dWt, float lambda_round, float* dV, float* round_loss,
                           uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/*
 * faar_softquant_fwd_bwd for callers that cannot hand over a workspace because they cannot allocate one: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without ws /
 * ws_bytes, same kernels, same results bit for bit.  The per-block Round-Loss partial sums live in a 512 KB array
 * that is part of the library's code object (each GPU the library runs on holds its copy until the process ends),
 * which bounds the tensor: O * K <= 2^27 weights, else FAAR_E_SHAPE.  The call allocates and frees nothing and does
 * not synchronise.  The first call with dWt != NULL on each device looks up that device's copy of the array (not an
 * allocation; make that call outside stream capture).  Every partial sum a call reads was written earlier in the same
 * call, so nothing needs clearing between calls; but all calls on one GPU share the one array: calls that overlap on
 * a GPU (two streams, two host threads) race on it and must be serialised by the caller.
 */
int faar_softquant_fwd_bwd_static(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                                  const float* s_global, const uint8_t* scales,
                                  const float* V, float beta, void* Wt,
                                  const float* dWt, float lambda_round, float* dV, float* round_loss,
                                  uint32_t flags, void* stream);

/*
 * Per-layer constants of the Stage-1 objective (Eq. 5, Table 2 steps 8-9), computed once before
 * the first faar_layer_step of a layer:
 *
 *   Xt = Xq^T                as bf16 [K, Tp], Tp = faar_padded_tokens(T), columns T..Tp-1 zero
 *   C  = Y_fp - Xq W^T       as float [ceil(T/4), O, 4]: element (t, o) at ((t / 4) * O + o) * 4 + t % 4,
 *                            rows T..4*ceil(T/4)-1 zero.  (Four consecutive tokens of one output channel are
 *                            what one lane of the step's GEMM epilogue holds: one 16-byte access.)  bf16
 *                            products are exact, float32 accumulation; a float32 W is split into three
 *                            bf16 terms.  The buffer holds 4 * ceil(T/4) * O floats.
 *
 * The residual of Eq. 5 is then  Xq W_q^T - Y_fp = Xq (W_q - W)^T - C,  which lets the step run its
 * GEMM on the small perturbation W_q - W without losing it to bf16 rounding of W_q.
 *
 * and the interval of every weight (Table 2 step 3; frozen with W and the scales), cached so that the
 * steps need neither the division nor the node search:
 *
 *   icodes = uint8 [O*K/2], element 2j of a row in the low nibble: signbit(w) << 3 | (w == 0 ? 7 : k_lo)
 *
 * and, optionally, the part of the gradient that does not depend on V.  With A = x_scale Xq (W_q - W)^T the residual is
 * R = A - C, so  dL_mse/dW_q = (2 a R)^T X_q = (2 a A)^T X_q - 2 a C^T X_q  and  ||R||^2 = ||A||^2 - 2 <A, C> + ||C||^2
 * with <A, C> = x_scale <W_q - W, C^T Xq>  (a = mse_scale).  Given
 *
 *   H       = C^T Xq     as float [O*K]  (products of three bf16 terms of C with Xq: exact; float32 accumulation)
 *   c_norm2 = ||C||^2    as double[1]
 *
 * a step's residual GEMM reads no constant in its epilogue (4 bytes per output of Y less), at the price of reading H
 * (4 bytes per weight) in the pass that updates V: a saving whenever T > K, and always when the step's dY comes
 * from upstream.  H and c_norm2 are both NULL or both given; pass the same pair to faar_layer_step.
 *
 *   s_global, scales  as written by faar_quant_rtn
 *   Xq   in bf16[T*K]   -- the activations fed to the quantised path (X_q of Sec. 3.4), in units of
 *   x_scale in, nullable device float[1] (NULL = 1): X_q = x_scale * Xq.  NVFP4-quantised activations are
 *        passed exactly as Xq = node * block scale (bf16-exact) and x_scale = their tensor scale.
 *   Y_fp in [T*O] of dtype ydt -- the frozen full-precision layer output X W^T.  Y_fp and C may both be NULL (a layer
 *        that is only stepped jointly, FAAR_STEP_JOINT): then only Xt and icodes are produced
 *   ws   FAAR_OP_LAYER_PREPARE workspace (queried with FAAR_WS_GRADIENT_CONSTANT when H is wanted; needed for a
 *        float32 W or with H)
 */
int faar_layer_prepare(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                       const float* s_global, const uint8_t* scales,
                       const void* Xq, const float* x_scale, const void* Y_fp, faar_dtype ydt, int64_t T,
                       void* Xt, float* C, uint8_t* icodes, float* H, double* c_norm2,
                       void* ws, size_t ws_bytes, void* stream);

/* Adam hyper-parameters; t is the 1-based index of the step being taken. */
typedef struct {
  float lr, beta1, beta2, eps;
  int32_t t;
} faar_adam;

/*
 * One rounding-optimisation step for one linear layer -- Table 2 steps 6-13, Eq. 5:
 *
 *   W_q(V) by Eq. 2-3;  R = Xq W_q^T - Y_fp;  L_mse = mse_scale * ||R||_F^2
 *   L_round = (1/N) sum (1 - (2 v - 1)^2);  L = L_mse + lambda_round * L_round
 *   dY = 2 mse_scale R (or dY_ext);  G = dY^T Xq;  dV as in faar_softquant_fwd_bwd with dWt = G
 *   Adam (bias-corrected, no weight decay) on V with state (adam_m, adam_v), then V clipped to [0, 1].
 *
 * GEMMs run on the bf16 matrix cores with float32 accumulation; three tensors are rounded to bf16
 * where they are stored: W_q - W, dY and dX.  Everything else is float32; loss sums are
 * accumulated in a fixed order (results are bit-reproducible run to run).
 *
 *   V, adam_m, adam_v   in/out float[O*K]
 *   Xq, x_scale, Xt, C, icodes   as for / from faar_layer_prepare
 *   H, c_norm2          nullable pair from faar_layer_prepare.  When given, the step uses the split form described
 *                       there: what is stored (and rounded to bf16) as dY is 2 a A instead of 2 a (A - C), and H
 *                       supplies the rest -- the same loss and gradient with one rounding point moved, so results
 *                       agree with the H-less form to rounding, not bit for bit.  With dY_ext the residual GEMM then
 *                       only sums the loss.  Ignored (the C form is used) when dX is wanted without dY_ext.
 *   dY_ext              in, nullable bf16[T*O]: upstream gradient replacing the locally derived dY
 *   dX                  out, nullable bf16[T*K]: dY W_q
 *   opt                 HOST pointer
 *   losses              out float[3]: L_mse, L_round, L
 *   ws                  FAAR_OP_LAYER_STEP workspace (queried with FAAR_WS_CHAINED when dY_ext or dX
 *                       is given; that mode also requires O % 8 == 0)
 *   beta_next           0, or the beta of the step that follows: the pass that updates V then also
 *                       evaluates Eq. 2-3 on the updated V at beta_next and leaves W_q - W (and W_q when dX
 *                       is requested) with that V's Round-Loss partial sums in ws, saving the next step
 *                       its forward kernel.  Same arithmetic, same results bit for bit.
 *   flags               FAAR_STEP_JOINT: a joint (Stage-2-style) step -- Table 2 steps 15-17 and 23: the loss is computed
 *                       downstream of the layer (faar_block_output_loss, faar_stage2_losses) and arrives as dY_ext, which
 *                       is required; the layer's own reconstruction loss is not evaluated (losses[0] = 0, no residual GEMM;
 *                       C may be NULL, H must be).  The activations Xq are the quantised model's own and change with
 *                       every step: the call writes their transpose into Xt itself (Xt is then scratch of
 *                       K * faar_padded_tokens(T) bf16, not an input; with FAAR_STEP_XT_READY it is an input again: the
 *                       transpose of this very Xq, left by the joint step of a sibling linear) -- unless
 *                       faar_dw_token_major(O, K, T), in which case Xt is not touched at all: a sibling that follows such a
 *                       step and does need Xt must not be given FAAR_STEP_XT_READY.  dX is normally requested.
 *                       FAAR_WS_CHAINED is accepted and has no effect on the computation.
 *                       FAAR_WS_FORWARD_READY: skip the forward kernel and use what ws holds.  That is valid
 *                       when the previous call on this ws was step opt->t - 1 of the same layer (same W, scales,
 *                       V, shapes, dX requested or not) with beta_next equal to this call's beta, and neither V
 *                       nor ws has been written since.  Checked ON THE DEVICE as far as it can be: the step that
 *                       leaves a forward in ws tags it with (step index, beta, addresses of V, W and scales, O*K,
 *                       dX requested, H), every call that overwrites that forward (a step without the flag,
 *                       faar_hardened_loss) clears the tag, and a step consumes the tag it checks.  On a mismatch
 *                       -- a stale or foreign workspace, a repeated or skipped step, another beta -- the step
 *                       writes NaN to losses[0..2], leaves V, adam_m and adam_v untouched (dX is undefined) and
 *                       leaves no forward behind, so every later FAAR_WS_FORWARD_READY step fails the same way
 *                       until one runs without the flag.  The return code is still FAAR_OK (the check runs on the
 *                       stream).  A write to V's memory between the two steps is the one violation it cannot see.
 */
int faar_layer_step(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                    const float* s_global, const uint8_t* scales,
                    float* V, float* adam_m, float* adam_v,
                    const void* Xq, const float* x_scale, const void* Xt, const float* C, const uint8_t* icodes,
                    const float* H, const double* c_norm2, int64_t T, const void* dY_ext, void* dX,
                    float beta, float beta_next, float lambda_round, float mse_scale, const faar_adam* opt,
                    float* losses, uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/*
 * The same step (Table 2 steps 6-13, Eq. 5) for a layer whose calibration activations stay the same from step to step,
 * as in the layer-wise first stage (Sec. 3.5): an OPTIONAL algebraic rearrangement, not what faar_layer_step does.
 * With D = W_q - W, A = x_scale Xq D^T, R = A - C and the token Gram matrix  Gm = Xq^T Xq  (K x K, constant per layer),
 *
 *   ||R||_F^2   = x_scale^2 <D Gm, D> - 2 x_scale <D, H> + ||C||^2
 *   dL_mse/dW_q = 2 a (x_scale^2 D Gm - x_scale H)                       (a = mse_scale, H and ||C||^2 as above)
 *
 * i.e. the loss and gradient of faar_layer_step without forming the layer output: one O x K x K product per step instead
 * of two T x O x K ones (a gain when 2 T > K).  The layer output, dY and dX do not exist in this form.
 *
 * faar_gram_prepare, once per layer, from the Xt that faar_layer_prepare wrote:
 *   gram     out bf16 [K*K]:  Gm rounded to bf16 (float32 accumulation of exact bf16 products over the tokens)
 *   gram_lo  out float [K]:   what the rounding took from the diagonal, Gm[k][k] - bf16(Gm[k][k]) -- the one place where
 *                             the rounding errors of a row would add up coherently; the step adds it back in float32
 *   ws       FAAR_OP_GRAM_PREPARE workspace
 *
 * faar_layer_step_gram: arguments as for faar_layer_step; H and c_norm2 are required.  Rounded to bf16: W_q - W and Gm.
 * Results agree with faar_layer_step to the rounding of those, not bit for bit.  flags: 0 or FAAR_WS_FORWARD_READY (same
 * contract; a workspace is good for one of the two step functions only).  ws: FAAR_OP_LAYER_STEP_GRAM workspace.
 */
int faar_gram_prepare(const void* Xt, int64_t K, int64_t T, void* gram, float* gram_lo, void* ws, size_t ws_bytes,
                      void* stream);
int faar_layer_step_gram(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                         const float* s_global, const uint8_t* scales,
                         float* V, float* adam_m, float* adam_v, const float* x_scale, const uint8_t* icodes,
                         const float* H, const double* c_norm2, const void* gram, const float* gram_lo,
                         float beta, float beta_next, float lambda_round, float mse_scale, const faar_adam* opt,
                         float* losses, uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/*
 * Hardening and NVFP4 packing -- Eq. 7 and Table 2 steps 25-26:
 *   v_hat = (v >= 0.5) on the stored float32 V;  nibble = signbit(w) << 3 | (w == 0 ? 0 : k_lo + v_hat).
 *
 *   codes      out uint8[O*K/2]
 *   decisions  out, nullable uint8[O*K/8]: bit i of byte j is v_hat of flattened element 8j+i
 *   W_final    out, nullable, dtype wdt: dequantised final weights (as W_dq of faar_quant_rtn)
 *   flip_count out, nullable uint64[1]: number of weights whose nibble differs from
 *              round-to-nearest.  The kernel ADDS to it: the caller zeroes it first.
 */
int faar_harden_pack(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                     const float* s_global, const uint8_t* scales, const float* V,
                     uint8_t* codes, uint8_t* decisions, void* W_final,
                     unsigned long long* flip_count, void* stream);

/*
 * The set-up and tear-down operations over MANY weight tensors in one call -- Table 2 steps 2-5 and 25-26 for every
 * linear layer of a model (the loops "for each layer" of Table 2).  Most tensors of a model are small (a 2 M-weight
 * projection is a launch of a few microseconds, half of it ramp-up and tail), so these calls put up to 72 tensors into
 * one launch.  Results are identical, bit for bit, to calling faar_quant_rtn / faar_init_v / faar_harden_pack on each
 * tensor.  A tensor is described by its flat weight count n = O * K (a multiple of 16: scale blocks are 16 consecutive
 * weights and rows are multiples of 16, so the row structure does not matter here).
 *
 *   items   HOST array of n_items descriptors (read during the call); every pointer in it is a device pointer
 *   wdt     storage type of every W in the batch
 */
typedef struct {
  const void* W;      /* in  [n] */
  float* s_global;    /* [1]: out of faar_quant_rtn_batch (in with FAAR_SGLOBAL_GIVEN); in of the other two */
  uint8_t* scales;    /* [n/16]: out of faar_quant_rtn_batch; in of the other two */
  float* V;           /* [n]: out of faar_init_v_batch; in of faar_harden_pack_batch; ignored by faar_quant_rtn_batch */
  uint8_t* codes;     /* [n/2]: out of faar_quant_rtn_batch (round-to-nearest nibbles) and faar_harden_pack_batch (hardened
                         nibbles); faar_init_v_batch: nullable out, floor codes signbit(w) << 3 | k_lo */
  int64_t n;          /* weights in the tensor */
} faar_tensor;

/* ws: FAAR_OP_QUANT_RTN_BATCH workspace (not needed with FAAR_SGLOBAL_GIVEN) */
int faar_quant_rtn_batch(const faar_tensor* items, int64_t n_items, faar_dtype wdt, uint32_t flags,
                         void* ws, size_t ws_bytes, void* stream);
int faar_init_v_batch(const faar_tensor* items, int64_t n_items, faar_dtype wdt, void* stream);
int faar_harden_pack_batch(const faar_tensor* items, int64_t n_items, faar_dtype wdt, void* stream);

/*
 * One stochastic-rounding candidate (the trials of Sec. 3.2 / Table 1, which the paper reports without defining
 * them; this is the standard unbiased rule): V[i] = 1 with probability v_init[i] (Eq. 4), else 0.  Element i
 * (row-major) draws word i % 4 of Philox-4x32-10(counter = (i / 4 low, i / 4 high, sample, 0), key = (seed low,
 * seed high)); u = (word >> 8) * 2^-24; V[i] = (u < v_init[i]).  The result is a valid V for
 * faar_harden_pack and faar_hardened_loss.
 *
 *   V  out float[O*K]
 */
int faar_stochastic_v(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                      const float* s_global, const uint8_t* scales,
                      unsigned long long seed, uint32_t sample, float* V, void* stream);

/*
 * Reconstruction loss of the HARDENED weights of a rounding candidate -- Eq. 5's first term at the weights of
 * Eq. 7:  loss = mse_scale * || Xq W_final(V)^T - Y_fp ||_F^2  with W_final = sign * node * block scale * tensor
 * scale in float32 -- what an NVFP4 decoder produces from the bytes faar_harden_pack writes (not rounded to bf16).
 * Computed like a step's forward half: the bf16 matrix cores see W_final - W and the per-layer constant C.
 * V = V_init gives the loss of round-to-nearest.
 *
 *   Xq, x_scale, C  as for / from faar_layer_prepare
 *   loss            out device float[1]
 *   ws              FAAR_OP_LAYER_STEP workspace (contents destroyed: a prepared forward is lost)
 */
int faar_hardened_loss(const void* W, faar_dtype wdt, int64_t O, int64_t K,
                       const float* s_global, const uint8_t* scales, const float* V,
                       const void* Xq, const float* x_scale, const float* C, int64_t T,
                       float mse_scale, float* loss, void* ws, size_t ws_bytes, void* stream);

/*
 * The operations between the quantised linears of a transformer block, for joint steps -- Sec. 3.5 "Stage 2", Table 2
 * steps 15-17 and 23: the assembled quantised model runs forward and ONE loss is back-propagated into every layer's V.
 * The paper evaluates Llama3 / Qwen3 models; these are the parts of their blocks around the seven linears (pre-norm
 * RMSNorm, also over each head of q and k; rotary position embedding; causal attention with grouped key / value heads;
 * gated SiLU; residual connections) and the squared error of the block output, the block-level form of Eq. 6's
 * hidden-state term.  faar_block_joint_step at the end of this section enqueues all of it in one call.  Activations and gradients between kernels are bf16 [rows * row length],
 * row-major; arithmetic is float32.  A joint step of the MLP half of a block is then
 *
 *   h = faar_rmsnorm_fwd(x1);  p = faar_linear_forward(gate, h);  q = faar_linear_forward(up, h);
 *   a = faar_silu_mul_fwd(p, q);  d = faar_linear_forward(down, a);  (L, dy) = faar_block_output_loss(x1, d, y_fp)
 *   da = dX of faar_layer_step(down, Xq = a, dY_ext = dy, FAAR_STEP_JOINT);  (dp, dq) = faar_silu_mul_bwd(da, p, q)
 *   dh1 = dX of faar_layer_step(gate, Xq = h, dY_ext = dp, ...);  dh2 = dX of faar_layer_step(up, Xq = h, dY_ext = dq, ...)
 *   dx1 = faar_rmsnorm_bwd(dh1, dh2, NULL, x1, d_res = dy)
 *
 * and of the attention half before it (x1 = x + o_proj(attention); its output gradient is dx1)
 *
 *   h = faar_rmsnorm_fwd(x);  q, k, v = faar_linear_forward(q_proj / k_proj / v_proj, h)
 *   [Qwen3: q, k = faar_rmsnorm_fwd over each head's dh entries: rows = T * heads, row length dh]
 *   q, k = faar_rope(q), faar_rope(k);  (o, lse) = faar_attention_fwd(q, k, v);  d = faar_linear_forward(o_proj, o)
 *   x1 = faar_residual_add(x, d)                                   ... the MLP half above, which returns dx1 ...
 *   do = dX of faar_layer_step(o_proj, Xq = o, dY_ext = dx1, FAAR_STEP_JOINT)
 *   (dq, dk, dv) = faar_attention_bwd(do, q, k, v, o, lse);  dq, dk = faar_rope(dq / dk, inverse)  [, faar_rmsnorm_bwd per head]
 *   dh1, dh2, dh3 = dX of faar_layer_step(q_proj / k_proj / v_proj, Xq = h, dY_ext = dq / dk / dv, ...)
 *   dx = faar_rmsnorm_bwd(dh1, dh2, dh3, x, d_res = dx1)
 */

/* Y = x_scale * Xq W_q(V)^T in bf16 [T*O]: the soft-quantised linear of Eq. 2-3 applied to activations [T*K] (bf16).
 * W_q is rounded to bf16 for the matrix cores, as a bf16 model's fake-quantised forward does.  ws: FAAR_OP_LINEAR_FORWARD. */
int faar_linear_forward(const void* W, faar_dtype wdt, int64_t O, int64_t K, const float* s_global, const uint8_t* scales,
                        const float* V, float beta, const void* Xq, const float* x_scale, int64_t T, void* Y,
                        void* ws, size_t ws_bytes, void* stream);

/* h[t, i] = x[t, i] g[i] rstd[t],  rstd[t] = 1 / sqrt(mean_i x[t, i]^2 + eps).
 *   x in [T*D] of dtype xdt; g in float[D]; h out bf16 [T*D]; rstd out float[T] (kept for the backward).  D % 8 == 0. */
int faar_rmsnorm_fwd(const void* x, faar_dtype xdt, int64_t T, int64_t D, const float* g, float eps, void* h, float* rstd,
                     void* stream);

/* dx = rstd g dh - x rstd^3 / D * sum_i (x g dh) + d_res  with dh = dh1 + dh2 + dh3 (g is frozen: no gradient for it).
 *   dh1 in bf16 [T*D]; dh2, dh3 in, nullable (further consumers of h: the up projection next to the gate projection; the
 *   k and v projections next to the q projection), added in float32 in that order;
 *   d_res in, nullable bf16 [T*D]: the gradient arriving over the residual connection; dx out bf16 [T*D]. */
int faar_rmsnorm_bwd(const void* dh1, const void* dh2, const void* dh3, const void* x, faar_dtype xdt, int64_t T, int64_t D,
                     const float* g, const float* rstd, const void* d_res, void* dx, void* stream);

/* Rotary position embedding of those models ("rotate-half" form): for every head of x [T * H * dh] (bf16) and i < dh / 2,
 *   y[i] = x[i] c - x[i + dh/2] s,  y[i + dh/2] = x[i + dh/2] c + x[i] s,  c = cos_t[(t % S) * dh/2 + i], s likewise from sin_t.
 * The tables (float [S * dh/2], device) are the caller's: position p of a sequence, frequency i.  inverse != 0 rotates by the
 * opposite angle, which is the backward pass (the rotation is orthogonal).  y out bf16, may be x.  dh % 16 == 0. */
int faar_rope(const void* x, int64_t T, int64_t H, int64_t dh, const float* cos_t, const float* sin_t, int64_t S,
              int32_t inverse, void* y, void* stream);

/* Causal softmax attention with grouped key / value heads, per sequence:
 *   o[t, j] = sum_{t' <= t, same sequence} softmax_t'(scale q[t, j] . k[t', j / (n_q / n_kv)]) v[t', j / (n_q / n_kv)]
 *   q in bf16 [T * n_q * dh], k, v in bf16 [T * n_kv * dh], T = n_seq * S tokens, sequence b = rows b*S .. (b+1)*S - 1;
 *   o out bf16 [T * n_q * dh]; lse out float [n_q * T]: log of the softmax denominator per head and query (for the backward).
 *   S % 32 == 0, dh 64 or 128, n_q % n_kv == 0, scale > 0.  float32 arithmetic, probabilities rounded to bf16 as matrix-core
 *   operands.  ws: FAAR_OP_ATTENTION_FWD (a transposed copy of v). */
int faar_attention_fwd(const void* q, const void* k, const void* v, int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv,
                       int64_t dh, float scale, void* o, float* lse, void* ws, size_t ws_bytes, void* stream);

/* (dq, dk, dv) of the above for the output gradient d_o (bf16 [T * n_q * dh]); o and lse from the forward call.
 *   dq out bf16 [T * n_q * dh]; dk, dv out bf16 [T * n_kv * dh] (summed over the query heads of a group in a fixed order).
 *   ws: FAAR_OP_ATTENTION_BWD (transposed copies of q, k, d_o and one float per head and query). */
int faar_attention_bwd(const void* d_o, const void* q, const void* k, const void* v, const void* o, const float* lse,
                       int64_t n_seq, int64_t S, int64_t n_q, int64_t n_kv, int64_t dh, float scale, void* dq, void* dk,
                       void* dv, void* ws, size_t ws_bytes, void* stream);

/* y = x + d: the residual connection after the attention half (x of dtype xdt, d and y bf16, [n], n % 8 == 0; y may be d) */
int faar_residual_add(const void* x, faar_dtype xdt, const void* d, int64_t n, void* y, void* stream);

/*
 * One joint step of a whole block: the sequence of calls listed above -- attention half, residual, MLP half, squared error
 * of the block output against the full-precision block's, and the gradient back through all of it into the rounding
 * variables of the seven linears (one Adam update each, Sec. 3.5 "Stage 2"; Table 2 steps 15-17, 23) and into the block's
 * input -- enqueued by one call, on one stream, with every intermediate tensor in the caller's workspace.
 */
typedef struct {
  const void* W;           /* in  [O*K], dtype faar_block.wdt */
  const float* s_global;   /* in  device scalar */
  const uint8_t* scales;   /* in  [O*K/16] */
  const uint8_t* icodes;   /* in  [O*K/2]: interval codes from faar_layer_prepare */
  float* V;                /* inout [O*K] */
  float* adam_m;           /* inout [O*K] */
  float* adam_u;           /* inout [O*K] */
  float* losses;           /* out device [3]: 0, Round Loss of the V the step started from, lambda_round times it */
} faar_block_linear;

enum faar_block_slot { FAAR_LIN_Q = 0, FAAR_LIN_K, FAAR_LIN_V, FAAR_LIN_O, FAAR_LIN_GATE, FAAR_LIN_UP, FAAR_LIN_DOWN, FAAR_LIN_COUNT };

typedef struct {
  int64_t n_seq, S;        /* T = n_seq * S tokens; S % 32 == 0 */
  int64_t D;               /* model width; q_proj is [n_q*dh, D], k/v_proj [n_kv*dh, D], o_proj [D, n_q*dh] */
  int64_t n_q, n_kv, dh;   /* heads; dh 64 or 128 */
  int64_t F;               /* MLP width: gate/up_proj [F, D], down_proj [D, F] */
  float eps;               /* of every RMSNorm */
  float attn_scale;        /* of the attention scores; 0: 1 / sqrt(dh) */
  faar_dtype wdt;          /* dtype of all seven W */
  const float* g_attn;     /* in  float[D]: weights of the norm before the attention half */
  const float* g_mlp;      /* in  float[D]: ... before the MLP half */
  const float* g_q;        /* in  float[dh], nullable: per-head norm of q (Qwen3); g_q and g_k both or neither */
  const float* g_k;
  const float* cos_t;      /* in  float[S * dh/2]: rotary tables, see faar_rope */
  const float* sin_t;
  faar_block_linear lin[FAAR_LIN_COUNT];
} faar_block;

/* Bytes of workspace faar_block_joint_step needs for this block (0 if the description is invalid).  Pure host function. */
size_t faar_block_workspace_bytes(const faar_block* blk);

/*   blk         HOST pointer; read during the call only
 *   x           in  bf16 [T*D]: the block's input;  y_fp in bf16 [T*D]: the full-precision block's output
 *   mse_scale   the block loss is mse_scale * ||y - y_fp||_F^2
 *   beta, lambda_round, opt   as in faar_layer_step, for all seven linears (opt->t is the step index)
 *   block_loss  out device float[1]
 *   dx          out, nullable bf16 [T*D]: dL/dx (the first block of a model does not need it; the dX GEMMs of q, k, v
 *               are then skipped)
 *   ws          faar_block_workspace_bytes(blk) bytes, 256-byte aligned; contents are scratch
 * Errors as everywhere: a negative code and nothing is launched for argument errors found up front. */
int faar_block_joint_step(const faar_block* blk, const void* x, const void* y_fp, float mse_scale, float beta,
                          float lambda_round, const faar_adam* opt, float* block_loss, void* dx, void* ws, size_t ws_bytes,
                          void* stream);

/* a = SiLU(p) q = p sigmoid(p) q, all bf16 [n], n % 8 == 0 */
int faar_silu_mul_fwd(const void* p, const void* q, int64_t n, void* a, void* stream);

/* dp = da q s (1 + p (1 - s)),  dq = da p s,  s = sigmoid(p); all bf16 [n] */
int faar_silu_mul_bwd(const void* da, const void* p, const void* q, int64_t n, void* dp, void* dq, void* stream);

/* y = x + d (residual connection);  loss = mse_scale * ||y - y_fp||_F^2;  dy = 2 mse_scale (y - y_fp)  (bf16).
 *   x in [T*D] of dtype xdt (the block's input stream); d in bf16 [T*D] (the MLP's output); y_fp in [T*D] of dtype ydt
 *   (the full-precision block output); y out, nullable bf16; dy out bf16; loss out float[1]; ws: FAAR_OP_BLOCK_OUTPUT_LOSS */
int faar_block_output_loss(const void* x, faar_dtype xdt, const void* d, const void* y_fp, faar_dtype ydt, int64_t T, int64_t D,
                           float mse_scale, void* y, void* dy, float* loss, void* ws, size_t ws_bytes, void* stream);

/*
 * The Stage-2 objective evaluated on given outputs of the two models -- Sec. 3.5 "Stage 2", Eq. 6,
 * Table 2 steps 18-22 (the models that produce the logits and hidden states are not part of this library):
 *
 *   P_fp = softmax(Z_fp / tau),  P_q = softmax(Z_q / tau)           row-wise over the vocabulary
 *   L_KL    = kl_scale  * sum_t sum_j P_fp[t,j] (log P_fp[t,j] - log P_q[t,j])
 *   L_MSE   = mse_scale * ||H_fp - H_q||_F^2
 *   L_round = sum_l round_losses[l]
 *   L       = lambda_kl L_KL + L_MSE + lambda_round L_round
 *   dZ_q = lambda_kl kl_scale / tau (P_q - P_fp),   dH_q = 2 mse_scale (H_q - H_fp)    (gradients of L)
 *
 * The paper does not say whether the KL is summed or averaged over tokens, nor whether its "MSE" (printed as a
 * squared Frobenius norm) is a mean: kl_scale and mse_scale are arguments (1 = as printed).  float32 arithmetic
 * with hardware exp / log; row sums are accumulated online (one pass over the logits for the loss, a second
 * one only when dZ_q is requested) and all sums are finished in a fixed order in double.
 *
 * A logit of -inf (a masked vocabulary entry) has probability 0 and, by the convention 0 log 0 = 0, adds nothing to
 * the KL term where P_fp = 0; where P_fp > 0 and Z_q = -inf the KL is +inf.  A row whose logits are all -inf has no
 * softmax: its results are NaN.  +inf and NaN logits are not supported.
 *
 *   Z_fp, Z_q   in  [T * vocab] of dtype zdt; vocab a multiple of 8
 *   H_fp, H_q   in  [T * D] of dtype hdt; D a multiple of 8
 *   round_losses in, nullable device float[n_layers]
 *   dZ_q        out, nullable [T * vocab] of dtype zdt (rounded to bf16 if zdt is bf16)
 *   dH_q        out, nullable [T * D] of dtype hdt
 *   losses      out float[4]: L_KL, L_MSE, L_round, L
 *   ws          FAAR_OP_STAGE2_LOSSES workspace
 */
int faar_stage2_losses(const void* Z_fp, const void* Z_q, faar_dtype zdt, int64_t T, int64_t vocab, float tau,
                       float kl_scale, const void* H_fp, const void* H_q, faar_dtype hdt, int64_t D, float mse_scale,
                       const float* round_losses, int64_t n_layers, float lambda_kl, float lambda_round,
                       void* dZ_q, void* dH_q, float* losses, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FAAR_H_ */
