"""CPU oracle for the FAAR per-layer rounding-optimisation path (NVFP4).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the tests, the smoke
check and the benchmark's cpu-baseline leg may import it; the HIP library never
does, and shares no code, table or constant with it.

It is a plain, slow, step-by-step numpy transcription of what the method
computes, in the paper's order and notation:

  * NVFP4 format (Sec. 3.1 "NVFP4 Overview"): node set N = {0, .5, 1, 1.5, 2, 3, 4, 6} x sign,
    one FP8-E4M3 scale s_g per block of 16 weights, one FP32 tensor scale s_global.
  * Table 2 steps 2-5 / Eq. 4: normalise, FindInterval, V_init.
  * Eq. 2-3 / Table 2 steps 6-7: soft-quantised weight through h_beta(v) = sigmoid(beta (v - 1/2)).
  * Eq. 5 / Table 2 steps 8-13: reconstruction loss + Round Loss, gradient, update, clip to [0, 1].
  * Eq. 7 / Table 2 steps 25-26: hardening and the final NVFP4 weights.
  * Eq. 6 / Table 2 steps 18-22: the Stage-2 objective on given logits and last hidden states
    (temperature softmax, KL(P_fp || P_q), Frobenius MSE, sum of the layers' Round Losses).

Precision rules
  * "Decision arithmetic" -- everything that ends in an integer (scale byte, interval index,
    up/down bit, packed nibble) and V_init -- is evaluated in IEEE float32, round-to-nearest-even,
    one operation at a time, because an integer result has to be taken in one stated precision
    by every implementation that wants to agree on it.
  * All other floating point (sigmoid, GEMMs, losses, gradients, Adam) is float64.

Where the paper is silent the reading taken is stated at the function that needs it.

Parity pins (tests/test_oracle_*.py): node-set enumeration, E4M3 against an independent library
cast, bf16 rounding against a library cast, harden(V_init) == RTN, interpolation identity,
on-grid property, per-element brute-force nearest node, Round-Loss closed forms, beta -> inf limit,
central finite differences for dL/dV and dL/dX, brute force over all 2^n roundings of a tiny layer,
Adam first-step identity; for the Stage-2 losses: a library relative-entropy / log-softmax routine, the
two-class closed form, KL(P||P) = 0, shift and temperature invariances, central finite differences.  The scale derivation (tensor_scale / block_scale_bytes rounding mode) and
the nibble packing order are conventions the paper does not fix: they are pinned to the published
NVFP4 format description only through the structural invariants tested there.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
BLOCK = 16                       # weights per scale block (Sec. 3.1)

# ----------------------------------------------------------------------------------------------
# Number formats
# ----------------------------------------------------------------------------------------------

def e2m1_decode(code) -> np.ndarray:
    """4-bit E2M1 code -> value (float64).  bit3 sign, bits2..1 exponent (bias 1), bit0 mantissa.
    exponent 0 is subnormal: m * 0.5.  Enumerating the 16 codes gives the paper's node set
    (Sec. 3.1)."""
    code = np.asarray(code).astype(np.int64)
    s = (code >> 3) & 1
    e = (code >> 1) & 3
    m = code & 1
    mag = np.where(e == 0, 0.5 * m, np.exp2(e - 1.0) * (1.0 + 0.5 * m))
    return np.where(s == 1, -mag, mag)


NODES = e2m1_decode(np.arange(8))            # magnitudes, ascending: index == magnitude code


def e4m3_decode(byte) -> np.ndarray:
    """OCP FP8 E4M3 byte -> value (float64).  1-4-3, bias 7, no infinities, 0x7F/0xFF are NaN;
    exponent field 0 is subnormal: m/8 * 2^-6."""
    byte = np.asarray(byte).astype(np.int64)
    s = (byte >> 7) & 1
    e = (byte >> 3) & 15
    m = byte & 7
    mag = np.where(e == 0, m / 8.0 * 2.0 ** -6, np.exp2(e - 7.0) * (1.0 + m / 8.0))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(s == 1, -mag, mag)


E4M3_POS = e4m3_decode(np.arange(0x7F))      # the 127 finite non-negative values, ascending
E4M3_MAX = float(E4M3_POS[-1])               # 448


def e4m3_encode(t) -> np.ndarray:
    """Non-negative float32 -> nearest E4M3 byte, ties to the even byte, saturating at 448.
    Found by search over the enumerated value table (midpoints of neighbours are exact in
    float64, so every comparison is exact)."""
    t64 = np.asarray(t, dtype=F32).astype(np.float64)
    mids = 0.5 * (E4M3_POS[:-1] + E4M3_POS[1:])
    idx = np.searchsorted(mids, t64, side="left")          # mids[idx-1] < t <= mids[idx]
    on_mid = (idx < mids.size) & (mids[np.minimum(idx, mids.size - 1)] == t64)
    idx = np.where(on_mid & (idx % 2 == 1), idx + 1, idx)   # tie -> even mantissa bit
    return idx.astype(np.uint8)


def bf16_round(x) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even); result returned as float32 values."""
    b = np.ascontiguousarray(x, dtype=F32).view(np.uint32).astype(np.uint64)
    lsb = (b >> np.uint64(16)) & np.uint64(1)
    r = (b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    return (r << np.uint64(16)).astype(np.uint32).view(F32).reshape(np.shape(x))


# ----------------------------------------------------------------------------------------------
# Two-level scaling, FindInterval, V_init  (Sec. 3.1; Table 2 steps 2-5; Eq. 4)
# ----------------------------------------------------------------------------------------------

def _check_w(W):
    W = np.asarray(W)
    if W.dtype != F32 or W.ndim != 2 or W.shape[1] % BLOCK:
        raise ValueError("W must be float32 [O, K] with K a multiple of 16")
    return W


def tensor_scale(W) -> np.float32:
    """s_global (Sec. 3.1: an FP32 scale-of-scales that keeps the FP8 block scales in range).
    The paper does not say how it is derived.  Reading: the largest weight should land on the
    largest node (6) under the largest E4M3 scale (448), so s_global = amax / (6 * 448).
    An all-zero tensor takes s_global = 1."""
    W = _check_w(W)
    amax = np.max(np.abs(W)) if W.size else F32(0)
    if amax == 0:
        return F32(1.0)
    return F32(amax) / F32(2688.0)


def block_scale_bytes(W, s_global) -> np.ndarray:
    """E4M3 byte of s_g for every block of 16 consecutive weights along K (Sec. 3.1).
    Direction and rounding are not stated in the paper.  Reading: blocks run along the
    contraction dimension and never straddle rows; the block's largest magnitude a_b should land
    on node 6, so the ideal scale is a_b / 6, expressed in units of s_global and rounded to the
    nearest E4M3 value (ties to even, saturating): byte = E4M3((a_b / 6) / s_global)."""
    W = _check_w(W)
    O, K = W.shape
    a_b = np.max(np.abs(W.reshape(O, K // BLOCK, BLOCK)), axis=2).astype(F32)
    t = (a_b / F32(6.0)) / F32(s_global)
    return e4m3_encode(t)


def effective_scale(scale_bytes, s_global) -> np.ndarray:
    """s = s_g * s_global as one float32 product per block (the denominator of w-tilde, Sec. 3.1)."""
    return e4m3_decode(scale_bytes).astype(F32) * F32(s_global)


def normalised_magnitude(W, scale_bytes, s_global) -> np.ndarray:
    """Table 2 step 2: w-tilde = |w| / (s_g * s_global), one float32 division per weight.
    A block whose scale is zero (all-zero block, or a scale that underflowed E4M3) has w-tilde = 0."""
    W = _check_w(W)
    s = np.repeat(effective_scale(scale_bytes, s_global), BLOCK, axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        wt = np.abs(W) / s
    return np.where(s == 0, F32(0), wt).astype(F32)


def find_interval(wt) -> np.ndarray:
    """Table 2 step 3: index k_lo of the lower neighbour, so that lower = N[k_lo], upper = N[k_lo+1].
    The paper's  lower <= w-tilde <= upper  admits two intervals when w-tilde sits on a node: the
    interval above is taken (v_init = 0), except at the top where only [4, 6] exists.  w-tilde can
    exceed 6 (the block scale was rounded down): it stays in [4, 6] and saturates."""
    wt = np.asarray(wt, dtype=F32)
    k = np.zeros(wt.shape, dtype=np.int64)
    for node in NODES[1:7]:                                  # 0.5, 1, 1.5, 2, 3, 4
        k += (wt >= F32(node))
    return k


def relative_position(wt, k_lo) -> np.ndarray:
    """Eq. 4 / Table 2 step 4: v_init = (w-tilde - lower) / (upper - lower), in float32, then
    limited to [0, 1] (only bites when w-tilde > 6)."""
    lo = NODES[k_lo].astype(F32)
    hi = NODES[k_lo + 1].astype(F32)
    v = (np.asarray(wt, dtype=F32) - lo) / (hi - lo)
    return np.minimum(np.maximum(v, F32(0)), F32(1)).astype(F32)


def pack_nibbles(codes) -> np.ndarray:
    """[O, K] 4-bit codes -> [O, K/2] bytes, element 2j in the low nibble of byte j.
    (Packing order is not in the paper: convention.)"""
    codes = np.asarray(codes, dtype=np.uint8)
    return (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed) -> np.ndarray:
    packed = np.asarray(packed, dtype=np.uint8)
    out = np.empty((packed.shape[0], packed.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = packed & 0xF
    out[:, 1::2] = packed >> 4
    return out


def _codes_from_decisions(W, k_lo, up) -> np.ndarray:
    """Nibble = sign bit of w, then the magnitude code k_lo + up (nodes are index-ordered).
    Eq. 2 multiplies by sign(w), and sign(0) = 0: a zero weight stays zero whatever its decision,
    so its magnitude code is forced to 0."""
    mag = np.where(W == 0, 0, k_lo + up).astype(np.uint8)
    return (np.signbit(W).astype(np.uint8) << 3) | mag


def dequantise(codes, scale_bytes, s_global, out_bf16: bool) -> np.ndarray:
    """Table 2 step 26 evaluated for a decided code:  sign * node * s_g * s_global.
    node * s_g is exact in float32 (<= 6 significant bits); one float32 rounding for * s_global;
    then rounded to bf16 if that is the weight dtype."""
    codes = np.asarray(codes, dtype=np.uint8)
    node = np.abs(e2m1_decode(codes & 7)).astype(F32)
    sg = np.repeat(e4m3_decode(scale_bytes).astype(F32), BLOCK, axis=1)
    mag = (node * sg) * F32(s_global)
    out = np.where((codes >> 3) == 1, -mag, mag).astype(F32)
    return bf16_round(out) if out_bf16 else out


def quant_rtn(W, w_is_bf16: bool, s_global=None) -> dict:
    """Round-to-nearest NVFP4 (the paper's baseline rounding, Sec. 3.1-3.2).
    The nearer neighbour is chosen by v_init >= 1/2, i.e. an exact midpoint goes UP: this is the
    only tie rule under which hardening V_init (Eq. 4 then Eq. 7) reproduces RTN."""
    W = _check_w(W)
    s_global = tensor_scale(W) if s_global is None else F32(s_global)
    scales = block_scale_bytes(W, s_global)
    wt = normalised_magnitude(W, scales, s_global)
    k_lo = find_interval(wt)
    up = (relative_position(wt, k_lo) >= F32(0.5)).astype(np.int64)
    codes = _codes_from_decisions(W, k_lo, up)
    return {"s_global": s_global, "scales": scales, "codes": pack_nibbles(codes),
            "W_dq": dequantise(codes, scales, s_global, w_is_bf16)}


def init_v(W, s_global, scale_bytes) -> dict:
    """Table 2 steps 2-5, Eq. 4: V_init, plus the 'floor' nibbles sign<<3 | k_lo."""
    W = _check_w(W)
    wt = normalised_magnitude(W, scale_bytes, s_global)
    k_lo = find_interval(wt)
    floor_codes = (np.signbit(W).astype(np.uint8) << 3) | k_lo.astype(np.uint8)
    return {"V": relative_position(wt, k_lo), "floor_codes": pack_nibbles(floor_codes)}


def harden_pack(W, w_is_bf16: bool, s_global, scale_bytes, V) -> dict:
    """Eq. 7 and Table 2 steps 25-26: v-hat = 1 if v >= 1/2 else 0 on the stored float32 V, then the
    final weights as packed NVFP4.  Also returns the decision bitmask (bit i of byte j is v-hat of
    element 8j+i of the flattened tensor), the dequantised final weights and the number of weights
    whose nibble differs from round-to-nearest."""
    W = _check_w(W)
    V = np.asarray(V, dtype=F32)
    wt = normalised_magnitude(W, scale_bytes, s_global)
    k_lo = find_interval(wt)
    vhat = (V >= F32(0.5)).astype(np.int64)
    codes = _codes_from_decisions(W, k_lo, vhat)
    rtn = _codes_from_decisions(W, k_lo, (relative_position(wt, k_lo) >= F32(0.5)).astype(np.int64))
    bits = vhat.reshape(-1, 8).astype(np.uint8)
    decisions = np.zeros(bits.shape[0], dtype=np.uint8)
    for i in range(8):
        decisions |= bits[:, i] << i
    return {"codes": pack_nibbles(codes), "decisions": decisions,
            "W_final": dequantise(codes, scale_bytes, s_global, w_is_bf16),
            "flip_count": int(np.count_nonzero(codes != rtn))}


# ----------------------------------------------------------------------------------------------
# Soft quantisation, losses, gradients  (Eq. 2, 3, 5; Table 2 steps 6-12) -- float64
# ----------------------------------------------------------------------------------------------

def interval_terms(W, s_global, scale_bytes):
    """(sign, lower, upper, s) of Eq. 2 for every weight, as float64 arrays."""
    W = _check_w(W)
    wt = normalised_magnitude(W, scale_bytes, s_global)
    k_lo = find_interval(wt)
    s = np.repeat(effective_scale(scale_bytes, s_global), BLOCK, axis=1).astype(np.float64)
    return np.sign(W).astype(np.float64), NODES[k_lo], NODES[k_lo + 1], s


def h_beta(V, beta) -> np.ndarray:
    """Eq. 3: temperature-scaled sigmoid of (v - 1/2)."""
    z = float(beta) * (np.asarray(V, dtype=np.float64) - 0.5)
    with np.errstate(over="ignore"):                      # exp(+large) = inf gives the correct limit 0
        return 1.0 / (1.0 + np.exp(-z))


def soft_weight(W, s_global, scale_bytes, V, beta) -> np.ndarray:
    """Eq. 2 / Table 2 step 7: W_q(V) = sign(W) [lower + h_beta(V) (upper - lower)] s_g s_global."""
    sign, lo, hi, s = interval_terms(W, s_global, scale_bytes)
    return sign * (lo + h_beta(V, beta) * (hi - lo)) * s


def round_loss(V) -> float:
    """Table 2 step 11: (1/N) sum (1 - (2 v_i - 1)^2)."""
    V = np.asarray(V, dtype=np.float64)
    return float(np.sum(1.0 - (2.0 * V - 1.0) ** 2) / V.size)


def stage1_loss_and_grads(W, s_global, scale_bytes, V, Xq, Y_fp, beta, lambda_round, alpha,
                          want_dX: bool = False, dY_ext=None, declared_rounding: bool = False) -> dict:
    """Eq. 5 with its gradient w.r.t. V (and optionally X_q).

      Y_q = X_q W_q^T,  R = Y_q - Y_fp,  L_mse = alpha * ||R||_F^2   (Table 2 steps 9-10; the paper
      calls a Frobenius norm "MSE": alpha = 1 is the literal sum, alpha = 1/(T*O) the mean)
      L_round as round_loss;  L = L_mse + lambda_round * L_round     (steps 11-12)
      dY = 2 alpha R;  G = dY^T X_q;  dV = G * sign s (upper-lower) beta h (1-h) + lambda/N (4 - 8 v)
      dX = dY W_q.

    dY_ext (if given) replaces the locally derived dY in G and dX (an upstream gradient when the
    layer is one link of a longer chain); the losses are still those of this layer.

    declared_rounding=True applies the three storage roundings a bf16 tensor-core implementation
    declares -- the weight perturbation (W_q - W), dY and dX are each rounded to bf16 where they
    are stored -- and nothing else; with it off, every quantity is exact float64.

    declared_rounding="split" is the same contract for an implementation that splits the constant
    part off the gradient: with d = W_q - W and C = Y_fp - X_q W^T (both as above),
        R = X_q d^T - C,   dY = 2 alpha R   =>   G = dY^T X_q = (2 alpha X_q d^T)^T X_q - 2 alpha C^T X_q,
    and only the first, V-dependent factor 2 alpha X_q d^T is stored (rounded to bf16); the constant
    C^T X_q is exact.  Same mathematics (Eq. 5 and its chain rule), another rounding point for dY.

    declared_rounding="gram" is the contract of an implementation that, for activations that stay the same
    from step to step, never forms the layer output: with Gm = X_q^T X_q,
        ||R||^2 = <d Gm, d> - 2 <d, C^T X_q> + ||C||^2,   G = 2 alpha (d Gm - C^T X_q)
    (Eq. 5 expanded, and its chain rule), where d is stored rounded to bf16 as above and Gm is stored rounded
    to bf16 off its diagonal (the diagonal is kept exact); dY does not exist.  No dY_ext, no dX.
    """
    W = _check_w(W)
    V64 = np.asarray(V, dtype=F32).astype(np.float64)
    Xq = np.asarray(Xq, dtype=np.float64)
    Y_fp = np.asarray(Y_fp, dtype=np.float64)
    sign, lo, hi, s = interval_terms(W, s_global, scale_bytes)
    h = h_beta(V64, beta)
    Wq = sign * (lo + h * (hi - lo)) * s
    W64 = W.astype(np.float64)
    if declared_rounding:
        delta = bf16_round((Wq - W64).astype(F32)).astype(np.float64)
        R = Xq @ delta.T - (Y_fp - Xq @ W64.T)
    else:
        R = Xq @ Wq.T - Y_fp
    N = W.size
    L_mse = float(alpha) * float(np.sum(R * R))
    L_round = round_loss(V64)
    if declared_rounding == "gram":
        if dY_ext is not None or want_dX:
            raise ValueError("the Gram-matrix form has neither dY nor dX")
        C = Y_fp - Xq @ W64.T
        Gm = Xq.T @ Xq
        Gm_stored = bf16_round(Gm.astype(F32)).astype(np.float64)
        np.fill_diagonal(Gm_stored, np.diag(Gm))
        Hc = C.T @ Xq
        dG = delta @ Gm_stored
        L_mse = float(alpha) * (float(np.sum(dG * delta)) - 2.0 * float(np.sum(delta * Hc)) + float(np.sum(C * C)))
        G = 2.0 * float(alpha) * (dG - Hc)
        dY = None
    elif dY_ext is None and declared_rounding == "split":
        C = Y_fp - Xq @ W64.T
        dYa = bf16_round((2.0 * float(alpha) * (Xq @ delta.T)).astype(F32)).astype(np.float64)
        dY = dYa - 2.0 * float(alpha) * C
        G = dYa.T @ Xq - 2.0 * float(alpha) * (C.T @ Xq)
    else:
        if dY_ext is None:
            dY = 2.0 * float(alpha) * R
            if declared_rounding:
                dY = bf16_round(dY.astype(F32)).astype(np.float64)
        else:
            dY = np.asarray(dY_ext, dtype=np.float64)
        G = dY.T @ Xq
    dV = G * sign * s * (hi - lo) * float(beta) * h * (1.0 - h) + float(lambda_round) / N * (4.0 - 8.0 * V64)
    out = {"Wq": Wq, "R": R, "dY": dY, "G": G, "dV": dV, "L_mse": L_mse, "L_round": L_round,
           "L": L_mse + float(lambda_round) * L_round}
    if want_dX:
        Wq_used = bf16_round(Wq.astype(F32)).astype(np.float64) if declared_rounding else Wq
        dX = dY @ Wq_used
        out["dX"] = bf16_round(dX.astype(F32)).astype(np.float64) if declared_rounding else dX
    return out


def adam_update(V, m, u, g, lr, beta1, beta2, eps, t):
    """Table 2 step 13 ("update V"); the optimiser is not named in the paper.  Reading: Adam with
    bias correction, no weight decay, then the clip of V to [0, 1] the paper requires after every
    update (Sec. 3.4, Stage 1).  t is the 1-based step count.  float64 throughout."""
    V = np.asarray(V, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    u = beta2 * np.asarray(u, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    u_hat = u / (1.0 - beta2 ** t)
    V_new = V - lr * m_hat / (np.sqrt(u_hat) + eps)
    return np.clip(V_new, 0.0, 1.0), m, u


def layer_step(W, s_global, scale_bytes, V, m, u, Xq, Y_fp, beta, lambda_round, alpha,
               lr, beta1, beta2, eps, t, want_dX=False, dY_ext=None, declared_rounding=False) -> dict:
    """One optimisation step of Table 2 steps 6-13 for one linear layer.  V, m, u are taken as
    float32 storage (what an implementation keeps between steps) and returned rounded to float32."""
    r = stage1_loss_and_grads(W, s_global, scale_bytes, V, Xq, Y_fp, beta, lambda_round, alpha,
                              want_dX=want_dX, dY_ext=dY_ext, declared_rounding=declared_rounding)
    V_new, m_new, u_new = adam_update(np.asarray(V, dtype=F32), np.asarray(m, dtype=F32),
                                      np.asarray(u, dtype=F32), r["dV"], lr, beta1, beta2, eps, t)
    r.update({"V": V_new.astype(F32), "m": m_new.astype(F32), "u": u_new.astype(F32),
              "V64": V_new, "m64": m_new, "u64": u_new})
    return r


def hardened_loss(W, w_is_bf16, s_global, scale_bytes, V, Xq, Y_fp, alpha) -> float:
    """alpha * ||X_q W_final^T - Y_fp||_F^2 with W_final from Eq. 7 (un-rounded float32 product
    sign*node*s_g*s_global, i.e. the values an NVFP4 decoder would produce)."""
    hp = harden_pack(W, False, s_global, scale_bytes, V)
    R = np.asarray(Xq, dtype=np.float64) @ hp["W_final"].astype(np.float64).T - np.asarray(Y_fp, dtype=np.float64)
    return float(alpha) * float(np.sum(R * R))


# ----------------------------------------------------------------------------------------------
# Stage-2 objective on given model outputs (Sec. 3.5 "Stage 2", Eq. 6; Table 2 steps 18-22)
# ----------------------------------------------------------------------------------------------

def log_softmax_t(Z, tau) -> np.ndarray:
    """log softmax(Z / tau) along the last axis (Table 2 step 18), float64, max-shifted."""
    a = np.asarray(Z, dtype=np.float64) / float(tau)
    a = a - a.max(axis=-1, keepdims=True)
    return a - np.log(np.exp(a).sum(axis=-1, keepdims=True))


def stage2_losses(Z_fp, Z_q, tau, kl_scale, H_fp, H_q, mse_scale, round_losses, lambda_kl, lambda_round) -> dict:
    """Eq. 6 / Table 2 steps 18-22 on logits Z [T, vocab] and last hidden states H [T, D]:

        P_fp = softmax(Z_fp / tau), P_q = softmax(Z_q / tau)
        L_KL    = kl_scale  * sum_t sum_j P_fp[t,j] (log P_fp[t,j] - log P_q[t,j])
        L_MSE   = mse_scale * ||H_fp - H_q||_F^2
        L_round = sum_l round_losses[l]
        L       = lambda_kl L_KL + L_MSE + lambda_round L_round

    and the gradients of L with respect to the quantised model's outputs,

        dZ_q = lambda_kl kl_scale / tau * (P_q - P_fp),     dH_q = 2 mse_scale (H_q - H_fp).

    The paper does not say whether the KL is summed or averaged over tokens, nor whether the "MSE" (written
    as a squared Frobenius norm) is a mean: both scales are arguments (1 = the formulas as printed)."""
    la, lb = log_softmax_t(Z_fp, tau), log_softmax_t(Z_q, tau)
    P_fp, P_q = np.exp(la), np.exp(lb)
    # a logit of -inf (a masked vocabulary entry) has probability 0; the KL divergence takes 0 log 0 = 0, so an
    # entry with P_fp = 0 contributes nothing whatever P_q is, and P_q = 0 under P_fp > 0 makes the sum +inf
    with np.errstate(invalid="ignore"):
        terms = np.where(P_fp > 0.0, P_fp * (la - lb), 0.0)
    kl = float(kl_scale) * float(terms.sum())
    dH = np.asarray(H_q, dtype=np.float64) - np.asarray(H_fp, dtype=np.float64)
    mse = float(mse_scale) * float((dH * dH).sum())
    rl = float(np.asarray(round_losses, dtype=np.float64).sum()) if round_losses is not None else 0.0
    return {"L_kl": kl, "L_mse": mse, "L_round": rl,
            "L": float(lambda_kl) * kl + mse + float(lambda_round) * rl,
            "dZ_q": float(lambda_kl) * float(kl_scale) / float(tau) * (P_q - P_fp),
            "dH_q": 2.0 * float(mse_scale) * dH}


# ----------------------------------------------------------------------------------------------
# Stochastic rounding candidates (Sec. 3.2, Table 1: "among only 100 stochastic rounding trials ...")
# ----------------------------------------------------------------------------------------------

def philox4x32_10(counter, key) -> np.ndarray:
    """Philox-4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3", SC'11):
    counter [..., 4] uint32, key [..., 2] uint32 -> [..., 4] uint32.  A counter-based generator, so that
    any other implementation can draw exactly the same numbers."""
    M0, M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
    W0, W1 = np.uint32(0x9E3779B9), np.uint32(0xBB67AE85)
    c = np.array(counter, dtype=np.uint32).copy()
    k = np.broadcast_to(np.array(key, dtype=np.uint32), c.shape[:-1] + (2,)).copy()
    with np.errstate(over="ignore"):
        for _ in range(10):
            p0 = M0 * c[..., 0].astype(np.uint64)
            p1 = M1 * c[..., 2].astype(np.uint64)
            hi0, lo0 = (p0 >> np.uint64(32)).astype(np.uint32), p0.astype(np.uint32)
            hi1, lo1 = (p1 >> np.uint64(32)).astype(np.uint32), p1.astype(np.uint32)
            c = np.stack([hi1 ^ c[..., 1] ^ k[..., 0], lo1, hi0 ^ c[..., 3] ^ k[..., 1], lo0], axis=-1)
            k = np.stack([k[..., 0] + W0, k[..., 1] + W1], axis=-1)
    return c


def stochastic_v(V_init, seed: int, sample: int) -> np.ndarray:
    """One stochastic-rounding candidate: v = 1 with probability v_init (the weight's relative position in its
    interval, Eq. 4), else 0.  The paper reports such trials (Table 1) without defining them; this is the
    standard unbiased rule.  Element i (row-major) draws word i % 4 of Philox(counter = (i / 4 low, i / 4 high,
    sample, 0), key = (seed low, seed high)); u = (word >> 8) * 2^-24; up iff u < v_init."""
    v = np.asarray(V_init, dtype=np.float32)
    n = v.size
    blocks = np.arange((n + 3) // 4, dtype=np.uint64)
    ctr = np.stack([(blocks & np.uint64(0xFFFFFFFF)).astype(np.uint32), (blocks >> np.uint64(32)).astype(np.uint32),
                    np.full(blocks.shape, np.uint32(sample & 0xFFFFFFFF)), np.zeros(blocks.shape, dtype=np.uint32)], axis=-1)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    words = philox4x32_10(ctr, key).reshape(-1)[:n]
    u = (words >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)
    return (u < v.reshape(-1)).astype(np.float32).reshape(v.shape)
