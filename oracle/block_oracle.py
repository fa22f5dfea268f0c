"""CPU oracle for the glue between the quantised linears of one transformer block (MLP half).

THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH (see faar_oracle.py: same rules, no code shared with the HIP
library).

Stage 2 of the method (Sec. 3.5 "Stage 2"; Table 2 steps 15-17 and 23) runs the assembled quantised model forward
and back-propagates one loss into every layer's rounding variables V.  Between the linears that means the ordinary
operations of the models the paper evaluates (Llama3 / Qwen3 blocks): pre-norm RMSNorm, the gated SiLU MLP, and the
residual connection; the paper does not restate them, so they are written here from their textbook definitions:

    h      = RMSNorm(x; g)        h_i = x_i g_i / sqrt(mean_j x_j^2 + eps)                     (per token)
    a      = SiLU(p) * q          SiLU(p) = p sigmoid(p);  p = gate_proj(h), q = up_proj(h)
    y      = x + down_proj(a)                                                                   (residual)
    L_blk  = mse_scale * ||y - y_fp||_F^2     ("MSE on block output": the block-level form of Eq. 6's hidden-state term)

and their backward passes.  All float64.  Every linear is y = X W_q(V)^T with W_q from Eq. 2-3 (faar_oracle.soft_weight);
dL/dV of a linear given dL/dY is faar_oracle.stage1_loss_and_grads(..., dY_ext=dL/dY).

bf16_storage=True rounds each tensor an implementation stores between kernels (h, p, q, a, the MLP output, every
gradient tensor) to bf16 -- the declared rounding points of the HIP path -- and nothing else.

The attention half of the same blocks, likewise from the textbook definitions (the paper does not restate them):

    h        = RMSNorm(x; g)
    q, k, v  = q_proj(h), k_proj(h), v_proj(h)          split into heads of width dh; n_q heads of q share n_kv heads of k, v
    q, k     = RMSNorm over each head's dh entries (weights gq, gk; Qwen3 only), then rotary position embedding
    o        = softmax(q k^T * scale, causal within a sequence) v     per head and sequence
    y        = x + o_proj(o)

Rotary embedding, "rotate-half" form of those models: with c, s the cosine and sine of pos * theta_i, i < dh/2,
    y_i = x_i c_i - x_{i+dh/2} s_i,    y_{i+dh/2} = x_{i+dh/2} c_i + x_i s_i.
The cosine / sine tables are inputs (one row per position), so that both sides rotate by the same angles.
"""
from __future__ import annotations

import numpy as np

from oracle import faar_oracle as fo

F32 = np.float32


def _store(x, bf16_storage):
    return fo.bf16_round(np.asarray(x, dtype=F32)).astype(np.float64) if bf16_storage else np.asarray(x, dtype=np.float64)


def rmsnorm(x, g, eps):
    """h_i = x_i g_i r with r = 1 / sqrt(mean(x^2) + eps), per row.  -> (h, r)."""
    x = np.asarray(x, dtype=np.float64)
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + float(eps))
    return x * r * np.asarray(g, dtype=np.float64), r[..., 0]


def rmsnorm_backward(dh, x, g, r):
    """dL/dx of h = x g r(x):  dx_i = r g_i dh_i - x_i r^3 / D * sum_j x_j g_j dh_j   (g is frozen)."""
    x = np.asarray(x, dtype=np.float64)
    gd = np.asarray(g, dtype=np.float64) * np.asarray(dh, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)[..., None]
    return r * gd - x * (r ** 3) * (x * gd).mean(axis=-1, keepdims=True)


def silu_mul(p, q):
    """a = p sigmoid(p) q."""
    p = np.asarray(p, dtype=np.float64)
    return p / (1.0 + np.exp(-p)) * np.asarray(q, dtype=np.float64)


def silu_mul_backward(da, p, q):
    """(dL/dp, dL/dq) of a = SiLU(p) q:  SiLU'(p) = s (1 + p (1 - s)), s = sigmoid(p)."""
    p, q, da = (np.asarray(t, dtype=np.float64) for t in (p, q, da))
    s = 1.0 / (1.0 + np.exp(-p))
    return da * q * s * (1.0 + p * (1.0 - s)), da * p * s


def block_output_loss(x, d, y_fp, mse_scale):
    """y = x + d;  L = mse_scale ||y - y_fp||_F^2;  dL/dy = 2 mse_scale (y - y_fp).  -> (y, L, dy)."""
    y = np.asarray(x, dtype=np.float64) + np.asarray(d, dtype=np.float64)
    r = y - np.asarray(y_fp, dtype=np.float64)
    return y, float(mse_scale) * float((r * r).sum()), 2.0 * float(mse_scale) * r


def mlp_block_step(x, g_norm, eps, layers, y_fp, mse_scale, beta, lambda_round, bf16_storage=False):
    """Forward and backward of the MLP half of a block whose three linears are FAAR-parameterised.

    layers: dict name -> (W, s_global, scale_bytes, V) for "gate", "up", "down" (W [O, K] as in faar_oracle).
    -> dict with the block loss, the Round Loss of each linear, dL/dV of each linear (block loss term plus
       lambda_round times that linear's Round-Loss gradient), dL/dx, and the intermediate activations.
    """
    st = lambda t: _store(t, bf16_storage)
    x = np.asarray(x, dtype=np.float64)
    h, r = rmsnorm(x, g_norm, eps)
    h = st(h)
    Wq = {}
    for name, (W, sg, sb, V) in layers.items():
        wq = fo.soft_weight(W, sg, sb, V, beta)
        Wq[name] = st(wq) if bf16_storage else wq        # the matrix cores see bf16 weights
    p = st(h @ Wq["gate"].T)
    q = st(h @ Wq["up"].T)
    a = st(silu_mul(p, q))
    d = st(a @ Wq["down"].T)
    y, L, dy = block_output_loss(x, d, y_fp, mse_scale)
    dy = st(dy)
    out = {"h": h, "rstd": r, "p": p, "q": q, "a": a, "d": d, "y": y, "L_block": L, "dy": dy, "dV": {}, "L_round": {}}

    def dv_of(name, X, dY):
        W, sg, sb, V = layers[name]
        # the reference output does not matter when dY is given: only the gradient terms are used
        res = fo.stage1_loss_and_grads(W, sg, sb, V, X, np.zeros((X.shape[0], W.shape[0])), beta, lambda_round, 0.0, dY_ext=dY)
        out["L_round"][name] = res["L_round"]
        return res["dV"]

    out["dV"]["down"] = dv_of("down", a, dy)
    da = st(dy @ Wq["down"])
    dp, dq = silu_mul_backward(da, p, q)
    dp, dq = st(dp), st(dq)
    out["dV"]["gate"] = dv_of("gate", h, dp)
    out["dV"]["up"] = dv_of("up", h, dq)
    dh_gate, dh_up = st(dp @ Wq["gate"]), st(dq @ Wq["up"])
    out["dx"] = st(rmsnorm_backward(dh_gate + dh_up, x, g_norm, r) + dy)     # norm path + residual path
    out["da"], out["dp"], out["dq"] = da, dp, dq
    return out


# ---- attention half -------------------------------------------------------------------------------------------------
def rope(x, cos, sin, pos, dh):
    """Rotate every head of x [T, H*dh] by its token's position: cos, sin [S, dh/2], pos [T] integer rows of the tables."""
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    xh = x.reshape(T, -1, dh)
    c = np.asarray(cos, dtype=np.float64)[pos][:, None, :]
    s_ = np.asarray(sin, dtype=np.float64)[pos][:, None, :]
    a, b = xh[..., :dh // 2], xh[..., dh // 2:]
    return np.concatenate([a * c - b * s_, b * c + a * s_], axis=-1).reshape(T, -1)


def rope_backward(dy, cos, sin, pos, dh):
    """dL/dx of y = rope(x): the rotation is orthogonal, so its transpose is the rotation by the opposite angle."""
    return rope(dy, cos, -np.asarray(sin, dtype=np.float64), pos, dh)


def attention(q, k, v, n_seq, n_q, n_kv, dh, scale):
    """Causal softmax attention.  q [T, n_q*dh], k, v [T, n_kv*dh]; T = n_seq * S tokens, sequence b = rows b*S..(b+1)*S-1;
    query head j reads key / value head j // (n_q // n_kv).  -> o [T, n_q*dh] and the probabilities [n_seq, n_q, S, S]."""
    q, k, v = (np.asarray(t, dtype=np.float64) for t in (q, k, v))
    T = q.shape[0]
    S = T // n_seq
    rep = n_q // n_kv
    o = np.zeros((T, n_q * dh))
    P = np.zeros((n_seq, n_q, S, S))
    allowed = np.tril(np.ones((S, S), dtype=bool))                  # key position <= query position
    for b in range(n_seq):
        rows = slice(b * S, (b + 1) * S)
        for j in range(n_q):
            qh = q[rows, j * dh:(j + 1) * dh]
            kh = k[rows, (j // rep) * dh:(j // rep + 1) * dh]
            vh = v[rows, (j // rep) * dh:(j // rep + 1) * dh]
            z = np.where(allowed, (qh @ kh.T) * scale, -np.inf)
            e = np.exp(z - z.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            P[b, j] = p
            o[rows, j * dh:(j + 1) * dh] = p @ vh
    return o, P


def attention_backward(do, q, k, v, P, n_seq, n_q, n_kv, dh, scale):
    """(dq, dk, dv) of o = attention(q, k, v): dV = P^T dO; dP = dO V^T; dZ = P * (dP - rowsum(P * dP)) (softmax Jacobian);
    dQ = scale dZ K; dK = scale dZ^T Q; the gradients of a shared key / value head add over its query heads."""
    do, q, k, v = (np.asarray(t, dtype=np.float64) for t in (do, q, k, v))
    T = q.shape[0]
    S = T // n_seq
    rep = n_q // n_kv
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b in range(n_seq):
        rows = slice(b * S, (b + 1) * S)
        for j in range(n_q):
            cq, ck = slice(j * dh, (j + 1) * dh), slice((j // rep) * dh, (j // rep + 1) * dh)
            p = P[b, j]
            dv[rows, ck] += p.T @ do[rows, cq]
            dp = do[rows, cq] @ v[rows, ck].T
            dz = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dq[rows, cq] = scale * (dz @ k[rows, ck])
            dk[rows, ck] += scale * (dz.T @ q[rows, cq])
    return dq, dk, dv


def attn_block_step(x, g_norm, eps, layers, n_seq, n_q, n_kv, dh, cos, sin, beta, lambda_round, y_fp=None, mse_scale=1.0,
                    d_out=None, qk_norm=None, bf16_storage=False):
    """Forward and backward of the attention half of a block whose four linears are FAAR-parameterised.

    layers: dict name -> (W, s_global, scale_bytes, V) for "q", "k", "v", "o".  qk_norm: None (Llama3) or (gq, gk) weights of
    the per-head RMSNorm of Qwen3.  The gradient entering at the half's output y = x + o_proj(o) is d_out if given (the
    MLP half's dL/dx when the whole block is stepped), else that of mse_scale ||y - y_fp||_F^2.
    -> dict with dL/dV and the Round Loss of each linear, dL/dx, y and the intermediates."""
    st = lambda t: _store(t, bf16_storage)
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    S = T // n_seq
    pos = np.arange(T) % S
    scale = 1.0 / np.sqrt(dh)
    h, r = rmsnorm(x, g_norm, eps)
    h = st(h)
    Wq = {}
    for name, (W, sg, sb, V) in layers.items():
        wq = fo.soft_weight(W, sg, sb, V, beta)
        Wq[name] = st(wq) if bf16_storage else wq
    q0, k0, v = st(h @ Wq["q"].T), st(h @ Wq["k"].T), st(h @ Wq["v"].T)
    if qk_norm is not None:
        q1, rq = rmsnorm(q0.reshape(-1, dh), qk_norm[0], eps)
        k1, rk = rmsnorm(k0.reshape(-1, dh), qk_norm[1], eps)
        q1, k1 = st(q1).reshape(T, -1), st(k1).reshape(T, -1)
    else:
        q1, k1 = q0, k0
    q2, k2 = st(rope(q1, cos, sin, pos, dh)), st(rope(k1, cos, sin, pos, dh))
    o, P = attention(q2, k2, v, n_seq, n_q, n_kv, dh, scale)
    o = st(o)
    d = st(o @ Wq["o"].T)
    out = {"h": h, "q0": q0, "k0": k0, "v": v, "q": q2, "k": k2, "o": o, "d": d, "dV": {}, "L_round": {}}
    if d_out is None:
        y, L, dy = block_output_loss(x, d, y_fp, mse_scale)
        out["L_block"] = L
    else:
        y, dy = x + d, np.asarray(d_out, dtype=np.float64)
    dy = st(dy)
    out["y"], out["dy"] = y, dy

    def dv_of(name, X, dY):
        W, sg, sb, V = layers[name]
        res = fo.stage1_loss_and_grads(W, sg, sb, V, X, np.zeros((X.shape[0], W.shape[0])), beta, lambda_round, 0.0, dY_ext=dY)
        out["L_round"][name] = res["L_round"]
        return res["dV"]

    out["dV"]["o"] = dv_of("o", o, dy)
    do = st(dy @ Wq["o"])
    dq2, dk2, dv = attention_backward(do, q2, k2, v, P, n_seq, n_q, n_kv, dh, scale)
    dq2, dk2, dv = st(dq2), st(dk2), st(dv)
    dq1, dk1 = st(rope_backward(dq2, cos, sin, pos, dh)), st(rope_backward(dk2, cos, sin, pos, dh))
    if qk_norm is not None:
        dq0 = st(rmsnorm_backward(dq1.reshape(-1, dh), q0.reshape(-1, dh), qk_norm[0], rq)).reshape(T, -1)
        dk0 = st(rmsnorm_backward(dk1.reshape(-1, dh), k0.reshape(-1, dh), qk_norm[1], rk)).reshape(T, -1)
    else:
        dq0, dk0 = dq1, dk1
    out["dV"]["q"], out["dV"]["k"], out["dV"]["v"] = dv_of("q", h, dq0), dv_of("k", h, dk0), dv_of("v", h, dv)
    dh_sum = st(dq0 @ Wq["q"]) + st(dk0 @ Wq["k"]) + st(dv @ Wq["v"])
    out["dx"] = st(rmsnorm_backward(dh_sum, x, g_norm, r) + dy)
    out.update({"do": do, "dq": dq2, "dk": dk2, "dv": dv, "dq0": dq0, "dk0": dk0})
    return out
