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
