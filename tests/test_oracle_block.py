"""Pins for the block-glue oracle (RMSNorm, gated SiLU, residual + block-output MSE, and their composition into the
MLP half of a block): an independent implementation with automatic differentiation (torch on the CPU, float64),
central finite differences, closed forms and invariances -- none of them the oracle's own formulas."""
import numpy as np
import pytest
import torch

from oracle import block_oracle as bo
from oracle import faar_oracle as fo
from workloads import synth


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def test_rmsnorm_against_a_library_and_closed_forms():
    x, g = _rand((5, 48), 1), _rand(48, 2) * 0.5 + 1.0
    h, r = bo.rmsnorm(x, g, 1e-6)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(h, want, rtol=1e-13, atol=0)
    # closed forms: a constant row c maps to sign(c) g; scaling the input leaves the output unchanged (eps -> 0)
    h1, _ = bo.rmsnorm(np.full((1, 48), -3.0), g, 0.0)
    assert np.allclose(h1, -g, rtol=1e-14)
    h2, _ = bo.rmsnorm(7.5 * x, g, 0.0)
    h0, r0 = bo.rmsnorm(x, g, 0.0)
    assert np.allclose(h2, h0, rtol=1e-13)
    assert np.allclose(r0, 1.0 / np.sqrt((x * x).mean(axis=1)), rtol=1e-14)
    # with g = 1 every output row has unit mean square
    h3, _ = bo.rmsnorm(x, np.ones(48), 0.0)
    assert np.allclose((h3 * h3).mean(axis=1), 1.0, rtol=1e-13)


def test_rmsnorm_backward_against_autograd_and_finite_differences():
    x, g, dh = _rand((4, 40), 3), _rand(40, 4) + 1.0, _rand((4, 40), 5)
    _, r = bo.rmsnorm(x, g, 1e-5)
    dx = bo.rmsnorm_backward(dh, x, g, r)
    xt = torch.from_numpy(x).requires_grad_(True)
    torch.nn.functional.rms_norm(xt, (40,), torch.from_numpy(g), 1e-5).backward(torch.from_numpy(dh))
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-11, atol=1e-14)
    f = lambda xx: float((bo.rmsnorm(xx, g, 1e-5)[0] * dh).sum())
    for (i, j) in [(0, 0), (1, 17), (3, 39)]:
        e = np.zeros_like(x); e[i, j] = 1e-6
        assert dx[i, j] == pytest.approx((f(x + e) - f(x - e)) / 2e-6, rel=1e-6, abs=1e-9)
    # the gradient is orthogonal to x when eps = 0 (the output does not depend on the scale of x)
    _, r0 = bo.rmsnorm(x, g, 0.0)
    assert np.abs((bo.rmsnorm_backward(dh, x, g, r0) * x).sum(axis=1)).max() < 1e-12


def test_silu_mul_forward_and_backward():
    p, q, da = _rand((6, 33), 6, 2.0), _rand((6, 33), 7), _rand((6, 33), 8)
    a = bo.silu_mul(p, q)
    assert np.allclose(a, (torch.nn.functional.silu(torch.from_numpy(p)) * torch.from_numpy(q)).numpy(), rtol=1e-13, atol=1e-16)
    # closed forms: SiLU(0) = 0, SiLU(p) -> p for large p, SiLU(p) + SiLU(-p) = p tanh(p / 2)
    assert bo.silu_mul(np.zeros(3), np.ones(3)).tolist() == [0.0, 0.0, 0.0]
    assert bo.silu_mul(np.array([40.0]), np.array([1.0]))[0] == pytest.approx(40.0, rel=1e-15)
    assert np.allclose(bo.silu_mul(p, 1.0) + bo.silu_mul(-p, 1.0), p * np.tanh(p / 2), rtol=1e-12, atol=1e-15)
    dp, dq = bo.silu_mul_backward(da, p, q)
    pt, qt = torch.from_numpy(p).requires_grad_(True), torch.from_numpy(q).requires_grad_(True)
    (torch.nn.functional.silu(pt) * qt).backward(torch.from_numpy(da))
    assert np.allclose(dp, pt.grad.numpy(), rtol=1e-12, atol=1e-15) and np.allclose(dq, qt.grad.numpy(), rtol=1e-12, atol=1e-15)
    # SiLU'(0) = 1/2
    assert bo.silu_mul_backward(np.ones(1), np.zeros(1), np.ones(1))[0][0] == 0.5


def test_block_output_loss():
    x, d, yf = _rand((3, 8), 9), _rand((3, 8), 10), _rand((3, 8), 11)
    y, L, dy = bo.block_output_loss(x, d, yf, 0.25)
    assert np.array_equal(y, x + d)
    assert L == pytest.approx(0.25 * np.linalg.norm(x + d - yf) ** 2, rel=1e-14)
    e = np.zeros_like(d); e[1, 2] = 1e-6
    fd = (bo.block_output_loss(x, d + e, yf, 0.25)[1] - bo.block_output_loss(x, d - e, yf, 0.25)[1]) / 2e-6
    assert dy[1, 2] == pytest.approx(fd, rel=1e-8)
    assert bo.block_output_loss(x, yf - x, yf, 1.0)[1] < 1e-28       # y = y_fp up to one rounding of x + (y_fp - x)


def _tiny_block(T=12, D=32, F=48, seed=0):
    rng = np.random.default_rng(seed)
    layers = {}
    for k, (name, O, K) in enumerate((("gate", F, D), ("up", F, D), ("down", D, F))):
        W = synth.student_t_weight(O, K, 300 + seed + k, scale=0.2)
        q = fo.quant_rtn(W, True)
        V = np.clip(fo.init_v(W, q["s_global"], q["scales"])["V"] + rng.uniform(-0.2, 0.2, W.shape), 0.05, 0.95).astype(np.float32)
        layers[name] = (W, q["s_global"], q["scales"], V)
    x = rng.standard_normal((T, D))
    g = rng.uniform(0.5, 1.5, D)
    y_fp = x + rng.standard_normal((T, D)) * 0.3
    return x, g, layers, y_fp


def test_mlp_block_step_against_autograd_through_an_independent_graph():
    """The whole MLP half: forward values and every gradient (dL/dV of the three linears, dL/dx) against torch autograd
    through a graph built from library ops and a re-statement of Eq. 2-3 on torch tensors."""
    x, g, layers, y_fp = _tiny_block()
    beta, lam, ms = 6.0, 0.02, 1.0 / (12 * 32)
    r = bo.mlp_block_step(x, g, 1e-6, layers, y_fp, ms, beta, lam)
    Vt, Wq = {}, {}
    for name, (W, sg, sb, V) in layers.items():
        sign, lo, hi, s = (torch.from_numpy(np.ascontiguousarray(t)) for t in fo.interval_terms(W, sg, sb))
        Vt[name] = torch.from_numpy(V.astype(np.float64)).requires_grad_(True)
        Wq[name] = sign * (lo + torch.sigmoid(beta * (Vt[name] - 0.5)) * (hi - lo)) * s
    xt = torch.from_numpy(x).requires_grad_(True)
    h = torch.nn.functional.rms_norm(xt, (32,), torch.from_numpy(g), 1e-6)
    a = torch.nn.functional.silu(h @ Wq["gate"].T) * (h @ Wq["up"].T)
    y = xt + a @ Wq["down"].T
    L = ms * ((y - torch.from_numpy(y_fp)) ** 2).sum()
    rl = sum((1 - (2 * v - 1) ** 2).mean() for v in Vt.values())
    (L + lam * rl).backward()
    assert r["L_block"] == pytest.approx(float(L.detach()), rel=1e-12)
    assert np.allclose(r["y"], y.detach().numpy(), rtol=1e-12, atol=1e-14)
    for name in layers:
        assert np.allclose(r["dV"][name], Vt[name].grad.numpy(), rtol=1e-9, atol=1e-15), name
        assert r["L_round"][name] == pytest.approx(float((1 - (2 * Vt[name] - 1) ** 2).mean()), rel=1e-12)
    assert np.allclose(r["dx"], xt.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_mlp_block_step_by_finite_differences_and_bf16_storage_is_a_small_perturbation():
    x, g, layers, y_fp = _tiny_block(seed=3)
    beta, lam, ms = 5.0, 0.0, 1.0 / (12 * 32)
    r = bo.mlp_block_step(x, g, 1e-6, layers, y_fp, ms, beta, lam)

    def loss_with(name, i, j, dv):
        mod = dict(layers)
        W, sg, sb, V = layers[name]
        V2 = V.astype(np.float64).copy(); V2[i, j] += dv
        mod[name] = (W, sg, sb, V2)
        # V is taken as float32 storage by the oracle: bypass by evaluating with float64 V through soft_weight directly
        return bo.mlp_block_step(x, g, 1e-6, mod, y_fp, ms, beta, lam)["L_block"]

    for name, (i, j) in (("gate", (3, 5)), ("up", (40, 31)), ("down", (7, 20))):
        eps = 2.0 ** -10            # exactly representable: V + eps survives the float32 storage of V
        fd = (loss_with(name, i, j, eps) - loss_with(name, i, j, -eps)) / (2 * eps)
        assert r["dV"][name][i, j] == pytest.approx(fd, rel=2e-4, abs=1e-12), name
    b = bo.mlp_block_step(x, g, 1e-6, layers, y_fp, ms, beta, lam, bf16_storage=True)
    n = np.linalg.norm
    assert b["L_block"] == pytest.approx(r["L_block"], rel=2e-2)
    for name in layers:
        assert 0 < n(b["dV"][name] - r["dV"][name]) <= 3e-2 * n(r["dV"][name])
    assert n(b["dx"] - r["dx"]) <= 3e-2 * n(r["dx"])


# ---- attention half ---------------------------------------------------------------------------------------------------
def _rope_tables(S, dh, base=10000.0):
    inv = base ** (-np.arange(dh // 2) * 2.0 / dh)
    ang = np.arange(S)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def test_rope_is_a_complex_rotation_with_relative_position_inner_products():
    S, H, dh = 10, 3, 8
    cos, sin = _rope_tables(S, dh)
    x = _rand((S, H * dh), 20)
    pos = np.arange(S)
    y = bo.rope(x, cos, sin, pos, dh)
    # an independent statement: the pair (x_i, x_{i+dh/2}) is the complex number x_i + 1j x_{i+dh/2} multiplied by exp(1j pos theta_i)
    xh = x.reshape(S, H, dh)
    z = (xh[..., :dh // 2] + 1j * xh[..., dh // 2:]) * np.exp(1j * np.arange(S)[:, None, None] * (10000.0 ** (-np.arange(dh // 2) * 2.0 / dh)))
    assert np.allclose(y.reshape(S, H, dh), np.concatenate([z.real, z.imag], axis=-1), rtol=1e-13, atol=1e-15)
    # position 0 is the identity; norms of heads are preserved
    assert np.array_equal(y[0], x[0])
    assert np.allclose(np.linalg.norm(y.reshape(S, H, dh), axis=-1), np.linalg.norm(xh, axis=-1), rtol=1e-13)
    # <rope(q, m), rope(k, n)> depends on m - n only
    q, k = _rand((1, dh), 21), _rand((1, dh), 22)
    at = lambda v, p: bo.rope(v, cos, sin, np.array([p]), dh)[0]
    assert at(q, 7) @ at(k, 4) == pytest.approx(at(q, 5) @ at(k, 2), rel=1e-12)
    assert at(q, 7) @ at(k, 4) != pytest.approx(at(q, 7) @ at(k, 5), rel=1e-3)
    # the backward pass is the transpose: <rope(x), w> = <x, rope_backward(w)>, and it undoes the rotation
    w = _rand((S, H * dh), 23)
    assert (y * w).sum() == pytest.approx((x * bo.rope_backward(w, cos, sin, pos, dh)).sum(), rel=1e-12)
    assert np.allclose(bo.rope_backward(y, cos, sin, pos, dh), x, rtol=1e-12, atol=1e-14)


def _sdpa(q, k, v, n_seq, n_q, n_kv, dh):
    """torch's scaled_dot_product_attention on [n_seq, heads, S, dh] tensors, key / value heads repeated for their query heads."""
    T = q.shape[0]
    S = T // n_seq
    sp = lambda t, H: t.reshape(n_seq, S, H, dh).permute(0, 2, 1, 3)
    rep = n_q // n_kv
    o = torch.nn.functional.scaled_dot_product_attention(sp(q, n_q), sp(k, n_kv).repeat_interleave(rep, dim=1),
                                                         sp(v, n_kv).repeat_interleave(rep, dim=1), is_causal=True)
    return o.permute(0, 2, 1, 3).reshape(T, n_q * dh)


def test_attention_forward_and_backward_against_a_library_and_its_autograd():
    n_seq, S, n_q, n_kv, dh = 2, 7, 4, 2, 8
    T = n_seq * S
    q, k, v, do = _rand((T, n_q * dh), 30), _rand((T, n_kv * dh), 31), _rand((T, n_kv * dh), 32), _rand((T, n_q * dh), 33)
    scale = 1.0 / np.sqrt(dh)
    o, P = bo.attention(q, k, v, n_seq, n_q, n_kv, dh, scale)
    qt, kt, vt = (torch.from_numpy(t).requires_grad_(True) for t in (q, k, v))
    ot = _sdpa(qt, kt, vt, n_seq, n_q, n_kv, dh)
    assert np.allclose(o, ot.detach().numpy(), rtol=1e-12, atol=1e-14)
    ot.backward(torch.from_numpy(do))
    dq, dk, dv = bo.attention_backward(do, q, k, v, P, n_seq, n_q, n_kv, dh, scale)
    for got, want in ((dq, qt.grad), (dk, kt.grad), (dv, vt.grad)):
        assert np.allclose(got, want.numpy(), rtol=1e-10, atol=1e-13)
    # rows of P sum to one, nothing above the diagonal; the first token of a sequence attends to itself only: o = v
    assert np.allclose(P.sum(axis=-1), 1.0, rtol=1e-14) and np.all(np.triu(P, 1) == 0.0)
    for b in range(n_seq):
        for j in range(n_q):
            assert np.allclose(o[b * S, j * dh:(j + 1) * dh], v[b * S, (j // 2) * dh:(j // 2 + 1) * dh], rtol=1e-14)
    # causal, and sequences do not see each other: changing later tokens (or another sequence) leaves earlier outputs alone
    k2, v2 = k.copy(), v.copy()
    k2[5:] += 1.0
    v2[5:] -= 2.0
    o2, _ = bo.attention(q, k2, v2, n_seq, n_q, n_kv, dh, scale)
    assert np.array_equal(o2[:5], o[:5]) and not np.allclose(o2[5:7], o[5:7])
    # a finite difference through the oracle's own forward, one entry each
    f = lambda qq, kk, vv: float((bo.attention(qq, kk, vv, n_seq, n_q, n_kv, dh, scale)[0] * do).sum())
    for arr, grad, idx in ((q, dq, (9, 13)), (k, dk, (3, 6)), (v, dv, (8, 11))):
        e = np.zeros_like(arr); e[idx] = 1e-6
        args = lambda d: tuple(a + d if a is arr else a for a in (q, k, v))
        assert grad[idx] == pytest.approx((f(*args(e)) - f(*args(-e))) / 2e-6, rel=1e-6, abs=1e-10)


def _tiny_attn_block(n_seq=2, S=6, D=32, n_q=4, n_kv=2, dh=8, seed=0):
    rng = np.random.default_rng(seed)
    T = n_seq * S
    layers = {}
    for i, (name, O, K) in enumerate((("q", n_q * dh, D), ("k", n_kv * dh, D), ("v", n_kv * dh, D), ("o", D, n_q * dh))):
        W = synth.student_t_weight(O, K, 400 + seed + i, scale=0.2)
        qz = fo.quant_rtn(W, True)
        V = np.clip(fo.init_v(W, qz["s_global"], qz["scales"])["V"] + rng.uniform(-0.2, 0.2, W.shape), 0.05, 0.95).astype(np.float32)
        layers[name] = (W, qz["s_global"], qz["scales"], V)
    x = rng.standard_normal((T, D))
    g = rng.uniform(0.5, 1.5, D)
    y_fp = x + rng.standard_normal((T, D)) * 0.3
    qk = (rng.uniform(0.5, 1.5, dh), rng.uniform(0.5, 1.5, dh))
    return x, g, layers, y_fp, qk


@pytest.mark.parametrize("with_qk_norm", [False, True])
def test_attn_block_step_against_autograd_through_an_independent_graph(with_qk_norm):
    """The whole attention half (norm, q / k / v projections, per-head norm, rotary embedding, causal grouped-query attention,
    output projection, residual, block-output MSE): values and every gradient against torch autograd through library ops."""
    n_seq, S, D, n_q, n_kv, dh = 2, 6, 32, 4, 2, 8
    T = n_seq * S
    x, g, layers, y_fp, qk = _tiny_attn_block()
    cos, sin = _rope_tables(S, dh)
    beta, lam, ms = 6.0, 0.02, 1.0 / (T * D)
    r = bo.attn_block_step(x, g, 1e-6, layers, n_seq, n_q, n_kv, dh, cos, sin, beta, lam, y_fp=y_fp, mse_scale=ms,
                           qk_norm=qk if with_qk_norm else None)
    Vt, Wq = {}, {}
    for name, (W, sg, sb, V) in layers.items():
        sign, lo, hi, s = (torch.from_numpy(np.ascontiguousarray(t)) for t in fo.interval_terms(W, sg, sb))
        Vt[name] = torch.from_numpy(V.astype(np.float64)).requires_grad_(True)
        Wq[name] = sign * (lo + torch.sigmoid(beta * (Vt[name] - 0.5)) * (hi - lo)) * s
    xt = torch.from_numpy(x).requires_grad_(True)
    h = torch.nn.functional.rms_norm(xt, (D,), torch.from_numpy(g), 1e-6)
    q, k, v = h @ Wq["q"].T, h @ Wq["k"].T, h @ Wq["v"].T
    if with_qk_norm:
        q = torch.nn.functional.rms_norm(q.reshape(T, n_q, dh), (dh,), torch.from_numpy(qk[0]), 1e-6).reshape(T, -1)
        k = torch.nn.functional.rms_norm(k.reshape(T, n_kv, dh), (dh,), torch.from_numpy(qk[1]), 1e-6).reshape(T, -1)

    def rot(t, H):      # rotate-half form written with torch ops on [T, H, dh]
        c = torch.from_numpy(np.tile(cos, (n_seq, 2)))[:, None, :]
        s_ = torch.from_numpy(np.tile(sin, (n_seq, 2)))[:, None, :]
        th = t.reshape(T, H, dh)
        half = torch.cat([-th[..., dh // 2:], th[..., :dh // 2]], dim=-1)
        return (th * c + half * s_).reshape(T, -1)

    o = _sdpa(rot(q, n_q), rot(k, n_kv), v, n_seq, n_q, n_kv, dh)
    y = xt + o @ Wq["o"].T
    L = ms * ((y - torch.from_numpy(y_fp)) ** 2).sum()
    rl = sum((1 - (2 * vv - 1) ** 2).mean() for vv in Vt.values())
    (L + lam * rl).backward()
    assert r["L_block"] == pytest.approx(float(L.detach()), rel=1e-12)
    assert np.allclose(r["y"], y.detach().numpy(), rtol=1e-11, atol=1e-13)
    for name in layers:
        assert np.allclose(r["dV"][name], Vt[name].grad.numpy(), rtol=1e-8, atol=1e-14), name
    assert np.allclose(r["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-13)
    # given an upstream gradient instead of its own loss, the half back-propagates exactly that gradient
    up = _rand((T, D), 40)
    r2 = bo.attn_block_step(x, g, 1e-6, layers, n_seq, n_q, n_kv, dh, cos, sin, beta, 0.0, d_out=up,
                            qk_norm=qk if with_qk_norm else None)
    for vv in Vt.values():
        vv.grad = None
    xt.grad = None
    Wq2 = {}
    for name, (W, sg, sb, V) in layers.items():
        sign, lo, hi, s = (torch.from_numpy(np.ascontiguousarray(t)) for t in fo.interval_terms(W, sg, sb))
        Wq2[name] = sign * (lo + torch.sigmoid(beta * (Vt[name] - 0.5)) * (hi - lo)) * s
    h = torch.nn.functional.rms_norm(xt, (D,), torch.from_numpy(g), 1e-6)
    q, k, v = h @ Wq2["q"].T, h @ Wq2["k"].T, h @ Wq2["v"].T
    if with_qk_norm:
        q = torch.nn.functional.rms_norm(q.reshape(T, n_q, dh), (dh,), torch.from_numpy(qk[0]), 1e-6).reshape(T, -1)
        k = torch.nn.functional.rms_norm(k.reshape(T, n_kv, dh), (dh,), torch.from_numpy(qk[1]), 1e-6).reshape(T, -1)
    y2 = xt + _sdpa(rot(q, n_q), rot(k, n_kv), v, n_seq, n_q, n_kv, dh) @ Wq2["o"].T
    y2.backward(torch.from_numpy(up))
    for name in layers:
        assert np.allclose(r2["dV"][name], Vt[name].grad.numpy(), rtol=1e-8, atol=1e-14), name
    assert np.allclose(r2["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-13)


def test_attn_block_step_bf16_storage_is_a_small_perturbation():
    n_seq, S, D, n_q, n_kv, dh = 2, 6, 32, 4, 2, 8
    x, g, layers, y_fp, qk = _tiny_attn_block(seed=5)
    cos, sin = _rope_tables(S, dh)
    a = dict(y_fp=y_fp, mse_scale=1.0 / (12 * 32), qk_norm=qk)
    r = bo.attn_block_step(x, g, 1e-6, layers, n_seq, n_q, n_kv, dh, cos, sin, 5.0, 0.01, **a)
    b = bo.attn_block_step(x, g, 1e-6, layers, n_seq, n_q, n_kv, dh, cos, sin, 5.0, 0.01, bf16_storage=True, **a)
    n = np.linalg.norm
    assert b["L_block"] == pytest.approx(r["L_block"], rel=2e-2)
    for name in layers:
        assert 0 < n(b["dV"][name] - r["dV"][name]) <= 4e-2 * n(r["dV"][name]), name
    assert 0 < n(b["dx"] - r["dx"]) <= 3e-2 * n(r["dx"])
