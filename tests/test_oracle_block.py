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
