"""Pins for the oracle's float arithmetic: soft quantiser (Eq. 2-3), Round Loss and Stage-1
objective (Eq. 5), their gradients, the update rule, the beta -> infinity limit and a brute
force over every rounding of a tiny layer (Sec. 3.3, Eq. 1)."""
import itertools

import numpy as np
import pytest

from oracle import faar_oracle as fo
from workloads import synth

NODES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def _tiny(O=6, K=32, T=10, seed=0, quantised_acts=True):
    rng = np.random.default_rng(seed)
    W = synth.student_t_weight(O, K, seed + 100)
    W[0, 3] = 0.0                                          # a zero weight: sign(0) = 0
    X = synth.activations(T, K, seed + 200, n_outlier=2, outlier_mult=10.0)
    Xq = synth.perturbed_activations(X, seed + 300) if quantised_acts else X
    Y = synth.frozen_output(X, W)
    sg = fo.tensor_scale(W)
    sb = fo.block_scale_bytes(W, sg)
    V = rng.uniform(0.05, 0.95, size=W.shape).astype(np.float32)
    return W, sg, sb, V, X, Xq, Y


def _loss(W, sg, sb, V, Xq, Y, beta, lam, alpha):
    """Eq. 5 retyped from the paper with plain loops over python floats (independent evaluator)."""
    O, K = W.shape
    T = Xq.shape[0]
    s_g = fo.e4m3_decode(sb)
    Wq = np.zeros((O, K))
    for o in range(O):
        for k in range(K):
            s = float(np.float32(s_g[o, k // 16]) * np.float32(sg))
            w = float(W[o, k])
            wt = float(np.float32(abs(w)) / np.float32(s)) if s > 0 else 0.0
            lo = max(n for n in NODES[:7] if n <= wt)
            hi = NODES[list(NODES).index(lo) + 1]
            h = 1.0 / (1.0 + np.exp(-beta * (float(V[o, k]) - 0.5)))
            sign = (w > 0) - (w < 0)
            Wq[o, k] = sign * (lo + h * (hi - lo)) * s
    mse = 0.0
    for t in range(T):
        for o in range(O):
            y = sum(float(Xq[t, k]) * Wq[o, k] for k in range(K))
            mse += (float(Y[t, o]) - y) ** 2
    rl = sum(1.0 - (2.0 * float(v) - 1.0) ** 2 for v in V.reshape(-1)) / V.size
    return alpha * mse + lam * rl, alpha * mse, rl


def test_losses_match_a_loop_evaluator():
    W, sg, sb, V, X, Xq, Y = _tiny(O=3, K=16, T=4)
    r = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, beta=7.0, lambda_round=0.3, alpha=0.5)
    L, mse, rl = _loss(W, sg, sb, V.astype(np.float64), Xq, Y, 7.0, 0.3, 0.5)
    assert r["L"] == pytest.approx(L, rel=1e-12)
    assert r["L_mse"] == pytest.approx(mse, rel=1e-12)
    assert r["L_round"] == pytest.approx(rl, rel=1e-12)


def test_round_loss_closed_forms():
    n = (8, 16)
    assert fo.round_loss(np.full(n, 0.5)) == 1.0
    assert fo.round_loss(np.zeros(n)) == 0.0
    assert fo.round_loss(np.ones(n)) == 0.0
    assert fo.round_loss(np.full(n, 0.25)) == 0.75
    v = np.zeros(n); v[0, 0] = 0.5
    assert fo.round_loss(v) == pytest.approx(1.0 / 128)


def test_h_beta_properties():
    v = np.linspace(0, 1, 101)
    assert fo.h_beta(0.5, 3.0) == 0.5
    assert np.allclose(fo.h_beta(v, 9.0) + fo.h_beta(1 - v, 9.0), 1.0, atol=1e-15)
    assert np.all(np.diff(fo.h_beta(v, 9.0)) > 0)
    assert fo.h_beta(0.75, 4.0) == pytest.approx(1 / (1 + np.exp(-1.0)))
    assert fo.h_beta(0.6, 1e5) == pytest.approx(1.0) and fo.h_beta(0.4, 1e5) == pytest.approx(0.0)


def test_large_beta_equals_hardened_weights():
    W, sg, sb, V, X, Xq, Y = _tiny(O=8, K=64)
    V[np.abs(V - 0.5) < 1e-3] = 0.7
    soft = fo.soft_weight(W, sg, sb, V, beta=1e6)
    hard = fo.harden_pack(W, False, sg, sb, V)["W_final"].astype(np.float64)
    assert np.allclose(soft, hard, rtol=2e-7, atol=0)
    # and the loss at beta -> inf equals the hardened loss
    r = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, beta=1e6, lambda_round=0.0, alpha=1.0)
    assert r["L_mse"] == pytest.approx(fo.hardened_loss(W, False, sg, sb, V, Xq, Y, 1.0), rel=1e-5)


@pytest.mark.parametrize("alpha,lam,beta", [(1.0, 0.0, 5.0), (1.0 / 60, 0.01, 12.0), (0.37, 2.5, 3.0)])
def test_dV_by_central_differences(alpha, lam, beta):
    W, sg, sb, V, X, Xq, Y = _tiny()
    V64 = V.astype(np.float64)
    r = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, beta, lam, alpha)
    # the oracle takes V as float32 storage; perturb in float64 around it through a float64 re-evaluation
    def L_of(Vd):
        sign, lo, hi, s = fo.interval_terms(W, sg, sb)
        Wq = sign * (lo + fo.h_beta(Vd, beta) * (hi - lo)) * s
        R = Xq.astype(np.float64) @ Wq.T - Y.astype(np.float64)
        return alpha * np.sum(R * R) + lam * fo.round_loss(Vd)
    assert L_of(V64) == pytest.approx(r["L"], rel=1e-13)
    eps = 1e-6
    rng = np.random.default_rng(1)
    idx = [(0, 3)] + [tuple(x) for x in np.stack([rng.integers(0, W.shape[0], 40), rng.integers(0, W.shape[1], 40)], 1)]
    scale = np.abs(r["dV"]).max()
    for (o, k) in idx:
        Vp = V64.copy(); Vp[o, k] += eps
        Vm = V64.copy(); Vm[o, k] -= eps
        fd = (L_of(Vp) - L_of(Vm)) / (2 * eps)
        assert abs(fd - r["dV"][o, k]) <= 1e-6 * scale + 1e-7 * abs(fd), (o, k)
    # the zero weight only feels the Round-Loss term
    assert r["dV"][0, 3] == pytest.approx(lam / W.size * (4 - 8 * V64[0, 3]), rel=1e-12, abs=1e-300)


def test_dX_by_central_differences():
    W, sg, sb, V, X, Xq, Y = _tiny()
    beta, lam, alpha = 6.0, 0.1, 0.25
    r = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, beta, lam, alpha, want_dX=True)
    Wq = fo.soft_weight(W, sg, sb, V, beta)
    def L_of(Xd):
        R = Xd @ Wq.T - Y.astype(np.float64)
        return alpha * np.sum(R * R)
    eps = 1e-6
    X64 = Xq.astype(np.float64)
    scale = np.abs(r["dX"]).max()
    for (t, k) in [(0, 0), (3, 17), (9, 31), (5, 8)]:
        Xp = X64.copy(); Xp[t, k] += eps
        Xm = X64.copy(); Xm[t, k] -= eps
        fd = (L_of(Xp) - L_of(Xm)) / (2 * eps)
        assert abs(fd - r["dX"][t, k]) <= 1e-6 * scale


def test_gradient_scales_with_interval_width():
    """Two weights identical except for the interval they fall in: dL/dV ratio = width ratio
    (Sec. 3.4: larger-interval weights receive stronger gradients)."""
    K = 16
    W = np.zeros((2, K), dtype=np.float32)
    # both rows: block amax 6 -> same scale; element 1 sits in [1, 1.5] (row 0) or [4, 6] (row 1)
    W[:, 0] = 6.0
    W[0, 1] = 1.25
    W[1, 1] = 5.0
    sg = np.float32(2.0 ** -7)                        # makes s = 1 for a block with amax 6 -> byte 0x70
    sb = fo.block_scale_bytes(W, sg)
    assert np.all(sb == 0x70)
    V = np.full((2, K), 0.5, dtype=np.float32)
    Xq = np.zeros((1, K), dtype=np.float32); Xq[0, 1] = 1.0
    sign, lo, hi, s = fo.interval_terms(W, sg, sb)
    Wq = fo.soft_weight(W, sg, sb, V, 4.0)
    Y = (Xq.astype(np.float64) @ Wq.T + 0.3).astype(np.float32)   # same residual (-0.3) for both outputs
    r = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 4.0, 0.0, 1.0)
    assert (hi - lo)[0, 1] == 0.5 and (hi - lo)[1, 1] == 2.0
    assert r["dV"][1, 1] / r["dV"][0, 1] == pytest.approx(4.0, rel=1e-6)


def test_dY_ext_replaces_local_gradient():
    W, sg, sb, V, X, Xq, Y = _tiny()
    rng = np.random.default_rng(3)
    dY = rng.standard_normal((Xq.shape[0], W.shape[0]))
    r = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 5.0, 0.0, 1.0, want_dX=True, dY_ext=dY)
    sign, lo, hi, s = fo.interval_terms(W, sg, sb)
    h = fo.h_beta(V, 5.0)
    want = np.einsum("to,tk->ok", dY, Xq.astype(np.float64)) * sign * s * (hi - lo) * 5.0 * h * (1 - h)
    assert np.allclose(r["dV"], want, rtol=1e-12, atol=1e-18)
    assert np.allclose(r["dX"], dY @ r["Wq"], rtol=1e-12, atol=1e-18)


def test_adam_first_step_identity_and_clip():
    rng = np.random.default_rng(0)
    V = rng.uniform(0.2, 0.8, (4, 16))
    g = rng.standard_normal((4, 16))
    Vn, m, u = fo.adam_update(V, np.zeros_like(V), np.zeros_like(V), g, 1e-2, 0.9, 0.999, 1e-8, 1)
    assert np.allclose(Vn, V - 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    assert np.allclose(m, 0.1 * g) and np.allclose(u, 0.001 * g * g)
    # second step by hand for one element
    g2 = rng.standard_normal((4, 16))
    Vn2, m2, u2 = fo.adam_update(Vn, m, u, g2, 1e-2, 0.9, 0.999, 1e-8, 2)
    m_h = (0.9 * 0.1 * g[0, 0] + 0.1 * g2[0, 0]) / (1 - 0.81)
    u_h = (0.999 * 0.001 * g[0, 0] ** 2 + 0.001 * g2[0, 0] ** 2) / (1 - 0.999 ** 2)
    assert Vn2[0, 0] == pytest.approx(Vn[0, 0] - 1e-2 * m_h / (np.sqrt(u_h) + 1e-8), rel=1e-12)
    # clip to [0, 1]
    Vc, _, _ = fo.adam_update(np.array([[0.001, 0.999]]), np.zeros((1, 2)), np.zeros((1, 2)),
                              np.array([[1.0, -1.0]]), 0.1, 0.9, 0.999, 1e-8, 1)
    assert Vc[0, 0] == 0.0 and Vc[0, 1] == 1.0


def test_declared_rounding_mode_is_a_small_perturbation():
    W, sg, sb, V, X, Xq, Y = _tiny(O=16, K=64, T=64)
    a = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, 1.0 / (64 * 16), want_dX=True)
    b = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, 1.0 / (64 * 16), want_dX=True,
                                 declared_rounding=True)
    assert b["L_mse"] == pytest.approx(a["L_mse"], rel=2e-3)
    assert np.linalg.norm(b["dV"] - a["dV"]) <= 1e-2 * np.linalg.norm(a["dV"])
    assert np.linalg.norm(b["dX"] - a["dX"]) <= 1e-2 * np.linalg.norm(a["dX"])
    assert b["L_round"] == a["L_round"]


def test_split_contract_mode_is_the_same_gradient_with_one_rounding_moved():
    """G = dY^T X_q with dY = 2 alpha (X_q d^T - C) splits into (2 alpha X_q d^T)^T X_q - 2 alpha C^T X_q.  The "split"
    contract rounds only the first factor to bf16: it must agree with the exact gradient to the size of that one
    rounding, agree with it EXACTLY when the factor happens to be bf16-representable (here: everything scaled so that
    the products are small integers), and leave the losses of the other contract untouched."""
    W, sg, sb, V, X, Xq, Y = _tiny(O=16, K=64, T=64)
    al = 1.0 / (64 * 16)
    a = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al)
    b = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al, declared_rounding=True)
    c = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al, declared_rounding="split")
    assert c["L_mse"] == b["L_mse"] and c["L_round"] == a["L_round"]
    n = np.linalg.norm
    assert 0 < n(c["dV"] - a["dV"]) <= 1e-2 * n(a["dV"])
    assert n(c["dV"] - b["dV"]) > 0                     # another rounding point: not the same numbers
    # the split itself is an identity: undo the roundings by hand and compare with the exact G
    W64, X64 = W.astype(np.float64), Xq.astype(np.float64)
    C = Y.astype(np.float64) - X64 @ W64.T
    d = a["Wq"] - W64
    G = (2 * al * (X64 @ d.T)).T @ X64 - 2 * al * (C.T @ X64)
    assert np.allclose(G, a["G"], rtol=1e-10, atol=1e-18)
    # an upstream gradient bypasses dY altogether: both contracts coincide
    dY = (np.arange(64 * 16).reshape(64, 16) % 7 - 3).astype(np.float32) * 2.0 ** -10
    e = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al, dY_ext=dY, declared_rounding=True)
    f = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al, dY_ext=dY, declared_rounding="split")
    assert np.array_equal(e["dV"], f["dV"])


def test_gram_contract_mode_is_eq5_expanded_over_the_token_gram_matrix():
    """||X d^T - C||^2 = <d Gm, d> - 2 <d, C^T X> + ||C||^2 and G = 2 alpha (d Gm - C^T X) with Gm = X^T X: the "gram"
    contract must agree with the exact loss and gradient to the size of its two roundings (d and the off-diagonal of
    Gm), and EXACTLY (to float64 summation order) when those roundings do nothing -- activations of small integers
    make Gm a matrix of small integers, and the rounding of d is shared with the plain declared mode, whose loss
    then has to coincide."""
    W, sg, sb, V, X, Xq, Y = _tiny(O=16, K=64, T=64)
    al = 1.0 / (64 * 16)
    a = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al)
    g = fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al, declared_rounding="gram")
    n = np.linalg.norm
    assert g["L_mse"] == pytest.approx(a["L_mse"], rel=4e-3) and g["L_round"] == a["L_round"]
    assert 0 < n(g["dV"] - a["dV"]) <= 1e-2 * n(a["dV"])
    # activations in {-1, 0, 1}: every entry of Gm is an integer of magnitude <= T = 64, which bf16 holds exactly
    rng = np.random.default_rng(5)
    Xi = rng.integers(-1, 2, size=Xq.shape).astype(np.float32)
    Gm = Xi.astype(np.float64).T @ Xi.astype(np.float64)
    assert np.array_equal(fo.bf16_round(Gm.astype(np.float32)).astype(np.float64), Gm)
    b = fo.stage1_loss_and_grads(W, sg, sb, V, Xi, Y, 8.0, 0.01, al, declared_rounding=True)
    gi = fo.stage1_loss_and_grads(W, sg, sb, V, Xi, Y, 8.0, 0.01, al, declared_rounding="gram")
    assert gi["L_mse"] == pytest.approx(b["L_mse"], rel=1e-11)
    # the gradient of the plain declared mode rounds dY as well; undo that by hand: G = (2 alpha R)^T X with the same d
    W64 = W.astype(np.float64)
    d = fo.bf16_round((b["Wq"] - W64).astype(np.float32)).astype(np.float64)
    R = Xi.astype(np.float64) @ d.T - (Y.astype(np.float64) - Xi.astype(np.float64) @ W64.T)
    assert np.allclose(gi["G"], (2 * al * R).T @ Xi.astype(np.float64), rtol=1e-10, atol=1e-18)
    with pytest.raises(ValueError):
        fo.stage1_loss_and_grads(W, sg, sb, V, Xq, Y, 8.0, 0.01, al, want_dX=True, declared_rounding="gram")


def test_brute_force_over_all_roundings_of_a_tiny_layer():
    """Eq. 1: enumerate every V in {0,1}^16 for one 16-weight row.  The oracle's hardened loss must
    agree with an independent evaluator (decode packed bytes -> dense matmul) at every assignment;
    RTN is one of the assignments, so min <= L(RTN); lower/upper-only are assignments too."""
    rng = np.random.default_rng(7)
    W = synth.student_t_weight(1, 16, 77)
    X = synth.activations(8, 16, 78, n_outlier=1, outlier_mult=8.0)
    Y = synth.frozen_output(X, W)
    q = fo.quant_rtn(W, True)
    sg, sb = q["s_global"], q["scales"]
    s_g = float(fo.e4m3_decode(sb)[0, 0])
    losses = {}
    for bits in itertools.product((0, 1), repeat=16):
        V = np.array(bits, dtype=np.float32).reshape(1, 16)
        hp = fo.harden_pack(W, False, sg, sb, V)
        nib = fo.unpack_nibbles(hp["codes"])[0]
        # independent decode of the packed bytes
        w = np.array([(-1.0 if c & 8 else 1.0) * NODES[c & 7] for c in nib]) * s_g * float(sg)
        L_ind = float(np.sum((X.astype(np.float64) @ w - Y[:, 0].astype(np.float64)) ** 2))
        L_orc = fo.hardened_loss(W, False, sg, sb, V, X, Y, 1.0)
        assert L_orc == pytest.approx(L_ind, rel=1e-4)   # W_final is float32; the residual cancels ~99%
        losses[bits] = L_ind
    V_rtn = (fo.init_v(W, sg, sb)["V"] >= 0.5).astype(int).reshape(-1)
    L_rtn = losses[tuple(V_rtn)]
    L_min = min(losses.values())
    assert L_min <= L_rtn
    assert fo.hardened_loss(W, False, sg, sb, fo.init_v(W, sg, sb)["V"], X, Y, 1.0) == pytest.approx(L_rtn, rel=1e-4)
    # the paper's empirical point (Sec. 3.2): RTN is not the optimum on a non-uniform grid
    assert L_min < L_rtn
    assert L_rtn <= max(losses[tuple([0] * 16)], losses[tuple([1] * 16)])


def test_optimisation_reduces_the_hardened_loss_on_config1():
    """A short run of the whole oracle loop (Table 2 steps 6-13) on the small parity config:
    V stays in [0,1], the soft loss falls, and the hardened loss ends at or below RTN's."""
    c = synth.config1(0)
    q = fo.quant_rtn(c.W, False)
    sg, sb = q["s_global"], q["scales"]
    V = fo.init_v(c.W, sg, sb)["V"]
    m = np.zeros_like(V); u = np.zeros_like(V)
    alpha = 1.0 / (c.T * c.O)
    L_rtn = fo.hardened_loss(c.W, False, sg, sb, V, c.Xq, c.Y_fp, alpha)
    first = None
    steps = 60
    for t in range(1, steps + 1):
        beta = 4.0 + (32.0 - 4.0) * (t - 1) / (steps - 1)
        r = fo.layer_step(c.W, sg, sb, V, m, u, c.Xq, c.Y_fp, beta, 1e-6, alpha, 1e-2, 0.9, 0.999, 1e-8, t)
        V, m, u = r["V"], r["m"], r["u"]
        assert V.min() >= 0.0 and V.max() <= 1.0
        first = r["L_mse"] if first is None else first
    L_end = fo.hardened_loss(c.W, False, sg, sb, V, c.Xq, c.Y_fp, alpha)
    assert L_end < L_rtn


def test_adam_matches_a_library_optimiser_over_several_steps():
    """Moments, bias correction and step size against torch.optim.Adam (float64, no weight decay), with the
    clip to [0, 1] applied to both after every update."""
    import torch
    rng = np.random.default_rng(12)
    V = rng.uniform(0.05, 0.95, size=(6, 16))
    p = torch.tensor(V.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=3e-2, betas=(0.9, 0.999), eps=1e-8)
    m = np.zeros_like(V)
    u = np.zeros_like(V)
    for t in range(1, 8):
        g = rng.standard_normal(V.shape) * (1.0 if t % 2 else 1e-3)
        V, m, u = fo.adam_update(V, m, u, g, 3e-2, 0.9, 0.999, 1e-8, t)
        p.grad = torch.tensor(g)
        opt.step()
        with torch.no_grad():
            p.clamp_(0.0, 1.0)
        assert np.allclose(np.asarray(V, dtype=np.float64), p.detach().numpy(), rtol=1e-6, atol=1e-7), t
