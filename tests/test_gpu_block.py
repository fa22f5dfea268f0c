"""GPU parity of the block glue (RMSNorm, gated SiLU, residual + block-output MSE, the soft-quantised linear's
forward) and of a whole joint step of a block's MLP half, against the float64 oracle.

Tolerances.  Each kernel reads bf16 or float32 inputs, computes in float32 and stores bf16: against the oracle given the
SAME inputs, an output element is one bf16 rounding (2^-9 relative; asserted 2^-8) of a float32 value that is itself
good to a few 1e-7 of the row's scale.  The composed step is compared with the oracle in its bf16-storage mode (the
same rounding points): what remains is float32 accumulation and rounding-boundary flips, a few 1e-3 of a tensor's rms
per element once several rounded tensors are chained; and with the exact float64 oracle norm-wise."""
import numpy as np
import pytest
import torch

from oracle import block_oracle as bo
from oracle import faar_oracle as fo
from workloads import synth

pytestmark = pytest.mark.gpu

import paper_2603_22370_amd as faar  # noqa: E402

U8 = 2.0 ** -8


def dev(a, bf16=True):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def bf(a):
    return synth.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)


def close(got, want, rel=U8, floor=0.0):
    return np.all(np.abs(got - want) <= rel * np.abs(want) + floor)


@pytest.mark.parametrize("T,D", [(1, 8), (7, 40), (300, 256), (65, 2048), (3, 6152)])
@pytest.mark.parametrize("xbf", [True, False])
def test_rmsnorm_forward_and_backward(T, D, xbf):
    rng = np.random.default_rng([T, D])
    x = rng.standard_normal((T, D)) * 2.0
    x[:, :: 17] *= 20.0                                   # outlier channels
    x = bf(x) if xbf else x.astype(np.float32).astype(np.float64)
    g = rng.uniform(0.5, 1.5, D).astype(np.float32)
    h, rstd = faar.faar_rmsnorm_fwd(dev(x, xbf), torch.from_numpy(g).cuda(), 1e-6)
    h_want, r_want = bo.rmsnorm(x, g, 1e-6)
    assert np.allclose(host(rstd), r_want, rtol=2e-6)
    assert close(host(h), h_want, floor=1e-30)
    dh1, dh2, dres = (bf(rng.standard_normal((T, D)) * s) for s in (1e-3, 1e-3, 1e-3))
    for use2, user in ((True, True), (False, False)):
        dx = faar.faar_rmsnorm_bwd(dev(dh1), dev(x, xbf), torch.from_numpy(g).cuda(), rstd, dh2=dev(dh2) if use2 else None,
                                   d_res=dev(dres) if user else None)
        want = bo.rmsnorm_backward(dh1 + (dh2 if use2 else 0.0), x, g, host(rstd)) + (dres if user else 0.0)
        # the two terms of dx cancel where x dominates: float32 noise is relative to their size, not to dx
        scale = np.abs(host(rstd))[:, None] * np.abs(g * (dh1 + (dh2 if use2 else 0.0))) + np.abs(dres if user else 0.0)
        assert close(host(dx), want, floor=4e-6 * scale.max(axis=1, keepdims=True) + 1e-30)


@pytest.mark.parametrize("n", [8, 2048 + 8, 300 * 640])
def test_silu_mul_forward_and_backward(n):
    rng = np.random.default_rng(n)
    p, q, da = bf(rng.standard_normal(n) * 3.0), bf(rng.standard_normal(n)), bf(rng.standard_normal(n) * 1e-3)
    p[:4] = [0.0, -30.0, 30.0, -0.0]
    a = faar.faar_silu_mul_fwd(dev(p), dev(q))
    assert close(host(a), bo.silu_mul(p, q), floor=1e-30)
    dp, dq = faar.faar_silu_mul_bwd(dev(da), dev(p), dev(q))
    dp_want, dq_want = bo.silu_mul_backward(da, p, q)
    assert close(host(dp), dp_want, floor=2e-6 * np.abs(da * q) + 1e-30) and close(host(dq), dq_want, floor=1e-30)


@pytest.mark.parametrize("T,D", [(3, 8), (300, 256), (1000, 2048)])
@pytest.mark.parametrize("dts", [(True, True), (False, False), (True, False)])
def test_block_output_loss(T, D, dts):
    xbf, ybf = dts
    rng = np.random.default_rng([T, D, 5])
    x, d, yf = rng.standard_normal((T, D)), rng.standard_normal((T, D)) * 0.5, rng.standard_normal((T, D))
    x = bf(x) if xbf else x.astype(np.float32).astype(np.float64)
    d = bf(d)
    yf = bf(yf) if ybf else yf.astype(np.float32).astype(np.float64)
    ms = 1.0 / (T * D)
    loss, dy, y = faar.faar_block_output_loss(dev(x, xbf), dev(d), dev(yf, ybf), ms, want_y=True)
    y_want, L_want, dy_want = bo.block_output_loss(x, d, yf, ms)
    assert loss.item() == pytest.approx(L_want, rel=2e-6)
    assert close(host(y), y_want, floor=1e-30)
    assert close(host(dy), dy_want, floor=2.0 * ms * 4e-7 * (np.abs(x) + np.abs(d) + np.abs(yf)) + 1e-30)


def _layer(O, K, seed):
    W = synth.student_t_weight(O, K, seed, scale=0.05)
    q = fo.quant_rtn(W, True)
    V = synth.rounding_variables(O, K, seed + 1)
    return W, q["s_global"], q["scales"], V


def test_linear_forward():
    # the last shape takes the 256x256-tile kernel with 32 contraction slices (the benchmark's gate projection, a slice of its tokens)
    # (100, 128) and (300, 64): output widths that are not multiples of 8 -- rows whose pitch rules out 16-byte stores, and a
    # last run of columns that is cut short -- through the 128x128-tile kernel and (the last two) both 64-wide-slice kernels
    for (O, K, T, seed) in ((96, 80, 100, 1), (640, 256, 300, 2), (2048, 512, 1024, 3), (6144, 2048, 2048, 4),
                            (100, 128, 200, 5), (300, 64, 2048, 6), (1028, 64, 4096, 7), (2052, 64, 4096, 8)):
        W, sg, sb, V = _layer(O, K, seed)
        X = synth.activations(T, K, seed)
        Wd = dev(W)
        sgd, scd, _, _ = faar.faar_quant_rtn(Wd)
        Y = faar.faar_linear_forward(Wd, sgd, scd, dev(V, False), 7.0, dev(X))
        Wq = bf(fo.soft_weight(W, sg, sb, V, 7.0))                       # the declared rounding of W_q
        want = X.astype(np.float64) @ Wq.T
        scale = np.abs(X.astype(np.float64)) @ np.abs(Wq).T
        # W_q is float32 arithmetic before its rounding to bf16: where that value sits on a rounding boundary the kernel
        # may round the other way than the float64 oracle, which moves that one term of the sum by 2^-8 of itself --
        # allow two such terms of the largest size in the row, on top of the output's own bf16 rounding
        big = np.abs(X.astype(np.float64)).max(axis=1)[:, None] * np.abs(Wq).max(axis=1)[None, :]
        assert np.all(np.abs(host(Y) - want) <= U8 * np.abs(want) + 2 * U8 * big + 4e-6 * scale + 1e-30)
        assert np.linalg.norm(host(Y) - want) <= 2.5e-3 * np.linalg.norm(want)


def test_joint_step_of_the_mlp_half_of_a_block():
    """RMSNorm -> gate / up -> SiLU * -> down -> residual -> block-output MSE, and back into the rounding variables of all
    three linears and into the block's input: every intermediate tensor and every gradient against the oracle, then one
    Adam update of each V (faar_layer_step in its joint form) against the oracle's update rule."""
    T, D, F = 300, 256, 640
    rng = np.random.default_rng(77)
    names = (("gate", F, D), ("up", F, D), ("down", D, F))
    layers = {n: _layer(O, K, 500 + i) for i, (n, O, K) in enumerate(names)}
    x = bf(synth.activations(T, D, 9))
    g = rng.uniform(0.5, 1.5, D).astype(np.float32)
    y_fp = bf(x + rng.standard_normal((T, D)) * 0.2)
    beta, lam, ms, eps = 6.0, 0.01, 1.0 / (T * D), 1e-6
    ref = bo.mlp_block_step(x, g, eps, layers, y_fp, ms, beta, lam, bf16_storage=True)
    exact = bo.mlp_block_step(x, g, eps, layers, y_fp, ms, beta, lam)

    L = {}
    for n, (W, sg, sb, V) in layers.items():
        Wd = dev(W)
        sgd, scd, _, _ = faar.faar_quant_rtn(Wd)
        Vd = dev(V, False)
        L[n] = dict(W=Wd, sg=sgd, sc=scd, V=Vd, m=torch.zeros_like(Vd), u=torch.zeros_like(Vd),
                    losses=torch.zeros(3, dtype=torch.float32, device="cuda"))
    xd, gd = dev(x), torch.from_numpy(g).cuda()
    h, rstd = faar.faar_rmsnorm_fwd(xd, gd, eps)
    fwd = lambda n, X: faar.faar_linear_forward(L[n]["W"], L[n]["sg"], L[n]["sc"], L[n]["V"], beta, X)
    p, q = fwd("gate", h), fwd("up", h)
    a = faar.faar_silu_mul_fwd(p, q)
    d = fwd("down", a)
    loss, dy, y = faar.faar_block_output_loss(xd, d, dev(y_fp), ms, want_y=True)

    def rms(t):
        return np.sqrt(np.mean(t ** 2))

    measured = {}

    def near(got, want, name, norm=3e-3):
        """Down a chain of kernels each tensor inherits the rounding-boundary flips of everything upstream (one bf16 ulp
        of an outlier activation moves SiLU' of that element by per cents), so the composed step is held norm-wise to
        the oracle with the same storage roundings -- measured 4e-5 ... 1.4e-3 -- and per element only loosely (8 ulp +
        0.05 rms, measured up to 0.023: what an indexing mistake would break); each kernel on its own is compared element by element above."""
        got = host(got)
        e_norm = np.linalg.norm(got - want) / np.linalg.norm(want)
        e_elem = float(((np.abs(got - want) - 8 * U8 * np.abs(want)) / rms(want)).max())
        measured[name] = (e_norm, e_elem)
        print(f"{name}: norm {e_norm:.2e}  element excess {e_elem:.2e} rms", flush=True)
        assert e_norm <= norm, (name, e_norm)
        assert e_elem <= 0.05, (name, e_elem)

    for got, key in ((h, "h"), (p, "p"), (q, "q"), (a, "a"), (d, "d"), (dy, "dy")):
        near(got, ref[key], key)
    assert loss.item() == pytest.approx(ref["L_block"], rel=2e-3)
    assert loss.item() == pytest.approx(exact["L_block"], rel=2e-2)

    hyp = dict(lr=5e-3, b1=0.9, b2=0.999, eps=1e-8)

    def back(n, X, dY):
        lay = L[n]
        O, K = lay["W"].shape
        Xt, _, ic = faar.faar_layer_prepare(lay["W"], lay["sg"], lay["sc"], X, None)
        ws = faar.layer_step_workspace(O, K, T, chained=True)
        dX = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
        V0 = lay["V"].clone()
        faar.faar_layer_step(lay["W"], lay["sg"], lay["sc"], lay["V"], lay["m"], lay["u"], X, Xt, None, ic, beta, lam, 0.0,
                             hyp["lr"], hyp["b1"], hyp["b2"], hyp["eps"], 1, lay["losses"], ws, dY_ext=dY, dX=dX, joint=True)
        torch.cuda.synchronize()
        grad = host(lay["m"]) / (1 - hyp["b1"])            # zero initial state: m = (1 - beta1) g
        want, want_exact = ref["dV"][n], exact["dV"][n]
        nrm = np.linalg.norm
        assert nrm(grad - want) <= 3e-3 * nrm(want), n
        assert nrm(grad - want_exact) <= 3e-2 * nrm(want_exact), n
        assert np.all(np.abs(grad - want) <= 2 ** -6 * np.abs(want) + 2e-2 * rms(want)), n
        Ls = host(lay["losses"])
        assert Ls[0] == 0.0 and Ls[1] == pytest.approx(ref["L_round"][n], rel=1e-5) and Ls[2] == pytest.approx(lam * ref["L_round"][n], rel=1e-5)
        Vn, _, _ = fo.adam_update(host(V0), np.zeros_like(grad), np.zeros_like(grad), grad, hyp["lr"], hyp["b1"], hyp["b2"], hyp["eps"], 1)
        assert np.all(np.abs(host(lay["V"]) - Vn) <= 1e-4 * hyp["lr"] + 1.2e-7), n
        return dX

    da = back("down", a, dy)
    near(da, ref["da"], "da")
    dp, dq = faar.faar_silu_mul_bwd(da, p, q)
    near(dp, ref["dp"], "dp")
    near(dq, ref["dq"], "dq")
    dh1, dh2 = back("gate", h, dp), back("up", h, dq)
    dx = faar.faar_rmsnorm_bwd(dh1, xd, gd, rstd, dh2=dh2, d_res=dy)
    near(dx, ref["dx"], "dx")
    assert np.linalg.norm(host(dx) - exact["dx"]) <= 3e-2 * np.linalg.norm(exact["dx"])
