"""GPU parity of the step in its Gram-matrix form (faar_gram_prepare + faar_layer_step_gram, constant activations)
against the same oracle as the token form: Eq. 5 expanded over Gm = X_q^T X_q, Table 2 steps 6-13."""
import numpy as np
import pytest
import torch

from oracle import faar_oracle as fo
from workloads import synth

from parity_cases import BY_NAME, GRAM_CASES, STEP_CASES
import test_gpu_parity as tp

pytestmark = pytest.mark.gpu

import paper_2603_22370_amd as faar  # noqa: E402
from paper_2603_22370_amd import binding  # noqa: E402

dev, host, HYP, U = tp.dev, tp.host, tp.HYP, tp.U

# Roundings of this form: W_q - W and the off-diagonal of Gm, both to bf16 (the token form: W_q - W and dY).
#  * Against the oracle with those declared roundings ("gram" contract) what remains is float32 accumulation noise and
#    bf16 boundary flips of single entries of Gm and of W_q - W.
#  * Against the exact float64 oracle: the same bounds as the token form (two independent roundings of rms u / sqrt(3)).
TOL_LOSS_DECLARED = 2e-5
TOL_GRAD_DECLARED = 5e-4

SMALL = [c.name for c in STEP_CASES + GRAM_CASES if not c.full_size]
FULL = [c.name for c in STEP_CASES if c.full_size]


def _gram_setup(c):
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic), hk = tp._setup(c, h=True)
    gram, gram_lo = binding.faar_gram_prepare(Xt, c.T)
    return Wd, sg, scales, q, ic, hk, gram, gram_lo


@pytest.mark.parametrize("name", ["ragged", "three_tiles"] + FULL[:1])
def test_gram_matrix(name):
    """bf16(X_q^T X_q) entry by entry (a float32 sum of exact products next to a rounding boundary may round the other
    way: one bf16 ulp, rarely), and the diagonal's remainder."""
    c = tp.build_case(name)
    *_, gram, gram_lo = _gram_setup(c)
    X = c.Xq.astype(np.float64)
    Gm = X.T @ X
    g = host(gram).astype(np.float64)
    assert g.shape == (c.K, c.K)
    mag = np.abs(X).T @ np.abs(X)
    err = np.abs(g - Gm)
    assert np.all(err <= 2.0 ** -7 * np.abs(Gm) + 4e-6 * mag + 1e-30)                 # within one ulp everywhere ...
    assert np.mean(err > 2.0 ** -8 * np.abs(Gm) + 4e-6 * mag + 1e-30) <= 2e-3           # ... and half an ulp but for flips
    # diagonal: bf16 part + float32 remainder restore the float32 sum
    assert np.all(np.abs(np.diag(g) + host(gram_lo).astype(np.float64) - np.diag(Gm)) <= 4e-6 * np.diag(mag) + 1e-30)


def _one_step_gram(c, beta, V0, t=1, m0=None, u0=None):
    Wd, sg, scales, q, ic, hk, gram, gram_lo = _gram_setup(c)
    alpha = 1.0 / (c.T * c.O)
    V = dev(V0.copy())
    m = dev(np.zeros_like(V0) if m0 is None else m0.copy())
    u = dev(np.zeros_like(V0) if u0 is None else u0.copy())
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = binding.layer_step_gram_workspace(c.O, c.K)
    binding.faar_layer_step_gram(Wd, sg, scales, V, m, u, ic, hk["H"], hk["c_norm2"], gram, gram_lo, beta, HYP["lambda_round"],
                                 alpha, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], t, losses, ws)
    torch.cuda.synchronize()
    out = host(V), host(m), host(u), host(losses)
    del Wd, V, m, u, ws, gram, hk
    torch.cuda.empty_cache()
    ref = {}
    for mode in (False, True):
        ref[mode] = fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0) if m0 is None else m0,
                                  np.zeros_like(V0) if u0 is None else u0, c.Xq, c.Y_fp, beta, HYP["lambda_round"], alpha,
                                  HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], t,
                                  declared_rounding=("gram" if mode else False))
        for k in ("R", "dY", "Wq"):
            ref[mode].pop(k, None)
    return out + (ref,)


def _assert_gram_case(name, beta):
    c = tp.build_case(name)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    V, m, u, losses, ref = _one_step_gram(c, beta, V0)
    ex, de = ref[False], ref[True]
    errs = {"loss_exact": abs(losses[0] - ex["L_mse"]) / ex["L_mse"], "loss_declared": abs(losses[0] - de["L_mse"]) / de["L_mse"],
            "round": abs(losses[1] - ex["L_round"]) / ex["L_round"], "total": abs(losses[2] - ex["L"]) / ex["L"]}
    g = m.astype(np.float64) / (1 - HYP["beta1"])
    errs["grad"] = tp.grad_errors(g, ref)
    assert errs["loss_exact"] <= tp.loss_tol(name), errs
    assert errs["loss_declared"] <= TOL_LOSS_DECLARED, errs
    assert errs["round"] <= 1e-5, errs
    assert errs["total"] <= tp.loss_tol(name), errs
    tp._check_grad(g, ref, tp.GRAD_ELEM_MAX_BY_CASE.get(name, tp.GRAD_ELEM_MAX), BY_NAME[name].full_size)
    tp._check_update(V, m, u, V0, np.zeros_like(V0), np.zeros_like(V0), 1)
    return errs


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("beta", [4.0, 20.0])
def test_gram_step_first_step(name, beta):
    _assert_gram_case(name, beta)


@pytest.mark.parametrize("name", FULL)
def test_gram_step_full_size(name):
    _assert_gram_case(name, 8.0)


def test_gram_step_with_state_and_random_v():
    """A later step: non-zero Adam state, V anywhere in [0, 1]; the update rule against the oracle's, fed the gradient
    the GPU itself used."""
    c = tp.build_case("three_tiles")
    rng = np.random.default_rng(23)
    V0 = rng.uniform(0, 1, (c.O, c.K)).astype(np.float32)
    m0 = (rng.standard_normal((c.O, c.K)) * 1e-6).astype(np.float32)
    u0 = (rng.uniform(0, 1, (c.O, c.K)) * 1e-12).astype(np.float32)
    V, m, u, losses, ref = _one_step_gram(c, 12.0, V0, t=7, m0=m0, u0=u0)
    assert losses[0] == pytest.approx(ref[True]["L_mse"], rel=TOL_LOSS_DECLARED)
    assert losses[1] == pytest.approx(ref[False]["L_round"], rel=1e-5)
    g = (m.astype(np.float64) - HYP["beta1"] * m0.astype(np.float64)) / (1 - HYP["beta1"])
    # recovered through a difference of float32 numbers: the per-element bound loosens by the rounding of m itself
    n = np.linalg.norm
    assert n(g - ref[True]["dV"]) <= 2e-3 * n(ref[True]["dV"])
    tp._check_update(V, m, u, V0, m0, u0, 7)


def test_gram_and_token_forms_follow_the_same_trajectory():
    """40 steps of the small fp32 configuration in both forms from the same start: the losses stay together to the size
    of the roundings that differ, and both end at the same hardened decisions but for weights whose V sits next to 1/2."""
    c = synth.config1(0)
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic), hk = tp._setup(c, h=True)
    gram, gram_lo = binding.faar_gram_prepare(Xt, c.T)
    alpha = 1.0 / (c.T * c.O)
    runs = {}
    for form in ("token", "gram"):
        V, _ = faar.faar_init_v(Wd, sg, scales)
        m, u = torch.zeros_like(V), torch.zeros_like(V)
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        ws = faar.layer_step_workspace(c.O, c.K, c.T) if form == "token" else binding.layer_step_gram_workspace(c.O, c.K)
        hist = []
        for i in range(40):
            beta = 4.0 + 0.5 * i
            if form == "token":
                faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, C, ic, beta, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, i + 1,
                                     losses, ws, **hk)
            else:
                binding.faar_layer_step_gram(Wd, sg, scales, V, m, u, ic, hk["H"], hk["c_norm2"], gram, gram_lo, beta, 0.01,
                                             alpha, 5e-3, 0.9, 0.999, 1e-8, i + 1, losses, ws)
            hist.append(host(losses))
        runs[form] = (host(V), np.array(hist))
    (Vt, Lt), (Vg, Lg) = runs["token"], runs["gram"]
    assert np.all(np.abs(Lt - Lg) <= 5e-3 * np.abs(Lt))
    assert Lt[-1, 0] < Lt[0, 0] and Lg[-1, 0] < Lg[0, 0]
    differ = (Vt >= 0.5) != (Vg >= 0.5)
    assert differ.mean() <= 2e-3
    assert np.all(np.abs(Vt[differ] - 0.5) <= 0.05) and np.all(np.abs(Vg[differ] - 0.5) <= 0.05)


def test_gram_forward_left_by_the_previous_step_is_identical_and_checked():
    """beta_next / forward_ready in the Gram form: bit-identical to the plain sequence; a stale workspace gives NaN losses
    and leaves the state untouched."""
    for c in (synth.config1(0), tp.build_case("three_tiles")):
        Wd, sg, scales, q, ic, hk, gram, gram_lo = _gram_setup(c)
        alpha = 1.0 / (c.T * c.O)
        ws = binding.layer_step_gram_workspace(c.O, c.K)
        betas = [4.0, 7.5, 9.0, 9.0, 16.0]

        def run(fused):
            V, _ = faar.faar_init_v(Wd, sg, scales)
            state = [V, torch.zeros_like(V), torch.zeros_like(V)]
            losses = torch.zeros(3, dtype=torch.float32, device="cuda")
            ws.zero_()
            out = []
            for i, beta in enumerate(betas):
                nxt = betas[i + 1] if fused and i + 1 < len(betas) else 0.0
                binding.faar_layer_step_gram(Wd, sg, scales, *state, ic, hk["H"], hk["c_norm2"], gram, gram_lo, beta, 0.01, alpha,
                                             5e-3, 0.9, 0.999, 1e-8, 2 + i, losses, ws, beta_next=nxt,
                                             forward_ready=fused and i > 0)
                out.append(losses.clone())
            return state, out

        a, oa = run(False)
        b, ob = run(True)
        for x, y in zip(a, b):
            assert torch.equal(x, y), c.name
        for la, lb in zip(oa, ob):
            assert torch.equal(la, lb), c.name
        # a workspace nobody prepared
        V, _ = faar.faar_init_v(Wd, sg, scales)
        state = [V, torch.zeros_like(V), torch.zeros_like(V)]
        snap = [x.clone() for x in state]
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        ws.fill_(0xA5)
        binding.faar_layer_step_gram(Wd, sg, scales, *state, ic, hk["H"], hk["c_norm2"], gram, gram_lo, 6.0, 0.01, alpha, 5e-3,
                                     0.9, 0.999, 1e-8, 2, losses, ws, forward_ready=True)
        torch.cuda.synchronize()
        assert bool(torch.isnan(losses).all()) and all(torch.equal(x, y) for x, y in zip(state, snap))


def test_gram_step_with_nvfp4_activations_in_units():
    """Activations passed as node * block scale with their tensor scale apart: the Gram matrix is built from the units
    and the step applies x_scale^2 (quadratic term) and x_scale (constant term)."""
    c = tp.build_case("three_tiles")
    X = synth.activations(c.T, c.K, 32)
    qx = fo.quant_rtn(X, True)
    sX, sc, cd, Xu = faar.faar_quant_rtn(dev(X, True), want_dq=True, dq_in_units=True)
    nib = fo.unpack_nibbles(qx["codes"])
    units = np.where(nib & 8, -1.0, 1.0) * fo.e2m1_decode(nib & 7) * np.repeat(fo.e4m3_decode(qx["scales"]), 16, axis=1)
    Xq = (units.astype(np.float32) * np.float32(qx["s_global"])).astype(np.float32)
    Wd = dev(c.W, c.w_is_bf16)
    sg, scales, _, _ = faar.faar_quant_rtn(Wd)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    Xt, C, ic, H, cn = faar.faar_layer_prepare(Wd, sg, scales, Xu, dev(c.Y_fp, True), x_scale=sX, gradient_constant=True)
    gram, gram_lo = binding.faar_gram_prepare(Xt, c.T)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    alpha = 1.0 / (c.T * c.O)
    V, m, u = dev(V0.copy()), dev(np.zeros_like(V0)), dev(np.zeros_like(V0))
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = binding.layer_step_gram_workspace(c.O, c.K)
    binding.faar_layer_step_gram(Wd, sg, scales, V, m, u, ic, H, cn, gram, gram_lo, 8.0, HYP["lambda_round"], alpha, HYP["lr"],
                                 HYP["beta1"], HYP["beta2"], HYP["eps"], 1, losses, ws, x_scale=sX)
    ref = {mode: fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0), np.zeros_like(V0), Xq, c.Y_fp, 8.0,
                               HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], 1,
                               declared_rounding=("gram" if mode else False)) for mode in (False, True)}
    L = host(losses)
    assert L[0] == pytest.approx(ref[False]["L_mse"], rel=tp.TOL_LOSS_EXACT_OUTLIER)
    # the Gram matrix of the units is rounded, not that of x_scale * units: the same relative rounding, other boundaries
    assert L[0] == pytest.approx(ref[True]["L_mse"], rel=2e-4)
    g = host(m).astype(np.float64) / (1 - HYP["beta1"])
    n = np.linalg.norm
    assert n(g - ref[False]["dV"]) <= tp.TOL_GRAD_EXACT * n(ref[False]["dV"])
