"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs.
Integer / byte / index results bit-exact; float results within the tolerances stated in the block above HYP below
(bf16 matrix-core path vs float64 oracle)."""
import functools

import numpy as np
import pytest
import torch

from oracle import faar_oracle as fo
from workloads import synth

from parity_cases import BY_NAME, STEP_CASES

pytestmark = pytest.mark.gpu

import paper_2603_22370_amd as faar  # noqa: E402


def dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def weight_cases():
    yield "config1_fp32", synth.config1(0).W, False
    yield "student_t_bf16_ragged", synth.student_t_weight(96, 320, 3), True      # 15 blocks of 256 threads, ragged
    yield "student_t_bf16_1tile", synth.student_t_weight(1, 16, 4), True         # a single scale block
    yield "adversarial_bf16", synth.adversarial_weight(1, True), True
    yield "adversarial_fp32", synth.adversarial_weight(2, False), False
    yield "qproj_slice_bf16", synth.student_t_weight(512, 2048, 5), True


WCASES = list(weight_cases())
WIDS = [c[0] for c in WCASES]


def extreme_weight_cases():
    """Magnitudes far outside anything a network holds: the kernels switch division routines on the size of the
    block scale and of the weights, and every route must give the decisions of the IEEE quotient."""
    base = synth.student_t_weight(8, 64, 6)
    yield "tiny_bf16", (base * np.float32(2.0 ** -80)).astype(np.float32), True          # scales below 2^-60
    yield "huge_fp32", (synth.config1(1).W[:8, :64] * np.float32(2.0 ** 90)).astype(np.float32), False
    rows = (2.0 ** (-12.0 * np.arange(8))).astype(np.float32)[:, None]                   # block scales that underflow
    yield "mixed_range_bf16", (base * rows).astype(np.float32), True
    w = base.copy()
    w[3, 5] = np.float32(2.0 ** 70)                                                      # one weight above 2^60
    yield "one_giant_bf16", w, True


XCASES = list(extreme_weight_cases())


@pytest.mark.parametrize("name,W,isbf", WCASES, ids=WIDS)
def test_quant_rtn_bit_exact(name, W, isbf):
    q = fo.quant_rtn(W, isbf)
    sg, scales, codes, Wdq = faar.faar_quant_rtn(dev(W, isbf), want_dq=True)
    assert host(sg)[0].view(np.uint32) == np.float32(q["s_global"]).view(np.uint32)
    assert np.array_equal(host(scales), q["scales"])
    assert np.array_equal(host(codes), q["codes"])
    assert np.array_equal(host(Wdq).view(np.uint32), q["W_dq"].view(np.uint32))
    # with a caller-supplied tensor scale
    sg2 = dev(np.array([q["s_global"] * np.float32(1.5)], dtype=np.float32))
    q2 = fo.quant_rtn(W, isbf, s_global=host(sg2)[0])
    _, scales2, codes2, _ = faar.faar_quant_rtn(dev(W, isbf), s_global=sg2)
    assert np.array_equal(host(scales2), q2["scales"]) and np.array_equal(host(codes2), q2["codes"])


@pytest.mark.parametrize("name,W,isbf", WCASES, ids=WIDS)
def test_init_v_and_harden_pack_bit_exact(name, W, isbf):
    q = fo.quant_rtn(W, isbf)
    Wd = dev(W, isbf)
    sg, scales, codes, _ = faar.faar_quant_rtn(Wd)
    iv = fo.init_v(W, q["s_global"], q["scales"])
    V, fc = faar.faar_init_v(Wd, sg, scales, want_floor_codes=True)
    assert np.array_equal(host(V).view(np.uint32), iv["V"].view(np.uint32))
    assert np.array_equal(host(fc), iv["floor_codes"])
    # hardening V_init reproduces RTN (Eq. 4 + Eq. 7), on the GPU path itself
    c2, _, _, flips = faar.faar_harden_pack(Wd, sg, scales, V, want_flips=True)
    assert torch.equal(c2, codes) and int(flips.item()) == 0
    # arbitrary V with planted 0, 0.5, 1, 0.5 -/+ 1 ulp, a denormal
    Vs = synth.rounding_variables(W.shape[0], W.shape[1], 7)
    hp = fo.harden_pack(W, isbf, q["s_global"], q["scales"], Vs)
    c3, dec, Wf, flips = faar.faar_harden_pack(Wd, sg, scales, dev(Vs), want_decisions=True, want_final=True,
                                               want_flips=True)
    assert np.array_equal(host(c3), hp["codes"])
    assert np.array_equal(host(dec), hp["decisions"])
    assert np.array_equal(host(Wf).view(np.uint32), hp["W_final"].view(np.uint32))
    assert int(flips.item()) == hp["flip_count"]
    # lower-only and upper-only rounding
    for const in (0.0, 1.0):
        Vc = np.full(W.shape, const, dtype=np.float32)
        c4, _, _, _ = faar.faar_harden_pack(Wd, sg, scales, dev(Vc))
        assert np.array_equal(host(c4), fo.harden_pack(W, isbf, q["s_global"], q["scales"], Vc)["codes"])


@pytest.mark.parametrize("name,W,isbf", XCASES, ids=[c[0] for c in XCASES])
def test_codec_bit_exact_on_extreme_magnitudes(name, W, isbf):
    test_quant_rtn_bit_exact(name, W, isbf)
    test_init_v_and_harden_pack_bit_exact(name, W, isbf)
    q = fo.quant_rtn(W, isbf)
    Wd = dev(W, isbf)
    sg, scales, _, _ = faar.faar_quant_rtn(Wd)
    X = np.ones((4, W.shape[1]), dtype=np.float32)
    _, _, ic = faar.faar_layer_prepare(Wd, sg, scales, dev(X, True), dev(np.zeros((4, W.shape[0]), dtype=np.float32)))
    wt = fo.normalised_magnitude(W, q["scales"], q["s_global"])
    want_ic = (np.signbit(W).astype(np.uint8) << 3) | np.where(W == 0, 7, fo.find_interval(wt)).astype(np.uint8)
    assert np.array_equal(host(ic), fo.pack_nibbles(want_ic))


@pytest.mark.parametrize("name,W,isbf", WCASES, ids=WIDS)
@pytest.mark.parametrize("beta", [4.0, 32.0])
def test_softquant_forward_and_backward(name, W, isbf, beta):
    q = fo.quant_rtn(W, isbf)
    Wd = dev(W, isbf)
    sg, scales, _, _ = faar.faar_quant_rtn(Wd)
    V = synth.rounding_variables(W.shape[0], W.shape[1], 8)
    Wq = fo.soft_weight(W, q["s_global"], q["scales"], V, beta)
    rng = np.random.default_rng(9)
    dWt = (rng.standard_normal(W.shape) * 1e-3).astype(np.float32)
    lam = 0.05
    for delta in (False, True):
        Wt, dV, rl = faar.faar_softquant_fwd_bwd(Wd, sg, scales, dev(V), beta, dWt=dev(dWt), lambda_round=lam,
                                                 emit_delta=delta)
        want = Wq - W.astype(np.float64) if delta else Wq
        # one bf16 rounding (2^-9 relative) plus float32 evaluation noise on the un-rounded value
        tol = 2.0 ** -8 * np.abs(want) + 4e-7 * np.abs(Wq) + 1e-30
        assert np.all(np.abs(host(Wt).astype(np.float64) - want) <= tol)
    sign, lo, hi, s = fo.interval_terms(W, q["s_global"], q["scales"])
    h = fo.h_beta(V, beta)
    dV_want = dWt.astype(np.float64) * sign * s * (hi - lo) * beta * h * (1 - h) + lam / W.size * (4 - 8 * V.astype(np.float64))
    err = np.abs(host(dV).astype(np.float64) - dV_want)
    assert np.all(err <= 2e-5 * np.abs(dV_want) + 1e-6 * np.abs(dV_want).max())
    assert host(rl)[0] == pytest.approx(fo.round_loss(V), rel=1e-6)


@functools.lru_cache(maxsize=2)
def build_case(name):
    """The seeded tensors of one parity case (see tests/parity_cases.py); the two most recent are kept."""
    p = BY_NAME[name]
    if p.fp32_small:
        return synth.config1(p.seed)
    return synth.llm_linear(p.name, p.O, p.K, p.T, p.seed, gated_input=p.gated_input, quantised_acts=p.quantised_acts)


SMALL = [c.name for c in STEP_CASES if not c.full_size]
FULL = [c.name for c in STEP_CASES if c.full_size]
# the cases other tests below reuse
RAGGED, THREE_TILES = "ragged", "three_tiles"


def _setup(c, h=False):
    """Device inputs of a case.  The last element holds the keyword arguments that make faar_layer_step use the
    split form of the gradient (H = C^T X_q, ||C||^2) -- empty unless h."""
    Wd = dev(c.W, c.w_is_bf16)
    sg, scales, _, _ = faar.faar_quant_rtn(Wd)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    Xq = dev(c.Xq, True)
    Y = dev(c.Y_fp, True)
    out = faar.faar_layer_prepare(Wd, sg, scales, Xq, Y, gradient_constant=h)
    hk = dict(H=out[3], c_norm2=out[4]) if h else {}
    return Wd, sg, scales, q, Xq, Y, out[0], (out[1], out[2]), hk


@pytest.mark.parametrize("name", SMALL + FULL)
def test_layer_prepare(name):
    c = build_case(name)
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic), _ = _setup(c)
    Tp = faar.faar_padded_tokens(c.T)
    xt = host(Xt)
    assert xt.shape == (c.K, Tp)
    assert np.array_equal(xt[:, :c.T], c.Xq.T) and not xt[:, c.T:].any()
    C_want = c.Y_fp.astype(np.float64) - c.Xq.astype(np.float64) @ c.W.astype(np.float64).T
    scale = np.abs(c.Xq.astype(np.float64)) @ np.abs(c.W.astype(np.float64)).T      # size of the summed terms
    Cg = host(C)                                        # [ceil(T/4), O, 4]: rows interleaved in groups of four
    assert Cg.shape == ((c.T + 3) // 4, c.O, 4)
    Cg = Cg.transpose(0, 2, 1).reshape(-1, c.O)
    assert not Cg[c.T:].any()
    assert np.all(np.abs(Cg[:c.T] - C_want) <= 2e-6 * scale + 1e-30)
    del Cg, C_want, scale
    # cached interval codes: sign bit and k_lo (7 for a zero weight)
    wt = fo.normalised_magnitude(c.W, q["scales"], q["s_global"])
    want_ic = (np.signbit(c.W).astype(np.uint8) << 3) | np.where(c.W == 0, 7, fo.find_interval(wt)).astype(np.uint8)
    assert np.array_equal(host(ic), fo.pack_nibbles(want_ic))
    # also with a float32 reference output
    Xt2, C2, ic2 = faar.faar_layer_prepare(Wd, sg, scales, Xq, dev(c.Y_fp))
    assert torch.equal(C2, C) and torch.equal(Xt2, Xt) and torch.equal(ic2, ic)
    del Xt2, C2, ic2
    # the gradient constant H = C^T X_q and ||C||^2, against float64 products of the C the library itself wrote
    # (three bf16 terms of C times X_q are exact products: only float32 accumulation noise remains)
    Xt3, C3, ic3, H, cn = faar.faar_layer_prepare(Wd, sg, scales, Xq, Y, gradient_constant=True)
    assert torch.equal(C3, C) and torch.equal(Xt3, Xt) and torch.equal(ic3, ic)
    Cg = host(C).transpose(0, 2, 1).reshape(-1, c.O)[:c.T].astype(np.float64)
    X64 = c.Xq.astype(np.float64)
    H_want = Cg.T @ X64
    assert np.all(np.abs(host(H) - H_want) <= 2e-6 * (np.abs(Cg).T @ np.abs(X64)) + 1e-30)
    assert float(cn.item()) == pytest.approx(float((Cg * Cg).sum()), rel=2e-6)


# ---- tolerances of the float results -------------------------------------------------------------------------
# Two bf16 roundings (unit roundoff u = 2^-9) sit between the inputs and the loss / gradient: the weight
# perturbation W_q - W and dY (a third, dX, on the input-gradient path).
#  * Against the oracle evaluated WITH those declared roundings only float32 accumulation noise and rounding-boundary
#    flips remain (a value that sits on a bf16 rounding boundary may round the other way in float32 than in float64).
#    Measured over all cases below: loss <= 6.2e-6, ||dV|| <= 3.4e-4, ||dX|| <= 4.8e-5.
#  * Against the EXACT float64 oracle the loss moves by 2 sum(d * err(d)) / sum(d^2) over the weights d = W_q - W that
#    carry it: at most 2u, and far less once many weights share the loss.  The full-size LLM-shaped layers measure
#    5.9e-5 ... 4.4e-4 and are held to 1e-3.  Small slices with outlier channels are dominated by a few dozen
#    heavy-tailed weights in the outlier columns (measured up to 2.05e-3 = 1.05u on 512x2048 with 640 tokens at
#    beta = 4) and are held to the bound 2u.
#  * The gradient against the exact oracle carries two independent roundings of rms u / sqrt(3) each (W_q - W, dY):
#    sqrt(2/3) u = 1.6e-3 expected, 1.2e-3 ... 2.6e-3 measured (the largest on the 256x256 configuration in the H form);
#    full-size layers 1.5e-3 ... 2.0e-3, held to 1.5u, the small cases to 2u.  With an upstream gradient given, dY is
#    not rounded and G does not depend on W_q: measured 5e-7.
#  * dX (bf16) against the exact oracle is the final rounding, u / sqrt(3) * ~2: measured 2.3e-3 ... 2.4e-3.
U = 2.0 ** -9
TOL_LOSS_EXACT_FULL = 1e-3       # full-size LLM-shaped layers
TOL_LOSS_EXACT_OUTLIER = 2 * U   # few-term or outlier-dominated sums: the worst-case bound
TOL_LOSS_DECLARED = 2e-5
TOL_GRAD_EXACT = 2 * U           # worst case of two roundings; full-size layers are held to 1.5u
TOL_GRAD_DECLARED = 5e-4
# per element, vs the oracle with the declared roundings: excess = (|g - g*| - GRAD_ELEM_A |g*|) / rms(g*).  A boundary
# flip of one W_q - W moves that weight's own gradient by up to 2^-8 of its own term 2 alpha ||X_k||^2 d, which is
# the size of g* itself unless the cross terms cancel it; a flip of one dY moves a whole row of G a little.
# Measured distribution over all cases (16.8 M elements in the largest): the fraction of elements with excess >
# 1e-3 is <= 8e-5 and with excess > 3e-3 is <= 2.7e-5; the largest excess is <= 1.4e-3 on the small cases, 1.2e-2 on
# the 16.8 M-weight gate projection (one element in ten million) -- and 5.8e-2 on the one case with 33 tokens, where
# the own terms of the outlier columns are ten times rms(g*) and largely cancelled by the other outlier columns
# (33 tokens cannot decorrelate 123 columns).  Held to: fraction above 1e-3 <= 2e-4; largest <= 2e-2 (9e-2 there).
GRAD_ELEM_A, GRAD_ELEM_FRAC_AT, GRAD_ELEM_FRAC, GRAD_ELEM_MAX = 2.0 ** -7, 1e-3, 2e-4, 2e-2
GRAD_ELEM_MAX_BY_CASE = {"dw_one_slice": 9e-2}
# dX per element: one ulp of the final bf16 rounding (a boundary flip).  With the upstream gradient given, measured
# excess <= 1.4e-6 rms and norm-wise <= 4.8e-5 against the declared oracle; with the locally derived dY its own
# boundary flips come on top (single terms of the sum over O): 1.9e-3 rms and 2.7e-4 measured.
DX_ELEM_A = 2.0 ** -7
DX_ELEM_B = {"upstream": 1e-4, "local": 5e-3}
TOL_DX_EXACT = 1.5 * U
TOL_DX_DECLARED = {"upstream": 2e-4, "local": 6e-4}

HYP = dict(lambda_round=0.01, lr=5e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def loss_tol(name):
    return TOL_LOSS_EXACT_FULL if BY_NAME[name].full_size else TOL_LOSS_EXACT_OUTLIER


def upstream_gradient(c, seed):
    """Synthetic upstream gradient of a chained step: bf16 N(0, 1) * 1e-3."""
    rng = np.random.default_rng([seed, 41])
    return synth.round_to_bf16((rng.standard_normal((c.T, c.O)) * 1e-3).astype(np.float32))


def _one_step(c, beta, V0, t=1, m0=None, u0=None, dY_ext=None, want_dX=False, split=False, whole_device=False):
    """split: the step is given the gradient constant H; its oracle of record is then the "split" contract."""
    Wd, sg, scales, q, Xq, Y, Xt, C, hk = _setup(c, h=split)
    alpha = 1.0 / (c.T * c.O)
    V = dev(V0.copy())
    m = dev(np.zeros_like(V0) if m0 is None else m0.copy())
    u = dev(np.zeros_like(V0) if u0 is None else u0.copy())
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    chained = dY_ext is not None or want_dX
    ws = faar.layer_step_workspace(c.O, c.K, c.T, chained=chained)
    dX = torch.empty((c.T, c.K), dtype=torch.bfloat16, device="cuda") if want_dX else None
    faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, *C, beta, HYP["lambda_round"], alpha, HYP["lr"],
                         HYP["beta1"], HYP["beta2"], HYP["eps"], t, losses, ws,
                         dY_ext=None if dY_ext is None else dev(dY_ext, True), dX=dX, whole_device=whole_device, **hk)
    torch.cuda.synchronize()
    out = host(V), host(m), host(u), host(losses), (None if dX is None else host(dX))
    del Wd, Xq, Y, Xt, C, V, m, u, ws, dX, hk
    torch.cuda.empty_cache()
    ref = {}
    for mode in (False, True):
        ref[mode] = fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0) if m0 is None else m0,
                                  np.zeros_like(V0) if u0 is None else u0, c.Xq, c.Y_fp, beta, HYP["lambda_round"],
                                  alpha, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], t, want_dX=want_dX,
                                  dY_ext=dY_ext, declared_rounding=("split" if split and mode else mode))
        for k in ("R", "dY", "Wq"):        # not compared; large
            ref[mode].pop(k, None)
    return out + (ref,)


def grad_errors(g, ref):
    """Error figures of a gradient against the two oracles (see the tolerance block above)."""
    exact, decl = ref[False]["dV"], ref[True]["dV"]
    n = np.linalg.norm
    rms = np.sqrt(np.mean(decl ** 2))
    excess = (np.abs(g - decl) - GRAD_ELEM_A * np.abs(decl)) / rms
    return {"norm_exact": n(g - exact) / n(exact), "norm_declared": n(g - decl) / n(decl),
            "elem_excess_over_rms": float(excess.max()),
            "frac_above": {thr: float(np.mean(excess > thr)) for thr in (3e-4, 1e-3, 3e-3)}}


def dx_errors(dX, ref):
    exact, decl = ref[False]["dX"], ref[True]["dX"]
    n = np.linalg.norm
    rms = np.sqrt(np.mean(decl ** 2))
    excess = np.abs(dX - decl) - DX_ELEM_A * np.abs(decl)  # in absolute units; divided by rms below
    return {"norm_exact": n(dX - exact) / n(exact), "norm_declared": n(dX - decl) / n(decl),
            "elem_excess_over_rms": float(excess.max() / rms)}


def _check_grad(g, ref, elem_max=GRAD_ELEM_MAX, full_size=False):
    e = grad_errors(g, ref)
    assert e["norm_exact"] <= (1.5 * U if full_size else TOL_GRAD_EXACT), e   # vs float64 oracle, no rounding anywhere
    assert e["norm_declared"] <= TOL_GRAD_DECLARED, e    # vs oracle with the declared bf16 roundings
    assert e["elem_excess_over_rms"] <= elem_max, e      # element by element: the largest ...
    assert e["frac_above"][GRAD_ELEM_FRAC_AT] <= GRAD_ELEM_FRAC, e   # ... and how many come anywhere near it


def _check_dx(dX, ref, dy="upstream"):
    """dX = dY W_q element by element against the oracle with the declared roundings (dY, W_q and dX itself in
    bf16), and norm-wise against the exact one (three roundings on this path).  dy: where dY came from."""
    e = dx_errors(dX, ref)
    assert e["norm_exact"] <= TOL_DX_EXACT, e
    assert e["norm_declared"] <= TOL_DX_DECLARED[dy], e
    assert e["elem_excess_over_rms"] <= DX_ELEM_B[dy], e


def _check_update(V, m, u, V0, m0, u0, t):
    """Adam is a sign-like update (first step: lr g / (|g| + eps)), so a sign flip of a near-zero
    gradient moves V by 2 lr: the update arithmetic is therefore checked against the oracle's
    update rule fed the gradient the GPU itself used (recovered exactly from its first moment)."""
    b1 = HYP["beta1"]
    g = (m.astype(np.float64) - b1 * m0.astype(np.float64)) / (1 - b1)
    Vn, mn, un = fo.adam_update(V0, m0, u0, g, HYP["lr"], b1, HYP["beta2"], HYP["eps"], t)
    assert np.allclose(u, un, rtol=2e-5, atol=1e-30)
    # float32 rounding of m, u and of the quotient: a few ulp of the step, plus the ulp of V itself
    assert np.all(np.abs(V - Vn) <= 1e-4 * HYP["lr"] + 1.2e-7)
    assert V.min() >= 0.0 and V.max() <= 1.0


def step_case_errors(name, beta, chained, split=False):
    """One first step of a parity case through the C ABI against both oracles -- chained: with an upstream gradient
    and dX; otherwise with the locally derived dY.  Asserts what is exact and returns the error figures of everything
    that has a tolerance."""
    p = BY_NAME[name]
    c = build_case(name)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    dY_ext = upstream_gradient(c, p.seed) if chained else None
    V, m, u, losses, dX, ref = _one_step(c, beta, V0, dY_ext=dY_ext, want_dX=chained, split=split, whole_device=p.whole_device)
    ex, de = ref[False], ref[True]
    errs = {"loss_exact": abs(losses[0] - ex["L_mse"]) / ex["L_mse"], "loss_declared": abs(losses[0] - de["L_mse"]) / de["L_mse"],
            "round": abs(losses[1] - ex["L_round"]) / ex["L_round"],
            "total": abs(losses[2] - ex["L"]) / ex["L"]}
    # with zero initial state, m = (1 - beta1) g: the gradient is observable through m
    errs["grad"] = grad_errors(m.astype(np.float64) / (1 - HYP["beta1"]), ref)
    if chained:
        errs["dx"] = dx_errors(dX, ref)
    _check_update(V, m, u, V0, np.zeros_like(V0), np.zeros_like(V0), 1)
    return errs, (m, dX, ref)


def _assert_step_case(name, beta):
    """Every case runs plainly (the residual GEMM's own dY^T feeds the dW GEMM) in both forms of the step -- with the
    constant C in the residual GEMM's epilogue, and with the gradient constant H instead; a chained case also runs with
    an upstream gradient and dX (three GEMMs), again in both forms (with H the residual GEMM then only sums the loss).
    So every output of every kernel variant a case reaches is compared."""
    modes = [(False, False), (False, True)] + ([(True, False), (True, True)] if BY_NAME[name].chained else [])
    for chained, split in modes:     # split: with the gradient constant H (no constant in the residual GEMM's epilogue)
        errs, (m, dX, ref) = step_case_errors(name, beta, chained, split)
        assert errs["loss_exact"] <= loss_tol(name), errs
        assert errs["loss_declared"] <= TOL_LOSS_DECLARED, errs
        assert errs["round"] <= 1e-5, errs
        assert errs["total"] <= loss_tol(name), errs
        _check_grad(m.astype(np.float64) / (1 - HYP["beta1"]), ref, GRAD_ELEM_MAX_BY_CASE.get(name, GRAD_ELEM_MAX),
                    BY_NAME[name].full_size)
        if dX is not None:
            _check_dx(dX, ref)
        del m, dX, ref


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("beta", [4.0, 20.0])
def test_layer_step_first_step(name, beta):
    _assert_step_case(name, beta)


@pytest.mark.parametrize("name", FULL)
def test_layer_step_full_size(name):
    """The benchmark's own shapes and launch configurations (all tiles, every contraction slice, the ring wrapping
    around): one whole step -- with an upstream gradient and dX where the case is chained -- element by element
    against the oracle.  The float64 products of the largest case take a few seconds on the host."""
    _assert_step_case(name, 8.0)


def test_layer_step_with_state_and_random_v():
    c = build_case(THREE_TILES)
    rng = np.random.default_rng(11)
    V0 = synth.rounding_variables(c.O, c.K, 12)
    m0 = (rng.standard_normal(V0.shape) * 1e-7).astype(np.float32)
    u0 = (rng.uniform(0, 1, V0.shape) * 1e-13).astype(np.float32)
    V, m, u, losses, _, ref = _one_step(c, 9.0, V0, t=7, m0=m0, u0=u0)
    decl = ref[True]
    g = (m.astype(np.float64) - HYP["beta1"] * m0) / (1 - HYP["beta1"])
    n = np.linalg.norm
    assert n(g - decl["dV"]) <= 1e-3 * n(decl["dV"])
    _check_update(V, m, u, V0, m0, u0, 7)
    assert losses[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_LOSS_EXACT_OUTLIER)
    assert losses[0] == pytest.approx(ref[True]["L_mse"], rel=2e-5)
    assert losses[1] == pytest.approx(ref[False]["L_round"], rel=1e-5)


def test_layer_step_chained_dY_ext_and_dX():
    c = build_case(THREE_TILES)
    rng = np.random.default_rng(13)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    dY = synth.round_to_bf16((rng.standard_normal((c.T, c.O)) * 1e-3).astype(np.float32))
    for ext in (dY, None):
        V, m, u, losses, dX, ref = _one_step(c, 6.0, V0, dY_ext=ext, want_dX=True)
        _check_grad(m.astype(np.float64) / (1 - HYP["beta1"]), ref)
        _check_dx(dX, ref, "upstream" if ext is not None else "local")
        assert losses[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_LOSS_EXACT_OUTLIER)


@pytest.mark.parametrize("name", ["dw_token_major_192x256_split", "dw_token_major_256x192"])
def test_whole_device_tiles_change_no_bit(name):
    """FAAR_STEP_WHOLE_DEVICE only changes which tile of the token-major dW GEMM an output element falls into: every sum runs
    over the same terms in the same order, so the step's state and losses are identical with and without it."""
    p = BY_NAME[name]
    assert faar.faar_dw_token_major(p.O, p.K, p.T, True) in (2, 3) and faar.faar_dw_token_major(p.O, p.K, p.T, False) == 1
    c = build_case(name)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    dY_ext = upstream_gradient(c, p.seed) if p.chained else None
    a = _one_step(c, 8.0, V0, dY_ext=dY_ext, want_dX=p.chained, split=True, whole_device=False)
    b = _one_step(c, 8.0, V0, dY_ext=dY_ext, want_dX=p.chained, split=True, whole_device=True)
    for x, y in zip(a[:4], b[:4]):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("split", [False, True], ids=["c_form", "h_form"])
def test_config1_trajectory_100_adam_steps(split):
    """The small parity config end to end: 100 Adam steps with beta annealed 4 -> 32.  The oracle is
    re-synchronised to the GPU's (V, m, u) every 10 steps; every step's losses must agree, V stays
    in [0,1], and the packed result of the GPU's final V is bit-exact with the oracle's packing.
    In both forms of the step (the constant C in the residual GEMM's epilogue / the gradient constant H)."""
    c = synth.config1(0)
    Wd, sg, scales, q, Xq, Y, Xt, C, hk = _setup(c, h=split)
    alpha = 1.0 / (c.T * c.O)
    V, _ = faar.faar_init_v(Wd, sg, scales)
    m = torch.zeros_like(V)
    u = torch.zeros_like(V)
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = faar.layer_step_workspace(c.O, c.K, c.T)
    Vo, mo, uo = host(V).copy(), host(m).copy(), host(u).copy()
    lr, steps = 1e-2, 100
    first = last = None
    for t in range(1, steps + 1):
        beta = 4.0 + 28.0 * (t - 1) / (steps - 1)
        faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, *C, beta, 0.01, alpha, lr, 0.9, 0.999, 1e-8, t, losses, ws, **hk)
        r = fo.layer_step(c.W, q["s_global"], q["scales"], Vo, mo, uo, c.Xq, c.Y_fp, beta, 0.01, alpha, lr, 0.9,
                          0.999, 1e-8, t)
        Vo, mo, uo = r["V"], r["m"], r["u"]
        L = host(losses)
        assert L[0] == pytest.approx(r["L_mse"], rel=TOL_LOSS_EXACT_OUTLIER), t
        assert L[1] == pytest.approx(r["L_round"], rel=1e-3), t
        first = L[0] if first is None else first
        last = L[0]
        if t % 10 == 0:
            Vg = host(V)
            assert Vg.min() >= 0.0 and Vg.max() <= 1.0
            agree = np.mean((Vg >= 0.5) == (Vo >= 0.5))
            assert agree > 0.999, (t, agree)
            Vo, mo, uo = Vg.copy(), host(m).copy(), host(u).copy()
    assert last < first
    codes, _, _, flips = faar.faar_harden_pack(Wd, sg, scales, V, want_flips=True)
    hp = fo.harden_pack(c.W, False, q["s_global"], q["scales"], host(V))
    assert np.array_equal(host(codes), hp["codes"]) and int(flips.item()) == hp["flip_count"]
    assert hp["flip_count"] > 0
    # and the optimised rounding beats round-to-nearest on the hardened reconstruction loss
    L_rtn = fo.hardened_loss(c.W, False, q["s_global"], q["scales"], fo.init_v(c.W, q["s_global"], q["scales"])["V"],
                             c.Xq, c.Y_fp, alpha)
    assert fo.hardened_loss(c.W, False, q["s_global"], q["scales"], host(V), c.Xq, c.Y_fp, alpha) < L_rtn


@pytest.mark.parametrize("split", [False, True], ids=["c_form", "h_form"])
def test_resume_is_bit_exact_and_runs_are_deterministic(split):
    c = build_case(THREE_TILES)
    Wd, sg, scales, q, Xq, Y, Xt, C, hk = _setup(c, h=split)
    alpha = 1.0 / (c.T * c.O)
    ws = faar.layer_step_workspace(c.O, c.K, c.T)

    def run(n_steps, state=None, t0=0):
        if state is None:
            V, _ = faar.faar_init_v(Wd, sg, scales)
            state = [V, torch.zeros_like(V), torch.zeros_like(V)]
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        for t in range(t0 + 1, t0 + n_steps + 1):
            faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, 4.0 + t, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, t,
                                 losses, ws, **hk)
        return state, losses.clone()

    a, la = run(6)
    b, lb = run(6)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert torch.equal(la, lb)
    half, _ = run(3)
    half = [x.cpu().clone().cuda() for x in half]          # state copied out and back in
    cc, lc = run(3, state=half, t0=3)
    for x, y in zip(a, cc):
        assert torch.equal(x, y)
    assert torch.equal(la, lc)


def test_forward_left_by_the_previous_step_gives_identical_results():
    """A step may leave the next step's soft-quantised weights in the workspace (beta_next) and the next
    step may consume them (forward_ready): same arithmetic, so losses and state must match the plain
    sequence bit for bit -- float32 and bf16 weights, with and without dX, odd and even step indices."""
    rng = np.random.default_rng(17)
    for c, want_dX, split in ((synth.config1(0), False, False), (build_case(THREE_TILES), False, False),
                              (build_case(THREE_TILES), True, False), (build_case(RAGGED), True, False),
                              (synth.config1(0), False, True), (build_case(THREE_TILES), False, True)):
        Wd, sg, scales, q, Xq, Y, Xt, C, hk = _setup(c, h=split)
        alpha = 1.0 / (c.T * c.O)
        ws = faar.layer_step_workspace(c.O, c.K, c.T, chained=want_dX)
        betas = [4.0, 7.5, 9.0, 9.0, 16.0, 30.0]

        def run(fused, t0=2):
            V, _ = faar.faar_init_v(Wd, sg, scales)
            state = [V, torch.zeros_like(V), torch.zeros_like(V)]
            losses = torch.zeros(3, dtype=torch.float32, device="cuda")
            dX = torch.zeros((c.T, c.K), dtype=torch.bfloat16, device="cuda") if want_dX else None
            ws.zero_()
            out = []
            for i, beta in enumerate(betas):
                nxt = betas[i + 1] if fused and i + 1 < len(betas) else 0.0
                faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, beta, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8,
                                     t0 + i, losses, ws, dX=dX, beta_next=nxt, forward_ready=fused and i > 0, **hk)
                out.append((losses.clone(), None if dX is None else dX.clone()))
            return state, out

        a, oa = run(False)
        b, ob = run(True)
        for x, y in zip(a, b):
            assert torch.equal(x, y), c.name
        for (la, xa), (lb, xb) in zip(oa, ob):
            assert torch.equal(la, lb), c.name
            assert xa is None or torch.equal(xa, xb)
        # a prepared forward that is not consumed does no harm
        V, _ = faar.faar_init_v(Wd, sg, scales)
        state = [V, torch.zeros_like(V), torch.zeros_like(V)]
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        dX = torch.zeros((c.T, c.K), dtype=torch.bfloat16, device="cuda") if want_dX else None
        for i, beta in enumerate(betas):
            faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, beta, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8,
                                 2 + i, losses, ws, dX=dX, beta_next=float(rng.uniform(1, 40)), **hk)
        for x, y in zip(a, state):
            assert torch.equal(x, y), c.name
        assert torch.equal(losses, oa[-1][0])


def test_forward_ready_is_checked_on_the_device():
    """A step told that its forward pass is already in the workspace verifies that claim against the tag the
    producing step left (step index, beta, the layer's buffers, dX or not).  Every violation must give NaN losses and
    leave V and the Adam state untouched; a following step without the flag recovers."""
    c = build_case(THREE_TILES)
    Wd, sg, scales, q, Xq, Y, Xt, C, _ = _setup(c)
    alpha = 1.0 / (c.T * c.O)
    nan3 = lambda L: bool(torch.isnan(L).all())

    def fresh(chained=False):
        V, _ = faar.faar_init_v(Wd, sg, scales)
        return dict(V=V, m=torch.zeros_like(V), u=torch.zeros_like(V), losses=torch.zeros(3, dtype=torch.float32, device="cuda"),
                    ws=faar.layer_step_workspace(c.O, c.K, c.T, chained=chained))

    def step(s, t, beta, beta_next=0.0, ready=False, V=None, dX=None, ws=None):
        faar.faar_layer_step(Wd, sg, scales, s["V"] if V is None else V, s["m"], s["u"], Xq, Xt, *C, beta, 0.01, alpha, 5e-3,
                             0.9, 0.999, 1e-8, t, s["losses"], s["ws"] if ws is None else ws, dX=dX, beta_next=beta_next,
                             forward_ready=ready)
        torch.cuda.synchronize()

    def snapshot(s):
        return [s[k].clone() for k in ("V", "m", "u")]

    def unchanged(s, snap):
        return all(torch.equal(s[k], x) for k, x in zip(("V", "m", "u"), snap))

    # the valid sequence works, and each violation below starts from it
    def prepared():
        s = fresh()
        step(s, 1, 4.0, beta_next=6.0)
        assert not nan3(s["losses"])
        return s, snapshot(s)

    s, snap = prepared()
    step(s, 2, 6.0, ready=True)
    assert not nan3(s["losses"]) and not unchanged(s, snap)
    # a workspace nobody prepared (zeroed, and one full of stale bytes)
    for fill in (0, 0xA5):
        s = fresh()
        s["ws"].fill_(fill)
        snap = snapshot(s)
        step(s, 2, 6.0, ready=True)
        assert nan3(s["losses"]) and unchanged(s, snap)
        step(s, 2, 6.0)                                   # without the flag the step is fine again
        assert not nan3(s["losses"]) and not unchanged(s, snap)
    # another beta than the one the forward was computed at; a skipped step; a repeated step
    s, snap = prepared()
    step(s, 2, 7.0, ready=True)
    assert nan3(s["losses"]) and unchanged(s, snap)
    s, snap = prepared()
    step(s, 3, 6.0, ready=True)
    assert nan3(s["losses"]) and unchanged(s, snap)
    s, snap = prepared()
    step(s, 2, 6.0, beta_next=8.0, ready=True)
    snap = snapshot(s)
    step(s, 2, 6.0, ready=True)                           # step 2 again: its forward was consumed
    assert nan3(s["losses"]) and unchanged(s, snap)
    step(s, 3, 8.0, ready=True)                           # and the failed step left nothing behind
    assert nan3(s["losses"]) and unchanged(s, snap)
    # another V buffer (another layer's state on the same workspace)
    s, snap = prepared()
    V2 = s["V"].clone()
    step(s, 2, 6.0, ready=True, V=V2)
    assert nan3(s["losses"]) and unchanged(s, snap) and torch.equal(V2, snap[0])
    # a forward prepared without W_q cannot serve a step that wants dX
    s = fresh(chained=True)
    step(s, 1, 4.0, beta_next=6.0)
    snap = snapshot(s)
    step(s, 2, 6.0, ready=True, dX=torch.empty((c.T, c.K), dtype=torch.bfloat16, device="cuda"))
    assert nan3(s["losses"]) and unchanged(s, snap)
    # a call that reuses the workspace in between destroys the forward and clears the tag
    s, snap = prepared()
    faar.faar_hardened_loss(Wd, sg, scales, s["V"], Xq, C[0], alpha, s["ws"])
    step(s, 2, 6.0, ready=True)
    assert nan3(s["losses"]) and unchanged(s, snap)
    # a forward left by a step in the C form lacks the loss's cross term: a step in the H form cannot use it, nor the
    # other way round
    *_, hk = _setup(c, h=True)
    s, snap = prepared()
    faar.faar_layer_step(Wd, sg, scales, s["V"], s["m"], s["u"], Xq, Xt, *C, 6.0, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, 2,
                         s["losses"], s["ws"], forward_ready=True, **hk)
    torch.cuda.synchronize()
    assert nan3(s["losses"]) and unchanged(s, snap)
    s = fresh()
    faar.faar_layer_step(Wd, sg, scales, s["V"], s["m"], s["u"], Xq, Xt, *C, 4.0, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, 1,
                         s["losses"], s["ws"], beta_next=6.0, **hk)
    snap = snapshot(s)
    step(s, 2, 6.0, ready=True)
    assert nan3(s["losses"]) and unchanged(s, snap)


def test_token_major_steps_chain_and_guard_their_prepared_forward():
    """The same two properties on a shape whose step runs the token-major kernels (H form, own gradient: the residual GEMM leaves
    dY token-major and carries the tag check, the dW GEMM reads dY and X_q as they are; 3 token slices, so the 2-stage ring
    wraps): steps chained through beta_next / forward_ready give the plain sequence bit for bit, and a forward nobody
    prepared, or one prepared at another beta, gives NaN losses and leaves the state untouched."""
    O, K, T = 2560, 3328, 192
    assert faar.faar_dw_token_major(O, K, T) == 1
    c = synth.llm_linear("token_major_chain", O, K, T, 51)
    Wd, sg, scales, q, Xq, Y, Xt, C, hk = _setup(c, h=True)
    alpha = 1.0 / (T * O)
    ws = faar.layer_step_workspace(O, K, T)
    betas = [4.0, 7.5, 9.0, 16.0]

    def run(fused):
        V, _ = faar.faar_init_v(Wd, sg, scales)
        state = [V, torch.zeros_like(V), torch.zeros_like(V)]
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        ws.zero_()
        out = []
        for i, beta in enumerate(betas):
            nxt = betas[i + 1] if fused and i + 1 < len(betas) else 0.0
            faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, beta, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, 1 + i, losses, ws,
                                 beta_next=nxt, forward_ready=fused and i > 0, **hk)
            out.append(losses.clone())
        torch.cuda.synchronize()
        return state, out

    a, la = run(False)
    b, lb = run(True)
    for x, y in zip(a + la, b + lb):
        assert torch.equal(x, y)
    assert not torch.isnan(la[-1]).any()
    # the first step agrees with the oracle (the later ones are covered bit for bit by the above and by the per-step cases)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    r = fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0), np.zeros_like(V0), c.Xq, c.Y_fp, betas[0], 0.01,
                      alpha, 5e-3, 0.9, 0.999, 1e-8, 1)
    assert float(la[0][0]) == pytest.approx(r["L_mse"], rel=TOL_LOSS_EXACT_OUTLIER)
    assert float(la[0][1]) == pytest.approx(r["L_round"], rel=1e-5)
    # the guard
    V, _ = faar.faar_init_v(Wd, sg, scales)
    state = [V, torch.zeros_like(V), torch.zeros_like(V)]
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    for fill in (0, 0xA5):
        ws.fill_(fill)
        snap = [x.clone() for x in state]
        faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, 6.0, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, 2, losses, ws,
                             forward_ready=True, **hk)
        torch.cuda.synchronize()
        assert torch.isnan(losses).all() and all(torch.equal(x, y) for x, y in zip(state, snap))
    faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, 4.0, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, 1, losses, ws, beta_next=6.0, **hk)
    torch.cuda.synchronize()
    assert not torch.isnan(losses).any()
    snap = [x.clone() for x in state]
    faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, 7.0, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, 2, losses, ws,
                         forward_ready=True, **hk)                       # prepared at beta 6
    torch.cuda.synchronize()
    assert torch.isnan(losses).all() and all(torch.equal(x, y) for x, y in zip(state, snap))


def test_nvfp4_activations_in_units_of_their_tensor_scale():
    """Activations quantised to NVFP4 by the same kernel (blocks along K, their own tensor scale): W_dq in units of
    s_global is the exact product node * block scale, and a step fed (Xq, x_scale) agrees with the oracle fed the
    dequantised activations x_scale * Xq."""
    for c, seed in ((build_case(RAGGED), 31), (build_case(THREE_TILES), 32)):          # ragged 96x80 T=100 (generic GEMM), 320x256 T=300
        X = synth.activations(c.T, c.K, seed)
        qx = fo.quant_rtn(X, True)
        sX, sc, cd, Xu = faar.faar_quant_rtn(dev(X, True), want_dq=True, dq_in_units=True)
        assert np.array_equal(host(cd), qx["codes"]) and np.array_equal(host(sc), qx["scales"])
        nib = fo.unpack_nibbles(qx["codes"])
        units = np.where(nib & 8, -1.0, 1.0) * fo.e2m1_decode(nib & 7) * np.repeat(fo.e4m3_decode(qx["scales"]), 16, axis=1)
        assert np.array_equal(host(Xu).astype(np.float64), units)                    # exact in bf16
        Xq = (units.astype(np.float32) * np.float32(qx["s_global"])).astype(np.float32)   # what the step must see
        Wd = dev(c.W, c.w_is_bf16)
        sg, scales, _, _ = faar.faar_quant_rtn(Wd)
        q = fo.quant_rtn(c.W, c.w_is_bf16)
        Xt, C, ic, H, cn = faar.faar_layer_prepare(Wd, sg, scales, Xu, dev(c.Y_fp, True), x_scale=sX, gradient_constant=True)
        Cg = host(C).transpose(0, 2, 1).reshape(-1, c.O)[:c.T]
        C_want = c.Y_fp.astype(np.float64) - Xq.astype(np.float64) @ c.W.astype(np.float64).T
        scale = np.abs(Xq.astype(np.float64)) @ np.abs(c.W.astype(np.float64)).T
        assert np.all(np.abs(Cg - C_want) <= 4e-6 * scale + 1e-30)
        V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
        alpha = 1.0 / (c.T * c.O)
        for hk, contract in (({}, True), (dict(H=H, c_norm2=cn), "split")):    # both forms of the step
            V, m, u = dev(V0.copy()), dev(np.zeros_like(V0)), dev(np.zeros_like(V0))
            losses = torch.zeros(3, dtype=torch.float32, device="cuda")
            ws = faar.layer_step_workspace(c.O, c.K, c.T)
            faar.faar_layer_step(Wd, sg, scales, V, m, u, Xu, Xt, C, ic, 8.0, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"],
                                 HYP["beta2"], HYP["eps"], 1, losses, ws, x_scale=sX, **hk)
            ref = {bool(mode): fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0), np.zeros_like(V0), Xq,
                                             c.Y_fp, 8.0, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"], HYP["beta2"],
                                             HYP["eps"], 1, declared_rounding=mode) for mode in (False, contract)}
            L = host(losses)
            assert L[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_LOSS_EXACT_OUTLIER)
            assert L[0] == pytest.approx(ref[True]["L_mse"], rel=2e-5)
            _check_grad(host(m).astype(np.float64) / (1 - HYP["beta1"]), ref)


def test_batched_codec_calls_match_the_single_tensor_calls_and_the_oracle():
    """faar_quant_rtn_batch / faar_init_v_batch / faar_harden_pack_batch over 90 tensors of mixed sizes (two launches of
    72 and 18; single-block, ragged and multi-block tensors; both storage types): every output bit-identical to the
    single-tensor entry points, and, for a subset, to the oracle."""
    shapes = [(1, 16), (8, 64), (96, 320), (16, 2048), (512, 2048), (33, 48), (1024, 1024), (7, 4112)]
    for isbf in (True, False):
        Ws_h = []
        for k in range(90):
            O, K = shapes[k % len(shapes)]
            if k == 5:
                Ws_h.append(synth.adversarial_weight(1, isbf))
            else:
                w = synth.student_t_weight(O, K, 100 + k) if isbf else synth.gaussian_weight(O, K, 100 + k)
                Ws_h.append(w)
        Ws = [dev(w, isbf) for w in Ws_h]
        Vs_h = [synth.rounding_variables(w.shape[0], w.shape[1], 200 + k) for k, w in enumerate(Ws_h)]
        mk = lambda shape, dt: torch.empty(shape, dtype=dt, device="cuda")
        sgs = [mk(1, torch.float32) for _ in Ws]
        scs = [mk((w.shape[0], w.shape[1] // 16), torch.uint8) for w in Ws]
        cds = [mk((w.shape[0], w.shape[1] // 2), torch.uint8) for w in Ws]
        ws = torch.empty(faar.faar_workspace_bytes(faar.binding.OP_QUANT_RTN_BATCH, 16, 16), dtype=torch.uint8, device="cuda")
        items, dt = faar.tensor_batch(Ws, sgs, scs, codes=cds)
        faar.faar_quant_rtn_batch(items, dt, ws)
        for k, W in enumerate(Ws):
            sg1, sc1, cd1, _ = faar.faar_quant_rtn(W)
            assert torch.equal(sgs[k], sg1) and torch.equal(scs[k], sc1) and torch.equal(cds[k], cd1), k
        # with given tensor scales: same codes again, no workspace
        cds2 = [torch.zeros_like(c) for c in cds]
        scs2 = [torch.zeros_like(c) for c in scs]
        items2, _ = faar.tensor_batch(Ws, sgs, scs2, codes=cds2)
        faar.faar_quant_rtn_batch(items2, dt, None, s_global_given=True)
        assert all(torch.equal(a, b) for a, b in zip(cds, cds2)) and all(torch.equal(a, b) for a, b in zip(scs, scs2))
        # V initialisation (with floor codes) and hardening of planted V
        Vg = [mk(w.shape, torch.float32) for w in Ws]
        fcs = [torch.zeros_like(c) for c in cds]
        items3, _ = faar.tensor_batch(Ws, sgs, scs, Vs=Vg, codes=fcs)
        faar.faar_init_v_batch(items3, dt)
        for k, W in enumerate(Ws):
            V1, fc1 = faar.faar_init_v(W, sgs[k], scs[k], want_floor_codes=True)
            assert torch.equal(Vg[k].view(torch.int32), V1.view(torch.int32)) and torch.equal(fcs[k], fc1), k
        Vd = [dev(v) for v in Vs_h]
        out = [torch.zeros_like(c) for c in cds]
        items4, _ = faar.tensor_batch(Ws, sgs, scs, Vs=Vd, codes=out)
        faar.faar_harden_pack_batch(items4, dt)
        for k, W in enumerate(Ws):
            c1, _, _, _ = faar.faar_harden_pack(W, sgs[k], scs[k], Vd[k])
            assert torch.equal(out[k], c1), k
        for k in (0, 2, 5, 6, 55):
            q = fo.quant_rtn(Ws_h[k], isbf)
            assert np.array_equal(host(cds[k]), q["codes"]) and np.array_equal(host(scs[k]), q["scales"])
            assert np.array_equal(host(out[k]), fo.harden_pack(Ws_h[k], isbf, q["s_global"], q["scales"], Vs_h[k])["codes"])


def test_stochastic_candidates_and_hardened_loss():
    """Candidate sampler bit-exact against the oracle's Philox draw; hardened reconstruction loss of arbitrary,
    round-to-nearest and sampled V against the oracle's float64 evaluation of the packed weights."""
    for name, W, isbf in WCASES[:3]:
        q = fo.quant_rtn(W, isbf)
        Wd = dev(W, isbf)
        sg, scales, _, _ = faar.faar_quant_rtn(Wd)
        V0 = fo.init_v(W, q["s_global"], q["scales"])["V"]
        for seed, sample in ((0, 0), (2 ** 40 + 17, 99)):
            Vs = faar.faar_stochastic_v(Wd, sg, scales, seed, sample)
            assert np.array_equal(host(Vs), fo.stochastic_v(V0, seed, sample)), name
    for c in (build_case("config1"), build_case(RAGGED), build_case(THREE_TILES)):
        Wd, sg, scales, q, Xq, Y, Xt, (C, ic), _ = _setup(c)
        alpha = 1.0 / (c.T * c.O)
        ws = faar.layer_step_workspace(c.O, c.K, c.T)
        V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
        cands = {"rtn": V0, "planted": synth.rounding_variables(c.O, c.K, 3), "sampled": fo.stochastic_v(V0, 7, 1)}
        got = {}
        for k, V in cands.items():
            got[k] = float(faar.faar_hardened_loss(Wd, sg, scales, dev(V), Xq, C, alpha, ws).item())
            want = fo.hardened_loss(c.W, c.w_is_bf16, q["s_global"], q["scales"], V, c.Xq, c.Y_fp, alpha)
            assert got[k] == pytest.approx(want, rel=TOL_LOSS_EXACT_OUTLIER), (c.name, k)
        assert got["rtn"] < got["planted"]          # arbitrary decisions are worse than round-to-nearest


def test_steps_captured_in_a_hip_graph_replay_identically():
    """Every entry point only enqueues kernels on the caller's stream (no allocation, host copy, memset or
    synchronisation), so a run of steps can be captured once and replayed.  Each replay starts from the same
    state and must reproduce the eager results bit for bit; eager work and synchronisations sit between replays."""
    c = synth.config1(0)
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic), hk = _setup(c, h=True)
    alpha = 1.0 / (c.T * c.O)
    ws = faar.layer_step_workspace(c.O, c.K, c.T)
    V0, _ = faar.faar_init_v(Wd, sg, scales)
    betas = [4.0, 8.0, 12.0, 16.0]

    def run_steps(V, m, u, losses):
        for i, beta in enumerate(betas):     # the first two steps in the C form, the last two in the H form
            kw = hk if i >= 2 else {}
            faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, C, ic, beta, 0.01, alpha, 1e-2, 0.9, 0.999, 1e-8, i + 1,
                                 losses[i], ws, beta_next=betas[i + 1] if i + 1 < len(betas) and i != 1 else 0.0,
                                 forward_ready=i in (1, 3), **kw)

    V, m, u = V0.clone(), torch.zeros_like(V0), torch.zeros_like(V0)
    losses = torch.zeros((len(betas), 3), dtype=torch.float32, device="cuda")
    run_steps(V, m, u, losses)
    torch.cuda.synchronize()
    want = [x.clone() for x in (V, m, u, losses)]

    gV, gm, gu = V0.clone(), torch.zeros_like(V0), torch.zeros_like(V0)
    glosses = torch.zeros_like(losses)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_steps(gV, gm, gu, glosses)            # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        run_steps(gV, gm, gu, glosses)
    for _ in range(3):
        gV.copy_(V0); gm.zero_(); gu.zero_(); glosses.zero_()      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip((gV, gm, gu, glosses), want):
            assert torch.equal(a, b)


@pytest.mark.parametrize("O,K,T", [(1, 16, 1), (8, 16, 3), (3, 32, 65), (130, 48, 1)])
def test_smallest_layers_run_the_whole_path(O, K, T):
    """Degenerate sizes: a single scale block, a single token, fewer rows than a lane group; every GEMM is one
    partly filled tile of the generic kernel.  Quantise, prepare, two steps (the second with a prepared forward),
    harden and pack, all against the oracle."""
    c = synth.llm_linear(f"tiny_{O}x{K}_T{T}", O, K, T, 50 + O)
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic), _ = _setup(c)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    V, _ = faar.faar_init_v(Wd, sg, scales)
    assert np.array_equal(host(V), V0)
    m, u = torch.zeros_like(V), torch.zeros_like(V)
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = faar.layer_step_workspace(O, K, T)
    alpha = 1.0 / (T * O)
    Vo, mo, uo = V0, np.zeros_like(V0), np.zeros_like(V0)
    for t, beta in ((1, 6.0), (2, 9.0)):
        faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, C, ic, beta, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"],
                             HYP["beta2"], HYP["eps"], t, losses, ws, beta_next=9.0 if t == 1 else 0.0, forward_ready=t == 2)
        r = fo.layer_step(c.W, q["s_global"], q["scales"], Vo, mo, uo, c.Xq, c.Y_fp, beta, HYP["lambda_round"], alpha,
                          HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], t)
        L = host(losses)
        assert L[0] == pytest.approx(r["L_mse"], rel=2 * TOL_LOSS_EXACT_OUTLIER, abs=1e-12)   # a handful of terms: no averaging
        assert L[1] == pytest.approx(r["L_round"], rel=1e-5, abs=1e-7)
        Vo, mo, uo = host(V).copy(), host(m).copy(), host(u).copy()               # re-synchronise
    codes, _, _, _ = faar.faar_harden_pack(Wd, sg, scales, V)
    assert np.array_equal(host(codes), fo.harden_pack(c.W, True, q["s_global"], q["scales"], host(V))["codes"])


@pytest.mark.parametrize("name", ["llama_q_proj", "llama_gate_proj"])
def test_full_size_codec_bit_exact(name):
    """Quantisation, V initialisation and hardening + packing of whole benchmark-sized tensors (4.2 M and 16.8 M
    weights, the launch configurations the benchmark times), bit for bit against the oracle."""
    c = build_case(name)
    q = fo.quant_rtn(c.W, True)
    Wd = dev(c.W, True)
    sg, scales, codes_g, Wdq = faar.faar_quant_rtn(Wd, want_dq=True)
    assert host(sg)[0].view(np.uint32) == np.float32(q["s_global"]).view(np.uint32)
    assert np.array_equal(host(scales), q["scales"]) and np.array_equal(host(codes_g), q["codes"])
    assert np.array_equal(host(Wdq).view(np.uint32), q["W_dq"].view(np.uint32))
    iv = fo.init_v(c.W, q["s_global"], q["scales"])
    Vg, fc = faar.faar_init_v(Wd, sg, scales, want_floor_codes=True)
    assert np.array_equal(host(Vg).view(np.uint32), iv["V"].view(np.uint32))
    assert np.array_equal(host(fc), iv["floor_codes"])
    Vs = synth.rounding_variables(c.O, c.K, 77)
    hp = fo.harden_pack(c.W, True, q["s_global"], q["scales"], Vs)
    codes2, dec, Wf, flips = faar.faar_harden_pack(Wd, sg, scales, dev(Vs), want_decisions=True, want_final=True, want_flips=True)
    assert np.array_equal(host(codes2), hp["codes"]) and np.array_equal(host(dec), hp["decisions"])
    assert np.array_equal(host(Wf).view(np.uint32), hp["W_final"].view(np.uint32))
    assert int(flips.item()) == hp["flip_count"]
