"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs.
Integer / byte / index results bit-exact; float results within the tolerances stated at TOL_EXACT below
(bf16 matrix-core path vs float64 oracle)."""
import numpy as np
import pytest
import torch

from oracle import faar_oracle as fo
from workloads import synth

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


def linear_cases():
    yield synth.config1(0)
    c = synth.llm_linear("ragged", 96, 80, 100, 21, quantised_acts=True)          # nothing a multiple of the tile
    yield c
    yield synth.llm_linear("kproj_slice", 512, 2048, 640, 22)
    yield synth.llm_linear("three_tiles", 320, 256, 300, 23, quantised_acts=True)
    # tile-shape coverage of the GEMM planner: 384 tiles of 256x256 with only two contraction slices,
    # and 192 tiles of 256x128; the dW GEMM of both splits its contraction over the tokens
    yield synth.llm_linear("wide_256x256_tiles", 12288, 64, 2048, 24)
    yield synth.llm_linear("mid_256x128_tiles", 3072, 96, 2048, 25, quantised_acts=True)


LCASES = list(linear_cases())
LIDS = [c.name for c in LCASES]


def _setup(c):
    Wd = dev(c.W, c.w_is_bf16)
    sg, scales, _, _ = faar.faar_quant_rtn(Wd)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    Xq = dev(c.Xq, True)
    Y = dev(c.Y_fp, True)
    Xt, C, ic = faar.faar_layer_prepare(Wd, sg, scales, Xq, Y)
    return Wd, sg, scales, q, Xq, Y, Xt, (C, ic)


@pytest.mark.parametrize("c", LCASES, ids=LIDS)
def test_layer_prepare(c):
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic) = _setup(c)
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
    # cached interval codes: sign bit and k_lo (7 for a zero weight)
    wt = fo.normalised_magnitude(c.W, q["scales"], q["s_global"])
    want_ic = (np.signbit(c.W).astype(np.uint8) << 3) | np.where(c.W == 0, 7, fo.find_interval(wt)).astype(np.uint8)
    assert np.array_equal(host(ic), fo.pack_nibbles(want_ic))
    # also with a float32 reference output
    Xt2, C2, ic2 = faar.faar_layer_prepare(Wd, sg, scales, Xq, dev(c.Y_fp))
    assert torch.equal(C2, C) and torch.equal(Xt2, Xt) and torch.equal(ic2, ic)


# Two bf16 roundings (unit roundoff u = 2^-9) sit between the inputs and the loss / gradient: the
# weight perturbation W_q - W and dY.  A loss or gradient dominated by a few outlier terms can move
# by up to 2u; sums over many terms average far below that.  Against the oracle evaluated with the
# same declared roundings only float32 accumulation noise remains.
TOL_EXACT = 2 * 2.0 ** -9

HYP = dict(lambda_round=0.01, lr=5e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def _one_step(c, beta, V0, t=1, m0=None, u0=None, dY_ext=None, want_dX=False):
    Wd, sg, scales, q, Xq, Y, Xt, C = _setup(c)
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
                         dY_ext=None if dY_ext is None else dev(dY_ext, True), dX=dX)
    torch.cuda.synchronize()
    ref = {}
    for mode in (False, True):
        ref[mode] = fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0) if m0 is None else m0,
                                  np.zeros_like(V0) if u0 is None else u0, c.Xq, c.Y_fp, beta, HYP["lambda_round"],
                                  alpha, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], t, want_dX=want_dX,
                                  dY_ext=dY_ext, declared_rounding=mode)
    return host(V), host(m), host(u), host(losses), (None if dX is None else host(dX)), ref


def _check_grad(g, ref):
    exact, decl = ref[False]["dV"], ref[True]["dV"]
    n = np.linalg.norm
    assert n(g - exact) <= TOL_EXACT * n(exact)                  # vs float64 oracle, no rounding anywhere
    assert n(g - decl) <= 5e-4 * n(decl)                         # vs oracle with the three declared bf16 roundings
    rms = np.sqrt(np.mean(decl ** 2))
    # a value on a bf16 rounding boundary may round the other way in float32 than in float64: one such
    # flip of W_q - W moves that weight's own gradient by up to 2^-8 relative (coherent over all tokens)
    assert np.all(np.abs(g - decl) <= 2.0 ** -7 * np.abs(decl) + 2e-2 * rms)


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


@pytest.mark.parametrize("c", LCASES, ids=LIDS)
@pytest.mark.parametrize("beta", [4.0, 20.0])
def test_layer_step_first_step(c, beta):
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    V, m, u, losses, _, ref = _one_step(c, beta, V0)
    ex = ref[False]
    assert losses[0] == pytest.approx(ex["L_mse"], rel=TOL_EXACT)
    assert losses[1] == pytest.approx(ex["L_round"], rel=1e-5)
    assert losses[2] == pytest.approx(ex["L"], rel=TOL_EXACT)
    assert losses[0] == pytest.approx(ref[True]["L_mse"], rel=2e-5)
    # with zero initial state, m = (1 - beta1) g: the gradient is observable through m
    _check_grad(m.astype(np.float64) / (1 - HYP["beta1"]), ref)
    _check_update(V, m, u, V0, np.zeros_like(V0), np.zeros_like(V0), 1)


def test_layer_step_with_state_and_random_v():
    c = LCASES[3]
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
    assert losses[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_EXACT)
    assert losses[0] == pytest.approx(ref[True]["L_mse"], rel=2e-5)
    assert losses[1] == pytest.approx(ref[False]["L_round"], rel=1e-5)


def test_layer_step_chained_dY_ext_and_dX():
    c = LCASES[3]
    rng = np.random.default_rng(13)
    q = fo.quant_rtn(c.W, c.w_is_bf16)
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    dY = synth.round_to_bf16((rng.standard_normal((c.T, c.O)) * 1e-3).astype(np.float32))
    for ext in (dY, None):
        V, m, u, losses, dX, ref = _one_step(c, 6.0, V0, dY_ext=ext, want_dX=True)
        _check_grad(m.astype(np.float64) / (1 - HYP["beta1"]), ref)
        n = np.linalg.norm
        assert n(dX - ref[False]["dX"]) <= 5e-3 * n(ref[False]["dX"])   # three roundings on this path: dY, W_q, dX
        assert n(dX - ref[True]["dX"]) <= 1e-3 * n(ref[True]["dX"])     # final bf16 rounding of dX included on both sides
        assert losses[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_EXACT)


def test_config1_trajectory_100_adam_steps():
    """The small parity config end to end: 100 Adam steps with beta annealed 4 -> 32.  The oracle is
    re-synchronised to the GPU's (V, m, u) every 10 steps; every step's losses must agree, V stays
    in [0,1], and the packed result of the GPU's final V is bit-exact with the oracle's packing."""
    c = synth.config1(0)
    Wd, sg, scales, q, Xq, Y, Xt, C = _setup(c)
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
        faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, *C, beta, 0.01, alpha, lr, 0.9, 0.999, 1e-8, t, losses, ws)
        r = fo.layer_step(c.W, q["s_global"], q["scales"], Vo, mo, uo, c.Xq, c.Y_fp, beta, 0.01, alpha, lr, 0.9,
                          0.999, 1e-8, t)
        Vo, mo, uo = r["V"], r["m"], r["u"]
        L = host(losses)
        assert L[0] == pytest.approx(r["L_mse"], rel=TOL_EXACT), t
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


def test_resume_is_bit_exact_and_runs_are_deterministic():
    c = LCASES[3]
    Wd, sg, scales, q, Xq, Y, Xt, C = _setup(c)
    alpha = 1.0 / (c.T * c.O)
    ws = faar.layer_step_workspace(c.O, c.K, c.T)

    def run(n_steps, state=None, t0=0):
        if state is None:
            V, _ = faar.faar_init_v(Wd, sg, scales)
            state = [V, torch.zeros_like(V), torch.zeros_like(V)]
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        for t in range(t0 + 1, t0 + n_steps + 1):
            faar.faar_layer_step(Wd, sg, scales, *state, Xq, Xt, *C, 4.0 + t, 0.01, alpha, 5e-3, 0.9, 0.999, 1e-8, t,
                                 losses, ws)
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
    for c, want_dX in ((synth.config1(0), False), (LCASES[3], False), (LCASES[3], True), (LCASES[1], True)):
        Wd, sg, scales, q, Xq, Y, Xt, C = _setup(c)
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
                                     t0 + i, losses, ws, dX=dX, beta_next=nxt, forward_ready=fused and i > 0)
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
                                 2 + i, losses, ws, dX=dX, beta_next=float(rng.uniform(1, 40)))
        for x, y in zip(a, state):
            assert torch.equal(x, y), c.name
        assert torch.equal(losses, oa[-1][0])


def test_nvfp4_activations_in_units_of_their_tensor_scale():
    """Activations quantised to NVFP4 by the same kernel (blocks along K, their own tensor scale): W_dq in units of
    s_global is the exact product node * block scale, and a step fed (Xq, x_scale) agrees with the oracle fed the
    dequantised activations x_scale * Xq."""
    for c, seed in ((LCASES[1], 31), (LCASES[3], 32)):          # ragged 96x80 T=100 (generic GEMM), 320x256 T=300
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
        Xt, C, ic = faar.faar_layer_prepare(Wd, sg, scales, Xu, dev(c.Y_fp, True), x_scale=sX)
        Cg = host(C).transpose(0, 2, 1).reshape(-1, c.O)[:c.T]
        C_want = c.Y_fp.astype(np.float64) - Xq.astype(np.float64) @ c.W.astype(np.float64).T
        scale = np.abs(Xq.astype(np.float64)) @ np.abs(c.W.astype(np.float64)).T
        assert np.all(np.abs(Cg - C_want) <= 4e-6 * scale + 1e-30)
        V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
        V, m, u = dev(V0.copy()), dev(np.zeros_like(V0)), dev(np.zeros_like(V0))
        losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        ws = faar.layer_step_workspace(c.O, c.K, c.T)
        alpha = 1.0 / (c.T * c.O)
        faar.faar_layer_step(Wd, sg, scales, V, m, u, Xu, Xt, C, ic, 8.0, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"],
                             HYP["beta2"], HYP["eps"], 1, losses, ws, x_scale=sX)
        ref = {mode: fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0), np.zeros_like(V0), Xq, c.Y_fp,
                                   8.0, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], 1,
                                   declared_rounding=mode) for mode in (False, True)}
        L = host(losses)
        assert L[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_EXACT)
        assert L[0] == pytest.approx(ref[True]["L_mse"], rel=2e-5)
        _check_grad(host(m).astype(np.float64) / (1 - HYP["beta1"]), ref)


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
    for c in (LCASES[0], LCASES[1], LCASES[3]):
        Wd, sg, scales, q, Xq, Y, Xt, (C, ic) = _setup(c)
        alpha = 1.0 / (c.T * c.O)
        ws = faar.layer_step_workspace(c.O, c.K, c.T)
        V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
        cands = {"rtn": V0, "planted": synth.rounding_variables(c.O, c.K, 3), "sampled": fo.stochastic_v(V0, 7, 1)}
        got = {}
        for k, V in cands.items():
            got[k] = float(faar.faar_hardened_loss(Wd, sg, scales, dev(V), Xq, C, alpha, ws).item())
            want = fo.hardened_loss(c.W, c.w_is_bf16, q["s_global"], q["scales"], V, c.Xq, c.Y_fp, alpha)
            assert got[k] == pytest.approx(want, rel=TOL_EXACT), (c.name, k)
        assert got["rtn"] < got["planted"]          # arbitrary decisions are worse than round-to-nearest


def test_steps_captured_in_a_hip_graph_replay_identically():
    """Every entry point only enqueues kernels on the caller's stream (no allocation, host copy, memset or
    synchronisation), so a run of steps can be captured once and replayed.  Each replay starts from the same
    state and must reproduce the eager results bit for bit; eager work and synchronisations sit between replays."""
    c = synth.config1(0)
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic) = _setup(c)
    alpha = 1.0 / (c.T * c.O)
    ws = faar.layer_step_workspace(c.O, c.K, c.T)
    V0, _ = faar.faar_init_v(Wd, sg, scales)
    betas = [4.0, 8.0, 12.0, 16.0]

    def run_steps(V, m, u, losses):
        for i, beta in enumerate(betas):
            faar.faar_layer_step(Wd, sg, scales, V, m, u, Xq, Xt, C, ic, beta, 0.01, alpha, 1e-2, 0.9, 0.999, 1e-8, i + 1,
                                 losses[i], ws, beta_next=betas[i + 1] if i + 1 < len(betas) else 0.0, forward_ready=i > 0)

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
    Wd, sg, scales, q, Xq, Y, Xt, (C, ic) = _setup(c)
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
        assert L[0] == pytest.approx(r["L_mse"], rel=2 * TOL_EXACT, abs=1e-12)   # a handful of terms: no averaging
        assert L[1] == pytest.approx(r["L_round"], rel=1e-5, abs=1e-7)
        Vo, mo, uo = host(V).copy(), host(m).copy(), host(u).copy()               # re-synchronise
    codes, _, _, _ = faar.faar_harden_pack(Wd, sg, scales, V)
    assert np.array_equal(host(codes), fo.harden_pack(c.W, True, q["s_global"], q["scales"], host(V))["codes"])


def test_full_size_q_proj_step_and_pack():
    """The benchmark's own workload and launch configuration (Llama3-1B-shaped q_proj, W 2048x2048 bf16,
    X 4096x2048): one whole step against the oracle -- the float64 matmuls of this size take a few seconds --
    and bit-exact quantisation / packing of all 4.2 M weights."""
    c = synth.llm_linear("q_proj", 2048, 2048, 4096, 0)
    q = fo.quant_rtn(c.W, True)
    Wd, sg, scales, _, Xq, Y, Xt, C = _setup(c)
    _, scales_g, codes_g, _ = faar.faar_quant_rtn(Wd)
    assert np.array_equal(host(scales_g), q["scales"]) and np.array_equal(host(codes_g), q["codes"])
    V0 = fo.init_v(c.W, q["s_global"], q["scales"])["V"]
    Vg, _ = faar.faar_init_v(Wd, sg, scales)
    assert np.array_equal(host(Vg).view(np.uint32), V0.view(np.uint32))
    alpha = 1.0 / (c.T * c.O)
    m = torch.zeros_like(Vg)
    u = torch.zeros_like(Vg)
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = faar.layer_step_workspace(c.O, c.K, c.T)
    faar.faar_layer_step(Wd, sg, scales, Vg, m, u, Xq, Xt, *C, 8.0, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"],
                         HYP["beta2"], HYP["eps"], 1, losses, ws)
    torch.cuda.synchronize()
    ref = {mode: fo.layer_step(c.W, q["s_global"], q["scales"], V0, np.zeros_like(V0), np.zeros_like(V0), c.Xq, c.Y_fp,
                               8.0, HYP["lambda_round"], alpha, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], 1,
                               declared_rounding=mode) for mode in (False, True)}
    L = host(losses)
    assert L[0] == pytest.approx(ref[False]["L_mse"], rel=TOL_EXACT)
    assert L[0] == pytest.approx(ref[True]["L_mse"], rel=2e-5)
    assert L[1] == pytest.approx(ref[False]["L_round"], rel=1e-5)
    _check_grad(host(m).astype(np.float64) / (1 - HYP["beta1"]), ref)
    _check_update(host(Vg), host(m), host(u), V0, np.zeros_like(V0), np.zeros_like(V0), 1)
    hp = fo.harden_pack(c.W, True, q["s_global"], q["scales"], host(Vg))
    codes2, dec, Wf, flips = faar.faar_harden_pack(Wd, sg, scales, Vg, want_decisions=True, want_final=True, want_flips=True)
    assert np.array_equal(host(codes2), hp["codes"]) and np.array_equal(host(dec), hp["decisions"])
    assert np.array_equal(host(Wf).view(np.uint32), hp["W_final"].view(np.uint32))
    assert int(flips.item()) == hp["flip_count"]
