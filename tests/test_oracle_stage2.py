"""Pins for the oracle's Stage-2 objective (Eq. 6; Table 2 steps 18-22): a library routine for the same
quantity, closed forms, invariances and finite differences -- none of them the oracle's own formula."""
import numpy as np
import pytest
from scipy.special import log_softmax, rel_entr, expit

from oracle import faar_oracle as fo


def _rand(T, V, D, seed):
    rng = np.random.default_rng(seed)
    Zf = rng.standard_normal((T, V)) * 3.0
    Zq = Zf + rng.standard_normal((T, V)) * 0.3
    Hf = rng.standard_normal((T, D))
    Hq = Hf + rng.standard_normal((T, D)) * 0.1
    return Zf, Zq, Hf, Hq


def test_kl_matches_library_relative_entropy_and_log_softmax():
    Zf, Zq, Hf, Hq = _rand(7, 53, 5, 0)
    for tau in (0.7, 1.0, 2.5):
        r = fo.stage2_losses(Zf, Zq, tau, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
        Pf, Pq = np.exp(log_softmax(Zf / tau, axis=-1)), np.exp(log_softmax(Zq / tau, axis=-1))
        assert r["L_kl"] == pytest.approx(rel_entr(Pf, Pq).sum(), rel=1e-12)
        assert np.allclose(fo.log_softmax_t(Zq, tau), log_softmax(Zq / tau, axis=-1), rtol=0, atol=1e-13)


def test_two_class_closed_form():
    # logits [x, 0] vs [y, 0]: P = (sigmoid(x), 1 - sigmoid(x)); KL of two Bernoulli distributions
    x, y, tau = 1.3, -0.4, 1.7
    r = fo.stage2_losses(np.array([[x, 0.0]]), np.array([[y, 0.0]]), tau, 1.0, np.zeros((1, 1)), np.zeros((1, 1)), 1.0,
                         None, 1.0, 0.0)
    p, q = expit(x / tau), expit(y / tau)
    want = p * np.log(p / q) + (1 - p) * np.log((1 - p) / (1 - q))
    assert r["L_kl"] == pytest.approx(want, rel=1e-12)
    # gradient with respect to y: d/dy KL = (q - p) / tau
    assert r["dZ_q"][0, 0] == pytest.approx((q - p) / tau, rel=1e-12)
    assert r["dZ_q"][0, 1] == pytest.approx(-(q - p) / tau, rel=1e-12)


def test_properties_zero_nonnegative_invariances():
    Zf, Zq, Hf, Hq = _rand(5, 40, 6, 1)
    same = fo.stage2_losses(Zf, Zf, 1.3, 1.0, Hf, Hf, 1.0, None, 1.0, 0.0)
    assert abs(same["L_kl"]) < 1e-14 and same["L_mse"] == 0.0 and not same["dZ_q"].any() and not same["dH_q"].any()
    r = fo.stage2_losses(Zf, Zq, 1.3, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
    assert r["L_kl"] > 0
    # a constant added to a row of logits changes nothing; scaling logits and temperature together changes nothing
    shift = np.arange(5)[:, None] * 7.0
    r2 = fo.stage2_losses(Zf + shift, Zq - 2 * shift, 1.3, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
    assert r2["L_kl"] == pytest.approx(r["L_kl"], rel=1e-10)
    r3 = fo.stage2_losses(4 * Zf, 4 * Zq, 4 * 1.3, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
    assert r3["L_kl"] == pytest.approx(r["L_kl"], rel=1e-12)
    # each row of the logit gradient sums to zero (softmax lives on the simplex)
    assert np.abs(r["dZ_q"].sum(axis=1)).max() < 1e-14
    # MSE and the total, written out
    assert r["L_mse"] == pytest.approx(np.linalg.norm(Hf - Hq) ** 2, rel=1e-12)
    full = fo.stage2_losses(Zf, Zq, 1.3, 0.2, Hf, Hq, 0.5, [0.25, 0.5, 0.125], 3.0, 0.01)
    assert full["L_round"] == 0.875
    assert full["L"] == pytest.approx(3.0 * 0.2 * r["L_kl"] + 0.5 * r["L_mse"] + 0.01 * 0.875, rel=1e-12)


def test_gradients_by_central_finite_differences():
    Zf, Zq, Hf, Hq = _rand(3, 11, 4, 2)
    args = dict(tau=1.9, kl_scale=0.37, mse_scale=0.6, round_losses=[0.3], lambda_kl=2.5, lambda_round=0.1)

    def L(zq, hq):
        return fo.stage2_losses(Zf, zq, args["tau"], args["kl_scale"], Hf, hq, args["mse_scale"], args["round_losses"],
                                args["lambda_kl"], args["lambda_round"])["L"]

    r = fo.stage2_losses(Zf, Zq, args["tau"], args["kl_scale"], Hf, Hq, args["mse_scale"], args["round_losses"],
                         args["lambda_kl"], args["lambda_round"])
    eps = 1e-6
    for (i, j) in [(0, 0), (1, 5), (2, 10), (0, 7)]:
        e = np.zeros_like(Zq); e[i, j] = eps
        fd = (L(Zq + e, Hq) - L(Zq - e, Hq)) / (2 * eps)
        assert r["dZ_q"][i, j] == pytest.approx(fd, rel=1e-6, abs=1e-10)
    for (i, j) in [(0, 0), (2, 3), (1, 1)]:
        e = np.zeros_like(Hq); e[i, j] = eps
        fd = (L(Zq, Hq + e) - L(Zq, Hq - e)) / (2 * eps)
        assert r["dH_q"][i, j] == pytest.approx(fd, rel=1e-6, abs=1e-10)


def test_masked_logits_follow_the_zero_log_zero_convention():
    """Logits of -inf (masked vocabulary entries) have probability 0.  An entry with P_fp = 0 contributes nothing to
    KL(P_fp || P_q) whatever P_q is; P_q = 0 where P_fp > 0 makes it +inf: the library relative entropy
    (rel_entr(0, y) = 0, rel_entr(x, 0) = inf) on library softmaxes, and the restriction to the unmasked entries."""
    Zf, Zq, Hf, Hq = _rand(4, 24, 3, 5)
    Zf[:, 3] = -np.inf                      # masked in both models
    Zq[:, 3] = -np.inf
    Zf[1, 7] = -np.inf                      # masked in the full-precision model only
    Zf[2, :5] = -np.inf                     # a masked prefix (the running maximum starts at -inf)
    r = fo.stage2_losses(Zf, Zq, 1.4, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
    Pf, Pq = np.exp(log_softmax(Zf / 1.4, axis=-1)), np.exp(log_softmax(Zq / 1.4, axis=-1))
    assert np.isfinite(r["L_kl"]) and r["L_kl"] == pytest.approx(rel_entr(Pf, Pq).sum(), rel=1e-12)
    assert np.isfinite(r["dZ_q"]).all() and not r["dZ_q"][:, 3].any()
    # masking an entry in both models is the same as deleting it
    keep = [j for j in range(24) if j != 3]
    r_del = fo.stage2_losses(Zf[:, keep], Zq[:, keep], 1.4, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
    assert r["L_kl"] == pytest.approx(r_del["L_kl"], rel=1e-12)
    Zq2 = Zq.copy()
    Zq2[0, 9] = -np.inf                     # P_q = 0 where P_fp > 0
    assert fo.stage2_losses(Zf, Zq2, 1.4, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)["L_kl"] == np.inf
