"""GPU parity of faar_stage2_losses (Eq. 6; Table 2 steps 18-22) against the float64 oracle.

Tolerances: the kernel works in float32 with the hardware exp (about 2 ulp).  A row's KL is w/sa - log(sa/sb) - ...
with sa, sb float32 sums over the vocabulary, each good to about 1e-6 relative, so the row's KL carries an ABSOLUTE
error of about 1e-6 whatever its size: losses are compared with 1e-5 relative plus 2e-6 per row.  The hardware
exp of an argument of size 10-15 is good to about 1e-6 relative (the argument is scaled by log2 e in float32
first), so each probability carries that relative error and a logit gradient coef * (P_q - P_fp) is compared per
element against 3e-6 * coef * (largest probability of the tensor).  bf16 outputs are the float32 values rounded
once more: one bf16 ulp."""
import numpy as np
import pytest
import torch

from oracle import faar_oracle as fo

pytestmark = pytest.mark.gpu

import paper_2603_22370_amd as faar  # noqa: E402


def _inputs(T, V, D, seed, spread=3.0, noise=0.3):
    rng = np.random.default_rng([seed, 41])
    Zf = (rng.standard_normal((T, V)) * spread).astype(np.float32)
    Zq = (Zf + rng.standard_normal((T, V)).astype(np.float32) * noise).astype(np.float32)
    Hf = rng.standard_normal((T, D)).astype(np.float32)
    Hq = (Hf + rng.standard_normal((T, D)).astype(np.float32) * 0.1).astype(np.float32)
    return Zf, Zq, Hf, Hq


def _bf16(a):
    return torch.from_numpy(a).to(torch.bfloat16).float().numpy()


CASES = [  # T, vocab, D, tau
    (5, 8, 8, 1.0),                 # a single chunk per row: most threads see no element
    (7, 1000, 24, 0.7),             # ragged: fewer chunks than threads
    (3, 8 * 1024 * 3 + 40, 64, 2.0),  # several strides of the workgroup plus a tail
    (33, 32000, 256, 1.0),
    (3, 128256, 16, 1.0),           # Llama3 vocabulary: the row of Z_fp held in registers (16 chunks per lane)
    (2, 151936, 16, 0.9),           # Qwen3 vocabulary: 19 chunks per lane
    (2, 163904, 16, 1.5),           # longer than a register-resident row: two passes over global memory
]


@pytest.mark.parametrize("T,V,D,tau", CASES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stage2_losses_and_gradients(T, V, D, tau, dtype):
    Zf, Zq, Hf, Hq = _inputs(T, V, D, T + V)
    if dtype == "bf16":
        Zf, Zq, Hf, Hq = _bf16(Zf), _bf16(Zq), _bf16(Hf), _bf16(Hq)
    rl = np.array([0.25, 0.5, 0.375], dtype=np.float32)
    kw = dict(kl_scale=1.0 / T, mse_scale=1.0 / (T * D), lambda_kl=2.0, lambda_round=0.01)
    ref = fo.stage2_losses(Zf, Zq, tau, kw["kl_scale"], Hf, Hq, kw["mse_scale"], rl, kw["lambda_kl"], kw["lambda_round"])
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda a: torch.from_numpy(a).cuda().to(td)
    losses, dZ, dH = faar.faar_stage2_losses(dev(Zf), dev(Zq), tau, dev(Hf), dev(Hq), round_losses=torch.from_numpy(rl).cuda(), **kw)
    L = losses.cpu().numpy().astype(np.float64)
    assert L[0] == pytest.approx(ref["L_kl"], rel=1e-5, abs=2e-6 * kw["kl_scale"] * T)
    assert L[1] == pytest.approx(ref["L_mse"], rel=1e-5)
    assert L[2] == pytest.approx(ref["L_round"], rel=1e-6)
    assert L[3] == pytest.approx(ref["L"], rel=1e-5, abs=2e-6 * kw["kl_scale"] * T * kw["lambda_kl"])
    gz, gh = dZ.float().cpu().numpy().astype(np.float64), dH.float().cpu().numpy().astype(np.float64)
    ulp = 2.0 ** -8 if dtype == "bf16" else 0.0
    pmax = max(np.exp(fo.log_softmax_t(Zf, tau)).max(), np.exp(fo.log_softmax_t(Zq, tau)).max())
    coef = kw["lambda_kl"] * kw["kl_scale"] / tau
    assert np.all(np.abs(gz - ref["dZ_q"]) <= 3e-6 * coef * pmax + ulp * np.abs(ref["dZ_q"]))
    assert np.all(np.abs(gh - ref["dH_q"]) <= 2e-6 * np.abs(ref["dH_q"]).max() + ulp * np.abs(ref["dH_q"]))
    # loss only: same numbers, no gradient buffers
    l2, z2, h2 = faar.faar_stage2_losses(dev(Zf), dev(Zq), tau, dev(Hf), dev(Hq), round_losses=torch.from_numpy(rl).cuda(),
                                         want_grads=False, **kw)
    assert z2 is None and h2 is None and torch.equal(l2, losses)


def test_stage2_degenerate_and_extreme_inputs():
    T, V, D = 4, 4096, 16
    Zf, Zq, Hf, Hq = _inputs(T, V, D, 9, spread=30.0, noise=5.0)     # logits of +-100: exp must not overflow
    Zf[1] += 1000.0                                                  # a row shifted as a whole
    dev = lambda a: torch.from_numpy(a).cuda()
    ref = fo.stage2_losses(Zf, Zq, 1.0, 1.0, Hf, Hq, 1.0, None, 1.0, 0.0)
    losses, dZ, _ = faar.faar_stage2_losses(dev(Zf), dev(Zq), 1.0, dev(Hf), dev(Hq))
    L = losses.cpu().numpy()
    assert np.isfinite(L).all() and L[0] == pytest.approx(ref["L_kl"], rel=2e-5)
    assert np.all(np.abs(dZ.cpu().numpy() - ref["dZ_q"]) <= 4e-6)
    # identical models: every loss and gradient is zero (up to float32 noise of the log-sum-exp)
    losses, dZ, dH = faar.faar_stage2_losses(dev(Zf), dev(Zf), 1.0, dev(Hf), dev(Hf))
    L = losses.cpu().numpy()
    assert abs(L[0]) <= 1e-5 * T and L[1] == 0.0 and L[2] == 0.0
    assert not dZ.any() and not dH.any()
    # two runs give the same bits
    a = faar.faar_stage2_losses(dev(Zf), dev(Zq), 1.3, dev(Hf), dev(Hq))
    b = faar.faar_stage2_losses(dev(Zf), dev(Zq), 1.3, dev(Hf), dev(Hq))
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


@pytest.mark.parametrize("V", [4096, 128256])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stage2_masked_logits(V, dtype):
    """Logits of -inf (masked vocabulary entries): probability 0, no contribution to the KL where P_fp = 0 (also when
    only the full-precision model masks the entry), finite losses and gradients; +inf where only the quantised model
    masks an entry the full-precision model gives weight to.  Both the plain and the register-resident row kernel."""
    T, D = 4, 16
    Zf, Zq, Hf, Hq = _inputs(T, V, D, 13)
    if dtype == "bf16":
        Zf, Zq, Hf, Hq = _bf16(Zf), _bf16(Zq), _bf16(Hf), _bf16(Hq)
    Zf[:, 100:164] = -np.inf
    Zq[:, 100:164] = -np.inf
    Zf[1, 7] = -np.inf
    Zf[2, :2048] = -np.inf          # the first chunks of every lane are all masked: the running maximum stays -inf
    Zq[2, :1024] = -np.inf
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda a: torch.from_numpy(a).cuda().to(td)
    ref = fo.stage2_losses(Zf, Zq, 1.0, 1.0 / T, Hf, Hq, 1.0, None, 1.0, 0.0)
    losses, dZ, _ = faar.faar_stage2_losses(dev(Zf), dev(Zq), 1.0, dev(Hf), dev(Hq), kl_scale=1.0 / T)
    L = losses.cpu().numpy().astype(np.float64)
    assert np.isfinite(L).all() and L[0] == pytest.approx(ref["L_kl"], rel=1e-5, abs=2e-6)
    gz = dZ.float().cpu().numpy().astype(np.float64)
    ulp = 2.0 ** -8 if dtype == "bf16" else 0.0
    assert np.isfinite(gz).all()
    assert np.all(np.abs(gz - ref["dZ_q"]) <= 3e-6 / T + ulp * np.abs(ref["dZ_q"]))
    Zq[0, 9] = -np.inf
    losses, _, _ = faar.faar_stage2_losses(dev(Zf), dev(Zq), 1.0, dev(Hf), dev(Hq), kl_scale=1.0 / T)
    assert losses[0].item() == np.inf
