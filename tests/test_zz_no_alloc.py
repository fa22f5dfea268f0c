"""The entry point that allocates nothing (faar_softquant_fwd_bwd_static) against the workspace-taking entry point
it is a variant of: same kernels, so every output must agree bit for bit -- on two calls in a row, the second on a
smaller tensor (the resident partial-sum array then still holds the first call's sums beyond the second call's
count), and for both weight storage types.  Also its size limit and argument checks."""
import ctypes

import numpy as np
import pytest
import torch

from workloads import synth

pytestmark = pytest.mark.gpu

import paper_2603_22370_amd as faar  # noqa: E402
from paper_2603_22370_amd import binding as fb  # noqa: E402


def _inputs(O, K, seed, bf16):
    W_h = synth.student_t_weight(O, K, seed) if bf16 else synth.gaussian_weight(O, K, seed)
    W = torch.from_numpy(W_h).cuda()
    W = W.to(torch.bfloat16) if bf16 else W
    sg, scales, _, _ = faar.faar_quant_rtn(W)
    V = torch.from_numpy(synth.rounding_variables(O, K, seed + 1)).cuda()
    rng = np.random.default_rng([seed, 43])
    dWt = torch.from_numpy((rng.standard_normal((O, K)) * 1e-3).astype(np.float32)).cuda()
    return W, sg, scales, V, dWt


def _both(W, sg, scales, V, dWt, beta, lam, delta):
    O, K = W.shape
    want = faar.faar_softquant_fwd_bwd(W, sg, scales, V, beta, dWt=dWt, lambda_round=lam, emit_delta=delta)
    Wt = torch.empty((O, K), dtype=torch.bfloat16, device="cuda")
    dV = torch.empty((O, K), dtype=torch.float32, device="cuda")
    rl = torch.empty(1, dtype=torch.float32, device="cuda")
    faar.faar_softquant_fwd_bwd_static(W, sg, scales, V, beta, Wt, dWt=dWt, lambda_round=lam, dV=dV, round_loss=rl,
                                       emit_delta=delta)
    torch.cuda.synchronize()
    return want, (Wt, dV, rl)


@pytest.mark.parametrize("bf16", [True, False])
def test_static_entry_point_matches_the_workspace_one_on_two_calls_in_a_row(bf16):
    # first a tensor of 2.1 M weights (1024 partial sums), then one of 30 k weights (15 partial sums, ragged last block)
    for (O, K, seed, beta, lam, delta) in ((1024, 2048, 3, 6.0, 0.05, True), (96, 320, 4, 11.0, 0.01, False)):
        want, got = _both(*_inputs(O, K, seed, bf16), beta, lam, delta)
        for a, b in zip(want, got):
            assert torch.equal(a, b), (O, K)
    # forward only: no partial sums, no backward outputs
    W, sg, scales, V, _ = _inputs(64, 256, 5, bf16)
    Wt = torch.empty((64, 256), dtype=torch.bfloat16, device="cuda")
    faar.faar_softquant_fwd_bwd_static(W, sg, scales, V, 9.0, Wt)
    assert torch.equal(Wt, faar.faar_softquant_fwd_bwd(W, sg, scales, V, 9.0)[0])


def test_static_entry_point_rejects_what_it_cannot_hold():
    L = fb.lib()
    p = ctypes.c_void_p(0x1000)      # never dereferenced: validation comes first
    f = L.faar_softquant_fwd_bwd_static
    assert f(p, 1, 1 << 14, 1 << 14, p, p, p, 4.0, p, p, 0.0, p, p, 0, None) == -2     # 2^28 weights > 2^27
    assert f(p, 1, 1 << 13, 1 << 14, p, p, p, 4.0, None, p, 0.0, p, p, 0, None) == -1  # at the limit: next check (Wt null)
    assert f(p, 1, 16, 16, p, p, p, -1.0, p, p, 0.0, p, p, 0, None) == -6
    assert f(p, 1, 16, 16, p, p, p, 4.0, p, p, 0.0, None, p, 0, None) == -1            # dWt without dV
    assert f(p, 1, 16, 24, p, p, p, 4.0, p, None, 0.0, None, None, 0, None) == -2
