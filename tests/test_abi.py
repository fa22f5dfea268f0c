"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, sizes workspaces consistently, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2603_22370_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "faar.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(faar_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_five_hot_path_calls():
    names = _declared()
    for n in ["faar_quant_rtn", "faar_init_v", "faar_softquant_fwd_bwd", "faar_layer_step", "faar_harden_pack"]:
        assert n in names


def test_library_exports_every_declared_symbol():
    L = fb.lib()
    for n in _declared():
        assert hasattr(L, n), n
    assert L.faar_version() >= 100


def test_workspace_sizes():
    assert fb.faar_workspace_bytes(fb.OP_QUANT_RTN, 256, 256) >= 4096
    assert fb.faar_workspace_bytes(fb.OP_QUANT_RTN, 256, 250) == 0           # K % 16
    assert fb.faar_workspace_bytes(fb.OP_LAYER_STEP, 256, 256, 0) == 0        # T missing
    assert fb.faar_workspace_bytes(99, 256, 256, 64) == 0
    a = fb.faar_workspace_bytes(fb.OP_LAYER_STEP, 2048, 2048, 4096)
    b = fb.faar_workspace_bytes(fb.OP_LAYER_STEP, 2048, 2048, 4096, fb.FAAR_WS_CHAINED)
    assert b > a >= 2048 * 2048 * (2 + 4) + 2048 * 4096 * 2
    assert fb.faar_padded_tokens(64) == 64 and fb.faar_padded_tokens(65) == 128 and fb.faar_padded_tokens(1) == 64


def test_error_codes_without_a_gpu():
    """Every call below must fail validation (negative code) before any kernel launch."""
    L = fb.lib()
    p = ctypes.c_void_p(0x1000)          # a non-null, 16-byte aligned dummy; never dereferenced
    odd = ctypes.c_void_p(0x1004)
    nul = None
    q = L.faar_quant_rtn
    assert q(nul, 1, 16, 16, p, p, p, nul, 0, p, 4096, nul) == -1
    assert q(p, 1, 16, 24, p, p, p, nul, 0, p, 4096, nul) == -2
    assert q(p, 1, 0, 16, p, p, p, nul, 0, p, 4096, nul) == -2
    assert q(p, 7, 16, 16, p, p, p, nul, 0, p, 4096, nul) == -3
    assert q(p, 1, 16, 16, p, p, p, nul, 0, p, 16, nul) == -4
    assert q(p, 1, 16, 16, p, p, p, nul, 0, nul, 0, nul) == -4
    assert q(p, 1, 16, 16, p, p, p, nul, 64, p, 4096, nul) == -6
    assert q(odd, 1, 16, 16, p, p, p, nul, 0, p, 4096, nul) == -6
    assert L.faar_init_v(p, 1, 16, 16, p, p, nul, nul, nul) == -1
    assert L.faar_init_v(p, 1, 16, 8, p, p, p, nul, nul) == -2
    sq = L.faar_softquant_fwd_bwd
    assert sq(p, 1, 16, 16, p, p, p, 0.0, p, nul, 0.0, nul, nul, 0, p, 4096, nul) == -6      # beta <= 0
    assert sq(p, 1, 16, 16, p, p, p, float("inf"), p, nul, 0.0, nul, nul, 0, p, 4096, nul) == -6
    assert sq(p, 1, 16, 16, p, p, p, 4.0, p, p, 0.0, nul, nul, 0, p, 4096, nul) == -1         # dWt without dV
    assert sq(p, 1, 16, 16, p, p, p, 4.0, p, p, 0.0, p, nul, 0, p, 1, nul) == -4
    lp = L.faar_layer_prepare
    assert lp(p, 1, 16, 16, p, p, p, nul, p, 1, 0, p, p, p, nul, nul, p, 1 << 20, nul) == -2   # T <= 0
    assert lp(p, 0, 16, 16, p, p, p, nul, p, 1, 8, p, p, p, nul, nul, nul, 0, nul) == -4       # fp32 W needs ws
    assert lp(p, 1, 16, 16, p, p, p, nul, p, 1, 8, p, p, nul, nul, nul, p, 1 << 20, nul) == -1 # icodes missing
    assert lp(p, 1, 16, 16, p, p, p, nul, p, 1, 8, p, p, p, p, nul, p, 1 << 20, nul) == -1     # H without c_norm2
    assert lp(p, 1, 16, 16, p, p, p, nul, p, 1, 8, p, p, p, p, p, nul, 0, nul) == -4           # H needs ws
    assert lp(p, 1, 16, 16, p, p, p, nul, p, 1, 8, p, p, p, p, p, p, 64, nul) == -4
    assert (fb.faar_workspace_bytes(fb.OP_LAYER_PREPARE, 2048, 2048, 4096, fb.FAAR_WS_GRADIENT_CONSTANT)
            > fb.faar_workspace_bytes(fb.OP_LAYER_PREPARE, 2048, 2048, 4096))
    opt = fb.faar_adam(1e-3, 0.9, 0.999, 1e-8, 1)
    st = L.faar_layer_step
    big = 1 << 30
    args = lambda **kw: [kw.get("W", p), 1, kw.get("O", 16), 16, p, p, p, p, p, p, nul, p, p, p, kw.get("H", nul),
                         kw.get("cn", nul), kw.get("T", 8),
                         kw.get("dYe", nul), kw.get("dX", nul), kw.get("beta", 4.0), kw.get("beta_next", 0.0), 0.01, 1.0,
                         ctypes.byref(kw.get("opt", opt)), p, kw.get("flags", 0), p, kw.get("ws", big), nul]
    assert st(*args(W=nul)) == -1
    assert st(*args(T=0)) == -2
    assert st(*args(beta=-1.0)) == -6
    assert st(*args(beta_next=-1.0)) == -6
    assert st(*args(beta_next=float("nan"))) == -6
    assert st(*args(flags=16)) == -6                                                       # unknown flag bit
    assert st(*args(opt=fb.faar_adam(-1.0, 0.9, 0.999, 1e-8, 1))) == -6
    assert st(*args(opt=fb.faar_adam(1e-3, 0.9, 0.999, 1e-8, 0))) == -6
    assert st(*args(ws=16)) == -4
    assert st(*args(O=12, dX=p)) == -2                                                     # chained needs O % 8 == 0
    assert st(*args(H=p)) == -1                                                            # H and c_norm2 come as a pair
    assert st(*args(cn=p)) == -1
    s2 = L.faar_stage2_losses
    s2a = lambda **kw: [kw.get("Zf", p), p, 1, kw.get("T", 4), kw.get("V", 64), kw.get("tau", 1.0), 1.0, p, p, 1, kw.get("D", 16), 1.0,
                        kw.get("rl", nul), kw.get("nl", 0), 1.0, 0.0, nul, nul, p, p, kw.get("ws", big), nul]
    assert s2(*s2a(Zf=nul)) == -1
    assert s2(*s2a(V=60)) == -2                                                            # vocabulary not a multiple of 8
    assert s2(*s2a(tau=0.0)) == -6
    assert s2(*s2a(nl=3)) == -1                                                            # layers announced, no array
    assert s2(*s2a(ws=8)) == -4
    hp = L.faar_harden_pack
    assert hp(p, 1, 16, 16, p, p, p, nul, nul, nul, nul, nul) == -1
    assert hp(p, 2, 16, 16, p, p, p, p, nul, nul, nul, nul) == -3
    assert L.faar_last_hip_error() == 0


def test_missing_library_is_a_loud_error(monkeypatch):
    monkeypatch.setattr(fb, "_lib", None)
    monkeypatch.setattr(fb, "LIB_PATH", "/nonexistent/libfaar.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        fb.lib()


def test_token_split_of_the_dw_gemm_is_sane():
    """faar_dw_split is pure host logic (the GEMM planner): 1..8 splits, at least 512 tokens per split, no
    empty split, and the workspace grows with it."""
    for O, K, T in [(2048, 2048, 4096), (512, 2048, 4096), (8192, 2048, 4096), (2048, 8192, 4096), (6144, 2048, 16384),
                    (1024, 2048, 16384), (256, 256, 64), (96, 80, 100), (16, 16, 1), (12288, 64, 2048)]:
        s = fb.faar_dw_split(O, K, T)
        Tp = fb.faar_padded_tokens(T)
        assert 1 <= s <= 16, (O, K, T, s)
        assert s == 1 or Tp // s >= 512, (O, K, T, s)
        assert fb.faar_workspace_bytes(fb.OP_LAYER_STEP, O, K, T) >= s * O * K * 4
    assert fb.faar_dw_split(0, 16, 8) == 0 and fb.faar_dw_split(16, 8, 8) == 0      # invalid shapes
    # small outputs with a long token axis split; large outputs do not
    assert fb.faar_dw_split(512, 2048, 4096) > 1
    assert fb.faar_dw_split(8192, 2048, 4096) == 1


def test_token_major_dw_gemm_choice_is_sane():
    """faar_dw_token_major is pure host logic: 0 where the token-major form does not apply, 256 x 256 tiles (1) beside other
    streams, and a 192-wide tile only for a step that has the device to itself and only where it saves rounds of the units."""
    assert fb.faar_dw_token_major(0, 16, 64) == 0 and fb.faar_dw_token_major(2048, 2048, 0) == 0    # invalid shapes
    assert fb.faar_dw_token_major(2048, 2048, 8192 + 32) == 0                                       # T not a multiple of 64
    assert fb.faar_dw_token_major(256, 256, 64) == 0                                                # too small for 256-wide tiles
    for O, K in [(2048, 2048), (6144, 2048), (2048, 6144)]:
        assert fb.faar_dw_token_major(O, K, 8192) == 1
    assert fb.faar_dw_token_major(6144, 2048, 8192, whole_device=True) == 2      # 192 tiles of 256 x 256, 256 of 192 x 256
    assert fb.faar_dw_token_major(2048, 6144, 8192, whole_device=True) == 3
    assert fb.faar_dw_token_major(2048, 2048, 8192, whole_device=True) == 1      # 64 tiles x 4 splits fill the device already


def test_batched_codec_calls_validate_every_descriptor_first():
    L = fb.lib()
    good = fb.faar_tensor(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 256)
    def batch(*ts):
        arr = (fb.faar_tensor * len(ts))(*ts)
        return arr, len(ts)
    ws = ctypes.c_void_p(0x9000)
    arr, n = batch(good, fb.faar_tensor(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 250))       # n % 16
    assert L.faar_quant_rtn_batch(arr, n, 1, 0, ws, 1 << 20, None) == -2
    arr, n = batch(good, fb.faar_tensor(0x1000, None, 0x3000, 0x4000, 0x5000, 256))          # missing tensor scale
    assert L.faar_harden_pack_batch(arr, n, 1, None) == -1
    arr, n = batch(fb.faar_tensor(0x1000, 0x2000, 0x3000, None, 0x5000, 256))                # V missing where it is used
    assert L.faar_init_v_batch(arr, n, 1, None) == -1
    assert L.faar_harden_pack_batch(arr, n, 1, None) == -1
    arr, n = batch(fb.faar_tensor(0x1004, 0x2000, 0x3000, 0x4000, 0x5000, 256))              # unaligned W
    assert L.faar_init_v_batch(arr, n, 1, None) == -6
    arr, n = batch(good)
    assert L.faar_quant_rtn_batch(arr, n, 1, 0, None, 0, None) == -4                         # workspace missing
    assert L.faar_quant_rtn_batch(arr, n, 5, 0, ws, 1 << 20, None) == -3
    assert L.faar_quant_rtn_batch(arr, 0, 1, 0, ws, 1 << 20, None) == -2
    assert L.faar_init_v_batch(None, 1, 1, None) == -1
    assert fb.faar_workspace_bytes(fb.OP_QUANT_RTN_BATCH, 16, 16) >= 48 * 64 * 4


def test_block_glue_calls_reject_bad_arguments_without_a_gpu():
    L = fb.lib()
    p, odd, nul = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004), None
    f = L.faar_linear_forward
    ws = fb.faar_workspace_bytes(fb.OP_LINEAR_FORWARD, 32, 32, 64)
    assert ws >= 32 * 32 * 2
    assert f(p, 1, 32, 32, p, p, nul, 1.0, p, nul, 64, p, p, ws, nul) == -1
    assert f(p, 5, 32, 32, p, p, p, 1.0, p, nul, 64, p, p, ws, nul) == -3
    assert f(p, 1, 32, 24, p, p, p, 1.0, p, nul, 64, p, p, ws, nul) == -2
    assert f(p, 1, 32, 32, p, p, p, 1.0, p, nul, 0, p, p, ws, nul) == -2
    assert f(p, 1, 32, 32, p, p, p, 0.0, p, nul, 64, p, p, ws, nul) == -6
    assert f(p, 1, 32, 32, p, p, p, 1.0, odd, nul, 64, p, p, ws, nul) == -6
    assert f(p, 1, 32, 32, p, p, p, 1.0, p, nul, 64, p, p, ws - 1, nul) == -4
    assert f(p, 1, 32, 32, p, p, p, 1.0, p, nul, 64, p, nul, 0, nul) == -4
    n = L.faar_rmsnorm_fwd
    assert n(p, 1, 4, 64, nul, 1e-6, p, p, nul) == -1
    assert n(p, 1, 4, 60, p, 1e-6, p, p, nul) == -2
    assert n(p, 1, 0, 64, p, 1e-6, p, p, nul) == -2
    assert n(p, 9, 4, 64, p, 1e-6, p, p, nul) == -3
    assert n(p, 1, 4, 64, p, -1.0, p, p, nul) == -6
    assert n(p, 1, 4, 64, p, float("nan"), p, p, nul) == -6
    assert n(odd, 1, 4, 64, p, 1e-6, p, p, nul) == -6
    b = L.faar_rmsnorm_bwd
    assert b(nul, nul, nul, p, 1, 4, 64, p, p, nul, p, nul) == -1
    assert b(p, nul, nul, p, 1, 4, 64, p, p, nul, nul, nul) == -1
    assert b(p, nul, nul, p, 1, 4, 12, p, p, nul, p, nul) == -2
    assert b(p, odd, nul, p, 1, 4, 64, p, p, nul, p, nul) == -6
    assert b(p, nul, odd, p, 1, 4, 64, p, p, nul, p, nul) == -6
    assert b(p, nul, nul, p, 1, 4, 64, p, p, odd, p, nul) == -6
    s = L.faar_silu_mul_fwd
    assert s(p, nul, 64, p, nul) == -1
    assert s(p, p, 60, p, nul) == -2
    assert s(p, p, 0, p, nul) == -2
    assert s(p, odd, 64, p, nul) == -6
    sb = L.faar_silu_mul_bwd
    assert sb(p, p, p, 64, p, nul, nul) == -1
    assert sb(p, p, p, 12, p, p, nul) == -2
    assert sb(p, p, p, 64, odd, p, nul) == -6
    o = L.faar_block_output_loss
    wsl = fb.faar_workspace_bytes(fb.OP_BLOCK_OUTPUT_LOSS, 64, 16, 4)
    assert wsl >= 8
    assert o(p, 1, p, p, 1, 4, 64, 1.0, nul, p, nul, p, wsl, nul) == -1
    assert o(p, 1, p, p, 4, 4, 64, 1.0, nul, p, p, p, wsl, nul) == -3
    assert o(p, 1, p, p, 1, 4, 20, 1.0, nul, p, p, p, wsl, nul) == -2
    assert o(p, 1, p, p, 1, 4, 64, float("inf"), nul, p, p, p, wsl, nul) == -6
    assert o(p, 1, p, p, 1, 4, 64, 1.0, odd, p, p, p, wsl, nul) == -6
    assert o(p, 1, p, p, 1, 4, 64, 1.0, nul, p, p, p, wsl - 1, nul) == -4
    assert o(p, 1, p, p, 1, 4, 64, 1.0, nul, p, p, nul, 0, nul) == -4


def test_attention_calls_reject_bad_arguments_without_a_gpu():
    L = fb.lib()
    p, odd, nul = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004), None
    r = L.faar_rope
    assert r(p, 64, 2, 64, p, nul, 32, 0, p, nul) == -1
    assert r(p, 64, 2, 24, p, p, 32, 0, p, nul) == -2          # dh % 16
    assert r(p, 0, 2, 64, p, p, 32, 0, p, nul) == -2
    assert r(p, 64, 2, 64, p, p, 0, 0, p, nul) == -2
    assert r(odd, 64, 2, 64, p, p, 32, 0, p, nul) == -6
    n_q, n_kv, dh, S, n_seq = 4, 2, 128, 64, 2
    wf = fb.faar_workspace_bytes(fb.OP_ATTENTION_FWD, n_q * dh, n_kv * dh, n_seq * S)
    wb = fb.faar_workspace_bytes(fb.OP_ATTENTION_BWD, n_q * dh, n_kv * dh, n_seq * S)
    assert wf >= n_kv * dh * 192 * 2 and wb >= (2 * n_q + n_kv) * dh * 192 * 2 + n_q * 128 * 4
    assert fb.faar_workspace_bytes(fb.OP_ATTENTION_FWD, n_q * dh, n_kv * dh, 0) == 0
    f = L.faar_attention_fwd
    assert f(p, p, nul, n_seq, S, n_q, n_kv, dh, 0.1, p, p, p, wf, nul) == -1
    assert f(p, p, p, n_seq, 48, n_q, n_kv, dh, 0.1, p, p, p, wf, nul) == -2        # S % 32
    assert f(p, p, p, n_seq, S, n_q, 3, dh, 0.1, p, p, p, wf, nul) == -2            # n_q % n_kv
    assert f(p, p, p, n_seq, S, n_q, n_kv, 96, 0.1, p, p, p, wf, nul) == -2         # dh
    assert f(p, p, p, 0, S, n_q, n_kv, dh, 0.1, p, p, p, wf, nul) == -2
    assert f(p, p, p, n_seq, S, n_q, n_kv, dh, 0.0, p, p, p, wf, nul) == -6
    assert f(p, odd, p, n_seq, S, n_q, n_kv, dh, 0.1, p, p, p, wf, nul) == -6
    assert f(p, p, p, n_seq, S, n_q, n_kv, dh, 0.1, p, p, p, wf - 1, nul) == -4
    assert f(p, p, p, n_seq, S, n_q, n_kv, dh, 0.1, p, p, nul, 0, nul) == -4
    b = L.faar_attention_bwd
    assert b(p, p, p, p, p, nul, n_seq, S, n_q, n_kv, dh, 0.1, p, p, p, p, wb, nul) == -1
    assert b(p, p, p, p, p, p, n_seq, S, n_q, n_kv, dh, 0.1, p, p, nul, p, wb, nul) == -1
    assert b(p, p, p, p, p, p, n_seq, 33, n_q, n_kv, dh, 0.1, p, p, p, p, wb, nul) == -2
    assert b(p, p, p, p, p, p, n_seq, S, n_q, n_kv, dh, float("nan"), p, p, p, p, wb, nul) == -6
    assert b(p, p, p, p, p, p, n_seq, S, n_q, n_kv, dh, 0.1, p, odd, p, p, wb, nul) == -6
    assert b(p, p, p, p, p, p, n_seq, S, n_q, n_kv, dh, 0.1, p, p, p, p, wb - 1, nul) == -4
    a = L.faar_residual_add
    assert a(p, 1, nul, 64, p, nul) == -1
    assert a(p, 3, p, 64, p, nul) == -3
    assert a(p, 1, p, 60, p, nul) == -2
    assert a(p, 1, odd, 64, p, nul) == -6


def test_block_joint_step_validates_its_description_without_a_gpu():
    L = fb.lib()
    p, nul = 0x1000, None

    def block(**kw):
        b = fb.faar_block()
        b.n_seq, b.S, b.D, b.n_q, b.n_kv, b.dh, b.F = 2, 64, 256, 4, 2, 64, 512
        b.eps, b.attn_scale, b.wdt = 1e-6, 0.0, 1
        b.g_attn = b.g_mlp = b.cos_t = b.sin_t = p
        for i in range(7):
            for f, _ in fb.faar_block_linear._fields_:
                setattr(b.lin[i], f, p)
        for k, v in kw.items():
            setattr(b, k, v)
        return b

    good = block()
    n = L.faar_block_workspace_bytes(ctypes.byref(good))
    T = 128
    assert n > T * (6 * 512 + 12 * 256) * 2                     # at least the activations it keeps
    assert L.faar_block_workspace_bytes(ctypes.byref(block(S=48))) == 0
    assert L.faar_block_workspace_bytes(ctypes.byref(block(dh=96))) == 0
    assert L.faar_block_workspace_bytes(ctypes.byref(block(n_kv=3))) == 0
    assert L.faar_block_workspace_bytes(ctypes.byref(block(D=100))) == 0
    assert L.faar_block_workspace_bytes(ctypes.byref(block(g_q=p))) == 0      # g_q without g_k
    opt = fb.faar_adam(1e-3, 0.9, 0.999, 1e-8, 1)
    ws = ctypes.c_void_p(0x10000)
    f = L.faar_block_joint_step
    P = ctypes.c_void_p(p)
    assert f(nul, P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -1
    assert f(ctypes.byref(good), nul, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -1
    assert f(ctypes.byref(good), P, P, 1.0, 4.0, 0.01, nul, P, P, ws, n, nul) == -1
    assert f(ctypes.byref(block(g_mlp=nul)), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -1
    bad_lin = block()
    bad_lin.lin[3].icodes = nul
    assert f(ctypes.byref(bad_lin), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -1
    assert f(ctypes.byref(block(S=40)), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -2
    assert f(ctypes.byref(block(wdt=7)), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -3
    assert f(ctypes.byref(good), P, P, 1.0, 0.0, 0.01, ctypes.byref(opt), P, P, ws, n, nul) == -6
    assert f(ctypes.byref(good), P, P, 1.0, 4.0, 0.01, ctypes.byref(fb.faar_adam(1e-3, 0.9, 0.999, 1e-8, 0)), P, P, ws, n, nul) == -6
    assert f(ctypes.byref(good), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ctypes.c_void_p(0x10010), n, nul) == -6
    assert f(ctypes.byref(good), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, ws, n - 1, nul) == -4
    assert f(ctypes.byref(good), P, P, 1.0, 4.0, 0.01, ctypes.byref(opt), P, P, nul, 0, nul) == -4


def test_gram_form_calls_reject_bad_arguments_without_a_gpu():
    L = fb.lib()
    P, nul = ctypes.c_void_p(0x1000), None
    O, K, T = 128, 256, 300
    n_prep = L.faar_workspace_bytes(fb.OP_GRAM_PREPARE, K, K, T, 0)
    n_step = L.faar_workspace_bytes(fb.OP_LAYER_STEP_GRAM, O, K, 1, 0)
    assert n_prep >= K * K * 4 and n_prep % (K * K * 4) == 0          # whole float32 partial matrices
    assert n_step > O * K * (2 + 4)                                   # W_q - W in bf16 and at least one float32 product
    assert L.faar_workspace_bytes(fb.OP_GRAM_PREPARE, K, 100, T, 0) == 0   # K not a multiple of 16
    ws = ctypes.c_void_p(0x10000)
    g = L.faar_gram_prepare
    assert g(nul, K, T, P, P, ws, n_prep, nul) == -1
    assert g(P, K, T, P, nul, ws, n_prep, nul) == -1
    assert g(P, 100, T, P, P, ws, n_prep, nul) == -2
    assert g(P, K, 0, P, P, ws, n_prep, nul) == -2
    assert g(ctypes.c_void_p(0x1008), K, T, P, P, ws, n_prep, nul) == -6
    assert g(P, K, T, P, P, ws, n_prep - 1, nul) == -4
    opt = fb.faar_adam(1e-3, 0.9, 0.999, 1e-8, 1)
    f = L.faar_layer_step_gram

    def call(W=P, wdt=1, O_=O, K_=K, H=P, cn=P, gram=P, lo=P, beta=4.0, beta_next=0.0, o=opt, flags=0, w=ws, n=n_step):
        return f(W, wdt, O_, K_, P, P, P, P, P, nul, P, H, cn, gram, lo, beta, beta_next, 0.01, 1.0,
                 ctypes.byref(o) if o is not None else nul, P, flags, w, n, nul)

    assert call(W=nul) == -1 and call(H=nul) == -1 and call(cn=nul) == -1 and call(gram=nul) == -1 and call(lo=nul) == -1
    assert call(o=None) == -1
    assert call(wdt=9) == -3
    assert call(K_=100) == -2 and call(O_=0) == -2
    assert call(beta=0.0) == -6 and call(beta_next=-1.0) == -6
    assert call(flags=fb.FAAR_STEP_JOINT) == -6 and call(flags=4) == -6      # only FAAR_WS_FORWARD_READY is meaningful here
    assert call(o=fb.faar_adam(1e-3, 1.0, 0.999, 1e-8, 1)) == -6
    assert call(cn=ctypes.c_void_p(0x1004)) == -6
    assert call(n=n_step - 1) == -4 and call(w=nul, n=0) == -4


def test_timing_hook_ring_validates_its_arguments_without_a_gpu():
    L = fb.lib()
    ev = (ctypes.c_void_p * 8)(*[0x1000 + 16 * i for i in range(8)])
    assert L.faar_time_kernel_ring(fb.K_GEMM_DW, ev, 4) == 0
    assert L.faar_time_kernel_count() == 0
    assert L.faar_time_kernel_ring(fb.K_GEMM_DW, ev, 0) == -6 and L.faar_time_kernel_ring(fb.K_GEMM_DW, ev, 4097) == -6
    assert L.faar_time_kernel_ring(fb.K_GEMM_DW, None, 4) == -6
    assert L.faar_time_kernel_ring(99, ev, 4) == -6 and L.faar_time_kernel_ring(fb.K_GEMM_C, ev, 4) == -6
    holes = (ctypes.c_void_p * 8)(*[0x1000, 0, 0x1020, 0x1030, 0x1040, 0x1050, 0x1060, 0x1070])
    assert L.faar_time_kernel_ring(fb.K_GEMM_DW, holes, 4) == -6
    assert L.faar_time_kernel_ring(fb.K_NONE, None, 0) == 0       # off; the old single-pair form still works
    assert L.faar_time_kernel(fb.K_GEMM_GRAM, ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1010)) == 0
    assert L.faar_time_kernel(fb.K_NONE, None, None) == 0
