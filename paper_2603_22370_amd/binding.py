"""ctypes binding of libfaar.so: same entry-point names as include/faar.h, argument marshalling
only.  torch is used for device memory and streams; every step of the method runs in the HIP
kernels behind the C ABI.  There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os
from ctypes import c_float, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfaar.so")

FAAR_F32, FAAR_BF16 = 0, 1
FAAR_SGLOBAL_GIVEN, FAAR_EMIT_DELTA, FAAR_WS_CHAINED, FAAR_WS_FORWARD_READY, FAAR_DQ_IN_UNITS = 1, 2, 4, 8, 16
FAAR_WS_GRADIENT_CONSTANT = 32
FAAR_STEP_JOINT = 64
FAAR_STEP_WHOLE_DEVICE = 256
OP_QUANT_RTN, OP_INIT_V, OP_SOFTQUANT, OP_LAYER_PREPARE, OP_LAYER_STEP, OP_HARDEN_PACK, OP_STAGE2_LOSSES, OP_QUANT_RTN_BATCH, OP_LINEAR_FORWARD, OP_BLOCK_OUTPUT_LOSS, OP_ATTENTION_FWD, OP_ATTENTION_BWD, OP_GRAM_PREPARE, OP_LAYER_STEP_GRAM = range(14)
ERRORS = {-1: "FAAR_E_NULL", -2: "FAAR_E_SHAPE", -3: "FAAR_E_DTYPE", -4: "FAAR_E_WORKSPACE",
          -5: "FAAR_E_HIP", -6: "FAAR_E_ARG", -7: "FAAR_E_UNSUPPORTED"}


class FaarError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = f" (hipError_t {lib().faar_last_hip_error()})" if code == -5 else ""
        super().__init__(f"{where}: {ERRORS.get(code, code)}{detail}")


class faar_tensor(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("s_global", c_void_p), ("scales", c_void_p), ("V", c_void_p), ("codes", c_void_p),
                ("n", c_int64)]


class faar_adam(ctypes.Structure):
    _fields_ = [("lr", c_float), ("beta1", c_float), ("beta2", c_float), ("eps", c_float), ("t", c_int32)]


class faar_block_linear(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("s_global", c_void_p), ("scales", c_void_p), ("icodes", c_void_p), ("V", c_void_p),
                ("adam_m", c_void_p), ("adam_u", c_void_p), ("losses", c_void_p)]


BLOCK_SLOTS = ("q", "k", "v", "o", "gate", "up", "down")


class faar_block(ctypes.Structure):
    _fields_ = [("n_seq", c_int64), ("S", c_int64), ("D", c_int64), ("n_q", c_int64), ("n_kv", c_int64), ("dh", c_int64),
                ("F", c_int64), ("eps", c_float), ("attn_scale", c_float), ("wdt", c_int), ("g_attn", c_void_p),
                ("g_mlp", c_void_p), ("g_q", c_void_p), ("g_k", c_void_p), ("cos_t", c_void_p), ("sin_t", c_void_p),
                ("lin", faar_block_linear * 7)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (python -m paper_2603_22370_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build(); "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.faar_version.restype = c_int
        L.faar_last_hip_error.restype = c_int
        L.faar_workspace_bytes.restype = c_size_t
        L.faar_workspace_bytes.argtypes = [c_int, c_int64, c_int64, c_int64, c_uint32]
        L.faar_time_kernel.restype = c_int
        L.faar_time_kernel.argtypes = [c_int, c_void_p, c_void_p]
        L.faar_time_kernel_ring.restype = c_int
        L.faar_time_kernel_ring.argtypes = [c_int, ctypes.POINTER(c_void_p), c_int]
        L.faar_time_kernel_count.restype = c_int64
        L.faar_time_kernel_count.argtypes = []
        L.faar_dw_split.restype = c_int
        L.faar_dw_split.argtypes = [c_int64, c_int64, c_int64]
        L.faar_gemm_plan.restype = c_int
        L.faar_gemm_plan.argtypes = [c_int, c_int64, c_int64, c_int64, ctypes.POINTER(c_int32)]
        L.faar_gemm_probe.restype = c_int
        L.faar_gemm_probe.argtypes = [c_int, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_int64, c_void_p,
                                      ctypes.POINTER(c_int32), c_void_p]
        L.faar_dw_token_major.restype = c_int
        L.faar_dw_token_major.argtypes = [c_int64, c_int64, c_int64, c_uint32]
        L.faar_padded_tokens.restype = c_int64
        L.faar_padded_tokens.argtypes = [c_int64]
        L.faar_quant_rtn.restype = c_int
        L.faar_quant_rtn.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_uint32, c_void_p, c_size_t, c_void_p]
        L.faar_init_v.restype = c_int
        L.faar_init_v.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        L.faar_softquant_fwd_bwd.restype = c_int
        L.faar_softquant_fwd_bwd.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_float,
                                             c_void_p, c_void_p, c_float, c_void_p, c_void_p, c_uint32, c_void_p,
                                             c_size_t, c_void_p]
        L.faar_quant_rtn_batch.restype = c_int
        L.faar_quant_rtn_batch.argtypes = [ctypes.POINTER(faar_tensor), c_int64, c_int, c_uint32, c_void_p, c_size_t, c_void_p]
        L.faar_init_v_batch.restype = c_int
        L.faar_init_v_batch.argtypes = [ctypes.POINTER(faar_tensor), c_int64, c_int, c_void_p]
        L.faar_harden_pack_batch.restype = c_int
        L.faar_harden_pack_batch.argtypes = [ctypes.POINTER(faar_tensor), c_int64, c_int, c_void_p]
        L.faar_softquant_fwd_bwd_static.restype = c_int
        L.faar_softquant_fwd_bwd_static.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_float,
                                                    c_void_p, c_void_p, c_float, c_void_p, c_void_p, c_uint32, c_void_p]
        L.faar_layer_prepare.restype = c_int
        L.faar_layer_prepare.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_void_p, c_int, c_int64, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_void_p, c_size_t, c_void_p]
        L.faar_layer_step.restype = c_int
        L.faar_layer_step.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_int64, c_void_p, c_void_p,
                                      c_float, c_float, c_float, c_float, ctypes.POINTER(faar_adam), c_void_p,
                                      c_uint32, c_void_p, c_size_t, c_void_p]
        L.faar_gram_prepare.restype = c_int
        L.faar_gram_prepare.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_layer_step_gram.restype = c_int
        L.faar_layer_step_gram.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                           c_float, c_float, c_float, c_float, ctypes.POINTER(faar_adam), c_void_p,
                                           c_uint32, c_void_p, c_size_t, c_void_p]
        L.faar_linear_forward.restype = c_int
        L.faar_linear_forward.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_float, c_void_p,
                                          c_void_p, c_int64, c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_rmsnorm_fwd.restype = c_int
        L.faar_rmsnorm_fwd.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_float, c_void_p, c_void_p, c_void_p]
        L.faar_rmsnorm_bwd.restype = c_int
        L.faar_block_workspace_bytes.restype = c_size_t
        L.faar_block_workspace_bytes.argtypes = [ctypes.POINTER(faar_block)]
        L.faar_block_joint_step.restype = c_int
        L.faar_block_joint_step.argtypes = [ctypes.POINTER(faar_block), c_void_p, c_void_p, c_float, c_float, c_float,
                                            ctypes.POINTER(faar_adam), c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_residual_add.restype = c_int
        L.faar_residual_add.argtypes = [c_void_p, c_int, c_void_p, c_int64, c_void_p, c_void_p]
        L.faar_rope.restype = c_int
        L.faar_rope.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_int64, ctypes.c_int32, c_void_p, c_void_p]
        L.faar_attention_fwd.restype = c_int
        L.faar_attention_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int64, c_int64, c_float, c_void_p,
                                         c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_attention_bwd.restype = c_int
        L.faar_attention_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64,
                                         c_int64, c_int64, c_float, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_rmsnorm_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p,
                                       c_void_p, c_void_p]
        L.faar_silu_mul_fwd.restype = c_int
        L.faar_silu_mul_fwd.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_void_p]
        L.faar_silu_mul_bwd.restype = c_int
        L.faar_silu_mul_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_void_p, c_void_p, c_void_p]
        L.faar_block_output_loss.restype = c_int
        L.faar_block_output_loss.argtypes = [c_void_p, c_int, c_void_p, c_void_p, c_int, c_int64, c_int64, c_float, c_void_p,
                                             c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_stochastic_v.restype = c_int
        L.faar_stochastic_v.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, ctypes.c_ulonglong, c_uint32,
                                        c_void_p, c_void_p]
        L.faar_hardened_loss.restype = c_int
        L.faar_hardened_loss.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_void_p, c_int64, c_float, c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_stage2_losses.restype = c_int
        L.faar_stage2_losses.argtypes = [c_void_p, c_void_p, c_int, c_int64, c_int64, c_float, c_float, c_void_p, c_void_p,
                                         c_int, c_int64, c_float, c_void_p, c_int64, c_float, c_float, c_void_p, c_void_p,
                                         c_void_p, c_void_p, c_size_t, c_void_p]
        L.faar_harden_pack.restype = c_int
        L.faar_harden_pack.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                       c_void_p, c_void_p, c_void_p, c_void_p]
        _lib = L
    return _lib


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FAAR_F32
    if t.dtype == torch.bfloat16:
        return FAAR_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def _check(rc: int, where: str):
    if rc != 0:
        raise FaarError(rc, where)


def faar_workspace_bytes(op: int, O: int, K: int, T: int = 0, flags: int = 0) -> int:
    return int(lib().faar_workspace_bytes(op, O, K, T, flags))


K_NONE, K_SOFTQUANT_FWD, K_GEMM_RESIDUAL, K_GEMM_DW, K_GEMM_DX, K_BWD_ADAM, K_QUANT_RTN, K_INIT_V, K_HARDEN_PACK, K_STAGE2_KL = range(10)


def faar_time_kernel(which: int, start_event=None, stop_event=None) -> None:
    """start_event / stop_event: raw hipEvent_t handles (integers)."""
    _check(lib().faar_time_kernel(which, c_void_p(start_event), c_void_p(stop_event)), "faar_time_kernel")


def faar_time_kernel_ring(which: int, events) -> None:
    """events: sequence of raw hipEvent_t handles (start 0, stop 0, start 1, ...); empty with K_NONE."""
    arr = (c_void_p * max(1, len(events)))(*events)
    _check(lib().faar_time_kernel_ring(which, arr, len(events) // 2), "faar_time_kernel_ring")


def faar_time_kernel_count() -> int:
    return int(lib().faar_time_kernel_count())


def faar_dw_split(O: int, K: int, T: int) -> int:
    return int(lib().faar_dw_split(O, K, T))


K_GEMM_C, K_GEMM_FWD, K_ATTENTION_FWD, K_ATTENTION_BWD, K_GEMM_GRAM = 10, 11, 12, 13, 14
GEMM_KINDS = ("generic", "L", "M", "S", "L64", "M64")


def faar_gemm_plan(which: int, O: int, K: int, T: int):
    """-> (variant name, tile rows, tile columns, contraction splits) of one GEMM of a layer of these sizes."""
    out = (c_int32 * 4)()
    _check(lib().faar_gemm_plan(which, O, K, T, out), "faar_gemm_plan")
    return GEMM_KINDS[out[0]], int(out[1]), int(out[2]), int(out[3])


PROBE_FULL, PROBE_MFMA_ONLY, PROBE_DMA_ONLY = 0, 1, 2
PROBE_TOKEN_MAJOR, PROBE_TOKEN_MAJOR_192 = 4, 12    # added to a mode / a mode of its own (whole loop on 192-wide tiles)
_probe_buffers = {}


def faar_gemm_probe(mode: int, A, B):
    """Runs one measurement variant of the GEMM main loop on A [M, Kd] x B [N, Kd]^T (bf16).
    -> (clocks int64 [items, 2]: shader-clock cycles and 100 MHz ticks per work item, variant name)."""
    _dev(A, B)
    M, Kd = A.shape
    N = B.shape[0]
    cap = 1 << 16
    if A.device not in _probe_buffers:
        _probe_buffers[A.device] = (torch.zeros((cap, 2), dtype=torch.int64, device=A.device),
                                    torch.zeros(1, dtype=torch.float32, device=A.device))
    clocks, sink = _probe_buffers[A.device]
    info = (c_int32 * 2)()
    _check(lib().faar_gemm_probe(mode, M, N, Kd, _ptr(A), _ptr(B), _ptr(clocks), cap, _ptr(sink), info, _stream()),
           "faar_gemm_probe")
    return clocks[:info[0]], GEMM_KINDS[info[1]]


def faar_dw_token_major(O: int, K: int, T: int, whole_device: bool = False) -> int:
    """0: the dW GEMM of such a step needs transposed operands; else the tile shape of its token-major form
    (1: 256 x 256; with whole_device also 2: 192 x 256, 3: 256 x 192)."""
    return int(lib().faar_dw_token_major(O, K, T, FAAR_STEP_WHOLE_DEVICE if whole_device else 0))


def faar_padded_tokens(T: int) -> int:
    return int(lib().faar_padded_tokens(T))


def _workspace(op, O, K, T=0, flags=0, device="cuda"):
    n = faar_workspace_bytes(op, O, K, T, flags)
    if n == 0:
        raise FaarError(-2, "faar_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def faar_quant_rtn(W, s_global=None, want_dq=False, ws=None, dq_in_units=False):
    """-> (s_global[1] f32, scales [O,K/16] u8, codes [O,K/2] u8, W_dq or None).
    dq_in_units: W_dq = sign * node * block scale (exact), to be multiplied by s_global by its consumer."""
    _dev(W, s_global, ws)
    O, K = W.shape
    flags = 0
    if s_global is None:
        s_global = torch.empty(1, dtype=torch.float32, device=W.device)
    else:
        flags |= FAAR_SGLOBAL_GIVEN
    if dq_in_units:
        flags |= FAAR_DQ_IN_UNITS
    scales = torch.empty((O, K // 16), dtype=torch.uint8, device=W.device)
    codes = torch.empty((O, K // 2), dtype=torch.uint8, device=W.device)
    W_dq = torch.empty_like(W) if want_dq else None
    ws = _workspace(OP_QUANT_RTN, O, K, device=W.device) if ws is None else ws
    _check(lib().faar_quant_rtn(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(codes), _ptr(W_dq),
                                flags, _ptr(ws), ws.numel(), _stream()), "faar_quant_rtn")
    return s_global, scales, codes, W_dq


def tensor_batch(Ws, s_globals, scales, Vs=None, codes=None):
    """A host array of faar_tensor descriptors over lists of device tensors (one entry per weight tensor; Vs / codes
    may be None where the batched call does not use them).  Build it once and reuse it: the calls only read it."""
    n = len(Ws)
    items = (faar_tensor * n)()
    dt = _dt(Ws[0])
    for k in range(n):
        _dev(Ws[k], s_globals[k], scales[k], None if Vs is None else Vs[k], None if codes is None else codes[k])
        if _dt(Ws[k]) != dt:
            raise TypeError("all tensors of a batch share one storage type")
        items[k] = faar_tensor(Ws[k].data_ptr(), s_globals[k].data_ptr(), scales[k].data_ptr(),
                               None if Vs is None else Vs[k].data_ptr(), None if codes is None else codes[k].data_ptr(),
                               Ws[k].numel())
    return items, dt


def faar_quant_rtn_batch(items, dt, ws, s_global_given=False):
    _check(lib().faar_quant_rtn_batch(items, len(items), dt, FAAR_SGLOBAL_GIVEN if s_global_given else 0, _ptr(ws),
                                      0 if ws is None else ws.numel(), _stream()), "faar_quant_rtn_batch")


def faar_init_v_batch(items, dt):
    _check(lib().faar_init_v_batch(items, len(items), dt, _stream()), "faar_init_v_batch")


def faar_harden_pack_batch(items, dt):
    _check(lib().faar_harden_pack_batch(items, len(items), dt, _stream()), "faar_harden_pack_batch")


def faar_init_v(W, s_global, scales, want_floor_codes=False):
    """-> (V [O,K] f32, floor_codes [O,K/2] u8 or None)."""
    _dev(W, s_global, scales)
    O, K = W.shape
    V = torch.empty((O, K), dtype=torch.float32, device=W.device)
    fc = torch.empty((O, K // 2), dtype=torch.uint8, device=W.device) if want_floor_codes else None
    _check(lib().faar_init_v(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), _ptr(fc), _stream()),
           "faar_init_v")
    return V, fc


def faar_softquant_fwd_bwd(W, s_global, scales, V, beta, dWt=None, lambda_round=0.0, emit_delta=False, ws=None):
    """-> (Wt bf16 [O,K], dV f32 or None, round_loss f32[1] or None)."""
    _dev(W, s_global, scales, V, dWt, ws)
    O, K = W.shape
    Wt = torch.empty((O, K), dtype=torch.bfloat16, device=W.device)
    dV = torch.empty((O, K), dtype=torch.float32, device=W.device) if dWt is not None else None
    rl = torch.empty(1, dtype=torch.float32, device=W.device) if dWt is not None else None
    ws = _workspace(OP_SOFTQUANT, O, K, device=W.device) if ws is None else ws
    flags = FAAR_EMIT_DELTA if emit_delta else 0
    _check(lib().faar_softquant_fwd_bwd(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), float(beta),
                                        _ptr(Wt), _ptr(dWt), float(lambda_round), _ptr(dV), _ptr(rl), flags,
                                        _ptr(ws), ws.numel(), _stream()), "faar_softquant_fwd_bwd")
    return Wt, dV, rl


def faar_softquant_fwd_bwd_static(W, s_global, scales, V, beta, Wt, dWt=None, lambda_round=0.0, dV=None, round_loss=None,
                                  emit_delta=False):
    """The same operation through the entry point that allocates nothing: outputs (Wt bf16 [O,K], and with dWt also
    dV f32 [O,K], round_loss f32[1]) are the caller's; no workspace."""
    _dev(W, s_global, scales, V, Wt, dWt, dV, round_loss)
    O, K = W.shape
    flags = FAAR_EMIT_DELTA if emit_delta else 0
    _check(lib().faar_softquant_fwd_bwd_static(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), float(beta),
                                               _ptr(Wt), _ptr(dWt), float(lambda_round), _ptr(dV), _ptr(round_loss), flags,
                                               _stream()), "faar_softquant_fwd_bwd_static")


def faar_layer_prepare(W, s_global, scales, Xq, Y_fp, ws=None, x_scale=None, gradient_constant=False):
    """-> (Xt bf16 [K, Tp], C f32 [ceil(T/4), O, 4] (tokens interleaved in groups of four), icodes u8 [O, K/2]);
    with gradient_constant also -> (..., H f32 [O, K] = C^T Xq, c_norm2 f64[1] = ||C||^2)."""
    _dev(W, s_global, scales, Xq, Y_fp, ws, x_scale)
    O, K = W.shape
    T = Xq.shape[0]
    if Xq.dtype != torch.bfloat16 or Xq.shape[1] != K or (Y_fp is not None and tuple(Y_fp.shape) != (T, O)):
        raise ValueError("Xq must be bf16 [T,K]; Y_fp must be [T,O]")
    Xt = torch.empty((K, faar_padded_tokens(T)), dtype=torch.bfloat16, device=W.device)
    # row groups of 4 interleaved; none without a reference output (a layer that is only stepped jointly)
    C = torch.empty(((T + 3) // 4, O, 4), dtype=torch.float32, device=W.device) if Y_fp is not None else None
    icodes = torch.empty((O, K // 2), dtype=torch.uint8, device=W.device)
    H = torch.empty((O, K), dtype=torch.float32, device=W.device) if gradient_constant else None
    cn = torch.empty(1, dtype=torch.float64, device=W.device) if gradient_constant else None
    flags = FAAR_WS_GRADIENT_CONSTANT if gradient_constant else 0
    ws = _workspace(OP_LAYER_PREPARE, O, K, T, flags, device=W.device) if ws is None else ws
    _check(lib().faar_layer_prepare(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(Xq), _ptr(x_scale),
                                    _ptr(Y_fp), FAAR_BF16 if Y_fp is None else _dt(Y_fp), T, _ptr(Xt), _ptr(C), _ptr(icodes), _ptr(H),
                                    _ptr(cn), _ptr(ws),
                                    ws.numel(), _stream()),
           "faar_layer_prepare")
    return (Xt, C, icodes, H, cn) if gradient_constant else (Xt, C, icodes)


def faar_layer_step(W, s_global, scales, V, adam_m, adam_v, Xq, Xt, C, icodes, beta, lambda_round, mse_scale,
                    lr, beta1, beta2, eps, t, losses, ws, dY_ext=None, dX=None, beta_next=0.0, forward_ready=False,
                    x_scale=None, H=None, c_norm2=None, joint=False, whole_device=False):
    """One step in place on (V, adam_m, adam_v); losses f32[3] receives (L_mse, L_round, L).
    beta_next > 0 leaves the next step's forward outputs in ws; forward_ready=True consumes them.
    H, c_norm2: the gradient constant of faar_layer_prepare(gradient_constant=True), or None.
    joint: a Stage-2-style step (dY_ext required; no local loss; Xt is rewritten from Xq; C may be None).
    whole_device: nothing else runs on the device beside the step (tiles that fill every compute unit)."""
    _dev(W, s_global, scales, V, adam_m, adam_v, Xq, Xt, C, icodes, losses, ws, dY_ext, dX, x_scale, H, c_norm2)
    O, K = W.shape
    T = Xq.shape[0]
    opt = faar_adam(float(lr), float(beta1), float(beta2), float(eps), int(t))
    _check(lib().faar_layer_step(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), _ptr(adam_m),
                                 _ptr(adam_v), _ptr(Xq), _ptr(x_scale), _ptr(Xt), _ptr(C), _ptr(icodes), _ptr(H),
                                 _ptr(c_norm2), T, _ptr(dY_ext), _ptr(dX),
                                 float(beta), float(beta_next), float(lambda_round), float(mse_scale),
                                 ctypes.byref(opt), _ptr(losses),
                                 (FAAR_WS_FORWARD_READY if forward_ready else 0) | (FAAR_STEP_JOINT if joint else 0)
                                 | (FAAR_STEP_WHOLE_DEVICE if whole_device else 0),
                                 _ptr(ws), ws.numel(), _stream()), "faar_layer_step")


def faar_gram_prepare(Xt, T, ws=None):
    """Xt bf16 [K, Tp] as written by faar_layer_prepare -> (gram bf16 [K, K] = bf16(Xq^T Xq), gram_lo f32 [K])."""
    _dev(Xt, ws)
    K = Xt.shape[0]
    if Xt.dtype != torch.bfloat16 or Xt.shape[1] != faar_padded_tokens(T):
        raise ValueError("Xt must be the bf16 [K, padded T] transpose written by faar_layer_prepare")
    gram = torch.empty((K, K), dtype=torch.bfloat16, device=Xt.device)
    gram_lo = torch.empty(K, dtype=torch.float32, device=Xt.device)
    ws = _workspace(OP_GRAM_PREPARE, K, K, T, device=Xt.device) if ws is None else ws
    _check(lib().faar_gram_prepare(_ptr(Xt), K, T, _ptr(gram), _ptr(gram_lo), _ptr(ws), ws.numel(), _stream()),
           "faar_gram_prepare")
    return gram, gram_lo


def faar_layer_step_gram(W, s_global, scales, V, adam_m, adam_v, icodes, H, c_norm2, gram, gram_lo, beta, lambda_round,
                         mse_scale, lr, beta1, beta2, eps, t, losses, ws, beta_next=0.0, forward_ready=False, x_scale=None):
    """faar_layer_step in its Gram-matrix form (constant activations): in place on (V, adam_m, adam_v); losses f32[3]."""
    _dev(W, s_global, scales, V, adam_m, adam_v, icodes, H, c_norm2, gram, gram_lo, losses, ws, x_scale)
    O, K = W.shape
    opt = faar_adam(float(lr), float(beta1), float(beta2), float(eps), int(t))
    _check(lib().faar_layer_step_gram(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), _ptr(adam_m), _ptr(adam_v),
                                      _ptr(x_scale), _ptr(icodes), _ptr(H), _ptr(c_norm2), _ptr(gram), _ptr(gram_lo),
                                      float(beta), float(beta_next), float(lambda_round), float(mse_scale), ctypes.byref(opt),
                                      _ptr(losses), FAAR_WS_FORWARD_READY if forward_ready else 0, _ptr(ws), ws.numel(),
                                      _stream()), "faar_layer_step_gram")


def layer_step_gram_workspace(O, K, device="cuda"):
    return _workspace(OP_LAYER_STEP_GRAM, O, K, 1, device=device)


def layer_step_workspace(O, K, T, chained=False, device="cuda"):
    return _workspace(OP_LAYER_STEP, O, K, T, FAAR_WS_CHAINED if chained else 0, device=device)


def faar_harden_pack(W, s_global, scales, V, want_decisions=False, want_final=False, want_flips=False):
    """-> (codes [O,K/2] u8, decisions [O*K/8] u8 or None, W_final or None, flip_count i64[1] or None)."""
    _dev(W, s_global, scales, V)
    O, K = W.shape
    codes = torch.empty((O, K // 2), dtype=torch.uint8, device=W.device)
    dec = torch.empty(O * K // 8, dtype=torch.uint8, device=W.device) if want_decisions else None
    Wf = torch.empty_like(W) if want_final else None
    flips = torch.zeros(1, dtype=torch.int64, device=W.device) if want_flips else None
    _check(lib().faar_harden_pack(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), _ptr(codes),
                                  _ptr(dec), _ptr(Wf), _ptr(flips), _stream()), "faar_harden_pack")
    return codes, dec, Wf, flips


def faar_stage2_losses(Z_fp, Z_q, tau, H_fp, H_q, kl_scale=1.0, mse_scale=1.0, round_losses=None, lambda_kl=1.0,
                       lambda_round=0.0, want_grads=True, ws=None):
    """-> (losses f32[4] = (L_KL, L_MSE, L_round, L), dZ_q or None, dH_q or None)."""
    _dev(Z_fp, Z_q, H_fp, H_q, round_losses, ws)
    T, vocab = Z_fp.shape
    D = H_fp.shape[1]
    if Z_q.shape != Z_fp.shape or Z_q.dtype != Z_fp.dtype or H_q.shape != H_fp.shape or H_q.dtype != H_fp.dtype:
        raise ValueError("Z_fp / Z_q and H_fp / H_q must agree in shape and dtype")
    losses = torch.empty(4, dtype=torch.float32, device=Z_fp.device)
    dZ = torch.empty_like(Z_q) if want_grads else None
    dH = torch.empty_like(H_q) if want_grads else None
    ws = _workspace(OP_STAGE2_LOSSES, vocab, D, T, device=Z_fp.device) if ws is None else ws
    n_layers = 0 if round_losses is None else int(round_losses.numel())
    _check(lib().faar_stage2_losses(_ptr(Z_fp), _ptr(Z_q), _dt(Z_fp), T, vocab, float(tau), float(kl_scale), _ptr(H_fp),
                                    _ptr(H_q), _dt(H_fp), D, float(mse_scale), _ptr(round_losses), n_layers,
                                    float(lambda_kl), float(lambda_round), _ptr(dZ), _ptr(dH), _ptr(losses), _ptr(ws),
                                    ws.numel(), _stream()), "faar_stage2_losses")
    return losses, dZ, dH


def faar_linear_forward(W, s_global, scales, V, beta, Xq, x_scale=None, ws=None, out=None):
    """-> Y bf16 [T, O] = x_scale * Xq W_q(V)^T."""
    _dev(W, s_global, scales, V, Xq, x_scale, ws, out)
    O, K = W.shape
    T = Xq.shape[0]
    Y = torch.empty((T, O), dtype=torch.bfloat16, device=W.device) if out is None else out
    ws = _workspace(OP_LINEAR_FORWARD, O, K, T, device=W.device) if ws is None else ws
    _check(lib().faar_linear_forward(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), float(beta), _ptr(Xq),
                                     _ptr(x_scale), T, _ptr(Y), _ptr(ws), ws.numel(), _stream()), "faar_linear_forward")
    return Y


def faar_rmsnorm_fwd(x, g, eps):
    """-> (h bf16 [T, D], rstd f32 [T])."""
    _dev(x, g)
    T, D = x.shape
    h = torch.empty((T, D), dtype=torch.bfloat16, device=x.device)
    rstd = torch.empty(T, dtype=torch.float32, device=x.device)
    _check(lib().faar_rmsnorm_fwd(_ptr(x), _dt(x), T, D, _ptr(g), float(eps), _ptr(h), _ptr(rstd), _stream()), "faar_rmsnorm_fwd")
    return h, rstd


def faar_rmsnorm_bwd(dh1, x, g, rstd, dh2=None, d_res=None, dh3=None):
    """-> dx bf16 [T, D]."""
    _dev(dh1, dh2, dh3, x, g, rstd, d_res)
    T, D = x.shape
    dx = torch.empty((T, D), dtype=torch.bfloat16, device=x.device)
    _check(lib().faar_rmsnorm_bwd(_ptr(dh1), _ptr(dh2), _ptr(dh3), _ptr(x), _dt(x), T, D, _ptr(g), _ptr(rstd), _ptr(d_res),
                                  _ptr(dx), _stream()), "faar_rmsnorm_bwd")
    return dx


def faar_residual_add(x, d, out=None):
    """-> y = x + d, bf16 like d."""
    _dev(x, d, out)
    y = torch.empty_like(d) if out is None else out
    _check(lib().faar_residual_add(_ptr(x), _dt(x), _ptr(d), d.numel(), _ptr(y), _stream()), "faar_residual_add")
    return y


def faar_rope(x, n_heads, cos_t, sin_t, inverse=False, out=None):
    """x bf16 [T, n_heads * dh]; cos_t, sin_t float32 [S, dh / 2] (row = position in the sequence, T a multiple of S).
    -> y bf16 like x (out may be x)."""
    _dev(x, cos_t, sin_t, out)
    T, HD = x.shape
    S, half = cos_t.shape
    if HD != n_heads * 2 * half or T % S != 0 or sin_t.shape != cos_t.shape:
        raise ValueError("faar_rope: x [T, n_heads * dh], tables [S, dh / 2], T a multiple of S")
    y = torch.empty_like(x) if out is None else out
    _check(lib().faar_rope(_ptr(x), T, n_heads, 2 * half, _ptr(cos_t), _ptr(sin_t), S, int(bool(inverse)), _ptr(y), _stream()),
           "faar_rope")
    return y


def faar_attention_fwd(q, k, v, n_seq, n_q, n_kv, scale=None, ws=None):
    """Causal grouped-query attention.  q bf16 [T, n_q * dh]; k, v bf16 [T, n_kv * dh]; T = n_seq * S.
    -> (o bf16 [T, n_q * dh], lse float32 [n_q, T])."""
    _dev(q, k, v, ws)
    T, QD = q.shape
    dh = QD // n_q
    S = T // n_seq
    if k.shape != (T, n_kv * dh) or v.shape != k.shape or S * n_seq != T:
        raise ValueError("faar_attention_fwd: shapes")
    scale = dh ** -0.5 if scale is None else scale
    o = torch.empty_like(q)
    lse = torch.empty((n_q, T), dtype=torch.float32, device=q.device)
    ws = _workspace(OP_ATTENTION_FWD, n_q * dh, n_kv * dh, T, device=q.device) if ws is None else ws
    _check(lib().faar_attention_fwd(_ptr(q), _ptr(k), _ptr(v), n_seq, S, n_q, n_kv, dh, float(scale), _ptr(o), _ptr(lse), _ptr(ws),
                                    ws.numel(), _stream()), "faar_attention_fwd")
    return o, lse


def faar_attention_bwd(d_o, q, k, v, o, lse, n_seq, n_q, n_kv, scale=None, ws=None):
    """-> (dq, dk, dv) bf16, shaped like q, k, v."""
    _dev(d_o, q, k, v, o, lse, ws)
    T, QD = q.shape
    dh = QD // n_q
    S = T // n_seq
    if d_o.shape != q.shape or o.shape != q.shape or k.shape != (T, n_kv * dh) or v.shape != k.shape or lse.shape != (n_q, T):
        raise ValueError("faar_attention_bwd: shapes")
    scale = dh ** -0.5 if scale is None else scale
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = _workspace(OP_ATTENTION_BWD, n_q * dh, n_kv * dh, T, device=q.device) if ws is None else ws
    _check(lib().faar_attention_bwd(_ptr(d_o), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), n_seq, S, n_q, n_kv, dh, float(scale),
                                    _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), ws.numel(), _stream()), "faar_attention_bwd")
    return dq, dk, dv


def faar_silu_mul_fwd(p, q):
    _dev(p, q)
    a = torch.empty_like(p)
    _check(lib().faar_silu_mul_fwd(_ptr(p), _ptr(q), p.numel(), _ptr(a), _stream()), "faar_silu_mul_fwd")
    return a


def faar_silu_mul_bwd(da, p, q):
    _dev(da, p, q)
    dp, dq = torch.empty_like(p), torch.empty_like(q)
    _check(lib().faar_silu_mul_bwd(_ptr(da), _ptr(p), _ptr(q), p.numel(), _ptr(dp), _ptr(dq), _stream()), "faar_silu_mul_bwd")
    return dp, dq


def faar_block_output_loss(x, d, y_fp, mse_scale, want_y=False, ws=None):
    """-> (loss f32[1], dy bf16 [T, D], y bf16 or None)."""
    _dev(x, d, y_fp, ws)
    T, D = x.shape
    dy = torch.empty((T, D), dtype=torch.bfloat16, device=x.device)
    y = torch.empty((T, D), dtype=torch.bfloat16, device=x.device) if want_y else None
    loss = torch.empty(1, dtype=torch.float32, device=x.device)
    ws = _workspace(OP_BLOCK_OUTPUT_LOSS, D, 16, T, device=x.device) if ws is None else ws
    _check(lib().faar_block_output_loss(_ptr(x), _dt(x), _ptr(d), _ptr(y_fp), _dt(y_fp), T, D, float(mse_scale), _ptr(y), _ptr(dy),
                                        _ptr(loss), _ptr(ws), ws.numel(), _stream()), "faar_block_output_loss")
    return loss, dy, y


def faar_stochastic_v(W, s_global, scales, seed, sample):
    """-> V f32 [O,K] in {0,1}: up with probability v_init, drawn from Philox keyed by (seed, sample)."""
    _dev(W, s_global, scales)
    O, K = W.shape
    V = torch.empty((O, K), dtype=torch.float32, device=W.device)
    _check(lib().faar_stochastic_v(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), int(seed), int(sample), _ptr(V),
                                   _stream()), "faar_stochastic_v")
    return V


def faar_hardened_loss(W, s_global, scales, V, Xq, C, mse_scale, ws, x_scale=None, loss=None):
    """-> loss f32[1]: mse_scale * ||Xq W_final(V)^T - Y_fp||^2 for the hardened V (ws: a layer-step workspace)."""
    _dev(W, s_global, scales, V, Xq, C, ws, x_scale, loss)
    O, K = W.shape
    T = Xq.shape[0]
    loss = torch.empty(1, dtype=torch.float32, device=W.device) if loss is None else loss
    _check(lib().faar_hardened_loss(_ptr(W), _dt(W), O, K, _ptr(s_global), _ptr(scales), _ptr(V), _ptr(Xq), _ptr(x_scale),
                                    _ptr(C), T, float(mse_scale), _ptr(loss), _ptr(ws), ws.numel(), _stream()),
           "faar_hardened_loss")
    return loss


def block_description(n_seq, S, D, n_q, n_kv, dh, F, eps, g_attn, g_mlp, cos_t, sin_t, linears, g_q=None, g_k=None, attn_scale=0.0):
    """A faar_block for faar_block_joint_step.  linears: dict slot name (BLOCK_SLOTS) -> dict with the device tensors
    W, s_global, scales, icodes, V, m, u, losses.  Keeps references to every tensor it points to."""
    _dev(g_attn, g_mlp, cos_t, sin_t, g_q, g_k)
    b = faar_block()
    b.n_seq, b.S, b.D, b.n_q, b.n_kv, b.dh, b.F = n_seq, S, D, n_q, n_kv, dh, F
    b.eps, b.attn_scale = float(eps), float(attn_scale)
    b.wdt = _dt(linears["q"]["W"])
    b.g_attn, b.g_mlp, b.g_q, b.g_k, b.cos_t, b.sin_t = (_ptr(t) for t in (g_attn, g_mlp, g_q, g_k, cos_t, sin_t))
    keep = [g_attn, g_mlp, g_q, g_k, cos_t, sin_t]
    for i, name in enumerate(BLOCK_SLOTS):
        lay = linears[name]
        ts = [lay[k] for k in ("W", "s_global", "scales", "icodes", "V", "m", "u", "losses")]
        _dev(*ts)
        if _dt(lay["W"]) != b.wdt:
            raise ValueError("block_description: all seven W must have one dtype")
        (b.lin[i].W, b.lin[i].s_global, b.lin[i].scales, b.lin[i].icodes, b.lin[i].V, b.lin[i].adam_m, b.lin[i].adam_u,
         b.lin[i].losses) = (_ptr(t) for t in ts)
        keep += ts
    b._keep = keep
    return b


def faar_block_workspace(block, device="cuda"):
    n = int(lib().faar_block_workspace_bytes(ctypes.byref(block)))
    if n == 0:
        raise FaarError(-2, "faar_block_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def faar_block_joint_step(block, x, y_fp, mse_scale, beta, lambda_round, lr, beta1, beta2, eps, t, ws, want_dx=True, block_loss=None):
    """One joint step of a whole block.  -> (block_loss float32[1], dx bf16 [T, D] or None)."""
    _dev(x, y_fp, ws, block_loss)
    loss = torch.empty(1, dtype=torch.float32, device=x.device) if block_loss is None else block_loss
    dx = torch.empty_like(x) if want_dx else None
    opt = faar_adam(float(lr), float(beta1), float(beta2), float(eps), int(t))
    _check(lib().faar_block_joint_step(ctypes.byref(block), _ptr(x), _ptr(y_fp), float(mse_scale), float(beta), float(lambda_round),
                                       ctypes.byref(opt), _ptr(loss), _ptr(dx), _ptr(ws), ws.numel(), _stream()),
           "faar_block_joint_step")
    return loss, dx
