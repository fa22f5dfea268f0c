"""Benchmark of the FAAR per-layer rounding-optimisation path on one MI355X.

Default workload (N=1): the Llama3-1B-shaped attention projection of the second configuration --
q_proj, W 2048x2048 bf16 Student-t(4) scaled to std 0.02, calibration X 4096 tokens x 2048 bf16
with 1% outlier channels x30 -- synthetic, seeded, resident in HBM before the timed region.
--workload picks another linear of the Llama3-1B- / Qwen3-1.7B-shaped blocks (see WORKLOADS).

Timed region: one whole per-layer job = faar_quant_rtn + faar_init_v + faar_layer_prepare, then
EXACTLY K faar_layer_step calls (soft-quant, residual GEMM + loss, dW GEMM, dV + Round Loss + Adam +
clip; beta annealed 4 -> 32), then faar_harden_pack.  value = K / elapsed (steps/s).

Also printed in the same JSON line:
  roofline      -- the dominant kernel's achieved rate from HIP-event brackets around each of its
                   launches (library hook faar_time_kernel), against the MI355X published peak
  kernels       -- the same measurement for every kernel of the path
  cpu_baseline  -- the CPU oracle timed on this host on a bounded number of steps of the same layer
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published

# name -> (O, K, T, gated_input): linears of the Llama3-1B-shaped (T = 4096), Qwen3-1.7B-shaped (T = 8192) and
# Llama3-8B-shaped (T = 4096) blocks
WORKLOADS = {
    "q_proj": (2048, 2048, 4096, False), "k_proj": (512, 2048, 4096, False),
    "gate_proj": (8192, 2048, 4096, False), "down_proj": (2048, 8192, 4096, True),
    "qwen_k_proj": (1024, 2048, 8192, False), "qwen_q_proj": (2048, 2048, 8192, False),
    "qwen_gate_proj": (6144, 2048, 8192, False), "qwen_down_proj": (2048, 6144, 8192, True),
    # Llama3-8B-shaped linears (the paper's larger model), T = 4096
    "llama8b_q_proj": (4096, 4096, 4096, False), "llama8b_k_proj": (1024, 4096, 4096, False),
    "llama8b_gate_proj": (14336, 4096, 4096, False), "llama8b_down_proj": (4096, 14336, 4096, True),
}


def bytes_per_weight(dw_split: int) -> dict:
    """Algorithmic bytes per weight element of each HBM-bound kernel (bf16 W, fp32 V/m/u, 1/16 B scale,
    1/2 B cached interval code), for the design as built: the dV kernel reads one fp32 partial per dW split
    and, in every step but a layer's last, also writes the next step's W_q - W."""
    return {
        "softquant_fwd": 2 + 4 + 0.5 + 1 / 16 + 2,             # read W, V, code, scale; write W_q - W (bf16)
        "bwd_adam": 4 * dw_split + 0.5 + 1 / 16 + 12 + 12 + 2 + 2,  # read G partials, code, scale, V, m, u, W; write V, m, u, W_q - W
        "quant_rtn": 2 + 0.5 + 1 / 16,                         # read W; write codes, scales
        "init_v": 2 + 1 / 16 + 4,                              # read W, scales; write V
        "harden_pack": 2 + 4 + 1 / 16 + 0.5,                   # read W, V, scales; write codes
        # stand-alone call: forward reads W, V, scale and writes W_q - W; backward reads dW_q, W, V, scale and writes dV
        "softquant_fwd_bwd_call": (2 + 4 + 1 / 16 + 2) + (4 + 2 + 4 + 1 / 16 + 4),
    }


class HipEvents:
    """Raw hipEvent_t pairs via the HIP runtime already loaded by torch (plumbing only)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return ev

    def elapsed_ms(self, a, b) -> float:
        self.hip.hipEventSynchronize(b)
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)


# The seven linears of one Qwen3-1.7B-shaped block: name -> (O, K, input group, gated input)
QWEN_BLOCK = [("q_proj", 2048, 2048, "attn_in", False), ("k_proj", 1024, 2048, "attn_in", False),
              ("v_proj", 1024, 2048, "attn_in", False), ("o_proj", 2048, 2048, "attn_out", False),
              ("gate_proj", 6144, 2048, "mlp_in", False), ("up_proj", 6144, 2048, "mlp_in", False),
              ("down_proj", 2048, 6144, "mlp_mid", True)]
QWEN_LAYERS = 28


def run_block_chained(args) -> dict:
    """All seven linears of one Qwen3-1.7B-shaped block stepped back to back at T = 16384, each with an
    upstream gradient supplied (dY_ext) and its input gradient requested (dX): three GEMMs per linear and step.
    One timed "step" is one step of every linear; `value` counts linear-layer steps."""
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb
    from workloads import synth

    T = 16384
    steps = min(args.steps, 50)
    warmup = min(args.warmup, 5)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    X_by_group, lin = {}, []
    for idx, (name, O, K, group, gated) in enumerate(QWEN_BLOCK):
        if group not in X_by_group:
            X_h = synth.silu_gated_activations(T, K, seed=idx) if gated else synth.activations(T, K, seed=idx)
            X_by_group[group] = torch.from_numpy(X_h).cuda().to(torch.bfloat16)
        Xq = X_by_group[group]
        W = torch.from_numpy(synth.student_t_weight(O, K, seed=idx)).cuda().to(torch.bfloat16)
        Y = Xq @ W.T                                                     # input generation only
        dY = (torch.randn((T, O), generator=gen, device="cuda") * 1e-3).to(torch.bfloat16)
        sg, scales, _, _ = faar.faar_quant_rtn(W)
        V, _ = faar.faar_init_v(W, sg, scales)
        Xt, C, ic = faar.faar_layer_prepare(W, sg, scales, Xq, Y)
        del Y
        lin.append(dict(name=name, O=O, K=K, W=W, sg=sg, scales=scales, V=V, m=torch.zeros_like(V), u=torch.zeros_like(V),
                        Xq=Xq, Xt=Xt, C=C, ic=ic, dY=dY, dX=torch.empty((T, K), dtype=torch.bfloat16, device="cuda"),
                        ws=faar.layer_step_workspace(O, K, T, chained=True),
                        losses=torch.zeros(3, dtype=torch.float32, device="cuda"), ready=False))
    lam, lr = 0.01, 5e-4

    def step_linear(L, t, beta=16.0, fused=True):
        faar.faar_layer_step(L["W"], L["sg"], L["scales"], L["V"], L["m"], L["u"], L["Xq"], L["Xt"], L["C"], L["ic"], beta,
                             lam, 1.0 / (T * L["O"]), lr, 0.9, 0.999, 1e-8, t, L["losses"], L["ws"], dY_ext=L["dY"],
                             dX=L["dX"], beta_next=beta if fused else 0.0, forward_ready=fused and L["ready"])
        L["ready"] = fused

    t = 0
    for _ in range(warmup):
        t += 1
        for L in lin:
            step_linear(L, t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        t += 1
        for L in lin:
            step_linear(L, t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    per_linear = {}
    total_flops = 0.0
    for L in lin:
        O, K = L["O"], L["K"]
        flops = 2.0 * T * O * K
        total_flops += 3 * flops
        row = {}
        for kname, kid in [("gemm_residual", fb.K_GEMM_RESIDUAL), ("gemm_dw", fb.K_GEMM_DW), ("gemm_dx", fb.K_GEMM_DX),
                           ("bwd_adam", fb.K_BWD_ADAM)]:
            ts = []
            fb.faar_time_kernel(kid, e0.value, e1.value)
            try:
                for _ in range(6):
                    t += 1
                    step_linear(L, t)
                    ts.append(ev.elapsed_ms(e0, e1))
            finally:
                fb.faar_time_kernel(fb.K_NONE)
            ms = sum(ts[2:]) / len(ts[2:])
            if kname.startswith("gemm"):
                row[kname] = {"ms": round(ms, 5), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                              "frac": round(flops / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, 4)}
            else:
                b = bytes_per_weight(fb.faar_dw_split(O, K, T))["bwd_adam"] + 2      # + W_q for the next dX
                row[kname] = {"ms": round(ms, 5), "gbs": round(b * O * K / (ms * 1e-3) / 1e9, 1),
                              "frac": round(b * O * K / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        row["dw_split"] = fb.faar_dw_split(O, K, T)
        per_linear[L["name"]] = row
    dom_l, dom_k = max(((l, k) for l in per_linear for k in ("gemm_residual", "gemm_dw", "gemm_dx")),
                       key=lambda lk: per_linear[lk[0]][lk[1]]["ms"])
    dom = per_linear[dom_l][dom_k]
    n_lin = len(lin)
    return {
        "metric": "FAAR layer steps/sec (fwd+bwd+Adam)", "value": round(n_lin * steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "qwen_block_chained: the 7 linears of one Qwen3-1.7B-shaped block (q/o 2048x2048, k/v "
                               "1024x2048, gate/up 6144x2048, down 2048x6144), T 16384, each stepped once per timed step "
                               "with dY supplied and dX produced (3 GEMMs per linear); value = linear-layer steps/s",
                   "T": T, "linears": n_lin},
        "block_step_gemm_tflops": round(total_flops / (elapsed / steps) / 1e12, 1),
        "roofline": {"kernel": f"{dom_l}.{dom_k}", "bound": "mfma", "achieved": dom["tflops"], "peak": BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": dom["frac"], "traffic": None, "launch_ms": dom["ms"]},
        "per_linear": per_linear,
    }


def run_pack_sweep(args) -> dict:
    """Set-up and tear-down kernels over every linear of a Qwen3-1.7B-shaped model (28 layers x 7 linears,
    1.409 G weights, each tensor in memory of its own): faar_quant_rtn, faar_init_v and faar_harden_pack,
    each timed as a sweep over all 196 tensors.  `value` is the harden+pack rate."""
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb
    from workloads import synth

    base = {}
    for idx, (name, O, K, _, _) in enumerate(QWEN_BLOCK):
        if (O, K) not in base:                       # one seeded draw per shape, copied into every layer's own tensor
            base[(O, K)] = torch.from_numpy(synth.student_t_weight(O, K, seed=idx)).cuda().to(torch.bfloat16)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    tensors = []
    n_total = 0
    for layer in range(QWEN_LAYERS):
        for name, O, K, _, _ in QWEN_BLOCK:
            W = base[(O, K)].clone()
            V = torch.rand((O, K), generator=gen, device="cuda", dtype=torch.float32)   # rounding variables mid-optimisation
            tensors.append([W, V, None, None])
            n_total += O * K
    ws_q = torch.empty(faar.faar_workspace_bytes(fb.OP_QUANT_RTN, 6144, 2048), dtype=torch.uint8, device="cuda")
    reps = 5

    def sweep(fn):
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            t0 = time.perf_counter()
            for rec in tensors:
                fn(rec)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        return best

    def do_quant(rec):
        rec[2], rec[3], _, _ = faar.faar_quant_rtn(rec[0], ws=ws_q)

    t_quant = sweep(do_quant)
    t_init = sweep(lambda rec: faar.faar_init_v(rec[0], rec[2], rec[3]))
    t_pack = sweep(lambda rec: faar.faar_harden_pack(rec[0], rec[2], rec[3], rec[1]))
    bpw = bytes_per_weight(1)
    rows = {}
    for name, tt, b in (("quant_rtn", t_quant, bpw["quant_rtn"] + 2), ("init_v", t_init, bpw["init_v"]),
                        ("harden_pack", t_pack, bpw["harden_pack"])):
        rows[name] = {"ms": round(tt * 1e3, 3), "gbs": round(b * n_total / tt / 1e9, 1),
                      "frac": round(b * n_total / tt / 1e9 / HBM_PEAK_GBS, 4), "bytes_per_weight": b}
    return {
        "metric": "NVFP4 harden+pack weight elements/sec", "value": round(n_total / t_pack, 1), "unit": "elems/s",
        "n_gpus": 1, "steps": reps, "warmup": 0, "ms_per_step": rows["harden_pack"]["ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"qwen_pack_sweep: {len(tensors)} weight tensors of a Qwen3-1.7B-shaped model "
                               f"({n_total / 1e9:.3f} G weights, bf16 W + float32 V in, NVFP4 codes out); best of {reps} sweeps; "
                               "times include the allocation of each output by the binding",
                   "weights": n_total},
        "roofline": {"kernel": "harden_pack", "bound": "hbm", "achieved": rows["harden_pack"]["gbs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": rows["harden_pack"]["frac"], "traffic": None},
        "sweeps": rows,
    }


def run_stage2(args) -> dict:
    """faar_stage2_losses on Llama3-1B-shaped model outputs: 4096 tokens, vocabulary 128256, hidden size 2048,
    bf16 logits and hidden states, losses and both gradients.  One timed step = one call."""
    import numpy as np
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb

    T, V, D, tau = 4096, 128256, 2048, 1.0
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    Zf = (torch.randn((T, V), generator=gen, device="cuda") * 3.0).to(torch.bfloat16)
    Zq = (Zf.float() + torch.randn((T, V), generator=gen, device="cuda") * 0.3).to(torch.bfloat16)
    Hf = torch.randn((T, D), generator=gen, device="cuda").to(torch.bfloat16)
    Hq = (Hf.float() + torch.randn((T, D), generator=gen, device="cuda") * 0.1).to(torch.bfloat16)
    rl = torch.rand(112, generator=gen, device="cuda")
    ws = torch.empty(faar.faar_workspace_bytes(fb.OP_STAGE2_LOSSES, V, D, T), dtype=torch.uint8, device="cuda")
    kw = dict(kl_scale=1.0 / T, mse_scale=1.0 / (T * D), round_losses=rl, lambda_kl=1.0, lambda_round=0.01, ws=ws)
    steps, warmup = min(args.steps, 50), min(args.warmup, 5)
    for _ in range(max(1, warmup)):
        losses, dZ, dH = faar.faar_stage2_losses(Zf, Zq, tau, Hf, Hq, **kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        losses, dZ, dH = faar.faar_stage2_losses(Zf, Zq, tau, Hf, Hq, **kw)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    ts = []
    fb.faar_time_kernel(fb.K_STAGE2_KL, e0.value, e1.value)
    try:
        for _ in range(8):
            faar.faar_stage2_losses(Zf, Zq, tau, Hf, Hq, **kw)
            ts.append(ev.elapsed_ms(e0, e1))
    finally:
        fb.faar_time_kernel(fb.K_NONE)
    ms = sum(ts[2:]) / len(ts[2:])
    algo = (T * V + T * D) * (2 + 2 + 2)            # read both tensors once, write the gradient (bf16)
    gbs = algo / (ms * 1e-3) / 1e9
    out = {
        "metric": "Stage-2 loss evaluations/sec (KL + MSE + gradients)", "value": round(steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"stage2_losses: logits {T}x{V} bf16 N(0, 3^2), quantised-model logits = those + N(0, 0.3^2); "
                               f"hidden states {T}x{D} bf16; tau 1; losses and both gradients", "T": T, "vocab": V, "D": D},
        "tokens_per_sec": round(T * steps / elapsed, 1),
        "final_losses": losses.cpu().numpy().tolist(),
        "roofline": {"kernel": "stage2 (KL rows + MSE + sums)", "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "launch_ms": round(ms, 5)},
    }
    if not args.no_cpu_baseline:
        from oracle import faar_oracle as fo
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        rows = 64
        zf, zq = Zf[:rows].float().cpu().numpy(), Zq[:rows].float().cpu().numpy()
        hf, hq = Hf[:rows].float().cpu().numpy(), Hq[:rows].float().cpu().numpy()
        n, t_cpu = 0, 0.0
        while n < 1 or (t_cpu < args.cpu_seconds and n < 50):
            c0 = time.perf_counter()
            fo.stage2_losses(zf, zq, tau, 1.0 / T, hf, hq, 1.0 / (T * D), rl.cpu().numpy(), 1.0, 0.01)
            t_cpu += time.perf_counter() - c0
            n += 1
        out["cpu_baseline"] = {"value": round(n * rows / T / t_cpu, 5), "unit": "steps/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{n} evaluations of {rows} of the {T} token rows (numpy float64, {t_cpu:.1f} s), "
                                         "scaled to whole steps"}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="q_proj", choices=sorted(WORKLOADS) + ["qwen_block_chained", "qwen_pack_sweep", "stage2_losses"])
    ap.add_argument("--quantised-acts", action="store_true",
                    help="W4A4: quantise the activations to NVFP4 with the same kernel and feed them as (units, tensor scale)")
    ap.add_argument("--stochastic-trials", type=int, default=0,
                    help="after the job, rank this many stochastic-rounding candidates by hardened reconstruction loss")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--probe-steps", type=int, default=20)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy three times (reference for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path has no collectives or sharding "
              "(layers and output rows are independent jobs: shard those across processes). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload == "qwen_block_chained":
        print(json.dumps(run_block_chained(args)))
        return 0
    if args.workload == "qwen_pack_sweep":
        print(json.dumps(run_pack_sweep(args)))
        return 0
    if args.workload == "stage2_losses":
        print(json.dumps(run_stage2(args)))
        return 0
    O, K, T, gated = WORKLOADS[args.workload]
    W_h = synth.student_t_weight(O, K, seed=0)
    X_h = synth.silu_gated_activations(T, K, seed=0) if gated else synth.activations(T, K, seed=0)
    W = torch.from_numpy(W_h).cuda().to(torch.bfloat16)
    Xq = torch.from_numpy(X_h).cuda().to(torch.bfloat16)
    Y = Xq @ W.T                       # the frozen BF16 layer output: an input of the method (input generation only)
    x_scale = None
    if args.quantised_acts:            # X_q = NVFP4(X): node * block scale in bf16 (exact) and the tensor scale on the side
        x_scale, _, _, Xq = faar.faar_quant_rtn(Xq, want_dq=True, dq_in_units=True)
        X_h = (Xq.float() * x_scale).cpu().numpy()
    torch.cuda.synchronize()
    N = O * K
    alpha, lam, lr = 1.0 / (T * O), 0.01, 5e-4
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ws = faar.layer_step_workspace(O, K, T)
    ws_q = torch.empty(faar.faar_workspace_bytes(fb.OP_QUANT_RTN, O, K), dtype=torch.uint8, device="cuda")
    ws_p = torch.empty(max(256, faar.faar_workspace_bytes(fb.OP_LAYER_PREPARE, O, K, T)), dtype=torch.uint8, device="cuda")

    def beta_at(t, total):
        return 4.0 + 28.0 * (t - 1) / max(1, total - 1)

    def layer_job(n_steps):
        sg, scales, codes, _ = faar.faar_quant_rtn(W, ws=ws_q)
        V, _ = faar.faar_init_v(W, sg, scales)
        Xt, C, ic = faar.faar_layer_prepare(W, sg, scales, Xq, Y, ws=ws_p, x_scale=x_scale)
        m = torch.zeros_like(V)
        u = torch.zeros_like(V)
        for t in range(1, n_steps + 1):
            # every step but the last also prepares the next step's soft-quantised weights (beta_next)
            faar.faar_layer_step(W, sg, scales, V, m, u, Xq, Xt, C, ic, beta_at(t, n_steps), lam, alpha, lr, 0.9, 0.999,
                                 1e-8, t, losses, ws, beta_next=beta_at(t + 1, n_steps) if t < n_steps else 0.0,
                                 forward_ready=t > 1, x_scale=x_scale)
        out, _, _, flips = faar.faar_harden_pack(W, sg, scales, V, want_flips=True)
        return sg, scales, V, m, u, Xt, C, ic, out, flips

    # warm-up (untimed)
    layer_job(max(1, args.warmup))
    torch.cuda.synchronize()

    # timed region: exactly K steps inside one whole per-layer job
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sg, scales, V, m, u, Xt, C, ic, packed, flips = layer_job(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    final_losses = losses.cpu().numpy().tolist()
    n_flips = int(flips.item())
    # what the optimisation bought, on the hardened (deployable) weights: reconstruction loss of round-to-nearest
    # against that of the hardened V (outside the timed region)
    V_rtn, _ = faar.faar_init_v(W, sg, scales)
    loss_rtn = float(faar.faar_hardened_loss(W, sg, scales, V_rtn, Xq, C, alpha, ws, x_scale=x_scale).item())
    loss_faar = float(faar.faar_hardened_loss(W, sg, scales, V, Xq, C, alpha, ws, x_scale=x_scale).item())
    stochastic = None
    if args.stochastic_trials > 0:
        trial = torch.empty(args.stochastic_trials, dtype=torch.float32, device="cuda")
        for k in range(args.stochastic_trials):
            Vs = faar.faar_stochastic_v(W, sg, scales, 2603, k)
            faar.faar_hardened_loss(W, sg, scales, Vs, Xq, C, alpha, ws, x_scale=x_scale, loss=trial[k:k + 1])
        tl = trial.cpu().numpy()
        stochastic = {"trials": int(tl.size), "better_than_rtn": int((tl < loss_rtn).sum()), "best": float(tl.min()),
                      "mean": float(tl.mean()), "std": float(tl.std())}

    # per-kernel durations: HIP events recorded by the library around each launch of one kernel
    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    probe = {}

    def timed_kernel(which, call, n):
        ts = []
        fb.faar_time_kernel(which, e0.value, e1.value)
        try:
            for i in range(n):
                call(i)
                ts.append(ev.elapsed_ms(e0, e1))
        finally:
            fb.faar_time_kernel(fb.K_NONE)
        ts = ts[2:] if len(ts) > 4 else ts
        return sum(ts) / len(ts)

    def first_step_call(i):      # a layer's first step: its own forward kernel, nothing prepared for the next
        faar.faar_layer_step(W, sg, scales, V, m, u, Xq, Xt, C, ic, 16.0, lam, alpha, lr, 0.9, 0.999, 1e-8,
                             args.steps + 1 + i, losses, ws, x_scale=x_scale)

    def step_call(i):            # every later step: forward taken from / left in the workspace
        faar.faar_layer_step(W, sg, scales, V, m, u, Xq, Xt, C, ic, 16.0, lam, alpha, lr, 0.9, 0.999, 1e-8,
                             args.steps + 1 + i, losses, ws, beta_next=16.0, forward_ready=i > 0, x_scale=x_scale)

    n_probe = max(5, args.probe_steps)
    probe["softquant_fwd"] = timed_kernel(fb.K_SOFTQUANT_FWD, first_step_call, n_probe)
    for name, kid in [("gemm_residual", fb.K_GEMM_RESIDUAL), ("gemm_dw", fb.K_GEMM_DW), ("bwd_adam", fb.K_BWD_ADAM)]:
        probe[name] = timed_kernel(kid, step_call, n_probe)
    # the stand-alone soft-quantisation entry point (forward + backward from a given dL/dW_q; it re-derives the
    # intervals from W and the scales on every call): torch events around the whole call, output allocation included
    dWt = torch.randn((O, K), device="cuda") * 1e-3
    te0, te1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(n_probe + 3):
        if i == 3:
            te0.record()
        faar.faar_softquant_fwd_bwd(W, sg, scales, V, 16.0, dWt=dWt, lambda_round=lam, emit_delta=True)
    te1.record()
    torch.cuda.synchronize()
    probe["softquant_fwd_bwd_call"] = te0.elapsed_time(te1) / n_probe
    del dWt
    probe["quant_rtn"] = timed_kernel(fb.K_QUANT_RTN, lambda i: faar.faar_quant_rtn(W, ws=ws_q), n_probe)
    probe["init_v"] = timed_kernel(fb.K_INIT_V, lambda i: faar.faar_init_v(W, sg, scales), n_probe)
    probe["harden_pack"] = timed_kernel(fb.K_HARDEN_PACK, lambda i: faar.faar_harden_pack(W, sg, scales, V), n_probe)

    gemm_flops = 2.0 * T * O * K
    dw_split = fb.faar_dw_split(O, K, T)
    bpw = bytes_per_weight(dw_split)
    kernels = {}
    for name, ms in probe.items():
        if name.startswith("gemm"):
            ach = gemm_flops / (ms * 1e-3) / 1e12
            kernels[name] = {"ms": round(ms, 5), "bound": "mfma", "achieved": round(ach, 2), "unit": "TFLOP/s",
                             "frac": round(ach / BF16_PEAK_TFLOPS, 4)}
        else:
            ach = bpw[name] * N / (ms * 1e-3) / 1e9
            kernels[name] = {"ms": round(ms, 5), "bound": "hbm", "achieved": round(ach, 1), "unit": "GB/s",
                             "frac": round(ach / HBM_PEAK_GBS, 4)}
    # HBM-side bytes per launch measured with rocprofv3 PMC counters (committed summary; None if not measured)
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) == 4 and f[0] == args.workload:
                traffic[f[1]] = int((float(f[2]) + float(f[3])) * 1e6)
    for name in kernels:
        kernels[name]["traffic"] = traffic.get(name)
    dom = max(("gemm_residual", "gemm_dw", "softquant_fwd", "bwd_adam"), key=lambda k: probe[k])
    roofline = {"kernel": dom, "bound": kernels[dom]["bound"], "achieved": kernels[dom]["achieved"],
                "peak": BF16_PEAK_TFLOPS if kernels[dom]["bound"] == "mfma" else HBM_PEAK_GBS,
                "unit": kernels[dom]["unit"], "frac": kernels[dom]["frac"], "traffic": kernels[dom]["traffic"],
                "launch_ms": kernels[dom]["ms"]}

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = elapsed / args.steps * 1e3
    out = {
        "metric": "FAAR layer steps/sec (fwd+bwd+Adam)", "value": round(args.steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: W {O}x{K} bf16 Student-t(4) std 0.02, X {T}x{K} "
                               f"{'NVFP4-quantised (W4A4)' if args.quantised_acts else 'bf16'}, NVFP4 block 16; "
                               "per-layer job = quant_rtn + init_v + prepare + K steps + harden_pack",
                   "O": O, "K": K, "T": T},
        "weight_elems_per_sec": round(N * args.steps / elapsed, 1),
        "step_gemm_tflops": round(2 * gemm_flops / (ms_per_step * 1e-3) / 1e12, 1),
        "dw_split": dw_split, "final_losses": final_losses, "flipped_decisions": n_flips,
        "hardened_loss": {"rtn": loss_rtn, "faar": loss_faar, "stochastic": stochastic},
        "roofline": roofline, "kernels": kernels,
    }

    if not args.no_cpu_baseline:
        from oracle import faar_oracle as fo
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        Y_h = Y.float().cpu().numpy()
        q = fo.quant_rtn(W_h, True)
        V0 = fo.init_v(W_h, q["s_global"], q["scales"])["V"]
        m0 = np.zeros_like(V0)
        u0 = np.zeros_like(V0)
        n_cpu, t_cpu = 0, 0.0
        while n_cpu < 1 or (t_cpu < args.cpu_seconds and n_cpu < 500):
            c0 = time.perf_counter()
            r = fo.layer_step(W_h, q["s_global"], q["scales"], V0, m0, u0, X_h, Y_h,
                              beta_at(n_cpu + 1, args.steps), lam, alpha, lr, 0.9, 0.999, 1e-8, n_cpu + 1)
            V0, m0, u0 = r["V"], r["m"], r["u"]
            t_cpu += time.perf_counter() - c0
            n_cpu += 1
        out["cpu_baseline"] = {"value": round(n_cpu / t_cpu, 4), "unit": "steps/s", "cores": int(cores),
                               "kind": "oracle",
                               "sample": f"{n_cpu} layer steps of the same {args.workload} layer (numpy float64, "
                                         f"{t_cpu:.1f} s)"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
