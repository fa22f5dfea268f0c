"""Benchmark of the FAAR per-layer rounding-optimisation path on one MI355X.

Default workload (N=1): one Qwen3-1.7B-shaped transformer layer -- the largest Stage-1 configuration of the
workload list: its seven linears (q/o 2048x2048, k/v 1024x2048, gate/up 6144x2048, down 2048x6144), bf16
Student-t(4) weights scaled to std 0.02, 8192 calibration tokens per linear with 1 % outlier channels x30
(silu(g)*u inputs for the down projection) -- synthetic, seeded, resident in HBM before the timed region.

Timed region: a whole per-layer job for each of the seven linears = faar_quant_rtn + faar_init_v +
faar_layer_prepare, then EXACTLY K faar_layer_step calls per linear (soft-quantisation, residual GEMM + loss,
dW GEMM, dV + Round Loss + Adam + clip; beta annealed 4 -> 32), then faar_harden_pack.  One "step" of the
command line is one optimisation step of every linear; value = 7 K / elapsed (linear-layer steps / s).

Other workloads (--workload): qwen_layer_gram (the same layer jobs with every step in its optional Gram-matrix form,
faar_layer_step_gram: one O x K x K product per step instead of two T x O x K ones -- valid because a layer's calibration
activations do not change between steps; NOT the default, which forms the layer output in every step); one linear of the Llama3-1B- / Qwen3-1.7B- / Llama3-8B-shaped blocks by name;
qwen_block_chained (the seven linears at 16384 tokens with dY supplied and dX produced); qwen_mlp_joint (one joint
step of the MLP half of the block: norm, three linears, gate, residual, block-output loss, and back); qwen_block_joint
(one joint step of the whole block, attention half included, by one faar_block_joint_step call); qwen_pack_sweep
(quantise / initialise / harden+pack all 196 weight tensors of the model); stage2_losses; gemm_ceiling (what
bounds the GEMM main loop: the loop with only its matrix instructions, with only its copies, and whole, with the
clock the compute units ran at).

Printed in the same JSON line:
  roofline      -- the dominant kernel's achieved rate from HIP-event brackets around each of its launches
                   (library hook faar_time_kernel), against the MI355X published peak
  kernels       -- the same measurement for every kernel of the path
  cpu_baseline  -- the CPU oracle timed on this host on a bounded sample of the same workload

Launch it as `python3 bench.py ...` (also under rocprofv3: the program itself after `--`).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import platform
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
    "llama8b_q_proj": (4096, 4096, 4096, False), "llama8b_k_proj": (1024, 4096, 4096, False),
    "llama8b_gate_proj": (14336, 4096, 4096, False), "llama8b_down_proj": (4096, 14336, 4096, True),
}

# The seven linears of one Qwen3-1.7B-shaped block: (name, O, K, input group, gated input)
QWEN_BLOCK = [("q_proj", 2048, 2048, "attn_in", False), ("k_proj", 1024, 2048, "attn_in", False),
              ("v_proj", 1024, 2048, "attn_in", False), ("o_proj", 2048, 2048, "attn_out", False),
              ("gate_proj", 6144, 2048, "mlp_in", False), ("up_proj", 6144, 2048, "mlp_in", False),
              ("down_proj", 2048, 6144, "mlp_mid", True)]
QWEN_LAYERS = 28
LAM, LR = 0.01, 5e-4


def bytes_per_weight(dw_split: int, use_h: bool = False) -> dict:
    """Algorithmic bytes per weight element of each HBM-bound kernel (bf16 W, fp32 V/m/u, 1/16 B scale,
    1/2 B cached interval code), for the design as built: the dV kernel reads one fp32 partial per dW split
    and, in every step but a layer's last, also writes the next step's W_q - W."""
    return {
        # read W, V, code, scale (and H, for the loss's cross term); write W_q - W (bf16)
        "softquant_fwd": 2 + 4 + 0.5 + 1 / 16 + 2 + (4 if use_h else 0),
        # read G partials (and H), code, scale, V, m, u, W; write V, m, u, W_q - W
        "bwd_adam": 4 * dw_split + (4 if use_h else 0) + 0.5 + 1 / 16 + 12 + 12 + 2 + 2,
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


class KernelTimer:
    """Average duration of one kernel of the path in steady state: the library brackets each of its launches with a pair
    of HIP events out of a ring, on the stream it is launched on; the calls are issued back to back without host
    synchronisation for long enough (BUSY_MS) that the chip runs at the clocks it holds during a real job (after idling,
    and between synchronised single launches, it runs ~20 % slower for the first tens of milliseconds), and the last RING
    launches are averaged."""
    RING, BUSY_MS, MAX_CALLS = 32, 80.0, 1500

    def __init__(self):
        self.ev = HipEvents()
        self.events = [self.ev.create() for _ in range(2 * self.RING)]

    def time(self, which, call, n, position=None):
        """Average duration (ms) of the launches of kernel `which` made by call(0), call(1), ...  position: when every call
        launches the kernel several times, average only the launches at that index within a call (-1 = the last)."""
        import torch

        from paper_2603_22370_amd import binding as fb
        handles = [e.value for e in self.events]
        fb.faar_time_kernel_ring(which, handles)
        try:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            first = max(4, min(n, self.RING))
            for i in range(first):
                call(i)
            torch.cuda.synchronize()
            per_call_ms = (time.perf_counter() - t0) * 1e3 / first
            per_call = fb.faar_time_kernel_count() // first          # launches of the kernel per call
            more = int(min(self.MAX_CALLS, max(self.RING + 8, self.BUSY_MS / max(per_call_ms, 1e-3))))
            fb.faar_time_kernel_ring(which, handles)                 # restart the count: call boundaries stay aligned
            for i in range(first, first + more):
                call(i)
            torch.cuda.synchronize()
            count = fb.faar_time_kernel_count()
        finally:
            fb.faar_time_kernel_ring(fb.K_NONE, [])
        if count < 1 or per_call < 1:
            raise RuntimeError(f"kernel {which} was not launched by every timed call")
        ts = []
        for g in range(max(0, count - self.RING), count):            # the launches still held by the ring
            if position is None or g % per_call == position % per_call:
                k = g % self.RING
                ts.append(self.ev.elapsed_ms(self.events[2 * k], self.events[2 * k + 1]))
        return sum(ts) / len(ts)


def host_description() -> dict:
    """CPU model, thread count and BLAS of the host the oracle is timed on."""
    model = platform.processor() or "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    threads, blas = os.cpu_count() or 1, "unknown BLAS"
    try:
        from threadpoolctl import threadpool_info
        pools = [p for p in threadpool_info() if p.get("user_api") == "blas"]
        if pools:
            threads = max(p.get("num_threads", 1) for p in pools)
            blas = ", ".join(f"{p.get('internal_api')} {p.get('version')}" for p in pools)
    except Exception:
        pass
    import numpy as np
    return {"cores": int(threads), "host": f"{model}; numpy {np.__version__} float64 on {blas}, {threads} threads"}


def traffic_for(kernel: str, O: int, K: int, T: int):
    """HBM-side bytes per launch of `kernel` on an O x K layer with T tokens, from the committed rocprofv3 counter
    summary (profiles/hbm_traffic.txt: lines `kernel O K T fetch_MB write_MB`).  None when that exact kernel and shape
    was not measured: a number is never carried over from another shape."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 6 and f[0] == kernel and f[1:4] == [str(O), str(K), str(T)]:
            return int((float(f[4]) + float(f[5])) * 1e6)
    return None


class LinearJob:
    """Device-resident inputs and state of one linear layer's rounding optimisation."""

    def __init__(self, name, O, K, T, W, Xq, quantised_acts=False, form="token"):
        import torch

        import paper_2603_22370_amd as faar
        from paper_2603_22370_amd import binding as fb
        self.name, self.O, self.K, self.T = name, O, K, T
        self.W, self.Xq = W, Xq
        self.Y = Xq @ W.T              # the frozen BF16 layer output: an input of the method (input generation only)
        self.x_scale = None
        if quantised_acts:             # X_q = NVFP4(X): node * block scale in bf16 (exact) and the tensor scale on the side
            self.x_scale, _, _, self.Xq = faar.faar_quant_rtn(Xq, want_dq=True, dq_in_units=True)
        self.alpha = 1.0 / (T * O)
        self.losses = torch.zeros(3, dtype=torch.float32, device="cuda")
        self.form = form               # "token": faar_layer_step; "gram": faar_layer_step_gram
        self.whole_device = False      # set when nothing runs beside this job's steps (one stream): tiles that fill every unit
        self.ws = faar.layer_step_workspace(O, K, T) if form == "token" else fb.layer_step_gram_workspace(O, K)
        self.ws_g = (torch.empty(faar.faar_workspace_bytes(fb.OP_GRAM_PREPARE, K, K, T), dtype=torch.uint8, device="cuda")
                     if form == "gram" else None)
        self.ws_q = torch.empty(faar.faar_workspace_bytes(fb.OP_QUANT_RTN, O, K), dtype=torch.uint8, device="cuda")
        self.ws_p = None
        self.dw_split = fb.faar_dw_split(O, K, T)
        # the gradient constant H = C^T X_q trades 4 bytes per output of Y in the residual GEMM's epilogue for 4 bytes
        # per weight in the pass that updates V: used where that is a saving
        self.use_h = T >= K or form == "gram"
        self.gram_split = fb.faar_gemm_plan(fb.K_GEMM_GRAM, O, K, 1)[3] if form == "gram" else 0
        self.state = None

    @staticmethod
    def beta_at(t, total):
        return 4.0 + 28.0 * (t - 1) / max(1, total - 1)

    def setup(self):
        import torch

        import paper_2603_22370_amd as faar
        self.state = None              # a previous job's buffers go back to torch's caching allocator first: no hipMalloc here
        sg, scales, codes, _ = faar.faar_quant_rtn(self.W, ws=self.ws_q)
        V, _ = faar.faar_init_v(self.W, sg, scales)
        if self.ws_p is None:
            from paper_2603_22370_amd import binding as fb
            flags = fb.FAAR_WS_GRADIENT_CONSTANT if self.use_h else 0
            self.ws_p = torch.empty(max(256, faar.faar_workspace_bytes(fb.OP_LAYER_PREPARE, self.O, self.K, self.T, flags)),
                                    dtype=torch.uint8, device="cuda")
        out = faar.faar_layer_prepare(self.W, sg, scales, self.Xq, self.Y, ws=self.ws_p, x_scale=self.x_scale,
                                      gradient_constant=self.use_h)
        self.state = dict(sg=sg, scales=scales, V=V, m=torch.zeros_like(V), u=torch.zeros_like(V), Xt=out[0], C=out[1], ic=out[2],
                          hk=dict(H=out[3], c_norm2=out[4]) if self.use_h else {})
        if self.form == "gram":
            from paper_2603_22370_amd import binding as fb
            self.state["gram"], self.state["gram_lo"] = fb.faar_gram_prepare(out[0], self.T, ws=self.ws_g)

    def step(self, t, total, beta=None, beta_next=None, forward_ready=None):
        import paper_2603_22370_amd as faar
        s = self.state
        beta = self.beta_at(t, total) if beta is None else beta
        if beta_next is None:      # every step but the last also prepares the next step's soft-quantised weights
            beta_next = self.beta_at(t + 1, total) if t < total else 0.0
        ready = (t > 1) if forward_ready is None else forward_ready
        if self.form == "gram":
            from paper_2603_22370_amd import binding as fb
            fb.faar_layer_step_gram(self.W, s["sg"], s["scales"], s["V"], s["m"], s["u"], s["ic"], s["hk"]["H"], s["hk"]["c_norm2"],
                                    s["gram"], s["gram_lo"], beta, LAM, self.alpha, LR, 0.9, 0.999, 1e-8, t, self.losses, self.ws,
                                    beta_next=beta_next, forward_ready=ready, x_scale=self.x_scale)
            return
        faar.faar_layer_step(self.W, s["sg"], s["scales"], s["V"], s["m"], s["u"], self.Xq, s["Xt"], s["C"], s["ic"], beta,
                             LAM, self.alpha, LR, 0.9, 0.999, 1e-8, t, self.losses, self.ws, beta_next=beta_next,
                             forward_ready=ready, x_scale=self.x_scale, whole_device=self.whole_device, **s["hk"])

    def finish(self):
        import paper_2603_22370_amd as faar
        s = self.state
        s["packed"], _, _, s["flips"] = faar.faar_harden_pack(self.W, s["sg"], s["scales"], s["V"], want_flips=True)

    def hardened_losses(self):
        import paper_2603_22370_amd as faar
        s = self.state
        ws = self.ws if self.form == "token" else faar.layer_step_workspace(self.O, self.K, self.T)
        V_rtn, _ = faar.faar_init_v(self.W, s["sg"], s["scales"])
        rtn = float(faar.faar_hardened_loss(self.W, s["sg"], s["scales"], V_rtn, self.Xq, s["C"], self.alpha, ws,
                                            x_scale=self.x_scale).item())
        opt = float(faar.faar_hardened_loss(self.W, s["sg"], s["scales"], s["V"], self.Xq, s["C"], self.alpha, ws,
                                            x_scale=self.x_scale).item())
        return rtn, opt

    def probe_kernels(self, timer, n_probe, t_base, codec=True):
        """Per-kernel durations of this linear: name -> ms."""
        import paper_2603_22370_amd as faar
        from paper_2603_22370_amd import binding as fb
        s = self.state
        probe = {}

        def first_step_call(i):      # a layer's first step: its own forward kernel, nothing prepared for the next
            self.step(t_base + i, 0, beta=16.0, beta_next=0.0, forward_ready=False)

        def step_call(i):            # every later step: forward taken from / left in the workspace
            self.step(t_base + i, 0, beta=16.0, beta_next=16.0, forward_ready=i > 0)

        probe["softquant_fwd"] = timer.time(fb.K_SOFTQUANT_FWD, first_step_call, n_probe)
        gemms = ([("gemm_residual", fb.K_GEMM_RESIDUAL), ("gemm_dw", fb.K_GEMM_DW)] if self.form == "token"
                 else [("gemm_gram", fb.K_GEMM_GRAM)])
        for name, kid in gemms + [("bwd_adam", fb.K_BWD_ADAM)]:
            probe[name] = timer.time(kid, step_call, n_probe)
        if codec:
            probe["quant_rtn"] = timer.time(fb.K_QUANT_RTN, lambda i: faar.faar_quant_rtn(self.W, ws=self.ws_q), n_probe)
            probe["init_v"] = timer.time(fb.K_INIT_V, lambda i: faar.faar_init_v(self.W, s["sg"], s["scales"]), n_probe)
            probe["harden_pack"] = timer.time(fb.K_HARDEN_PACK,
                                              lambda i: faar.faar_harden_pack(self.W, s["sg"], s["scales"], s["V"]), n_probe)
        return probe

    def kernel_table(self, probe):
        gemm_flops = 2.0 * self.T * self.O * self.K if self.form == "token" else 2.0 * self.O * self.K * self.K
        bpw = bytes_per_weight(self.dw_split if self.form == "token" else self.gram_split, self.use_h)
        N = self.O * self.K
        # working set of one step: W, V, m, u, W_q - W, G partials, X_q, X_q^T, C, dY^T
        step_bytes = N * (2 + 12 + 2 + 4 * self.dw_split) + self.T * self.K * 4 + self.T * self.O * 6
        out = {}
        for name, ms in probe.items():
            if name.startswith("gemm"):
                ach = gemm_flops / (ms * 1e-3) / 1e12
                out[name] = {"ms": round(ms, 5), "bound": "mfma", "achieved": round(ach, 2), "unit": "TFLOP/s",
                             "frac": round(ach / BF16_PEAK_TFLOPS, 4)}
            else:
                ach = bpw[name] * N / (ms * 1e-3) / 1e9
                out[name] = {"ms": round(ms, 5), "bound": "hbm", "achieved": round(ach, 1), "unit": "GB/s",
                             "frac": round(ach / HBM_PEAK_GBS, 4)}
                if step_bytes < 256e6:     # the step's working set fits the 256 MB Infinity Cache: not an HBM rate
                    out[name]["note"] = "effective rate: working set resident in the Infinity Cache"
            # the dW GEMM has its own counter rows for the 192-wide tiles a step takes when it has the device to itself
            from paper_2603_22370_amd import binding as fb
            wide = (name == "gemm_dw" and self.form == "token" and self.whole_device
                    and fb.faar_dw_token_major(self.O, self.K, self.T, True) in (2, 3))
            out[name]["traffic"] = traffic_for(name + ("_whole_device" if wide else ""), self.O, self.K, self.T)
        return out


def oracle_step_time(job_inputs, seconds, max_steps=500):
    """Times fo.layer_step (exact mode) on host copies of one linear's inputs: (steps done, seconds)."""
    import numpy as np

    from oracle import faar_oracle as fo
    W_h, X_h, Y_h, alpha = job_inputs
    q = fo.quant_rtn(W_h, True)
    V0 = fo.init_v(W_h, q["s_global"], q["scales"])["V"]
    m0, u0 = np.zeros_like(V0), np.zeros_like(V0)
    n, t_cpu = 0, 0.0
    while n < 1 or (t_cpu < seconds and n < max_steps):
        c0 = time.perf_counter()
        r = fo.layer_step(W_h, q["s_global"], q["scales"], V0, m0, u0, X_h, Y_h, LinearJob.beta_at(n + 1, 500), LAM, alpha,
                          LR, 0.9, 0.999, 1e-8, n + 1)
        V0, m0, u0 = r["V"], r["m"], r["u"]
        t_cpu += time.perf_counter() - c0
        n += 1
    return n, t_cpu


def make_block_jobs(T, quantised_acts=False, form="token"):
    import torch

    from workloads import synth
    X_by_group, jobs = {}, []
    for idx, (name, O, K, group, gated) in enumerate(QWEN_BLOCK):
        if group not in X_by_group:
            X_h = synth.silu_gated_activations(T, K, seed=idx) if gated else synth.activations(T, K, seed=idx)
            X_by_group[group] = torch.from_numpy(X_h).cuda().to(torch.bfloat16)
        W = torch.from_numpy(synth.student_t_weight(O, K, seed=idx)).cuda().to(torch.bfloat16)
        jobs.append(LinearJob(name, O, K, T, W, X_by_group[group], quantised_acts, form))
    return jobs


def run_layer(args) -> dict:
    """The default: one Qwen3-1.7B-shaped layer, all seven linears, 8192 tokens (see the module docstring)."""
    import torch

    T = 8192
    gram = args.workload == "qwen_layer_gram"
    jobs = make_block_jobs(T, args.quantised_acts, "gram" if gram else "token")
    for j in jobs:                           # one stream: nothing runs beside a step, so it may take tiles that fill every unit
        j.whole_device = args.streams == 1 if args.whole_device == "auto" else args.whole_device == "on"
    torch.cuda.synchronize()
    # Stage 1 optimises every linear against frozen inputs: the seven jobs are independent, so they are issued on
    # several HIP streams (default priority).  While one job's workgroups sit in a GEMM epilogue or in the
    # memory-bound pass that updates V, compute units that fall idle pick up another job's GEMM tiles.
    by_name = {j.name: j for j in jobs}
    groups = {1: [["q_proj", "k_proj", "v_proj", "o_proj", "gate_proj", "up_proj", "down_proj"]],
              2: [["gate_proj", "q_proj", "k_proj", "v_proj", "o_proj"], ["up_proj", "down_proj"]],
              3: [["gate_proj", "q_proj", "k_proj"], ["up_proj", "v_proj", "o_proj"], ["down_proj"]]}[args.streams]
    streams = [torch.cuda.Stream() for _ in groups] if args.streams > 1 else [torch.cuda.current_stream()]

    def job_ops(j, n_steps):
        yield j.setup
        for t in range(1, n_steps + 1):
            yield lambda t=t: j.step(t, n_steps)
        yield j.finish

    def layer_job(n_steps):
        cur = torch.cuda.current_stream()
        for st in streams:
            st.wait_stream(cur)
        pending = [iter([op for name in g for op in job_ops(by_name[name], n_steps)]) for g in groups]
        streams_live = list(streams)
        while pending:                       # round-robin over the streams so that every queue stays fed
            for k in range(len(pending) - 1, -1, -1):
                op = next(pending[k], None)
                if op is None:
                    pending.pop(k)
                    streams_live.pop(k)
                    continue
                with torch.cuda.stream(streams_live[k]):
                    op()
        for st in streams:
            cur.wait_stream(st)

    # Untimed: first a 100-step job that only brings the process to its working state (code objects loaded, the runtime's
    # queues and signal pools at their working size, clocks settled: the first job of a process runs ~20 % slower whatever
    # its length), then the W warm-up steps asked for
    if args.warmup < 100:
        layer_job(100)
    layer_job(max(1, args.warmup))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    layer_job(args.steps)                    # timed region: exactly K steps of every linear inside whole per-layer jobs
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    n_lin = len(jobs)
    weights = sum(j.O * j.K for j in jobs)
    flops_per_set = sum(2.0 * j.O * j.K * j.K if gram else 2 * 2.0 * T * j.O * j.K for j in jobs)
    per_linear, timer = {}, KernelTimer()
    n_probe = max(5, args.probe_steps)
    for j in jobs:
        rtn, opt = j.hardened_losses()
        table = j.kernel_table(j.probe_kernels(timer, n_probe, args.steps + 1, codec=True))
        per_linear[j.name] = {"O": j.O, "K": j.K, "dw_split": j.dw_split, "gradient_constant": j.use_h, "final_losses": j.losses.cpu().numpy().tolist(),
                              "flipped_decisions": int(j.state["flips"].item()), "hardened_loss": {"rtn": rtn, "faar": opt},
                              "kernels": table}
    # the kernel that takes the largest share of a step of the whole layer
    dom_l, dom_k = max(((l, k) for l in per_linear for k in (("gemm_gram", "bwd_adam") if gram else ("gemm_residual", "gemm_dw", "bwd_adam"))),
                       key=lambda lk: per_linear[lk[0]]["kernels"][lk[1]]["ms"])
    dom = per_linear[dom_l]["kernels"][dom_k]
    ms_per_step = elapsed / args.steps * 1e3
    out = {
        "metric": "FAAR layer steps/sec (fwd+bwd+Adam)", "value": round(n_lin * args.steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": ("qwen_layer_gram (every step in its Gram-matrix form, faar_layer_step_gram: no layer output is formed; "
                                "NOT the default workload): " if gram else "qwen_layer: ") +
                               "the 7 linears of one Qwen3-1.7B-shaped layer (q/o 2048x2048, k/v 1024x2048, gate/up "
                               "6144x2048, down 2048x6144; bf16 Student-t(4) std 0.02), X 8192 tokens "
                               f"{'NVFP4-quantised (W4A4)' if args.quantised_acts else 'bf16'} with 1% outlier channels x30, "
                               "NVFP4 block 16; per linear: quant_rtn + init_v + prepare" + (" + gram_prepare" if gram else "") +
                               " + K steps + harden_pack; one timed step = "
                               f"one step of every linear; value = linear-layer steps/s; the 7 independent jobs issued on {args.streams} "
                               "HIP stream(s)",
                   "T": T, "linears": n_lin, "weights": weights, "streams": args.streams,
                   "whole_device_tiles": bool(jobs[0].whole_device)},
        "weight_elems_per_sec": round(weights * args.steps / elapsed, 1),
        "step_gemm_tflops": round(flops_per_set / (ms_per_step * 1e-3) / 1e12, 1),
        "roofline": {"kernel": f"{dom_l}.{dom_k}", "bound": dom["bound"], "achieved": dom["achieved"],
                     "peak": BF16_PEAK_TFLOPS if dom["bound"] == "mfma" else HBM_PEAK_GBS, "unit": dom["unit"],
                     "frac": dom["frac"], "traffic": dom["traffic"], "launch_ms": dom["ms"]},
        "per_linear": per_linear,
    }
    if not args.no_cpu_baseline:
        # the same number of steps of each of the seven linears (the layer's mix of shapes): 3 by default, about 10 s of
        # float64 products (2 x 824 GF per step of all seven)
        each = max(1, int(round(args.cpu_seconds / 5.0)))
        t_cpu, n_cpu = 0.0, 0
        for j in jobs:
            xs = j.x_scale if j.x_scale is not None else 1.0
            n, t = oracle_step_time((j.W.float().cpu().numpy(), (j.Xq.float() * xs).cpu().numpy(), j.Y.float().cpu().numpy(),
                                     j.alpha), seconds=1e9, max_steps=each)
            n_cpu += n
            t_cpu += t
        out["cpu_baseline"] = {"value": round(n_cpu / t_cpu, 4), "unit": "steps/s", "kind": "oracle",
                               "sample": f"{each} step(s) of each of the {len(jobs)} linears of the same layer ({t_cpu:.1f} s)",
                               **host_description()}
    return out


def run_linear(args) -> dict:
    """One linear layer's whole job (the shapes of WORKLOADS)."""
    import torch

    import paper_2603_22370_amd as faar
    from workloads import synth

    O, K, T, gated = WORKLOADS[args.workload]
    W_h = synth.student_t_weight(O, K, seed=0)
    X_h = synth.silu_gated_activations(T, K, seed=0) if gated else synth.activations(T, K, seed=0)
    W = torch.from_numpy(W_h).cuda().to(torch.bfloat16)
    Xq = torch.from_numpy(X_h).cuda().to(torch.bfloat16)
    j = LinearJob(args.workload, O, K, T, W, Xq, args.quantised_acts, args.form)
    j.whole_device = args.whole_device != "off"
    gram = args.form == "gram"
    torch.cuda.synchronize()

    def layer_job(n_steps):
        j.setup()
        for t in range(1, n_steps + 1):
            j.step(t, n_steps)
        j.finish()

    if args.warmup < 100:                    # untimed: brings the process to its working state (see run_layer)
        layer_job(100)
    layer_job(max(1, args.warmup))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    layer_job(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    final_losses = j.losses.cpu().numpy().tolist()
    n_flips = int(j.state["flips"].item())
    loss_rtn, loss_faar = j.hardened_losses()
    s = j.state
    stochastic = None
    if args.stochastic_trials > 0:
        trial = torch.empty(args.stochastic_trials, dtype=torch.float32, device="cuda")
        for k in range(args.stochastic_trials):
            Vs = faar.faar_stochastic_v(W, s["sg"], s["scales"], 2603, k)
            faar.faar_hardened_loss(W, s["sg"], s["scales"], Vs, j.Xq, s["C"], j.alpha,
                                    j.ws if not gram else faar.layer_step_workspace(O, K, T), x_scale=j.x_scale, loss=trial[k:k + 1])
        tl = trial.cpu().numpy()
        stochastic = {"trials": int(tl.size), "better_than_rtn": int((tl < loss_rtn).sum()), "best": float(tl.min()),
                      "mean": float(tl.mean()), "std": float(tl.std())}

    timer = KernelTimer()
    n_probe = max(5, args.probe_steps)
    probe = j.probe_kernels(timer, n_probe, args.steps + 1)
    # the stand-alone soft-quantisation entry point (forward + backward from a given dL/dW_q; it re-derives the
    # intervals from W and the scales on every call): torch events around the whole call, output allocation included
    dWt = torch.randn((O, K), device="cuda") * 1e-3
    te0, te1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(n_probe + 3):
        if i == 3:
            te0.record()
        faar.faar_softquant_fwd_bwd(W, s["sg"], s["scales"], s["V"], 16.0, dWt=dWt, lambda_round=LAM, emit_delta=True)
    te1.record()
    torch.cuda.synchronize()
    probe["softquant_fwd_bwd_call"] = te0.elapsed_time(te1) / n_probe
    del dWt
    kernels = j.kernel_table(probe)
    dom = max(("gemm_gram", "bwd_adam") if gram else ("gemm_residual", "gemm_dw", "bwd_adam"), key=lambda k: probe[k])
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
    gemm_flops = 2.0 * T * O * K if not gram else 1.0 * O * K * K      # per GEMM; two GEMMs (token form) or "half of two" (Gram form)
    out = {
        "metric": "FAAR layer steps/sec (fwd+bwd+Adam)", "value": round(args.steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}{' in the optional Gram-matrix form of the step (faar_layer_step_gram)' if gram else ''}: W {O}x{K} bf16 Student-t(4) std 0.02, X {T}x{K} "
                               f"{'NVFP4-quantised (W4A4)' if args.quantised_acts else 'bf16'}, NVFP4 block 16; "
                               "per-layer job = quant_rtn + init_v + prepare + K steps + harden_pack",
                   "O": O, "K": K, "T": T},
        "weight_elems_per_sec": round(O * K * args.steps / elapsed, 1),
        "step_gemm_tflops": round(2 * gemm_flops / (ms_per_step * 1e-3) / 1e12, 1),
        "dw_split": j.dw_split, "gradient_constant": j.use_h, "final_losses": final_losses, "flipped_decisions": n_flips,
        "hardened_loss": {"rtn": loss_rtn, "faar": loss_faar, "stochastic": stochastic},
        "roofline": roofline, "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        X_used = (j.Xq.float() * (j.x_scale if j.x_scale is not None else 1.0)).cpu().numpy()
        n_cpu, t_cpu = oracle_step_time((W_h, X_used, j.Y.float().cpu().numpy(), j.alpha), args.cpu_seconds)
        out["cpu_baseline"] = {"value": round(n_cpu / t_cpu, 4), "unit": "steps/s", "kind": "oracle",
                               "sample": f"{n_cpu} layer steps of the same {args.workload} layer ({t_cpu:.1f} s)",
                               **host_description()}
    return out


def run_block_chained(args) -> dict:
    """All seven linears of one Qwen3-1.7B-shaped block stepped back to back at T = 16384, each with an
    upstream gradient supplied (dY_ext) and its input gradient requested (dX): three GEMMs per linear and step.
    One timed "step" is one step of every linear; `value` counts linear-layer steps."""
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb

    T = 16384
    steps = min(args.steps, 50)
    warmup = min(args.warmup, 30)           # ~0.2 s under load before the timed region: the chip's clocks have settled
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    jobs = make_block_jobs(T)
    lin = []
    for j in jobs:
        j.use_h = True          # with dY from upstream the residual GEMM then only sums the loss
        j.setup()
        j.Y = None
        j.ws = None
        dY = (torch.randn((T, j.O), generator=gen, device="cuda") * 1e-3).to(torch.bfloat16)
        lin.append(dict(j=j, dY=dY, dX=torch.empty((T, j.K), dtype=torch.bfloat16, device="cuda"),
                        ws=faar.layer_step_workspace(j.O, j.K, T, chained=True), t=0, ready=False))

    def step_linear(L, beta=16.0):
        j, s = L["j"], L["j"].state
        L["t"] += 1
        faar.faar_layer_step(j.W, s["sg"], s["scales"], s["V"], s["m"], s["u"], j.Xq, s["Xt"], s["C"], s["ic"], beta,
                             LAM, j.alpha, LR, 0.9, 0.999, 1e-8, L["t"], j.losses, L["ws"], dY_ext=L["dY"],
                             dX=L["dX"], beta_next=beta, forward_ready=L["ready"], whole_device=True, **s["hk"])
        L["ready"] = True

    for _ in range(warmup):
        for L in lin:
            step_linear(L)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for L in lin:
            step_linear(L)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    timer = KernelTimer()
    per_linear = {}
    total_flops = 0.0
    for L in lin:
        j = L["j"]
        O, K = j.O, j.K
        flops = 2.0 * T * O * K
        total_flops += 3 * flops
        row = {}
        for kname, kid in [("gemm_residual", fb.K_GEMM_RESIDUAL), ("gemm_dw", fb.K_GEMM_DW), ("gemm_dx", fb.K_GEMM_DX),
                           ("bwd_adam", fb.K_BWD_ADAM)]:
            ms = timer.time(kid, lambda i: step_linear(L), 6)
            if kname.startswith("gemm"):
                row[kname] = {"ms": round(ms, 5), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                              "frac": round(flops / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, 4)}
            else:
                b = bytes_per_weight(j.dw_split, True)["bwd_adam"] + 2      # + W_q for the next dX
                row[kname] = {"ms": round(ms, 5), "gbs": round(b * O * K / (ms * 1e-3) / 1e9, 1),
                              "frac": round(b * O * K / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        row["dw_split"] = j.dw_split
        row["losses"] = j.losses.cpu().numpy().tolist()
        per_linear[j.name] = row
    dom_l, dom_k = max(((l, k) for l in per_linear for k in ("gemm_residual", "gemm_dw", "gemm_dx")),
                       key=lambda lk: per_linear[lk[0]][lk[1]]["ms"])
    dom = per_linear[dom_l][dom_k]
    n_lin = len(lin)
    out = {
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
    if not args.no_cpu_baseline:
        # the oracle's chained step (dY given, dX produced) on the smallest linear of the block, k_proj; the other six
        # are scaled by their share of the products: labelled as extrapolated
        import numpy as np

        from oracle import faar_oracle as fo
        L = lin[1]
        j = L["j"]
        W_h, X_h = j.W.float().cpu().numpy(), j.Xq.float().cpu().numpy()
        Y_h = (j.Xq @ j.W.T).float().cpu().numpy()
        dY_h = L["dY"].float().cpu().numpy()
        q = fo.quant_rtn(W_h, True)
        V0 = fo.init_v(W_h, q["s_global"], q["scales"])["V"]
        z = np.zeros_like(V0)
        n, t_cpu = 0, 0.0
        while n < 1 or (t_cpu < args.cpu_seconds and n < 20):
            c0 = time.perf_counter()
            fo.layer_step(W_h, q["s_global"], q["scales"], V0, z, z, X_h, Y_h, 16.0, LAM, j.alpha, LR, 0.9, 0.999, 1e-8, n + 1,
                          want_dX=True, dY_ext=dY_h)
            t_cpu += time.perf_counter() - c0
            n += 1
        share = (j.O * j.K) / sum(x["j"].O * x["j"].K for x in lin)
        out["cpu_baseline"] = {"value": round(n_lin / (t_cpu / n / share), 4), "unit": "steps/s", "kind": "oracle",
                               "sample": f"{n} chained steps of k_proj 1024x2048 at T 16384 measured ({t_cpu / n:.2f} s each); the block's "
                                         f"7 linears extrapolated by weight count (k_proj is {share:.3f} of the block)",
                               **host_description()}
    return out


def run_mlp_joint(args) -> dict:
    """One joint step of the MLP half of a Qwen3-1.7B-shaped block at T = 16384: RMSNorm, gate / up projections,
    SiLU * up, down projection, residual and block-output MSE forward; then the gradient back through all of it into
    the rounding variables of the three linears (one Adam update each) and into the block's input.  Nine GEMMs per
    step.  `value` counts linear-layer steps (three per block step)."""
    import numpy as np
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb
    from workloads import synth

    T, D, F = 16384, 2048, 6144
    steps, warmup = min(args.steps, 100), min(args.warmup, 30)
    beta, eps, ms_scale = 16.0, 1e-6, 1.0 / (T * D)
    shapes = (("gate", F, D), ("up", F, D), ("down", D, F))
    x_h = synth.activations(T, D, 31)
    x = torch.from_numpy(x_h).cuda().to(torch.bfloat16)
    g = torch.ones(D, dtype=torch.float32, device="cuda")
    lin = {}
    for i, (n, O, K) in enumerate(shapes):
        W = torch.from_numpy(synth.student_t_weight(O, K, 40 + i)).cuda().to(torch.bfloat16)
        sg, sc, _, _ = faar.faar_quant_rtn(W)
        V, _ = faar.faar_init_v(W, sg, sc)
        X0 = torch.zeros((T, K), dtype=torch.bfloat16, device="cuda")
        Xt, _, ic = faar.faar_layer_prepare(W, sg, sc, X0, None)          # only the node codes depend on W alone
        lin[n] = dict(W=W, sg=sg, sc=sc, V=V, m=torch.zeros_like(V), u=torch.zeros_like(V), Xt=Xt, ic=ic, O=O, K=K, t=0,
                      losses=torch.zeros(3, dtype=torch.float32, device="cuda"),
                      ws=faar.layer_step_workspace(O, K, T, chained=True), fws=fb._workspace(fb.OP_LINEAR_FORWARD, O, K, T, device="cuda"),
                      Y=torch.empty((T, O), dtype=torch.bfloat16, device="cuda"),
                      dX=torch.empty((T, K), dtype=torch.bfloat16, device="cuda"))
        del X0
    # the full-precision block's output: the same MLP with the unquantised weights, computed once with library GEMMs
    with torch.no_grad():
        xf = x.float()
        hf = (xf * torch.rsqrt((xf * xf).mean(-1, keepdim=True) + eps)).to(torch.bfloat16)
        pf, qf = hf @ lin["gate"]["W"].T, hf @ lin["up"]["W"].T
        y_fp = (xf + ((torch.nn.functional.silu(pf.float()) * qf.float()).to(torch.bfloat16) @ lin["down"]["W"].T).float()).to(torch.bfloat16)
        del xf, hf, pf, qf
    state = {"loss": None}

    def fwd(n, X):
        L = lin[n]
        return faar.faar_linear_forward(L["W"], L["sg"], L["sc"], L["V"], beta, X, ws=L["fws"], out=L["Y"])

    def back(n, X, dY):
        L = lin[n]
        L["t"] += 1
        faar.faar_layer_step(L["W"], L["sg"], L["sc"], L["V"], L["m"], L["u"], X, L["Xt"], None, L["ic"], beta, LAM, 0.0, LR,
                             0.9, 0.999, 1e-8, L["t"], L["losses"], L["ws"], dY_ext=dY, dX=L["dX"], joint=True)
        return L["dX"]

    def block_step():
        h, rstd = faar.faar_rmsnorm_fwd(x, g, eps)
        p, q = fwd("gate", h), fwd("up", h)
        a = faar.faar_silu_mul_fwd(p, q)
        d = fwd("down", a)
        state["loss"], dy, _ = faar.faar_block_output_loss(x, d, y_fp, ms_scale)
        da = back("down", a, dy)
        dp, dq = faar.faar_silu_mul_bwd(da, p, q)
        dh1, dh2 = back("gate", h, dp), back("up", h, dq)
        return faar.faar_rmsnorm_bwd(dh1, x, g, rstd, dh2=dh2, d_res=dy)

    for _ in range(warmup):
        block_step()
    torch.cuda.synchronize()
    first_loss = float(state["loss"].item())
    t0 = time.perf_counter()
    for _ in range(steps):
        block_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    timer = KernelTimer()
    kernels = {}
    flops = 2.0 * T * F * D
    for kname, kid in [("gemm_fwd", fb.K_GEMM_FWD), ("gemm_dw", fb.K_GEMM_DW), ("gemm_dx", fb.K_GEMM_DX), ("bwd_adam", fb.K_BWD_ADAM)]:
        # three launches of each per block step, of equal size; the last one is timed (down_proj's forward GEMM,
        # up_proj's backward kernels)
        ms = timer.time(kid, lambda i: block_step(), 4, position=-1)
        if kname.startswith("gemm"):
            kernels[kname] = {"ms": round(ms, 5), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                              "frac": round(flops / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, 4)}
        else:
            kernels[kname] = {"ms": round(ms, 5)}
    dom_k = max((k for k in kernels if k.startswith("gemm")), key=lambda k: kernels[k]["ms"])
    dom = kernels[dom_k]
    gemm_ms = 3 * sum(kernels[k]["ms"] for k in kernels if k.startswith("gemm"))
    out = {
        "metric": "FAAR layer steps/sec (fwd+bwd+Adam)", "value": round(3 * steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "qwen_mlp_joint: the MLP half of one Qwen3-1.7B-shaped block (RMSNorm, gate/up 6144x2048, SiLU*, "
                               "down 2048x6144, residual, block-output MSE), T 16384, one joint step = forward + backward + Adam "
                               "on the rounding variables of all three linears (9 GEMMs); value = linear-layer steps/s",
                   "T": T, "D": D, "F": F, "linears": 3},
        "block_step_gemm_tflops": round(9 * flops / (elapsed / steps) / 1e12, 1),
        "gemm_share_of_step": round(gemm_ms / (elapsed / steps * 1e3), 3),
        "block_loss": {"after_warmup": first_loss, "at_end": float(state["loss"].item())},
        "roofline": {"kernel": dom_k, "bound": "mfma", "achieved": dom["tflops"], "peak": BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": dom["frac"], "traffic": None, "launch_ms": dom["ms"]},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        # the oracle's joint step at two small token counts; its cost is linear in T (a part per weight plus a part per
        # token), extrapolated to T = 16384 and labelled so
        from oracle import block_oracle as bo
        from oracle import faar_oracle as fo
        layers = {}
        for n in lin:
            W_h = lin[n]["W"].float().cpu().numpy()
            qh = fo.quant_rtn(W_h, True)
            layers[n] = (W_h, qh["s_global"], qh["scales"], fo.init_v(W_h, qh["s_global"], qh["scales"])["V"])
        times = {}
        for Ts in (256, 512):
            xs, ys = x_h[:Ts].astype(np.float64), y_fp[:Ts].float().cpu().numpy()
            c0 = time.perf_counter()
            bo.mlp_block_step(xs, np.ones(D), eps, layers, ys, 1.0 / (Ts * D), beta, LAM, bf16_storage=True)
            times[Ts] = time.perf_counter() - c0
        per_tok = max(times[512] - times[256], 0.0) / 256
        t_full = times[256] + per_tok * (T - 256)
        out["cpu_baseline"] = {"value": round(3 / t_full, 5), "unit": "steps/s", "kind": "oracle",
                               "sample": f"joint MLP step of the oracle (gradients only, no Adam) at T 256 ({times[256]:.1f} s) and T 512 "
                                         f"({times[512]:.1f} s), extrapolated linearly in T to 16384 ({t_full:.0f} s per block step)",
                               **host_description()}
    return out


def run_block_joint(args) -> dict:
    """One joint step of a whole Qwen3-1.7B-shaped block at T = 16384 (32 sequences of 512 tokens): RMSNorm, q / k / v
    projections, per-head norm, rotary embedding, causal grouped-query attention (16 query heads on 8 key / value heads of
    128), output projection, residual, RMSNorm, gated-SiLU MLP, residual, squared error against the full-precision block's
    output; then the gradient back through all of it into the rounding variables of the seven linears (one Adam update
    each) and into the block's input.  One call of faar_block_joint_step per step; 21 GEMMs.  `value` counts linear-layer
    steps (seven per block step)."""
    import numpy as np
    import torch

    import paper_2603_22370_amd as faar
    from paper_2603_22370_amd import binding as fb
    from workloads import synth

    n_seq, S, D, n_q, n_kv, dh, F = 32, 512, 2048, 16, 8, 128, 6144
    T = n_seq * S
    steps, warmup = min(args.steps, 100), min(args.warmup, 30)
    beta, eps, ms_scale = 16.0, 1e-6, 1.0 / (T * D)
    shapes = dict(q=(n_q * dh, D), k=(n_kv * dh, D), v=(n_kv * dh, D), o=(D, n_q * dh), gate=(F, D), up=(F, D), down=(D, F))
    x_h = synth.activations(T, D, 51)
    x = torch.from_numpy(x_h).cuda().to(torch.bfloat16)
    ones_d, ones_h = torch.ones(D, dtype=torch.float32, device="cuda"), torch.ones(dh, dtype=torch.float32, device="cuda")
    inv = 1.0e6 ** (-np.arange(dh // 2) * 2.0 / dh)                    # rotary base of the Qwen3 models
    ang = np.arange(S)[:, None] * inv[None, :]
    cos_h, sin_h = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    cos_t, sin_t = torch.from_numpy(cos_h).cuda(), torch.from_numpy(sin_h).cuda()
    lin, W_h = {}, {}
    for i, (n, (O, K)) in enumerate(shapes.items()):
        W_h[n] = synth.student_t_weight(O, K, 60 + i)
        W = torch.from_numpy(W_h[n]).cuda().to(torch.bfloat16)
        sg, sc, _, _ = faar.faar_quant_rtn(W)
        V, _ = faar.faar_init_v(W, sg, sc)
        _, _, ic = faar.faar_layer_prepare(W, sg, sc, torch.zeros((T, K), dtype=torch.bfloat16, device="cuda"), None)
        lin[n] = dict(W=W, s_global=sg, scales=sc, icodes=ic, V=V, m=torch.zeros_like(V), u=torch.zeros_like(V),
                      losses=torch.zeros(3, dtype=torch.float32, device="cuda"))
    # the full-precision block's output, from library ops on the unquantised weights (input synthesis, outside the path)
    with torch.no_grad():
        def norm(t, width):
            tf = t.float()
            return (tf * torch.rsqrt((tf * tf).mean(-1, keepdim=True) + eps)).to(torch.bfloat16)

        def rot(t, H):
            th = t.float().view(T, H, dh)
            c = cos_t.repeat(n_seq, 2)[:, None, :]
            s_ = sin_t.repeat(n_seq, 2)[:, None, :]
            half = torch.cat([-th[..., dh // 2:], th[..., :dh // 2]], dim=-1)
            return (th * c + half * s_).to(torch.bfloat16).view(T, H * dh)

        h = norm(x, D)
        q, k, v = (h @ lin[n]["W"].T for n in ("q", "k", "v"))
        q, k = rot(norm(q.view(T * n_q, dh), dh).view(T, -1), n_q), rot(norm(k.view(T * n_kv, dh), dh).view(T, -1), n_kv)
        sp = lambda t, H: t.view(n_seq, S, H, dh).permute(0, 2, 1, 3)
        o = torch.nn.functional.scaled_dot_product_attention(sp(q, n_q), sp(k, n_kv).repeat_interleave(n_q // n_kv, dim=1),
                                                             sp(v, n_kv).repeat_interleave(n_q // n_kv, dim=1), is_causal=True)
        x1 = (x.float() + (o.permute(0, 2, 1, 3).reshape(T, n_q * dh) @ lin["o"]["W"].T).float()).to(torch.bfloat16)
        h2 = norm(x1, D)
        a = (torch.nn.functional.silu((h2 @ lin["gate"]["W"].T).float()) * (h2 @ lin["up"]["W"].T).float()).to(torch.bfloat16)
        y_fp = (x1.float() + (a @ lin["down"]["W"].T).float()).to(torch.bfloat16)
        del h, q, k, v, o, x1, h2, a
    blk = faar.block_description(n_seq, S, D, n_q, n_kv, dh, F, eps, ones_d, ones_d.clone(), cos_t, sin_t, lin, g_q=ones_h, g_k=ones_h.clone())
    ws = faar.faar_block_workspace(blk)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    dx_keep = {}
    state = {"t": 0}

    def block_step():
        state["t"] += 1
        _, dx_keep["dx"] = faar.faar_block_joint_step(blk, x, y_fp, ms_scale, beta, LAM, LR, 0.9, 0.999, 1e-8, state["t"], ws,
                                                      block_loss=loss)

    for _ in range(warmup):
        block_step()
    torch.cuda.synchronize()
    first_loss = float(loss.item())
    t0 = time.perf_counter()
    for _ in range(steps):
        block_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    timer = KernelTimer()
    kernels = {}
    flops_mlp = 2.0 * T * F * D
    for kname, kid, fl, what in [("gemm_fwd", fb.K_GEMM_FWD, flops_mlp, "down_proj forward"), ("gemm_dw", fb.K_GEMM_DW, 2.0 * T * n_kv * dh * D, "v_proj dW"),
                                 ("gemm_dx", fb.K_GEMM_DX, 2.0 * T * n_kv * dh * D, "v_proj dX"), ("bwd_adam", fb.K_BWD_ADAM, 0.0, "v_proj"),
                                 ("attention_fwd", fb.K_ATTENTION_FWD, 2.0 * n_seq * n_q * S * S * dh, "causal: half the S x S scores count"),
                                 ("attention_bwd", fb.K_ATTENTION_BWD, 5.0 * n_seq * n_q * S * S * dh, "three kernels; causal half of five S x S x dh products")]:
        ms = timer.time(kid, lambda i: block_step(), 4, position=-1)     # the last launch of that kernel in a block step
        row = {"ms": round(ms, 5), "launch": what}
        if fl:
            row["tflops"] = round(fl / (ms * 1e-3) / 1e12, 1)
            row["frac"] = round(fl / (ms * 1e-3) / 1e12 / BF16_PEAK_TFLOPS, 4)
        kernels[kname] = row
    gemm_flops = 3 * 2.0 * T * (2 * n_q * dh * D + 2 * n_kv * dh * D + 3 * F * D)
    attn_flops = 7.0 * n_seq * n_q * S * S * dh
    dom = kernels["gemm_fwd"]
    out = {
        "metric": "FAAR layer steps/sec (fwd+bwd+Adam)", "value": round(7 * steps / elapsed, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "qwen_block_joint: one joint step of a whole Qwen3-1.7B-shaped block (attention half with per-head norm, "
                               "rotary embedding and causal grouped-query attention 16/8 heads of 128; gated-SiLU MLP 6144; residuals; "
                               "block-output MSE), 32 sequences of 512 tokens, forward + backward + Adam on the rounding variables of "
                               "all seven linears (21 GEMMs) by one faar_block_joint_step call; value = linear-layer steps/s",
                   "T": T, "n_seq": n_seq, "S": S, "D": D, "F": F, "n_q": n_q, "n_kv": n_kv, "dh": dh, "linears": 7},
        "block_step_tflops": round((gemm_flops + attn_flops) / (elapsed / steps) / 1e12, 1),
        "block_loss": {"after_warmup": first_loss, "at_end": float(loss.item())},
        "roofline": {"kernel": "gemm_fwd (down_proj forward, 16384 x 2048 x 6144)", "bound": "mfma", "achieved": dom["tflops"],
                     "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": dom["frac"], "traffic": None, "launch_ms": dom["ms"]},
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        # the oracle's joint block step on one and on two sequences of 512 tokens; its cost is a part per weight plus a part per
        # sequence, extrapolated linearly to 32 sequences and labelled so
        from oracle import block_oracle as bo
        from oracle import faar_oracle as fo
        layers = {}
        for n in lin:
            qh = fo.quant_rtn(W_h[n], True)
            layers[n] = (W_h[n], qh["s_global"], qh["scales"], fo.init_v(W_h[n], qh["s_global"], qh["scales"])["V"])
        attn_l, mlp_l = {n: layers[n] for n in ("q", "k", "v", "o")}, {n: layers[n] for n in ("gate", "up", "down")}
        one = np.ones(D)
        times = {}
        for ns in (1, 2):
            Ts = ns * S
            xs, ys = x_h[:Ts].astype(np.float64), y_fp[:Ts].float().cpu().numpy()
            c0 = time.perf_counter()
            a0 = bo.attn_block_step(xs, one, eps, attn_l, ns, n_q, n_kv, dh, cos_h, sin_h, beta, LAM, d_out=np.zeros((Ts, D)),
                                    qk_norm=(np.ones(dh), np.ones(dh)), bf16_storage=True)
            m = bo.mlp_block_step(a0["y"], one, eps, mlp_l, ys, 1.0 / (Ts * D), beta, LAM, bf16_storage=True)
            bo.attn_block_step(xs, one, eps, attn_l, ns, n_q, n_kv, dh, cos_h, sin_h, beta, LAM, d_out=m["dx"],
                               qk_norm=(np.ones(dh), np.ones(dh)), bf16_storage=True)
            times[ns] = time.perf_counter() - c0
        per_seq = max(times[2] - times[1], 0.0)
        t_full = times[1] + per_seq * (n_seq - 1)
        out["cpu_baseline"] = {"value": round(7 / t_full, 5), "unit": "steps/s", "kind": "oracle",
                               "sample": f"joint block step of the oracle (gradients only, no Adam; its attention half evaluated twice) on 1 "
                                         f"sequence ({times[1]:.1f} s) and 2 sequences ({times[2]:.1f} s) of 512 tokens, extrapolated linearly "
                                         f"to 32 sequences ({t_full:.0f} s per block step)",
                               **host_description()}
    return out


def run_pack_sweep(args) -> dict:
    """Set-up and tear-down over every linear of a Qwen3-1.7B-shaped model (28 layers x 7 linears, 1.409 G weights,
    each tensor in memory of its own): quantisation, V initialisation and hardening + packing, each as ONE batched call
    over all 196 tensors (5 launches of up to 48 tensors), outputs preallocated.  `value` is the harden+pack rate.
    The same sweeps as 196 single-tensor calls are reported beside them."""
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
    Ws, Vs, sgs, scs, cds = [], [], [], [], []
    n_total = 0
    for layer in range(QWEN_LAYERS):
        for name, O, K, _, _ in QWEN_BLOCK:
            Ws.append(base[(O, K)].clone())
            Vs.append(torch.rand((O, K), generator=gen, device="cuda", dtype=torch.float32))   # rounding variables mid-optimisation
            sgs.append(torch.empty(1, dtype=torch.float32, device="cuda"))
            scs.append(torch.empty((O, K // 16), dtype=torch.uint8, device="cuda"))
            cds.append(torch.empty((O, K // 2), dtype=torch.uint8, device="cuda"))
            n_total += O * K
    ws_b = torch.empty(faar.faar_workspace_bytes(fb.OP_QUANT_RTN_BATCH, 16, 16), dtype=torch.uint8, device="cuda")
    ws_q = torch.empty(faar.faar_workspace_bytes(fb.OP_QUANT_RTN, 6144, 2048), dtype=torch.uint8, device="cuda")
    items_q, dt = faar.tensor_batch(Ws, sgs, scs, codes=cds)
    Vout = [torch.empty_like(v) for v in Vs]         # V initialisation writes 5.6 GB: every tensor gets its own output
    items_i, _ = faar.tensor_batch(Ws, sgs, scs, Vs=Vout)
    items_p, _ = faar.tensor_batch(Ws, sgs, scs, Vs=Vs, codes=cds)
    reps = max(3, min(args.steps, 10))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def sweep(fn):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            dt_ms = e0.elapsed_time(e1)
            best = dt_ms if best is None else min(best, dt_ms)
        return best * 1e-3

    L = fb.lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())

    def single_quant():
        for k, W in enumerate(Ws):
            L.faar_quant_rtn(ptr(W), 1, W.shape[0], W.shape[1], ptr(sgs[k]), ptr(scs[k]), ptr(cds[k]), None, 0, ptr(ws_q), ws_q.numel(), st)

    def single_init():
        for k, W in enumerate(Ws):
            L.faar_init_v(ptr(W), 1, W.shape[0], W.shape[1], ptr(sgs[k]), ptr(scs[k]), ptr(Vout[k]), None, st)

    def single_pack():
        for k, W in enumerate(Ws):
            L.faar_harden_pack(ptr(W), 1, W.shape[0], W.shape[1], ptr(sgs[k]), ptr(scs[k]), ptr(Vs[k]), ptr(cds[k]), None, None, None, st)

    t = {"quant_rtn": sweep(lambda: faar.faar_quant_rtn_batch(items_q, dt, ws_b)),
         "init_v": sweep(lambda: faar.faar_init_v_batch(items_i, dt)),
         "harden_pack": sweep(lambda: faar.faar_harden_pack_batch(items_p, dt))}
    t1 = {"quant_rtn": sweep(single_quant), "init_v": sweep(single_init), "harden_pack": sweep(single_pack)}
    bpw = bytes_per_weight(1)
    bytes_of = {"quant_rtn": bpw["quant_rtn"] + 2, "init_v": bpw["init_v"], "harden_pack": bpw["harden_pack"]}
    rows = {}
    for name in t:
        b = bytes_of[name]
        rows[name] = {"ms": round(t[name] * 1e3, 3), "gbs": round(b * n_total / t[name] / 1e9, 1),
                      "frac": round(b * n_total / t[name] / 1e9 / HBM_PEAK_GBS, 4), "bytes_per_weight": b,
                      "single_tensor_calls_ms": round(t1[name] * 1e3, 3),
                      "single_tensor_calls_gbs": round(b * n_total / t1[name] / 1e9, 1)}
    out = {
        "metric": "NVFP4 harden+pack weight elements/sec", "value": round(n_total / t["harden_pack"], 1), "unit": "elems/s",
        "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": rows["harden_pack"]["ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"qwen_pack_sweep: {len(Ws)} weight tensors of a Qwen3-1.7B-shaped model "
                               f"({n_total / 1e9:.3f} G weights, bf16 W + float32 V in, NVFP4 codes out), one batched call per "
                               f"operation; best of {reps} sweeps, GPU time between events on the launch stream",
                   "weights": n_total},
        "roofline": {"kernel": "harden_pack (batched)", "bound": "hbm", "achieved": rows["harden_pack"]["gbs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": rows["harden_pack"]["frac"], "traffic": None, "launch_ms": rows["harden_pack"]["ms"]},
        "sweeps": rows,
    }
    if not args.no_cpu_baseline:
        # the oracle's quantise / initialise / harden+pack on the smallest tensor of the model (k_proj, 2.1 M weights);
        # the model's 1.409 G weights are extrapolated linearly (the work is O(N))
        from oracle import faar_oracle as fo
        W_h = base[(1024, 2048)].float().cpu().numpy()
        V_h = Vs[1].cpu().numpy()
        n, t_cpu = 0, 0.0
        while n < 1 or (t_cpu < args.cpu_seconds and n < 100):
            c0 = time.perf_counter()
            q = fo.quant_rtn(W_h, True)
            fo.init_v(W_h, q["s_global"], q["scales"])
            fo.harden_pack(W_h, True, q["s_global"], q["scales"], V_h)
            t_cpu += time.perf_counter() - c0
            n += 1
        out["cpu_baseline"] = {"value": round(W_h.size * n / t_cpu, 1), "unit": "elems/s", "kind": "oracle",
                               "sample": f"quantise + initialise + harden+pack of one k_proj tensor (2.1 M weights) {n} times "
                                         f"({t_cpu:.1f} s); all three operations, so a lower bound of the pack rate; the model's "
                                         "196 tensors extrapolated linearly (O(N) work)",
                               **host_description()}
    return out


def run_stage2(args) -> dict:
    """faar_stage2_losses on Llama3-1B-shaped model outputs: 4096 tokens, vocabulary 128256, hidden size 2048,
    bf16 logits and hidden states, losses and both gradients.  One timed step = one call."""
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
    steps, warmup = min(args.steps, 100), min(args.warmup, 30)
    for _ in range(max(1, warmup)):
        losses, dZ, dH = faar.faar_stage2_losses(Zf, Zq, tau, Hf, Hq, **kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        losses, dZ, dH = faar.faar_stage2_losses(Zf, Zq, tau, Hf, Hq, **kw)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = KernelTimer().time(fb.K_STAGE2_KL, lambda i: faar.faar_stage2_losses(Zf, Zq, tau, Hf, Hq, **kw), 8)
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
        rows = 64
        zf, zq = Zf[:rows].float().cpu().numpy(), Zq[:rows].float().cpu().numpy()
        hf, hq = Hf[:rows].float().cpu().numpy(), Hq[:rows].float().cpu().numpy()
        n, t_cpu = 0, 0.0
        while n < 1 or (t_cpu < args.cpu_seconds and n < 50):
            c0 = time.perf_counter()
            fo.stage2_losses(zf, zq, tau, 1.0 / T, hf, hq, 1.0 / (T * D), rl.cpu().numpy(), 1.0, 0.01)
            t_cpu += time.perf_counter() - c0
            n += 1
        out["cpu_baseline"] = {"value": round(n * rows / T / t_cpu, 5), "unit": "steps/s", "kind": "oracle",
                               "sample": f"{n} evaluations of {rows} of the {T} token rows ({t_cpu:.1f} s), "
                                         "scaled to whole steps", **host_description()}
    return out


def run_gemm_ceiling(args) -> dict:
    """What bounds the GEMM main loop, measured through the library's own kernel (faar_gemm_probe) on one product
    (default: the Llama3-1B-shaped gate_proj dW GEMM, 8192 x 2048 outputs, contraction over 4096 tokens), random bf16 operands: the
    loop with only its matrix instructions (operands read from LDS, nothing copied), with only its global->LDS copies,
    and whole -- each with the core clock the compute units ran at (shader clock counter / constant 100 MHz counter), in
    steady state; then with the operands evicted from the last-level cache before every launch, and the vendor library."""
    import torch

    from paper_2603_22370_amd import binding as fb

    M, N, Kd = (int(v) for v in args.gemm_shape.split(","))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    A = torch.randn((M, Kd), generator=gen, device="cuda").to(torch.bfloat16)
    B = torch.randn((N, Kd), generator=gen, device="cuda").to(torch.bfloat16)
    A0, B0 = torch.zeros_like(A), torch.zeros_like(B)
    flops = 2.0 * M * N * Kd
    est_ms = flops / 1.0e12                                   # ~1 PFLOP/s: only sizes the loops below
    n_warm, n_time = max(10, int(80.0 / est_ms)), max(10, int(25.0 / est_ms))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rows = {}

    def row_of(us, clocks, variant, with_flops=True):
        c = clocks.cpu().numpy().astype("float64")
        core, wall = c[:, 0], c[:, 1]
        mhz = float((core / (wall / 100.0)).mean())            # the constant counter ticks at 100 MHz
        row = {"us": round(us, 1), "core_mhz": round(mhz, 0), "core_cycles_per_item": round(float(core.mean()), 0), "variant": variant}
        if with_flops:
            row["tflops"] = round(flops / us / 1e6, 1)
            row["frac_of_published_peak"] = round(flops / us / 1e6 / BF16_PEAK_TFLOPS, 4)
            # what the matrix cores can deliver at the clock they actually ran at
            row["frac_of_peak_at_measured_clock"] = round(flops / us / 1e6 / (BF16_PEAK_TFLOPS * mhz / 2400.0), 4)
        return row

    # steady state: ~80 ms of back-to-back launches before the timed ones (from idle the clocks take tens of ms to settle)
    for label, mode, a, b in (("whole loop", fb.PROBE_FULL, A, B), ("matrix instructions only", fb.PROBE_MFMA_ONLY, A, B),
                              ("copies only", fb.PROBE_DMA_ONLY, A, B), ("whole loop, all-zero operands", fb.PROBE_FULL, A0, B0)):
        for _ in range(n_warm):
            clocks, variant = fb.faar_gemm_probe(mode, a, b)
        e0.record()
        for _ in range(n_time):
            clocks, variant = fb.faar_gemm_probe(mode, a, b)
        e1.record()
        torch.cuda.synchronize()
        rows[label] = row_of(e0.elapsed_time(e1) / n_time * 1e3, clocks, variant, mode != fb.PROBE_DMA_ONLY)
    # the token-major form of the same product (the buffers read as [Kd, M] and [Kd, N]: same bytes, transposing LDS reads),
    # on 256 x 256 tiles and on the 192-wide tiles a step that has the device to itself may take
    if fb.faar_dw_token_major(M, N, Kd):
        for label, mode in (("whole loop, token-major operands", fb.PROBE_FULL + fb.PROBE_TOKEN_MAJOR),
                            ("matrix instructions only, token-major operands", fb.PROBE_MFMA_ONLY + fb.PROBE_TOKEN_MAJOR),
                            ("whole loop, token-major operands, 192-wide tiles", fb.PROBE_TOKEN_MAJOR_192)):
            for _ in range(n_warm):
                clocks, variant = fb.faar_gemm_probe(mode, A, B)
            e0.record()
            for _ in range(n_time):
                clocks, variant = fb.faar_gemm_probe(mode, A, B)
            e1.record()
            torch.cuda.synchronize()
            rows[label] = row_of(e0.elapsed_time(e1) / n_time * 1e3, clocks, variant)
    # the same loops when the operands are NOT in the 256 MB last-level cache, as a step's dW GEMM finds them: 512 MB are
    # read (nothing written) before every launch; the events bracket the launch alone
    evict = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").view(torch.int32)
    n_cold = max(40, n_time)
    for label, mode in (("whole loop, operands from HBM", fb.PROBE_FULL), ("copies only, operands from HBM", fb.PROBE_DMA_ONLY)):
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_cold)]
        for x, y in pairs:
            evict.sum()
            x.record()
            clocks, variant = fb.faar_gemm_probe(mode, A, B)
            y.record()
        torch.cuda.synchronize()
        ts = [x.elapsed_time(y) * 1e3 for x, y in pairs[n_cold // 2:]]
        rows[label] = row_of(sum(ts) / len(ts), clocks, variant, mode != fb.PROBE_DMA_ONLY)
    # the vendor GEMM library on the same operands (a plain product with a bf16 output), same schedule
    Bt = B.t()
    for _ in range(n_warm):
        C = A @ Bt
    e0.record()
    for _ in range(n_time):
        C = A @ Bt
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / n_time * 1e3
    rows["vendor library product (torch.matmul), with its bf16 output"] = {
        "us": round(us, 1), "tflops": round(flops / us / 1e6, 1), "frac_of_published_peak": round(flops / us / 1e6 / BF16_PEAK_TFLOPS, 4)}
    whole = rows["whole loop"]
    return {
        "metric": "GEMM main-loop ceiling", "value": whole["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": n_time, "warmup": n_warm,
        "ms_per_step": round(whole["us"] * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"gemm_ceiling: {M}x{N} outputs, contraction {Kd}, bf16 N(0,1) operands, float32 output", "M": M, "N": N, "Kd": Kd},
        "roofline": {"kernel": f"gemm main loop ({whole['variant']})", "bound": "mfma", "achieved": whole["tflops"],
                     "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": whole["frac_of_published_peak"], "traffic": None,
                     "launch_ms": round(whole["us"] * 1e-3, 5)},
        "modes": rows,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 500 steps per layer is the job length of the workload list; the untimed warm-up is a 100-step job of the same kind:
    # the chip needs about 0.2 s under load before its clocks settle (the first 100 steps after idling run ~20 % slower)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="qwen_layer",
                    choices=["qwen_layer", "qwen_layer_gram"] + sorted(WORKLOADS) + ["qwen_block_chained", "qwen_mlp_joint", "qwen_block_joint", "qwen_pack_sweep", "stage2_losses", "gemm_ceiling"])
    ap.add_argument("--quantised-acts", action="store_true",
                    help="W4A4: quantise the activations to NVFP4 with the same kernel and feed them as (units, tensor scale)")
    ap.add_argument("--stochastic-trials", type=int, default=0,
                    help="single-linear workloads: after the job, rank this many stochastic-rounding candidates by hardened reconstruction loss")
    ap.add_argument("--gemm-shape", default="8192,2048,4096",
                    help="gemm_ceiling: outputs M x N and contraction, default the Llama3-1B-shaped gate_proj dW GEMM")
    ap.add_argument("--form", default="token", choices=["token", "gram"],
                    help="single-linear workloads: faar_layer_step (token) or the optional faar_layer_step_gram (gram)")
    ap.add_argument("--streams", type=int, default=3, choices=[1, 2, 3],
                    help="qwen_layer: HIP streams the seven independent per-linear jobs are issued on")
    ap.add_argument("--whole-device", default="auto", choices=["auto", "on", "off"],
                    help="layer jobs: step with FAAR_STEP_WHOLE_DEVICE (auto: when the jobs are issued on one stream)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--probe-steps", type=int, default=12)
    ap.add_argument("--calib-copy", action="store_true",
                    help="single-linear workloads: also run a plain 256 MiB device copy three times (reference for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path has no collectives or sharding "
              "(layers and output rows are independent jobs: shard those across processes). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    runners = {"qwen_layer": run_layer, "qwen_layer_gram": run_layer, "qwen_block_chained": run_block_chained, "qwen_mlp_joint": run_mlp_joint, "qwen_block_joint": run_block_joint,
               "qwen_pack_sweep": run_pack_sweep,
               "stage2_losses": run_stage2, "gemm_ceiling": run_gemm_ceiling}
    out = runners.get(args.workload, run_linear)(args)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
