"""Shapes of the layer-step parity cases (pure data, importable without a GPU).

Every case is one linear layer [O, K] with T calibration tokens.  `chained` cases are stepped with an
upstream gradient and with dX requested (three GEMMs), the others with the locally derived dY (two GEMMs);
every case also runs faar_layer_prepare with a bf16 and with a float32 reference output.  The list is
chosen so that, together, the cases reach every GEMM kernel variant the library's planner can pick for any
layer shape (tests/test_plan_coverage.py proves that on the CPU from faar_gemm_plan), and so that the shapes
the benchmark times are compared with the oracle at their full size.
"""
from __future__ import annotations

import dataclasses


@dataclasses.dataclass(frozen=True)
class StepCase:
    name: str
    O: int
    K: int
    T: int
    seed: int
    quantised_acts: bool = False    # X_q = X with seeded relative noise (stand-in for low-precision activations)
    gated_input: bool = False       # silu(g) * u activations (input of a down projection)
    chained: bool = False           # dY_ext given and dX requested
    full_size: bool = False         # a benchmark shape at its real size: one beta, no repeated variants
    fp32_small: bool = False        # the 256x256 float32 parity configuration (own generator)
    whole_device: bool = False      # stepped with FAAR_STEP_WHOLE_DEVICE: the token-major dW GEMM may take 192-wide tiles


STEP_CASES = [
    StepCase("config1", 256, 256, 64, 0, fp32_small=True),
    StepCase("ragged", 96, 80, 100, 21, quantised_acts=True, chained=True),   # nothing a multiple of a tile
    StepCase("kproj_slice", 512, 2048, 640, 22),
    StepCase("three_tiles", 320, 256, 300, 23, quantised_acts=True, chained=True),
    StepCase("wide_two_slices", 12288, 64, 2048, 24),
    StepCase("mid_k96", 3072, 96, 2048, 25, quantised_acts=True),
    # small shapes that exist to reach one kernel variant each
    StepCase("tall_k32", 14336, 32, 640, 26),                    # residual / C GEMMs on 256x256 tiles, 32-wide slices
    StepCase("dx_o32_t640", 32, 12288, 640, 27, chained=True),   # dX GEMM: contraction 32, 256x256 tiles
    StepCase("dx_o32_t300", 32, 12288, 300, 28, chained=True),   # dX GEMM: contraction 32, 256x128 tiles
    StepCase("dx_o80", 80, 96, 100, 29, chained=True),           # dX GEMM: ragged contraction
    StepCase("dw_split_256x256", 288, 6144, 4096, 30),           # dW GEMM: 256x256 tiles, contraction split
    StepCase("dw_one_slice", 288, 12288, 33, 31),                # dW GEMM: 256x128 tiles, a single 64-token slice
    # dW GEMM on token-major operands (upstream gradient given): last tiles 8 rows / 16 columns wide, 32 slices split 11 + 11 + 10
    StepCase("dw_token_major_ragged", 3592, 1040, 2048, 32, chained=True),
    # ... with the device to itself: on 192 x 256 tiles (last tile 72 rows x 80 columns) and on 256 x 192 tiles (last 152 x 160),
    # whole and split in three
    StepCase("dw_token_major_192x256", 1032, 7248, 512, 34, chained=True, whole_device=True),
    StepCase("dw_token_major_256x192", 8088, 1312, 512, 35, chained=True, whole_device=True),
    StepCase("dw_token_major_192x256_split", 528, 6576, 2048, 36, whole_device=True),
    StepCase("dw_token_major_256x192_split", 6576, 528, 2048, 37, whole_device=True),
    # token-major dY out of the residual GEMM (with H) on 256x256 tiles with 32-wide slices: K a multiple of 32 only
    StepCase("rows_k160", 12288, 160, 4096, 33),
    # the shapes the benchmark times, at full size
    StepCase("llama_q_proj", 2048, 2048, 4096, 0, full_size=True),
    StepCase("llama_gate_proj", 8192, 2048, 4096, 1, chained=True, full_size=True),
    StepCase("llama_down_proj", 2048, 8192, 4096, 2, gated_input=True, chained=True, full_size=True),
    StepCase("qwen_k_proj", 1024, 2048, 8192, 3, quantised_acts=True, chained=True, full_size=True),
    StepCase("qwen_q_proj", 2048, 2048, 8192, 5, full_size=True),                       # the default benchmark's q / o projection
    StepCase("qwen_down_proj", 2048, 6144, 8192, 6, gated_input=True, full_size=True, whole_device=True),   # ... its down projection
    StepCase("qwen_gate_proj", 6144, 2048, 8192, 7, full_size=True, whole_device=True),   # ... and its gate / up projection
    StepCase("qwen_gate_proj_T16384", 6144, 2048, 16384, 4, chained=True, full_size=True),
]

# Cases only the Gram-matrix form of the step runs (tests/test_gpu_gram.py, next to all of STEP_CASES): shapes whose
# O x K x K product takes a kernel variant none of the above reaches with that epilogue
GRAM_CASES = [
    StepCase("gram_256x128_split", 1024, 2112, 256, 41),          # 256x128 tiles, 64-wide slices, contraction split
    StepCase("gram_256x128_k64", 4096, 1088, 192, 42),            # 256x128 tiles, 64-wide slices, whole
    StepCase("gram_256x128_k32", 4096, 1056, 192, 43),            # 256x128 tiles, 32-wide slices
]

BY_NAME = {c.name: c for c in STEP_CASES + GRAM_CASES}
