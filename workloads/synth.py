"""Seeded synthetic stand-ins for LLM linear layers and their calibration activations.

The method under test is calibrated on real model weights and activations, which
are not available here; these generators reproduce their shapes and the two
statistical features that matter for NVFP4 rounding: heavy-tailed weights and a
few outlier activation channels.  Every tensor is a pure function of its seed.

Arrays are numpy.  "bf16" tensors are returned as float32 arrays whose values
are exactly representable in bfloat16; `to_bf16_bits` gives the 16-bit patterns.
Only format conversion and a reference matmul (the frozen layer output, which
is an *input* of the method) happen here -- no quantisation arithmetic.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array -> nearest bfloat16 values (ties to even), returned as float32."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array holding bf16-representable values -> uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    if np.any(bits & np.uint32(0xFFFF)):
        raise ValueError("array holds values that are not bfloat16-representable")
    return (bits >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass
class LinearCase:
    """One linear layer's calibration problem.  W is [O, K]; X, Xq are [T, K]; Y_fp is [T, O]."""
    name: str
    W: np.ndarray          # float32 values (bf16-representable iff w_is_bf16)
    w_is_bf16: bool
    X: np.ndarray          # bf16-representable float32
    Xq: np.ndarray         # bf16-representable float32 (the quantised-path activations)
    Y_fp: np.ndarray       # bf16-representable float32: frozen layer output X @ W.T

    @property
    def O(self) -> int:
        return self.W.shape[0]

    @property
    def K(self) -> int:
        return self.W.shape[1]

    @property
    def T(self) -> int:
        return self.X.shape[0]


def gaussian_weight(O: int, K: int, seed: int, std: float = 0.02,
                    outlier_frac: float = 0.01, outlier_mult: float = 8.0) -> np.ndarray:
    """fp32 N(0, std^2) weights with a seeded fraction of entries multiplied by outlier_mult."""
    rng = np.random.default_rng([seed, 11])
    W = rng.standard_normal((O, K)).astype(np.float32) * np.float32(std)
    n_out = int(round(outlier_frac * O * K))
    if n_out:
        idx = rng.choice(O * K, size=n_out, replace=False)
        W.reshape(-1)[idx] *= np.float32(outlier_mult)
    return W


def student_t_weight(O: int, K: int, seed: int, scale: float = 0.02 / np.sqrt(2.0),
                     nu: float = 4.0) -> np.ndarray:
    """bf16 heavy-tailed weights: scale * Student-t(nu).  scale=0.02/sqrt(2) gives std 0.02 at nu=4."""
    rng = np.random.default_rng([seed, 13])
    W = rng.standard_t(nu, size=(O, K)).astype(np.float32) * np.float32(scale)
    return round_to_bf16(W)


def activations(T: int, K: int, seed: int, outlier_frac: float = 0.01,
                outlier_mult: float = 30.0, n_outlier: int | None = None) -> np.ndarray:
    """bf16 N(0,1) activations with seeded outlier channels (columns) scaled by outlier_mult."""
    rng = np.random.default_rng([seed, 17])
    X = rng.standard_normal((T, K)).astype(np.float32)
    n = int(round(outlier_frac * K)) if n_outlier is None else n_outlier
    if n:
        cols = rng.choice(K, size=n, replace=False)
        X[:, cols] *= np.float32(outlier_mult)
    return round_to_bf16(X)


def silu_gated_activations(T: int, K: int, seed: int) -> np.ndarray:
    """bf16 silu(g) * u with g, u ~ N(0,1): the input statistics of an MLP down-projection."""
    rng = np.random.default_rng([seed, 19])
    g = rng.standard_normal((T, K)).astype(np.float32)
    u = rng.standard_normal((T, K)).astype(np.float32)
    return round_to_bf16(g / (1.0 + np.exp(-g)) * u)


def perturbed_activations(X: np.ndarray, seed: int, rel: float = 0.05) -> np.ndarray:
    """A stand-in for low-precision activations: X with seeded relative noise, re-rounded to bf16."""
    rng = np.random.default_rng([seed, 23])
    noise = rng.uniform(-rel, rel, size=X.shape).astype(np.float32)
    return round_to_bf16(X * (np.float32(1.0) + noise))


def frozen_output(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """The reference layer output X @ W.T, accumulated in fp32 and stored as bf16."""
    y = torch.from_numpy(X) @ torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).T
    return y.to(torch.bfloat16).to(torch.float32).numpy()


def make_case(name: str, W: np.ndarray, w_is_bf16: bool, X: np.ndarray,
              Xq: np.ndarray | None = None) -> LinearCase:
    Xq = X if Xq is None else Xq
    return LinearCase(name, W, w_is_bf16, X, Xq, frozen_output(X, W))


def config1(seed: int = 0) -> LinearCase:
    """Small parity case: fp32 W 256x256 ~ N(0, 0.02^2) with 1% x8 outliers; X 64x256 with 4 channels x20."""
    W = gaussian_weight(256, 256, seed)
    X = activations(64, 256, seed, outlier_mult=20.0, n_outlier=4)
    return make_case("config1_256x256_T64", W, False, X)


# (name, O, K) of the linears of one transformer block; T is the calibration token count.
LLAMA3_1B_LINEARS = [("q_proj", 2048, 2048), ("k_proj", 512, 2048), ("v_proj", 512, 2048),
                     ("o_proj", 2048, 2048), ("gate_proj", 8192, 2048), ("up_proj", 8192, 2048),
                     ("down_proj", 2048, 8192)]
QWEN3_1P7B_LINEARS = [("q_proj", 2048, 2048), ("k_proj", 1024, 2048), ("v_proj", 1024, 2048),
                      ("o_proj", 2048, 2048), ("gate_proj", 6144, 2048), ("up_proj", 6144, 2048),
                      ("down_proj", 2048, 6144)]


def llm_linear(name: str, O: int, K: int, T: int, seed: int, scale: float = 0.02 / np.sqrt(2.0),
               gated_input: bool = False, quantised_acts: bool = False) -> LinearCase:
    """An LLM-shaped linear: Student-t(4) bf16 weights, bf16 activations with 1% outlier channels x30."""
    W = student_t_weight(O, K, seed, scale=scale)
    X = silu_gated_activations(T, K, seed) if gated_input else activations(T, K, seed)
    Xq = perturbed_activations(X, seed) if quantised_acts else None
    return make_case(f"{name}_{O}x{K}_T{T}", W, True, X, Xq)


def rounding_variables(O: int, K: int, seed: int) -> np.ndarray:
    """fp32 V in [0,1] with planted exact 0, 0.5, 1 and values one ulp either side of 0.5."""
    rng = np.random.default_rng([seed, 29])
    V = rng.uniform(0.0, 1.0, size=(O, K)).astype(np.float32)
    flat = V.reshape(-1)
    n = flat.size
    special = np.array([0.0, 0.5, 1.0, np.nextafter(np.float32(0.5), np.float32(0)),
                        np.nextafter(np.float32(0.5), np.float32(1)), 1e-40], dtype=np.float32)
    idx = rng.choice(n, size=min(n, 6 * max(1, n // 64)), replace=False)
    flat[idx] = np.resize(special, idx.size)
    return V


def adversarial_weight(seed: int, bf16: bool) -> np.ndarray:
    """A 16x64 tensor of hand-picked hard blocks: zeros, signed zeros, ties, on-node values,
    one huge outlier, denormals, a block whose scale underflows E4M3."""
    rng = np.random.default_rng([seed, 31])
    W = (rng.standard_normal((16, 64)) * 0.02).astype(np.float32)
    W[0, 0:16] = 0.0                                    # all-zero block
    W[0, 16:32] = 0.0
    W[0, 17] = -0.0                                     # negative zero inside a zero block
    W[1, 0:16] = np.array([6, 5, 4, 3.5, 3, 2.5, 2, 1.75, 1.5, 1.25, 1, 0.75, 0.5, 0.25, 0, -0.25],
                          dtype=np.float32)             # nodes and exact midpoints when scale is 1*s_global...
    W[1, 16:32] = -W[1, 0:16]
    W[2, 0] = 21.0                                      # tensor amax = 2688 * 2^-7: one huge outlier
    W[2, 1:16] = 1e-3
    W[3, 0:16] = 1e-30                                  # scale underflows to 0 relative to amax
    W[3, 16:32] = np.float32(1e-39)                     # fp32 denormals
    W[4, 0:16] = 2.0 ** -7 * np.array([6, 5, 4, 3.5, 3, 2.5, 2, 1.75, 1.5, 1.25, 1, 0.75, 0.5, 0.25, 0, 6],
                                           dtype=np.float32)
    W[5, 0:16] = -0.0
    W[6, 0:16] = np.linspace(-0.3, 0.3, 16, dtype=np.float32)
    W[7, 0:16] = 0.02
    W[7, 3] = -0.02
    return round_to_bf16(W) if bf16 else W
