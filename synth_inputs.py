"""Seeded synthetic inputs for the layer-stack workloads.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds none of the method's arithmetic: it only draws numbers,
lays them out and rounds them to a storage type.

The paper's workloads are shapes, not data (Table B.1 gives model shapes; no
dataset is used anywhere), so nothing here stands in for a public benchmark.

Recipe (one generator, numpy PCG64 seeded with `seed`, float64 standard normals,
drawn in this fixed order, then cast to float32):
  1. x  [n_mu, b_mu, d_s, d_m]  ~ N(0, 1)      stack input
  2. G  [n_mu, b_mu, d_s, d_m]  ~ N(0, 1)      upstream gradient, loss = sum(y * G)
  3. for each layer 0..d_l-1, in canonical order: w_qkv, w_o, w_1, w_2 ~ N(0, std^2)
     with std = 0.02; layer-norm gains are 1, every bias (linear and layer-norm) is 0.
With `bias_std > 0` the biases and gains are perturbed too (drawn after all of the
above, layer by layer in canonical order) so that tests exercise non-trivial values.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

PARAM_ORDER = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2",
)
MATRICES = ("w_qkv", "w_o", "w_1", "w_2")
GAINS = ("ln1_g", "ln2_g")


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    d_ff: int
    seq_len: int
    micro_batch: int
    n_micro: int
    dtype: str            # "fp32", "bf16" or "fp16": activation / GEMM-input type on the GPU

    @property
    def tokens(self) -> int:
        return self.n_micro * self.micro_batch * self.seq_len

    @property
    def params_per_layer(self) -> int:
        d, f = self.d_model, self.d_ff
        return 4 * d * d + 2 * d * f + 9 * d + f


# The five benchmark configurations (shapes only).
CONFIGS: Tuple[Workload, ...] = (
    Workload("cfg0_tiny_fp32", 2, 64, 4, 256, 32, 2, 4, "fp32"),
    Workload("cfg1_gpt2small_bf16", 12, 768, 12, 3072, 1024, 4, 8, "bf16"),
    Workload("cfg2_mid_bf16", 24, 2048, 16, 8192, 2048, 2, 16, "bf16"),
    Workload("cfg3_gpt3_share_bf16", 4, 12288, 96, 49152, 2048, 1, 32, "bf16"),
    Workload("cfg4_x160_share_bf16", 1, 25600, 160, 102400, 2048, 1, 64, "bf16"),
)

# Micro-batches per kernel launch (`group`) with which the benchmark runs each configuration, and the full-size parity
# tests with it: the narrow configurations gain from more tokens per launch (their GEMMs have few tiles per round of
# 256 workgroups and short contractions), the wide ones do not (within 0.5 % for 2 ... 16).
BENCH_GROUP = {0: 4, 1: 8, 2: 8, 3: 4, 4: 4}


def x_family(x: int, n_micro: int, micro_batch: int = 1, n_layers: int = 0, dtype: str = "bf16") -> Workload:
    """Shape of the paper's X_[x] model family (appendix B, table B.1): d_a = x/2 heads of size d_h = 2x,
    d_l = x layers (or `n_layers` of them), d_s = 16x, d_m = x^2, d_I = 4x^2."""
    if x < 2 or x % 2:
        raise ValueError("x must be even and >= 2")
    return Workload(f"X{x}", n_layers or x, x * x, x // 2, 4 * x * x, 16 * x, micro_batch, n_micro, dtype)


def parity_slice(w: Workload, n_layers: int = 1, n_micro: int = 2, seq_len: int = 256) -> Workload:
    """Same width, heads, feed-forward width and dtype; fewer layers, micro-batches, tokens."""
    return Workload(w.name + "_slice", n_layers, w.d_model, w.n_heads, w.d_ff, seq_len,
                    w.micro_batch, n_micro, w.dtype)


def tensor_shapes(d_model: int, d_ff: int) -> Dict[str, Tuple[int, ...]]:
    d, f = d_model, d_ff
    return {
        "ln1_g": (d,), "ln1_b": (d,), "w_qkv": (d, 3 * d), "b_qkv": (3 * d,),
        "w_o": (d, d), "b_o": (d,), "ln2_g": (d,), "ln2_b": (d,),
        "w_1": (d, f), "b_1": (f,), "w_2": (f, d), "b_2": (d,),
    }


def tensor_slices(d_model: int, d_ff: int) -> Dict[str, slice]:
    """Where each tensor sits in a layer's flat canonical vector."""
    out, off = {}, 0
    for name, shp in tensor_shapes(d_model, d_ff).items():
        n = int(np.prod(shp))
        out[name] = slice(off, off + n)
        off += n
    return out


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bias = ((bits >> 16) & 1) + 0x7FFF
    rounded = ((bits + bias) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 values that are exactly bf16-representable -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def round_to_fp16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest IEEE half (ties to even); result stays float32."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def from_16bit_bits(b: np.ndarray, dtype: str) -> np.ndarray:
    """uint16 bit patterns of a 16-bit workload's tensor -> float32."""
    if dtype == "fp16":
        return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)
    return from_bf16_bits(b)


def make_inputs(w: Workload, seed: int = 0, weight_std: float = 0.02, bias_std: float = 0.0):
    """Return (x, G, params): x and G float32 [n, b, s, d]; params a list of flat float32
    vectors, one per layer, in canonical order.  In 16-bit workloads x and G hold values
    representable in the workload's format (so storing them in it on the GPU loses nothing)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    shp = (w.n_micro, w.micro_batch, w.seq_len, w.d_model)
    x = rng.standard_normal(shp).astype(np.float32)
    G = rng.standard_normal(shp).astype(np.float32)
    if w.dtype == "bf16":
        x, G = round_to_bf16(x), round_to_bf16(G)
    elif w.dtype == "fp16":
        x, G = round_to_fp16(x), round_to_fp16(G)
    shapes = tensor_shapes(w.d_model, w.d_ff)
    sl = tensor_slices(w.d_model, w.d_ff)
    params: List[np.ndarray] = []
    for _ in range(w.n_layers):
        flat = np.zeros(w.params_per_layer, dtype=np.float32)
        for name in GAINS:
            flat[sl[name]] = 1.0
        for name in MATRICES:
            n = int(np.prod(shapes[name]))
            flat[sl[name]] = (weight_std * rng.standard_normal(n)).astype(np.float32)
        params.append(flat)
    if bias_std > 0.0:
        for flat in params:
            for name in PARAM_ORDER:
                if name in MATRICES:
                    continue
                n = int(np.prod(shapes[name]))
                flat[sl[name]] += (bias_std * rng.standard_normal(n)).astype(np.float32)
    return x, G, params
