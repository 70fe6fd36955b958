"""Seeded synthetic inputs for the HiNM sparse-GEMM path.

This module only *draws data*: Gaussian weights and activations rounded to the
16-bit storage type, and random channel permutations.  It contains none of the
method's arithmetic (no masks, no packing, no products) and is the only module
that both the CPU oracle's tests and the HIP path's tests/benchmarks share.

Storage convention used everywhere in this repository: a 16-bit floating-point
tensor travels as a ``numpy.uint16`` array of raw bit patterns plus a dtype tag
(``"f16"`` = IEEE binary16, ``"bf16"`` = bfloat16).

The workloads are stand-ins for the layers the paper measures (Section 5: a
BERT-base / DeiT-base feed-forward layer, ResNet convolutions as GEMMs) and
for larger LLM-MLP shapes; trained weights and datasets are not available, and
the kernel's work depends only on shapes and on the sparsity structure.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import numpy as np

SEED_BASE = 20496 * 100

# tensor ids inside one config (second chain layer adds 5)
T_W, T_X, T_PI_IN, T_PI_OUT = 0, 1, 2, 3
LAYER2 = 5


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return uint16 bits.

    Data preparation only; inputs drawn here are finite.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f16":
        return f32_to_f16_bits(x)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(f"unknown dtype tag {dtype!r}")


def bits_to_f32(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored 16-bit patterns to float32 (for feeding dense
    library references in benchmarks; not part of the method)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(f"unknown dtype tag {dtype!r}")


def seed_for(config_id: int, tensor_id: int) -> int:
    return SEED_BASE + 10 * config_id + tensor_id


def gaussian_bits(shape: Tuple[int, ...], std: float, dtype: str, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_bits(x, dtype)


def permutation(n: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).permutation(n).astype(np.int32)


@dataclasses.dataclass(frozen=True)
class Case:
    """One single-layer workload: W is M x K, X is K x N."""
    name: str
    config_id: int
    M: int
    K: int
    V: int
    Kv: int
    N: int
    dtype: str
    seed_salt: int = 0  # distinguishes sub-cases of one config (shape / sparsity)

    @property
    def T(self) -> int:
        return self.M // self.V

    def weights(self, layer: int = 0) -> np.ndarray:
        off = LAYER2 if layer == 1 else 0
        return gaussian_bits((self.M, self.K), 0.02, self.dtype,
                             seed_for(self.config_id, T_W + off) + 1000 * self.seed_salt)

    def activations(self, n: Optional[int] = None) -> np.ndarray:
        n = self.N if n is None else n
        return gaussian_bits((self.K, n), 1.0, self.dtype,
                             seed_for(self.config_id, T_X) + 1000 * self.seed_salt)

    def pi_in(self, layer: int = 0) -> np.ndarray:
        off = LAYER2 if layer == 1 else 0
        return permutation(self.K, seed_for(self.config_id, T_PI_IN + off) + 1000 * self.seed_salt)

    def pi_out(self, layer: int = 0) -> np.ndarray:
        off = LAYER2 if layer == 1 else 0
        return permutation(self.M, seed_for(self.config_id, T_PI_OUT + off) + 1000 * self.seed_salt)


def c1() -> Case:
    return Case("C1 tiny 256x256 f16 V16 N64", 0, 256, 256, 16, 128, 64, "f16")


def c2() -> Case:
    return Case("C2 encoder-FFN 3072x768 f16 V64 N4096", 1, 3072, 768, 64, 384, 4096, "f16")


def c3_cases() -> List[Case]:
    out = []
    salt = 0
    for (M, K) in ((11008, 4096), (4096, 11008)):
        for keep_div in (2, 4):
            for N in (1, 16, 2048):
                out.append(Case(
                    f"C3 LLM-MLP {M}x{K} bf16 V128 keep1/{keep_div} N{N}",
                    2, M, K, 128, K // keep_div, N, "bf16", seed_salt=salt))
            salt += 1
    return out


def c4() -> Case:
    """Two-layer chain; both layers are 4096 x 4096, layer index selects seeds."""
    return Case("C4 chain 2x(4096x4096) f16 V64 N1024", 3, 4096, 4096, 64, 2048, 1024, "f16")


def c5() -> Case:
    return Case("C5 large 16384x16384 bf16 V128 N8192", 4, 16384, 16384, 128, 8192, 8192, "bf16")


def small_case(M: int, K: int, V: int, Kv: int, N: int, dtype: str, salt: int) -> Case:
    """Free-form case for unit tests (config id 9 keeps seeds apart from the
    five named workloads)."""
    return Case(f"unit {M}x{K} V{V} Kv{Kv} N{N} {dtype}", 9, M, K, V, Kv, N, dtype, seed_salt=salt)


def sweep_layers(which):
    """GEMM shapes (name, M, K, N) behind the latency figure of Section 5.3 (BERT-base, all linear layers of one
    encoder layer at 8 x 512 tokens) and behind the V = 32 convolution experiments of Section 5.1.1 (3x3
    convolutions of the four ResNet stages as GEMMs, M = output channels, K = 9 x input channels, N = 8 images x
    output pixels).  Weights and activations are seeded synthetic tensors of these shapes."""
    if which == "sweep-bert":
        return [("attention q", 768, 768, 4096), ("attention k", 768, 768, 4096), ("attention v", 768, 768, 4096),
                ("attention out", 768, 768, 4096), ("ffn up", 3072, 768, 4096), ("ffn down", 768, 3072, 4096)]
    return [("stage1 3x3 64ch 56x56", 64, 576, 8 * 56 * 56), ("stage2 3x3 128ch 28x28", 128, 1152, 8 * 28 * 28),
            ("stage3 3x3 256ch 14x14", 256, 2304, 8 * 14 * 14), ("stage4 3x3 512ch 7x7", 512, 4608, 8 * 7 * 7)]
