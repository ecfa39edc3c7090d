"""Seeded synthetic inputs shared by the CPU oracle's tests, the GPU parity tests and the benchmark.

This module holds no attention or partition arithmetic: it only draws numbers.  Values are a pure
function of (seed, tensor id, head index), drawn from numpy's counter-based Philox generator, so the
host oracle and the device upload see bit-identical inputs without either side depending on the other.

The paper trains GPT-style models on token streams and reports throughput only (Section 4.1, Table 1);
the attention operands of one pipeline stage are stood in for by i.i.d. N(0,1) tensors of the same shape.
"""
from __future__ import annotations

import dataclasses
import numpy as np

TENSOR_IDS = {"q": 0, "k": 1, "v": 2, "dout": 3}


@dataclasses.dataclass(frozen=True)
class Workload:
    """One attention workload: a full sequence of `seq_len` tokens cut into `n_seg` segments."""
    name: str
    seq_len: int
    n_seg: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    hidden: int          # model width fed to the partitioner
    dtype: str           # "f32" or "bf16"
    partition: str       # "uniform" or "cwp" (computation-wise partition, Section 3.4)
    seed: int


# The five workloads named by the benchmark contract (shapes follow Table 1 of the paper where they
# coincide; the 30B-class and GQA shapes are the contract's own).
WORKLOADS = {
    "tiny": Workload("tiny", 1024, 4, 4, 4, 64, 256, "f32", "uniform", 20240603),
    "2.7b": Workload("2.7b", 8192, 4, 32, 32, 80, 2560, "bf16", "cwp", 20240604),
    "7b": Workload("7b", 32768, 8, 32, 32, 128, 4096, "bf16", "cwp", 20240605),
    "30b": Workload("30b", 65536, 16, 56, 56, 128, 7168, "bf16", "cwp", 20240606),
    "30b-uniform": Workload("30b-uniform", 65536, 16, 56, 56, 128, 7168, "bf16", "uniform", 20240606),
    "gqa": Workload("gqa", 131072, 32, 64, 8, 128, 8192, "bf16", "cwp", 20240607),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even) and return them as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    bias = np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    r = ((u + bias) >> np.uint64(16)) << np.uint64(16)
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Bit pattern (uint16) of bf16-representable fp32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def head_tensor(seed: int, name: str, head: int, seq_len: int, head_dim: int, dtype: str,
                scale: float = 1.0) -> np.ndarray:
    """[seq_len, head_dim] fp32 array of N(0,1)*scale values for one head of tensor `name`.

    In "bf16" mode the values are rounded to bf16 (and returned as fp32), so that the oracle and the
    device consume exactly the same numbers.
    """
    gen = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF,
                                                     (TENSOR_IDS[name] << 32) | head]))
    x = gen.standard_normal((seq_len, head_dim), dtype=np.float32)
    if scale != 1.0:
        x = x * np.float32(scale)
    if dtype == "bf16":
        x = round_to_bf16(x)
    elif dtype != "f32":
        raise ValueError(dtype)
    return x


def tensor(seed: int, name: str, n_heads: int, seq_len: int, head_dim: int, dtype: str,
           scale: float = 1.0, heads=None) -> np.ndarray:
    """[n_heads, seq_len, head_dim] fp32 array (or only the listed `heads`, stacked in that order)."""
    hs = range(n_heads) if heads is None else heads
    return np.stack([head_tensor(seed, name, h, seq_len, head_dim, dtype, scale) for h in hs])


def uniform_boundaries(seq_len: int, n_seg: int):
    """Equal-length split (the baseline the paper's Table 6 ablates against)."""
    return [(i * seq_len) // n_seg for i in range(n_seg + 1)]
