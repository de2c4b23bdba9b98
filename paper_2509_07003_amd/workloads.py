"""The benchmark workloads (shapes, meshes, placements, seeds) and their seeded synthetic
inputs.  This module serves the tests, the benchmark and the smoke check alike and holds
none of the method's arithmetic: no generator, no index map, no conversion.

The shapes stand in for the paper's LLaMA-3-8B-like training workloads (hidden 4096,
MLP 14336, 32 heads, sequence 4096); datasets and weights are not needed because the
path's inputs are only shapes, shardings, seeds and - for dropout - an activation tensor.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass
class Workload:
    name: str
    op: str                     # "uniform" | "normal" | "dropout"
    dtype: str                  # "f32" | "bf16"
    global_shape: List[int]
    mesh_shape: List[int]
    placements: List[Tuple]
    seed: int
    offset: int = 0
    params: dict = field(default_factory=dict)
    input_seed: Optional[int] = None   # dropout: seed of the synthetic activations
    input_kind: Optional[str] = None   # "normal" | "softmax"
    bench_coord: Optional[List[int]] = None   # the rank whose shard is timed

    def sharding_args(self, coord):
        return self.global_shape, self.mesh_shape, self.placements, list(coord)


C1 = Workload("C1 uniform f32 [1024,1024] mesh(4) Shard(0)", "uniform", "f32", [1024, 1024], [4],
              [("S", 0)], seed=1234, params=dict(low=0.0, high=1.0), bench_coord=[0])
C2 = Workload("C2 normal f32 [4096,4096] mesh(3) Shard(1) uneven", "normal", "f32", [4096, 4096], [3],
              [("S", 1)], seed=7, params=dict(mean=0.0, std=1.0), bench_coord=[1])
C3 = Workload("C3 normal bf16 N(0,0.02) [4096,14336] mesh(2,4) (Shard(0),Shard(1))", "normal", "bf16",
              [4096, 14336], [2, 4], [("S", 0), ("S", 1)], seed=3, params=dict(mean=0.0, std=0.02),
              bench_coord=[1, 2])
C4 = Workload("C4 dropout bf16 p=0.1 [8,4096,4096] mesh(8) Shard(1)", "dropout", "bf16", [8, 4096, 4096],
              [8], [("S", 1)], seed=1234, params=dict(p=0.1), input_seed=11, input_kind="normal",
              bench_coord=[3])
C5 = Workload("C5 dropout bf16 p=0.1 [8,32,4096,4096] mesh(4,2) (Shard(1),Shard(1))", "dropout", "bf16",
              [8, 32, 4096, 4096], [4, 2], [("S", 1), ("S", 1)], seed=1234, params=dict(p=0.1),
              input_seed=11, input_kind="softmax", bench_coord=[2, 1])
# Second reading of "interleaved 8-way": heads dealt out round-robin in 4 groups of 8.
C5_INTERLEAVED = Workload("C5 dropout bf16 p=0.1 [8,32,4096,4096] mesh(8) InterleavedShard(1,4)", "dropout",
                          "bf16", [8, 32, 4096, 4096], [8], [("IS", 1, 4)], seed=1234, params=dict(p=0.1),
                          input_seed=11, input_kind="softmax", bench_coord=[5])
ALL = [C1, C2, C3, C4, C5]


def bf16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """fp32 array -> bfloat16 bit patterns (uint16) through torch's own conversion."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def f16_bits_from_f32(a: np.ndarray) -> np.ndarray:
    """float32 -> IEEE binary16 bit patterns (nearest even; overflow becomes infinity)."""
    with np.errstate(over="ignore"):
        return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def bits16_from_f32(a: np.ndarray, dtype: str) -> np.ndarray:
    return f16_bits_from_f32(a) if dtype == "f16" else bf16_bits_from_f32(a)


def host_activations(shape, seed, kind="normal", dtype="bf16") -> np.ndarray:
    """Seeded synthetic dropout input on the host: N(0,1) values, or softmax-normalised rows of
    N(0,1) logits (attention probabilities).  Returns float32, or uint16 bf16 bit patterns."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=tuple(shape), dtype=np.float32)
    if kind == "softmax":
        a = a - a.max(axis=-1, keepdims=True)
        np.exp(a, out=a)
        a /= a.sum(axis=-1, keepdims=True)
    return bf16_bits_from_f32(a) if dtype == "bf16" else a


def device_activations(shape, seed, kind="normal", dtype="bf16"):
    """The same kind of input generated on the GPU with torch (used where the shard is too
    large to make on the host quickly).  Values differ from host_activations; only the
    distribution is the same."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    a = torch.randn(tuple(shape), generator=gen, device="cuda", dtype=torch.float32)
    if kind == "softmax":
        a = torch.softmax(a, dim=-1)
    return a.to(torch.bfloat16) if dtype == "bf16" else a


def adversarial_f32(n: int, seed: int) -> np.ndarray:
    """Activations seasoned with the values that break careless dropout code."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n).astype(np.float32)
    specials = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-39, -1e-39, 1e-45, 3.3e38, -3.3e38,
                         1.0, -1.0, 65504.0, 2.0 ** -126, 2.0 ** -133,
                         6.0e-8, -6.0e-8, 3.0e-5, 6.1e-5, 60000.0, -65504.0], dtype=np.float32)  # binary16's edges
    idx = rng.permutation(n)[: min(n, 8 * len(specials))]
    a[idx] = np.resize(specials, idx.size)
    return a
