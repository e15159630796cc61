"""Seeded synthetic inputs for the LUT mpGEMV/mpGEMM path.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no bit planes, no tables, no matmul).  Both the CPU oracle
tests and the HIP path's tests/bench take their inputs from here, so that the
two sides always see exactly the same arrays.

The shapes stand in for the layer shapes of Llama-2-7B/13B and BitNet-b1.58-3B
used in the paper's kernel benchmarks (Section 5.1 "Kernels and models",
Section 5.2, Table 3); the trained weights themselves are not needed because
the kernels' cost and correctness do not depend on the values.

Seed rule: ``20240700 + 100*config + case_index``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, Optional

import numpy as np

SEED_BASE = 20240700


@dataclass
class Problem:
    """One mpGEMM problem instance: R[N,M] = A[N,K] x W[M,K]^T.

    Weights are unsigned codes ``q`` in [0, 2^bits) with ``w = s*(q - z)``.
    ``group`` is the quantisation group along K; ``group == 0`` means one
    scale (``weight_scale``) and one zero (``zero_point``) for the whole tensor.
    Activations are fp16 (``act``) or int8 with a per-row fp32 scale
    (``act_q``, ``act_scale``).
    """
    name: str
    config: int
    N: int
    M: int
    K: int
    bits: int
    group: int
    q: np.ndarray                      # uint8 [M, K]
    scales: Optional[np.ndarray]       # float16 [M, K/group] or None
    zeros: Optional[np.ndarray]        # float16 [M, K/group] or None
    weight_scale: float = 1.0          # per-tensor scale (group == 0)
    zero_point: float = 0.0            # per-tensor zero (group == 0)
    act: Optional[np.ndarray] = None   # float16 [N, K]
    act_q: Optional[np.ndarray] = None     # int8 [N, K]
    act_scale: Optional[np.ndarray] = None  # float32 [N]
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def int_path(self) -> bool:
        return self.act_q is not None


def seed_for(config: int, case: int) -> int:
    return SEED_BASE + 100 * config + case


def _rng(config: int, case: int) -> np.random.Generator:
    return np.random.default_rng(seed_for(config, case))


def gaussian_act(rng: np.random.Generator, N: int, K: int) -> np.ndarray:
    """fp16 activations ~ N(0,1)."""
    return rng.standard_normal((N, K), dtype=np.float32).astype(np.float16)


def uniform_codes(rng: np.random.Generator, M: int, K: int, bits: int) -> np.ndarray:
    return rng.integers(0, 1 << bits, size=(M, K), dtype=np.uint8)


def group_scales(rng: np.random.Generator, M: int, ngroups: int) -> np.ndarray:
    return rng.uniform(0.01, 0.1, size=(M, ngroups)).astype(np.float16)


def group_zeros(rng: np.random.Generator, M: int, ngroups: int, bits: int) -> np.ndarray:
    return rng.uniform(0.0, float((1 << bits) - 1), size=(M, ngroups)).astype(np.float16)


def absmax_int8(act_f16: np.ndarray):
    """Per-token absmax quantisation of activations to int8 (done upstream of the
    path, as BitNet does): s_a = max|a|/127, a_q = clip(rint(a/s_a), -127, 127)."""
    a = act_f16.astype(np.float32)
    amax = np.abs(a).max(axis=1)
    s_a = (amax / np.float32(127.0)).astype(np.float32)
    s_a = np.where(s_a == 0, np.float32(1.0), s_a).astype(np.float32)
    a_q = np.clip(np.rint(a / s_a[:, None]), -127, 127).astype(np.int8)
    return a_q, s_a


def make_grouped(config: int, case: int, N: int, M: int, K: int, bits: int, group: int,
                 name: Optional[str] = None) -> Problem:
    """Uniform codes, fp16 group scales ~U(0.01,0.1), fp16 zeros ~U(0,2^b-1),
    fp16 activations ~N(0,1)."""
    rng = _rng(config, case)
    q = uniform_codes(rng, M, K, bits)
    ng = K // group
    s = group_scales(rng, M, ng)
    z = group_zeros(rng, M, ng, bits)
    a = gaussian_act(rng, N, K)
    return Problem(name or f"cfg{config}_{M}x{K}_w{bits}_n{N}", config, N, M, K, bits, group,
                   q, s, z, act=a, seed=seed_for(config, case))


def make_ternary(config: int, case: int, N: int, M: int, K: int,
                 weight_scale: float = 0.02, name: Optional[str] = None) -> Problem:
    """Ternary weights t in {-1,0,+1} with p=(.25,.5,.25), stored as 2-bit codes
    q=t+1 with zero point 1 and one fp32 scale; int8 absmax activations."""
    rng = _rng(config, case)
    t = rng.choice(np.array([-1, 0, 1], dtype=np.int8), size=(M, K), p=[0.25, 0.5, 0.25])
    q = (t + 1).astype(np.uint8)
    a = gaussian_act(rng, N, K)
    a_q, s_a = absmax_int8(a)
    return Problem(name or f"cfg{config}_{M}x{K}_ternary_n{N}", config, N, M, K, 2, 0,
                   q, None, None, weight_scale=float(np.float32(weight_scale)), zero_point=1.0,
                   act_q=a_q, act_scale=s_a, seed=seed_for(config, case))


LLAMA7B_SHAPES = [(4096, 4096), (11008, 4096), (4096, 11008)]
BITNET3B_SHAPES = [(3200, 3200), (8640, 3200), (3200, 8640)]
LLAMA13B_SHAPES = [(5120, 5120), (13824, 5120), (5120, 13824)]


def config1() -> Problem:
    """Tiny mpGEMV: N=1, K=M=256, 2-bit asymmetric, group 32."""
    return make_grouped(1, 0, 1, 256, 256, 2, 32, name="cfg1_tiny_256x256_w2")


def config2(i: int) -> Problem:
    """Llama-2-7B-shaped W4A16 decode GEMV, shape index i in 0..2."""
    M, K = LLAMA7B_SHAPES[i]
    return make_grouped(2, i, 1, M, K, 4, 128)


def config3(bits: int) -> Problem:
    """Bit-width sweep at M=K=4096, N=1."""
    return make_grouped(3, bits, 1, 4096, 4096, bits, 128)


def config4(i: int) -> Problem:
    """BitNet-b1.58-3B-shaped ternary GEMV, shape index i in 0..2."""
    M, K = BITNET3B_SHAPES[i]
    return make_ternary(4, i, 1, M, K)


def config5(i: int, bits: int, N: int = 256) -> Problem:
    """Llama-2-13B-shaped prefill mpGEMM, N=256 tokens."""
    M, K = LLAMA13B_SHAPES[i]
    return make_grouped(5, 10 * bits + i, N, M, K, bits, 128)


def all_full_size() -> Iterator[Problem]:
    yield config1()
    for i in range(3):
        yield config2(i)
    for b in (1, 2, 3, 4):
        yield config3(b)
    for i in range(3):
        yield config4(i)
    for b in (2, 4):
        for i in range(3):
            yield config5(i, b)
