"""Seeded synthetic shapes and tensor values for the five benchmark configurations.

No dataset is involved: every workload is synthetic, drawn from a seed, with the shapes, value
distributions and structure the benchmark configuration states.  Shapes come from
``numpy.random.default_rng``; values from a ``torch.Generator`` on the requested device.  This
module evaluates no operator of the method: it only draws inputs (the RoPE cos/sin tables are
inputs of that program and are produced here in float64, then stored as float32).
"""
from __future__ import annotations

import math
from typing import Dict, List, Tuple

import numpy as np
import torch

BASE_SEED = 26032423

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def randn(shape, seed, device="cpu", dtype="f32", mean=0.0, std=1.0) -> torch.Tensor:
    g = _gen(seed, device)
    t = torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(_TORCH_DT[dtype])


def rand_uniform(shape, seed, lo, hi, device="cpu", dtype="f32") -> torch.Tensor:
    g = _gen(seed, device)
    t = torch.rand(tuple(shape), generator=g, device=device, dtype=torch.float32)
    return (t * (hi - lo) + lo).to(_TORCH_DT[dtype])


# ----------------------------------------------------------------------------------------------
# shape streams
# ----------------------------------------------------------------------------------------------

def c2_shapes(n: int = 200, seed: int = BASE_SEED + 2) -> List[Tuple[int, int]]:
    """(B, S) pairs, B uniform in 1..32, S uniform in 1..2048, all distinct (rejection sampling)."""
    rng = np.random.default_rng(seed)
    seen, out = set(), []
    while len(out) < n:
        b, s = int(rng.integers(1, 33)), int(rng.integers(1, 2049))
        if (b, s) not in seen:
            seen.add((b, s))
            out.append((b, s))
    return out


def c3_shapes(n: int = 50, seed: int = BASE_SEED + 3) -> List[Tuple[int, int]]:
    """(B, S) pairs, B uniform in 1..4, S uniform in 128..4096."""
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, 5)), int(rng.integers(128, 4097))) for _ in range(n)]


def c4_shapes(n: int = 100, seed: int = BASE_SEED + 4) -> List[int]:
    """T uniform in 1..16384."""
    rng = np.random.default_rng(seed)
    return [int(rng.integers(1, 16385)) for _ in range(n)]


def c5_steps(n: int = 64, seed: int = BASE_SEED + 5, sigma: float = 1.0) -> List[int]:
    """T per step: log-normal with median 512 (sigma 1.0), rounded and clipped to 1..8192."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal(n)
    t = np.clip(np.rint(np.exp(math.log(512.0) + sigma * z)), 1, 8192)
    return [int(v) for v in t]


def layernorm_paper_shapes(n: int = 60, seed: int = BASE_SEED + 6) -> List[Tuple[int, int, int]]:
    """The paper's LayerNorm subgraph range (Table 2): [b, 8192, h], b in 1..60, h in {1024..4096}."""
    rng = np.random.default_rng(seed)
    hs = (1024, 2048, 3072, 4096)
    return [(int(rng.integers(1, 61)), 8192, hs[int(rng.integers(0, 4))]) for _ in range(n)]


def column_sum_shapes(n: int = 48, seed: int = BASE_SEED + 8) -> List[Tuple[int, int, int]]:
    """A dynamic stream for Table 1's Sum in its general form, [M, size, N] reduced along `size`:
    M log-uniform in 1..256, size log-uniform in 16..4096, N in {512, 1024, 2048, 4096}; instances above
    2^27 elements are drawn again (the oracle evaluates whole instances)."""
    rng = np.random.default_rng(seed)
    ns = (512, 1024, 2048, 4096)
    out: List[Tuple[int, int, int]] = []
    while len(out) < n:
        m = int(round(2.0 ** rng.uniform(0.0, 8.0)))
        size = int(round(2.0 ** rng.uniform(4.0, 12.0)))
        nn = ns[int(rng.integers(0, 4))]
        if m * size * nn <= 2 ** 27:
            out.append((m, size, nn))
    return out


def column_sum_bytes(m: int, size: int, n: int) -> int:
    return m * size * n * 4 + m * n * 4


def if_else_add_shapes(n: int = 60, seed: int = BASE_SEED + 7) -> List[Tuple[int, int, int, bool]]:
    """The paper's if-else-add range (Table 2): [b, s, f] plus a random branch flag."""
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, 257)), int(rng.integers(1, 513)), int(rng.integers(1, 8193)),
             bool(rng.integers(0, 2))) for _ in range(n)]


# ----------------------------------------------------------------------------------------------
# inputs per configuration: name -> tensor, in the program's input order
# ----------------------------------------------------------------------------------------------

def c1_inputs(seed: int = BASE_SEED + 1, device="cpu", rows: int = 4, cols: int = 1000) -> Dict[str, torch.Tensor]:
    return {
        "x": randn((rows, cols), seed, device),
        "a": rand_uniform((cols,), seed + 1, -1.0, 1.0, device),
        "b": rand_uniform((cols,), seed + 2, -1.0, 1.0, device),
    }


def c2_inputs(B: int, S: int, seed: int, device="cpu", H: int = 4096) -> Dict[str, torch.Tensor]:
    return {
        "x": randn((B, S, H), seed, device, "bf16"),
        "w": randn((H,), seed + 1, device, "bf16", mean=1.0, std=0.1),
    }


def causal_mask(S: int, device="cpu") -> torch.Tensor:
    """Additive causal mask: 0 on and below the diagonal, -inf above it."""
    m = torch.zeros((S, S), dtype=torch.float32, device=device)
    m.masked_fill_(torch.ones((S, S), dtype=torch.bool, device=device).triu(1), float("-inf"))
    return m


def c3_inputs(B: int, S: int, seed: int, device="cpu", heads: int = 32) -> Dict[str, torch.Tensor]:
    return {"z": randn((B, heads, S, S), seed, device, "f32", std=3.0), "mask": causal_mask(S, device)}


def c4_inputs(T: int, seed: int, device="cpu", H: int = 8192) -> Dict[str, torch.Tensor]:
    g = _gen(seed + 5, device)
    keep = torch.rand((T, H), generator=g, device=device) < 0.9
    mask = torch.where(keep, torch.tensor(1.0 / (1.0 - 0.1), device=device), torch.tensor(0.0, device=device))
    return {
        "x": randn((T, H), seed, device, "bf16"),
        "r": randn((T, H), seed + 1, device, "bf16"),
        "gamma": randn((H,), seed + 2, device, "bf16", mean=1.0, std=0.1),
        "beta": randn((H,), seed + 3, device, "bf16", std=0.1),
        "bias": randn((H,), seed + 4, device, "bf16", std=0.1),
        "mask": mask.to(torch.bfloat16),
    }


def rope_tables(T: int, half: int = 64, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """cos/sin of theta[t, i] = t * 10000**(-i/half), evaluated in float64, stored as float32 [T, half]."""
    t = np.arange(T, dtype=np.float64)[:, None]
    inv = 10000.0 ** (-np.arange(half, dtype=np.float64) / half)[None, :]
    th = t * inv
    return (torch.from_numpy(np.cos(th)).to(torch.float32).to(device),
            torch.from_numpy(np.sin(th)).to(torch.float32).to(device))


def c5_inputs(T: int, seed: int, device="cpu", hidden: int = 4096, heads: int = 32, head_dim: int = 128,
              ffn: int = 14336) -> Dict[str, Dict[str, torch.Tensor]]:
    """Inputs of the six per-layer programs for one layer at sequence length T.

    The "GEMM outputs" of the configuration are seeded N(0,1) bf16 tensors.  RoPE gets the full
    [T, heads, head_dim] tensor under the key ``q``; its program reads the two halves of the last
    axis as strided views and the cos/sin tables [T, 1, head_dim/2] broadcast over heads.
    """
    cos, sin = rope_tables(T, head_dim // 2, device)
    q = randn((T, heads, head_dim), seed + 10, device, "bf16")
    half = head_dim // 2
    return {
        "c5_rmsnorm": {"x": randn((T, hidden), seed, device, "bf16"),
                       "w": randn((hidden,), seed + 1, device, "bf16", mean=1.0, std=0.1)},
        "c5_rope": {"x1": q[..., :half], "x2": q[..., half:], "cos": cos.view(T, 1, half),
                    "sin": sin.view(T, 1, half)},
        "c5_softmax": {"z": randn((heads, T, T // 8 + 1), seed + 20, device, "bf16")},
        "c5_residual_a": {"a": randn((T, hidden), seed + 30, device, "bf16"),
                          "b": randn((T, hidden), seed + 31, device, "bf16")},
        "c5_silu_gate": {"g": randn((T, ffn), seed + 40, device, "bf16"),
                         "u": randn((T, ffn), seed + 41, device, "bf16")},
        "c5_residual_b": {"a": randn((T, hidden), seed + 50, device, "bf16"),
                          "b": randn((T, hidden), seed + 51, device, "bf16")},
    }


# ----------------------------------------------------------------------------------------------
# algorithmic bytes: one read of every distinct input element + one write of every output element
# ----------------------------------------------------------------------------------------------

def c2_bytes(B: int, S: int, H: int = 4096) -> int:
    return 2 * B * S * H * 2 + H * 2


def layernorm_inputs(b: int, s: int, h: int, seed: int, device="cpu") -> Dict[str, torch.Tensor]:
    return {
        "x": randn((b, s, h), seed, device, "bf16"),
        "gamma": randn((h,), seed + 1, device, "bf16", mean=1.0, std=0.1),
        "beta": randn((h,), seed + 2, device, "bf16", std=0.1),
    }


def layernorm_bytes(b: int, s: int, h: int) -> int:
    return 2 * b * s * h * 2 + 2 * h * 2


def c3_bytes(B: int, S: int, heads: int = 32) -> int:
    return 2 * B * heads * S * S * 4 + S * S * 4


def c4_bytes(T: int, H: int = 8192) -> int:
    return 4 * T * H * 2 + 3 * H * 2


def c5_layer_bytes(T: int, hidden: int = 4096, heads: int = 32, head_dim: int = 128, ffn: int = 14336) -> int:
    L = T // 8 + 1
    return ((2 * T * hidden + hidden) * 2            # rmsnorm
            + 2 * T * heads * head_dim * 2 + 2 * T * (head_dim // 2) * 4   # rope
            + 2 * heads * T * L * 2                  # softmax
            + 2 * 3 * T * hidden * 2                 # two residual adds
            + 3 * T * ffn * 2)                       # silu gate
