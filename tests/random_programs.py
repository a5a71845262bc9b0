"""Seeded random operator programs for differential tests (generator only: no arithmetic of the method).

A program is a chain of elementwise ops, broadcasts, row reductions over the last axis and their
consumers, built so that every value stays bounded (no overflow, no division by something near
zero) and the comparison with the oracle is meaningful at the stated tolerances.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

from workloads.programs import _p

ROW_LENGTHS = [1, 2, 3, 7, 8, 9, 31, 33, 64, 100, 127, 128, 129, 255, 257, 513, 1000, 1024, 1025, 2047, 4096, 4100, 5000, 9001]
OUTER = [1, 2, 3, 5, 8, 17, 40, 130]

UNARY_BOUNDED = ["tanh", "sigmoid", "neg", "abs", "gelu_tanh", "gelu_erf", "silu", "erf"]


def make(seed: int):
    """Returns (program description, dict name -> (shape, strides or None, dtype), budget of elements)."""
    rng = np.random.default_rng(seed)
    rank = int(rng.integers(1, 4))
    d0 = int(rng.choice(ROW_LENGTHS))
    outer = [int(rng.choice(OUTER)) for _ in range(rank - 1)]
    while int(np.prod(outer + [d0])) > 400000 and outer:
        outer[int(np.argmax(outer))] = max(1, max(outer) // 2)
    dom = tuple(outer + [d0])
    bf16_prog = bool(rng.integers(0, 2))
    n_in = int(rng.integers(1, 5))
    inputs: List[Tuple[str, str]] = []
    specs: Dict[str, Tuple[Tuple[int, ...], str, str]] = {}
    for i in range(n_in):
        name = f"in{i}"
        if i == 0:
            shape = dom
        else:
            kind = int(rng.integers(0, 5))
            if kind == 0:
                shape = dom
            elif kind == 1:
                shape = (d0,)                                   # row vector
            elif kind == 2:
                shape = tuple(list(dom[:-1]) + [1])             # one value per row
            elif kind == 3:
                shape = tuple(1 if rng.integers(0, 2) else s for s in dom)   # random broadcast pattern
            else:
                shape = dom[-2:] if rank >= 2 else dom          # leading dims broadcast
        dt = "bf16" if (bf16_prog and rng.integers(0, 4) != 0) else "f32"
        layout = "contig"
        if len(shape) >= 2 and rng.integers(0, 4) == 0:
            layout = "padded_rows"                               # row stride larger than the row
        elif len(shape) == 3 and rng.integers(0, 5) == 0:
            layout = "swapped_outer"                             # a permuted view of the outer dims
        inputs.append((name, dt))
        specs[name] = (shape, dt, layout)

    ops = []
    full_vals = ["in0"]          # values with the dominant shape (or broadcastable tiles)
    any_vals = [n for n, _ in inputs]
    row_vals: List[str] = [n for n, (s, _, _) in specs.items() if len(s) == rank and s[-1] == 1 and d0 > 1]
    counter = [0]

    def new(prefix="v"):
        counter[0] += 1
        return f"{prefix}{counter[0]}"

    n_ops = int(rng.integers(1, 11))
    has_red = False
    cur = "in0"
    for _ in range(n_ops):
        r = int(rng.integers(0, 100))
        out = new()
        if r < 25:
            u = str(rng.choice(UNARY_BOUNDED))
            ops.append((out, u, [cur], {}))
        elif r < 35:
            t = new("t")
            ops.append((t, "tanh", [cur], {}))
            ops.append((out, str(rng.choice(["exp", "square", "sqrt_abs"])), [t], {}))
            if ops[-1][1] == "sqrt_abs":
                a = new("a")
                ops[-1] = (a, "abs", [t], {})
                ops.append((out, "sqrt", [a], {}))
        elif r < 60:
            other = str(rng.choice(any_vals + full_vals))
            b = str(rng.choice(["add", "sub", "mul", "min", "max"]))
            args = [cur, other] if rng.integers(0, 2) else [other, cur]
            ops.append((out, b, args, {}))
        elif r < 68:
            other = str(rng.choice(any_vals))
            a = new("a")
            d = new("d")
            ops.append((a, "abs", [other], {}))
            ops.append((d, "adds", [a], {"imm": 1.0}))
            ops.append((out, "div", [cur, d], {}))
        elif r < 76:
            ops.append((out, str(rng.choice(["adds", "muls"])), [cur], {"imm": float(np.round(rng.uniform(-2, 2), 3))}))
        elif r < 90:
            red = str(rng.choice(["sum", "rmax", "rmin", "mean", "meansq"]))
            rv = new("r")
            ops.append((rv, red, [cur], {}))
            has_red = True
            row_vals.append(rv)
            if red == "sum":      # keep magnitudes bounded: scale a sum back to a mean-like value
                sv = new("r")
                ops.append((sv, "muls", [rv], {"imm": 1.0 / d0}))
                rv = sv
                row_vals.append(rv)
            how = int(rng.integers(0, 3))
            if how == 0:
                ops.append((out, "sub", [cur, rv], {}))
            elif how == 1:
                a = new("a")
                d = new("d")
                ops.append((a, "abs", [rv], {}))
                ops.append((d, "adds", [a], {"imm": 0.5}))
                ops.append((out, "div", [cur, d], {}))
            else:
                ops.append((out, "mul", [cur, rv], {}))
        elif r < 95:
            # the condition compares two inputs: both sides then decide on identical values
            lhs, rhs = str(rng.choice(any_vals)), str(rng.choice(any_vals))
            c = new("c")
            alt = new("alt")
            ops.append((c, "cmp", [lhs, rhs], {"cmp": str(rng.choice(["lt", "ge", "eq", "ne", "gt", "le"]))}))
            ops.append((alt, "muls", [cur], {"imm": -0.5}))
            ops.append((out, "select", [c, cur, alt], {}))
        else:
            ops.append((out, str(rng.choice(["softmax"])), [cur], {}))
            has_red = True
        cur = ops[-1][0]
        full_vals.append(cur)
        if len(full_vals) > 4:
            full_vals.pop(0)
    out_dt = "bf16" if bf16_prog else "f32"
    outputs = [(cur, out_dt)]
    # sometimes a second output: an earlier full value or a row value
    if rng.integers(0, 3) == 0:
        cand = [v for v in full_vals[:-1] if not v.startswith("in")] + [v for v in row_vals if not v.startswith("in")]
        if cand:
            extra = str(rng.choice(cand))
            if extra != cur:
                outputs.append((extra, out_dt))
    desc = _p(f"random_{seed}", inputs, ops, outputs)
    return desc, specs, dom, has_red


def layout_of(shape, layout):
    """(storage shape, strides in elements) for the layouts the generator names."""
    shape = tuple(int(x) for x in shape)
    if layout == "padded_rows" and len(shape) >= 2:
        pad = shape[-1] + 3
        strides = [1]
        ext = pad
        for s in reversed(shape[:-1]):
            strides.append(ext)
            ext *= s
        return tuple(reversed(strides))
    if layout == "swapped_outer" and len(shape) == 3:
        a, b, c = shape                      # stored as [b, a, c], viewed as [a, b, c]
        return (c, a * c, 1)
    strides = [1]
    for s in reversed(shape[1:]):
        strides.append(strides[-1] * s)
    return tuple(reversed(strides))
