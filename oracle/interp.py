"""Plain per-op eager CPU interpreter of an operator program.  TEST INFRASTRUCTURE ONLY.

What it computes: the unfused definition of the program.  Each op is evaluated over whole arrays
in float64, its result fully materialised, with NumPy broadcasting (a broadcast or reduced
dimension has extent 1: Algorithm 1, the "skip broadcasting or reduction dimensions" step).
Per-op semantics are Table 1 of the paper ("Tile-level Virtual Instructions"); compound ops are
written out from their textbook definitions (the paper decomposes compound operators into basic
ones, Section 3 "Operator Compiler").

Numeric contract:
  * storage dtypes are fp32 or bf16; inputs arrive as arrays of exactly representable values;
  * all arithmetic is float64; an output is rounded once, to its storage dtype, at the very end
    (round-to-nearest-even).  ``cast`` is the only op that rounds an intermediate (Table 1, Cast);
  * ops whose result is an integer decision (cmp, select's condition, round, floor, isfinite) take
    that decision on operands rounded to fp32 first, the precision the device computes in;
  * reductions (Table 1 Sum / Max / Min with N = 1, i.e. over the last axis) accumulate
    sequentially in float64.

Nothing here is blocked, fused or reordered.  This module imports nothing from the HIP package.
"""
from __future__ import annotations

import math
from typing import Dict, Mapping, Tuple

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------------------------

def round_to_bf16(x) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (8 exponent bits, 7 fraction bits), ties to even.

    Written from the format definition: a finite value with binade exponent e (clamped below at
    the smallest normal exponent -126, so subnormals share the spacing 2**-133) is a multiple of
    2**(e-7); rounding is rint() of the value expressed in that unit.  Overflow goes to infinity.
    Returned as float64 holding exactly representable values.
    """
    x = np.asarray(x, dtype=F64)
    out = np.array(x, dtype=F64, copy=True)
    fin = np.isfinite(x) & (x != 0.0)
    if np.any(fin):
        v = x[fin]
        _, e = np.frexp(v)              # v = m * 2**e, 0.5 <= |m| < 1  -> binade exponent is e-1
        e = np.maximum(e - 1, -126)
        unit = np.ldexp(1.0, e - 7)
        r = np.rint(v / unit) * unit    # np.rint rounds half to even
        max_bf16 = (2.0 - 2.0 ** -7) * 2.0 ** 127
        r = np.where(np.abs(r) > max_bf16, np.sign(r) * np.inf, r)
        out[fin] = r
    return out


def round_to_f32(x) -> np.ndarray:
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=F64).astype(np.float32).astype(F64)


def round_to_storage(x, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return round_to_f32(x)
    if dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# ----------------------------------------------------------------------------------------------
# per-op definitions
# ----------------------------------------------------------------------------------------------

_erf = np.vectorize(math.erf, otypes=[F64])


def _gelu_tanh(u):
    return 0.5 * u * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u ** 3)))


def _gelu_erf(u):
    return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))


def _sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def _rowsum(x):
    """Sequential float64 sum over the last axis, kept with extent 1 (Table 1, Sum, N = 1)."""
    x = np.asarray(x, dtype=F64)
    acc = np.zeros(x.shape[:-1] + (1,), dtype=F64)
    for j in range(x.shape[-1]):
        acc[..., 0] += x[..., j]
    return acc


_CMP = {"eq": np.equal, "ne": np.not_equal, "lt": np.less, "le": np.less_equal,
        "gt": np.greater, "ge": np.greater_equal}


def _f32(x):
    return round_to_f32(x)


def _eval(name: str, a: Tuple[np.ndarray, ...], attrs: Mapping[str, object]) -> np.ndarray:
    with np.errstate(all="ignore"):
        # --- Table 1, computation ---------------------------------------------------------
        if name == "copy":
            return a[0].copy()
        if name == "sqrt":
            return np.sqrt(a[0])
        if name == "abs":
            return np.abs(a[0])
        if name == "log":
            return np.log(a[0])
        if name == "exp":
            return np.exp(a[0])
        if name == "pow":
            return np.power(a[0], a[1])
        if name == "round":
            return np.rint(_f32(a[0]))                  # nearest integer, halves to even
        if name == "floor":
            return np.floor(_f32(a[0]))
        if name == "isfinite":
            return np.isfinite(_f32(a[0])).astype(F64)
        if name == "adds":
            return a[0] + float(attrs["imm"])
        if name == "muls":
            return a[0] * float(attrs["imm"])
        if name == "add":
            return a[0] + a[1]
        if name == "sub":
            return a[0] - a[1]
        if name == "mul":
            return a[0] * a[1]
        if name == "div":
            return a[0] / a[1]
        if name == "min":
            return np.minimum(a[0], a[1])
        if name == "max":
            return np.maximum(a[0], a[1])
        if name == "cmp":
            return _CMP[str(attrs["cmp"])](_f32(a[0]), _f32(a[1])).astype(F64)
        if name == "cast":
            return round_to_storage(a[0], str(attrs["to"]))
        if name == "sum":
            return _rowsum(a[0])
        if name == "rmax":
            return np.max(a[0], axis=-1, keepdims=True)
        if name == "rmin":
            return np.min(a[0], axis=-1, keepdims=True)
        # Table 1's reductions in their general form: [M, size, N] reduced along `size` to [M, 1, N]
        # (the penultimate axis; the row reductions above are the N = 1 case)
        if name == "csum":
            return np.sum(a[0], axis=-2, keepdims=True)
        if name == "cmax":
            return np.max(a[0], axis=-2, keepdims=True)
        if name == "cmin":
            return np.min(a[0], axis=-2, keepdims=True)
        if name == "select":
            cond, xm, xn = a
            return np.where(_f32(cond) != 0.0, xm, xn)
        # --- extras built from Table 1's Exp / Div / Sqrt / Mul -----------------------------
        if name == "neg":
            return -a[0]
        if name == "rsqrt":
            return 1.0 / np.sqrt(a[0])
        if name == "rcp":
            return 1.0 / a[0]
        if name == "tanh":
            return np.tanh(a[0])
        if name == "erf":
            return _erf(a[0])
        if name == "sigmoid":
            return _sigmoid(a[0])
        if name == "square":
            return a[0] * a[0]
        if name == "gelu_tanh":
            return _gelu_tanh(a[0])
        if name == "gelu_erf":
            return _gelu_erf(a[0])
        if name == "silu":
            return a[0] * _sigmoid(a[0])
        # --- row statistics and compound ops, last axis of length H --------------------------
        if name == "mean":
            return _rowsum(a[0]) / a[0].shape[-1]
        if name == "meansq":
            return _rowsum(a[0] * a[0]) / a[0].shape[-1]
        if name == "softmax":
            z = a[0]
            e = np.exp(z - np.max(z, axis=-1, keepdims=True))
            return e / _rowsum(e)
        if name == "rmsnorm":
            x, w = a
            ms = _rowsum(x * x) / x.shape[-1]
            return x * (1.0 / np.sqrt(ms + float(attrs["eps"]))) * w
        if name == "layernorm":
            h, gamma, beta = a
            mu = _rowsum(h) / h.shape[-1]
            d = h - mu
            var = _rowsum(d * d) / h.shape[-1]           # biased variance, two passes
            return d * (1.0 / np.sqrt(var + float(attrs["eps"]))) * gamma + beta
    raise ValueError(f"oracle: unknown op {name!r}")


# ----------------------------------------------------------------------------------------------
# the interpreter
# ----------------------------------------------------------------------------------------------

def run(program, inputs: Mapping[str, np.ndarray], keep_intermediates: bool = False):
    """Evaluate ``program`` (a workloads.programs.Program) op by op.

    ``inputs`` maps input names to arrays of values already representable in the input's storage
    dtype.  Returns ``(rounded, exact)``: two dicts keyed by output name, holding the outputs
    rounded once to their storage dtype and the unrounded float64 results.  With
    ``keep_intermediates`` the second dict holds every value of the program.
    """
    env: Dict[str, np.ndarray] = {}
    for name, _dtype in program.inputs:
        env[name] = np.array(inputs[name], dtype=F64)
    for op in program.ops:
        env[op.out] = np.asarray(_eval(op.name, tuple(env[n] for n in op.args), op.attrs), dtype=F64)
    rounded = {n: round_to_storage(env[n], dt) for n, dt in program.outputs}
    exact = dict(env) if keep_intermediates else {n: env[n] for n, _ in program.outputs}
    return rounded, exact


def row_scale(exact: np.ndarray) -> np.ndarray:
    """RMS of the finite reference values over each output row (last axis), the natural scale used
    by the mixed tolerance ``|got-ref| <= rtol*|ref| + rtol*row_scale``."""
    x = np.asarray(exact, dtype=F64)
    fin = np.isfinite(x)
    xs = np.where(fin, x, 0.0)
    n = np.maximum(fin.sum(axis=-1, keepdims=True), 1)
    return np.sqrt((xs * xs).sum(axis=-1, keepdims=True) / n)
