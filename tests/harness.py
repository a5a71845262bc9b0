"""Shared helpers of the parity tests: run a program on the HIP VM, run it on the oracle, compare.

Tolerance (stated per test through `kind`):
  fp32 outputs  rtol 1e-5 for purely elementwise programs, 1e-4 when the program contains a reduction;
  bf16 outputs  rtol 2e-2 (fp32 accumulation, one rounding at the output).
An element passes iff |got - ref| <= rtol * |ref| + a * rtol * s_row, with s_row the RMS of the
reference over that output row and a = 1 for programs with a reduction, 0.01 for purely element-wise
ones: cancellation can drive a reference value to ~0, where a purely relative bound is unattainable
for any fp32 evaluation.  Non-finite references must be matched
in kind (NaN with NaN, +-inf with the same infinity).
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np
import torch

from oracle import interp
from paper_2603_24239_amd import binding as B

RTOL = {("f32", False): 1e-5, ("f32", True): 1e-4, ("bf16", False): 2e-2, ("bf16", True): 2e-2}

_REDUCING = {"sum", "rmax", "rmin", "mean", "meansq", "softmax", "rmsnorm", "layernorm"}


def has_reduction(desc) -> bool:
    return any(op.name in _REDUCING for op in desc.ops)


_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}

_ctx_cache: Dict[int, B.Context] = {}
_prog_cache: Dict[str, B.Program] = {}


def gpu_ctx() -> B.Context:
    dev = torch.cuda.current_device()
    if dev not in _ctx_cache:
        _ctx_cache[dev] = B.Context(dev)
    return _ctx_cache[dev]


def program(desc) -> B.Program:
    key = repr((desc.name, desc.inputs, desc.ops, desc.outputs))
    if key not in _prog_cache:
        _prog_cache[key] = B.Program(desc)
    return _prog_cache[key]


def run_vm(desc, inputs: Dict[str, torch.Tensor], outputs: Optional[Dict[str, torch.Tensor]] = None,
           ctx: Optional[B.Context] = None, sync: bool = True):
    """Encode + run `desc` on the GPU.  `inputs` maps input names to CUDA tensors (views allowed).
    `outputs` may supply pre-allocated output tensors/views; otherwise contiguous ones are made.
    Returns (dict of output tensors, Bytecode)."""
    ctx = ctx or gpu_ctx()
    prog = program(desc)
    ins = [inputs[n] for n, _ in desc.inputs]
    for (n, dt), t in zip(desc.inputs, ins):
        assert t.dtype == _TORCH_DT[dt], (n, t.dtype, dt)
        assert t.is_cuda
    if outputs is None:
        code = B.encode_for(ctx, prog, ins)
        outs = [torch.empty(shape, dtype=_TORCH_DT[dt], device=ins[0].device)
                for (_, dt), shape in zip(desc.outputs, code.out_shapes)]
    else:
        outs = [outputs[n] for n, _ in desc.outputs]
        code = B.encode_for(ctx, prog, ins, outs)
    B.run_on(ctx, code, ins + outs)
    if sync:
        torch.cuda.synchronize()
    return {n: t for (n, _), t in zip(desc.outputs, outs)}, code


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def run_oracle(desc, inputs: Dict[str, torch.Tensor]):
    return interp.run(desc, {n: to_np64(inputs[n]) for n, _ in desc.inputs})


def compare(got: torch.Tensor, rounded: np.ndarray, exact: np.ndarray, dtype: str, reducing: bool,
            what: str = "") -> float:
    """Assert `got` matches the oracle; returns the largest error in units of the tolerance."""
    rtol = RTOL[(dtype, reducing)]
    g = to_np64(got)
    ref = np.asarray(rounded, dtype=np.float64)
    assert g.shape == ref.shape, (what, g.shape, ref.shape)
    if g.size == 0:
        return 0.0
    fin = np.isfinite(ref)
    # non-finite references must be matched in kind
    nan_ref = np.isnan(ref)
    assert np.array_equal(np.isnan(g), nan_ref), f"{what}: NaN pattern differs"
    inf_ref = np.isinf(ref)
    assert np.array_equal(g[inf_ref], ref[inf_ref]), f"{what}: infinities differ"
    scale = interp.row_scale(exact)
    scale = np.broadcast_to(scale, ref.shape)
    err = np.abs(g - ref)
    # the absolute term covers cancellation: in full for programs that reduce (a row statistic is subtracted or
    # divided by), at a hundredth for purely element-wise ones (a difference of two inputs of the row's size)
    tol = rtol * np.abs(ref) + rtol * (1.0 if reducing else 1e-2) * scale
    tol = np.where(tol > 0, tol, np.finfo(np.float64).tiny)
    ratio = np.where(fin, err / tol, 0.0)
    worst = float(ratio.max())
    if worst > 1.0:
        idx = np.unravel_index(int(np.argmax(ratio)), ratio.shape)
        raise AssertionError(f"{what}: |got-ref| exceeds tolerance x{worst:.3g} at {idx}: got {g[idx]!r} ref {ref[idx]!r} "
                             f"(rtol {rtol}, row scale {scale[idx]!r})")
    return worst


def check_program(desc, inputs: Dict[str, torch.Tensor], outputs: Optional[Dict[str, torch.Tensor]] = None,
                  what: str = "", ctx: Optional[B.Context] = None):
    outs, code = run_vm(desc, inputs, outputs, ctx=ctx)
    rounded, exact = run_oracle(desc, inputs)
    red = has_reduction(desc)
    worst = 0.0
    for n, dt in desc.outputs:
        worst = max(worst, compare(outs[n], rounded[n], exact[n], dt, red, f"{what or desc.name}:{n}"))
    return outs, code, worst
