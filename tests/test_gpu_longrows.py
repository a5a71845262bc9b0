"""Rows longer than the widest tile (16 384 elements) with reductions along them: the interpreter passes over such a
row once per reduction and once more for the stores.  Parity with the oracle for softmax, RMSNorm, LayerNorm and a
row-sum at 16 385 .. 100 003 columns, fp32 and bf16 storage."""
from __future__ import annotations

import pytest
import torch

from workloads import gen
from workloads import programs as W
from workloads.programs import _p, single_op_program

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cols", [16385, 32768, 100000, 100003])
def test_softmax_over_long_rows(cols, dtype):
    say(f"softmax {dtype} [19, {cols}]")
    z = gen.randn((19, cols), 9000 + cols, DEV, dtype, std=3.0)
    z[3, cols - 1] = 30.0           # the row maximum in the last, ragged tile
    z[5, 0] = 25.0                  # and in the first
    outs, code, _ = H.check_program(single_op_program("softmax", 1, dtype), {"a0": z})
    assert "rows longer than a tile: 3 passes" in code.disasm()
    sums = outs["y"].float().sum(dim=-1)
    assert float((sums - 1).abs().max()) < (2e-2 if dtype == "bf16" else 1e-3)


@pytest.mark.parametrize("cols", [32768, 100000])
def test_rmsnorm_and_layernorm_over_long_rows(cols):
    say(f"rmsnorm / layernorm bf16 [2, 7, {cols}]")
    d = gen.c2_inputs(2, 7, 9100 + cols, DEV, hidden=cols) if "hidden" in gen.c2_inputs.__code__.co_varnames else None
    if d is None:
        d = {"x": gen.randn((2, 7, cols), 9100, DEV, "bf16"), "w": gen.randn((cols,), 9101, DEV, "bf16", mean=1.0, std=0.1)}
    _, code, _ = H.check_program(W.get_program("c2_rmsnorm"), d)
    assert "rows longer than a tile: 2 passes" in code.disasm()
    ln = {"x": gen.randn((11, cols), 9102, DEV, "bf16"), "gamma": gen.randn((cols,), 9103, DEV, "bf16", mean=1.0, std=0.1),
          "beta": gen.randn((cols,), 9104, DEV, "bf16", std=0.1)}
    _, code, _ = H.check_program(W.get_program("layernorm_bf16"), ln)
    assert "rows longer than a tile: 3 passes" in code.disasm()


def test_row_value_output_and_a_view_over_long_rows():
    say("row sum and scaled rows, fp32 [5, 3, 40000] read through a strided view")
    base = gen.randn((5, 3, 40010), 9200, DEV)
    x = base[..., 5:40005]                                  # rows of 40000 inside rows of 40010: unaligned starts
    desc = _p("sum_and_scale", [("x", "f32")], [("s", "sum", ["x"], {}), ("y", "div", ["x", "s"], {})], [("s", "f32"), ("y", "f32")])
    outs, code, _ = H.check_program(desc, {"x": x})
    assert "rows longer than a tile" in code.disasm()
    assert outs["s"].shape == (5, 3, 1)
