"""The interpreter variant with 64 elements per lane and one tile register, on the GPU against the oracle: programs that
need at most one tile register beside the accumulator, planned for it through the context's limits."""
from __future__ import annotations

import pytest
import torch

from paper_2603_24239_amd import binding as B
from workloads import gen
from workloads import programs as W
from workloads.programs import single_op_program

from . import harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(torch.cuda.current_device())
    c.set_limits(64, 1)
    return c


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("rows,cols", [(37, 4096), (300, 4095), (100, 8192), (33, 16384), (50, 8200), (64, 2049), (1000, 513),
                                       (700, 257), (2000, 65), (5, 100003)])
def test_softmax_rows(ctx, dt, rows, cols):
    say(f"64 elements per lane: softmax {dt} [{rows},{cols}]")
    _, code, _ = H.check_program(single_op_program("softmax", 1, dt), {"a0": gen.randn((rows, cols), 11, DEV, dt)}, ctx=ctx)
    assert code.info().variant_nr <= 1


def test_config_programs(ctx):
    for name, d in [("c2_rmsnorm", gen.c2_inputs(3, 700, 5, DEV)), ("c3_masked_softmax", gen.c3_inputs(1, 1000, 6, DEV)),
                    ("c3_masked_softmax", gen.c3_inputs(2, 517, 7, DEV))]:
        say(f"64 elements per lane: {name}")
        _, code, _ = H.check_program(W.get_program(name), d, ctx=ctx)
        assert code.info().variant_k == 64 and code.info().variant_nr == 1
    d = gen.c5_inputs(300, 8, DEV)
    for name, key in [("c5_rmsnorm", "c5_rmsnorm"), ("c5_softmax", "c5_softmax"), ("c5_residual", "c5_residual_a"), ("c5_silu_gate", "c5_silu_gate")]:
        say(f"64 elements per lane: {name}")
        H.check_program(W.get_program(name), d[key], ctx=ctx)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(1000, 5000), (3, 100000), (70000,), (129, 4096), (7,)])
def test_elementwise(ctx, dt, shape):
    say(f"64 elements per lane: add and gelu {dt} {shape}")
    H.check_program(single_op_program("add", 2, dt), {"a0": gen.randn(shape, 1, DEV, dt), "a1": gen.randn(shape, 2, DEV, dt)}, ctx=ctx)
    H.check_program(single_op_program("gelu_tanh", 1, dt), {"a0": gen.randn(shape, 3, DEV, dt)}, ctx=ctx)


def test_a_program_that_needs_two_tile_registers_is_refused(ctx):
    with pytest.raises(B.DvmError) as e:
        B.encode_for(ctx, H.program(W.get_program("c4_chain")), [gen.c4_inputs(8, 1, DEV)[n] for n, _ in W.get_program("c4_chain").inputs])
    assert e.value.status == -5
