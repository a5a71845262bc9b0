"""The interpreter variant with 64 elements per lane and one tile register, on the GPU against the oracle.  A context whose
limits allow 64 elements plans programs with rows long enough that need at most one tile register beside the accumulator
for it; programs that need more registers and flat element-wise programs keep the 32-element variants."""
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
    c.set_limits(64, 2)
    return c


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("rows,cols", [(37, 4096), (300, 4095), (100, 8192), (33, 16384), (50, 8200), (64, 2049), (1000, 513),
                                       (700, 257), (2000, 65), (5, 100003)])
def test_softmax_rows(ctx, dt, rows, cols):
    say(f"64 elements per lane: softmax {dt} [{rows},{cols}]")
    _, code, _ = H.check_program(single_op_program("softmax", 1, dt), {"a0": gen.randn((rows, cols), 11, DEV, dt)}, ctx=ctx)
    if cols >= 4095 and rows >= 33:
        assert (code.info().variant_k, code.info().variant_nr) == (64, 1)


def test_config_programs(ctx):
    for name, d, k in [("c2_rmsnorm", gen.c2_inputs(3, 700, 5, DEV), 64), ("c3_masked_softmax", gen.c3_inputs(1, 2300, 6, DEV), 64),
                       ("c4_chain", gen.c4_inputs(333, 7, DEV), 32)]:
        say(f"64 elements per lane allowed: {name}")
        _, code, _ = H.check_program(W.get_program(name), d, ctx=ctx)
        assert code.info().variant_k == k
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


def test_parts_planned_for_different_variants_stack_by_the_registers_they_use(ctx):
    """A long-row part planned for (64, 1) and a short-row part planned for a two-register variant of which it uses one
    register share the (64, 1) launch."""
    desc = W.get_program("c2_rmsnorm")
    big, small = gen.c2_inputs(2, 300, 21, DEV), gen.c2_inputs(1, 3, 22, DEV)
    small["x"] = small["x"][..., :48].contiguous()
    small["w"] = small["w"][:48].contiguous()
    codes, tensors, outs = [], [], []
    for d in (big, small):
        ins = [d[n] for n, _ in desc.inputs]
        code = B.encode_for(ctx, H.program(desc), ins)
        o = [torch.zeros(s_, dtype=torch.bfloat16, device=DEV) for s_ in code.out_shapes]
        codes.append(code); tensors += ins + o; outs.append(o[0])
    assert codes[0].info().variant_k == 64 and codes[1].info().variant_k < 64
    st = B.dvm_stack(codes)
    assert (st.info().variant_k, st.info().variant_nr) == (64, 1)
    B.dvm_run(ctx, st, [t.data_ptr() for t in tensors], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for d, got in zip((big, small), outs):
        rounded, exact = H.run_oracle(desc, d)
        H.compare(got, rounded["y"], exact["y"], "bf16", True, "stacked rmsnorm parts of different variants")
