"""Parity of the HIP virtual machine against the CPU oracle, element by element, through the C ABI.
Every test prints its case before touching the GPU so that a fault names its case."""
import sys

import numpy as np
import pytest
import torch

from paper_2603_24239_amd import binding as B
from tests import harness as H
from workloads import gen
from workloads import programs as W
from workloads.programs import single_op_program

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


UNARY = ["sqrt", "abs", "log", "exp", "round", "floor", "isfinite", "neg", "rsqrt", "rcp", "tanh", "erf", "sigmoid",
         "square", "gelu_tanh", "gelu_erf", "silu", "copy"]
BINARY = ["add", "sub", "mul", "div", "min", "max", "pow"]
POSITIVE = {"sqrt", "log", "rsqrt", "pow"}


def _vals(shape, seed, op="", dtype="f32"):
    x = gen.randn(shape, seed, DEV, "f32", std=2.0)
    if op in POSITIVE:
        x = x.abs() + 0.05
    if op in ("round", "floor"):
        x = x * 3
    return x.to(torch.bfloat16) if dtype == "bf16" else x


# ---------------------------------------------------------------------------------------- aligned shapes

def test_c1_config():
    say("c1 gelu(x*a+b) fp32 [4,1000]")
    for variant in ("c1_gelu_erf", "c1_gelu_tanh"):
        H.check_program(W.get_program(variant), gen.c1_inputs(device=DEV))


def test_identity_bit_exact():
    say("identity x*1+0")
    x = gen.randn((33, 512), 5, DEV)
    outs, _ = H.run_vm(W.get_program("identity_affine"), {"x": x})
    assert torch.equal(outs["y"].view(torch.int32), x.view(torch.int32))


@pytest.mark.parametrize("op", UNARY)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unary_ops(op, dtype):
    say("unary", op, dtype)
    x = _vals((8, 1024), 11, op, dtype)
    if op == "isfinite":
        x = x.clone()
        x[0, :4] = torch.tensor([float("inf"), float("-inf"), float("nan"), 1.0], device=DEV).to(x.dtype)
    H.check_program(single_op_program(op, 1, dtype), {"a0": x})


@pytest.mark.parametrize("op", BINARY)
def test_binary_ops(op):
    say("binary", op)
    a = _vals((8, 1024), 21, op)
    b = _vals((8, 1024), 22, op)
    if op == "pow":
        b = gen.randn((8, 1024), 23, DEV)
    H.check_program(single_op_program(op, 2), {"a0": a, "a1": b})


@pytest.mark.parametrize("c", ["eq", "ne", "lt", "le", "gt", "ge"])
def test_cmp_ops(c):
    say("cmp", c)
    a = gen.randn((4, 2048), 31, DEV)
    b = gen.randn((4, 2048), 32, DEV)
    b[:, ::5] = a[:, ::5]
    outs, _, _ = H.check_program(single_op_program("cmp", 2, cmp=c), {"a0": a, "a1": b})
    assert set(outs["y"].unique().tolist()) <= {0.0, 1.0}


def test_select_and_if_else_add():
    say("select / if_else_add")
    a, b = gen.randn((6, 7, 64), 41, DEV), gen.randn((6, 7, 64), 42, DEV)
    x, y = gen.randn((6, 7, 64), 43, DEV), gen.randn((6, 7, 64), 44, DEV)
    H.check_program(W.get_program("if_else_add"), {"a": a, "b": b, "x": x, "y": y})
    H.check_program(W.get_program("if_else_add_true"), {"x": x, "y": y})
    H.check_program(W.get_program("if_else_add_false"), {"x": x, "y": y})


def test_scalar_imm_and_cast():
    say("adds / muls / cast")
    x = gen.randn((16, 256), 51, DEV)
    H.check_program(single_op_program("adds", 1, imm=2.5), {"a0": x})
    H.check_program(single_op_program("muls", 1, imm=-0.75), {"a0": x})
    H.check_program(single_op_program("cast", 1, to="bf16"), {"a0": x})


@pytest.mark.parametrize("op", ["sum", "rmax", "rmin", "mean", "meansq"])
@pytest.mark.parametrize("cols", [64, 256, 4096, 8192])
def test_row_reductions(op, cols):
    say("reduce", op, cols)
    x = gen.randn((9, cols), 61, DEV)
    outs, _, _ = H.check_program(single_op_program(op, 1), {"a0": x})
    assert outs["y"].shape == (9, 1)


def test_rmsnorm_small():
    say("rmsnorm bf16 [2,5,4096]")
    ins = gen.c2_inputs(2, 5, 71, DEV)
    H.check_program(W.get_program("c2_rmsnorm"), ins)
    H.check_program(W.get_program("c2_rmsnorm_basic"), ins)


def test_softmax_aligned():
    say("masked softmax fp32 [2,4,64,64]")
    z = gen.randn((2, 4, 64, 64), 81, DEV, std=3.0)
    mask = gen.causal_mask(64, DEV)
    outs, _, _ = H.check_program(W.get_program("c3_masked_softmax"), {"z": z, "mask": mask})
    p = outs["p"]
    assert torch.all(p[..., torch.triu(torch.ones(64, 64, dtype=torch.bool, device=DEV), 1)] == 0)
    H.check_program(W.get_program("softmax_f32"), {"z": z})
    H.check_program(W.get_program("softmax_bf16"), {"z": z.to(torch.bfloat16)})


def test_layernorm_small():
    say("layernorm f32/bf16 [3,7,1024]")
    x = gen.randn((3, 7, 1024), 91, DEV, std=2.0) + 0.5
    g = gen.randn((1024,), 92, DEV, mean=1.0, std=0.1)
    b = gen.randn((1024,), 93, DEV, std=0.1)
    H.check_program(W.get_program("layernorm_f32"), {"x": x, "gamma": g, "beta": b})
    bf = torch.bfloat16
    H.check_program(W.get_program("layernorm_bf16"), {"x": x.to(bf), "gamma": g.to(bf), "beta": b.to(bf)})


def test_c4_chain_small():
    say("c4 chain bf16 [9,8192]")
    ins = gen.c4_inputs(9, 101, DEV)
    H.check_program(W.get_program("c4_chain"), ins)
    H.check_program(W.get_program("c4_chain_ln"), ins)


def test_c5_programs_small():
    T = 16
    say("c5 programs T=16")
    d = gen.c5_inputs(T, 111, DEV)
    H.check_program(W.get_program("c5_rmsnorm"), d["c5_rmsnorm"])
    H.check_program(W.get_program("c5_residual"), d["c5_residual_a"])
    H.check_program(W.get_program("c5_silu_gate"), d["c5_silu_gate"])
    say("c5 rope T=16 (view load / view store)")
    rope_in = d["c5_rope"]
    out = torch.full((T, 32, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    views = {"y1": out[..., :64], "y2": out[..., 64:]}
    H.check_program(W.get_program("c5_rope"), rope_in, views)
    assert not torch.isnan(out.float()).any()


def test_broadcast_forms():
    say("broadcast: row vector, column vector, leading dims")
    prog = single_op_program("add", 2)
    x = gen.randn((5, 6, 128), 121, DEV)
    for shape in [(128,), (6, 1), (5, 1, 1), (1, 6, 128), (5, 1, 128), (1,)]:
        y = gen.randn(shape, 122, DEV)
        H.check_program(prog, {"a0": x, "a1": y}, what=f"add {tuple(x.shape)}+{shape}")
        H.check_program(single_op_program("sub", 2), {"a0": y, "a1": x}, what=f"sub {shape}-{tuple(x.shape)}")


def test_determinism_bitwise():
    say("determinism: same bytecode twice")
    ins = gen.c4_inputs(33, 131, DEV)
    o1, c1 = H.run_vm(W.get_program("c4_chain"), ins)
    o2, c2 = H.run_vm(W.get_program("c4_chain"), ins)
    assert c1.raw == c2.raw
    assert torch.equal(o1["y"].view(torch.int16), o2["y"].view(torch.int16))


# ---------------------------------------------------------------------------------------- ragged shapes

@pytest.mark.parametrize("shape", [(1, 1), (3, 5), (7, 333), (5, 1001), (2, 4099), (1, 70001), (129, 17)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_elementwise(shape, dtype):
    say("ragged elementwise", shape, dtype)
    x = _vals(shape, 141, "", dtype)
    y = _vals(shape, 142, "", dtype)
    H.check_program(single_op_program("mul", 2, dtype), {"a0": x, "a1": y})
    v = _vals(shape[-1:], 143, "", dtype)
    H.check_program(single_op_program("add", 2, dtype), {"a0": x, "a1": v})


@pytest.mark.parametrize("cols", [1, 3, 17, 63, 65, 333, 1001, 2100, 4095, 5000])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_softmax(cols, dtype):
    say("ragged softmax", cols, dtype)
    z = gen.randn((11, cols), 151, DEV, dtype, std=3.0)
    H.check_program(W.get_program("softmax_f32" if dtype == "f32" else "softmax_bf16"), {"z": z})


def test_ragged_masked_softmax():
    say("ragged masked softmax S=333, S=129")
    for S in (333, 129):
        ins = gen.c3_inputs(2, S, 161, DEV, heads=3)
        outs, _, _ = H.check_program(W.get_program("c3_masked_softmax"), ins)
        tri = torch.triu(torch.ones(S, S, dtype=torch.bool, device=DEV), 1)
        assert torch.all(outs["p"][..., tri] == 0)


def test_c5_softmax_odd_rows():
    for T in (1, 8, 37, 200):
        say("c5 softmax bf16 [32, T, T//8+1], T =", T)
        H.check_program(W.get_program("c5_softmax"), {"z": gen.randn((32, T, T // 8 + 1), 171, DEV, "bf16")})


def test_strided_input_rows():
    say("row-strided views")
    base = gen.randn((16, 640), 181, DEV)
    x = base[:, :600]                     # row stride 640, row length 600
    y = base[:, 40:640]
    H.check_program(single_op_program("add", 2), {"a0": x, "a1": y})
    H.check_program(W.get_program("softmax_f32"), {"z": x})


def test_empty_and_tiny():
    say("empty tensor / single element")
    x = torch.empty((0, 128), device=DEV)
    outs, code = H.run_vm(single_op_program("exp", 1), {"a0": x})
    assert outs["y"].shape == (0, 128)
    one = torch.tensor([[1.5]], device=DEV)
    H.check_program(single_op_program("exp", 1), {"a0": one})
    H.check_program(W.get_program("softmax_f32"), {"z": one})


def test_operand_pinned_along_the_fastest_outer_dim():
    """A mask [S, L] under scores [N, S, L]: the N dim is visited fastest and the mask row stays in a tile
    register until the S index changes; N not a multiple of the rows per tile makes tiles straddle."""
    desc = W.get_program("c3_masked_softmax")
    blocked = B.Context(torch.cuda.current_device())
    blocked.set_assignment("blocked")
    inter = B.Context(torch.cuda.current_device())
    inter.set_assignment("interleaved")     # (the pinned mask row is reloaded for nearly every tile)
    for (n, s_, l) in [(17, 40, 100), (19, 33, 257), (64, 7, 1000), (16, 300, 64), (130, 5, 33)]:
        say(f"pinned mask rows: scores [{n},{s_},{l}]")
        z = gen.randn((n, s_, l), 500 + n, DEV, "f32", std=3.0)
        mask = torch.zeros((s_, l), dtype=torch.float32, device=DEV)
        mask.masked_fill_(torch.rand((s_, l), generator=torch.Generator(DEV).manual_seed(n), device=DEV) < 0.3, float("-inf"))
        mask[:, 0] = 0.0            # no fully masked row
        _, code, _ = H.check_program(desc, {"z": z, "mask": mask}, ctx=blocked)
        assert "again whenever the second outer index changes" in code.disasm()
        _, code, _ = H.check_program(desc, {"z": z, "mask": mask}, ctx=inter)
        assert "again whenever the second outer index changes" in code.disasm()
        H.check_program(desc, {"z": z, "mask": mask})
